// Host side of the structured-binary library: layout closed forms, the bit-exact packer and the host
// dequantiser.  Pure C++ (no HIP).  Must be compiled with -ffp-contract=off: the packer's results are
// defined by a fixed sequence of IEEE double operations (sequential ascending-index sums, one divide
// per mean, fp64 -> fp32 -> fp16 rounding for stored scales).
#include "stb_internal.h"
#include "stb_f16.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

inline uint16_t f32_to_f16_bits(float f) { return stb_f32_to_f16_bits(f); }
inline float f16_bits_to_f32(uint16_t h) { return stb_f16_bits_to_f32(h); }
inline uint16_t f64_to_f16_bits(double v) { return stb_f64_to_f16_bits(v); }   // fp64 -> fp32 -> fp16

int check_cfg(const stb_cfg_t* c) {
    if (!c) return STB_ENULL;
    if (c->block != STB_BLOCK) return STB_EINVAL;
    if (c->M != 4 && c->M != 8) return STB_EINVAL;
    if (c->N < 1 || c->N > c->M) return STB_EINVAL;
    if (c->n_out < 1 || c->k_in < STB_BLOCK || c->k_in % STB_BLOCK != 0) return STB_EINVAL;
    if (c->n_salient < 0 || c->n_salient > c->k_in) return STB_EINVAL;
    if (c->region_mode != 0 && c->region_mode != 1) return STB_EINVAL;
    return STB_OK;
}

template <class F>
void parallel_for(int64_t count, int n_threads, F&& body) {
    if (n_threads <= 1 || count <= 1) {
        for (int64_t i = 0; i < count; i++) body(i);
        return;
    }
    std::atomic<int64_t> next(0);
    std::vector<std::thread> pool;
    int nt = (int)std::min<int64_t>(n_threads, count);
    for (int t = 0; t < nt; t++)
        pool.emplace_back([&]() {
            for (;;) {
                int64_t i = next.fetch_add(1);
                if (i >= count) break;
                body(i);
            }
        });
    for (auto& th : pool) th.join();
}

inline bool sal_bit(const uint32_t* bm, int j) { return (bm[j >> 5] >> (j & 31)) & 1u; }

}  // namespace

namespace {

void place_planes(stb_layout_t* out) {
    out->total_bytes = out->mask_bytes + out->sign_bytes + out->region_bytes + out->res_bytes +
                       out->scales_bytes + out->res_scale_bytes + out->salmap_bytes + out->salprefix_bytes +
                       out->saltab_bytes + out->res_t_bytes;
    int64_t off = 0;
    auto place = [&](int64_t bytes) {
        int64_t o = off;
        off = round_up(off + bytes, STB_PLANE_ALIGN);
        return o;
    };
    out->off_mask = place(out->mask_bytes);
    out->off_sign = place(out->sign_bytes);
    out->off_region = place(out->region_bytes);
    out->off_res = place(out->res_bytes);
    out->off_scales = place(out->scales_bytes);
    out->off_res_scale = place(out->res_scale_bytes);
    out->off_salmap = place(out->salmap_bytes);
    out->off_salprefix = place(out->salprefix_bytes);
    out->off_saltab = place(out->saltab_bytes);
    out->off_res_t = place(out->res_t_bytes);
    out->image_bytes = off;
}

}  // namespace

extern "C" int stb_layout_sizes(const stb_cfg_t* cfg, stb_layout_t* out) {
    if (!out) return STB_ENULL;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    std::memset(out, 0, sizeof(*out));
    out->cfg = *cfg;
    out->kind = STB_KIND_ROWMAJOR;
    const int64_t n = cfg->n_out, k = cfg->k_in, nb = k / STB_BLOCK;
    const int64_t slots = k * cfg->N / cfg->M;
    out->n_blocks = (int32_t)nb;
    out->n_salient_pad = cfg->n_salient > 0 ? (int32_t)round_up(cfg->n_salient, 128) : 0;
    out->mask_stride = k / 8;
    out->sign_stride = round_up(round_up(slots, 8) / 8, 16);
    out->region_stride = round_up(round_up(2 * slots, 8) / 8, 16);
    out->res_stride = out->n_salient_pad / 8;
    out->mask_bytes = n * out->mask_stride;
    out->sign_bytes = n * out->sign_stride;
    out->region_bytes = n * out->region_stride;
    out->res_bytes = n * out->res_stride;
    out->scales_bytes = n * nb * 4 * 2;
    out->res_scale_bytes = n * nb * 2;
    out->salmap_bytes = k / 8;
    out->salprefix_bytes = 4 * (nb + 1);
    out->saltab_bytes = 0;
    place_planes(out);
    return STB_OK;
}

extern "C" int stb_tiled_sizes(const stb_cfg_t* cfg, stb_layout_t* out) {
    if (!out) return STB_ENULL;
    int rc = check_cfg(cfg);
    if (rc) return rc;
    std::memset(out, 0, sizeof(*out));
    out->cfg = *cfg;
    out->kind = STB_KIND_TILED;
    const int64_t n = cfg->n_out, k = cfg->k_in, nb = k / STB_BLOCK;
    const int64_t nrt = (n + 15) / 16, nsb = (nb + 3) / 4;
    const int64_t rec = nrt * nsb * 64;                          // lane records
    out->n_blocks = (int32_t)nb;
    out->n_row_tiles = (int32_t)nrt;
    out->n_super = (int32_t)nsb;
    out->n_salient_pad = cfg->n_salient > 0 ? (int32_t)round_up(cfg->n_salient, 128) : 0;
    out->sal_chunks = cfg->n_salient > 0 ? (int32_t)((std::min<int64_t>(cfg->n_salient, 64) + 7) / 8) : 0;
    out->mask_stride = 16;
    out->sign_stride = 16 * cfg->N / cfg->M;                     // 128*N/M sign bits per block
    out->region_stride = 32 * cfg->N / cfg->M;
    if (stb_tiled_padded(cfg)) {                                 // 3 or 5 of 8: stored with the slots of 4 or 6 of 8
        out->sign_stride = 2 * stb_tiled_slots(cfg);
        out->region_stride = 4 * stb_tiled_slots(cfg);
    }
    out->res_stride = out->n_salient_pad / 8;
    out->mask_bytes = rec * out->mask_stride;
    out->sign_bytes = rec * out->sign_stride;
    out->region_bytes = rec * out->region_stride;
    out->res_bytes = nrt * 16 * out->res_stride;
    out->scales_bytes = rec * 8;
    out->res_scale_bytes = rec * 2;
    out->salmap_bytes = nsb * 4 * 16;
    out->salprefix_bytes = 4 * (nsb * 4 + 1);
    out->saltab_bytes = nsb * 4 * 2 * out->sal_chunks * 48;
    out->res_t_bytes = cfg->n_salient > 0 ? rec * 4 : 0;
    place_planes(out);
    return STB_OK;
}

extern "C" int stb_layout_bind(stb_layout_t* L, void* base) {
    if (!L || !base) return STB_ENULL;
    if ((uintptr_t)base % STB_PLANE_ALIGN) return STB_EALIGN;
    char* b = (char*)base;
    L->mask = (uint32_t*)(b + L->off_mask);
    L->sign = (uint32_t*)(b + L->off_sign);
    L->region = (uint32_t*)(b + L->off_region);
    L->res_sign = (uint32_t*)(b + L->off_res);
    L->scales = (uint16_t*)(b + L->off_scales);
    L->res_scale = (uint16_t*)(b + L->off_res_scale);
    L->sal_bitmap = (uint32_t*)(b + L->off_salmap);
    L->sal_block_prefix = (uint32_t*)(b + L->off_salprefix);
    L->sal_tab = (uint32_t*)(b + L->off_saltab);
    L->res_t = (uint32_t*)(b + L->off_res_t);
    return STB_OK;
}

// Validates that the size fields agree with the closed form for L->cfg and that the plane pointers are
// set and 16-byte aligned.  Shared by the host and device entry points.
extern "C" int stb_layout_check(const stb_layout_t* L) {
    if (!L) return STB_ENULL;
    stb_layout_t ref;
    int rc;
    if (L->kind == STB_KIND_ROWMAJOR) rc = stb_layout_sizes(&L->cfg, &ref);
    else if (L->kind == STB_KIND_TILED) rc = stb_tiled_sizes(&L->cfg, &ref);
    else rc = STB_EINVAL;
    if (rc) return rc;
    if (L->n_salient_pad != ref.n_salient_pad || L->n_blocks != ref.n_blocks ||
        L->n_row_tiles != ref.n_row_tiles || L->n_super != ref.n_super || L->sal_chunks != ref.sal_chunks ||
        L->mask_stride != ref.mask_stride || L->sign_stride != ref.sign_stride ||
        L->region_stride != ref.region_stride || L->res_stride != ref.res_stride ||
        L->total_bytes != ref.total_bytes)
        return STB_EINVAL;
    if (L->kind == STB_KIND_TILED && (L->max_sal_block < 0 || L->max_sal_block > 16 * L->sal_chunks ||
                                      L->max_sal_half < 0 || L->max_sal_half > 8 * L->sal_chunks)) return STB_EINVAL;
    const void* ptrs[10] = {L->mask, L->sign, L->region, L->res_sign, L->scales, L->res_scale,
                            L->sal_bitmap, L->sal_block_prefix, L->sal_tab, L->res_t};
    for (int i = 0; i < 10; i++) {
        if ((i == 3 || i >= 8) && L->cfg.n_salient == 0) continue;   // res_sign / sal_tab / res_t may be absent
        if (i >= 8 && L->kind == STB_KIND_ROWMAJOR) continue;
        if (!ptrs[i]) return STB_ENULL;
        if ((uintptr_t)ptrs[i] % 16) return STB_EALIGN;
    }
    return STB_OK;
}

// ------------------------------------------------------------------------------------------------
// STB1 <-> tiled device order (byte permutation plus zero padding)
// ------------------------------------------------------------------------------------------------
namespace {

bool same_cfg(const stb_cfg_t& a, const stb_cfg_t& b) {
    return a.n_out == b.n_out && a.k_in == b.k_in && a.N == b.N && a.M == b.M && a.block == b.block &&
           a.n_salient == b.n_salient;
}

// Copies every (row, block) record between the two orders; to_tiled selects the direction.
// Returns STB_EINVAL when a padded layout (3 or 5 kept of 8) meets a mask byte with another number of bits.
int permute_records(const stb_layout_t* rm, const stb_layout_t* tl, bool to_tiled) {
    const int n = rm->cfg.n_out, nb = rm->n_blocks, nsb = tl->n_super;
    const int64_t SB = tl->sign_stride, RB = tl->region_stride;
    const bool padded = stb_tiled_padded(&rm->cfg);
    const int t8 = stb_tiled_slots(&rm->cfg), n8 = 8 * rm->cfg.N / rm->cfg.M;
    const int64_t RSB = 2 * n8, RRB = 4 * n8;               // row-major bytes per block when padded (M = 8)
    uint8_t* rmask = (uint8_t*)rm->mask; uint8_t* tmask = (uint8_t*)tl->mask;
    uint8_t* rsign = (uint8_t*)rm->sign; uint8_t* tsign = (uint8_t*)tl->sign;
    uint8_t* rreg = (uint8_t*)rm->region; uint8_t* treg = (uint8_t*)tl->region;
    auto mv = [&](uint8_t* a_rm, uint8_t* a_tl, int64_t bytes) {
        if (to_tiled) std::memcpy(a_tl, a_rm, bytes); else std::memcpy(a_rm, a_tl, bytes);
    };
    for (int r = 0; r < n; r++)
        for (int q = 0; q < nb; q++) {
            const int64_t tile = (int64_t)(r / 16) * nsb + q / 4, lane = 16 * (q % 4) + (r % 16);
            const int64_t rec = tile * 64 + lane;
            // a plane whose block record splits into two halves of whole 4-byte words is stored half by half
            // ([tile][half][lane]): a wavefront that works on one half of the columns then reads contiguous bytes
            auto mv_rec = [&](uint8_t* a_rm, uint8_t* t_plane, int64_t bytes) {
                if (bytes % 8 == 0) {
                    for (int h = 0; h < 2; h++)
                        mv(a_rm + h * (bytes / 2), t_plane + tile * 64 * bytes + h * 32 * bytes + lane * (bytes / 2), bytes / 2);
                } else {
                    mv(a_rm, t_plane + rec * bytes, bytes);
                }
            };
            uint8_t* mrow = rmask + (int64_t)r * rm->mask_stride + 16 * q;
            mv_rec(mrow, tmask, 16);                       // from here on the row-major mask is valid in both directions
            if (!padded) {
                mv_rec(rsign + (int64_t)r * rm->sign_stride + SB * q, tsign, SB);
                mv_rec(rreg + (int64_t)r * rm->region_stride + RB * q, treg, RB);
            } else {
                // slot s of the block (kept weights in column order) <-> slot t8 * group + rank of its column among
                // the group's kept columns and the lowest pruned one
                uint8_t* srow = rsign + (int64_t)r * rm->sign_stride + RSB * q;
                uint8_t* grow = rreg + (int64_t)r * rm->region_stride + RRB * q;
                uint8_t ps[12] = {0}, pr[24] = {0};
                if (!to_tiled) {
                    mv_rec(ps, tsign, SB);
                    mv_rec(pr, treg, RB);
                    std::memset(srow, 0, (size_t)RSB);
                    std::memset(grow, 0, (size_t)RRB);
                }
                int slot = 0;
                for (int g = 0; g < 16; g++) {
                    const unsigned mb = mrow[g];
                    if (__builtin_popcount(mb) != n8) return STB_EINVAL;
                    const unsigned aug = mb | (~mb & (mb + 1u));
                    for (int c = 0; c < 8; c++) {
                        if (!((mb >> c) & 1u)) continue;
                        const int t = t8 * g + __builtin_popcount(aug & ((1u << c) - 1u));
                        if (to_tiled) {
                            ps[t >> 3] |= (uint8_t)(((srow[slot >> 3] >> (slot & 7)) & 1u) << (t & 7));
                            pr[t >> 2] |= (uint8_t)(((grow[slot >> 2] >> ((slot & 3) * 2)) & 3u) << ((t & 3) * 2));
                        } else {
                            srow[slot >> 3] |= (uint8_t)(((ps[t >> 3] >> (t & 7)) & 1u) << (slot & 7));
                            grow[slot >> 2] |= (uint8_t)(((pr[t >> 2] >> ((t & 3) * 2)) & 3u) << ((slot & 3) * 2));
                        }
                        slot++;
                    }
                }
                if (to_tiled) {
                    mv_rec(ps, tsign, SB);
                    mv_rec(pr, treg, RB);
                }
            }
            mv((uint8_t*)(rm->scales + ((int64_t)r * nb + q) * 4), (uint8_t*)(tl->scales + rec * 4), 8);
            mv((uint8_t*)(rm->res_scale + (int64_t)r * nb + q), (uint8_t*)(tl->res_scale + rec), 2);
        }
    if (rm->cfg.n_salient) {
        const int words = (int)(rm->res_stride / 4);
        for (int r = 0; r < n; r++)
            for (int w = 0; w < words; w++)
                mv((uint8_t*)rm->res_sign + (int64_t)r * rm->res_stride + 4 * w,
                   (uint8_t*)tl->res_sign + (((int64_t)(r / 16) * words + w) * 16 + r % 16) * 4, 4);
    }
    return STB_OK;
}

// Fills the derived table of salient columns (layout in stb.h); returns the largest count of one block.
int fill_sal_tab(const stb_layout_t* tl, const uint32_t* bitmap, int k, const uint32_t* prefix, int* max_half) {
    const int nsb = tl->n_super, C = tl->sal_chunks;
    int mx = 0;
    *max_half = 0;
    std::vector<int> cols;
    for (int sb = 0; sb < nsb; sb++) {
        int need[2] = {0, 0};
        for (int g = 0; g < 4; g++) {
            int blk = 0;
            for (int h = 0; h < 2; h++) {
                int c = 0;
                const int j0 = (4 * sb + g) * 128 + 64 * h;
                for (int j = j0; j < std::min(k, j0 + 64); j++) c += sal_bit(bitmap, j);
                need[h] = std::max(need[h], (c + 7) / 8);
                *max_half = std::max(*max_half, c);
                blk += c;
            }
            mx = std::max(mx, blk);
        }
        for (int g = 0; g < 4; g++) {
            const int q = 4 * sb + g;
            uint32_t ord = prefix[q];                               // ordinal of the block's first salient column
            for (int h = 0; h < 2; h++) {
                cols.clear();
                const int j0 = q * 128 + 64 * h;
                for (int j = j0; j < std::min(k, j0 + 64); j++)
                    if (sal_bit(bitmap, j)) cols.push_back(j - q * 128);
                for (int c = 0; c < C; c++) {
                    uint32_t* rec = tl->sal_tab + (((int64_t)q * 2 + h) * C + c) * 12;
                    uint32_t sel[2] = {0, 0}, bit[2] = {0, 0};
                    uint16_t* pos = reinterpret_cast<uint16_t*>(rec + 8);
                    int cnt = 0;
                    for (int e = 0; e < 8; e++) {
                        const int idx = 8 * c + e;
                        const bool valid = idx < (int)cols.size();
                        const uint32_t pcol = valid ? (uint32_t)cols[idx] : 0xFFFFu;
                        const uint32_t byte = valid ? ((pcol >> 3) & 7u) : 0x0Cu;   // byte inside the half's 8 mask bytes
                        sel[e >> 2] |= byte << (8 * (e & 3));
                        if (valid) bit[e >> 2] |= (1u << (pcol & 7u)) << (8 * (e & 3));
                        pos[e] = (uint16_t)pcol;
                        cnt += valid;
                    }
                    rec[0] = sel[0]; rec[1] = sel[1];
                    rec[2] = bit[0]; rec[3] = bit[1];
                    rec[4] = ord + 8u * (uint32_t)c;
                    rec[5] = (uint32_t)need[h];
                    rec[6] = (uint32_t)cnt;
                    rec[7] = 0;
                }
                ord += (uint32_t)cols.size();
            }
        }
    }
    return mx;
}

}  // namespace

// res_t of the tiled order: per (row, block) the res_sign bits of the first 16 salient columns of each half block,
// half 0 in bits 0..15, half 1 in bits 16..31, at the lane record of (row, block).
void fill_res_t(const stb_layout_t* rm, const stb_layout_t* tl) {
    const int n = rm->cfg.n_out, nb = rm->n_blocks, nsb = tl->n_super;
    std::memset(tl->res_t, 0, (size_t)tl->res_t_bytes);
    for (int r = 0; r < n; r++) {
        const uint32_t* row = (const uint32_t*)((const uint8_t*)rm->res_sign + (int64_t)r * rm->res_stride);
        for (int q = 0; q < nb; q++) {
            uint32_t ord = rm->sal_block_prefix[q], word = 0;
            for (int h = 0; h < 2; h++) {
                int e = 0;
                for (int c = 64 * h; c < 64 * h + 64; c++) {
                    if (!sal_bit(rm->sal_bitmap, q * STB_BLOCK + c)) continue;
                    if (e < 16 && ((row[ord >> 5] >> (ord & 31)) & 1u)) word |= 1u << (16 * h + e);
                    e++;
                    ord++;
                }
            }
            const int64_t tile = (int64_t)(r / 16) * nsb + q / 4;
            tl->res_t[tile * 64 + 16 * (q % 4) + (r % 16)] = word;
        }
    }
}

// The derived tables of the tiled order from the salient bitmap alone (host arrays): bitmap and prefix padded to whole
// superblocks, the table of salient columns, the two maxima.  Shared by stb_tile and the device tiling.
extern "C" int stb_host_tiled_tables(const stb_layout_t* tl, const uint32_t* bitmap, const uint32_t* prefix,
                                     uint32_t* bitmap_out, uint32_t* prefix_out, uint32_t* sal_tab_out, int* max_block,
                                     int* max_half) {
    const int nb = tl->n_blocks, nsb = tl->n_super, k = tl->cfg.k_in;
    std::memset(bitmap_out, 0, (size_t)tl->salmap_bytes);
    std::memcpy(bitmap_out, bitmap, (size_t)k / 8);
    for (int q = 0; q <= nsb * 4; q++) prefix_out[q] = prefix[std::min(q, nb)];
    *max_block = 0;
    *max_half = 0;
    if (tl->cfg.n_salient) {
        stb_layout_t tmp = *tl;
        tmp.sal_tab = sal_tab_out;
        *max_block = fill_sal_tab(&tmp, bitmap, k, prefix_out, max_half);
    }
    return STB_OK;
}

extern "C" int stb_tile(const stb_layout_t* src, stb_layout_t* dst) {
    int rc = stb_layout_check(src);
    if (rc) return rc;
    if (!dst) return STB_ENULL;
    dst->max_sal_block = 0;
    dst->max_sal_half = 0;
    rc = stb_layout_check(dst);
    if (rc) return rc;
    if (src->kind != STB_KIND_ROWMAJOR || dst->kind != STB_KIND_TILED || !same_cfg(src->cfg, dst->cfg))
        return STB_EINVAL;
    std::memset(dst->mask, 0, dst->mask_bytes);
    std::memset(dst->sign, 0, dst->sign_bytes);
    std::memset(dst->region, 0, dst->region_bytes);
    if (dst->res_bytes) std::memset(dst->res_sign, 0, dst->res_bytes);
    std::memset(dst->scales, 0, dst->scales_bytes);
    std::memset(dst->res_scale, 0, dst->res_scale_bytes);
    std::memset(dst->sal_bitmap, 0, dst->salmap_bytes);
    rc = permute_records(src, dst, true);
    if (rc) return rc;
    const int nb = src->n_blocks, nsb = dst->n_super, k = src->cfg.k_in;
    std::memcpy(dst->sal_bitmap, src->sal_bitmap, src->salmap_bytes);
    for (int q = 0; q <= nsb * 4; q++) dst->sal_block_prefix[q] = src->sal_block_prefix[std::min(q, nb)];
    int mh = 0;
    const int mx = dst->cfg.n_salient ? fill_sal_tab(dst, src->sal_bitmap, k, dst->sal_block_prefix, &mh) : 0;
    if (dst->cfg.n_salient) fill_res_t(src, dst);
    dst->max_sal_block = mx;
    dst->max_sal_half = mh;
    return STB_OK;
}

extern "C" int stb_untile(const stb_layout_t* src, stb_layout_t* dst) {
    int rc = stb_layout_check(src);
    if (rc) return rc;
    rc = stb_layout_check(dst);
    if (rc) return rc;
    if (src->kind != STB_KIND_TILED || dst->kind != STB_KIND_ROWMAJOR || !same_cfg(src->cfg, dst->cfg))
        return STB_EINVAL;
    std::memset(dst->sign, 0, dst->sign_bytes);       // row padding of the sign / region planes
    std::memset(dst->region, 0, dst->region_bytes);
    rc = permute_records(dst, src, false);
    if (rc) return rc;
    std::memcpy(dst->sal_bitmap, src->sal_bitmap, dst->salmap_bytes);
    for (int q = 0; q <= dst->n_blocks; q++) dst->sal_block_prefix[q] = src->sal_block_prefix[q];
    return STB_OK;
}

// ------------------------------------------------------------------------------------------------
// packer
// ------------------------------------------------------------------------------------------------
namespace {

struct BlockScratch {
    std::vector<double> a;        // kept non-salient magnitudes, row after row
    std::vector<int32_t> start;   // first entry of each row in `a` (n + 1)
    std::vector<uint8_t> col;     // column inside the block of each entry
};

// Error of binarising the three regions separately (Eq. 5-6), rows left to right then top to bottom.
double trisection_error(const BlockScratch& s, int n, double p1, double p2) {
    double total = 0.0;
    for (int i = 0; i < n; i++) {
        const double* a = s.a.data() + s.start[i];
        const int cnt = s.start[i + 1] - s.start[i];
        double sum[3] = {0.0, 0.0, 0.0};
        int c[3] = {0, 0, 0};
        for (int e = 0; e < cnt; e++) {
            const int r = a[e] > p2 ? 2 : (a[e] > p1 ? 1 : 0);
            sum[r] += a[e];
            c[r]++;
        }
        double alpha[3];
        for (int r = 0; r < 3; r++) alpha[r] = c[r] > 0 ? sum[r] / (double)c[r] : 0.0;
        double row = 0.0;
        for (int e = 0; e < cnt; e++) {
            const int r = a[e] > p2 ? 2 : (a[e] > p1 ? 1 : 0);
            const double d = a[e] - alpha[r];
            row += d * d;
        }
        total += row;
    }
    return total;
}

// One block of 128 columns: residual binarisation of the kept salient weights (Eq. 4), break points and region
// scales of the kept non-salient ones (Alg. 2 NonSalientAwareQuant / Trisection, Eq. 6).  W has row stride `ldw`;
// `keep`, `ids`, `tpos` are n x k byte maps.  `nt` threads share the break-point candidates.
template <class T>
void quantise_block(const T* W, size_t ldw, int q, const stb_cfg_t& cfg, const uint8_t* keep, const uint32_t* sal_bitmap,
                    uint8_t* ids, uint8_t* tpos, uint16_t* scales, uint16_t* res_scale, int nt) {
    const int n = cfg.n_out, k = cfg.k_in, N = cfg.N, M = cfg.M, nb = k / STB_BLOCK;
    const int c0 = q * STB_BLOCK;
    BlockScratch s;
    s.start.resize(n + 1);
    s.a.reserve((size_t)n * STB_BLOCK * N / M);
    s.col.reserve((size_t)n * STB_BLOCK * N / M);
    double mx = 0.0;
    for (int i = 0; i < n; i++) {
        const T* w = W + (size_t)i * ldw + c0;
        const uint8_t* kp = keep + (size_t)i * k + c0;
        // salient part of this (row, block): Eq. 4
        double so = 0.0;
        int co = 0;
        for (int c = 0; c < STB_BLOCK; c++)
            if (kp[c] && sal_bit(sal_bitmap, c0 + c)) { so += std::fabs((double)w[c]); co++; }
        const uint16_t ao16 = f64_to_f16_bits(co > 0 ? so / (double)co : 0.0);
        const double ao = (double)f16_bits_to_f32(ao16);
        double sr = 0.0;
        for (int c = 0; c < STB_BLOCK; c++)
            if (kp[c] && sal_bit(sal_bitmap, c0 + c)) {
                const double sg = w[c] >= (T)0 ? 1.0 : -1.0;
                const double r = (double)w[c] - ao * sg;
                sr += std::fabs(r);
                tpos[(size_t)i * k + c0 + c] = r >= 0.0 ? 1 : 0;
            }
        scales[((size_t)i * nb + q) * 4 + 3] = ao16;
        res_scale[(size_t)i * nb + q] = f64_to_f16_bits(co > 0 ? sr / (double)co : 0.0);
        // non-salient kept magnitudes
        s.start[i] = (int32_t)s.a.size();
        for (int c = 0; c < STB_BLOCK; c++)
            if (kp[c] && !sal_bit(sal_bitmap, c0 + c)) {
                const double a = std::fabs((double)w[c]);
                s.a.push_back(a);
                s.col.push_back((uint8_t)c);
                if (a > mx) mx = a;
            }
    }
    s.start[n] = (int32_t)s.a.size();

    double p1 = 0.0, p2 = 0.0;
    if (cfg.region_mode == 0) {
        // Alg. 2 NonSalientAwareQuant: 160 candidates c_t = 0.1 + t*(0.8/159), p2 = 2*p1,
        // skipped when p2 > 0.9*max; first strict minimum wins
        const double step = (0.9 - 0.1) / 159.0;
        double best = std::numeric_limits<double>::infinity();
        // the candidates' errors are independent of each other: taken by `nt` threads, compared in order afterwards
        double err[160];
        parallel_for(160, nt, [&](int64_t t) {
            const double c = (t == 159) ? 0.9 : (double)t * step + 0.1;
            const double q1 = c * mx, q2 = 2.0 * q1;
            err[t] = q2 > 0.9 * mx ? std::numeric_limits<double>::infinity() : trisection_error(s, n, q1, q2);
        });
        for (int t = 0; t < 160; t++) {
            const double c = (t == 159) ? 0.9 : (double)t * step + 0.1;
            const double q1 = c * mx, q2 = 2.0 * q1;
            if (q2 > 0.9 * mx) continue;
            if (err[t] < best) { best = err[t]; p1 = q1; p2 = q2; }
        }
    } else {
        std::vector<double> sorted(s.a);
        std::sort(sorted.begin(), sorted.end());
        const size_t m = sorted.size();
        if (m > 0) {
            p1 = sorted[(m + 2) / 3 - 1];
            p2 = sorted[(2 * m + 2) / 3 - 1];
        }
    }
    for (int i = 0; i < n; i++) {
        const double* a = s.a.data() + s.start[i];
        const uint8_t* col = s.col.data() + s.start[i];
        const int cnt = s.start[i + 1] - s.start[i];
        double sum[3] = {0.0, 0.0, 0.0};
        int c3[3] = {0, 0, 0};
        for (int e = 0; e < cnt; e++) {
            const int r = a[e] > p2 ? 2 : (a[e] > p1 ? 1 : 0);
            sum[r] += a[e];
            c3[r]++;
            ids[(size_t)i * k + c0 + col[e]] = (uint8_t)r;
        }
        for (int r = 0; r < 3; r++)
            scales[((size_t)i * nb + q) * 4 + r] = f64_to_f16_bits(c3[r] > 0 ? sum[r] / (double)c3[r] : 0.0);
        const uint8_t* kp = keep + (size_t)i * k + c0;
        for (int c = 0; c < STB_BLOCK; c++)
            if (kp[c] && sal_bit(sal_bitmap, c0 + c)) ids[(size_t)i * k + c0 + c] = 3;
    }
}

// The bit planes, the salient bitmap and its per-block prefix from the per-weight decisions.  The sign plane takes
// the sign of W as it was when its block was quantised (row stride `ldw`).
template <class T>
int emit_planes(const T* W, size_t ldw, const stb_cfg_t& cfg, const uint8_t* keep, const uint8_t* ids, const uint8_t* tpos,
                const uint32_t* sal_bitmap, stb_layout_t* out, int nt) {
    const int n = cfg.n_out, k = cfg.k_in, nb = k / STB_BLOCK;
    const int slots = k * cfg.N / cfg.M;
    std::vector<int32_t> ordinal(k);   // index of column j among the salient columns
    {
        int u = 0;
        for (int j = 0; j < k; j++) { ordinal[j] = u; u += sal_bit(sal_bitmap, j); }
    }
    std::atomic<int> badrow(0);
    parallel_for(n, nt, [&](int64_t i) {
        uint8_t* mrow = (uint8_t*)out->mask + (size_t)i * out->mask_stride;
        uint8_t* srow = (uint8_t*)out->sign + (size_t)i * out->sign_stride;
        uint8_t* rrow = (uint8_t*)out->region + (size_t)i * out->region_stride;
        uint8_t* trow = cfg.n_salient ? (uint8_t*)out->res_sign + (size_t)i * out->res_stride : nullptr;
        std::memset(mrow, 0, out->mask_stride);
        std::memset(srow, 0, out->sign_stride);
        std::memset(rrow, 0, out->region_stride);
        if (trow) std::memset(trow, 0, out->res_stride);
        const T* w = W + (size_t)i * ldw;
        const uint8_t* kp = keep + (size_t)i * k;
        int slot = 0;
        for (int j = 0; j < k; j++) {
            if (!kp[j]) continue;
            mrow[j >> 3] |= (uint8_t)(1u << (j & 7));
            if (w[j] >= (T)0) srow[slot >> 3] |= (uint8_t)(1u << (slot & 7));
            const unsigned id = ids[(size_t)i * k + j];
            rrow[slot >> 2] |= (uint8_t)(id << ((slot & 3) * 2));
            if (id == 3 && tpos[(size_t)i * k + j]) {
                const int u = ordinal[j];
                trow[u >> 3] |= (uint8_t)(1u << (u & 7));
            }
            slot++;
        }
        if (slot != slots) badrow.store(1);
    });
    if (badrow.load()) return STB_EINVAL;
    std::memcpy(out->sal_bitmap, sal_bitmap, (size_t)k / 8);
    {
        uint32_t run = 0;
        for (int q = 0; q <= nb; q++) {
            out->sal_block_prefix[q] = run;
            if (q < nb)
                for (int c = 0; c < STB_BLOCK; c++) run += sal_bit(sal_bitmap, q * STB_BLOCK + c);
        }
    }
    return STB_OK;
}

}  // namespace

extern "C" int stb_pack(const float* W, const float* xnorm, const uint32_t* sal_bitmap, stb_layout_t* out,
                        int32_t n_threads) {
    if (!W || !xnorm || !sal_bitmap || !out) return STB_ENULL;
    int rc = stb_layout_check(out);
    if (rc) return rc;
    if (out->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    const stb_cfg_t cfg = out->cfg;
    const int n = cfg.n_out, k = cfg.k_in, N = cfg.N, M = cfg.M, nb = k / STB_BLOCK;
    int nt = n_threads > 0 ? n_threads : (int)std::thread::hardware_concurrency();
    if (nt < 1) nt = 1;

    // salient columns: count must match the configuration
    {
        int cnt = 0;
        for (int j = 0; j < k; j++) cnt += sal_bit(sal_bitmap, j);
        if (cnt != cfg.n_salient) return STB_EINVAL;
    }
    for (int j = 0; j < k; j++)
        if (!(xnorm[j] >= 0.0f) || !std::isfinite(xnorm[j])) return STB_ENONFINITE;

    // ---- Standardized Importance (Eq. 3): row sums, column sums of |W| ----
    std::vector<double> rs(n), cs(k, 0.0);
    std::atomic<int> bad(0);
    parallel_for(n, nt, [&](int64_t i) {
        const float* w = W + (size_t)i * k;
        double s = 0.0;
        for (int j = 0; j < k; j++) {
            if (!std::isfinite(w[j])) bad.store(1);
            s += std::fabs((double)w[j]);
        }
        rs[i] = s;
    });
    if (bad.load()) return STB_ENONFINITE;
    {
        // column sums must add rows in ascending order: split the columns over the threads
        const int chunks = std::min(nt, std::max(1, k / 256));
        parallel_for(chunks, nt, [&](int64_t c) {
            const int j0 = (int)((int64_t)k * c / chunks), j1 = (int)((int64_t)k * (c + 1) / chunks);
            for (int i = 0; i < n; i++) {
                const float* w = W + (size_t)i * k;
                for (int j = j0; j < j1; j++) cs[j] += std::fabs((double)w[j]);
            }
        });
    }
    auto mu_at = [&](int i, int j) -> double {
        const double a = std::fabs((double)W[(size_t)i * k + j]);
        const double t1 = rs[i] > 0.0 ? a / rs[i] : 0.0;
        const double t2 = cs[j] > 0.0 ? a / cs[j] : 0.0;
        return t1 + t2;
    };
    std::vector<double> rowacc(n);
    parallel_for(n, nt, [&](int64_t i) {
        double s = 0.0;
        for (int j = 0; j < k; j++) s += mu_at((int)i, j);
        rowacc[i] = s;
    });
    double tot = 0.0;
    for (int i = 0; i < n; i++) tot += rowacc[i];
    const double mean = tot / ((double)n * (double)k);
    parallel_for(n, nt, [&](int64_t i) {
        double s = 0.0;
        for (int j = 0; j < k; j++) {
            const double d = mu_at((int)i, j) - mean;
            s += d * d;
        }
        rowacc[i] = s;
    });
    tot = 0.0;
    for (int i = 0; i < n; i++) tot += rowacc[i];
    double sd = std::sqrt(tot / ((double)n * (double)k));
    if (sd == 0.0) sd = 1.0;

    // ---- N:M mask: the N highest scores of each group, equal scores keep the lower column ----
    std::vector<uint8_t> keep((size_t)n * k);       // 0 / 1 per weight
    parallel_for(n, nt, [&](int64_t i) {
        uint8_t* kp = keep.data() + (size_t)i * k;
        double sc[8];
        for (int g = 0; g < k / M; g++) {
            for (int p = 0; p < M; p++) {
                const int j = g * M + p;
                sc[p] = ((mu_at((int)i, j) - mean) / sd) * (double)xnorm[j];
                kp[j] = 0;
            }
            for (int p = 0; p < M; p++) {
                int better = 0;   // entries that rank before p
                for (int o = 0; o < M; o++)
                    if (sc[o] > sc[p] || (sc[o] == sc[p] && o < p)) better++;
                if (better < N) kp[g * M + p] = 1;
            }
        }
    });

    // ---- per block: salient residual binarisation, break points, region ids, scales ----
    std::vector<uint8_t> ids((size_t)n * k, 0);      // group id of each kept weight
    std::vector<uint8_t> tpos((size_t)n * k, 0);     // residual sign is +1 (kept salient weights)
    uint16_t* scales = out->scales;
    uint16_t* res_scale = out->res_scale;
    parallel_for(nb, nt, [&](int64_t q) {
        quantise_block(W, (size_t)k, (int)q, cfg, keep.data(), sal_bitmap, ids.data(), tpos.data(), scales, res_scale, 1);
    });

    return emit_planes(W, (size_t)k, cfg, keep.data(), ids.data(), tpos.data(), sal_bitmap, out, nt);
}

// ------------------------------------------------------------------------------------------------
// packer with the block loop of Alg. 1: Standardized Importance per 128-column slice and block-wise error
// compensation of the later columns
// ------------------------------------------------------------------------------------------------
// ------------------------------------------------------------------------------------------------
// H^c of Alg. 1 from calibration activations: H = 2 X^T X, H^c = upper Cholesky factor of (H + lambda I)^-1.
// With H + lambda I = R R^T, R upper triangular (the factorisation that starts at the last column), the inverse is
// R^-T R^-1, so H^c = R^-1: one factorisation and one triangular inverse, both in place in the output array.
// Every entry is one thread's float64 sum in a fixed order (dot4 below): the result does not depend on n_threads.
// ------------------------------------------------------------------------------------------------
namespace {
// sum_t a[t] * b[t] over [0, n) as four interleaved partial sums (t mod 4), added ((s0 + s1) + (s2 + s3)) and then
// the tail in order: a fixed order, and four independent addition chains for the processor.
inline double dot4(const double* a, const double* b, int64_t n) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int64_t t = 0;
    for (; t + 4 <= n; t += 4) {
        s0 += a[t] * b[t];
        s1 += a[t + 1] * b[t + 1];
        s2 += a[t + 2] * b[t + 2];
        s3 += a[t + 3] * b[t + 3];
    }
    double s = (s0 + s1) + (s2 + s3);
    for (; t < n; t++) s += a[t] * b[t];
    return s;
}
}  // namespace

extern "C" int stb_hessian_factor(const float* X, int32_t r, int32_t k, double lambda, double* Hc, float* xnorm,
                                  int32_t n_threads) {
    if (!X || !Hc) return STB_ENULL;
    if (r < 1 || k < 1 || !(lambda >= 0.0) || !std::isfinite(lambda)) return STB_EINVAL;
    const int nt = n_threads > 0 ? n_threads : (int)std::thread::hardware_concurrency();
    const int64_t K = k;
    std::atomic<bool> bad(false);
    // upper triangle of H + lambda I (sums over the samples in ascending order); zeros below the diagonal.
    // (X is transposed first so that a feature's samples are contiguous: k * r doubles of scratch.)
    std::vector<double> Xt((size_t)K * (size_t)r);
    parallel_for(K, nt, [&](int64_t i) {
        double* dst = Xt.data() + (size_t)i * r;
        for (int64_t t = 0; t < r; t++) dst[t] = (double)X[t * K + i];
    });
    parallel_for(K, nt, [&](int64_t i) {
        double* row = Hc + i * K;
        const double* xi = Xt.data() + (size_t)i * r;
        for (int64_t j = 0; j < i; j++) row[j] = 0.0;
        for (int64_t j = i; j < K; j++) {
            const double* xj = Xt.data() + (size_t)j * r;
            const double s = dot4(xi, xj, r);
            row[j] = 2.0 * s + (i == j ? lambda : 0.0);
            if (!std::isfinite(row[j])) bad.store(true);
            if (i == j && xnorm) xnorm[i] = (float)std::sqrt(s);
        }
    });
    std::vector<double>().swap(Xt);
    if (bad.load()) return STB_ENONFINITE;
    // R R^T = H, from the last column to the first: R[j][j] = sqrt(H[j][j] - sum_{m>j} R[j][m]^2),
    // R[i][j] = (H[i][j] - sum_{m>j} R[i][m] R[j][m]) / R[j][j] for i < j.  Columns are taken in panels of NB: the
    // panel's own rows first (one thread), then every row above the panel on its own (row i needs rows j of the
    // panel, which are final by then, and its own entries right of j).
    const int64_t NB = 32, CH = 16;                        // panel width, rows per task
    std::vector<double> piv((size_t)NB);
    for (int64_t j1 = K; j1 > 0; j1 -= NB) {
        const int64_t j0 = std::max<int64_t>(0, j1 - NB);
        for (int64_t j = j1 - 1; j >= j0; j--) {
            double* rj = Hc + j * K;
            const double d = rj[j] - dot4(rj + j + 1, rj + j + 1, K - j - 1);
            if (!(d > 0.0) || !std::isfinite(d)) return STB_ENONFINITE;      // not positive definite in floating point
            const double pv = std::sqrt(d);
            piv[(size_t)(j - j0)] = pv;
            rj[j] = pv;
            for (int64_t i = j0; i < j; i++) {
                double* ri = Hc + i * K;
                ri[j] = (ri[j] - dot4(ri + j + 1, rj + j + 1, K - j - 1)) / pv;
            }
        }
        const int64_t tasks = (j0 + CH - 1) / CH;
        parallel_for(tasks, nt, [&](int64_t c) {
            const int64_t hi = std::min<int64_t>(j0, (c + 1) * CH);
            for (int64_t i = c * CH; i < hi; i++) {
                double* ri = Hc + i * K;
                for (int64_t j = j1 - 1; j >= j0; j--)
                    ri[j] = (ri[j] - dot4(ri + j + 1, Hc + j * K + j + 1, K - j - 1)) / piv[(size_t)(j - j0)];
            }
        });
    }
    // U = R^-1 in place, panel after panel from the left: U[j][j] = 1 / R[j][j],
    // U[i][j] = -(sum_{m=i}^{j-1} U[i][m] R[m][j]) U[j][j] for i < j.  The panel's columns of R are copied out, its
    // diagonal is set, then every row is on its own (entries left of j in the row are final or made just before).
    std::vector<double> cols((size_t)NB * (size_t)K), ujj((size_t)NB);
    for (int64_t j0 = 0; j0 < K; j0 += NB) {
        const int64_t j1 = std::min<int64_t>(K, j0 + NB);
        for (int64_t j = j0; j < j1; j++) {
            double* col = cols.data() + (size_t)(j - j0) * K;
            for (int64_t m = 0; m <= j; m++) col[m] = Hc[m * K + j];
            ujj[(size_t)(j - j0)] = 1.0 / col[j];
        }
        for (int64_t j = j0; j < j1; j++) Hc[j * K + j] = ujj[(size_t)(j - j0)];
        const int64_t tasks = (j1 - 1 + CH - 1) / CH;
        parallel_for(tasks, nt, [&](int64_t c) {
            const int64_t hi = std::min<int64_t>(j1 - 1, (c + 1) * CH);
            for (int64_t i = c * CH; i < hi; i++) {
                double* ui = Hc + i * K;
                for (int64_t j = std::max<int64_t>(j0, i + 1); j < j1; j++)
                    ui[j] = -dot4(ui + i, cols.data() + (size_t)(j - j0) * K + i, j - i) * ujj[(size_t)(j - j0)];
            }
        });
    }
    for (int64_t i = 0; i < K; i++)
        if (!std::isfinite(Hc[i * K + i])) return STB_ENONFINITE;
    return STB_OK;
}

// The block loop of Alg. 1.  `accel` == nullptr: everything on the host.  Otherwise the float64 working copy that
// receives the compensation lives with the accelerator (a GPU): `start` hands it the initial copy, `fetch` brings the
// current values of a block's 128 columns back into the host copy before the block is quantised, `update` takes the
// block's error matrix E (n x 128, row-major) and applies W[:, later] -= E . H^c[block, later] there.  The arithmetic
// of `update` is fixed (see below), so both ways give the same bytes.
extern "C" int stb_pack_obc_with(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                                 stb_layout_t* out, int32_t n_threads, const stb_obc_accel_t* accel) {
    if (!W || !xnorm || !sal_bitmap || !out) return STB_ENULL;
    int rc = stb_layout_check(out);
    if (rc) return rc;
    if (out->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    const stb_cfg_t cfg = out->cfg;
    const int n = cfg.n_out, k = cfg.k_in, N = cfg.N, M = cfg.M, nb = k / STB_BLOCK;
    int nt = n_threads > 0 ? n_threads : (int)std::thread::hardware_concurrency();
    if (nt < 1) nt = 1;
    {
        int cnt = 0;
        for (int j = 0; j < k; j++) cnt += sal_bit(sal_bitmap, j);
        if (cnt != cfg.n_salient) return STB_EINVAL;
    }
    for (int j = 0; j < k; j++)
        if (!(xnorm[j] >= 0.0f) || !std::isfinite(xnorm[j])) return STB_ENONFINITE;
    if (Hc)
        for (int j = 0; j < k; j++) {
            const double d = Hc[(size_t)j * k + j];
            if (!std::isfinite(d) || d == 0.0) return STB_ENONFINITE;
        }

    // float64 working copy: columns right of the current block receive the compensation
    std::vector<double> Wd((size_t)n * k);
    std::atomic<int> bad(0);
    parallel_for(n, nt, [&](int64_t i) {
        for (int j = 0; j < k; j++) {
            const float v = W[(size_t)i * k + j];
            if (!std::isfinite(v)) bad.store(1);
            Wd[(size_t)i * k + j] = (double)v;
        }
    });
    if (bad.load()) return STB_ENONFINITE;
    if (accel && Hc) {
        rc = accel->start(accel->ctx, Wd.data());
        if (rc) return rc;
    }

    std::vector<uint8_t> keep((size_t)n * k), ids((size_t)n * k, 0), tpos((size_t)n * k, 0);
    std::vector<double> rs(n), rowacc(n), cs(STB_BLOCK), E(Hc ? (size_t)n * STB_BLOCK : 0);
    uint16_t* scales = out->scales;
    uint16_t* res_scale = out->res_scale;
    const double cnt = (double)n * (double)STB_BLOCK;

    for (int q = 0; q < nb; q++) {
        const int c0 = q * STB_BLOCK, c1 = c0 + STB_BLOCK;
        if (accel && Hc && q > 0) {
            rc = accel->fetch(accel->ctx, q, Wd.data());
            if (rc) return rc;
        }
        // ---- Standardized Importance over the slice (Eq. 3 with the sums, mean and deviation of the slice) ----
        parallel_for(n, nt, [&](int64_t i) {
            const double* w = Wd.data() + (size_t)i * k + c0;
            double s = 0.0;
            for (int c = 0; c < STB_BLOCK; c++) s += std::fabs(w[c]);
            rs[i] = s;
        });
        parallel_for(8, nt, [&](int64_t part) {         // column sums add the rows in ascending order
            for (int c = (int)part * 16; c < (int)part * 16 + 16; c++) cs[c] = 0.0;
            for (int i = 0; i < n; i++) {
                const double* w = Wd.data() + (size_t)i * k + c0;
                for (int c = (int)part * 16; c < (int)part * 16 + 16; c++) cs[c] += std::fabs(w[c]);
            }
        });
        auto mu_at = [&](int i, int c) -> double {
            const double a = std::fabs(Wd[(size_t)i * k + c0 + c]);
            const double t1 = rs[i] > 0.0 ? a / rs[i] : 0.0;
            const double t2 = cs[c] > 0.0 ? a / cs[c] : 0.0;
            return t1 + t2;
        };
        parallel_for(n, nt, [&](int64_t i) {
            double s = 0.0;
            for (int c = 0; c < STB_BLOCK; c++) s += mu_at((int)i, c);
            rowacc[i] = s;
        });
        double tot = 0.0;
        for (int i = 0; i < n; i++) tot += rowacc[i];
        const double mean = tot / cnt;
        parallel_for(n, nt, [&](int64_t i) {
            double s = 0.0;
            for (int c = 0; c < STB_BLOCK; c++) {
                const double d = mu_at((int)i, c) - mean;
                s += d * d;
            }
            rowacc[i] = s;
        });
        tot = 0.0;
        for (int i = 0; i < n; i++) tot += rowacc[i];
        double sd = std::sqrt(tot / cnt);
        if (sd == 0.0) sd = 1.0;
        parallel_for(n, nt, [&](int64_t i) {
            uint8_t* kp = keep.data() + (size_t)i * k + c0;
            double sc[8];
            for (int g = 0; g < STB_BLOCK / M; g++) {
                for (int p = 0; p < M; p++) {
                    sc[p] = ((mu_at((int)i, g * M + p) - mean) / sd) * (double)xnorm[c0 + g * M + p];
                    kp[g * M + p] = 0;
                }
                for (int p = 0; p < M; p++) {
                    int better = 0;
                    for (int o = 0; o < M; o++)
                        if (sc[o] > sc[p] || (sc[o] == sc[p] && o < p)) better++;
                    if (better < N) kp[g * M + p] = 1;
                }
            }
        });

        quantise_block(Wd.data(), (size_t)k, q, cfg, keep.data(), sal_bitmap, ids.data(), tpos.data(), scales, res_scale, nt);

        if (!Hc || c1 >= k) continue;
        // ---- E = (W_block - B) / diag(H^c): B is the block as inference sees it (fp16 scales, one fp32 addition) ----
        parallel_for(n, nt, [&](int64_t i) {
            const double* w = Wd.data() + (size_t)i * k + c0;
            const uint8_t* kp = keep.data() + (size_t)i * k + c0;
            float sc4[4];
            for (int r = 0; r < 4; r++) sc4[r] = f16_bits_to_f32(scales[((size_t)i * nb + q) * 4 + r]);
            const float ar = f16_bits_to_f32(res_scale[(size_t)i * nb + q]);
            for (int c = 0; c < STB_BLOCK; c++) {
                float b = 0.0f;
                if (kp[c]) {
                    const unsigned id = ids[(size_t)i * k + c0 + c];
                    b = w[c] >= 0.0 ? sc4[id] : -sc4[id];
                    if (id == 3) b = b + (tpos[(size_t)i * k + c0 + c] ? ar : -ar);
                }
                E[(size_t)i * STB_BLOCK + c] = (w[c] - (double)b) / Hc[(size_t)(c0 + c) * k + c0 + c];
            }
        });
        // ---- W[:, later] -= E . H^c[block, later]: per output the block's 128 terms in ascending order ----
        if (accel) {
            rc = accel->update(accel->ctx, q, E.data());
            if (rc) return rc;
            continue;
        }
        const int TJ = 256;
        const int tiles = (k - c1 + TJ - 1) / TJ;
        parallel_for(tiles, nt, [&](int64_t t) {
            const int j0 = c1 + (int)t * TJ, jn = std::min(TJ, k - j0);
            double acc[TJ];
            for (int i = 0; i < n; i++) {
                const double* e = E.data() + (size_t)i * STB_BLOCK;
                for (int j = 0; j < jn; j++) acc[j] = 0.0;
                for (int c = 0; c < STB_BLOCK; c++) {
                    const double ec = e[c];
                    const double* h = Hc + (size_t)(c0 + c) * k + j0;
                    for (int j = 0; j < jn; j++) acc[j] += ec * h[j];
                }
                double* w = Wd.data() + (size_t)i * k + j0;
                for (int j = 0; j < jn; j++) w[j] -= acc[j];
            }
        });
    }
    return emit_planes(Wd.data(), (size_t)k, cfg, keep.data(), ids.data(), tpos.data(), sal_bitmap, out, nt);
}

extern "C" int stb_pack_obc(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                            stb_layout_t* out, int32_t n_threads) {
    return stb_pack_obc_with(W, Hc, xnorm, sal_bitmap, out, n_threads, nullptr);
}

// ------------------------------------------------------------------------------------------------
// host dequantiser
// ------------------------------------------------------------------------------------------------
extern "C" int stb_unpack(const stb_layout_t* L, float* W_hat) {
    if (!W_hat) return STB_ENULL;
    int rc = stb_layout_check(L);
    if (rc) return rc;
    if (L->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    const int n = L->cfg.n_out, k = L->cfg.k_in, nb = k / STB_BLOCK;
    const int slots = k * L->cfg.N / L->cfg.M;
    std::vector<int32_t> ordinal(k);
    {
        int u = 0;
        for (int j = 0; j < k; j++) { ordinal[j] = u; u += sal_bit(L->sal_bitmap, j); }
    }
    for (int i = 0; i < n; i++) {
        const uint8_t* mrow = (const uint8_t*)L->mask + (size_t)i * L->mask_stride;
        const uint8_t* srow = (const uint8_t*)L->sign + (size_t)i * L->sign_stride;
        const uint8_t* rrow = (const uint8_t*)L->region + (size_t)i * L->region_stride;
        const uint8_t* trow = L->cfg.n_salient ? (const uint8_t*)L->res_sign + (size_t)i * L->res_stride : nullptr;
        float* o = W_hat + (size_t)i * k;
        int slot = 0;
        for (int j = 0; j < k; j++) {
            if (!((mrow[j >> 3] >> (j & 7)) & 1)) { o[j] = 0.0f; continue; }
            if (slot >= slots) return STB_EINVAL;
            const float s = ((srow[slot >> 3] >> (slot & 7)) & 1) ? 1.0f : -1.0f;
            const unsigned id = (rrow[slot >> 2] >> ((slot & 3) * 2)) & 3u;
            const int q = j / STB_BLOCK;
            const float a = f16_bits_to_f32(L->scales[((size_t)i * nb + q) * 4 + id]);
            if (id == 3) {
                if (!trow) return STB_EINVAL;
                const int u = ordinal[j];
                const float t = ((trow[u >> 3] >> (u & 7)) & 1) ? 1.0f : -1.0f;
                const float ar = f16_bits_to_f32(L->res_scale[(size_t)i * nb + q]);
                o[j] = s * a + t * ar;
            } else {
                o[j] = s * a;
            }
            slot++;
        }
        if (slot != slots) return STB_EINVAL;
    }
    return STB_OK;
}

// ------------------------------------------------------------------------------------------------
// Layer-wise N:M assignment (Sec. 3.3): alpha_i = omega_i / sum omega, N_i / M = alpha_i + (1 - alpha_i) R_target.
// ------------------------------------------------------------------------------------------------
extern "C" int stb_layer_l2_norm(const float* W, int64_t count, double* omega) {
    if (!W || !omega) return STB_ENULL;
    if (count < 0) return STB_EINVAL;
    double s = 0.0;
    for (int64_t q = 0; q < count; q++) {
        const double v = (double)W[q];
        if (!std::isfinite(v)) return STB_ENONFINITE;
        s += v * v;
    }
    *omega = std::sqrt(s);
    return STB_OK;
}

extern "C" int stb_layer_nm_assignment(const double* omega, int32_t n_layers, double r_target, int32_t M, int32_t* N_out) {
    if (!omega || !N_out) return STB_ENULL;
    if (n_layers < 1 || M < 1 || !(r_target >= 0.0 && r_target <= 1.0)) return STB_EINVAL;
    double total = 0.0;
    for (int i = 0; i < n_layers; i++) {
        if (!std::isfinite(omega[i]) || omega[i] < 0.0) return STB_ENONFINITE;
        total += omega[i];
    }
    for (int i = 0; i < n_layers; i++) {
        const double alpha = total > 0.0 ? omega[i] / total : 1.0 / (double)n_layers;
        const double ratio = alpha + (1.0 - alpha) * r_target;
        double nn = std::floor((double)M * ratio + 0.5);
        if (nn < 1.0) nn = 1.0;
        if (nn > (double)M) nn = (double)M;
        N_out[i] = (int32_t)nn;
    }
    return STB_OK;
}

// ------------------------------------------------------------------------------------------------
// Salient columns (Alg. 2 "Salient"), block by block, on the diagonal of the Hessian of Alg. 1:
// S_ij = w_ij^2 (2 xnorm_j^2 + lambda); candidates = the columns with the largest column sums of S; the number
// kept is the one whose two-group binarisation (Eq. 1, per row over each group) has the smallest squared error.
// All sums are float64, sequential in ascending index, so that the result is reproducible bit for bit.
// ------------------------------------------------------------------------------------------------
namespace {
// Salient() of Alg. 2 after the salient matrix: S_ij = w_ij^2 * f_j (divide == false) or w_ij^2 / f_j (divide == true).
int salient_select(const float* W, int n, int k, const double* f, bool divide, int max_per_block, uint32_t* sal_bitmap,
                   int32_t* n_selected) {
    for (size_t q = 0; q < (size_t)n * k; q++)
        if (!std::isfinite(W[q])) return STB_ENONFINITE;
    std::memset(sal_bitmap, 0, (size_t)k / 32 * sizeof(uint32_t));
    int total = 0;
    std::vector<double> score(STB_BLOCK);
    std::vector<int> order(STB_BLOCK);
    std::vector<char> sal(STB_BLOCK);
    for (int b = 0; b < k; b += STB_BLOCK) {
        const double* h = f + b;
        for (int j = 0; j < STB_BLOCK; j++) score[j] = 0.0;
        for (int i = 0; i < n; i++) {
            const float* w = W + (size_t)i * k + b;
            for (int j = 0; j < STB_BLOCK; j++) {
                const double v = (double)w[j];
                score[j] += divide ? (v * v) / h[j] : (v * v) * h[j];
            }
        }
        for (int j = 0; j < STB_BLOCK; j++) order[j] = j;
        std::stable_sort(order.begin(), order.end(), [&](int a, int c) { return score[a] > score[c]; });
        double best = std::numeric_limits<double>::infinity();
        int n_star = 0;
        std::fill(sal.begin(), sal.end(), 0);
        for (int c = 1; c <= max_per_block; c++) {
            sal[order[c - 1]] = 1;
            double e = 0.0;
            for (int i = 0; i < n; i++) {
                const float* w = W + (size_t)i * k + b;
                double s1 = 0.0, s2 = 0.0;
                for (int j = 0; j < STB_BLOCK; j++) {
                    const double a = std::fabs((double)w[j]);
                    if (sal[j]) s1 += a; else s2 += a;
                }
                const double a1 = s1 / (double)c;
                const double a2 = c < STB_BLOCK ? s2 / (double)(STB_BLOCK - c) : 0.0;
                double er = 0.0;
                for (int j = 0; j < STB_BLOCK; j++) {
                    const double v = (double)w[j];
                    const double bq = (sal[j] ? a1 : a2) * (v >= 0.0 ? 1.0 : -1.0);
                    er += (v - bq) * (v - bq);
                }
                e += er;
            }
            if (e < best) { best = e; n_star = c; }
        }
        for (int c = 0; c < n_star; c++) {
            const int j = b + order[c];
            sal_bitmap[j >> 5] |= 1u << (j & 31);
        }
        total += n_star;
    }
    if (n_selected) *n_selected = total;
    return STB_OK;
}
}  // namespace

extern "C" int stb_salient_columns(const float* W, int32_t n, int32_t k, const float* xnorm, double lambda,
                                   int32_t max_per_block, uint32_t* sal_bitmap, int32_t* n_selected) {
    if (!W || !xnorm || !sal_bitmap) return STB_ENULL;
    if (n < 1 || k < STB_BLOCK || k % STB_BLOCK || max_per_block < 0 || max_per_block > STB_BLOCK) return STB_EINVAL;
    if (!(lambda >= 0.0) || !std::isfinite(lambda)) return STB_EINVAL;
    for (int j = 0; j < k; j++)
        if (!(xnorm[j] >= 0.0f) || !std::isfinite(xnorm[j])) return STB_ENONFINITE;
    std::vector<double> f((size_t)k);
    for (int j = 0; j < k; j++) {
        const double x = (double)xnorm[j];
        f[(size_t)j] = 2.0 * x * x + lambda;
    }
    return salient_select(W, n, k, f.data(), false, max_per_block, sal_bitmap, n_selected);
}

extern "C" int stb_salient_columns_hc(const float* W, int32_t n, int32_t k, const double* Hc, int32_t max_per_block,
                                      uint32_t* sal_bitmap, int32_t* n_selected) {
    if (!W || !Hc || !sal_bitmap) return STB_ENULL;
    if (n < 1 || k < STB_BLOCK || k % STB_BLOCK || max_per_block < 0 || max_per_block > STB_BLOCK) return STB_EINVAL;
    std::vector<double> f((size_t)k);
    for (int j = 0; j < k; j++) {
        const double d = Hc[(size_t)j * k + j];
        if (!std::isfinite(d) || d == 0.0) return STB_ENONFINITE;
        f[(size_t)j] = d * d;
    }
    return salient_select(W, n, k, f.data(), true, max_per_block, sal_bitmap, n_selected);
}

// ------------------------------------------------------------------------------------------------
// The 2:4 group code of App. C: a 16-bit meta index per four groups of four columns (which two of the four
// are kept) and a byte of eight sign bits (1 -> +1) for the same 16 columns: six bits per group.
// ------------------------------------------------------------------------------------------------
namespace {
int code24_shape_ok(const stb_layout_t* L) {
    int rc = stb_layout_check(L);
    if (rc) return rc;
    if (L->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    if (L->cfg.N != 2 || L->cfg.M != 4) return STB_EUNSUPPORTED;
    return STB_OK;
}
}  // namespace

extern "C" int stb_code24_export(const stb_layout_t* L, uint16_t* E, uint8_t* V) {
    if (!E || !V) return STB_ENULL;
    int rc = code24_shape_ok(L);
    if (rc) return rc;
    const int n = L->cfg.n_out, k16 = L->cfg.k_in / 16;
    for (int i = 0; i < n; i++) {
        const uint8_t* mrow = (const uint8_t*)L->mask + (size_t)i * L->mask_stride;
        const uint8_t* srow = (const uint8_t*)L->sign + (size_t)i * L->sign_stride;
        for (int c = 0; c < k16; c++) {
            const unsigned m16 = mrow[2 * c] | ((unsigned)mrow[2 * c + 1] << 8);
            unsigned e = 0;
            for (int g = 0; g < 4; g++) {
                const unsigned nib = (m16 >> (4 * g)) & 15u;
                int pos[2], cnt = 0;
                for (int j = 0; j < 4; j++)
                    if ((nib >> j) & 1u) { if (cnt < 2) pos[cnt] = j; cnt++; }
                if (cnt != 2) return STB_EINVAL;
                e |= (unsigned)(pos[0] | (pos[1] << 2)) << (4 * g);
            }
            E[(size_t)i * k16 + c] = (uint16_t)e;
            V[(size_t)i * k16 + c] = srow[c];
        }
    }
    return STB_OK;
}

extern "C" int stb_code24_import(stb_layout_t* L, const uint16_t* E, const uint8_t* V) {
    if (!E || !V) return STB_ENULL;
    int rc = code24_shape_ok(L);
    if (rc) return rc;
    const int n = L->cfg.n_out, k16 = L->cfg.k_in / 16;
    for (size_t q = 0; q < (size_t)n * k16; q++)
        for (int g = 0; g < 4; g++) {
            const unsigned nib = (E[q] >> (4 * g)) & 15u;
            if ((nib & 3u) >= (nib >> 2)) return STB_EINVAL;      // two different positions, lower one first
        }
    for (int i = 0; i < n; i++) {
        uint8_t* mrow = (uint8_t*)L->mask + (size_t)i * L->mask_stride;
        uint8_t* srow = (uint8_t*)L->sign + (size_t)i * L->sign_stride;
        std::memset(mrow, 0, (size_t)L->mask_stride);
        std::memset(srow, 0, (size_t)L->sign_stride);
        for (int c = 0; c < k16; c++) {
            const unsigned e = E[(size_t)i * k16 + c];
            unsigned m16 = 0;
            for (int g = 0; g < 4; g++) {
                const unsigned nib = (e >> (4 * g)) & 15u;
                m16 |= ((1u << (nib & 3u)) | (1u << (nib >> 2))) << (4 * g);
            }
            mrow[2 * c] = (uint8_t)(m16 & 255u);
            mrow[2 * c + 1] = (uint8_t)(m16 >> 8);
            srow[c] = V[(size_t)i * k16 + c];
        }
    }
    return STB_OK;
}

extern "C" const char* stb_strerror(int status) {
    switch (status) {
        case STB_OK: return "ok";
        case STB_EINVAL: return "invalid configuration or argument";
        case STB_ENULL: return "required pointer is NULL";
        case STB_EALIGN: return "pointer is not sufficiently aligned";
        case STB_ENONFINITE: return "NaN/Inf in W or xnorm, or negative xnorm";
        case STB_EHIP: return "HIP call failed (see stb_last_hip_error)";
        case STB_EUNSUPPORTED: return "no kernel for this configuration";
        case STB_ETOOBIG: return "problem needs more scratch than the library's static device array holds";
        default: return "unknown status";
    }
}
