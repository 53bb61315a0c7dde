// Device-side building blocks shared by the kernels that read the tiled device order (STB_KIND_TILED).
//
// A tile is 16 output rows x 4 column blocks (512 columns): lane = 16*g + i owns (row i of the tile, block g of
// the superblock); its record holds that block's 16 mask bytes, its sign and id bits and its scales.  mask and
// id bytes (and sign bytes where they split into whole words) are stored half by half (64 columns), so that a
// wavefront working on one half of every block reads contiguous bytes.  A lane expands 8 columns at a time into
// the A operand (4 VGPRs of fp16) of v_mfma_f32_16x16x32_f16.  Expansion works on whole registers:
//   * ids -> byte selectors -> v_perm_b32 over the block's scale table gives two kept weights per register
//     in slot order (the order of the sign / id planes),
//   * sign bits are moved to bit 15 / 31 with one packed 16-bit shift and merged with one and-or,
//   * a 256-entry table in LDS, indexed by the mask byte, holds the four v_perm selectors that spread the
//     slot-ordered weights to their column positions (zero where the mask bit is clear).
// Stored sign bit 1 means +1 (Eq. 2 / App. C "1 -> +1, 0 -> -1"); the bit is copied into the fp16 sign bit
// as it is, so every expanded weight is the negative of W_hat and the consumer negates its accumulator.
// Salient columns (Eq. 4): alpha_o rides in the scale table as id 3; the residual term t*alpha_r is a second,
// short operand built per block from the table of salient columns (residual_chunk below).
#ifndef STB_TILED_HPP
#define STB_TILED_HPP
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "stb_internal.h"

namespace stbt {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef short short2_t __attribute__((ext_vector_type(2)));

struct TiledPlanes {
    const uint4* mask;          // [nrt][nsb][64] x 16 B
    const uint8_t* sign;        // [nrt][nsb][64] x sign_stride
    const uint8_t* region;      // [nrt][nsb][64] x region_stride
    const uint2* scales;        // [nrt][nsb][64] x 4 fp16
    const uint16_t* res_scale;  // [nrt][nsb][64]
    const uint32_t* res_sign;   // [nrt][res_words][16]
    const uint32_t* sal_bitmap; // [nsb*4][4]
    const uint32_t* sal_prefix; // [nsb*4 + 1]
    const uint32_t* sal_tab;    // [nsb*4][2][sal_chunks][12]
    int n, k, nb, nrt, nsb;
    int res_words;              // uint32 per row of res_sign (0 if no salient columns)
    int sal_chunks;
};

inline TiledPlanes make_tiled(const stb_layout_t* L) {
    TiledPlanes p;
    p.mask = (const uint4*)L->mask;
    p.sign = (const uint8_t*)L->sign;
    p.region = (const uint8_t*)L->region;
    p.scales = (const uint2*)L->scales;
    p.res_scale = (const uint16_t*)L->res_scale;
    p.res_sign = (const uint32_t*)L->res_sign;
    p.sal_bitmap = L->sal_bitmap;
    p.sal_prefix = L->sal_block_prefix;
    p.sal_tab = L->sal_tab;
    p.n = L->cfg.n_out;
    p.k = L->cfg.k_in;
    p.nb = L->n_blocks;
    p.nrt = L->n_row_tiles;
    p.nsb = L->n_super;
    p.res_words = (int)(L->res_stride / 4);
    p.sal_chunks = L->sal_chunks;
    return p;
}

__device__ inline uint32_t perm(uint32_t hi, uint32_t lo, uint32_t sel) {
    return __builtin_amdgcn_perm(hi, lo, sel);      // selector bytes 0-3 pick from lo, 4-7 from hi, 0x0C -> 0x00
}

__device__ inline uint32_t pk_shl(uint32_t v, unsigned lo, unsigned hi) {
    ushort2_t x = __builtin_bit_cast(ushort2_t, v);
    const ushort2_t s = {(unsigned short)lo, (unsigned short)hi};
    x = x << s;
    return __builtin_bit_cast(uint32_t, x);
}

// (a & b) | c in one instruction with all three operands in VGPRs (two constants cannot share the one
// constant-bus slot a VOP3 instruction has, so the compiler would otherwise split it in two).
__device__ inline uint32_t and_or(uint32_t a, uint32_t b, uint32_t c) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}

// (a & b) | c for operands of which at most one is a literal constant: the compiler picks v_and_or_b32 itself,
// and schedules it better than an asm statement (after which it also pads dependent instructions with s_nop).
__device__ inline uint32_t and_or_v(uint32_t a, uint32_t b, uint32_t c) { return (a & b) | c; }

// Low 16-bit products of the two halves (v_pk_mul_lo_u16).
__device__ inline uint32_t pk_mul_u16(uint32_t a, uint32_t b) {
    const ushort2_t r = __builtin_bit_cast(ushort2_t, a) * __builtin_bit_cast(ushort2_t, b);
    return __builtin_bit_cast(uint32_t, r);
}

// 32 bits of a little-endian bit string held in words w[], starting at bit `off` (compile-time constant
// after unrolling).  WORDS = number of valid words.
template <int WORDS>
__device__ inline uint32_t window32(const uint32_t* w, int off) {
    const int i = off >> 5, s = off & 31;
    if (s == 0) return w[i];
    if (i + 1 < WORDS) return __builtin_amdgcn_alignbit(w[i + 1], w[i], s);
    return w[i] >> s;
}

// ------------------------------------------------------------------------------------------------
// Scatter table: for mask byte mb, four v_perm selectors that place the slot-ordered weights of the
// 8-column group at their columns.  N8 = slots per 8 columns (4 for 2:4, 4:8 and 3:8; 6 for 6:8 and 5:8).
// Registers W0 = slots 0,1; W1 = slots 2,3; W2 = slots 4,5.  Selectors 0,1 address {W1:W0}; for N8 = 6
// selectors 2,3 address {W2:W1} (columns 4..7 can only hold slots 2..5), for N8 = 4 they address {W1:W0}.
// ------------------------------------------------------------------------------------------------
// A workgroup keeps the scatter table in LDS, eight times: entry mb of copy c sits at [mb][c], and lane l reads
// copy l % 8, so the eight lanes that an LDS cycle serves hit eight different groups of four banks whatever
// their mask bytes are.
struct ScatterLds {
    uint4 e[256][8];
};

template <int N8>
__device__ inline uint4 scatter_entry(uint32_t mb) {
    uint32_t sel[4];
#pragma unroll
    for (int v = 0; v < 4; v++) {
        uint32_t s = 0;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int pcol = 2 * v + h;
            uint32_t two = 0x0C0Cu;
            if ((mb >> pcol) & 1u) {
                // a group that keeps one column less than the table's N8 (3 of 8 with N8 = 4, 5 of 8 with N8 = 6) numbers
                // its slots as if its lowest pruned column were kept as well: that slot is padding in the planes
                const uint32_t aug = __popc(mb) == N8 - 1 ? (mb | (~mb & (mb + 1u))) : mb;
                int r = __popc(aug & ((1u << pcol) - 1u));
                if (N8 == 6 && v >= 2) r -= 2;
                r = r < 0 ? 0 : (r > 3 ? 3 : r);
                two = (uint32_t)(2 * r) | ((uint32_t)(2 * r + 1) << 8);
            }
            s |= two << (16 * h);
        }
        sel[v] = s;
    }
    return make_uint4(sel[0], sel[1], sel[2], sel[3]);
}

// Fills the table (any block size; a barrier must follow before it is read).
template <int N8>
__device__ inline void build_luts(ScatterLds* L) {
    for (int mb = threadIdx.x; mb < 256; mb += blockDim.x) {
        const uint4 v = scatter_entry<N8>((uint32_t)mb);
#pragma unroll
        for (int c = 0; c < 8; c++) L->e[mb][c] = v;
    }
}

// ------------------------------------------------------------------------------------------------
// Per-lane operands of one (row, half block): 64 columns = 8 groups of 8.  A wavefront that works on half h of
// its superblock reads, from each lane record, mask bytes 8h .. 8h+7, the sign bits of slots 8*N8*h ..
// (N8 = 4: one word; N8 = 6: a 64-bit window at byte 4h, shifted right by 16h), the id fields of the same
// slots (N8 = 4: two words; N8 = 6: three), the four scales and alpha_r.
// ------------------------------------------------------------------------------------------------
template <int N8>
struct HalfData {
    static constexpr int SW = N8 == 4 ? 1 : 2;   // sign words held
    static constexpr int RW = N8 == 4 ? 2 : 3;   // region words held
    uint32_t m[2];
    uint32_t s[2];
    uint32_t r[3];
    uint2 sc;                           // the four scales {dense, inter, sparse, alpha_o} as stored
    uint32_t ar;                        // alpha_r (fp16 bits)
    uint32_t rlo, rhi;                  // the two res_sign words of the row that hold the half's first bits
};

// Byte offsets of the lane's pieces inside one tile of each plane (lane = 16*g + i, half h).
struct LaneOffsets {
    uint32_t omask, osign, oregion, o8, o2;
    uint32_t ores0, ores1;     // byte offsets of the two res_sign words inside the row tile
};

template <int N8>
__device__ inline LaneOffsets lane_offsets(int lane, int half) {
    LaneOffsets lo;
    // mask, region (and sign for N8 = 4) are stored [tile][half][lane]: the 64 lanes of a half read contiguous bytes
    lo.omask = 512u * half + (uint32_t)lane * 8u;
    lo.osign = N8 == 4 ? 256u * half + (uint32_t)lane * 4u : (uint32_t)lane * 12u + 4u * half;
    lo.oregion = N8 == 4 ? 512u * half + (uint32_t)lane * 8u : 768u * half + (uint32_t)lane * 12u;
    lo.o8 = (uint32_t)lane * 8u;
    lo.o2 = (uint32_t)lane * 2u;
    lo.ores0 = 0u;
    lo.ores1 = 0u;
    return lo;
}

// Plain loads of one half record (verification kernel and prefill kernel).
template <int N8>
__device__ inline void load_half(const TiledPlanes& p, int64_t tile, const LaneOffsets& lo, int half, HalfData<N8>& d) {
    const char* bm = reinterpret_cast<const char*>(p.mask) + tile * (64 * 16);
    const char* bs = reinterpret_cast<const char*>(p.sign) + tile * (64 * 2 * N8);
    const char* br = reinterpret_cast<const char*>(p.region) + tile * (64 * 4 * N8);
    const uint2 m = *reinterpret_cast<const uint2*>(bm + lo.omask);
    d.m[0] = m.x; d.m[1] = m.y;
    if (N8 == 4) {
        d.s[0] = *reinterpret_cast<const uint32_t*>(bs + lo.osign); d.s[1] = 0u;
        const uint2 r = *reinterpret_cast<const uint2*>(br + lo.oregion);
        d.r[0] = r.x; d.r[1] = r.y; d.r[2] = 0u;
    } else {
        const uint32_t s0 = *reinterpret_cast<const uint32_t*>(bs + lo.osign);
        const uint32_t s1 = *reinterpret_cast<const uint32_t*>(bs + lo.osign + 4);
        d.s[0] = __builtin_amdgcn_alignbit(s1, s0, 16u * half);
        d.s[1] = s1 >> (16u * half);
        const uint32_t* rp = reinterpret_cast<const uint32_t*>(br + lo.oregion);
        d.r[0] = rp[0]; d.r[1] = rp[1]; d.r[2] = rp[2];
    }
    d.sc = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(p.scales) + tile * (64 * 8) + lo.o8);
    d.ar = *reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(p.res_scale) + tile * (64 * 2) + lo.o2);
    d.rlo = 0u; d.rhi = 0u;
}

// ------------------------------------------------------------------------------------------------
// Software-pipelined fetch of half records.  The loads are written as asm statements with the plane base
// in SGPRs and a 32-bit lane offset, and the matching wait names every destination register as a read-write
// operand: the loads of several tiles stay in flight exactly as written (the compiler neither moves them
// nor waits for them), and no register of a tile can be read before wait_tile has been executed on it.
// Rules for callers: every fetch is followed, on every path, by a wait_tile on the same object before the
// object dies; K = number of such loads issued after the last load of the tile.
// ------------------------------------------------------------------------------------------------
typedef uint32_t uint3_t __attribute__((ext_vector_type(3)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

template <int N8>
struct TileRegs;
template <>
struct TileRegs<4> {
    uint2_t m; uint32_t s; uint2_t r; uint2_t sc; uint32_t ar, rlo, rhi;
};
template <>
struct TileRegs<6> {
    uint2_t m; uint2_t s; uint3_t r; uint2_t sc; uint32_t ar, rlo, rhi;
};
template <bool HAS_RES>
struct TileLoads {
    static constexpr int count = 5 + (HAS_RES ? 2 : 0);
};

template <int N8>
__device__ inline void fetch_main(TileRegs<N8>& d, const TiledPlanes& p, int64_t tile, const LaneOffsets& lo) {
    const char* bm = reinterpret_cast<const char*>(p.mask) + tile * (64 * 16);
    const char* bs = reinterpret_cast<const char*>(p.sign) + tile * (64 * 2 * N8);
    const char* br = reinterpret_cast<const char*>(p.region) + tile * (64 * 4 * N8);
    const char* bc = reinterpret_cast<const char*>(p.scales) + tile * (64 * 8);
    const char* ba = reinterpret_cast<const char*>(p.res_scale) + tile * (64 * 2);
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(d.m) : "v"(lo.omask), "s"(bm));
    if constexpr (N8 == 4) {
        asm volatile("global_load_dword %0, %1, %2" : "=v"(d.s) : "v"(lo.osign), "s"(bs));
        asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(d.r) : "v"(lo.oregion), "s"(br));
    } else {
        asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(d.s) : "v"(lo.osign), "s"(bs));
        asm volatile("global_load_dwordx3 %0, %1, %2" : "=v"(d.r) : "v"(lo.oregion), "s"(br));
    }
    asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(d.sc) : "v"(lo.o8), "s"(bc));
    asm volatile("global_load_ushort %0, %1, %2" : "=v"(d.ar) : "v"(lo.o2), "s"(ba));
}

// The two res_sign words of the lane's row in row tile rt (lo.ores0 / lo.ores1 must be final).
template <int N8, bool HAS_RES>
__device__ inline void fetch_res(TileRegs<N8>& d, const TiledPlanes& p, int64_t rt, const LaneOffsets& lo) {
    if constexpr (HAS_RES) {
        const char* bres = reinterpret_cast<const char*>(p.res_sign) + rt * ((int64_t)p.res_words * 64);
        asm volatile("global_load_dword %0, %1, %2" : "=v"(d.rlo) : "v"(lo.ores0), "s"(bres));
        asm volatile("global_load_dword %0, %1, %2" : "=v"(d.rhi) : "v"(lo.ores1), "s"(bres));
    } else {
        d.rlo = 0u; d.rhi = 0u;
    }
}

template <int N8, bool HAS_RES>
__device__ inline void fetch_tile(TileRegs<N8>& d, const TiledPlanes& p, int64_t tile, int64_t rt,
                                  const LaneOffsets& lo) {
    fetch_main<N8>(d, p, tile, lo);
    fetch_res<N8, HAS_RES>(d, p, rt, lo);
}

// Waits until at most K of the loads above are outstanding and hands the tile's registers over.
template <int K, int N8>
__device__ inline void wait_tile(TileRegs<N8>& d) {
    asm volatile("s_waitcnt vmcnt(%7)" : "+v"(d.m), "+v"(d.s), "+v"(d.r), "+v"(d.sc), "+v"(d.ar), "+v"(d.rlo), "+v"(d.rhi) : "n"(K));
}

template <int N8>
__device__ inline void unpack_tile(const TileRegs<N8>& t, int half, HalfData<N8>& d) {
    d.m[0] = t.m[0]; d.m[1] = t.m[1];
    if constexpr (N8 == 4) {
        d.s[0] = t.s; d.s[1] = 0u;
        d.r[0] = t.r[0]; d.r[1] = t.r[1]; d.r[2] = 0u;
    } else {
        d.s[0] = __builtin_amdgcn_alignbit(t.s[1], t.s[0], 16u * half);
        d.s[1] = t.s[1] >> (16u * half);
        d.r[0] = t.r[0]; d.r[1] = t.r[1]; d.r[2] = t.r[2];
    }
    d.sc = make_uint2(t.sc[0], t.sc[1]);
    d.ar = t.ar & 0xFFFFu;
    d.rlo = t.rlo; d.rhi = t.rhi;
}

// Scatter selectors of group t (issued ahead of the arithmetic that uses them).
template <int N8>
__device__ inline uint4 lut_fetch(const HalfData<N8>& d, int t, const ScatterLds* L, int copy) {
    const uint32_t mb = (d.m[t >> 2] >> (8 * (t & 3))) & 0xFFu;
    return L->e[mb][copy];
}

// Expands columns 8t .. 8t+7 (t < 8) of the lane's half block into four registers of fp16 pairs (negated
// weights).  TL / TH = low / high bytes of the four scales; L = the group's scatter selectors.
template <int N8>
__device__ inline void expand_group(const HalfData<N8>& d, uint32_t TL, uint32_t TH, int t, const uint4& L,
                                    uint32_t out[4]) {
    uint32_t W[3];
    if (N8 == 4) {
        const uint32_t rw = d.r[t >> 2], r2 = rw >> 2;
        const uint32_t b = t & 3;
        const uint32_t Z = perm(r2, rw, b | (b << 8) | ((4 + b) << 16) | ((4 + b) << 24));
        const uint32_t sel0 = and_or(Z, 0x03030303u, 0x04000400u);
        const uint32_t sel1 = and_or(Z >> 4, 0x03030303u, 0x04000400u);
        W[0] = perm(TH, TL, sel0);
        W[1] = perm(TH, TL, sel1);
        const uint32_t sw = d.s[0];
        const uint32_t sb = (t >> 1) & 3;
        const uint32_t X = perm(sw, sw, 0x000C000Cu | (sb << 8) | (sb << 24));     // halves = sign byte << 8
        const int base = 4 * (t & 1);
        W[0] = and_or(pk_shl(X, 7 - base, 6 - base), 0x80008000u, W[0]);   // scales are >= 0: their sign bit is clear
        W[1] = and_or(pk_shl(X, 5 - base, 4 - base), 0x80008000u, W[1]);
        out[0] = perm(W[1], W[0], L.x);
        out[1] = perm(W[1], W[0], L.y);
        out[2] = perm(W[1], W[0], L.z);
        out[3] = perm(W[1], W[0], L.w);
    } else {
        const uint32_t v = window32<3>(d.r, 12 * t), v2 = v >> 2;
        const uint32_t Z = perm(v2, v, 0x04040000u);
        const uint32_t Z1 = perm(v2, v, 0x05050101u);
        const uint32_t sel0 = and_or(Z, 0x03030303u, 0x04000400u);
        const uint32_t sel1 = and_or(Z >> 4, 0x03030303u, 0x04000400u);
        const uint32_t sel2 = and_or(Z1, 0x03030303u, 0x04000400u);
        W[0] = perm(TH, TL, sel0);
        W[1] = perm(TH, TL, sel1);
        W[2] = perm(TH, TL, sel2);
        const uint32_t sv = window32<2>(d.s, 6 * t);
        const uint32_t X = perm(sv, sv, 0x000C000Cu);                               // halves = (sign bits) << 8
        W[0] = and_or(pk_shl(X, 7, 6), 0x80008000u, W[0]);
        W[1] = and_or(pk_shl(X, 5, 4), 0x80008000u, W[1]);
        W[2] = and_or(pk_shl(X, 3, 2), 0x80008000u, W[2]);
        out[0] = perm(W[1], W[0], L.x);
        out[1] = perm(W[1], W[0], L.y);
        out[2] = perm(W[2], W[1], L.z);
        out[3] = perm(W[2], W[1], L.w);
    }
}

__device__ inline half8_t as_half8(const uint32_t v[4]) {
    const uint4 u = make_uint4(v[0], v[1], v[2], v[3]);
    return __builtin_bit_cast(half8_t, u);
}

// ------------------------------------------------------------------------------------------------
// Residual term of the salient columns (Eq. 4, second binarisation): one record of the salient-column
// table covers 8 salient columns of the lane's half block.
// ------------------------------------------------------------------------------------------------
struct ResSel {
    uint32_t sel0, sel1;     // gather selectors for the mask bytes of entries 0..3 / 4..7
    uint32_t bit0, bit1;     // per entry: the bit of the column inside its mask byte
};

// A operand (negated weights) of 8 salient columns: entry e is -t_e * alpha_r where the column is kept, 0
// where it is pruned.  m = the half's mask words, rb8 = the 8 residual sign bits of the entries (bit e in
// bit e; other bits ignored), ar2 = alpha_r in both halves.
__device__ inline void residual_chunk(const uint32_t m[2], uint32_t rb8, uint32_t ar2, const ResSel& s,
                                      uint32_t out[4]) {
    // per entry: the mask byte that holds its column, reduced to its bit, then to a 0 / 1 flag (a byte b <= 128 is
    // non-zero iff b + 127 has bit 7 set)
    const uint32_t G0 = perm(m[1], m[0], s.sel0) & s.bit0;
    const uint32_t G1 = perm(m[1], m[0], s.sel1) & s.bit1;
    const uint32_t F0 = ((G0 + 0x7F7F7F7Fu) >> 7) & 0x01010101u;
    const uint32_t F1 = ((G1 + 0x7F7F7F7Fu) >> 7) & 0x01010101u;
    uint32_t K[4];
    K[0] = perm(0u, F0, 0x0C010C00u);      // halves = flag of entry 0 / 1
    K[1] = perm(0u, F0, 0x0C030C02u);
    K[2] = perm(0u, F1, 0x0C010C00u);
    K[3] = perm(0u, F1, 0x0C030C02u);
    const uint32_t X = perm(rb8, rb8, 0x000C000Cu);          // halves = rb8 << 8
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const uint32_t val = and_or_v(pk_shl(X, 7 - 2 * v, 6 - 2 * v), 0x80008000u, ar2);
        out[v] = pk_mul_u16(val, K[v]);
    }
}

}  // namespace stbt
#endif
