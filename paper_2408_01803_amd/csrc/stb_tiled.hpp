// Device-side building blocks shared by the kernels that read the tiled device order (STB_KIND_TILED).
//
// One wavefront works on a tile of 16 output rows x 4 column blocks (512 columns): lane = 16*g + i owns
// (row i of the tile, block g of the superblock) and receives that block's 16 mask bytes, its sign and id
// bits and its scales with one coalesced load per plane.  The lane expands 8 columns at a time into the
// A operand (4 VGPRs of fp16) of v_mfma_f32_16x16x32_f16.  Expansion works on whole registers:
//   * ids -> byte selectors (a 256-entry table in LDS indexed by the id byte for 2:4 and 4:8, bit arithmetic
//     for 6:8) -> v_perm_b32 over the block's scale table gives two kept weights per register in slot order
//     (the order of the sign / id planes),
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
    const uint32_t* sal_tab;    // [nsb*4][sal_chunks][12]
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

__device__ inline uint32_t pk_min_u16(uint32_t a, uint32_t b) {
    const ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    const ushort2_t r = __builtin_elementwise_min(x, y);
    return __builtin_bit_cast(uint32_t, r);
}

__device__ inline uint32_t pk_mul_u16(uint32_t a, uint32_t b) {
    const ushort2_t x = __builtin_bit_cast(ushort2_t, a), y = __builtin_bit_cast(ushort2_t, b);
    const ushort2_t r = x * y;
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
// 8-column group at their columns.  N8 = kept weights per 8 columns (4 for 2:4 and 4:8, 6 for 6:8).
// Registers W0 = slots 0,1; W1 = slots 2,3; W2 = slots 4,5.  Selectors 0,1 address {W1:W0}; for N8 = 6
// selectors 2,3 address {W2:W1} (columns 4..7 can only hold slots 2..5), for N8 = 4 they address {W1:W0}.
// ------------------------------------------------------------------------------------------------
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
                int r = __popc(mb & ((1u << pcol) - 1u));
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

// ------------------------------------------------------------------------------------------------
// Per-lane operands of one (row, block)
// ------------------------------------------------------------------------------------------------
template <int N8>
struct BlockData {
    static constexpr int SW = N8 / 2;   // sign words   (128*N8/8 bits = 16*N8 bits)
    static constexpr int RW = N8;       // region words
    uint32_t m[4];
    uint32_t s[SW];
    uint32_t r[RW];
    uint2 sc;                           // the four scales {dense, inter, sparse, alpha_o} as stored
    uint32_t ar;                        // alpha_r (fp16 bits)
    uint32_t rlo, rhi;                  // the two res_sign words of the row that hold the block's first bits
};

// Issues the loads of lane record `rec`.  res0 = index of the first res_sign word of the lane's row in this
// row tile (already offset by the block's first word), res1 = the next word (clamped); has_res is uniform.
template <int N8>
__device__ inline void load_block(const TiledPlanes& p, int64_t rec, bool has_res, int64_t res0, int64_t res1,
                                  BlockData<N8>& d) {
    const uint4 m = p.mask[rec];
    d.m[0] = m.x; d.m[1] = m.y; d.m[2] = m.z; d.m[3] = m.w;
    const uint32_t* sp = reinterpret_cast<const uint32_t*>(p.sign + rec * (4 * BlockData<N8>::SW));
    const uint32_t* rp = reinterpret_cast<const uint32_t*>(p.region + rec * (4 * BlockData<N8>::RW));
    if (N8 == 4) {
        const uint2 s = *reinterpret_cast<const uint2*>(sp);
        d.s[0] = s.x; d.s[1] = s.y;
        const uint4 r = *reinterpret_cast<const uint4*>(rp);
        d.r[0] = r.x; d.r[1] = r.y; d.r[2] = r.z; d.r[3] = r.w;
    } else {
#pragma unroll
        for (int v = 0; v < BlockData<N8>::SW; v++) d.s[v] = sp[v];
#pragma unroll
        for (int v = 0; v < BlockData<N8>::RW; v += 2) {
            const uint2 r = *reinterpret_cast<const uint2*>(rp + v);
            d.r[v] = r.x; d.r[v + 1] = r.y;
        }
    }
    d.sc = p.scales[rec];
    d.ar = p.res_scale[rec];
    d.rlo = 0; d.rhi = 0;
    if (has_res) {
        d.rlo = p.res_sign[res0];
        d.rhi = p.res_sign[res1];
    }
}

// ------------------------------------------------------------------------------------------------
// Software-pipelined fetch of lane records.  The loads are written as asm statements with the plane base
// in SGPRs and a 32-bit lane offset, and the matching wait names every destination register as a read-write
// operand: the loads of several tiles stay in flight exactly as written (the compiler neither moves them
// nor waits for them), and no register of a tile can be read before wait_tile has been executed on it.
// Rules for callers: every fetch_tile is followed, on every path, by a wait_tile (or wait_tiles_all) on the
// same object before the object dies; K = number of such loads issued after the last load of the tile.
// ------------------------------------------------------------------------------------------------
typedef uint32_t uint3_t __attribute__((ext_vector_type(3)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

template <int N8>
struct TileRegs;
template <>
struct TileRegs<4> {
    uint4_t m; uint2_t s; uint4_t r; uint2_t sc; uint32_t ar, rlo, rhi;
};
template <>
struct TileRegs<6> {
    uint4_t m; uint3_t s; uint4_t r; uint2_t r2; uint2_t sc; uint32_t ar, rlo, rhi;
};
template <int N8, bool HAS_RES>
struct TileLoads {
    static constexpr int count = (N8 == 4 ? 5 : 6) + (HAS_RES ? 2 : 0);
};

// Per-lane byte offsets of the lane's record inside one tile of each plane.
struct LaneOffsets {
    uint32_t o16, o8, o2;      // lane * 16, lane * 8, lane * 2
    uint32_t osign, oregion;   // lane * sign_stride, lane * region_stride
    uint32_t ores0, ores1;     // byte offsets of the two res_sign words inside the row tile
};

template <int N8>
__device__ inline void fetch_main(TileRegs<N8>& d, const TiledPlanes& p, int64_t tile, const LaneOffsets& lo) {
    const char* bm = reinterpret_cast<const char*>(p.mask) + tile * (64 * 16);
    const char* bs = reinterpret_cast<const char*>(p.sign) + tile * (64 * 2 * N8);
    const char* br = reinterpret_cast<const char*>(p.region) + tile * (64 * 4 * N8);
    const char* bc = reinterpret_cast<const char*>(p.scales) + tile * (64 * 8);
    const char* ba = reinterpret_cast<const char*>(p.res_scale) + tile * (64 * 2);
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(d.m) : "v"(lo.o16), "s"(bm));
    if constexpr (N8 == 4) {
        asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(d.s) : "v"(lo.osign), "s"(bs));
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(d.r) : "v"(lo.oregion), "s"(br));
    } else {
        asm volatile("global_load_dwordx3 %0, %1, %2" : "=v"(d.s) : "v"(lo.osign), "s"(bs));
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(d.r) : "v"(lo.oregion), "s"(br));
        asm volatile("global_load_dwordx2 %0, %1, %2 offset:16" : "=v"(d.r2) : "v"(lo.oregion), "s"(br));
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
    if constexpr (N8 == 4)
        asm volatile("s_waitcnt vmcnt(%7)" : "+v"(d.m), "+v"(d.s), "+v"(d.r), "+v"(d.sc), "+v"(d.ar), "+v"(d.rlo), "+v"(d.rhi) : "n"(K));
    else
        asm volatile("s_waitcnt vmcnt(%8)" : "+v"(d.m), "+v"(d.s), "+v"(d.r), "+v"(d.r2), "+v"(d.sc), "+v"(d.ar), "+v"(d.rlo), "+v"(d.rhi) : "n"(K));
}

template <int N8>
__device__ inline void unpack_tile(const TileRegs<N8>& t, BlockData<N8>& d) {
    d.m[0] = t.m[0]; d.m[1] = t.m[1]; d.m[2] = t.m[2]; d.m[3] = t.m[3];
    if constexpr (N8 == 4) {
        d.s[0] = t.s[0]; d.s[1] = t.s[1];
        d.r[0] = t.r[0]; d.r[1] = t.r[1]; d.r[2] = t.r[2]; d.r[3] = t.r[3];
    } else {
        d.s[0] = t.s[0]; d.s[1] = t.s[1]; d.s[2] = t.s[2];
        d.r[0] = t.r[0]; d.r[1] = t.r[1]; d.r[2] = t.r[2]; d.r[3] = t.r[3]; d.r[4] = t.r2[0]; d.r[5] = t.r2[1];
    }
    d.sc = make_uint2(t.sc[0], t.sc[1]);
    d.ar = t.ar & 0xFFFFu;
    d.rlo = t.rlo; d.rhi = t.rhi;
}

// Second table (N8 = 4 only): for the byte holding the four 2-bit ids of an 8-column group, the two v_perm
// selectors that pick the low / high bytes of the scales of slots (0,1) and (2,3) out of {TH:TL}.
__device__ inline uint2 id_entry(uint32_t idb) {
    uint32_t sel[2];
#pragma unroll
    for (int v = 0; v < 2; v++) {
        const uint32_t a = (idb >> (4 * v)) & 3u, b = (idb >> (4 * v + 2)) & 3u;
        sel[v] = a | ((a | 4u) << 8) | (b << 16) | ((b | 4u) << 24);
    }
    return make_uint2(sel[0], sel[1]);
}

struct ExpandLuts {
    uint4 scatter[256];
    uint2 ids[256];
};

template <int N8>
__device__ inline void build_luts(ExpandLuts* L) {
    for (int e = threadIdx.x; e < 256; e += blockDim.x) {
        L->scatter[e] = scatter_entry<N8>((uint32_t)e);
        L->ids[e] = id_entry((uint32_t)e);
    }
}

// Table entries of group t (issued ahead of the arithmetic that uses them).
struct GroupLut {
    uint4 sc;
    uint2 id;
};

template <int N8>
__device__ inline GroupLut lut_fetch(const BlockData<N8>& d, int t, const ExpandLuts* L) {
    GroupLut g;
    const uint32_t mb = (d.m[t >> 2] >> (8 * (t & 3))) & 0xFFu;
#if defined(STB_VARIANT) && STB_VARIANT == 2
    g.sc = make_uint4(mb, mb * 3u, 0x01000302u, 0x05040706u);
    g.id = make_uint2(d.r[t >> 2], d.r[t >> 2] >> 3);
    return g;
#endif
    g.sc = L->scatter[mb];
    g.id = make_uint2(0u, 0u);
    if (N8 == 4) {
        const uint32_t idb = (d.r[t >> 2] >> (8 * (t & 3))) & 0xFFu;
        g.id = L->ids[idb];
    }
    return g;
}

// Expands columns 8t .. 8t+7 of the lane's block into four registers of fp16 pairs (negated weights).
// TL / TH = low / high bytes of the four scales; gl = the group's table entries.
template <int N8>
__device__ inline void expand_group(const BlockData<N8>& d, uint32_t TL, uint32_t TH, int t, const GroupLut& gl,
                                    uint32_t out[4]) {
    const uint4 L = gl.sc;
    uint32_t W[3];
    if (N8 == 4) {
        W[0] = perm(TH, TL, gl.id.x);
        W[1] = perm(TH, TL, gl.id.y);
        const uint32_t sw = d.s[t >> 3];
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
        const uint32_t v = window32<BlockData<N8>::RW>(d.r, 12 * t), v2 = v >> 2;
        const uint32_t Z = perm(v2, v, 0x04040000u);
        const uint32_t Z1 = perm(v2, v, 0x05050101u);
        const uint32_t sel0 = and_or(Z, 0x03030303u, 0x04000400u);
        const uint32_t sel1 = and_or(Z >> 4, 0x03030303u, 0x04000400u);
        const uint32_t sel2 = and_or(Z1, 0x03030303u, 0x04000400u);
        W[0] = perm(TH, TL, sel0);
        W[1] = perm(TH, TL, sel1);
        W[2] = perm(TH, TL, sel2);
        const uint32_t sv = window32<BlockData<N8>::SW>(d.s, 6 * t);
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
// table covers 8 salient columns of the lane's block.
// ------------------------------------------------------------------------------------------------
struct ResSel {
    uint32_t selA0, selB0, selA1, selB1;   // gather selectors for the mask bytes of entries 0..3 / 4..7
    uint32_t bit0, bit1;                   // per entry: the bit of the column inside its mask byte
};

__device__ inline ResSel load_res_sel(const uint32_t* rec) {
    const uint4 a = *reinterpret_cast<const uint4*>(rec);
    const uint2 b = *reinterpret_cast<const uint2*>(rec + 4);
    ResSel s;
    s.selA0 = a.x; s.selB0 = a.y; s.selA1 = a.z; s.selB1 = a.w;
    s.bit0 = b.x; s.bit1 = b.y;
    return s;
}

// A operand (negated weights) of 8 salient columns: entry e is -t_e * alpha_r where the column is kept, 0
// where it is pruned.  m = the block's mask words, rb8 = the 8 residual sign bits of the entries (bit e in
// bit e; other bits ignored), ar2 = alpha_r in both halves.
__device__ inline void residual_chunk(const uint32_t m[4], uint32_t rb8, uint32_t ar2, const ResSel& s,
                                      uint32_t out[4]) {
    const uint32_t G0 = (perm(m[1], m[0], s.selA0) | perm(m[3], m[2], s.selB0)) & s.bit0;
    const uint32_t G1 = (perm(m[1], m[0], s.selA1) | perm(m[3], m[2], s.selB1)) & s.bit1;
    uint32_t K[4];
    K[0] = perm(0u, G0, 0x0C010C00u);      // halves = byte of entry 0 / 1: non-zero iff kept
    K[1] = perm(0u, G0, 0x0C030C02u);
    K[2] = perm(0u, G1, 0x0C010C00u);
    K[3] = perm(0u, G1, 0x0C030C02u);
    const uint32_t X = perm(rb8, rb8, 0x000C000Cu);          // halves = rb8 << 8
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const uint32_t val = (pk_shl(X, 7 - 2 * v, 6 - 2 * v) & 0x80008000u) | ar2;
        out[v] = pk_mul_u16(val, pk_min_u16(K[v], 0x00010001u));
    }
}

}  // namespace stbt
#endif
