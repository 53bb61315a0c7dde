// Wavefront-tiled kernels for the tiled device order (STB_KIND_TILED), gfx950.
//
// One wavefront works on a tile of 16 output rows x 4 column blocks (512 columns): lane = 16*g + i owns
// (row i of the tile, block g of the superblock) and receives that block's 16 mask bytes, its sign and id
// bits and its scales with one coalesced load per plane.  The lane expands 8 columns at a time into the
// A operand (4 VGPRs of fp16) of v_mfma_f32_16x16x32_f16; the B operand is x (decode) or a token tile
// (prefill).  Expansion works on whole registers:
//   * ids -> byte selectors -> v_perm_b32 over the block's scale table gives two kept weights per register
//     in slot order (the order of the sign / id planes),
//   * sign bits are moved to bit 15 / 31 with one packed 16-bit shift and merged with one bit-select,
//   * a 256-entry table in LDS, indexed by the mask byte, holds the four v_perm selectors that spread the
//     slot-ordered weights to their column positions (zero where the mask bit is clear).
// Stored sign bit 1 means +1 (Eq. 2 / App. C "1 -> +1, 0 -> -1"); the bit is copied into the fp16 sign bit
// as it is, so every expanded weight is the negative of W_hat and the epilogue negates the accumulator.
// Salient columns (Eq. 4): alpha_o rides in the scale table as id 3; the residual term t*alpha_r is a second,
// short MFMA chain over the salient columns of the superblock (kept bit looked up in an LDS copy of the
// tile's mask bytes).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include "stb_internal.h"

namespace {

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
    const uint32_t* res_sign;   // [nrt*16][res_words]
    const uint32_t* sal_prefix; // [nsb*4 + 1]
    const uint16_t* sal_pos;    // [nsb][sal_stride]
    int n, k, nb, nrt, nsb;
    int res_words;              // uint32 per row of res_sign (0 if no salient columns)
    int sal_stride;
};

TiledPlanes make_tiled(const stb_layout_t* L) {
    TiledPlanes p;
    p.mask = (const uint4*)L->mask;
    p.sign = (const uint8_t*)L->sign;
    p.region = (const uint8_t*)L->region;
    p.scales = (const uint2*)L->scales;
    p.res_scale = (const uint16_t*)L->res_scale;
    p.res_sign = (const uint32_t*)L->res_sign;
    p.sal_prefix = L->sal_block_prefix;
    p.sal_pos = L->sal_pos;
    p.n = L->cfg.n_out;
    p.k = L->cfg.k_in;
    p.nb = L->n_blocks;
    p.nrt = L->n_row_tiles;
    p.nsb = L->n_super;
    p.res_words = (int)(L->res_stride / 4);
    p.sal_stride = L->sal_stride;
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

__device__ inline uint32_t pk_sar15(uint32_t v) {
    short2_t x = __builtin_bit_cast(short2_t, v);
    const short2_t s = {15, 15};
    x = x >> s;
    return __builtin_bit_cast(uint32_t, x);
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

template <int N8>
__device__ inline void build_scatter_lut(uint4* lut) {
    for (int mb = threadIdx.x; mb < 256; mb += blockDim.x) lut[mb] = scatter_entry<N8>((uint32_t)mb);
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
    uint32_t TL, TH;                    // low / high bytes of the four scales {dense, inter, sparse, alpha_o}
    uint32_t ar;                        // alpha_r (fp16 bits)
};

template <int N8>
__device__ inline void load_block(const TiledPlanes& p, int64_t rec, BlockData<N8>& d) {
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
    const uint2 sc = p.scales[rec];
    d.TL = perm(sc.y, sc.x, 0x06040200u);
    d.TH = perm(sc.y, sc.x, 0x07050301u);
    d.ar = p.res_scale[rec];
}

// Expands columns 8t .. 8t+7 of the lane's block into four registers of fp16 pairs (negated weights).
template <int N8>
__device__ inline void expand_group(const BlockData<N8>& d, int t, const uint4* lut, uint32_t out[4]) {
    const uint32_t mb = (d.m[t >> 2] >> (8 * (t & 3))) & 0xFFu;
    const uint4 L = lut[mb];
    uint32_t W[3];
    if (N8 == 4) {
        const uint32_t rw = d.r[t >> 2], r2 = rw >> 2;
        const uint32_t b = t & 3;
        const uint32_t Z = perm(r2, rw, b | (b << 8) | ((4 + b) << 16) | ((4 + b) << 24));
        const uint32_t sel0 = (Z & 0x03030303u) | 0x04000400u;
        const uint32_t sel1 = ((Z >> 4) & 0x03030303u) | 0x04000400u;
        W[0] = perm(d.TH, d.TL, sel0);
        W[1] = perm(d.TH, d.TL, sel1);
        const uint32_t sw = d.s[t >> 3];
        const uint32_t sb = (t >> 1) & 3;
        const uint32_t X = perm(sw, sw, 0x000C000Cu | (sb << 8) | (sb << 24));     // halves = sign byte << 8
        const int base = 4 * (t & 1);
        W[0] = (W[0] & 0x7FFF7FFFu) | (pk_shl(X, 7 - base, 6 - base) & 0x80008000u);
        W[1] = (W[1] & 0x7FFF7FFFu) | (pk_shl(X, 5 - base, 4 - base) & 0x80008000u);
        out[0] = perm(W[1], W[0], L.x);
        out[1] = perm(W[1], W[0], L.y);
        out[2] = perm(W[1], W[0], L.z);
        out[3] = perm(W[1], W[0], L.w);
    } else {
        const uint32_t v = window32<BlockData<N8>::RW>(d.r, 12 * t), v2 = v >> 2;
        const uint32_t Z = perm(v2, v, 0x04040000u);
        const uint32_t Z1 = perm(v2, v, 0x05050101u);
        const uint32_t sel0 = (Z & 0x03030303u) | 0x04000400u;
        const uint32_t sel1 = ((Z >> 4) & 0x03030303u) | 0x04000400u;
        const uint32_t sel2 = (Z1 & 0x03030303u) | 0x04000400u;
        W[0] = perm(d.TH, d.TL, sel0);
        W[1] = perm(d.TH, d.TL, sel1);
        W[2] = perm(d.TH, d.TL, sel2);
        const uint32_t sv = window32<BlockData<N8>::SW>(d.s, 6 * t);
        const uint32_t X = perm(sv, sv, 0x000C000Cu);                               // halves = (sign bits) << 8
        W[0] = (W[0] & 0x7FFF7FFFu) | (pk_shl(X, 7, 6) & 0x80008000u);
        W[1] = (W[1] & 0x7FFF7FFFu) | (pk_shl(X, 5, 4) & 0x80008000u);
        W[2] = (W[2] & 0x7FFF7FFFu) | (pk_shl(X, 3, 2) & 0x80008000u);
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
// Residual term of the salient columns of one superblock, 8 entries per lane: lane (i, g) of chunk ch owns
// entries 32*ch + 8*g + j, j < 8, of the superblock's ascending list of salient columns.
// ------------------------------------------------------------------------------------------------
struct ResCtx {
    int cs;          // salient columns in this superblock
    int ord;         // salient columns before it (index of its first bit in a res_sign row)
};

// pos[j] = column inside the superblock (0..511) or 0xFFFF.  mcopy = LDS copy of the tile's mask bytes,
// [16 rows][64 bytes]; rcopy = LDS copy of the tile's alpha_r, [16 rows][4].  Returns negated weights.
__device__ inline void expand_residual(const TiledPlanes& p, const ResCtx& rc, int ch, int i, int g, int row,
                                       const uint4 posv, const uint8_t* mcopy, const uint16_t* rcopy,
                                       uint32_t out[4]) {
    const int e0 = 32 * ch + 8 * g;
    const uint32_t pw[4] = {posv.x, posv.y, posv.z, posv.w};
    uint32_t kb = 0;
    uint32_t arp[4];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const uint32_t pos = ((pw[j >> 1] >> (16 * (j & 1))) & 0xFFFFu) & 511u;
        const uint32_t byte = mcopy[i * 64 + (pos >> 3)];
        kb |= ((byte >> (pos & 7u)) & 1u) << j;
        const uint32_t a = rcopy[i * 4 + (pos >> 7)];
        if (j & 1) arp[j >> 1] |= a << 16; else arp[j >> 1] = a;
    }
    int nvalid = rc.cs - e0;
    nvalid = nvalid < 0 ? 0 : (nvalid > 8 ? 8 : nvalid);
    kb &= (1u << nvalid) - 1u;
    // residual sign bits of the 8 entries
    const int u0 = rc.ord + e0;
    int w0 = u0 >> 5;
    w0 = w0 < p.res_words - 1 ? w0 : p.res_words - 1;
    const int w1 = w0 + 1 < p.res_words ? w0 + 1 : w0;
    const uint32_t* rr = p.res_sign + (int64_t)row * p.res_words;
    const uint32_t lo = rr[w0], hi = rr[w1];
    const uint32_t tb = (u0 & 31) ? __builtin_amdgcn_alignbit(hi, lo, u0 & 31) : lo;
    const uint32_t X = perm(tb, tb, 0x000C000Cu);
    const uint32_t K = perm(kb, kb, 0x000C000Cu);
#pragma unroll
    for (int v = 0; v < 4; v++) {
        const uint32_t sgn = pk_shl(X, 7 - 2 * v, 6 - 2 * v);
        const uint32_t keep = pk_sar15(pk_shl(K, 7 - 2 * v, 6 - 2 * v));
        out[v] = ((arp[v] & 0x7FFF7FFFu) | (sgn & 0x80008000u)) & keep;
    }
}

// ------------------------------------------------------------------------------------------------
// Tile driver shared by the kernels: calls f(t, a, d) for each of the 16 column groups of the superblock
// (a = A operand of columns 8t..8t+7 of every lane's block, d = the lane's packed operands) and
// fr(ch, a, posv) for each residual chunk.
// ------------------------------------------------------------------------------------------------
struct TileLds {
    uint8_t mcopy[16 * 64];
    uint16_t rcopy[16 * 4];
};

template <int N8, class F, class FR>
__device__ inline void for_tile(const TiledPlanes& p, int rt, int sb, const uint4* lut, TileLds* tl, F&& f, FR&& fr) {
    const int lane = threadIdx.x & 63, i = lane & 15, g = lane >> 4;
    const int64_t rec = ((int64_t)rt * p.nsb + sb) * 64 + lane;
    BlockData<N8> d;
    load_block<N8>(p, rec, d);
    ResCtx rc;
    rc.ord = (int)p.sal_prefix[4 * sb];
    rc.cs = p.res_words ? (int)p.sal_prefix[4 * sb + 4] - rc.ord : 0;
    const int nch = (rc.cs + 31) >> 5;
    if (nch > 0) {
        *reinterpret_cast<uint4*>(&tl->mcopy[i * 64 + g * 16]) = make_uint4(d.m[0], d.m[1], d.m[2], d.m[3]);
        tl->rcopy[i * 4 + g] = (uint16_t)d.ar;
    }
#pragma unroll
    for (int t = 0; t < 16; t++) {
        uint32_t o[4];
        expand_group<N8>(d, t, lut, o);
        f(t, as_half8(o), d);
    }
    if (nch > 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        for (int ch = 0; ch < nch; ch++) {
            const uint4 posv = *reinterpret_cast<const uint4*>(p.sal_pos + (int64_t)sb * p.sal_stride + 32 * ch + 8 * g);
            uint32_t o[4];
            expand_residual(p, rc, ch, i, g, rt * 16 + i, posv, tl->mcopy, tl->rcopy, o);
            fr(ch, as_half8(o), posv);
        }
        __builtin_amdgcn_wave_barrier();
    }
}

// ------------------------------------------------------------------------------------------------
// stb_dequant on the tiled order: expands every tile with the same code the product kernels use and writes
// dense fp32.  Salient weights are reassembled as f32(s*alpha_o + t*alpha_r) from the two fp16 terms.
// One wavefront per tile; the tile is staged in LDS as fp32 [16 rows][512 columns].
// ------------------------------------------------------------------------------------------------
template <int N8>
__global__ __launch_bounds__(64) void dequant_tiled_kernel(TiledPlanes p, float* __restrict__ out) {
    __shared__ uint4 lut[256];
    __shared__ TileLds tl;
    __shared__ float stage[16 * 512];
    build_scatter_lut<N8>(lut);
    __syncthreads();
    const int rt = blockIdx.x / p.nsb, sb = blockIdx.x % p.nsb;
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    for_tile<N8>(
        p, rt, sb, lut, &tl,
        [&](int t, half8_t a, const BlockData<N8>& d) {
            const uint32_t mb = d.m[t >> 2] >> (8 * (t & 3));
#pragma unroll
            for (int e = 0; e < 8; e++)
                stage[i * 512 + g * 128 + 8 * t + e] = ((mb >> e) & 1u) ? -(float)a[e] : 0.0f;
        },
        [&](int ch, half8_t a, uint4 posv) {
            const uint32_t pw[4] = {posv.x, posv.y, posv.z, posv.w};
#pragma unroll
            for (int e = 0; e < 8; e++) {
                const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                // the main term was stored by the lane that owns the column's block: same wavefront
                if (pos < 512u) stage[i * 512 + pos] = stage[i * 512 + pos] + (-(float)a[e]);
            }
        });
    __syncthreads();
    for (int idx = lane; idx < 16 * 512; idx += 64) {
        const int r = rt * 16 + idx / 512, c = sb * 512 + idx % 512;
        if (r < p.n && c < p.k) out[(int64_t)r * p.k + c] = stage[idx];
    }
}

// ------------------------------------------------------------------------------------------------
// Decode GEMV: workgroup = W wavefronts that split the superblocks of one 16-row tile; x (B <= 16 rows) is
// the B operand, read from global memory (it stays in L1/L2) by the lanes with lane % 16 < B.
// ------------------------------------------------------------------------------------------------
template <int N8>
__global__ __launch_bounds__(512) void gemv_tiled_kernel(TiledPlanes p, const __half* __restrict__ x, int B,
                                                          void* __restrict__ y, int y_fp32) {
    __shared__ uint4 lut[256];
    __shared__ TileLds tls[8];
    __shared__ float red[8][4][64];
    build_scatter_lut<N8>(lut);
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, W = blockDim.x >> 6;
    const int bcol = lane & 15, g = lane >> 4;
    const int rt = blockIdx.x;
    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int sb = wave; sb < p.nsb; sb += W) {
        const int q = 4 * sb + g;
        const bool xok = bcol < B && q < p.nb;
        const __half* xrow = x + (int64_t)bcol * p.k + (int64_t)q * 128;
        const __half* xsb = x + (int64_t)bcol * p.k + (int64_t)sb * 512;
        for_tile<N8>(
            p, rt, sb, lut, &tls[wave],
            [&](int t, half8_t a, const BlockData<N8>&) {
                uint4 xb = make_uint4(0u, 0u, 0u, 0u);
                if (xok) xb = *reinterpret_cast<const uint4*>(xrow + 8 * t);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, __builtin_bit_cast(half8_t, xb), acc, 0, 0, 0);
            },
            [&](int ch, half8_t a, uint4 posv) {
                const uint32_t pw[4] = {posv.x, posv.y, posv.z, posv.w};
                uint32_t xv[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    uint32_t h = 0;
                    if (bcol < B && pos < 512u && sb * 512 + (int)pos < p.k)
                        h = *reinterpret_cast<const uint16_t*>(xsb + pos);
                    xv[e >> 1] |= h << (16 * (e & 1));
                }
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, as_half8(xv), acc, 0, 0, 0);
            });
    }
#pragma unroll
    for (int v = 0; v < 4; v++) red[wave][v][lane] = acc[v];
    __syncthreads();
    // D[row][b]: lane holds b = lane % 16, rows 4*(lane / 16) + v
    for (int o = threadIdx.x; o < 256; o += blockDim.x) {
        const int v = o >> 6, l = o & 63;
        float s = 0.0f;
        for (int w = 0; w < W; w++) s += red[w][v][l];
        const int b = l & 15, row = rt * 16 + 4 * (l >> 4) + v;
        if (b < B && row < p.n) {
            if (y_fp32) reinterpret_cast<float*>(y)[(int64_t)b * p.n + row] = -s;
            else reinterpret_cast<__half*>(y)[(int64_t)b * p.n + row] = __float2half(-s);
        }
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// launchers (internal ABI, see stb_internal.h)
// ------------------------------------------------------------------------------------------------
static int kept_per_8(const stb_layout_t* L) { return 8 * L->cfg.N / L->cfg.M; }

extern "C" int stb_tiled_supported(const stb_layout_t* L) {
    const int n8 = kept_per_8(L);
    return (8 * L->cfg.N) % L->cfg.M == 0 && (n8 == 4 || n8 == 6);
}

extern "C" int stb_tiled_dequant(const stb_layout_t* L, float* out, void* stream, int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    const TiledPlanes p = make_tiled(L);
    const dim3 grid(p.nrt * p.nsb);
    if (kept_per_8(L) == 4)
        hipLaunchKernelGGL(dequant_tiled_kernel<4>, grid, dim3(64), 0, (hipStream_t)stream, p, out);
    else
        hipLaunchKernelGGL(dequant_tiled_kernel<6>, grid, dim3(64), 0, (hipStream_t)stream, p, out);
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}

extern "C" int stb_tiled_gemv(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* stream,
                              int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    const TiledPlanes p = make_tiled(L);
    const int per = (p.nsb + 7) / 8;                 // superblocks per wavefront
    const int W = (p.nsb + per - 1) / per;           // wavefronts per workgroup, <= 8
    const dim3 grid(p.nrt), block(64 * W);
    if (kept_per_8(L) == 4)
        hipLaunchKernelGGL(gemv_tiled_kernel<4>, grid, block, 0, (hipStream_t)stream, p, (const __half*)x, B, y, y_fp32);
    else
        hipLaunchKernelGGL(gemv_tiled_kernel<6>, grid, block, 0, (hipStream_t)stream, p, (const __half*)x, B, y, y_fp32);
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}
