// Decode GEMV and verification dequantiser for the tiled device order (STB_KIND_TILED), gfx950.
// The expansion of packed bits into matrix-core operands is in stb_tiled.hpp.
#include "stb_tiled.hpp"

#include <cstdlib>

using namespace stbt;

#ifndef STB_VARIANT
#define STB_VARIANT 0
#endif
#ifndef STB_LUT_AHEAD
#define STB_LUT_AHEAD 2
#endif

#ifdef STB_TRACE
__device__ long long stb_trace_buf[4096 * 32];
#define TRACE(slot) do { if (lane == 0) stb_trace_buf[((blockIdx.y * gridDim.x + blockIdx.x) * 8 + wave) % 4096 * 32 + (slot)] = wall_clock64(); } while (0)
extern "C" int stb_trace_read(long long* host) { return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(stb_trace_buf), sizeof(long long) * 4096 * 32); }
#else
#define TRACE(slot) do {} while (0)
#endif

namespace {

// ------------------------------------------------------------------------------------------------
// stb_dequant on the tiled order: one wavefront per tile, lane (i, g) writes the 128 columns of its
// (row, block) with the same expansion code the product kernels use.  Salient weights are reassembled as
// f32(s*alpha_o + t*alpha_r) from the two fp16 terms with one fp32 addition.
// ------------------------------------------------------------------------------------------------
template <int N8>
__global__ __launch_bounds__(64) void dequant_tiled_kernel(TiledPlanes p, float* __restrict__ out) {
    __shared__ ExpandLuts lut;
    build_luts<N8>(&lut);
    __syncthreads();
    const int rt = blockIdx.x / p.nsb, sb = blockIdx.x % p.nsb;
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    const int q = 4 * sb + g, row = rt * 16 + i;
    const int64_t rec = ((int64_t)rt * p.nsb + sb) * 64 + lane;
    BlockData<N8> d;
    load_block<N8>(p, rec, false, 0, 0, d);
    if (row >= p.n || q >= p.nb) return;
    const uint32_t TL = perm(d.sc.y, d.sc.x, 0x06040200u), TH = perm(d.sc.y, d.sc.x, 0x07050301u);
    const float ar = __half2float(__ushort_as_half((unsigned short)d.ar));
    uint32_t ord = p.sal_prefix[q];                        // index of the block's first salient column
    float* o = out + (int64_t)row * p.k + (int64_t)q * 128;
#pragma unroll
    for (int t = 0; t < 16; t++) {
        uint32_t e[4];
        expand_group<N8>(d, TL, TH, t, lut_fetch<N8>(d, t, &lut), e);
        const half8_t a = as_half8(e);
        const uint32_t mb = (d.m[t >> 2] >> (8 * (t & 3))) & 0xFFu;
        const uint32_t salb = p.res_words ? (p.sal_bitmap[4 * q + (t >> 2)] >> (8 * (t & 3))) & 0xFFu : 0u;
        float vals[8];
#pragma unroll
        for (int c = 0; c < 8; c++) {
            float v = ((mb >> c) & 1u) ? -(float)a[c] : 0.0f;
            if ((salb >> c) & 1u) {
                if ((mb >> c) & 1u) {
                    const uint32_t w = p.res_sign[((int64_t)rt * p.res_words + (ord >> 5)) * 16 + i];
                    v = v + (((w >> (ord & 31u)) & 1u) ? ar : -ar);
                }
                ord++;
            }
            vals[c] = v;
        }
        *reinterpret_cast<float4*>(o + 8 * t) = make_float4(vals[0], vals[1], vals[2], vals[3]);
        *reinterpret_cast<float4*>(o + 8 * t + 4) = make_float4(vals[4], vals[5], vals[6], vals[7]);
    }
}

// ------------------------------------------------------------------------------------------------
// Decode GEMV (App. C: the memory-bound regime).  A workgroup owns R consecutive 16-row tiles; its W
// wavefronts split the superblocks (wavefront w takes superblocks w, w + W, ...), so everything that depends
// on the columns only -- the 16 B operands holding x for the superblock, the salient-column selectors and
// the gathered x of the salient columns -- is loaded once per (wavefront, superblock) and stays in registers
// while the wavefront streams the R tiles of packed weights, three tiles in flight.  Partial products go to
// LDS ([wavefront][tile][256] fp32) and are summed in a fixed order at the end.
// ------------------------------------------------------------------------------------------------
struct ResInv {
    ResSel sel;
    uint32_t xs[4];     // x at the 8 salient columns of the record (B operand)
};

// xrow = x of batch row min(i, B - 1) at the first column of block q (any valid address if the lane has no
// x to supply); live = the lane supplies x (i < B and q < nb).  All loads are unconditional so that they
// issue back to back; entries that do not exist read column 0 and are zeroed afterwards.
__device__ inline ResInv load_res_inv(const TiledPlanes& p, int q, int c, const unsigned short* __restrict__ xrow,
                                      bool live) {
    const uint32_t* rec = p.sal_tab + ((int64_t)q * p.sal_chunks + c) * 12;
    ResInv r;
    r.sel = load_res_sel(rec);
    const uint4 pv = *reinterpret_cast<const uint4*>(rec + 8);
    const uint32_t pw[4] = {pv.x, pv.y, pv.z, pv.w};
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
        h[e] = xrow[pos & 127u];
        if (!(live && pos < 128u)) h[e] = 0u;
    }
#pragma unroll
    for (int v = 0; v < 4; v++) r.xs[v] = h[2 * v] | (h[2 * v + 1] << 16);
    return r;
}

// Workgroup (gr, ks) of the grid owns the 16-row tiles [gr*R, gr*R + R) and the eight superblocks
// 8*ks .. 8*ks + 7, one per wavefront.  With more than eight superblocks (k > 4096) the grid has several
// column splits: each writes its partial sums to the workspace, takes a ticket, and the last split to finish
// a row group adds the partial sums in split order and writes y.
template <int N8, bool HAS_RES>
__global__ __launch_bounds__(512) void gemv_stream_kernel(TiledPlanes p, const __half* __restrict__ x, int B,
                                                           void* __restrict__ y, int y_fp32, int R,
                                                           float* __restrict__ ws_part, uint32_t* __restrict__ ws_count) {
    __shared__ ExpandLuts lut;
    __shared__ uint32_t ticket;
    extern __shared__ float part[];                  // [8][R][256]
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 15, g = lane >> 4;
    const int gr = blockIdx.x, ks = blockIdx.y, S = gridDim.y;
    const int r0 = gr * R;
    const int r1 = r0 + R < p.nrt ? r0 + R : p.nrt;
    const int rl = r1 - 1;
    const int sb = 8 * ks + wave;
    const bool active = sb < p.nsb;                  // uniform per wavefront
    const int Wa = p.nsb - 8 * ks < 8 ? p.nsb - 8 * ks : 8;     // wavefronts of this workgroup that have a superblock
    constexpr int L = TileLoads<N8, HAS_RES>::count;
    const int q = 4 * sb + g;

    LaneOffsets lo;
    lo.o16 = lane * 16u; lo.o8 = lane * 8u; lo.o2 = lane * 2u;
    lo.osign = lane * (2u * N8); lo.oregion = lane * (4u * N8);
    lo.ores0 = 0u; lo.ores1 = 0u;
    auto tile_of = [&](int rt) { return (int64_t)rt * p.nsb + sb; };
    auto clamp = [&](int rt) { return rt < rl ? rt : rl; };

    TRACE(0);
    // ---- the packed planes of the first two tiles and the column tables go out before anything else ----
    TileRegs<N8> t0, t1, t2;
    uint32_t ord = 0u;
    int nch = 0;
    if (active) {
        fetch_main<N8>(t0, p, tile_of(r0), lo);
        fetch_main<N8>(t1, p, tile_of(clamp(r0 + 1)), lo);
        if (HAS_RES) {
            ord = p.sal_prefix[q];
            nch = (int)p.sal_tab[((int64_t)q * p.sal_chunks) * 12 + 7];
        }
    }
    build_luts<N8>(&lut);
    TRACE(1);
    __syncthreads();
    TRACE(2);

    if (active) {
        const bool live = i < B && q < p.nb;
        const __half* xrow = x + (int64_t)(i < B ? i : B - 1) * p.k + (int64_t)(q < p.nb ? q : 0) * 128;
        int rsh = 0;
        if (HAS_RES) {
            nch = __builtin_amdgcn_readfirstlane(nch);
            rsh = (int)(ord & 31u);
            const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
            const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
            lo.ores0 = (uint32_t)(wa * 16 + i) * 4u;
            lo.ores1 = (uint32_t)(wb * 16 + i) * 4u;
        }
        fetch_res<N8, HAS_RES>(t0, p, r0, lo);
        fetch_res<N8, HAS_RES>(t1, p, clamp(r0 + 1), lo);

        // ---- operands that depend on the columns only ----
        uint4 xr[16];
#pragma unroll
        for (int t = 0; t < 16; t++) xr[t] = reinterpret_cast<const uint4*>(xrow)[t];
        ResInv inv0, inv1;
        if (HAS_RES) {
            inv0 = load_res_inv(p, q, 0, reinterpret_cast<const unsigned short*>(xrow), live);
            inv1 = load_res_inv(p, q, p.sal_chunks > 1 ? 1 : 0, reinterpret_cast<const unsigned short*>(xrow), live);
        }
        if (!live) {
#pragma unroll
            for (int t = 0; t < 16; t++) xr[t] = make_uint4(0u, 0u, 0u, 0u);
        }
        // Everything issued so far has arrived before the streaming loop starts: the compiler then places no
        // wait of its own inside the loop (such a wait would also drain the prefetched tiles), and the fixed
        // wait counts of the loop hold from its first iteration.
        __builtin_amdgcn_s_waitcnt(0x0F70);          // vmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
        TRACE(3);

        auto product = [&](const TileRegs<N8>& tr, int rt) {
            BlockData<N8> d;
            unpack_tile<N8>(tr, d);
            const uint32_t TL = perm(d.sc.y, d.sc.x, 0x06040200u), TH = perm(d.sc.y, d.sc.x, 0x07050301u);
            float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
            constexpr int D = STB_LUT_AHEAD;                             // table reads run D groups ahead
            GroupLut gl[D];
#pragma unroll
            for (int t = 0; t < D; t++) gl[t] = lut_fetch<N8>(d, t, &lut);
#pragma unroll
            for (int t = 0; t < 16; t++) {
                const GroupLut cur = gl[t % D];
                if (t + D < 16) gl[t % D] = lut_fetch<N8>(d, t + D, &lut);
                __builtin_amdgcn_sched_barrier(0);
                uint32_t o[4];
                expand_group<N8>(d, TL, TH, t, cur, o);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), __builtin_bit_cast(half8_t, xr[t]), acc, 0, 0, 0);
            }
            if (HAS_RES && nch > 0) {
                const uint32_t ar2 = d.ar | (d.ar << 16);
                const uint32_t rb = __builtin_amdgcn_alignbit(d.rhi, d.rlo, (uint32_t)rsh);   // the block's first 32 bits
                uint32_t o[4];
                residual_chunk(d.m, rb, ar2, inv0.sel, o);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(inv0.xs), acc, 0, 0, 0);
                if (nch > 1) {
                    residual_chunk(d.m, rb >> 8, ar2, inv1.sel, o);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(inv1.xs), acc, 0, 0, 0);
                }
            }
            float* dst = part + ((int64_t)(wave * R + (rt - r0)) * 256 + lane);
#pragma unroll
            for (int v = 0; v < 4; v++) dst[64 * v] = acc[v];
            TRACE(8 + (rt - r0 < 20 ? rt - r0 : 20));
        };

        // Three tiles in flight: while tile rt is expanded, the loads of rt + 1 and rt + 2 are outstanding.
        // Fetches past the last tile of the workgroup re-read that tile (cache hits), which keeps the number of
        // loads between a fetch and its wait the same on every path.
        for (int rt = r0; rt < r1; rt += 3) {
            fetch_tile<N8, HAS_RES>(t2, p, tile_of(clamp(rt + 2)), clamp(rt + 2), lo);
            wait_tile<2 * L>(t0);
            product(t0, rt);
            if (rt + 1 >= r1) break;
            fetch_tile<N8, HAS_RES>(t0, p, tile_of(clamp(rt + 3)), clamp(rt + 3), lo);
            wait_tile<2 * L>(t1);
            product(t1, rt + 1);
            if (rt + 2 >= r1) break;
            fetch_tile<N8, HAS_RES>(t1, p, tile_of(clamp(rt + 4)), clamp(rt + 4), lo);
            wait_tile<2 * L>(t2);
            product(t2, rt + 2);
        }
        TRACE(4);
        wait_tile<0>(t0);                            // drain: no load may still target a register that is reused
        wait_tile<0>(t1);
        wait_tile<0>(t2);

        // Blocks with more than 16 salient columns: the remaining records, outside the streaming loop so that
        // its load/wait pattern stays fixed.  Rare; every operand is re-read.
        if (HAS_RES && nch > 2) {
            const int64_t rstride = (int64_t)p.res_words * 16;
            for (int rt = r0; rt < r1; rt++) {
                const int64_t rec = tile_of(rt) * 64 + lane;
                const uint4 mv = p.mask[rec];
                const uint32_t m[4] = {mv.x, mv.y, mv.z, mv.w};
                const uint32_t ar = p.res_scale[rec];
                const uint32_t ar2 = ar | (ar << 16);
                float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                for (int c = 2; c < nch; c++) {
                    const ResInv inv = load_res_inv(p, q, c, reinterpret_cast<const unsigned short*>(xrow), live);
                    const uint32_t u0 = ord + 8u * (uint32_t)c;
                    const int wa = (int)(u0 >> 5) < p.res_words ? (int)(u0 >> 5) : p.res_words - 1;
                    const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
                    const uint32_t rlo = p.res_sign[rt * rstride + (int64_t)wa * 16 + i];
                    const uint32_t rhi = p.res_sign[rt * rstride + (int64_t)wb * 16 + i];
                    uint32_t o[4];
                    residual_chunk(m, __builtin_amdgcn_alignbit(rhi, rlo, u0 & 31u), ar2, inv.sel, o);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(inv.xs), acc, 0, 0, 0);
                }
                float* dst = part + ((int64_t)(wave * R + (rt - r0)) * 256 + lane);
#pragma unroll
                for (int v = 0; v < 4; v++) dst[64 * v] += acc[v];
            }
        }
    }
    TRACE(5);
    __syncthreads();
    TRACE(6);

    // D[row][b] of a tile: lane l holds b = l % 16, rows 4*(l / 16) + v.  Consecutive threads take consecutive rows.
    const int total = (r1 - r0) * 256;
    const int64_t n16 = (int64_t)p.nrt * 16;
    auto wg_sum = [&](int o) {
        const int j = o >> 8, b = (o >> 4) & 15, r16 = o & 15;
        const int l = b + 16 * (r16 >> 2), v = r16 & 3;
        float s = 0.0f;
        for (int w = 0; w < Wa; w++) s += part[(int64_t)(w * R + j) * 256 + 64 * v + l];
        return s;
    };
    auto store_y = [&](int o, float s) {
        const int b = (o >> 4) & 15, row = (r0 + (o >> 8)) * 16 + (o & 15);
        if (b < B && row < p.n) {
            if (y_fp32) reinterpret_cast<float*>(y)[(int64_t)b * p.n + row] = -s;
            else reinterpret_cast<__half*>(y)[(int64_t)b * p.n + row] = __float2half(-s);
        }
    };
    if (S == 1) {
        for (int o = threadIdx.x; o < total; o += blockDim.x) store_y(o, wg_sum(o));
        TRACE(7);
        return;
    }
    // ---- several column splits: partial sums to the workspace [split][16][n16], then a ticket ----
    // The partial sums are written and read with agent-scope accesses (they go through to the level all
    // compute dies share), so no cache write-back or invalidate is needed around the ticket: the stores have
    // completed (vmcnt = 0, then the barrier) before thread 0 takes the ticket, and the last arrival issues
    // its loads after it has seen the ticket.
    for (int o = threadIdx.x; o < total; o += blockDim.x) {
        const int b = (o >> 4) & 15, row = (r0 + (o >> 8)) * 16 + (o & 15);
        if (b < B) __hip_atomic_store(ws_part + ((int64_t)ks * 16 + b) * n16 + row, wg_sum(o), __ATOMIC_RELAXED,
                                      __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicInc(ws_count + gr, (uint32_t)(S - 1));    // wraps to 0 after S arrivals
    __syncthreads();
    if (ticket != (uint32_t)(S - 1)) return;
    for (int o = threadIdx.x; o < total; o += blockDim.x) {
        const int b = (o >> 4) & 15, row = (r0 + (o >> 8)) * 16 + (o & 15);
        if (b >= B) continue;
        float s = 0.0f;
        for (int c = 0; c < S; c++)
            s += __hip_atomic_load(ws_part + ((int64_t)c * 16 + b) * n16 + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        store_y(o, s);
    }
}

int env_int(const char* name, int dflt) {
    const char* v = std::getenv(name);
    return v && *v ? std::atoi(v) : dflt;
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

static int64_t round_up256(int64_t v) { return (v + 255) / 256 * 256; }

extern "C" int64_t stb_tiled_gemv_workspace(int n_row_tiles, int n_super) {
    const int S = (n_super + 7) / 8;
    if (S <= 1) return 0;
    return round_up256(4 * (int64_t)n_row_tiles) + (int64_t)S * 16 * 16 * n_row_tiles * 4;
}

template <int N8, bool HAS_RES>
static hipError_t launch_gemv_stream(const TiledPlanes& p, const __half* x, int B, void* y, int y_fp32, int R,
                                     dim3 grid, size_t lds, float* ws_part, uint32_t* ws_count, hipStream_t st) {
    static const hipError_t attr = hipFuncSetAttribute((const void*)gemv_stream_kernel<N8, HAS_RES>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024);
    if (attr != hipSuccess) return attr;
    hipLaunchKernelGGL((gemv_stream_kernel<N8, HAS_RES>), grid, dim3(512), lds, st, p, x, B, y, y_fp32, R, ws_part, ws_count);
    return hipGetLastError();
}

extern "C" int stb_tiled_gemv(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* workspace,
                              int64_t workspace_bytes, void* stream, int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    const TiledPlanes p = make_tiled(L);
    const int S = (p.nsb + 7) / 8;                                 // column splits of eight superblocks
    const int64_t need = stb_tiled_gemv_workspace(p.nrt, p.nsb);
    if (need > 0) {
        if (!workspace) return STB_ENULL;
        if (workspace_bytes < need) return STB_EINVAL;
        if ((uintptr_t)workspace % 256) return STB_EALIGN;
    }
    static const int wg_target = env_int("STB_GEMV_WGS", 256);     // workgroups the launch aims for
    int groups = wg_target / S;                                    // row groups
    if (groups < 1) groups = 1;
    int R = (p.nrt + groups - 1) / groups;                         // row tiles per workgroup
    if (R > 16) R = 16;                                            // 8 x R KB of partial sums in LDS
    const int G = (p.nrt + R - 1) / R;
    const size_t lds = (size_t)8 * R * 256 * sizeof(float);
    const dim3 grid(G, S);
    const hipStream_t st = (hipStream_t)stream;
    const __half* xh = (const __half*)x;
    uint32_t* cnt = (uint32_t*)workspace;
    float* part = need > 0 ? (float*)((char*)workspace + round_up256(4 * (int64_t)p.nrt)) : nullptr;
    const bool res = p.res_words > 0;
    hipError_t e;
    if (kept_per_8(L) == 4)
        e = res ? launch_gemv_stream<4, true>(p, xh, B, y, y_fp32, R, grid, lds, part, cnt, st)
                : launch_gemv_stream<4, false>(p, xh, B, y, y_fp32, R, grid, lds, part, cnt, st);
    else
        e = res ? launch_gemv_stream<6, true>(p, xh, B, y, y_fp32, R, grid, lds, part, cnt, st)
                : launch_gemv_stream<6, false>(p, xh, B, y, y_fp32, R, grid, lds, part, cnt, st);
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}
