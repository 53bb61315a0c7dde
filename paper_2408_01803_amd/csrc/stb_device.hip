// Device side of libstb for gfx950: dequantisation, decode GEMV and prefill GEMM on the packed planes.
// C ABI in include/stb.h.  Everything here runs on the caller's stream; nothing allocates.
#include <hip/hip_runtime.h>

#include <atomic>
#include <mutex>
#include <vector>
#include <hip/hip_fp16.h>

#include "stb_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

inline int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return STB_EHIP;
}

// Plane pointers and sizes in the form the kernels take them (passed by value).
struct Planes {
    const uint32_t* mask;
    const uint8_t* sign;
    const uint8_t* region;
    const uint8_t* res_sign;
    const __half* scales;       // [n][nb][4]
    const __half* res_scale;    // [n][nb]
    const uint32_t* sal_bitmap;
    const uint32_t* sal_prefix;
    int n, k, N, M, nb, wpr;    // wpr = mask words per row = k/32
    int sign_stride, region_stride, res_stride;
    int spw;                    // kept weights ("slots") per mask word = 32*N/M
};

Planes make_planes(const stb_layout_t* L) {
    Planes p;
    p.mask = L->mask;
    p.sign = (const uint8_t*)L->sign;
    p.region = (const uint8_t*)L->region;
    p.res_sign = (const uint8_t*)L->res_sign;
    p.scales = (const __half*)L->scales;
    p.res_scale = (const __half*)L->res_scale;
    p.sal_bitmap = L->sal_bitmap;
    p.sal_prefix = L->sal_block_prefix;
    p.n = L->cfg.n_out;
    p.k = L->cfg.k_in;
    p.N = L->cfg.N;
    p.M = L->cfg.M;
    p.nb = L->n_blocks;
    p.wpr = p.k / 32;
    p.sign_stride = (int)L->sign_stride;
    p.region_stride = (int)L->region_stride;
    p.res_stride = (int)L->res_stride;
    p.spw = 32 * p.N / p.M;
    return p;
}

// ------------------------------------------------------------------------------------------------
// Decoder of one mask word (32 consecutive columns of one row), generic in N:M.
// Because every M-group keeps exactly N weights, the first slot of mask word w is w * 32*N/M.
// ------------------------------------------------------------------------------------------------
struct WordCtx {
    uint32_t m;            // mask bits
    uint32_t salw;         // salient-column bits of the same 32 columns
    int slot0;             // slot of the first kept weight of the word
    int ord0;              // index among salient columns of the word's first column
    float a0, a1, a2, a3;  // dense, intermediate, sparse, alpha_o
    float ar;              // alpha_r
    const uint8_t* srow;
    const uint8_t* rrow;
    const uint8_t* trow;
};

__device__ inline WordCtx load_word(const Planes& p, int row, int w) {
    WordCtx c;
    c.m = p.mask[(size_t)row * p.wpr + w];
    c.salw = p.sal_bitmap[w];
    c.slot0 = w * p.spw;
    const int q = w >> 2;
    int ord = (int)p.sal_prefix[q];
    for (int v = q * 4; v < w; v++) ord += __popc(p.sal_bitmap[v]);
    c.ord0 = ord;
    const uint2 sc = *reinterpret_cast<const uint2*>(p.scales + ((size_t)row * p.nb + q) * 4);
    const __half2 s01 = *reinterpret_cast<const __half2*>(&sc.x);
    const __half2 s23 = *reinterpret_cast<const __half2*>(&sc.y);
    c.a0 = __low2float(s01);
    c.a1 = __high2float(s01);
    c.a2 = __low2float(s23);
    c.a3 = __high2float(s23);
    c.ar = __half2float(p.res_scale[(size_t)row * p.nb + q]);
    c.srow = p.sign + (size_t)row * p.sign_stride;
    c.rrow = p.region + (size_t)row * p.region_stride;
    c.trow = p.res_sign ? p.res_sign + (size_t)row * p.res_stride : nullptr;
    return c;
}

// Dequantised value of bit position `pos` of the word (must be a kept position), `rank` = number of
// kept positions below it inside the word.
// The two terms of a kept position: s * scale (an fp16 value) and, on a salient column, t * alpha_r (else 0).
__device__ inline float decode_kept_terms(const WordCtx& c, int pos, int rank, float* residual) {
    const int slot = c.slot0 + rank;
    const bool plus = (c.srow[slot >> 3] >> (slot & 7)) & 1;
    const unsigned id = (c.rrow[slot >> 2] >> ((slot & 3) * 2)) & 3u;
    const float a = id == 0 ? c.a0 : (id == 1 ? c.a1 : (id == 2 ? c.a2 : c.a3));
    *residual = 0.0f;
    if (id == 3 && c.trow) {
        const int u = c.ord0 + __popc(c.salw & ((1u << pos) - 1u));
        const bool tplus = (c.trow[u >> 3] >> (u & 7)) & 1;
        *residual = tplus ? c.ar : -c.ar;
    }
    return plus ? a : -a;
}
__device__ inline float decode_kept(const WordCtx& c, int pos, int rank) {
    float r;
    const float v = decode_kept_terms(c, pos, rank, &r);
    return v + r;                            // one fp32 addition (adding 0 changes nothing)
}

// ------------------------------------------------------------------------------------------------
// stb_dequant: one thread per (row, mask word)
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dequant_kernel(Planes p, float* __restrict__ out) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (int64_t)p.n * p.wpr) return;
    const int row = (int)(gid / p.wpr), w = (int)(gid % p.wpr);
    const WordCtx c = load_word(p, row, w);
    float* o = out + (size_t)row * p.k + (size_t)w * 32;
    int rank = 0;
    for (int pos = 0; pos < 32; pos++) {
        float v = 0.0f;
        if ((c.m >> pos) & 1u) {
            v = decode_kept(c, pos, rank);
            rank++;
        }
        o[pos] = v;
    }
}

// ------------------------------------------------------------------------------------------------
// Generic decode GEMV (any N:M): one wavefront per output row, lanes stride over the mask words.
// ------------------------------------------------------------------------------------------------
template <int B>
__global__ __launch_bounds__(256) void gemv_generic_kernel(Planes p, const __half* __restrict__ x,
                                                            void* __restrict__ y, int y_fp32) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + wave;
    if (row >= p.n) return;
    float acc[B];
#pragma unroll
    for (int b = 0; b < B; b++) acc[b] = 0.0f;
    for (int w = lane; w < p.wpr; w += 64) {
        const WordCtx c = load_word(p, row, w);
        uint32_t m = c.m;
        int rank = 0;
        while (m) {
            const int pos = __ffs(m) - 1;
            m &= m - 1;
            const float v = decode_kept(c, pos, rank);
            rank++;
            const int j = w * 32 + pos;
#pragma unroll
            for (int b = 0; b < B; b++) acc[b] += v * __half2float(x[(size_t)b * p.k + j]);
        }
    }
#pragma unroll
    for (int b = 0; b < B; b++) {
        float s = acc[b];
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) {
            if (y_fp32) reinterpret_cast<float*>(y)[(size_t)b * p.n + row] = s;
            else reinterpret_cast<__half*>(y)[(size_t)b * p.n + row] = __float2half(s);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Generic prefill GEMM (any N:M): 64 tokens x 64 output rows per workgroup, one 128-column block per
// step; the W tile is dequantised to fp16 in LDS, the contraction runs on v_mfma_f32_32x32x8_f16.
// A salient weight s * alpha_o + t * alpha_r is not an fp16 value in general: its two terms (both fp16 values) go
// to two tiles and two contractions, as in the tiled kernels, so that no product is taken with a rounded weight.
// ------------------------------------------------------------------------------------------------
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int GT = 64;           // tokens per tile
constexpr int GN = 64;           // output rows per tile
constexpr int GK = 128;          // columns per step
constexpr int GPAD = 8;          // halves of row padding in LDS

__global__ __launch_bounds__(256) void gemm_generic_kernel(Planes p, const __half* __restrict__ X, int T,
                                                            void* __restrict__ Y, int y_fp32) {
    __shared__ __attribute__((aligned(16))) _Float16 Ws[GN][GK + GPAD];
    __shared__ __attribute__((aligned(16))) _Float16 Rs[GN][GK + GPAD];     // residual terms (layers with salient columns)
    __shared__ __attribute__((aligned(16))) _Float16 Xs[GT][GK + GPAD];
    const bool has_res = p.res_sign != nullptr;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int n0 = blockIdx.x * GN, t0 = blockIdx.y * GT;
    const int wt = (wave >> 1) * 32, wn = (wave & 1) * 32;     // sub-tile of this wavefront
    float16_t acc;
#pragma unroll
    for (int v = 0; v < 16; v++) acc[v] = 0.0f;

    const int r = tid >> 2, seg = tid & 3;                     // (row | token) and 32-column segment
    for (int q = 0; q < p.nb; q++) {
        // ---- W tile: thread (r, seg) decodes mask word 4q + seg of row n0 + r ----
        {
            _Float16* dst = &Ws[r][seg * 32];
            _Float16* dres = &Rs[r][seg * 32];
            const int row = n0 + r;
            if (row < p.n) {
                const WordCtx c = load_word(p, row, q * 4 + seg);
                int rank = 0;
                for (int pos = 0; pos < 32; pos++) {
                    float v = 0.0f, res = 0.0f;
                    if ((c.m >> pos) & 1u) {
                        v = decode_kept_terms(c, pos, rank, &res);
                        rank++;
                    }
                    dst[pos] = (_Float16)v;                        // exact: v and res are +- an fp16 scale, or 0
                    if (has_res) dres[pos] = (_Float16)res;
                }
            } else {
                for (int pos = 0; pos < 32; pos++) { dst[pos] = (_Float16)0.0f; if (has_res) dres[pos] = (_Float16)0.0f; }
            }
        }
        // ---- X tile: thread (r, seg) copies 32 halves of token t0 + r ----
        {
            uint4* dst = reinterpret_cast<uint4*>(&Xs[r][seg * 32]);
            const int t = t0 + r;
            if (t < T) {
                const uint4* src = reinterpret_cast<const uint4*>(X + (size_t)t * p.k + (size_t)q * GK + seg * 32);
#pragma unroll
                for (int v = 0; v < 4; v++) dst[v] = src[v];
            } else {
                const uint4 z = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int v = 0; v < 4; v++) dst[v] = z;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GK / 8; kk++) {
            const int kc = kk * 8 + (lane >> 5) * 4;
            const half4_t a = *reinterpret_cast<const half4_t*>(&Xs[wt + (lane & 31)][kc]);
            const half4_t b = *reinterpret_cast<const half4_t*>(&Ws[wn + (lane & 31)][kc]);
            acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b, acc, 0, 0, 0);
            if (has_res) {
                const half4_t b2 = *reinterpret_cast<const half4_t*>(&Rs[wn + (lane & 31)][kc]);
                acc = __builtin_amdgcn_mfma_f32_32x32x8f16(a, b2, acc, 0, 0, 0);
            }
        }
        __syncthreads();
    }
    // D[token][row]: lane holds column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4
    const int col = n0 + wn + (lane & 31);
    if (col < p.n) {
#pragma unroll
        for (int v = 0; v < 16; v++) {
            const int t = t0 + wt + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (t < T) {
                if (y_fp32) reinterpret_cast<float*>(Y)[(size_t)t * p.n + col] = acc[v];
                else reinterpret_cast<__half*>(Y)[(size_t)t * p.n + col] = __float2half(acc[v]);
            }
        }
    }
}

// Streaming read of a buffer: every workgroup pulls a contiguous slice, 4 x 16 bytes per lane in flight.
__global__ __launch_bounds__(512) void probe_read_kernel(const uint4* __restrict__ src, int64_t n16, uint32_t* __restrict__ sink) {
    const int64_t per = (n16 + gridDim.x - 1) / gridDim.x;
    const int64_t lo = per * blockIdx.x, hi = lo + per < n16 ? lo + per : n16;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (int64_t i = lo + threadIdx.x; i < hi; i += 4 * blockDim.x) {
        uint4 v[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int64_t idx = i + (int64_t)j * blockDim.x;
            v[j] = idx < hi ? src[idx] : make_uint4(0u, 0u, 0u, 0u);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) { acc.x ^= v[j].x; acc.y ^= v[j].y; acc.z ^= v[j].z; acc.w ^= v[j].w; }
    }
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int off = 32; off > 0; off >>= 1) r ^= __shfl_xor(r, off, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(sink + (blockIdx.x & 1023), r);
}

// ------------------------------------------------------------------------------------------------
// Generic decode GEMV, second form (any N:M; used when B rows of x fit in LDS): a workgroup stages x once, in a
// transposed order, and takes 16 output rows, four per wavefront one after the other.  A lane owns one mask word
// (32 columns) at a time and reads that word's sign bits, id fields and residual-sign bits as bit windows (two or
// three aligned 32-bit loads each) instead of one byte load per kept weight.
// LDS order: x[b][32 w + pos] at ((b * 32 + pos) * (W + 1) + w), W = k / 32: the lanes of a wavefront differ in w.
// ------------------------------------------------------------------------------------------------
__device__ inline uint32_t bit_window(const uint32_t* words, int n_words, int bit) {
    // 32 bits of a little-endian bit string starting at `bit`; words past the end read as the last word (their
    // bits are never used: a window is cut to its own length by the caller)
    const int dw = bit >> 5;
    const uint32_t lo = words[dw < n_words ? dw : n_words - 1];
    const uint32_t hi = words[dw + 1 < n_words ? dw + 1 : n_words - 1];
    return __builtin_amdgcn_alignbit(hi, lo, (uint32_t)(bit & 31));
}

template <int B>
__global__ __launch_bounds__(256) void gemv_rows_kernel(Planes p, const __half* __restrict__ x, void* __restrict__ y, int y_fp32) {
    extern __shared__ __attribute__((aligned(16))) __half xs[];
    const int W = p.wpr, WP = W + 1;
    for (int idx = threadIdx.x; idx < B * p.k; idx += 256) {
        const int b = idx / p.k, j = idx - b * p.k;
        xs[(b * 32 + (j & 31)) * WP + (j >> 5)] = x[idx];
    }
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int sign_words = p.sign_stride / 4, region_words = p.region_stride / 4, res_words = p.res_stride / 4;
    for (int rr = 0; rr < 4; rr++) {
        const int row = blockIdx.x * 16 + wave * 4 + rr;
        if (row >= p.n) break;                                      // uniform per wavefront
        const uint32_t* srow = reinterpret_cast<const uint32_t*>(p.sign + (size_t)row * p.sign_stride);
        const uint32_t* rrow = reinterpret_cast<const uint32_t*>(p.region + (size_t)row * p.region_stride);
        const uint32_t* trow = p.res_sign ? reinterpret_cast<const uint32_t*>(p.res_sign + (size_t)row * p.res_stride) : nullptr;
        float acc[B];
#pragma unroll
        for (int b = 0; b < B; b++) acc[b] = 0.0f;
        for (int w = lane; w < W; w += 64) {
            uint32_t m = p.mask[(size_t)row * W + w];
            const uint32_t salw = p.sal_bitmap[w];
            const int slot0 = w * p.spw, q = w >> 2;
            const uint32_t sw = bit_window(srow, sign_words, slot0);                 // spw <= 32 sign bits
            const uint32_t r0 = bit_window(rrow, region_words, 2 * slot0);           // ids of the first 16 slots
            const uint32_t r1 = bit_window(rrow, region_words, 2 * slot0 + 32);      // ... of the next 16
            uint32_t tw = 0u;
            if (trow) {
                int ord = (int)p.sal_prefix[q];
                for (int v = q * 4; v < w; v++) ord += __popc(p.sal_bitmap[v]);
                tw = bit_window(trow, res_words, ord);                               // residual signs of the word's salient columns
            }
            const uint2 sc = *reinterpret_cast<const uint2*>(p.scales + ((size_t)row * p.nb + q) * 4);
            const __half2 s01 = *reinterpret_cast<const __half2*>(&sc.x);
            const __half2 s23 = *reinterpret_cast<const __half2*>(&sc.y);
            const float a0 = __low2float(s01), a1 = __high2float(s01), a2 = __low2float(s23), a3 = __high2float(s23);
            const float ar = __half2float(p.res_scale[(size_t)row * p.nb + q]);
            const __half* xw = xs + w;
            int rank = 0;
            while (m) {                                             // every word keeps 32 N / M weights: the same trip count in all lanes
                const int pos = __ffs(m) - 1;
                m &= m - 1;
                const bool plus = (sw >> rank) & 1u;
                const uint32_t id = ((rank < 16 ? r0 >> (2 * rank) : r1 >> (2 * rank - 32))) & 3u;
                const float a = id == 0 ? a0 : (id == 1 ? a1 : (id == 2 ? a2 : a3));
                float v = plus ? a : -a;
                if (id == 3 && trow) {
                    const int u = __popc(salw & ((1u << pos) - 1u));
                    v = v + (((tw >> u) & 1u) ? ar : -ar);          // one fp32 addition
                }
                rank++;
#pragma unroll
                for (int b = 0; b < B; b++) acc[b] += v * __half2float(xw[(b * 32 + pos) * WP]);
            }
        }
#pragma unroll
        for (int b = 0; b < B; b++) {
            float s = acc[b];
            for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            if (lane == 0) {
                if (y_fp32) reinterpret_cast<float*>(y)[(size_t)b * p.n + row] = s;
                else reinterpret_cast<__half*>(y)[(size_t)b * p.n + row] = __float2half(s);
            }
        }
    }
}

constexpr int64_t GEMV_ROWS_LDS_MAX = 120 * 1024;
static int64_t gemv_rows_lds(const Planes& p, int B) { return (int64_t)B * 32 * (p.wpr + 1) * 2; }

template <int B>
hipError_t launch_gemv_rows(const Planes& p, const void* x, void* y, int y_fp32, hipStream_t s) {
    static std::atomic<bool> attr_set{false};         // a failure is not remembered: the next call tries again
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute((const void*)gemv_rows_kernel<B>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)GEMV_ROWS_LDS_MAX);
        if (attr != hipSuccess) return attr;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(gemv_rows_kernel<B>, dim3((p.n + 15) / 16), dim3(256), (size_t)gemv_rows_lds(p, B), s, p, (const __half*)x, y, y_fp32);
    return hipGetLastError();
}

template <int B>
hipError_t launch_gemv_generic(const Planes& p, const void* x, void* y, int y_fp32, hipStream_t s) {
    const int blocks = (p.n + 3) / 4;
    hipLaunchKernelGGL(gemv_generic_kernel<B>, dim3(blocks), dim3(256), 0, s, p, (const __half*)x, y, y_fp32);
    return hipGetLastError();
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" int stb_last_hip_error(void) { return g_last_hip_error; }

// ------------------------------------------------------------------------------------------------
// packer on the GPU
// ------------------------------------------------------------------------------------------------
extern "C" int stb_tile_device(const stb_layout_t* src, stb_layout_t* dst, void* stream) {
    int rc = stb_layout_check(src);
    if (rc) return rc;
    if (!dst) return STB_ENULL;
    dst->max_sal_block = 0;
    dst->max_sal_half = 0;
    rc = stb_layout_check(dst);
    if (rc) return rc;
    const stb_cfg_t &a = src->cfg, &b = dst->cfg;
    if (src->kind != STB_KIND_ROWMAJOR || dst->kind != STB_KIND_TILED || a.n_out != b.n_out || a.k_in != b.k_in ||
        a.N != b.N || a.M != b.M || a.block != b.block || a.n_salient != b.n_salient)
        return STB_EINVAL;
    int herr = 0;
    rc = stb_tile_gpu(src, dst, stream, &herr);
    if (rc == STB_EHIP) g_last_hip_error = herr;
    return rc;
}

extern "C" int64_t stb_pack_device_workspace_bytes(const stb_cfg_t* cfg, int32_t si_per_block) {
    stb_layout_t probe;
    const int rc = stb_layout_sizes(cfg, &probe);       // validates cfg
    if (rc) return rc;
    return stb_pack_gpu_workspace(cfg, si_per_block != 0);
}

extern "C" int stb_pack_device(const float* W, const float* xnorm, const uint32_t* sal_bitmap, const stb_layout_t* out,
                               int32_t si_per_block, void* workspace, int64_t workspace_bytes, void* stream) {
    if (!W || !xnorm || !sal_bitmap || !out || !workspace) return STB_ENULL;
    const int rc0 = stb_layout_check(out);
    if (rc0) return rc0;
    if (out->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    if ((uintptr_t)W % 16 || (uintptr_t)xnorm % 4 || (uintptr_t)sal_bitmap % 4 || (uintptr_t)workspace % 256) return STB_EALIGN;
    if (workspace_bytes < stb_pack_gpu_workspace(&out->cfg, si_per_block != 0)) return STB_EINVAL;
    int herr = 0;
    const int rc = stb_pack_gpu(W, xnorm, sal_bitmap, out, si_per_block != 0, workspace, stream, &herr);
    if (rc == STB_EHIP) g_last_hip_error = herr;
    return rc;
}


extern "C" int64_t stb_pack_obc_hybrid_workspace_bytes(const stb_cfg_t* cfg) {
    stb_layout_t tmp;
    const int rc = stb_layout_sizes(cfg, &tmp);
    if (rc) return rc;
    return stb_pack_obc_gpu_workspace(cfg);
}

extern "C" int stb_pack_obc_hybrid(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                                   stb_layout_t* out, int32_t n_threads, void* workspace, int64_t workspace_bytes,
                                   void* stream) {
    if (!Hc) return stb_pack_obc(W, nullptr, xnorm, sal_bitmap, out, n_threads);     // no compensation: nothing for the GPU
    if (!W || !xnorm || !sal_bitmap || !out || !workspace) return STB_ENULL;
    const int rc0 = stb_layout_check(out);
    if (rc0) return rc0;
    if (out->kind != STB_KIND_ROWMAJOR) return STB_EINVAL;
    if ((uintptr_t)workspace % 256) return STB_EALIGN;
    if (workspace_bytes < stb_pack_obc_gpu_workspace(&out->cfg)) return STB_EINVAL;
    int herr = 0;
    const int rc = stb_pack_obc_gpu(W, Hc, xnorm, sal_bitmap, out, n_threads, workspace, stream, &herr);
    if (rc == STB_EHIP) g_last_hip_error = herr;
    return rc;
}

static std::atomic<int> g_override[4] = {{0}, {0}, {0}, {0}};

extern "C" int stb_kernel_override(int which) { return which >= 0 && which < 4 ? g_override[which].load(std::memory_order_relaxed) : 0; }

extern "C" int stb_set_kernel_override(int32_t gemv_kernel, int32_t gemv_visits, int32_t gemv_splits, int32_t gemm_kernel) {
    if (gemv_kernel < 0 || gemv_kernel > 1 || gemv_visits < 0 || gemv_visits > 8 || gemv_splits < 0 || gemv_splits > 64 ||
        gemm_kernel < 0 || gemm_kernel > 4)
        return STB_EINVAL;
    g_override[0].store(gemv_kernel, std::memory_order_relaxed);
    g_override[1].store(gemv_visits, std::memory_order_relaxed);
    g_override[2].store(gemm_kernel, std::memory_order_relaxed);
    g_override[3].store(gemv_splits, std::memory_order_relaxed);
    return STB_OK;
}

extern "C" int stb_probe_read(const void* src, int64_t bytes, void* sink, void* stream) {
    if (!src || !sink) return STB_ENULL;
    if (bytes < 16 || bytes % 16) return STB_EINVAL;
    if ((uintptr_t)src % 16 || (uintptr_t)sink % 4) return STB_EALIGN;
    hipLaunchKernelGGL(probe_read_kernel, dim3(1024), dim3(512), 0, (hipStream_t)stream, (const uint4*)src, bytes / 16,
                       (uint32_t*)sink);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? STB_OK : hip_fail(e);
}

extern "C" int stb_probe_mfma(int32_t kind, int32_t valu, int32_t steps, int32_t n_workgroups, void* sink, void* stream) {
    if (!sink) return STB_ENULL;
    if (steps < 1 || n_workgroups < 1 || n_workgroups > 65536) return STB_EINVAL;
    if ((uintptr_t)sink % 16) return STB_EALIGN;
    int herr = 0;
    const int rc = stb_tiled_probe_mfma(kind, valu, steps, n_workgroups, sink, stream, &herr);
    if (rc == STB_EHIP) g_last_hip_error = herr;
    return rc;
}

extern "C" int stb_dequant(const stb_layout_t* dev, float* W_hat_dev, void* stream) {
    if (!W_hat_dev) return STB_ENULL;
    int rc = stb_layout_check(dev);
    if (rc) return rc;
    if ((uintptr_t)W_hat_dev % 16) return STB_EALIGN;
    if (dev->kind == STB_KIND_TILED) {
        int herr = 0;
        rc = stb_tiled_dequant(dev, W_hat_dev, stream, &herr);
        if (rc == STB_EHIP) g_last_hip_error = herr;
        return rc;
    }
    const Planes p = make_planes(dev);
    const int64_t threads = (int64_t)p.n * p.wpr;
    const int blocks = (int)((threads + 255) / 256);
    hipLaunchKernelGGL(dequant_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, p, W_hat_dev);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? STB_OK : hip_fail(e);
}

extern "C" int stb_code24_index(const stb_layout_t* dev, uint16_t* E_dev, void* stream) {
    if (!E_dev) return STB_ENULL;
    int rc = stb_layout_check(dev);
    if (rc) return rc;
    if (dev->kind != STB_KIND_TILED) return STB_EINVAL;
    if (dev->cfg.N != 2 || dev->cfg.M != 4) return STB_EUNSUPPORTED;
    if ((uintptr_t)E_dev % 16) return STB_EALIGN;
    int herr = 0;
    rc = stb_tiled_meta_index(dev, E_dev, stream, &herr);
    if (rc == STB_EHIP) g_last_hip_error = herr;
    return rc;
}

// Batches above 16 on layers that the dense matrix instruction serves: one pass of the prefill kernel's small-token
// form instead of two passes of the decode kernel (the weights are expanded once for all rows of x).  Its scratch
// sits behind the decode kernel's, whose arrival counters must stay zero.
static bool gemv_takes_gemm(const stb_layout_t* L, int B) {
    return B > 16 && L->kind == STB_KIND_TILED && !(L->cfg.N == 2 && L->cfg.M == 4) &&
           stb_kernel_override(0) == 0 && stb_kernel_override(1) == 0 && stb_kernel_override(2) == 0 && stb_kernel_override(3) == 0;
}
static int64_t gemv_area(const stb_layout_t* L) { return (stb_tiled_gemv_workspace(L->n_row_tiles, L->n_super) + 255) / 256 * 256; }

extern "C" int64_t stb_gemv_workspace_bytes(const stb_cfg_t* cfg, int32_t B) {
    stb_layout_t tmp;
    int rc = stb_tiled_sizes(cfg, &tmp);
    if (rc) return rc;
    if (B < 1 || B > STB_MAX_BATCH) return STB_EINVAL;
    const int64_t decode = stb_tiled_gemv_workspace(tmp.n_row_tiles, tmp.n_super);
    if (B <= 16 || (cfg->N == 2 && cfg->M == 4) || stb_tiled_slots(cfg) == 0) return decode;
    tmp.max_sal_half = 8 * tmp.sal_chunks;             // sized for any placement of the salient columns
    return gemv_area(&tmp) + stb_tiled_gemm_workspace(&tmp, B);
}

// stb_gemv with the partial sums of the column splits at byte offset part_off of the workspace (-1: directly behind
// the arrival counters, the layout stb_gemv documents).
static int gemv_impl(const stb_layout_t* dev, const void* x, int32_t B, void* y, int32_t y_fp32,
                     void* workspace, int64_t workspace_bytes, int64_t part_off, void* stream) {
    if (!x || !y) return STB_ENULL;
    int rc = stb_layout_check(dev);
    if (rc) return rc;
    if (B < 1 || B > STB_MAX_BATCH || (y_fp32 != 0 && y_fp32 != 1) || workspace_bytes < 0) return STB_EINVAL;
    if ((uintptr_t)x % 16 || (uintptr_t)y % 4) return STB_EALIGN;
    if (dev->kind == STB_KIND_TILED) {
        if (part_off < 0 && gemv_takes_gemm(dev, B) && workspace && (uintptr_t)workspace % 256 == 0 &&
            workspace_bytes >= gemv_area(dev) + stb_tiled_gemm_workspace(dev, B)) {
            int herr = 0;
            const int64_t off = gemv_area(dev);
            rc = stb_tiled_gemm(dev, x, B, y, y_fp32, (char*)workspace + off, workspace_bytes - off, stream, &herr);
            if (rc == STB_EHIP) g_last_hip_error = herr;
            if (rc != STB_EUNSUPPORTED) return rc;
        }
        // the decode kernel takes up to 16 rows of x per launch
        for (int done = 0; done < B; done += 16) {
            const int nb = B - done < 16 ? B - done : 16;
            const void* xb = (const __half*)x + (size_t)done * dev->cfg.k_in;
            void* yb = y_fp32 ? (void*)((float*)y + (size_t)done * dev->cfg.n_out)
                              : (void*)((__half*)y + (size_t)done * dev->cfg.n_out);
            int herr = 0;
            rc = stb_tiled_gemv(dev, xb, nb, yb, y_fp32, workspace, workspace_bytes, part_off, stream, &herr);
            if (rc == STB_EHIP) g_last_hip_error = herr;
            if (rc) return rc;
        }
        return STB_OK;
    }
    const Planes p = make_planes(dev);
    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    int done = 0;
    // batch rows are processed in chunks of 8, 4, 2, 1 columns of x
    while (done < B && e == hipSuccess) {
        const int left = B - done;
        const __half* xb = (const __half*)x + (size_t)done * p.k;
        void* yb = y_fp32 ? (void*)((float*)y + (size_t)done * p.n) : (void*)((__half*)y + (size_t)done * p.n);
        // (the kernel with x in LDS where that many rows of x fit, the older one otherwise)
        if (left >= 8 && gemv_rows_lds(p, 8) <= GEMV_ROWS_LDS_MAX) { e = launch_gemv_rows<8>(p, xb, yb, y_fp32, s); done += 8; }
        else if (left >= 4 && gemv_rows_lds(p, 4) <= GEMV_ROWS_LDS_MAX) { e = launch_gemv_rows<4>(p, xb, yb, y_fp32, s); done += 4; }
        else if (left >= 2 && gemv_rows_lds(p, 2) <= GEMV_ROWS_LDS_MAX) { e = launch_gemv_rows<2>(p, xb, yb, y_fp32, s); done += 2; }
        else if (gemv_rows_lds(p, 1) <= GEMV_ROWS_LDS_MAX) { e = launch_gemv_rows<1>(p, xb, yb, y_fp32, s); done += 1; }
        else if (left >= 8) { e = launch_gemv_generic<8>(p, xb, yb, y_fp32, s); done += 8; }
        else if (left >= 4) { e = launch_gemv_generic<4>(p, xb, yb, y_fp32, s); done += 4; }
        else if (left >= 2) { e = launch_gemv_generic<2>(p, xb, yb, y_fp32, s); done += 2; }
        else { e = launch_gemv_generic<1>(p, xb, yb, y_fp32, s); done += 1; }
    }
    return e == hipSuccess ? STB_OK : hip_fail(e);
}

extern "C" int stb_gemv(const stb_layout_t* dev, const void* x, int32_t B, void* y, int32_t y_fp32,
                        void* workspace, int64_t workspace_bytes, void* stream) {
    return gemv_impl(dev, x, B, y, y_fp32, workspace, workspace_bytes, -1, stream);
}

// ------------------------------------------------------------------------------------------------
// stb_gemv_static: the scratch lives in a device array of this library instead of a caller's buffer.
// ------------------------------------------------------------------------------------------------
// [0, STB_STATIC_COUNTER_BYTES): arrival counters (zero when the library is loaded; every call leaves them zero);
// behind them the partial sums of the column splits (no initialisation needed).
static __device__ __align__(256) unsigned char scratch[STB_GEMV_STATIC_SCRATCH_BYTES];
constexpr int64_t STB_STATIC_COUNTER_BYTES = 65536;
constexpr int STB_STATIC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[STB_STATIC_MAX_DEVICES] = {};   // the array's address on each device, once looked up

// The device address of `scratch` on the current device (each GPU holds its own copy of the array).  The array's name
// is a host-side handle: only the pointer that hipGetSymbolAddress returns may be given to a kernel.
static int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= STB_STATIC_MAX_DEVICES) return STB_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!ptr || (uintptr_t)ptr % 256) return STB_EALIGN;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return STB_OK;
}

extern "C" int stb_gemv_static(const stb_layout_t* dev, const void* x, int32_t B, void* y, int32_t y_fp32, void* stream) {
    if (!dev) return STB_ENULL;
    // the counters of ceil(n / 16) row tiles must fit their fixed area; the partial sums are checked by the launcher
    // against what is left of the array (it knows how many column splits it takes)
    if (dev->kind == STB_KIND_TILED && 4 * (int64_t)dev->n_row_tiles > STB_STATIC_COUNTER_BYTES) return STB_ETOOBIG;
    void* ptr = nullptr;
    int rc = static_scratch(&ptr);
    if (rc) return rc;
    rc = gemv_impl(dev, x, B, y, y_fp32, ptr, STB_GEMV_STATIC_SCRATCH_BYTES, STB_STATIC_COUNTER_BYTES, stream);
    // the only size check a valid layout can fail with this buffer is the one on the partial sums
    if (rc == STB_EINVAL && dev->kind == STB_KIND_TILED && stb_layout_check(dev) == STB_OK && x && y && B >= 1 &&
        B <= STB_MAX_BATCH && (y_fp32 == 0 || y_fp32 == 1))
        return STB_ETOOBIG;
    return rc;
}

// Each layer of a batched call owns a slice of the workspace: its arrival counters, then its partial sums.
static int64_t round_up256_(int64_t v) { return (v + 255) / 256 * 256; }
static int64_t batched_slice(const stb_cfg_t* cfg, int32_t B, int64_t* counter_bytes) {
    stb_layout_t tmp;
    int rc = stb_tiled_sizes(cfg, &tmp);
    if (rc) return rc;
    if (B < 1 || B > STB_MAX_BATCH) return STB_EINVAL;
    const int64_t total = stb_tiled_gemv_workspace(tmp.n_row_tiles, tmp.n_super);
    if (counter_bytes) *counter_bytes = round_up256_(4 * (int64_t)tmp.n_row_tiles);
    return round_up256_(total);
}

extern "C" int64_t stb_gemv_batched_workspace_bytes(int32_t n_layers, const stb_cfg_t* const* cfgs, int32_t B) {
    if (!cfgs) return STB_ENULL;
    if (n_layers < 1) return STB_EINVAL;
    int64_t total = 0;
    for (int l = 0; l < n_layers; l++) {
        if (!cfgs[l]) return STB_ENULL;
        const int64_t b = batched_slice(cfgs[l], B, nullptr);
        if (b < 0) return b;
        total += b;
    }
    return total;
}

extern "C" int stb_gemv_batched(int32_t n_layers, const stb_layout_t* const* dev, const void* const* x,
                                int32_t B, void* const* y, int32_t y_fp32, void* workspace,
                                int64_t workspace_bytes, void* stream) {
    if (!dev || !x || !y) return STB_ENULL;
    if (n_layers < 1 || B < 1 || B > STB_MAX_BATCH || (y_fp32 != 0 && y_fp32 != 1) || workspace_bytes < 0) return STB_EINVAL;
    if (workspace && (uintptr_t)workspace % 256) return STB_EALIGN;
    // validate everything before the first launch; cut the workspace into one slice per layer
    std::vector<int64_t> off(n_layers), cnt_bytes(n_layers), len(n_layers);
    int64_t total = 0;
    bool grouped = true;
    for (int l = 0; l < n_layers; l++) {
        if (!dev[l] || !x[l] || !y[l]) return STB_ENULL;
        const int rc = stb_layout_check(dev[l]);
        if (rc) return rc;
        if ((uintptr_t)x[l] % 16 || (uintptr_t)y[l] % 4) return STB_EALIGN;
        const int64_t b = batched_slice(&dev[l]->cfg, B, &cnt_bytes[l]);
        if (b < 0) return (int)b;
        off[l] = total; len[l] = b;
        total += b;
        if (dev[l]->kind != STB_KIND_TILED || !stb_tiled_supported(dev[l])) grouped = false;
    }
    const bool have_ws = workspace && workspace_bytes >= total;
    if (!have_ws && workspace && workspace_bytes > 0) return STB_EINVAL;      // a workspace that is too small
    if (grouped && stb_kernel_override(0) == 0) {
        // layers in runs of up to 8 per launch, batch rows in chunks of 16
        bool fell_back = false;
        for (int l0 = 0; l0 < n_layers && !fell_back; l0 += 8) {
            const int nl = n_layers - l0 < 8 ? n_layers - l0 : 8;
            for (int done = 0; done < B; done += 16) {
                const int nb = B - done < 16 ? B - done : 16;
                const void* xs[8]; void* ys[8]; void* cnts[8]; void* parts[8]; int64_t pbytes[8];
                for (int j = 0; j < nl; j++) {
                    const stb_layout_t* L = dev[l0 + j];
                    xs[j] = (const __half*)x[l0 + j] + (size_t)done * L->cfg.k_in;
                    ys[j] = y_fp32 ? (void*)((float*)y[l0 + j] + (size_t)done * L->cfg.n_out)
                                   : (void*)((__half*)y[l0 + j] + (size_t)done * L->cfg.n_out);
                    cnts[j] = have_ws ? (char*)workspace + off[l0 + j] : nullptr;
                    parts[j] = have_ws ? (char*)workspace + off[l0 + j] + cnt_bytes[l0 + j] : nullptr;
                    pbytes[j] = have_ws ? len[l0 + j] - cnt_bytes[l0 + j] : 0;
                }
                int herr = 0;
                const int rc = stb_tiled_gemv24_group(nl, dev + l0, xs, nb, ys, y_fp32, cnts, parts, pbytes, stream, &herr);
                if (rc == STB_EUNSUPPORTED && l0 == 0 && done == 0) { fell_back = true; break; }   // nothing was launched yet
                if (rc == STB_EHIP) g_last_hip_error = herr;
                if (rc) return rc;
            }
        }
        if (!fell_back) return STB_OK;
    }
    for (int l = 0; l < n_layers; l++) {
        const int rc = gemv_impl(dev[l], x[l], B, y[l], y_fp32, have_ws ? (char*)workspace + off[l] : nullptr,
                                 have_ws ? len[l] : 0, -1, stream);
        if (rc) return rc;
    }
    return STB_OK;
}

extern "C" int64_t stb_gemm_workspace_bytes(const stb_layout_t* layout, int32_t T) {
    if (!layout) return STB_ENULL;
    stb_layout_t ref;
    int rc = layout->kind == STB_KIND_TILED ? stb_tiled_sizes(&layout->cfg, &ref)
                                            : (layout->kind == STB_KIND_ROWMAJOR ? stb_layout_sizes(&layout->cfg, &ref) : STB_EINVAL);
    if (rc) return rc;
    if (T < 1) return STB_EINVAL;
    if (layout->kind == STB_KIND_ROWMAJOR || !stb_tiled_supported(layout)) return 0;
    if (layout->max_sal_half < 0 || layout->max_sal_half > 8 * ref.sal_chunks) return STB_EINVAL;
    stb_layout_t tmp = ref;
    tmp.max_sal_half = layout->max_sal_half;
    return stb_tiled_gemm_workspace(&tmp, T);      // gathered salient columns of X, partial tiles of a K split
}

extern "C" int stb_gemm(const stb_layout_t* dev, const void* X, int32_t T, void* Y, int32_t y_fp32,
                        void* workspace, int64_t workspace_bytes, void* stream) {
    if (!X || !Y) return STB_ENULL;
    int rc = stb_layout_check(dev);
    if (rc) return rc;
    if (T < 1 || (y_fp32 != 0 && y_fp32 != 1) || workspace_bytes < 0) return STB_EINVAL;
    if ((uintptr_t)X % 16 || (uintptr_t)Y % 4) return STB_EALIGN;
    if (dev->kind == STB_KIND_TILED) {
        int herr = 0;
        rc = stb_tiled_gemm(dev, X, T, Y, y_fp32, workspace, workspace_bytes, stream, &herr);
        if (rc == STB_EHIP) g_last_hip_error = herr;
        return rc;
    }
    const Planes p = make_planes(dev);
    dim3 grid((p.n + GN - 1) / GN, (T + GT - 1) / GT);
    hipLaunchKernelGGL(gemm_generic_kernel, grid, dim3(256), 0, (hipStream_t)stream, p, (const __half*)X, T,
                       Y, y_fp32);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? STB_OK : hip_fail(e);
}
