// The packer of stb_pack on the GPU: Standardized Importance (Eq. 3), N:M mask (Sec. 3.1), residual binarisation of the
// kept salient weights (Eq. 4), break-point search and trisection of the kept non-salient ones (Alg. 2, Eq. 5-6), bit
// planes of STB1 in device memory.
//
// The result must agree with the host packer bit for bit, so every floating-point value is computed by the same
// expression in the same order as there: float64 throughout, sums over a row's columns from left to right, sums over
// rows from top to bottom, no fused multiply-add (contraction is switched off for this file), and the three roundings
// of a scale (fp64 -> fp32 -> fp16) through the integer routine the host uses.  Parallelism comes from what the
// definition leaves independent: rows, columns, blocks and break-point candidates; a sum over n rows is one thread's
// loop.  Division and square root of float64 are correctly rounded on this hardware, as on the host.
#include <hip/hip_runtime.h>

#include <vector>

#include "stb_f16.h"
#include "stb_internal.h"

#pragma clang fp contract(off)

namespace {

constexpr int CAND = 160;                  // break-point candidates of Alg. 2
constexpr uint32_t ST_NONFINITE = 1u, ST_SALIENT = 2u;

struct PK {
    const float* W;
    const float* xnorm;
    const uint32_t* sal;
    int n, k, N, M, nb, nbS, per_block, region_mode, n_salient;
    uint8_t* mask;
    uint8_t* sign;
    uint8_t* region;
    uint32_t* res_sign;
    uint16_t* scales;
    uint16_t* res_scale;
    uint32_t* sal_out;
    uint32_t* prefix;
    int64_t mask_stride, sign_stride, region_stride, res_stride;
    uint32_t* status;       // [0] error bits
    double* rs;             // [n][nbS] row sums of |W| (whole row, or per block)
    double* cs;             // [k] column sums of |W|
    double* rowacc;         // [n][nbS]
    double* stats;          // [nbS][2] mean, deviation
    uint32_t* mxbits;       // [nb] largest kept non-salient magnitude of the block (fp32 bits)
    uint32_t* cnt;          // [nb] number of kept non-salient weights of the block
    double* p12;            // [nb][2] break points
    uint32_t* hist;         // [nb][2][256]
    uint32_t* sel;          // [nb][2][2] prefix, remaining rank of the two order statistics
    double* err;            // [blocks of a batch][n][CAND]
};

__device__ inline bool sal_bit(const uint32_t* bm, int j) { return (bm[j >> 5] >> (j & 31)) & 1u; }

__device__ inline double mu_of(double a, double rs, double cs) {
    const double t1 = rs > 0.0 ? a / rs : 0.0;
    const double t2 = cs > 0.0 ? a / cs : 0.0;
    return t1 + t2;
}

// ---- Standardized Importance: sums ------------------------------------------------------------------------------
// One thread per row: |w| from left to right.  MODE 0: the row sums themselves (and the finiteness check);
// 1: the sum of mu over the row; 2: the sum of (mu - mean)^2.
template <int MODE>
__global__ void k_row_pass(PK a) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= a.n) return;
    const float4* w4 = reinterpret_cast<const float4*>(a.W + (size_t)i * a.k);
    double s = 0.0;
    bool bad = false;
    for (int q = 0; q < a.nb; q++) {
        const int sc = a.per_block ? q : 0;
        double rsv = 0.0, mean = 0.0;
        if (MODE >= 1) rsv = a.rs[(size_t)i * a.nbS + sc];
        if (MODE == 2) mean = a.stats[2 * sc];
        for (int c4 = 0; c4 < 32; c4++) {
            const float4 v = w4[q * 32 + c4];
            const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const double av = fabs((double)e[u]);
                if (MODE == 0) {
                    bad |= !__builtin_isfinite(e[u]);
                    s += av;
                } else {
                    const double mu = mu_of(av, rsv, a.cs[q * 128 + c4 * 4 + u]);
                    if (MODE == 1) s += mu;
                    else { const double d = mu - mean; s += d * d; }
                }
            }
        }
        if (a.per_block) {
            (MODE == 0 ? a.rs : a.rowacc)[(size_t)i * a.nbS + q] = s;
            s = 0.0;
        }
    }
    if (!a.per_block) (MODE == 0 ? a.rs : a.rowacc)[i] = s;
    if (MODE == 0 && bad) atomicOr(a.status, ST_NONFINITE);
}

// One thread per column: |w| from the top row down.  Also checks xnorm.
__global__ void k_col_sums(PK a) {
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= a.k) return;
    double s = 0.0;
#pragma unroll 32
    for (int i = 0; i < a.n; i++) s += fabs((double)a.W[(size_t)i * a.k + j]);
    a.cs[j] = s;
    const float x = a.xnorm[j];
    if (!(x >= 0.0f) || !__builtin_isfinite(x)) atomicOr(a.status, ST_NONFINITE);
}

// One thread per scope (the layer, or a block): the row accumulators from the top row down.  MODE 0 -> mean, 1 -> deviation.
template <int MODE>
__global__ void k_total(PK a) {
    const int sc = blockIdx.x * blockDim.x + threadIdx.x;
    if (sc >= a.nbS) return;
    double tot = 0.0;
#pragma unroll 32
    for (int i = 0; i < a.n; i++) tot += a.rowacc[(size_t)i * a.nbS + sc];
    const double cnt = (double)a.n * (double)(a.per_block ? STB_BLOCK : a.k);
    if (MODE == 0) a.stats[2 * sc] = tot / cnt;
    else {
        double sd = sqrt(tot / cnt);
        if (sd == 0.0) sd = 1.0;
        a.stats[2 * sc + 1] = sd;
    }
}

// ---- N:M mask: one thread per (row, 8 columns) -------------------------------------------------------------------
__global__ void k_mask(PK a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int g8n = a.k / 8;
    if (idx >= (int64_t)a.n * g8n) return;
    const int i = (int)(idx / g8n), g8 = (int)(idx % g8n);
    const int j0 = 8 * g8, q = j0 / STB_BLOCK, sc = a.per_block ? q : 0;
    const double rsv = a.rs[(size_t)i * a.nbS + sc], mean = a.stats[2 * sc], sd = a.stats[2 * sc + 1];
    double s[8];
#pragma unroll
    for (int p = 0; p < 8; p++) {
        const double av = fabs((double)a.W[(size_t)i * a.k + j0 + p]);
        s[p] = ((mu_of(av, rsv, a.cs[j0 + p]) - mean) / sd) * (double)a.xnorm[j0 + p];
    }
    uint32_t byte = 0;
    const int M = a.M;
    for (int g = 0; g < 8; g += M)
        for (int p = 0; p < M; p++) {
            int better = 0;                 // entries that rank before p: a higher score, or an equal one further left
            for (int o = 0; o < M; o++)
                if (s[g + o] > s[g + p] || (s[g + o] == s[g + p] && o < p)) better++;
            if (better < a.N) byte |= 1u << (g + p);
        }
    a.mask[(size_t)i * a.mask_stride + g8] = (uint8_t)byte;
}

// ---- per (row, block): salient part, largest non-salient magnitude ------------------------------------------------
__global__ void k_block_salient(PK a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.nb) return;
    const int i = (int)(idx / a.nb), q = (int)(idx % a.nb), c0 = q * STB_BLOCK;
    const float* w = a.W + (size_t)i * a.k + c0;
    const uint8_t* mrow = a.mask + (size_t)i * a.mask_stride + 16 * q;
    uint32_t m[4], sb[4];
    for (int u = 0; u < 4; u++) {
        m[u] = (uint32_t)mrow[4 * u] | ((uint32_t)mrow[4 * u + 1] << 8) | ((uint32_t)mrow[4 * u + 2] << 16) | ((uint32_t)mrow[4 * u + 3] << 24);
        sb[u] = a.sal[4 * q + u];
    }
    double so = 0.0;
    int co = 0;
    uint32_t mx = 0, members = 0;
    const float4* w4 = reinterpret_cast<const float4*>(w);          // 16 bytes per load: a cache line serves 8 loads, not 32
    for (int c4 = 0; c4 < STB_BLOCK / 4; c4++) {
        const float4 v = w4[c4];
        const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int c = 4 * c4 + u;
            if (!((m[c >> 5] >> (c & 31)) & 1u)) continue;
            const float wf = e[u];
            if ((sb[c >> 5] >> (c & 31)) & 1u) { so += fabs((double)wf); co++; }
            else {
                const uint32_t bits = __float_as_uint(fabsf(wf));      // magnitudes order like their bit patterns
                mx = bits > mx ? bits : mx;
                members++;
            }
        }
    }
    const uint16_t ao16 = stb_f64_to_f16_bits(co > 0 ? so / (double)co : 0.0);
    const double ao = (double)stb_f16_bits_to_f32(ao16);
    double sr = 0.0;
    if (co > 0) {
        int u = (int)a.prefix[q];           // index of the block's first salient column among all salient columns
        uint32_t* trow = a.res_sign + (size_t)i * (a.res_stride / 4);
        for (int c = 0; c < STB_BLOCK; c++) {
            if (!((sb[c >> 5] >> (c & 31)) & 1u)) continue;
            if ((m[c >> 5] >> (c & 31)) & 1u) {
                const double wd = (double)w[c];
                const double sg = w[c] >= 0.0f ? 1.0 : -1.0;
                const double r = wd - ao * sg;
                sr += fabs(r);
                if (r >= 0.0) atomicOr(trow + (u >> 5), 1u << (u & 31));     // neighbouring blocks share words
            }
            u++;
        }
    }
    a.scales[((size_t)i * a.nb + q) * 4 + 3] = ao16;
    a.res_scale[(size_t)i * a.nb + q] = stb_f64_to_f16_bits(co > 0 ? sr / (double)co : 0.0);
    if (mx) atomicMax(a.mxbits + q, mx);
    if (members) atomicAdd(a.cnt + q, members);
}

// ---- break-point search (Alg. 2 NonSalientAwareQuant) --------------------------------------------------------------
__device__ inline void candidate(int t, double mx, double& q1, double& q2, bool& skip) {
    const double step = (0.9 - 0.1) / 159.0;
    const double c = (t == CAND - 1) ? 0.9 : (double)t * step + 0.1;
    q1 = c * mx;
    q2 = 2.0 * q1;
    skip = q2 > 0.9 * mx;
}

// One thread per (row, candidate, block of the batch): the error of binarising the row's three regions separately
// (Eq. 5-6), its kept non-salient magnitudes taken from left to right.  grid = (ceil(n / 4), 3, blocks), block = (64, 4).
__global__ void k_candidate_errors(PK a, int q_first) {
    const int i = blockIdx.x * blockDim.y + threadIdx.y;
    const int t = blockIdx.y * 64 + threadIdx.x;
    const int qb = blockIdx.z, q = q_first + qb;
    if (i >= a.n || t >= CAND) return;
    const double mx = (double)__uint_as_float(a.mxbits[q]);
    double p1, p2;
    bool skip;
    candidate(t, mx, p1, p2, skip);
    double* out = a.err + ((size_t)qb * a.n + i) * CAND + t;
    if (skip) { *out = 0.0; return; }           // never read
    const float* w = a.W + (size_t)i * a.k + q * STB_BLOCK;
    const uint8_t* mrow = a.mask + (size_t)i * a.mask_stride + 16 * q;
    double sum0 = 0.0, sum1 = 0.0, sum2 = 0.0;
    int n0 = 0, n1 = 0, n2 = 0;
    for (int b = 0; b < 16; b++) {
        const uint32_t keep = mrow[b] & ~((a.sal[4 * q + (b >> 2)] >> (8 * (b & 3))) & 0xFFu);
        for (int c = 0; c < 8; c++) {
            if (!((keep >> c) & 1u)) continue;
            const double av = fabs((double)w[8 * b + c]);
            if (av > p2) { sum2 += av; n2++; }
            else if (av > p1) { sum1 += av; n1++; }
            else { sum0 += av; n0++; }
        }
    }
    const double al0 = n0 > 0 ? sum0 / (double)n0 : 0.0;
    const double al1 = n1 > 0 ? sum1 / (double)n1 : 0.0;
    const double al2 = n2 > 0 ? sum2 / (double)n2 : 0.0;
    double row = 0.0;
    for (int b = 0; b < 16; b++) {
        const uint32_t keep = mrow[b] & ~((a.sal[4 * q + (b >> 2)] >> (8 * (b & 3))) & 0xFFu);
        for (int c = 0; c < 8; c++) {
            if (!((keep >> c) & 1u)) continue;
            const double av = fabs((double)w[8 * b + c]);
            const double d = av - (av > p2 ? al2 : (av > p1 ? al1 : al0));
            row += d * d;
        }
    }
    *out = row;
}

// One workgroup per block of the batch, one thread per candidate: the rows' errors from the top row down, then the
// first strict minimum over the candidates in their order.
__global__ void k_pick_breakpoints(PK a, int q_first) {
    __shared__ double tot[CAND];
    const int t = threadIdx.x, qb = blockIdx.x, q = q_first + qb;
    const double mx = (double)__uint_as_float(a.mxbits[q]);
    double p1, p2;
    bool skip;
    if (t < CAND) {
        candidate(t, mx, p1, p2, skip);
        double s = 0.0;
        if (!skip) {
            const double* e = a.err + (size_t)qb * a.n * CAND + t;
#pragma unroll 32
            for (int i = 0; i < a.n; i++) s += e[(size_t)i * CAND];           // the loads run ahead, the additions stay in order
        }
        tot[t] = s;
    }
    __syncthreads();
    if (t == 0) {
        double best = __builtin_inf(), b1 = 0.0, b2 = 0.0;
        for (int c = 0; c < CAND; c++) {
            candidate(c, mx, p1, p2, skip);
            if (skip) continue;
            if (tot[c] < best) { best = tot[c]; b1 = p1; b2 = p2; }
        }
        a.p12[2 * q] = b1;
        a.p12[2 * q + 1] = b2;
    }
}

// ---- tertile split (region_mode 1): two order statistics per block by radix selection on the fp32 bit patterns ----
// sel[q][s] = {bits fixed so far, rank still to find among the values that share them}
__global__ void k_select_init(PK a) {
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= a.nb) return;
    const uint32_t m = a.cnt[q];
    a.sel[4 * q + 0] = 0; a.sel[4 * q + 1] = m ? (m + 2) / 3 - 1 : 0;
    a.sel[4 * q + 2] = 0; a.sel[4 * q + 3] = m ? (uint32_t)((2ull * m + 2) / 3 - 1) : 0;
}

// One thread per (row, block): counts, for both statistics, the next 8 bits of the values whose higher bits match.
__global__ void k_select_hist(PK a, int pass) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.nb) return;
    const int i = (int)(idx / a.nb), q = (int)(idx % a.nb);
    const float* w = a.W + (size_t)i * a.k + q * STB_BLOCK;
    const uint8_t* mrow = a.mask + (size_t)i * a.mask_stride + 16 * q;
    const int shift = 24 - 8 * pass;
    const uint32_t pre0 = a.sel[4 * q + 0], pre1 = a.sel[4 * q + 2];
    const float4* w4 = reinterpret_cast<const float4*>(w);
    for (int b = 0; b < 16; b++) {
        const uint32_t keep = mrow[b] & ~((a.sal[4 * q + (b >> 2)] >> (8 * (b & 3))) & 0xFFu);
        const float4 v0 = w4[2 * b], v1 = w4[2 * b + 1];
        const float e[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int c = 0; c < 8; c++) {
            if (!((keep >> c) & 1u)) continue;
            const uint32_t bits = __float_as_uint(fabsf(e[c]));
            const uint32_t hi = pass == 0 ? 0u : bits >> (shift + 8), dig = (bits >> shift) & 255u;
            if (hi == pre0) atomicAdd(a.hist + ((size_t)q * 2 + 0) * 256 + dig, 1u);
            if (hi == pre1) atomicAdd(a.hist + ((size_t)q * 2 + 1) * 256 + dig, 1u);
        }
    }
}

// One thread per (block, statistic): the digit whose bucket holds the rank; clears the histogram for the next pass.
__global__ void k_select_step(PK a, int pass) {
    const int id = blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= 2 * a.nb) return;
    uint32_t* h = a.hist + (size_t)id * 256;
    uint32_t rank = a.sel[2 * id + 1], run = 0;
    int dig = 255;
    bool found = false;
    for (int d = 0; d < 256; d++) {
        const uint32_t c = h[d];
        if (!found && rank < run + c) { dig = d; rank -= run; found = true; }
        run += c;
        h[d] = 0;
    }
    if (!found) { dig = 0; rank = 0; }             // an empty block
    a.sel[2 * id] = (a.sel[2 * id] << 8) | (uint32_t)dig;
    a.sel[2 * id + 1] = rank;
    if (pass == 3) {
        const int q = id >> 1;
        a.p12[2 * q + (id & 1)] = a.cnt[q] ? (double)__uint_as_float(a.sel[2 * id]) : 0.0;
    }
}

// ---- per (row, block): region ids, the three scales, sign and id bits of the block ---------------------------------
__global__ void k_assign(PK a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.nb) return;
    const int i = (int)(idx / a.nb), q = (int)(idx % a.nb);
    const float* w = a.W + (size_t)i * a.k + q * STB_BLOCK;
    const uint8_t* mrow = a.mask + (size_t)i * a.mask_stride + 16 * q;
    const double p1 = a.p12[2 * q], p2 = a.p12[2 * q + 1];
    const int sbytes = 16 * a.N / a.M, rbytes = 32 * a.N / a.M;
    uint8_t* srow = a.sign + (size_t)i * a.sign_stride + (size_t)q * sbytes;
    uint8_t* rrow = a.region + (size_t)i * a.region_stride + (size_t)q * rbytes;
    double sum[3] = {0.0, 0.0, 0.0};
    int c3[3] = {0, 0, 0};
    uint32_t sacc = 0, racc = 0;        // bits of the sign byte / id byte being filled
    int slot = 0;
    const float4* w4 = reinterpret_cast<const float4*>(w);
    for (int b = 0; b < 16; b++) {
        const uint32_t mb = mrow[b], sb = (a.sal[4 * q + (b >> 2)] >> (8 * (b & 3))) & 0xFFu;
        const float4 v0 = w4[2 * b], v1 = w4[2 * b + 1];
        const float e[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
        for (int c = 0; c < 8; c++) {
            if (!((mb >> c) & 1u)) continue;
            const float wf = e[c];
            uint32_t id = 3;
            if (!((sb >> c) & 1u)) {
                const double av = fabs((double)wf);
                id = av > p2 ? 2 : (av > p1 ? 1 : 0);
                if (id == 2) { sum[2] += av; c3[2]++; }
                else if (id == 1) { sum[1] += av; c3[1]++; }
                else { sum[0] += av; c3[0]++; }
            }
            if (wf >= 0.0f) sacc |= 1u << (slot & 7);
            racc |= id << ((slot & 3) * 2);
            slot++;
            if ((slot & 7) == 0) { srow[(slot >> 3) - 1] = (uint8_t)sacc; sacc = 0; }
            if ((slot & 3) == 0) { rrow[(slot >> 2) - 1] = (uint8_t)racc; racc = 0; }
        }
    }
    // a row keeps 128 N / M weights of every block, a multiple of 16: both accumulators are empty here
    if (slot != 8 * sbytes) atomicOr(a.status, ST_SALIENT << 1);
    for (int r = 0; r < 3; r++)
        a.scales[((size_t)i * a.nb + q) * 4 + r] = stb_f64_to_f16_bits(c3[r] > 0 ? sum[r] / (double)c3[r] : 0.0);
}

// ---- the salient bitmap and its per-block prefix; one thread ------------------------------------------------------
__global__ void k_salient_tables(PK a) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    uint32_t run = 0;
    for (int q = 0; q < a.nb; q++) {
        a.prefix[q] = run;
        for (int u = 0; u < 4; u++) {
            const uint32_t wv = a.sal[4 * q + u];
            a.sal_out[4 * q + u] = wv;
            run += (uint32_t)__popc(wv);
        }
    }
    a.prefix[a.nb] = run;
    if (run != (uint32_t)a.n_salient) atomicOr(a.status, ST_SALIENT);
}

inline int64_t up256(int64_t v) { return (v + 255) / 256 * 256; }

struct WsPlan {
    int64_t status, rs, cs, rowacc, stats, mxbits, cnt, p12, hist, sel, err, total;
    int batch;                  // blocks whose candidate errors are held at once
};

WsPlan plan_workspace(const stb_cfg_t& c, int per_block) {
    const int64_t n = c.n_out, k = c.k_in, nb = k / STB_BLOCK, nbS = per_block ? nb : 1;
    WsPlan p;
    int64_t o = 0;
    p.status = o; o += 256;
    p.rs = o; o += up256(n * nbS * 8);
    p.cs = o; o += up256(k * 8);
    p.rowacc = o; o += up256(n * nbS * 8);
    p.stats = o; o += up256(nbS * 16);
    p.mxbits = o; o += up256(nb * 4);
    p.cnt = o; o += up256(nb * 4);
    p.p12 = o; o += up256(nb * 16);
    p.hist = o; o += up256(nb * 2 * 256 * 4);
    p.sel = o; o += up256(nb * 16);
    // candidate errors: as many blocks at once as fit into 1 GiB, at least one
    const int64_t per_block_bytes = n * CAND * 8;
    int64_t batch = (1ll << 30) / per_block_bytes;
    batch = batch < 1 ? 1 : (batch > nb ? nb : batch);
    p.batch = (int)batch;
    p.err = o; o += up256(c.region_mode == 0 ? batch * per_block_bytes : 0);
    p.total = o;
    return p;
}

}  // namespace

extern "C" int64_t stb_pack_gpu_workspace(const stb_cfg_t* cfg, int per_block) {
    return plan_workspace(*cfg, per_block).total;
}

// ------------------------------------------------------------------------------------------------
// The compensation step of Alg. 1 on the GPU: the float64 working copy of W and the factor H^c stay in HBM, the host
// quantises block after block (stb_pack_obc_with) and sends each block's error matrix E.
//   W[i][j] -= sum_c E[i][c] * Hc[c0 + c][j]   for the columns j right of the block,
// the 128 terms in ascending c, one multiplication and one addition per term (no fused multiply-add: see the pragma
// at the top), the sum subtracted once -- the host loop's arithmetic, so the bytes that come out are the same.
// A workgroup takes OBC_TI rows x 256 columns: E's rows from LDS (every lane reads the same word), H^c coalesced.
// ------------------------------------------------------------------------------------------------
namespace {

constexpr int OBC_TI = 8;

__global__ __launch_bounds__(256) void k_obc_update(double* __restrict__ Wd, const double* __restrict__ E,
                                                    const double* __restrict__ Hc, int n, int k, int c0) {
    __shared__ double e[OBC_TI][STB_BLOCK];
    const int c1 = c0 + STB_BLOCK;
    const int i0 = (int)blockIdx.y * OBC_TI;
    for (int t = threadIdx.x; t < OBC_TI * STB_BLOCK; t += 256) {
        const int r = t / STB_BLOCK, c = t % STB_BLOCK;
        e[r][c] = i0 + r < n ? E[(size_t)(i0 + r) * STB_BLOCK + c] : 0.0;
    }
    __syncthreads();
    const int j = c1 + (int)blockIdx.x * 256 + (int)threadIdx.x;
    if (j >= k) return;
    double acc[OBC_TI];
#pragma unroll
    for (int r = 0; r < OBC_TI; r++) acc[r] = 0.0;
    const double* h = Hc + (size_t)c0 * k + j;
    for (int c = 0; c < STB_BLOCK; c++) {
        const double hv = h[(size_t)c * k];
#pragma unroll
        for (int r = 0; r < OBC_TI; r++) acc[r] += e[r][c] * hv;
    }
#pragma unroll
    for (int r = 0; r < OBC_TI; r++)
        if (i0 + r < n) Wd[(size_t)(i0 + r) * k + j] -= acc[r];
}

struct ObcGpu {
    int n, k;
    double* Wd;
    double* Hc;
    double* E;
    hipStream_t st;
    int hip_err;
};

int obc_fail(ObcGpu* g, hipError_t e) { g->hip_err = (int)e; return STB_EHIP; }

int obc_start(void* ctx, const double* Wd_host) {
    ObcGpu* g = (ObcGpu*)ctx;
    hipError_t e = hipMemcpyAsync(g->Wd, Wd_host, (size_t)g->n * g->k * 8, hipMemcpyHostToDevice, g->st);
    if (e == hipSuccess) e = hipStreamSynchronize(g->st);
    return e == hipSuccess ? STB_OK : obc_fail(g, e);
}

int obc_fetch(void* ctx, int q, double* Wd_host) {
    ObcGpu* g = (ObcGpu*)ctx;
    const size_t pitch = (size_t)g->k * 8, off = (size_t)q * STB_BLOCK;
    hipError_t e = hipMemcpy2DAsync(Wd_host + off, pitch, g->Wd + off, pitch, (size_t)STB_BLOCK * 8, (size_t)g->n,
                                    hipMemcpyDeviceToHost, g->st);
    if (e == hipSuccess) e = hipStreamSynchronize(g->st);      // the update kernels of the blocks before are done too
    return e == hipSuccess ? STB_OK : obc_fail(g, e);
}

int obc_update(void* ctx, int q, const double* E_host) {
    ObcGpu* g = (ObcGpu*)ctx;
    const int c1 = (q + 1) * STB_BLOCK;
    if (c1 >= g->k) return STB_OK;
    hipError_t e = hipMemcpyAsync(g->E, E_host, (size_t)g->n * STB_BLOCK * 8, hipMemcpyHostToDevice, g->st);
    if (e == hipSuccess) e = hipStreamSynchronize(g->st);      // the host reuses its E for the next block
    if (e != hipSuccess) return obc_fail(g, e);
    const dim3 grid((unsigned)((g->k - c1 + 255) / 256), (unsigned)((g->n + OBC_TI - 1) / OBC_TI));
    hipLaunchKernelGGL(k_obc_update, grid, dim3(256), 0, g->st, g->Wd, g->E, g->Hc, g->n, g->k, q * STB_BLOCK);
    e = hipGetLastError();
    return e == hipSuccess ? STB_OK : obc_fail(g, e);
}


}  // namespace

extern "C" int64_t stb_pack_obc_gpu_workspace(const stb_cfg_t* cfg) {
    const int64_t n = cfg->n_out, k = cfg->k_in;
    return up256(n * k * 8) + up256(k * k * 8) + up256(n * STB_BLOCK * 8);
}

// W, Hc (not NULL), xnorm, sal_bitmap, out: host, as stb_pack_obc takes them; workspace: device.
extern "C" int stb_pack_obc_gpu(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                                stb_layout_t* out, int32_t n_threads, void* workspace, void* stream, int* hip_err) {
    const int64_t n = out->cfg.n_out, k = out->cfg.k_in;
    if ((n + OBC_TI - 1) / OBC_TI > 65535) return STB_EUNSUPPORTED;          // rows of the update grid
    ObcGpu g;
    g.n = (int)n; g.k = (int)k; g.st = (hipStream_t)stream; g.hip_err = 0;
    g.Wd = (double*)workspace;
    g.Hc = (double*)((char*)workspace + up256(n * k * 8));
    g.E = (double*)((char*)workspace + up256(n * k * 8) + up256(k * k * 8));
    hipError_t e = hipMemcpyAsync(g.Hc, Hc, (size_t)k * k * 8, hipMemcpyHostToDevice, g.st);
    if (e == hipSuccess) e = hipStreamSynchronize(g.st);
    if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
    stb_obc_accel_t accel;
    accel.ctx = &g; accel.start = obc_start; accel.fetch = obc_fetch; accel.update = obc_update;
    const int rc = stb_pack_obc_with(W, Hc, xnorm, sal_bitmap, out, n_threads, &accel);
    e = hipStreamSynchronize(g.st);                    // nothing of this call is still running when it returns
    if (rc == STB_EHIP) *hip_err = g.hip_err;
    else if (rc == STB_OK && e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
    return rc;
}

// out: row-major layout bound to device memory (checked by the caller).  Runs on `stream` and waits for it: the status
// word comes back before the call returns.
extern "C" int stb_pack_gpu(const float* W, const float* xnorm, const uint32_t* sal_bitmap, const stb_layout_t* out,
                            int per_block, void* workspace, void* stream, int* hip_err) {
    const stb_cfg_t& c = out->cfg;
    const WsPlan wp = plan_workspace(c, per_block);
    char* ws = (char*)workspace;
    const hipStream_t st = (hipStream_t)stream;
    PK a;
    a.W = W; a.xnorm = xnorm; a.sal = sal_bitmap;
    a.n = c.n_out; a.k = c.k_in; a.N = c.N; a.M = c.M; a.nb = c.k_in / STB_BLOCK; a.per_block = per_block ? 1 : 0;
    a.nbS = a.per_block ? a.nb : 1; a.region_mode = c.region_mode; a.n_salient = c.n_salient;
    a.mask = (uint8_t*)out->mask; a.sign = (uint8_t*)out->sign; a.region = (uint8_t*)out->region;
    a.res_sign = (uint32_t*)out->res_sign; a.scales = out->scales; a.res_scale = out->res_scale;
    a.sal_out = out->sal_bitmap; a.prefix = out->sal_block_prefix;
    a.mask_stride = out->mask_stride; a.sign_stride = out->sign_stride; a.region_stride = out->region_stride;
    a.res_stride = out->res_stride;
    a.status = (uint32_t*)(ws + wp.status); a.rs = (double*)(ws + wp.rs); a.cs = (double*)(ws + wp.cs);
    a.rowacc = (double*)(ws + wp.rowacc); a.stats = (double*)(ws + wp.stats); a.mxbits = (uint32_t*)(ws + wp.mxbits);
    a.cnt = (uint32_t*)(ws + wp.cnt); a.p12 = (double*)(ws + wp.p12); a.hist = (uint32_t*)(ws + wp.hist);
    a.sel = (uint32_t*)(ws + wp.sel); a.err = (double*)(ws + wp.err);

    hipError_t e = hipSuccess;
    auto ok = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; return e == hipSuccess; };
    // everything that is accumulated into, and every padding byte of the planes, starts at zero
    ok(hipMemsetAsync(ws, 0, (size_t)wp.err, st));
    ok(hipMemsetAsync(out->mask, 0, (size_t)out->mask_bytes, st));
    ok(hipMemsetAsync(out->sign, 0, (size_t)out->sign_bytes, st));
    ok(hipMemsetAsync(out->region, 0, (size_t)out->region_bytes, st));
    if (out->res_bytes) ok(hipMemsetAsync(out->res_sign, 0, (size_t)out->res_bytes, st));
    if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }

    const int T = 256;
    const auto blocks = [&](int64_t items) { return dim3((unsigned)((items + T - 1) / T)); };
    const int64_t rb = (int64_t)a.n * a.nb;
    // the salient bitmap must hold exactly cfg.n_salient columns before anything indexes the res_sign rows by it
    hipLaunchKernelGGL(k_salient_tables, dim3(1), dim3(64), 0, st, a);
    uint32_t status = 0;
    ok(hipGetLastError());
    ok(hipMemcpyAsync(&status, a.status, 4, hipMemcpyDeviceToHost, st));
    ok(hipStreamSynchronize(st));
    if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
    if (status & ST_SALIENT) return STB_EINVAL;
    hipLaunchKernelGGL(k_row_pass<0>, dim3((a.n + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_col_sums, dim3((a.k + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_row_pass<1>, dim3((a.n + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_total<0>, dim3((a.nbS + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_row_pass<2>, dim3((a.n + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_total<1>, dim3((a.nbS + 63) / 64), dim3(64), 0, st, a);
    hipLaunchKernelGGL(k_mask, blocks((int64_t)a.n * (a.k / 8)), dim3(T), 0, st, a);
    hipLaunchKernelGGL(k_block_salient, blocks(rb), dim3(T), 0, st, a);
    if (a.region_mode == 0) {
        for (int q0 = 0; q0 < a.nb; q0 += wp.batch) {
            const int nq = a.nb - q0 < wp.batch ? a.nb - q0 : wp.batch;
            hipLaunchKernelGGL(k_candidate_errors, dim3((a.n + 3) / 4, 3, nq), dim3(64, 4), 0, st, a, q0);
            hipLaunchKernelGGL(k_pick_breakpoints, dim3(nq), dim3(192), 0, st, a, q0);
        }
    } else {
        hipLaunchKernelGGL(k_select_init, dim3((a.nb + 63) / 64), dim3(64), 0, st, a);
        for (int pass = 0; pass < 4; pass++) {
            hipLaunchKernelGGL(k_select_hist, blocks(rb), dim3(T), 0, st, a, pass);
            hipLaunchKernelGGL(k_select_step, dim3((2 * a.nb + 63) / 64), dim3(64), 0, st, a, pass);
        }
    }
    hipLaunchKernelGGL(k_assign, blocks(rb), dim3(T), 0, st, a);
    ok(hipGetLastError());
    ok(hipMemcpyAsync(&status, a.status, 4, hipMemcpyDeviceToHost, st));
    ok(hipStreamSynchronize(st));
    *hip_err = (int)e;
    if (e != hipSuccess) return STB_EHIP;
    if (status & ST_NONFINITE) return STB_ENONFINITE;
    if (status & ~ST_NONFINITE) return STB_EINVAL;
    return STB_OK;
}

// ------------------------------------------------------------------------------------------------
// stb_tile in device memory: the record permutation of the host routine, one thread per (row, block)
// ------------------------------------------------------------------------------------------------
namespace {

static __device__ uint32_t tile_status;

struct TK {
    const uint8_t* rmask; const uint8_t* rsign; const uint8_t* rreg; const uint16_t* rscales; const uint16_t* rres_scale;
    const uint32_t* rres_sign;
    uint8_t* tmask; uint8_t* tsign; uint8_t* treg; uint16_t* tscales; uint16_t* tres_scale; uint32_t* tres_sign;
    int64_t rmask_stride, rsign_stride, rreg_stride, rres_stride;
    int n, nb, nsb, SB, RB, RSB, RRB, padded, t8, n8, res_words;
    uint32_t* status;
};

// bytes [0, bytes) of a record: whole, or cut in two halves stored [tile][half][lane] when it is a multiple of 8 bytes
__device__ inline void put_record(uint8_t* plane, int64_t tile, int lane, const uint8_t* src, int bytes) {
    if (bytes % 8 == 0) {
        const int hb = bytes / 2;
        for (int h = 0; h < 2; h++) {
            uint8_t* dst = plane + tile * 64 * bytes + (int64_t)h * 32 * bytes + (int64_t)lane * hb;
            for (int b = 0; b < hb; b++) dst[b] = src[h * hb + b];
        }
    } else {
        uint8_t* dst = plane + (tile * 64 + lane) * bytes;
        for (int b = 0; b < bytes; b++) dst[b] = src[b];
    }
}

__global__ void k_tile_records(TK a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.nb) return;
    const int r = (int)(idx / a.nb), q = (int)(idx % a.nb);
    const int64_t tile = (int64_t)(r / 16) * a.nsb + q / 4;
    const int lane = 16 * (q % 4) + (r % 16);
    const uint8_t* mrow = a.rmask + (int64_t)r * a.rmask_stride + 16 * q;
    put_record(a.tmask, tile, lane, mrow, 16);
    if (!a.padded) {
        put_record(a.tsign, tile, lane, a.rsign + (int64_t)r * a.rsign_stride + (int64_t)a.SB * q, a.SB);
        put_record(a.treg, tile, lane, a.rreg + (int64_t)r * a.rreg_stride + (int64_t)a.RB * q, a.RB);
    } else {
        // 3 or 5 kept of 8: slot s of the block -> slot t8 * group + rank of its column among the group's kept columns
        // and the lowest pruned one
        const uint8_t* srow = a.rsign + (int64_t)r * a.rsign_stride + (int64_t)a.RSB * q;
        const uint8_t* grow = a.rreg + (int64_t)r * a.rreg_stride + (int64_t)a.RRB * q;
        uint8_t ps[12], pr[24];
        for (int b = 0; b < 12; b++) ps[b] = 0;
        for (int b = 0; b < 24; b++) pr[b] = 0;
        int slot = 0;
        bool bad = false;
        for (int g = 0; g < 16; g++) {
            const unsigned mb = mrow[g];
            if (__popc(mb) != a.n8) { bad = true; break; }
            const unsigned aug = mb | (~mb & (mb + 1u));
            for (int c = 0; c < 8; c++) {
                if (!((mb >> c) & 1u)) continue;
                const int t = a.t8 * g + __popc(aug & ((1u << c) - 1u));
                ps[t >> 3] |= (uint8_t)(((srow[slot >> 3] >> (slot & 7)) & 1u) << (t & 7));
                pr[t >> 2] |= (uint8_t)(((grow[slot >> 2] >> ((slot & 3) * 2)) & 3u) << ((t & 3) * 2));
                slot++;
            }
        }
        if (bad) { atomicOr(a.status, 4u); return; }
        put_record(a.tsign, tile, lane, ps, a.SB);
        put_record(a.treg, tile, lane, pr, a.RB);
    }
    const int64_t rec = tile * 64 + lane;
    for (int u = 0; u < 4; u++) a.tscales[rec * 4 + u] = a.rscales[((int64_t)r * a.nb + q) * 4 + u];
    a.tres_scale[rec] = a.rres_scale[(int64_t)r * a.nb + q];
}

// res_sign: the row strings cut into 32-bit words and transposed inside each 16-row tile; one thread per (row, word)
__global__ void k_tile_res(TK a) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.res_words) return;
    const int r = (int)(idx / a.res_words), w = (int)(idx % a.res_words);
    a.tres_sign[((int64_t)(r / 16) * a.res_words + w) * 16 + r % 16] = a.rres_sign[(int64_t)r * (a.rres_stride / 4) + w];
}

// res_t: per (row, block) the res_sign bits of the first 16 salient columns of each half block; one thread per record
__global__ void k_tile_res_t(TK a, const uint32_t* __restrict__ bitmap, const uint32_t* __restrict__ prefix,
                             uint32_t* __restrict__ res_t) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.nb) return;
    const int r = (int)(idx / a.nb), q = (int)(idx % a.nb);
    const uint32_t* row = a.rres_sign + (int64_t)r * (a.rres_stride / 4);
    uint32_t ord = prefix[q], word = 0;
    for (int h = 0; h < 2; h++) {
        int e = 0;
        for (int u = 0; u < 2; u++) {
            uint32_t bits = bitmap[4 * q + 2 * h + u];
            while (bits) {
                bits &= bits - 1;
                if (e < 16 && ((row[ord >> 5] >> (ord & 31)) & 1u)) word |= 1u << (16 * h + e);
                e++;
                ord++;
            }
        }
    }
    const int64_t tile = (int64_t)(r / 16) * a.nsb + q / 4;
    res_t[tile * 64 + 16 * (q % 4) + (r % 16)] = word;
}

}  // namespace

// src: checked row-major layout, dst: checked tiled layout of the same cfg, both bound to device memory.
extern "C" int stb_tile_gpu(const stb_layout_t* src, stb_layout_t* dst, void* stream, int* hip_err) {
    const hipStream_t st = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    auto ok = [&](hipError_t r) { if (e == hipSuccess && r != hipSuccess) e = r; return e == hipSuccess; };
    const int k = src->cfg.k_in, nb = src->n_blocks;
    // the derived tables depend on the salient bitmap only: they are made on the host and copied
    std::vector<uint32_t> bitmap((size_t)k / 32), prefix((size_t)nb + 1);
    ok(hipMemcpyAsync(bitmap.data(), src->sal_bitmap, (size_t)k / 8, hipMemcpyDeviceToHost, st));
    ok(hipMemcpyAsync(prefix.data(), src->sal_block_prefix, 4 * ((size_t)nb + 1), hipMemcpyDeviceToHost, st));
    ok(hipStreamSynchronize(st));
    if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
    {   // the kernels index the res_sign rows through these tables: they must describe cfg.n_salient columns
        uint32_t run = 0;
        for (int q = 0; q < nb; q++) {
            if (prefix[q] != run) return STB_EINVAL;
            for (int u = 0; u < 4; u++) run += (uint32_t)__builtin_popcount(bitmap[4 * q + u]);
        }
        if (prefix[nb] != run || run != (uint32_t)src->cfg.n_salient) return STB_EINVAL;
    }
    std::vector<uint32_t> bm_out((size_t)dst->salmap_bytes / 4), pf_out((size_t)dst->salprefix_bytes / 4),
        tab((size_t)dst->saltab_bytes / 4 + 1, 0u);
    int mx = 0, mh = 0;
    stb_host_tiled_tables(dst, bitmap.data(), prefix.data(), bm_out.data(), pf_out.data(), tab.data(), &mx, &mh);
    ok(hipMemcpyAsync(dst->sal_bitmap, bm_out.data(), (size_t)dst->salmap_bytes, hipMemcpyHostToDevice, st));
    ok(hipMemcpyAsync(dst->sal_block_prefix, pf_out.data(), (size_t)dst->salprefix_bytes, hipMemcpyHostToDevice, st));
    if (dst->saltab_bytes) ok(hipMemcpyAsync(dst->sal_tab, tab.data(), (size_t)dst->saltab_bytes, hipMemcpyHostToDevice, st));
    // padding rows and blocks of the planes are zero
    ok(hipMemsetAsync(dst->mask, 0, (size_t)dst->mask_bytes, st));
    ok(hipMemsetAsync(dst->sign, 0, (size_t)dst->sign_bytes, st));
    ok(hipMemsetAsync(dst->region, 0, (size_t)dst->region_bytes, st));
    ok(hipMemsetAsync(dst->scales, 0, (size_t)dst->scales_bytes, st));
    ok(hipMemsetAsync(dst->res_scale, 0, (size_t)dst->res_scale_bytes, st));
    if (dst->res_bytes) ok(hipMemsetAsync(dst->res_sign, 0, (size_t)dst->res_bytes, st));
    if (dst->res_t_bytes) ok(hipMemsetAsync(dst->res_t, 0, (size_t)dst->res_t_bytes, st));
    TK a;
    a.rmask = (const uint8_t*)src->mask; a.rsign = (const uint8_t*)src->sign; a.rreg = (const uint8_t*)src->region;
    a.rscales = src->scales; a.rres_scale = src->res_scale; a.rres_sign = (const uint32_t*)src->res_sign;
    a.tmask = (uint8_t*)dst->mask; a.tsign = (uint8_t*)dst->sign; a.treg = (uint8_t*)dst->region;
    a.tscales = dst->scales; a.tres_scale = dst->res_scale; a.tres_sign = (uint32_t*)dst->res_sign;
    a.rmask_stride = src->mask_stride; a.rsign_stride = src->sign_stride; a.rreg_stride = src->region_stride;
    a.rres_stride = src->res_stride;
    a.n = src->cfg.n_out; a.nb = nb; a.nsb = dst->n_super;
    a.SB = (int)dst->sign_stride; a.RB = (int)dst->region_stride;
    a.padded = stb_tiled_padded(&src->cfg); a.t8 = stb_tiled_slots(&src->cfg); a.n8 = 8 * src->cfg.N / src->cfg.M;
    a.RSB = 2 * a.n8; a.RRB = 4 * a.n8;
    a.res_words = (int)(src->res_stride / 4);
    // what the kernel finds (a mask byte with the wrong number of bits in a padded layout) comes back through a word
    // of the library's own device memory; calls that overlap on one GPU share it
    uint32_t* status_dev = nullptr;
    ok(hipGetSymbolAddress((void**)&status_dev, HIP_SYMBOL(tile_status)));
    if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
    ok(hipMemsetAsync(status_dev, 0, 4, st));
    a.status = status_dev;
    const int64_t recs = (int64_t)a.n * a.nb;
    hipLaunchKernelGGL(k_tile_records, dim3((unsigned)((recs + 255) / 256)), dim3(256), 0, st, a);
    if (a.res_words > 0) {
        const int64_t words = (int64_t)a.n * a.res_words;
        hipLaunchKernelGGL(k_tile_res, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, a);
        hipLaunchKernelGGL(k_tile_res_t, dim3((unsigned)((recs + 255) / 256)), dim3(256), 0, st, a, src->sal_bitmap,
                           src->sal_block_prefix, dst->res_t);
    }
    ok(hipGetLastError());
    uint32_t status = 0;
    ok(hipMemcpyAsync(&status, status_dev, 4, hipMemcpyDeviceToHost, st));
    ok(hipStreamSynchronize(st));          // also: the host arrays of the tables must outlive their copies
    *hip_err = (int)e;
    if (e != hipSuccess) return STB_EHIP;
    if (status) return STB_EINVAL;
    dst->max_sal_block = mx;
    dst->max_sal_half = mh;
    return STB_OK;
}
