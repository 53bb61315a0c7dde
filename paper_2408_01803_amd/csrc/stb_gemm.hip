// Prefill GEMM for the tiled device order (STB_KIND_TILED), gfx950 (App. C: the compute-bound regime).
//
//   Y[t][i] = sum_j X[t][j] * W_hat[i][j]
//
// A workgroup of four wavefronts owns 256 output rows x 128 tokens; wavefront w owns the four 16-row tiles
// 4w .. 4w+3 of the block.  The weights never pass through memory in dequantised form: every lane expands
// its (row, half block) bits straight into the A operand of v_mfma_f32_16x16x32_f16 (the code of
// stb_tiled.hpp, as in the decode kernel), so K slot g of an MFMA is 8 columns of block g of the superblock.
// The tokens are the B operand: a window of X (128 tokens x 4 blocks x 32 columns) is staged in LDS, double
// buffered, and every B operand read from it feeds four MFMAs (one per row tile).
// The residual term of the salient columns (Eq. 4) is a second, short contraction: its A operand comes from
// residual_chunk, its B operand from a compact copy of the salient columns of X that gemm_gather_kernel
// writes to the workspace beforehand.
#include "stb_tiled.hpp"

using namespace stbt;

namespace {

constexpr int GM_TOK = 128;           // tokens per workgroup
constexpr int GM_ROWT = 16;           // 16-row tiles per workgroup (four per wavefront)
constexpr int GM_XROW = 136;          // halves per token row of the LDS window: 4 x 32 columns + 8 of padding
constexpr int GM_XROW1 = 168;         // second buffer: + 4 x 8 gathered salient columns (residual contraction)

// Workspace: xsal[T][E] fp16, E = nsb * 2 * cfix * 32; entry ((sb*2 + half)*cfix + c)*32 + g*8 + e holds X at the
// e-th salient column of record c of (block 4*sb + g, half), 0 where the record has no such entry.
__global__ __launch_bounds__(256) void gemm_gather_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                           __half* __restrict__ xsal, int cfix) {
    const int per_tok = p.nsb * 2 * cfix * 4;                       // 16-byte pieces per token
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= (int64_t)T * per_tok) return;
    const int tok = (int)(id / per_tok), piece = (int)(id % per_tok);
    const int g = piece & 3, c = (piece >> 2) % cfix, sh = (piece >> 2) / cfix;
    const int q = 4 * (sh >> 1) + g, half = sh & 1;
    uint32_t out[4] = {0u, 0u, 0u, 0u};
    if (c < p.sal_chunks) {
        const uint32_t* rec = p.sal_tab + (((int64_t)q * 2 + half) * p.sal_chunks + c) * 12;
        const uint4 pv = *reinterpret_cast<const uint4*>(rec + 8);
        const uint32_t pw[4] = {pv.x, pv.y, pv.z, pv.w};
        const unsigned short* xrow = reinterpret_cast<const unsigned short*>(X) + (int64_t)tok * p.k + (int64_t)q * 128;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
            if (pos < 128u && q < p.nb) out[e >> 1] |= (uint32_t)xrow[pos] << (16 * (e & 1));
        }
    }
    *reinterpret_cast<uint4*>(xsal + ((int64_t)tok * per_tok + piece) * 8) = make_uint4(out[0], out[1], out[2], out[3]);
}

template <int N8, bool HAS_RES>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                          void* __restrict__ Y, int y_fp32,
                                                          const __half* __restrict__ xsal, int cfix) {
    __shared__ ScatterLds lut;
    __shared__ __attribute__((aligned(16))) _Float16 xs0[GM_TOK * GM_XROW];
    __shared__ __attribute__((aligned(16))) _Float16 xs1[GM_TOK * GM_XROW1];
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * GM_TOK;
    const int rtw = blockIdx.y * GM_ROWT + wave * 4;                // first row tile of this wavefront
    build_luts<N8>(&lut);

    float4_t acc[4][8];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
        for (int tt = 0; tt < 8; tt++) acc[r][tt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    // ---- staging of the X window: 2048 pieces of 16 bytes, 8 per thread ----
    // piece c: token c / 16, block (c / 4) % 4, 8 columns (c % 4) of the window
    auto x_gload = [&](int sb, int half, int win, uint4 (&st)[8]) {
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const int c = tid + 256 * u;
            const int tok = t0 + (c >> 4), gb = (c >> 2) & 3, cc = c & 3;
            const int q = 4 * sb + gb;
            st[u] = make_uint4(0u, 0u, 0u, 0u);
            if (tok < T && q < p.nb)
                st[u] = *reinterpret_cast<const uint4*>(X + (int64_t)tok * p.k + (int64_t)q * 128 + 64 * half + 32 * win + 8 * cc);
        }
    };
    auto x_lstore = [&](int buf, const uint4 (&st)[8]) {
        _Float16* dst = buf ? xs1 : xs0;
        const int stride = buf ? GM_XROW1 : GM_XROW;
#pragma unroll
        for (int u = 0; u < 8; u++) {
            const int c = tid + 256 * u;
            *reinterpret_cast<uint4*>(&dst[(c >> 4) * stride + ((c >> 2) & 3) * 32 + (c & 3) * 8]) = st[u];
        }
    };
    // the gathered salient columns of this (superblock, half), record c: 128 tokens x 4 pieces of 16 bytes
    const int64_t E = (int64_t)p.nsb * 2 * cfix * 32;               // halves per token in xsal
    auto r_gload = [&](int sh, int c, uint4 (&sr)[2]) {
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int pc = tid + 256 * u;
            const int tok = t0 + (pc >> 2), gb = pc & 3;
            sr[u] = make_uint4(0u, 0u, 0u, 0u);
            if (HAS_RES && tok < T) sr[u] = *reinterpret_cast<const uint4*>(xsal + (int64_t)tok * E + ((int64_t)sh * cfix + c) * 32 + gb * 8);
        }
    };
    auto r_lstore = [&](const uint4 (&sr)[2]) {
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int pc = tid + 256 * u;
            *reinterpret_cast<uint4*>(&xs1[(pc >> 2) * GM_XROW1 + 128 + (pc & 3) * 8]) = sr[u];
        }
    };
    // four K steps on one window: groups 4*win .. 4*win + 3 of every lane's half block.  The B operands and the
    // expanded A operands of step s + 1 are produced while the 32 MFMAs of step s run.
    auto bload = [&](int buf, int tq, uint4 (&b)[8]) {
        const _Float16* src = buf ? xs1 : xs0;
        const int stride = buf ? GM_XROW1 : GM_XROW;
#pragma unroll
        for (int tt = 0; tt < 8; tt++)
            b[tt] = *reinterpret_cast<const uint4*>(&src[(16 * tt + i) * stride + g * 32 + tq * 8]);
    };
    auto bload_res = [&](uint4 (&b)[8]) {
#pragma unroll
        for (int tt = 0; tt < 8; tt++)
            b[tt] = *reinterpret_cast<const uint4*>(&xs1[(16 * tt + i) * GM_XROW1 + 128 + g * 8]);
    };
    auto expand4 = [&](const HalfData<N8> (&hd)[4], const uint32_t (&TL)[4], const uint32_t (&TH)[4], int t, uint32_t (&a)[4][4]) {
#pragma unroll
        for (int r = 0; r < 4; r++) expand_group<N8>(hd[r], TL[r], TH[r], t, lut_fetch<N8>(hd[r], t, &lut, lane & 7), a[r]);
    };
    auto mfma32 = [&](const uint32_t (&a)[4][4], const uint4 (&b)[8]) {
#pragma unroll
        for (int tt = 0; tt < 8; tt++) {
            const half8_t bv = __builtin_bit_cast(half8_t, b[tt]);
#pragma unroll
            for (int r = 0; r < 4; r++)
                acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(a[r]), bv, acc[r][tt], 0, 0, 0);
        }
    };
    auto window = [&](const HalfData<N8> (&hd)[4], const uint32_t (&TL)[4], const uint32_t (&TH)[4], int win, int buf) {
        uint4 b0[8], b1[8];
        uint32_t a0[4][4], a1[4][4];
        bload(buf, 0, b0);
        expand4(hd, TL, TH, 4 * win, a0);
        bload(buf, 1, b1);
        expand4(hd, TL, TH, 4 * win + 1, a1);
        mfma32(a0, b0);
        bload(buf, 2, b0);
        expand4(hd, TL, TH, 4 * win + 2, a0);
        mfma32(a1, b1);
        bload(buf, 3, b1);
        expand4(hd, TL, TH, 4 * win + 3, a1);
        mfma32(a0, b0);
        mfma32(a1, b1);
    };
    auto load_hd = [&](int sb, int half, HalfData<N8> (&hd)[4]) {
        const LaneOffsets lo = lane_offsets<N8>(lane, half);
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int rt = rtw + r < p.nrt ? rtw + r : p.nrt - 1;
            load_half<N8>(p, (int64_t)rt * p.nsb + sb, lo, half, hd[r]);
        }
    };

    uint4 st[8];
    x_gload(0, 0, 0, st);
    x_lstore(0, st);
    __syncthreads();

    const int nsh = p.nsb * 2;                                      // (superblock, half) pairs
    auto load_res_words = [&](uint32_t ord, uint32_t (&rlo)[4], uint32_t (&rhi)[4]) {
        const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
        const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            const int rt = rtw + r < p.nrt ? rtw + r : p.nrt - 1;
            rlo[r] = p.res_sign[((int64_t)rt * p.res_words + wa) * 16 + i];
            rhi[r] = p.res_sign[((int64_t)rt * p.res_words + wb) * 16 + i];
        }
    };
    // residual contraction of one record: A from the mask / res_sign bits, B = the gathered columns in xs1
    auto residual = [&](const HalfData<N8> (&hd)[4], const uint4& ra, uint32_t ord, const uint32_t (&rlo)[4],
                        const uint32_t (&rhi)[4]) {
        ResSel sel;
        sel.sel0 = ra.x; sel.sel1 = ra.y; sel.bit0 = ra.z; sel.bit1 = ra.w;
        uint4 b[8];
        bload_res(b);
        uint32_t a[4][4];
#pragma unroll
        for (int r = 0; r < 4; r++)
            residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], ord & 31u), hd[r].ar | (hd[r].ar << 16), sel, a[r]);
        mfma32(a, b);
    };

    for (int sh = 0; sh < nsh; sh++) {
        const int sb = sh >> 1, half = sh & 1;
        const bool more = sh + 1 < nsh;
        HalfData<N8> hd[4];
        load_hd(sb, half, hd);
        // the table record of this (superblock, half) and, through it, the residual sign words of the rows
        uint4 ra = make_uint4(0u, 0u, 0u, 0u);
        uint2 rb = make_uint2(0u, 0u);
        const uint32_t* rec0 = nullptr;
        if (HAS_RES) {
            rec0 = p.sal_tab + (((int64_t)(4 * sb + g) * 2 + half) * p.sal_chunks) * 12;
            ra = *reinterpret_cast<const uint4*>(rec0);
            rb = *reinterpret_cast<const uint2*>(rec0 + 4);
        }
        uint32_t TL[4], TH[4];
#pragma unroll
        for (int r = 0; r < 4; r++) {
            TL[r] = perm(hd[r].sc.y, hd[r].sc.x, 0x06040200u);
            TH[r] = perm(hd[r].sc.y, hd[r].sc.x, 0x07050301u);
        }
        // window 0 is in xs0; fetch window 1 and the gathered salient columns while it is used
        uint4 sr[2];
        x_gload(sb, half, 1, st);
        r_gload(sh, 0, sr);
        window(hd, TL, TH, 0, 0);
        x_lstore(1, st);
        if (HAS_RES) r_lstore(sr);
        uint32_t rlo[4] = {0u, 0u, 0u, 0u}, rhi[4] = {0u, 0u, 0u, 0u};
        int nch = 0;
        if (HAS_RES) {
            nch = __builtin_amdgcn_readfirstlane((int)rb.y);
            if (nch > 0) load_res_words(rb.x, rlo, rhi);
        }
        __syncthreads();
        if (more) x_gload((sh + 1) >> 1, (sh + 1) & 1, 0, st);
        window(hd, TL, TH, 1, 1);
        if (HAS_RES && nch > 0) {
            residual(hd, ra, rb.x, rlo, rhi);
            for (int c = 1; c < nch; c++) {              // half blocks with more than 8 salient columns (rare)
                __syncthreads();                         // every wavefront is done with the gathered columns
                r_gload(sh, c, sr);
                r_lstore(sr);
                const uint32_t* rec = rec0 + c * 12;
                const uint4 rc = *reinterpret_cast<const uint4*>(rec);
                const uint32_t ord = rec[4];
                load_res_words(ord, rlo, rhi);
                __syncthreads();
                residual(hd, rc, ord, rlo, rhi);
            }
        }
        if (more) x_lstore(0, st);
        __syncthreads();
    }

    // ---- epilogue: D[row][token] of an MFMA: lane l holds token l % 16, rows 4*(l / 16) + v ----
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int row = (rtw + r) * 16 + 4 * g;
        if (rtw + r >= p.nrt) continue;
#pragma unroll
        for (int tt = 0; tt < 8; tt++) {
            const int tok = t0 + 16 * tt + i;
            if (tok >= T) continue;
#pragma unroll
            for (int v = 0; v < 4; v++) {
                if (row + v >= p.n) continue;
                const float val = -acc[r][tt][v];
                if (y_fp32) reinterpret_cast<float*>(Y)[(int64_t)tok * p.n + row + v] = val;
                else reinterpret_cast<__half*>(Y)[(int64_t)tok * p.n + row + v] = __float2half(val);
            }
        }
    }
}

}  // namespace

static int64_t round_up256(int64_t v) { return (v + 255) / 256 * 256; }
static int cfix_of(const stb_layout_t* L) { return (L->max_sal_half + 7) / 8; }

extern "C" int64_t stb_tiled_gemm_workspace(const stb_layout_t* L, int T) {
    return round_up256((int64_t)T * L->n_super * 2 * cfix_of(L) * 32 * 2);
}

extern "C" int stb_tiled_gemm(const stb_layout_t* L, const void* X, int T, void* Y, int y_fp32, void* workspace,
                              int64_t workspace_bytes, void* stream, int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    const TiledPlanes p = make_tiled(L);
    const int cfix = cfix_of(L);
    const bool res = p.res_words > 0 && cfix > 0;
    const hipStream_t st = (hipStream_t)stream;
    if (res) {
        if (!workspace) return STB_ENULL;
        if (workspace_bytes < stb_tiled_gemm_workspace(L, T)) return STB_EINVAL;
        if ((uintptr_t)workspace % 256) return STB_EALIGN;
        const int64_t pieces = (int64_t)T * p.nsb * 2 * cfix * 4;
        hipLaunchKernelGGL(gemm_gather_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, p,
                           (const __half*)X, T, (__half*)workspace, cfix);
    }
    const dim3 grid((T + GM_TOK - 1) / GM_TOK, (p.nrt + GM_ROWT - 1) / GM_ROWT);
    const int n8 = 8 * L->cfg.N / L->cfg.M;
    const __half* xh = (const __half*)X;
    const __half* xs = (const __half*)workspace;
    if (n8 == 4) {
        if (res) hipLaunchKernelGGL((gemm_tiled_kernel<4, true>), grid, dim3(256), 0, st, p, xh, T, Y, y_fp32, xs, cfix);
        else hipLaunchKernelGGL((gemm_tiled_kernel<4, false>), grid, dim3(256), 0, st, p, xh, T, Y, y_fp32, xs, cfix);
    } else {
        if (res) hipLaunchKernelGGL((gemm_tiled_kernel<6, true>), grid, dim3(256), 0, st, p, xh, T, Y, y_fp32, xs, cfix);
        else hipLaunchKernelGGL((gemm_tiled_kernel<6, false>), grid, dim3(256), 0, st, p, xh, T, Y, y_fp32, xs, cfix);
    }
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}
