// Prefill GEMM for the tiled device order (STB_KIND_TILED), gfx950 (App. C: the compute-bound regime).
//
//   Y[t][i] = sum_j X[t][j] * W_hat[i][j]
//
// A workgroup of four wavefronts (one per SIMD) owns 256 output rows x 128 tokens; wavefront w owns the four
// 16-row tiles 4w .. 4w+3 of the block and their 128 accumulator registers.  The weights never pass through
// memory in dequantised form: every lane expands its (row, half block) bits straight into the A operand of the
// matrix instruction (the code of stb_tiled.hpp, as in the decode kernel), so K slot g of an instruction is 8 (dense)
// or 16 (sparse) columns of block g of the superblock.  The tokens are the B operand: windows of X (128 tokens x 4
// blocks x 32 columns) go from global memory straight to LDS, two per half block, and every B operand read from
// them feeds four matrix instructions (one per row tile).
// The main loop is a software pipeline of K steps: a step issues its 32 matrix instructions and, between them,
// builds the A operands and reloads the B operands of the next step; the global loads of later steps are spread
// over the steps as asm statements with hand-written waits.
//   gemm_tiled_kernel  4:8 and 6:8 layers (and 2:4 on request): v_mfma_f32_16x16x32_f16 on the expanded operand
//   gemm24_kernel      2:4 layers: v_smfmac_f32_16x16x64_f16 on the kept weights and an index word
// The residual term of the salient columns (Eq. 4) is a second, short contraction: its A operand comes from
// residual_chunk, its B operand from a compact copy of the salient columns of X that gemm_gather_kernel
// writes to the workspace beforehand.
#include <atomic>

#include "stb_tiled.hpp"

using namespace stbt;

namespace {

// Tokens per workgroup: 16 * TT, TT token tiles per wavefront (a multiple of 4).

constexpr int GM_ROWT = 16;           // 16-row tiles per workgroup (four per wavefront)
// LDS of the main kernel (dynamic, carved by hand so that the positions are fixed):
//   (sizes for 128 tokens; they grow with the tile)
//   [0, 64 KB)    two X windows: 128 token rows x 256 bytes (4 blocks x 32 columns); the 16-byte piece p of row r
//                 sits at position p ^ (r % 16), so the 16 lanes that read one piece of 16 consecutive rows (a B
//                 operand) hit 16 different positions and a wavefront's global->LDS load fills 4 whole rows
//   [64, 80 KB)   gathered salient columns, by parity of the pass: 128 rows x 64 bytes, piece g of row r at
//                 position g ^ ((r / 4) % 4)
//   [80, 112 KB)  the scatter table
template <int TT>
struct GmLds {
    static constexpr int TOK = 16 * TT;
    static constexpr int XW = 0, XWSZ = TOK * 256, XG = 2 * XWSZ, XGSZ = TOK * 64, LUT = XG + 2 * XGSZ;
    static constexpr int TOTAL = LUT + 32768;      // with the scatter table (dense kernel)
    static constexpr int TOTAL24 = LUT;            // without (sparse kernel)
};
constexpr int GM_TT = 8, GM_TT24 = 8;       // (12 in the dense kernel was measured: 15 - 30 % slower, fewer and fatter workgroups)
constexpr int GM_SMALL_TT = 4, GM_SMALL_TOK = 16 * GM_SMALL_TT;     // launches of up to 64 tokens

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

template <int V> struct IntC { static constexpr int value = V; };

// Writes a wavefront's 64 rows x 128 tokens: D[row][token] of an MFMA, lane l holds token l % 16, rows 4*(l / 16) + v.
// (The caller has passed a barrier after the last use of LDS.)
template <int TT>
__device__ inline void store_tile(const float4_t (&acc)[4][TT], char* lds, const TiledPlanes& p, void* __restrict__ Y, int y_fp32,
                                  int T, int t0, int rtw, int wave, int lane) {
    const int i = lane & 15, g = lane >> 4;
    // fp16 output whose rows of Y can be written in 16-byte pieces: the wavefront transposes its 64 rows x 128 tokens
    // through LDS (its own region; token rows of 144 bytes), so that a store instruction writes whole 128-byte runs
    // of Y (8 tokens x the wavefront's 64 rows) instead of 32-byte pieces.
    const bool wide = !y_fp32 && (p.n & 7) == 0 && ((uintptr_t)Y & 15) == 0 && (rtw + 4) * 16 <= p.n;     // uniform per wavefront
    if (wide) {
        char* const ep = lds + wave * (16 * TT * 144);
#pragma unroll
        for (int r = 0; r < 4; r++)
#pragma unroll
            for (int tt = 0; tt < TT; tt++) {
                const __half2 lo = __floats2half2_rn(-acc[r][tt][0], -acc[r][tt][1]);
                const __half2 hi = __floats2half2_rn(-acc[r][tt][2], -acc[r][tt][3]);
                uint2 v;
                v.x = __builtin_bit_cast(uint32_t, lo);
                v.y = __builtin_bit_cast(uint32_t, hi);
                *reinterpret_cast<uint2*>(ep + (16 * tt + i) * 144 + (16 * r + 4 * g) * 2) = v;
            }
        // (the wavefront reads back only what it wrote itself: LDS keeps a wavefront's accesses in order)
        __half* const Yh = reinterpret_cast<__half*>(Y);
#pragma unroll
        for (int it = 0; it < 2 * TT; it++) {
            const int tl = 8 * it + (lane >> 3), tok = t0 + tl;
            const uint4 v = *reinterpret_cast<const uint4*>(ep + tl * 144 + (lane & 7) * 16);
            if (tok < T) *reinterpret_cast<uint4*>(Yh + (int64_t)tok * p.n + rtw * 16 + (lane & 7) * 8) = v;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < 4; r++) {
        const int row = (rtw + r) * 16 + 4 * g;
        if (rtw + r >= p.nrt) continue;
#pragma unroll
        for (int tt = 0; tt < TT; tt++) {
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

// One wavefront-wide global -> LDS load of 16 bytes per lane: lane l's bytes land at LDS address m0 + 16 * l.
// No register is written: the data is in LDS once vmcnt has counted the load down.
__device__ inline void load_to_lds(uint32_t lds_addr, uint32_t voff, const void* base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}

// ------------------------------------------------------------------------------------------------
// What the two main kernels share: the per-lane constants and the loads of a pass.
// Every global load of a main loop is an asm statement, and every use sits behind a vmcnt wait written by hand
// (for loads into registers the wait names them, the rules of the fetch helpers in stb_tiled.hpp): the loads go
// out where they are written, K steps ahead of their use, and the compiler neither sinks them down to it nor
// waits for them on its own (a load the compiler knows of makes it wait for everything in flight).
// ------------------------------------------------------------------------------------------------
// WIDE (the kernel on the 32x32x16 instruction): lane 16 g + i is row 16 (g % 2) + i of a 32-row operand and K half
// g / 2, so its record r = 2 rs + bs (0..3) is (row tile 2 rs + g % 2 of the wavefront, block 2 (g / 2) + bs of the
// superblock) instead of (row tile r, block g): the same 256 records per wavefront and pass, dealt differently.
template <int N8, bool HAS_RES, int TT, bool WIDE = false>
struct GemmStage {
    typedef GmLds<TT> G;
    static constexpr int NGL = TT / 4;         // gathered-column loads per wavefront (16 token rows each)
    const TiledPlanes& p;
    const __half* Xt;                          // X at the workgroup's first token
    const __half* xsal_t;                      // gathered salient columns at the workgroup's first token
    const uint32_t* rsbase[4];                 // res_sign words of the wavefront's four row tiles (uniform)
    uint32_t lds0, tok_last, k2, xpc[4], grow[NGL];
    uint32_t dn[2], dres[2];                   // WIDE: from the uniform base of row-tile pair rs to the lane's own row tile, in tiles / res_sign bytes
    int cfix, rtw, wave, lane, i, g;

    __device__ GemmStage(const TiledPlanes& p_, const __half* X, const __half* xsal, int T, int cfix_, uint32_t lds0_, int t0,
                         int rtw_, int wave_, int lane_)
        : p(p_), lds0(lds0_), cfix(cfix_), rtw(rtw_), wave(wave_), lane(lane_), i(lane_ & 15), g(lane_ >> 4) {
        tok_last = (uint32_t)(T - 1 - t0);
        k2 = (uint32_t)p.k * 2u;
        Xt = X + (int64_t)t0 * p.k;
        // X window -> LDS: 4 TT wavefront loads of 4 token rows each, TT per wavefront.  Load u of wavefront w covers
        // rows 4 * (TT w + u) ..; lane l = row l / 16 of them, position l % 16, i.e. piece (l % 16) ^ (row % 16):
        // block piece / 4, 8 columns (piece % 4).  Tokens past T are clamped to the last token (their outputs are
        // never stored); a piece past column k is clamped to the row's last 16 bytes (it meets zero weights).
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const uint32_t pc = (uint32_t)i ^ (uint32_t)(4 * j + g);   // rows 4 * (TT w + u) + g: row % 16 = 4 * (u % 4) + g
            xpc[j] = (pc >> 2) * 256u + (pc & 3u) * 16u;
        }
        // gathered salient columns: TT wavefront loads of 16 token rows, NGL per wavefront; lane l = row l / 4 of
        // them, position l % 4 = piece (l % 4) ^ ((row / 4) % 4)
        const int64_t E = (int64_t)p.nsb * 2 * cfix * 32;           // halves per token in xsal
        xsal_t = xsal + (int64_t)t0 * E;
#pragma unroll
        for (int u = 0; u < NGL; u++) {
            const uint32_t row = (uint32_t)(16 * (NGL * wave + u) + (lane >> 2));
            grow[u] = (row < tok_last ? row : tok_last) * (uint32_t)E * 2u + (((uint32_t)lane & 3u) ^ (((uint32_t)lane >> 4) & 3u)) * 16u;
        }
#pragma unroll
        for (int rs = 0; rs < 2; rs++) {
            const int mine = rtw + 2 * rs + (g & 1) < p.nrt ? rtw + 2 * rs + (g & 1) : p.nrt - 1;
            dn[rs] = WIDE ? (uint32_t)((mine - row_tile(2 * rs)) * p.nsb) : 0u;
            dres[rs] = WIDE ? (uint32_t)((mine - row_tile(2 * rs)) * p.res_words) * 64u : 0u;
        }
#pragma unroll
        for (int r = 0; r < 4; r++) rsbase[r] = p.res_sign + (int64_t)base_tile(r) * p.res_words * 16;
    }
    __device__ int row_tile(int r) const { return rtw + r < p.nrt ? rtw + r : p.nrt - 1; }
    // record r of the lane: the uniform row tile its loads start from, its block, its offsets inside the planes
    __device__ int base_tile(int r) const { return WIDE ? row_tile(2 * (r >> 1)) : row_tile(r); }
    __device__ int block_of(int r) const { return WIDE ? 2 * (g >> 1) + (r & 1) : g; }
    __device__ LaneOffsets offsets(int sh, int r) const {
        LaneOffsets lo = lane_offsets<N8>(WIDE ? 16 * block_of(r) + i : lane, sh & 1);
        if (WIDE) {
            const uint32_t d = dn[r >> 1];
            lo.omask += d * (64u * 16u);
            lo.osign += d * (64u * 2u * N8);
            lo.oregion += d * (64u * 4u * N8);
            lo.o8 += d * (64u * 8u);
            lo.o2 += d * (64u * 2u);
        }
        return lo;
    }

    // load u (0 .. TT-1) of the wavefront's share of window `win` of (superblock, half) sh into window buffer `buf`
    __device__ void x_gload1(int sh, int win, int buf, int u) const {
        const uint32_t wcol = (uint32_t)((sh >> 1) * 1024 + (sh & 1) * 128 + win * 64);      // bytes inside a token row
        const uint32_t dst = lds0 + G::XW + buf * G::XWSZ + wave * (TT * 1024);
        const uint32_t c = xpc[u & 3] + wcol;
        const uint32_t row = (uint32_t)(4 * (TT * wave + u)) + (uint32_t)g;
        load_to_lds(dst + u * 1024, __umul24(row < tok_last ? row : tok_last, k2) + (c < k2 - 16u ? c : k2 - 16u), Xt);
    }
    __device__ void x_gload(int sh, int win, int buf) const {
#pragma unroll
        for (int u = 0; u < TT; u++) x_gload1(sh, win, buf, u);
    }
    // load u (0 .. NGL-1) of the gathered salient columns of (superblock, half) sh, record c, into buffer `par`
    __device__ void r_gload1(int sh, int c, int par, int u) const {
        if (HAS_RES) load_to_lds(lds0 + G::XG + par * G::XGSZ + (NGL * wave + u) * 1024, grow[u] + (uint32_t)(sh * cfix + c) * 64u, xsal_t);
    }
    __device__ void r_gload(int sh, int c, int par) const {
#pragma unroll
        for (int u = 0; u < NGL; u++) r_gload1(sh, c, par, u);
    }
    // plain loads (tail loop only)
    __device__ void load_hd(int sh, HalfData<N8> (&hd)[4]) const {
#pragma unroll
        for (int r = 0; r < 4; r++) load_half<N8>(p, (int64_t)base_tile(r) * p.nsb + (sh >> 1), offsets(sh, r), sh & 1, hd[r]);
    }
    __device__ void load_res_words(uint32_t ord, uint32_t (&rlo)[4], uint32_t (&rhi)[4]) const {
        const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
        const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
#pragma unroll
        for (int r = 0; r < 4; r++) {
            rlo[r] = rsbase[r][wa * 16 + i];
            rhi[r] = rsbase[r][wb * 16 + i];
        }
    }
    // (WIDE: the words of record r alone, at the lane's own row tile)
    __device__ void load_res_words1(uint32_t ord, uint32_t (&rlo)[4], uint32_t (&rhi)[4], int r) const {
        const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
        const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
        const char* base = reinterpret_cast<const char*>(rsbase[r]) + dres[r >> 1];
        rlo[r] = *reinterpret_cast<const uint32_t*>(base + (wa * 16 + i) * 4);
        rhi[r] = *reinterpret_cast<const uint32_t*>(base + (wb * 16 + i) * 4);
    }
    // asm loads: the table record of (superblock, half) sh (2 loads), the half records of row tile r (5 loads), the
    // res_sign words of row tile r (2 loads)
    __device__ void fetch_rec(int sh, uint4_t& ra, uint2_t& rb, int r = 0) const {
        if (HAS_RES) {
            const uint32_t off = (uint32_t)(((4 * (sh >> 1) + block_of(r)) * 2 + (sh & 1)) * p.sal_chunks) * 48u;
            asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(ra) : "v"(off), "s"(p.sal_tab));
            asm volatile("global_load_dwordx2 %0, %1, %2 offset:16" : "=v"(rb) : "v"(off), "s"(p.sal_tab));
        }
    }
    __device__ void fetch_hd1(int sh, TileRegs<N8> (&tn)[4], int r) const {
        const LaneOffsets lo = offsets(sh, r);
        fetch_main<N8>(tn[r], p, (int64_t)__builtin_amdgcn_readfirstlane(base_tile(r) * p.nsb + (sh >> 1)), lo);
    }
    __device__ void fetch_res_words1(uint32_t ord, uint32_t (&rlo)[4], uint32_t (&rhi)[4], int r) const {
        const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
        const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
        const uint32_t oa = (uint32_t)(wa * 16 + i) * 4u + dres[r >> 1], ob = (uint32_t)(wb * 16 + i) * 4u + dres[r >> 1];
        asm volatile("global_load_dword %0, %1, %2" : "=v"(rlo[r]) : "v"(oa), "s"(rsbase[r]));
        asm volatile("global_load_dword %0, %1, %2" : "=v"(rhi[r]) : "v"(ob), "s"(rsbase[r]));
    }
    __device__ void fetch_res_words(uint32_t ord, uint32_t (&rlo)[4], uint32_t (&rhi)[4]) const {
#pragma unroll
        for (int r = 0; r < 4; r++) fetch_res_words1(ord, rlo, rhi, r);
    }
    __device__ static void scale_tables(const HalfData<N8> (&hd)[4], uint32_t (&TL)[4], uint32_t (&TH)[4]) {
#pragma unroll
        for (int r = 0; r < 4; r++) {
            TL[r] = perm(hd[r].sc.y, hd[r].sc.x, 0x06040200u);
            TH[r] = perm(hd[r].sc.y, hd[r].sc.x, 0x07050301u);
        }
    }
    // the first pass's half records and table record (asm loads here too), waited for on the spot
    __device__ void first_records(int shb, HalfData<N8> (&hd)[4], uint4& ra, uint2& rb, uint4* ra_odd = nullptr, uint2* rb_odd = nullptr) const {
        TileRegs<N8> t0r[4];
        uint4_t ra0 = {0u, 0u, 0u, 0u}, ra1 = {0u, 0u, 0u, 0u};
        uint2_t rb0 = {0u, 0u}, rb1 = {0u, 0u};
#pragma unroll
        for (int r = 0; r < 4; r++) fetch_hd1(shb, t0r, r);
        fetch_rec(shb, ra0, rb0);
        if (WIDE) fetch_rec(shb, ra1, rb1, 1);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(ra0), "+v"(rb0), "+v"(ra1), "+v"(rb1) : : "memory");
        if (WIDE) {
            *ra_odd = make_uint4(ra1.x, ra1.y, ra1.z, ra1.w);
            *rb_odd = make_uint2(rb1.x, rb1.y);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) {
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t0r[r].m), "+v"(t0r[r].s), "+v"(t0r[r].r), "+v"(t0r[r].sc), "+v"(t0r[r].ar));
            t0r[r].rlo = 0u; t0r[r].rhi = 0u;
            unpack_tile<N8>(t0r[r], shb & 1, hd[r]);
        }
        ra = make_uint4(ra0.x, ra0.y, ra0.z, ra0.w);
        rb = make_uint2(rb0.x, rb0.y);
    }
    // Half blocks with more than 8 salient columns: their further records, one at a time and without any overlap
    // (few: a record covers 8 of the 64 columns).  Kept out of the main loops so that they stay one straight line of
    // K steps (a branch around matrix instructions costs two register copies of the accumulators).
    __device__ void further_records(float4_t (&acc)[4][TT], HalfData<N8> (&hd)[4], uint32_t (&a1)[4][4], uint32_t (&rlo)[4],
                                    uint32_t (&rhi)[4], const char* lds, int shb, int nsh) const {
        if (!(HAS_RES && p.sal_chunks > 1)) return;
        const uint32_t gx = (uint32_t)(i * 64 + (g ^ ((i >> 2) & 3)) * 16);
        for (int sh0 = shb; sh0 < nsh; sh0 += 64) {
            // which of the next 64 half blocks have such records: lane l looks at half block sh0 + l
            const int shl = sh0 + lane < nsh ? sh0 + lane : nsh - 1;
            const uint32_t need_l = p.sal_tab[(((int64_t)(4 * (shl >> 1)) * 2 + (shl & 1)) * p.sal_chunks) * 12 + 5];
            uint64_t todo = __ballot(need_l > 1u && sh0 + lane < nsh);
            while (todo) {
                const int sh = sh0 + __builtin_ctzll(todo);
                todo &= todo - 1;
                const uint32_t* rec0 = p.sal_tab + (((int64_t)(4 * (sh >> 1) + g) * 2 + (sh & 1)) * p.sal_chunks) * 12;
                const int nch = __builtin_amdgcn_readfirstlane((int)rec0[5]);          // the same for the four blocks
                load_hd(sh, hd);
                for (int c = 1; c < nch; c++) {
                    __syncthreads();                             // every wavefront is done with the gathered columns
                    r_gload(sh, c, 0);
                    const uint4 rc = *reinterpret_cast<const uint4*>(rec0 + c * 12);
                    const uint32_t ord = rec0[c * 12 + 4];
                    load_res_words(ord, rlo, rhi);
                    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
                    __syncthreads();
                    ResSel sel;
                    sel.sel0 = rc.x; sel.sel1 = rc.y; sel.bit0 = rc.z; sel.bit1 = rc.w;
#pragma unroll
                    for (int r = 0; r < 4; r++)
                        residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], ord & 31u), hd[r].ar | (hd[r].ar << 16), sel, a1[r]);
#pragma unroll
                    for (int tt = 0; tt < TT; tt++) {
                        const uint4 bt = *reinterpret_cast<const uint4*>(lds + G::XG + tt * 1024 + gx);
                        const half8_t bv = __builtin_bit_cast(half8_t, bt);
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(a1[r]), bv, acc[r][tt], 0, 0, 0);
                    }
                }
            }
        }
    }
    // The same for the kernels on the 32x32 instructions (WIDE records; acc[rs][q] = 32 rows x 32 tokens; gx[bs] = the
    // lane's offset inside the gathered columns for block 2 (g / 2) + bs).
    template <typename Acc>
    __device__ void further_records_wide(Acc (&acc)[2][TT / 2], HalfData<N8> (&hd)[4], uint32_t (&a1)[4][4], uint32_t (&rlo)[4],
                                         uint32_t (&rhi)[4], const char* lds, int shb, int nsh, const uint32_t (&gx)[2]) const {
        constexpr int TQ = TT / 2;
        if (!(HAS_RES && p.sal_chunks > 1)) return;
        for (int sh0 = shb; sh0 < nsh; sh0 += 64) {
            const int shl = sh0 + lane < nsh ? sh0 + lane : nsh - 1;
            const uint32_t need_l = p.sal_tab[(((int64_t)(4 * (shl >> 1)) * 2 + (shl & 1)) * p.sal_chunks) * 12 + 5];
            uint64_t todo = __ballot(need_l > 1u && sh0 + lane < nsh);
            while (todo) {
                const int sh = sh0 + __builtin_ctzll(todo);
                todo &= todo - 1;
                const uint32_t* rec0[2];
#pragma unroll
                for (int bs = 0; bs < 2; bs++)
                    rec0[bs] = p.sal_tab + (((int64_t)(4 * (sh >> 1) + 2 * (g >> 1) + bs) * 2 + (sh & 1)) * p.sal_chunks) * 12;
                const int nch = __builtin_amdgcn_readfirstlane((int)rec0[0][5]);       // the same for the four blocks
                load_hd(sh, hd);
                for (int c = 1; c < nch; c++) {
                    __syncthreads();                             // every wavefront is done with the gathered columns
                    r_gload(sh, c, 0);
                    uint4 rc[2];
                    uint32_t ord[2];
#pragma unroll
                    for (int bs = 0; bs < 2; bs++) {
                        rc[bs] = *reinterpret_cast<const uint4*>(rec0[bs] + c * 12);
                        ord[bs] = rec0[bs][c * 12 + 4];
                    }
#pragma unroll
                    for (int r = 0; r < 4; r++) load_res_words1(ord[r & 1], rlo, rhi, r);
                    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
                    __syncthreads();
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        ResSel sel;
                        sel.sel0 = rc[r & 1].x; sel.sel1 = rc[r & 1].y; sel.bit0 = rc[r & 1].z; sel.bit1 = rc[r & 1].w;
                        residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], ord[r & 1] & 31u), hd[r].ar | (hd[r].ar << 16), sel, a1[r]);
                    }
#pragma unroll
                    for (int u = 0; u < TT; u++) {
                        const uint4 bt = *reinterpret_cast<const uint4*>(lds + G::XG + (u % TQ) * 2048 + gx[u / TQ]);
                        const half8_t bv = __builtin_bit_cast(half8_t, bt);
#pragma unroll
                        for (int rs = 0; rs < 2; rs++)
                            acc[rs][u % TQ] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_half8(a1[2 * rs + u / TQ]), bv, acc[rs][u % TQ], 0, 0, 0);
                    }
                }
            }
        }
    }
};

template <int N8, bool HAS_RES, bool SPLIT, int TT = GM_TT>
__global__ __launch_bounds__(256) void gemm_tiled_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                          void* __restrict__ Y, int y_fp32,
                                                          const __half* __restrict__ xsal, int cfix, int sbs, float* __restrict__ part) {
    typedef GmLds<TT> G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    ScatterLds& lut = *reinterpret_cast<ScatterLds*>(lds + G::LUT);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;     // LDS address of lds[0]
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * G::TOK;
    const int rtw = blockIdx.y * GM_ROWT + wave * 4;                // first row tile of this wavefront
    // K split: this workgroup contracts the superblocks [sbs * blockIdx.z, + sbs) and leaves an fp32 partial tile
    // (a template parameter: the kernel without a split keeps the registers it had before the split existed)
    const int shb = SPLIT ? 2 * sbs * (int)blockIdx.z : 0;         // first (superblock, half) pair: even
    const int nsh = SPLIT && 2 * sbs * ((int)blockIdx.z + 1) < p.nsb * 2 ? 2 * sbs * ((int)blockIdx.z + 1) : p.nsb * 2;   // one past the last
    if constexpr (SPLIT) { Y = part + (int64_t)blockIdx.z * T * p.n; y_fp32 = 1; }
    build_luts<N8>(&lut);

    float4_t acc[4][TT];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
        for (int tt = 0; tt < TT; tt++) acc[r][tt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const GemmStage<N8, HAS_RES, TT> st(p, X, xsal, T, cfix, lds0, t0, rtw, wave, lane);
    constexpr int NGL = TT / 4;

    // ---- the K step: 32 MFMAs (4 row tiles x 8 token tiles) on the A operands `ac` and the B operands b[]; in
    //      their shadow the lane builds the A operands of the next step (`next_a(r)` for row tile r) and, as soon
    //      as the four MFMAs of a token tile have been issued, reloads that tile's B operand for the next step
    //      (`next_b(tt)`).  `extra(tt)` is the share of the staging work that goes with token tile tt. ----
    uint4 b[TT];
    auto kstep = [&](const uint32_t (&ac)[4][4], auto&& next_a, auto&& next_b, auto&& extra) {
#pragma unroll
        for (int tt = 0; tt < TT; tt++) {
            const half8_t bv = __builtin_bit_cast(half8_t, b[tt]);
#pragma unroll
            for (int r = 0; r < 4; r++)
                acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(ac[r]), bv, acc[r][tt], 0, 0, 0);
            next_b(tt);
            if (tt % (TT / 4) == 0) next_a(tt / (TT / 4));
            extra(tt);
        }
        // (Asking the scheduler for an MFMA / LDS read / three vector instructions rhythm through sched_group_barrier
        //  was measured: 6 - 8 % slower on 4:8 layers than its own order, and 20 times the compile time.)
    };
    // B operand of token tile tt: rows 16 tt + i, piece 4 g + tq, at position piece ^ i
    uint32_t bx[2][4];                                              // per window buffer (the offset of a token tile is an immediate)
#pragma unroll
    for (int buf = 0; buf < 2; buf++)
#pragma unroll
        for (int tq = 0; tq < 4; tq++) bx[buf][tq] = (uint32_t)(G::XW + buf * G::XWSZ + i * 256 + ((4 * g + tq) ^ i) * 16);
    auto bread = [&](int buf, int tq, int tt) {
        b[tt] = *reinterpret_cast<const uint4*>(lds + tt * 4096 + bx[buf][tq]);
    };
    const uint32_t gx = (uint32_t)(i * 64 + (g ^ ((i >> 2) & 3)) * 16);

    // ---- prologue: both windows of the first half block, its records, the operands of step 0 ----
    HalfData<N8> hd[4];
    uint32_t TL[4], TH[4];
    uint4 ra = make_uint4(0u, 0u, 0u, 0u);
    uint2 rb = make_uint2(0u, 0u);
    uint32_t a0[4][4], a1[4][4];
    uint32_t rlo[4] = {0u, 0u, 0u, 0u}, rhi[4] = {0u, 0u, 0u, 0u};
    st.x_gload(shb, 0, 0);
    st.x_gload(shb, 1, 1);
    st.r_gload(shb, 0, 0);
    st.first_records(shb, hd, ra, rb);
    if (HAS_RES) st.fetch_res_words(rb.x, rlo, rhi);
    st.scale_tables(hd, TL, TH);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; r++) expand_group<N8>(hd[r], TL[r], TH[r], 0, lut_fetch<N8>(hd[r], 0, &lut, lane & 7), a0[r]);
#pragma unroll
    for (int tt = 0; tt < TT; tt++) bread(0, 0, tt);

    // Loads of one pass, in issue order (NR res_sign words of this pass are older than all of them):
    //   [step 3, after the first barrier]  window 0 of the next pass (8)
    //   [step 4]                           the next pass's half records (NH) and table record (NC)
    //   [step 7, after the second barrier] window 1 (8) and gathered columns (NG) of the next pass
    //   [residual step]                    res_sign words of the next pass (NR)
    constexpr int NG = HAS_RES ? 2 : 0, NR = HAS_RES ? 8 : 0, NC = HAS_RES ? 2 : 0, NH = 4 * TileLoads<false>::count;
    for (int sh = shb; sh < nsh; sh++) {
        const int shn = sh + 1 < nsh ? sh + 1 : sh;                 // the last pass prefetches its own data again
        const int par = sh & 1;
        TileRegs<N8> tn[4];
        uint4_t ran = {0u, 0u, 0u, 0u};
        uint2_t rbn = {0u, 0u};
        auto produce = [&](int t, uint32_t (&an)[4][4]) {
            return [&, t](int r) { expand_group<N8>(hd[r], TL[r], TH[r], t, lut_fetch<N8>(hd[r], t, &lut, lane & 7), an[r]); };
        };
        auto reload = [&](int t) { return [&, t](int tt) { bread(t >> 2, t & 3, tt); }; };
        auto nothing = [](int) {};

        // steps 0 .. 7 = column groups 0 .. 7 of the half block; window 0 holds groups 0..3, window 1 groups 4..7
        kstep(a0, produce(1, a1), reload(1), nothing);
        kstep(a1, produce(2, a0), reload(2), nothing);
        kstep(a0, produce(3, a1), reload(3), nothing);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NR) : "memory");  // window 1 and the gathered columns of this pass are in LDS
        __syncthreads();                                            // ... everyone's; and everyone is done with window 0
        // (the loads are spread over the token tiles of a step, a few at a time: the four wavefronts share one path
        //  to memory, and a burst of loads stalls them all)
        kstep(a1, produce(4, a0), reload(4), [&](int tt) { st.x_gload1(shn, 0, 0, tt); });
        kstep(a0, produce(5, a1), reload(5), [&](int tt) { if (tt % (TT / 4) == 0) st.fetch_hd1(shn, tn, tt / (TT / 4)); if (tt == TT - 1) st.fetch_rec(shn, ran, rbn); });
        kstep(a1, produce(6, a0), reload(6), nothing);
        kstep(a0, produce(7, a1), reload(7), nothing);
        // everything in flight has arrived: window 0 of the next pass, its half records and table record, and the
        // res_sign words of this pass
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]),
                     "+v"(ran), "+v"(rbn) : : "memory");
#pragma unroll
        for (int r = 0; r < 4; r++) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tn[r].m), "+v"(tn[r].s), "+v"(tn[r].r), "+v"(tn[r].sc), "+v"(tn[r].ar));
        __syncthreads();                                            // everyone is done with window 1
        HalfData<N8> hn[4];
        uint32_t TLn[4], THn[4];
#pragma unroll
        for (int r = 0; r < 4; r++) { tn[r].rlo = 0u; tn[r].rhi = 0u; unpack_tile<N8>(tn[r], shn & 1, hn[r]); }
        st.scale_tables(hn, TLn, THn);
        auto produce_n = [&](uint32_t (&an)[4][4]) {
            return [&](int r) { expand_group<N8>(hn[r], TLn[r], THn[r], 0, lut_fetch<N8>(hn[r], 0, &lut, lane & 7), an[r]); };
        };
        auto reload_n = [&](int tt) { bread(0, 0, tt); };
        auto next_loads = [&](int tt) { st.x_gload1(shn, 1, 1, tt); if (tt >= TT - NGL) st.r_gload1(shn, 0, par ^ 1, tt - (TT - NGL)); };
        if (HAS_RES) {
            // residual contraction (Eq. 4) of the first 8 salient columns of every half block: A from the mask and
            // res_sign bits, B = the gathered columns.  (A half block without salient columns has an all-zero A.)
            auto res_a = [&](int r) {
                ResSel sel;
                sel.sel0 = ra.x; sel.sel1 = ra.y; sel.bit0 = ra.z; sel.bit1 = ra.w;
                residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], rb.x & 31u), hd[r].ar | (hd[r].ar << 16), sel, a0[r]);
            };
            const uint32_t gxp = gx + (uint32_t)(G::XG + par * G::XGSZ);
            auto reload_g = [&](int tt) { b[tt] = *reinterpret_cast<const uint4*>(lds + tt * 1024 + gxp); };
            kstep(a1, res_a, reload_g, next_loads);
            // (the res_sign words of the next pass: its table record arrived before the barrier above)
            kstep(a0, produce_n(a1), reload_n, [&](int tt) { if (tt < 4) st.fetch_res_words1(rbn.x, rlo, rhi, tt); });
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int v = 0; v < 4; v++) a0[r][v] = a1[r][v];
        } else {
            kstep(a1, produce_n(a0), reload_n, next_loads);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) { hd[r] = hn[r]; TL[r] = TLn[r]; TH[r] = THn[r]; }
        ra = make_uint4(ran.x, ran.y, ran.z, ran.w);
        rb = make_uint2(rbn.x, rbn.y);
    }
    // nothing may still be on its way to this workgroup's LDS or registers from here on
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]) : : "memory");

    st.further_records(acc, hd, a1, rlo, rhi, lds, shb, nsh);

    __syncthreads();                                                // every wavefront is done with LDS
    store_tile<TT>(acc, lds, p, Y, y_fp32, T, t0, rtw, wave, lane);
}

// ------------------------------------------------------------------------------------------------
// The same pipeline on v_mfma_f32_32x32x16_f16 (asked for by name, see stb_tiled_gemm): half as many matrix
// instructions for the same work, each of which hides more of the vector instructions that follow it (the probe
// below: five against two).  In this pipeline the two forms take the same time to within 1 %: what a wavefront
// issues besides the matrix instructions is what holds it up.
// Per wavefront the tile is the same (64 rows x 128 tokens, 128 accumulator
// registers: 2 x 4 tiles of 32 x 32) and so are the windows, the expansion and the loads; what differs is who holds
// what (WIDE in GemmStage): an instruction contracts 8 columns of block 2 (g / 2) + bs from each K half, bs = 0 / 1
// alternating, so a "step" below is the pair of them: 16 instructions, four operand builds, eight B reads.
//   A  lane 16 g + i: row 16 (g % 2) + i of the 32-row tile rs (row tiles 2 rs, 2 rs + 1), K half g / 2
//   B  lane 16 g + i: token 16 (g % 2) + i of the 32-token tile q, K half g / 2
//   D  lane l, register v: token l % 32, row 8 (v / 4) + 4 (l / 32) + v % 4
// ------------------------------------------------------------------------------------------------
typedef float float16_t __attribute__((ext_vector_type(16)));

template <int TT>
__device__ inline void store_tile_wide(const float16_t (&acc)[2][TT / 2], char* lds, const TiledPlanes& p, void* __restrict__ Y,
                                       int y_fp32, int T, int t0, int rtw, int wave, int lane) {
    const int i = lane & 15, g = lane >> 4;
    const int tl0 = 16 * (g & 1) + i, rl0 = 4 * (g >> 1);           // token inside a 32-token tile, first row inside an 8-row band
    const bool wide = !y_fp32 && (p.n & 7) == 0 && ((uintptr_t)Y & 15) == 0 && (rtw + 4) * 16 <= p.n;     // uniform per wavefront
    if (wide) {
        // through LDS as in store_tile: token rows of 144 bytes, the wavefront's 64 rows in each
        char* const ep = lds + wave * (16 * TT * 144);
#pragma unroll
        for (int rs = 0; rs < 2; rs++)
#pragma unroll
            for (int q = 0; q < TT / 2; q++)
#pragma unroll
                for (int vq = 0; vq < 4; vq++) {
                    const __half2 lo = __floats2half2_rn(-acc[rs][q][4 * vq + 0], -acc[rs][q][4 * vq + 1]);
                    const __half2 hi = __floats2half2_rn(-acc[rs][q][4 * vq + 2], -acc[rs][q][4 * vq + 3]);
                    uint2 v;
                    v.x = __builtin_bit_cast(uint32_t, lo);
                    v.y = __builtin_bit_cast(uint32_t, hi);
                    *reinterpret_cast<uint2*>(ep + (32 * q + tl0) * 144 + (32 * rs + 8 * vq + rl0) * 2) = v;
                }
        __half* const Yh = reinterpret_cast<__half*>(Y);
#pragma unroll
        for (int it = 0; it < 2 * TT; it++) {
            const int tl = 8 * it + (lane >> 3), tok = t0 + tl;
            const uint4 v = *reinterpret_cast<const uint4*>(ep + tl * 144 + (lane & 7) * 16);
            if (tok < T) *reinterpret_cast<uint4*>(Yh + (int64_t)tok * p.n + rtw * 16 + (lane & 7) * 8) = v;
        }
        return;
    }
#pragma unroll
    for (int rs = 0; rs < 2; rs++)
#pragma unroll
        for (int q = 0; q < TT / 2; q++) {
            const int tok = t0 + 32 * q + tl0;
            if (tok >= T) continue;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int row = rtw * 16 + 32 * rs + 8 * (v >> 2) + rl0 + (v & 3);
                if (row >= p.n) continue;
                const float val = -acc[rs][q][v];
                if (y_fp32) reinterpret_cast<float*>(Y)[(int64_t)tok * p.n + row] = val;
                else reinterpret_cast<__half*>(Y)[(int64_t)tok * p.n + row] = __float2half(val);
            }
        }
}

template <int N8, bool HAS_RES, bool SPLIT>
__global__ __launch_bounds__(256) void gemm_wide_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                         void* __restrict__ Y, int y_fp32,
                                                         const __half* __restrict__ xsal, int cfix, int sbs, float* __restrict__ part) {
    constexpr int TT = GM_TT;                                       // B operands per step: 4 token tiles of 32 x the 2 blocks of a K half
    constexpr int TQ = TT / 2;
    typedef GmLds<TT> G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    ScatterLds& lut = *reinterpret_cast<ScatterLds*>(lds + G::LUT);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * G::TOK;
    const int rtw = blockIdx.y * GM_ROWT + wave * 4;
    // K split: this workgroup contracts the superblocks [sbs * blockIdx.z, + sbs) and leaves an fp32 partial tile
    // (a template parameter: the kernel without a split keeps the registers it had before the split existed)
    const int shb = SPLIT ? 2 * sbs * (int)blockIdx.z : 0;         // first (superblock, half) pair: even
    const int nsh = SPLIT && 2 * sbs * ((int)blockIdx.z + 1) < p.nsb * 2 ? 2 * sbs * ((int)blockIdx.z + 1) : p.nsb * 2;   // one past the last
    if constexpr (SPLIT) { Y = part + (int64_t)blockIdx.z * T * p.n; y_fp32 = 1; }
    build_luts<N8>(&lut);

    float16_t acc[2][TQ];
#pragma unroll
    for (int rs = 0; rs < 2; rs++)
#pragma unroll
        for (int q = 0; q < TQ; q++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[rs][q][v] = 0.0f;

    const GemmStage<N8, HAS_RES, TT, true> st(p, X, xsal, T, cfix, lds0, t0, rtw, wave, lane);
    constexpr int NGL = TT / 4;

    // ---- the step: B operand u = (bs = u / TQ, token tile q = u % TQ) meets the A operands of records 2 rs + bs;
    //      the two uses of an accumulator are TT instructions apart ----
    uint4 b[TT];
    auto kstep = [&](const uint32_t (&ac)[4][4], auto&& next_a, auto&& next_b, auto&& extra) {
#pragma unroll
        for (int u = 0; u < TT; u++) {
            const half8_t bv = __builtin_bit_cast(half8_t, b[u]);
#pragma unroll
            for (int rs = 0; rs < 2; rs++)
                acc[rs][u % TQ] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_half8(ac[2 * rs + u / TQ]), bv, acc[rs][u % TQ], 0, 0, 0);
            next_b(u);
            if (u % (TT / 4) == 0) next_a(u / (TT / 4));
            extra(u);
        }
    };
    // B operand u: row 32 q + 16 (g % 2) + i of the window, piece 4 (2 (g / 2) + bs) + tq, at position piece ^ i
    uint32_t bx[2][2][4];
#pragma unroll
    for (int buf = 0; buf < 2; buf++)
#pragma unroll
        for (int bs = 0; bs < 2; bs++)
#pragma unroll
            for (int tq = 0; tq < 4; tq++)
                bx[buf][bs][tq] = (uint32_t)(G::XW + buf * G::XWSZ + (16 * (g & 1) + i) * 256 + ((4 * (2 * (g >> 1) + bs) + tq) ^ i) * 16);
    auto bread = [&](int buf, int tq, int u) {
        b[u] = *reinterpret_cast<const uint4*>(lds + (u % TQ) * 8192 + bx[buf][u / TQ][tq]);
    };
    // gathered columns: row as above (64 bytes each), piece 2 (g / 2) + bs at position piece ^ ((row / 4) % 4)
    uint32_t gx[2];
#pragma unroll
    for (int bs = 0; bs < 2; bs++) gx[bs] = (uint32_t)((16 * (g & 1) + i) * 64 + ((2 * (g >> 1) + bs) ^ ((i >> 2) & 3)) * 16);

    // ---- prologue ----
    HalfData<N8> hd[4];
    uint32_t TL[4], TH[4];
    uint4 ra[2] = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u)};
    uint2 rb[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};
    uint32_t a0[4][4], a1[4][4];
    uint32_t rlo[4] = {0u, 0u, 0u, 0u}, rhi[4] = {0u, 0u, 0u, 0u};
    st.x_gload(shb, 0, 0);
    st.x_gload(shb, 1, 1);
    st.r_gload(shb, 0, 0);
    st.first_records(shb, hd, ra[0], rb[0], &ra[1], &rb[1]);
    if (HAS_RES) {
#pragma unroll
        for (int r = 0; r < 4; r++) st.fetch_res_words1(rb[r & 1].x, rlo, rhi, r);
    }
    st.scale_tables(hd, TL, TH);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; r++) expand_group<N8>(hd[r], TL[r], TH[r], 0, lut_fetch<N8>(hd[r], 0, &lut, lane & 7), a0[r]);
#pragma unroll
    for (int u = 0; u < TT; u++) bread(0, 0, u);

    // Loads of one pass, in issue order (the NR res_sign words of this pass are older than all of them):
    //   [step 3, after the first barrier]  window 0 of the next pass (8)
    //   [step 4]                           the next pass's half records and table records
    //   [step 7, after the second barrier] window 1 (8) and gathered columns of the next pass
    //   [residual step]                    res_sign words of the next pass (NR)
    constexpr int NR = HAS_RES ? 8 : 0;
    for (int sh = shb; sh < nsh; sh++) {
        const int shn = sh + 1 < nsh ? sh + 1 : sh;
        const int par = sh & 1;
        TileRegs<N8> tn[4];
        uint4_t ran[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
        uint2_t rbn[2] = {{0u, 0u}, {0u, 0u}};
        auto produce = [&](int t, uint32_t (&an)[4][4]) {
            return [&, t](int r) { expand_group<N8>(hd[r], TL[r], TH[r], t, lut_fetch<N8>(hd[r], t, &lut, lane & 7), an[r]); };
        };
        auto reload = [&](int t) { return [&, t](int u) { bread(t >> 2, t & 3, u); }; };
        auto nothing = [](int) {};

        kstep(a0, produce(1, a1), reload(1), nothing);
        kstep(a1, produce(2, a0), reload(2), nothing);
        kstep(a0, produce(3, a1), reload(3), nothing);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NR) : "memory");  // window 1 and the gathered columns of this pass are in LDS
        __syncthreads();
        kstep(a1, produce(4, a0), reload(4), [&](int u) { st.x_gload1(shn, 0, 0, u); });
        kstep(a0, produce(5, a1), reload(5), [&](int u) {
            if (u % 2 == 0) st.fetch_hd1(shn, tn, u / 2);
            if (u == 5) st.fetch_rec(shn, ran[0], rbn[0], 0);
            if (u == 7) st.fetch_rec(shn, ran[1], rbn[1], 1);
        });
        kstep(a1, produce(6, a0), reload(6), nothing);
        kstep(a0, produce(7, a1), reload(7), nothing);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]),
                     "+v"(ran[0]), "+v"(rbn[0]), "+v"(ran[1]), "+v"(rbn[1]) : : "memory");
#pragma unroll
        for (int r = 0; r < 4; r++) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tn[r].m), "+v"(tn[r].s), "+v"(tn[r].r), "+v"(tn[r].sc), "+v"(tn[r].ar));
        __syncthreads();                                            // everyone is done with window 1
        HalfData<N8> hn[4];
        uint32_t TLn[4], THn[4];
#pragma unroll
        for (int r = 0; r < 4; r++) { tn[r].rlo = 0u; tn[r].rhi = 0u; unpack_tile<N8>(tn[r], shn & 1, hn[r]); }
        st.scale_tables(hn, TLn, THn);
        auto produce_n = [&](uint32_t (&an)[4][4]) {
            return [&](int r) { expand_group<N8>(hn[r], TLn[r], THn[r], 0, lut_fetch<N8>(hn[r], 0, &lut, lane & 7), an[r]); };
        };
        auto reload_n = [&](int u) { bread(0, 0, u); };
        auto next_loads = [&](int u) { st.x_gload1(shn, 1, 1, u); if (u >= TT - NGL) st.r_gload1(shn, 0, par ^ 1, u - (TT - NGL)); };
        if (HAS_RES) {
            // residual contraction (Eq. 4) of the first 8 salient columns of every half block
            auto res_a = [&](int r) {
                ResSel sel;
                sel.sel0 = ra[r & 1].x; sel.sel1 = ra[r & 1].y; sel.bit0 = ra[r & 1].z; sel.bit1 = ra[r & 1].w;
                residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], rb[r & 1].x & 31u), hd[r].ar | (hd[r].ar << 16), sel, a0[r]);
            };
            const uint32_t gbase = (uint32_t)(G::XG + par * G::XGSZ);
            auto reload_g = [&](int u) { b[u] = *reinterpret_cast<const uint4*>(lds + (u % TQ) * 2048 + gbase + gx[u / TQ]); };
            kstep(a1, res_a, reload_g, next_loads);
            kstep(a0, produce_n(a1), reload_n, [&](int u) { if (u < 4) st.fetch_res_words1(rbn[u & 1].x, rlo, rhi, u); });
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int v = 0; v < 4; v++) a0[r][v] = a1[r][v];
        } else {
            kstep(a1, produce_n(a0), reload_n, next_loads);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) { hd[r] = hn[r]; TL[r] = TLn[r]; TH[r] = THn[r]; }
#pragma unroll
        for (int bs = 0; bs < 2; bs++) {
            ra[bs] = make_uint4(ran[bs].x, ran[bs].y, ran[bs].z, ran[bs].w);
            rb[bs] = make_uint2(rbn[bs].x, rbn[bs].y);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]) : : "memory");

    st.further_records_wide(acc, hd, a1, rlo, rhi, lds, shb, nsh, gx);

    __syncthreads();                                                // every wavefront is done with LDS
    store_tile_wide<TT>(acc, lds, p, Y, y_fp32, T, t0, rtw, wave, lane);
}

// ------------------------------------------------------------------------------------------------
// 2:4 layers on the structured-sparse matrix instruction (Sec. 3.1 / App. C: the paper's own kernel form):
// v_smfmac_f32_16x16x64_f16 takes the kept weights only (8 per lane = 16 columns of the lane's block) and an index
// word that says which 2 of every 4 columns they are, and contracts them with 64 columns of X at once.  Half the
// matrix instructions of the dense kernel above, no scatter table, and a cheaper operand (nothing to spread).
// A pass over a half block is 4 sparse steps of 16 columns per block plus the dense residual step.
// ------------------------------------------------------------------------------------------------
typedef _Float16 half16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint8_t32 __attribute__((ext_vector_type(8)));

// Index register for 32 columns: every mask nibble (two bits set) becomes the positions of its two kept weights,
// low one in bits 1:0, high one in bits 3:2, looked up in an 8-byte table by (nibble >> 1) & 7.
__device__ inline uint32_t index_word24(uint32_t m, uint32_t T0, uint32_t T1, uint32_t K7) {
    const uint32_t t = m >> 1;
    const uint32_t lo = perm(T1, T0, t & K7);
    const uint32_t hi = perm(T1, T0, (t >> 4) & K7);
    return (hi << 4) | lo;
}

// A operand of a sparse step s (columns 16 s .. 16 s + 15 of a half block): the 8 kept weights in slot order, scale
// by region id and sign bit merged in (the first half of expand_group; nothing to spread).  K3, K4, KS: the constants
// 0x03030303, 0x04000400, 0x80008000 in registers (a VOP3 instruction takes one literal).
__device__ inline void sparse_operand(const HalfData<4>& d, uint32_t TLr, uint32_t THr, int s, uint32_t K3, uint32_t K4,
                                      uint32_t KS, uint32_t (&W)[4]) {
    const uint32_t rw = d.r[s >> 1], r2 = rw >> 2;
#pragma unroll
    for (int c = 0; c < 2; c++) {                             // byte 2 (s % 2) + c of the id word: 4 kept weights
        const uint32_t bb = 2 * (s & 1) + c;
        const uint32_t Z = perm(r2, rw, bb | (bb << 8) | ((4 + bb) << 16) | ((4 + bb) << 24));
        W[2 * c] = perm(THr, TLr, and_or_v(Z, K3, K4));
        W[2 * c + 1] = perm(THr, TLr, and_or_v(Z >> 4, K3, K4));
    }
    const uint32_t sbi = (uint32_t)s;                         // byte of the half's sign word
    const uint32_t Xs = perm(d.s[0], d.s[0], 0x000C000Cu | (sbi << 8) | (sbi << 24));
#pragma unroll
    for (int q = 0; q < 4; q++) W[q] = and_or_v(pk_shl(Xs, 7 - 2 * q, 6 - 2 * q), KS, W[q]);
}

template <bool HAS_RES, bool SPLIT, int TT = GM_TT24>
__global__ __launch_bounds__(256) void gemm24_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                      void* __restrict__ Y, int y_fp32,
                                                      const __half* __restrict__ xsal, int cfix, int sbs, float* __restrict__ part) {
    constexpr int N8 = 4;
    typedef GmLds<TT> G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * G::TOK;
    const int rtw = blockIdx.y * GM_ROWT + wave * 4;
    // K split: this workgroup contracts the superblocks [sbs * blockIdx.z, + sbs) and leaves an fp32 partial tile
    // (a template parameter: the kernel without a split keeps the registers it had before the split existed)
    const int shb = SPLIT ? 2 * sbs * (int)blockIdx.z : 0;         // first (superblock, half) pair: even
    const int nsh = SPLIT && 2 * sbs * ((int)blockIdx.z + 1) < p.nsb * 2 ? 2 * sbs * ((int)blockIdx.z + 1) : p.nsb * 2;   // one past the last
    if constexpr (SPLIT) { Y = part + (int64_t)blockIdx.z * T * p.n; y_fp32 = 1; }

    float4_t acc[4][TT];
#pragma unroll
    for (int r = 0; r < 4; r++)
#pragma unroll
        for (int tt = 0; tt < TT; tt++) acc[r][tt] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

    const GemmStage<N8, HAS_RES, TT> st(p, X, xsal, T, cfix, lds0, t0, rtw, wave, lane);
    constexpr int NGL = TT / 4;
    // constants of the operand build, in VGPRs (a VOP3 instruction takes one literal)
    uint32_t T0 = 0x09080404u, T1 = 0x0E0E0D0Cu, K7 = 0x07070707u, K3 = 0x03030303u, K4 = 0x04000400u, KS = 0x80008000u;
    asm volatile("" : "+v"(T0), "+v"(T1), "+v"(K7), "+v"(K3), "+v"(K4), "+v"(KS));
    // A operand of step s (columns 16 s .. 16 s + 15 of the half block of the record's block)
    auto build_a = [&](const HalfData<N8>& d, uint32_t TLr, uint32_t THr, int s, uint32_t (&W)[4]) {
        sparse_operand(d, TLr, THr, s, K3, K4, KS, W);
    };

    // B operand of a sparse step, lane 16 g + n of token tile tt: elements 0..7 = X[token][block g / 2, columns
    // 16 s + 8 (g % 2) ..], elements 8..15 = the same columns of block 2 + g / 2: pieces P and P + 8 of the window row.
    uint32_t bxl[2];
#pragma unroll
    for (int u = 0; u < 2; u++) bxl[u] = (uint32_t)(i * 256 + ((4 * (g >> 1) + 2 * u + (g & 1)) ^ i) * 16);
    uint8_t32 b[TT];
    auto bread = [&](int buf, int u, int tt) {
        const char* base = lds + G::XW + buf * G::XWSZ + tt * 4096;
        const uint4 lo = *reinterpret_cast<const uint4*>(base + bxl[u]);
        const uint4 hi = *reinterpret_cast<const uint4*>(base + (bxl[u] ^ 128u));
        b[tt] = uint8_t32{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    const uint32_t gx = (uint32_t)(i * 64 + (g ^ ((i >> 2) & 3)) * 16);

    // ---- K steps: a sparse one (32 sparse instructions) and the dense residual one (32 MFMAs on the low half of b[]) ----
    auto sstep = [&](auto abid_, const uint32_t (&ac)[4][4], const uint32_t (&idx)[4], auto&& next_a, auto&& next_b, auto&& extra) {
        constexpr int ABID = decltype(abid_)::value;
#pragma unroll
        for (int tt = 0; tt < TT; tt++) {
            const half16_t bv = __builtin_bit_cast(half16_t, b[tt]);
#pragma unroll
            for (int r = 0; r < 4; r++)
                acc[r][tt] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(ac[r]), bv, acc[r][tt], (int)idx[r], 0, ABID);
            next_b(tt);
            if (tt % (TT / 4) == 0) next_a(tt / (TT / 4));
            extra(tt);
        }
    };
    auto dstep = [&](const uint32_t (&ac)[4][4], auto&& next_a, auto&& next_b, auto&& extra) {
#pragma unroll
        for (int tt = 0; tt < TT; tt++) {
            const uint4 bl = make_uint4(b[tt][0], b[tt][1], b[tt][2], b[tt][3]);
            const half8_t bv = __builtin_bit_cast(half8_t, bl);
#pragma unroll
            for (int r = 0; r < 4; r++)
                acc[r][tt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(ac[r]), bv, acc[r][tt], 0, 0, 0);
            next_b(tt);
            if (tt % (TT / 4) == 0) next_a(tt / (TT / 4));
            extra(tt);
        }
    };

    // ---- prologue ----
    HalfData<N8> hd[4];
    uint32_t TL[4], TH[4];
    uint4 ra = make_uint4(0u, 0u, 0u, 0u);
    uint2 rb = make_uint2(0u, 0u);
    uint32_t a0[4][4], a1[4][4], ia[4], ib[4];
    uint32_t rlo[4] = {0u, 0u, 0u, 0u}, rhi[4] = {0u, 0u, 0u, 0u};
    st.x_gload(shb, 0, 0);
    st.x_gload(shb, 1, 1);
    st.r_gload(shb, 0, 0);
    st.first_records(shb, hd, ra, rb);
    if (HAS_RES) {
#pragma unroll
        for (int r = 0; r < 4; r++) st.fetch_res_words1(rb.x, rlo, rhi, r);
    }
    st.scale_tables(hd, TL, TH);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; r++) { build_a(hd[r], TL[r], TH[r], 0, a0[r]); ia[r] = index_word24(hd[r].m[0], T0, T1, K7); }
#pragma unroll
    for (int tt = 0; tt < TT; tt++) bread(0, 0, tt);

    // Loads of one pass, in issue order (the NR res_sign words of this pass are older than all of them):
    //   [step 0]                           the next pass's half records (NH) and table record (NC)
    //   [step 1, after the first barrier]  window 0 of the next pass (8)
    //   [step 3, after the second barrier] window 1 (8) and gathered columns (NG) of the next pass
    //   [residual step]                    res_sign words of the next pass (NR)
    constexpr int NR = HAS_RES ? 8 : 0, NC = HAS_RES ? 2 : 0, NH = 4 * TileLoads<false>::count;
    for (int sh = shb; sh < nsh; sh++) {
        const int shn = sh + 1 < nsh ? sh + 1 : sh;
        const int par = sh & 1;
        TileRegs<N8> tn[4];
        uint4_t ran = {0u, 0u, 0u, 0u};
        uint2_t rbn = {0u, 0u};
        auto nothing = [](int) {};
        // step 0 (window 0): builds step 1, fetches the next pass's records
        sstep(IntC<0>{}, a0, ia, [&](int r) { build_a(hd[r], TL[r], TH[r], 1, a1[r]); }, [&](int tt) { bread(0, 1, tt); },
              [&](int tt) { if (tt % (TT / 4) == 0) st.fetch_hd1(shn, tn, tt / (TT / 4)); if (tt == TT - 1) st.fetch_rec(shn, ran, rbn); });
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NR + NH + NC) : "memory");     // window 1 and the gathered columns of this pass
        __syncthreads();                                            // ... everyone's; and everyone is done with window 0
        // step 1: builds step 2 (window 1) and its index word, loads window 0 of the next pass
        sstep(IntC<1>{}, a1, ia, [&](int r) { build_a(hd[r], TL[r], TH[r], 2, a0[r]); ib[r] = index_word24(hd[r].m[1], T0, T1, K7); },
              [&](int tt) { bread(1, 0, tt); }, [&](int tt) { st.x_gload1(shn, 0, 0, tt); });
        sstep(IntC<0>{}, a0, ib, [&](int r) { build_a(hd[r], TL[r], TH[r], 3, a1[r]); }, [&](int tt) { bread(1, 1, tt); }, nothing);
        // everything in flight has arrived
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]),
                     "+v"(ran), "+v"(rbn) : : "memory");
#pragma unroll
        for (int r = 0; r < 4; r++) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tn[r].m), "+v"(tn[r].s), "+v"(tn[r].r), "+v"(tn[r].sc), "+v"(tn[r].ar));
        __syncthreads();                                            // everyone is done with window 1
        HalfData<N8> hn[4];
        uint32_t TLn[4], THn[4];
#pragma unroll
        for (int r = 0; r < 4; r++) { tn[r].rlo = 0u; tn[r].rhi = 0u; unpack_tile<N8>(tn[r], shn & 1, hn[r]); }
        st.scale_tables(hn, TLn, THn);
        auto next_loads = [&](int tt) { st.x_gload1(shn, 1, 1, tt); if (tt >= TT - NGL) st.r_gload1(shn, 0, par ^ 1, tt - (TT - NGL)); };
        auto reload_n = [&](int tt) { bread(0, 0, tt); };
        if (HAS_RES) {
            auto res_a = [&](int r) {
                ResSel sel;
                sel.sel0 = ra.x; sel.sel1 = ra.y; sel.bit0 = ra.z; sel.bit1 = ra.w;
                residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], rb.x & 31u), hd[r].ar | (hd[r].ar << 16), sel, a0[r]);
            };
            const uint32_t gxp = gx + (uint32_t)(G::XG + par * G::XGSZ);
            auto reload_g = [&](int tt) {
                const uint4 v = *reinterpret_cast<const uint4*>(lds + tt * 1024 + gxp);
                b[tt][0] = v.x; b[tt][1] = v.y; b[tt][2] = v.z; b[tt][3] = v.w;
            };
            sstep(IntC<1>{}, a1, ib, res_a, reload_g, next_loads);
            dstep(a0, [&](int r) { build_a(hn[r], TLn[r], THn[r], 0, a1[r]); ia[r] = index_word24(hn[r].m[0], T0, T1, K7); }, reload_n,
                  [&](int tt) { if (tt < 4) st.fetch_res_words1(rbn.x, rlo, rhi, tt); });
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int v = 0; v < 4; v++) a0[r][v] = a1[r][v];
        } else {
            sstep(IntC<1>{}, a1, ib, [&](int r) { build_a(hn[r], TLn[r], THn[r], 0, a0[r]); }, reload_n, next_loads);
#pragma unroll
            for (int r = 0; r < 4; r++) ia[r] = index_word24(hn[r].m[0], T0, T1, K7);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) { hd[r] = hn[r]; TL[r] = TLn[r]; TH[r] = THn[r]; }
        ra = make_uint4(ran.x, ran.y, ran.z, ran.w);
        rb = make_uint2(rbn.x, rbn.y);
    }
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]) : : "memory");

    st.further_records(acc, hd, a1, rlo, rhi, lds, shb, nsh);
    __syncthreads();
    store_tile<TT>(acc, lds, p, Y, y_fp32, T, t0, rtw, wave, lane);
}

// ------------------------------------------------------------------------------------------------
// The 2:4 kernel on v_smfmac_f32_32x32x32_f16, the one that runs by default: gemm24_kernel with the lane mapping of
// gemm_wide_kernel.  Half the matrix instructions for the same work (2 - 3 % faster with salient columns, a third
// faster without: there the 16x16x64 kernel shuffles 200 accumulator registers per pass).  Operand layout of the instruction (found by probing single-element operands on the
// device): A lane l = row l % 32, its 8 kept weights belong to dense K 16 (l / 32) .. + 15 (element e sits in the
// group of four 4 (e / 2), at the position its two index bits 2e+1:2e of the half chosen by ABID name); B lane l =
// token l % 32, element j = dense K 16 (j / 8) + 8 (l / 32) + j % 8; D as for the dense 32x32 form.
// So K 0..15 of an instruction are 16 columns of block bs and K 16..31 the same columns of block 2 + bs, and a B
// operand is two 16-byte pieces of the window row, P and P ^ 8, as in gemm24_kernel.
// ------------------------------------------------------------------------------------------------
template <bool HAS_RES, bool SPLIT>
__global__ __launch_bounds__(256) void gemm24_wide_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                           void* __restrict__ Y, int y_fp32,
                                                           const __half* __restrict__ xsal, int cfix, int sbs, float* __restrict__ part) {
    constexpr int N8 = 4;
    constexpr int TT = GM_TT24;                                     // B operands per step: 4 token tiles of 32 x 2 (bs)
    constexpr int TQ = TT / 2;
    static_assert(TT == 8, "four records are built over eight B operand slots");
    typedef GmLds<TT> G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4;
    const int t0 = blockIdx.x * G::TOK;
    const int rtw = blockIdx.y * GM_ROWT + wave * 4;
    // K split: this workgroup contracts the superblocks [sbs * blockIdx.z, + sbs) and leaves an fp32 partial tile
    // (a template parameter: the kernel without a split keeps the registers it had before the split existed)
    const int shb = SPLIT ? 2 * sbs * (int)blockIdx.z : 0;         // first (superblock, half) pair: even
    const int nsh = SPLIT && 2 * sbs * ((int)blockIdx.z + 1) < p.nsb * 2 ? 2 * sbs * ((int)blockIdx.z + 1) : p.nsb * 2;   // one past the last
    if constexpr (SPLIT) { Y = part + (int64_t)blockIdx.z * T * p.n; y_fp32 = 1; }

    float16_t acc[2][TQ];
#pragma unroll
    for (int rs = 0; rs < 2; rs++)
#pragma unroll
        for (int q = 0; q < TQ; q++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[rs][q][v] = 0.0f;

    const GemmStage<N8, HAS_RES, TT, true> st(p, X, xsal, T, cfix, lds0, t0, rtw, wave, lane);
    constexpr int NGL = TT / 4;
    uint32_t T0 = 0x09080404u, T1 = 0x0E0E0D0Cu, K7 = 0x07070707u, K3 = 0x03030303u, K4 = 0x04000400u, KS = 0x80008000u;
    asm volatile("" : "+v"(T0), "+v"(T1), "+v"(K7), "+v"(K3), "+v"(K4), "+v"(KS));
    // A operand of step s (columns 16 s .. 16 s + 15 of the half block of the record's block)
    auto build_a = [&](const HalfData<N8>& d, uint32_t TLr, uint32_t THr, int s, uint32_t (&W)[4]) {
        sparse_operand(d, TLr, THr, s, K3, K4, KS, W);
    };

    // B operand u = (bs = u / TQ, token tile q = u % TQ) of step s, lane 16 g + i: row 32 q + 16 (g % 2) + i of the
    // window s / 2, pieces P = 4 bs + 2 (s % 2) + g / 2 (block bs) and P + 8 (block 2 + bs), at positions P ^ i, (P + 8) ^ i
    uint32_t bxl[2][2];
#pragma unroll
    for (int bs = 0; bs < 2; bs++)
#pragma unroll
        for (int u2 = 0; u2 < 2; u2++) bxl[bs][u2] = (uint32_t)((16 * (g & 1) + i) * 256 + ((4 * bs + 2 * u2 + (g >> 1)) ^ i) * 16);
    uint8_t32 b[TT];
    auto bread = [&](int buf, int u2, int u) {
        const char* base = lds + G::XW + buf * G::XWSZ + (u % TQ) * 8192;
        const uint4 lo = *reinterpret_cast<const uint4*>(base + bxl[u / TQ][u2]);
        const uint4 hi = *reinterpret_cast<const uint4*>(base + (bxl[u / TQ][u2] ^ 128u));
        b[u] = uint8_t32{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    uint32_t gx[2];
#pragma unroll
    for (int bs = 0; bs < 2; bs++) gx[bs] = (uint32_t)((16 * (g & 1) + i) * 64 + ((2 * (g >> 1) + bs) ^ ((i >> 2) & 3)) * 16);

    // ---- K steps: a sparse one (16 sparse instructions) and the dense residual one (16 MFMAs on the low half of b[]) ----
    auto sstep = [&](auto abid_, const uint32_t (&ac)[4][4], const uint32_t (&idx)[4], auto&& next_a, auto&& next_b, auto&& extra) {
        constexpr int ABID = decltype(abid_)::value;
#pragma unroll
        for (int u = 0; u < TT; u++) {
            const half16_t bv = __builtin_bit_cast(half16_t, b[u]);
#pragma unroll
            for (int rs = 0; rs < 2; rs++)
                acc[rs][u % TQ] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(as_half8(ac[2 * rs + u / TQ]), bv, acc[rs][u % TQ], (int)idx[2 * rs + u / TQ], 0, ABID);
            next_b(u);
            if (u % 2 == 0) next_a(u / 2);
            extra(u);
        }
    };
    auto dstep = [&](const uint32_t (&ac)[4][4], auto&& next_a, auto&& next_b, auto&& extra) {
#pragma unroll
        for (int u = 0; u < TT; u++) {
            const uint4 bl = make_uint4(b[u][0], b[u][1], b[u][2], b[u][3]);
            const half8_t bv = __builtin_bit_cast(half8_t, bl);
#pragma unroll
            for (int rs = 0; rs < 2; rs++)
                acc[rs][u % TQ] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_half8(ac[2 * rs + u / TQ]), bv, acc[rs][u % TQ], 0, 0, 0);
            next_b(u);
            if (u % 2 == 0) next_a(u / 2);
            extra(u);
        }
    };

    // ---- prologue ----
    HalfData<N8> hd[4];
    uint32_t TL[4], TH[4];
    uint4 ra[2] = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u)};
    uint2 rb[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};
    uint32_t a0[4][4], a1[4][4], ia[4], ib[4];
    uint32_t rlo[4] = {0u, 0u, 0u, 0u}, rhi[4] = {0u, 0u, 0u, 0u};
    st.x_gload(shb, 0, 0);
    st.x_gload(shb, 1, 1);
    st.r_gload(shb, 0, 0);
    st.first_records(shb, hd, ra[0], rb[0], &ra[1], &rb[1]);
    if (HAS_RES) {
#pragma unroll
        for (int r = 0; r < 4; r++) st.fetch_res_words1(rb[r & 1].x, rlo, rhi, r);
    }
    st.scale_tables(hd, TL, TH);
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 4; r++) { build_a(hd[r], TL[r], TH[r], 0, a0[r]); ia[r] = index_word24(hd[r].m[0], T0, T1, K7); }
#pragma unroll
    for (int u = 0; u < TT; u++) bread(0, 0, u);

    // Loads of one pass, in issue order (the NR res_sign words of this pass are older than all of them):
    //   [step 0]                           the next pass's half records (NH) and table records (NC)
    //   [step 1, after the first barrier]  window 0 of the next pass (8)
    //   [step 3, after the second barrier] window 1 (8) and gathered columns of the next pass
    //   [residual step]                    res_sign words of the next pass (NR)
    constexpr int NR = HAS_RES ? 8 : 0, NC = HAS_RES ? 4 : 0, NH = 4 * TileLoads<false>::count;
    for (int sh = shb; sh < nsh; sh++) {
        const int shn = sh + 1 < nsh ? sh + 1 : sh;
        const int par = sh & 1;
        TileRegs<N8> tn[4];
        uint4_t ran[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
        uint2_t rbn[2] = {{0u, 0u}, {0u, 0u}};
        auto nothing = [](int) {};
        sstep(IntC<0>{}, a0, ia, [&](int r) { build_a(hd[r], TL[r], TH[r], 1, a1[r]); }, [&](int u) { bread(0, 1, u); },
              [&](int u) {
                  if (u % 2 == 0) st.fetch_hd1(shn, tn, u / 2);
                  if (u == 5) st.fetch_rec(shn, ran[0], rbn[0], 0);
                  if (u == 7) st.fetch_rec(shn, ran[1], rbn[1], 1);
              });
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(NR + NH + NC) : "memory");     // window 1 and the gathered columns of this pass
        __syncthreads();
        sstep(IntC<1>{}, a1, ia, [&](int r) { build_a(hd[r], TL[r], TH[r], 2, a0[r]); ib[r] = index_word24(hd[r].m[1], T0, T1, K7); },
              [&](int u) { bread(1, 0, u); }, [&](int u) { st.x_gload1(shn, 0, 0, u); });
        sstep(IntC<0>{}, a0, ib, [&](int r) { build_a(hd[r], TL[r], TH[r], 3, a1[r]); }, [&](int u) { bread(1, 1, u); }, nothing);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]),
                     "+v"(ran[0]), "+v"(rbn[0]), "+v"(ran[1]), "+v"(rbn[1]) : : "memory");
#pragma unroll
        for (int r = 0; r < 4; r++) asm volatile("s_waitcnt vmcnt(0)" : "+v"(tn[r].m), "+v"(tn[r].s), "+v"(tn[r].r), "+v"(tn[r].sc), "+v"(tn[r].ar));
        __syncthreads();                                            // everyone is done with window 1
        HalfData<N8> hn[4];
        uint32_t TLn[4], THn[4];
#pragma unroll
        for (int r = 0; r < 4; r++) { tn[r].rlo = 0u; tn[r].rhi = 0u; unpack_tile<N8>(tn[r], shn & 1, hn[r]); }
        st.scale_tables(hn, TLn, THn);
        auto next_loads = [&](int u) { st.x_gload1(shn, 1, 1, u); if (u >= TT - NGL) st.r_gload1(shn, 0, par ^ 1, u - (TT - NGL)); };
        auto reload_n = [&](int u) { bread(0, 0, u); };
        if (HAS_RES) {
            auto res_a = [&](int r) {
                ResSel sel;
                sel.sel0 = ra[r & 1].x; sel.sel1 = ra[r & 1].y; sel.bit0 = ra[r & 1].z; sel.bit1 = ra[r & 1].w;
                residual_chunk(hd[r].m, __builtin_amdgcn_alignbit(rhi[r], rlo[r], rb[r & 1].x & 31u), hd[r].ar | (hd[r].ar << 16), sel, a0[r]);
            };
            const uint32_t gbase = (uint32_t)(G::XG + par * G::XGSZ);
            auto reload_g = [&](int u) {
                const uint4 v = *reinterpret_cast<const uint4*>(lds + (u % TQ) * 2048 + gbase + gx[u / TQ]);
                b[u][0] = v.x; b[u][1] = v.y; b[u][2] = v.z; b[u][3] = v.w;
            };
            sstep(IntC<1>{}, a1, ib, res_a, reload_g, next_loads);
            dstep(a0, [&](int r) { build_a(hn[r], TLn[r], THn[r], 0, a1[r]); ia[r] = index_word24(hn[r].m[0], T0, T1, K7); }, reload_n,
                  [&](int u) { if (u < 4) st.fetch_res_words1(rbn[u & 1].x, rlo, rhi, u); });
#pragma unroll
            for (int r = 0; r < 4; r++)
#pragma unroll
                for (int v = 0; v < 4; v++) a0[r][v] = a1[r][v];
        } else {
            sstep(IntC<1>{}, a1, ib, [&](int r) { build_a(hn[r], TLn[r], THn[r], 0, a0[r]); }, reload_n, next_loads);
#pragma unroll
            for (int r = 0; r < 4; r++) ia[r] = index_word24(hn[r].m[0], T0, T1, K7);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) { hd[r] = hn[r]; TL[r] = TLn[r]; TH[r] = THn[r]; }
#pragma unroll
        for (int bs = 0; bs < 2; bs++) {
            ra[bs] = make_uint4(ran[bs].x, ran[bs].y, ran[bs].z, ran[bs].w);
            rb[bs] = make_uint2(rbn[bs].x, rbn[bs].y);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(rlo[0]), "+v"(rlo[1]), "+v"(rlo[2]), "+v"(rlo[3]), "+v"(rhi[0]), "+v"(rhi[1]), "+v"(rhi[2]), "+v"(rhi[3]) : : "memory");

    st.further_records_wide(acc, hd, a1, rlo, rhi, lds, shb, nsh, gx);
    __syncthreads();
    store_tile_wide<TT>(acc, lds, p, Y, y_fp32, T, t0, rtw, wave, lane);
}

// K split: the partial tiles [split][T][n] (fp32, already negated back) are added in split order and stored as Y.
__global__ __launch_bounds__(256) void gemm_splitk_reduce_kernel(const float* __restrict__ part, int S, int64_t count,
                                                                 void* __restrict__ Y, int y_fp32) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= count) return;
    float s = part[e];
    for (int c = 1; c < S; c++) s += part[(int64_t)c * count + e];
    if (y_fp32) reinterpret_cast<float*>(Y)[e] = s;
    else reinterpret_cast<__half*>(Y)[e] = __float2half(s);
}

#include "stb_gemm_shared.hpp"

template <int N8, bool HAS_RES, int TT = GM_TT>
hipError_t launch_gemm(dim3 grid, hipStream_t st, const TiledPlanes& p, const __half* X, int T, void* Y, int y_fp32,
                       const __half* xsal, int cfix, int sbs, float* part) {
    // two instantiations: with and without the K split
    static std::atomic<bool> attr_set[2] = {{false}, {false}};         // a failure is not remembered: the next call tries again
    const int sp = sbs ? 1 : 0;
    const void* fn = sp ? (const void*)gemm_tiled_kernel<N8, HAS_RES, true, TT> : (const void*)gemm_tiled_kernel<N8, HAS_RES, false, TT>;
    if (!attr_set[sp].load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, GmLds<TT>::TOTAL);
        if (attr != hipSuccess) return attr;
        attr_set[sp].store(true, std::memory_order_release);
    }
    if (sp) hipLaunchKernelGGL((gemm_tiled_kernel<N8, HAS_RES, true, TT>), grid, dim3(256), GmLds<TT>::TOTAL, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    else hipLaunchKernelGGL((gemm_tiled_kernel<N8, HAS_RES, false, TT>), grid, dim3(256), GmLds<TT>::TOTAL, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    return hipGetLastError();
}

template <int N8, bool HAS_RES>
hipError_t launch_gemm_wide(dim3 grid, hipStream_t st, const TiledPlanes& p, const __half* X, int T, void* Y, int y_fp32,
                            const __half* xsal, int cfix, int sbs, float* part) {
    // two instantiations: with and without the K split
    static std::atomic<bool> attr_set[2] = {{false}, {false}};         // a failure is not remembered: the next call tries again
    const int sp = sbs ? 1 : 0;
    const void* fn = sp ? (const void*)gemm_wide_kernel<N8, HAS_RES, true> : (const void*)gemm_wide_kernel<N8, HAS_RES, false>;
    if (!attr_set[sp].load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, GmLds<GM_TT>::TOTAL);
        if (attr != hipSuccess) return attr;
        attr_set[sp].store(true, std::memory_order_release);
    }
    if (sp) hipLaunchKernelGGL((gemm_wide_kernel<N8, HAS_RES, true>), grid, dim3(256), GmLds<GM_TT>::TOTAL, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    else hipLaunchKernelGGL((gemm_wide_kernel<N8, HAS_RES, false>), grid, dim3(256), GmLds<GM_TT>::TOTAL, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    return hipGetLastError();
}

template <bool HAS_RES>
hipError_t launch_gemm24_wide(dim3 grid, hipStream_t st, const TiledPlanes& p, const __half* X, int T, void* Y, int y_fp32,
                              const __half* xsal, int cfix, int sbs, float* part) {
    // two instantiations: with and without the K split
    static std::atomic<bool> attr_set[2] = {{false}, {false}};         // a failure is not remembered: the next call tries again
    const int sp = sbs ? 1 : 0;
    const void* fn = sp ? (const void*)gemm24_wide_kernel<HAS_RES, true> : (const void*)gemm24_wide_kernel<HAS_RES, false>;
    if (!attr_set[sp].load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, GmLds<GM_TT24>::TOTAL24);
        if (attr != hipSuccess) return attr;
        attr_set[sp].store(true, std::memory_order_release);
    }
    if (sp) hipLaunchKernelGGL((gemm24_wide_kernel<HAS_RES, true>), grid, dim3(256), GmLds<GM_TT24>::TOTAL24, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    else hipLaunchKernelGGL((gemm24_wide_kernel<HAS_RES, false>), grid, dim3(256), GmLds<GM_TT24>::TOTAL24, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    return hipGetLastError();
}

template <bool HAS_RES, int TT = GM_TT24>
hipError_t launch_gemm24(dim3 grid, hipStream_t st, const TiledPlanes& p, const __half* X, int T, void* Y, int y_fp32,
                         const __half* xsal, int cfix, int sbs, float* part) {
    // two instantiations: with and without the K split
    static std::atomic<bool> attr_set[2] = {{false}, {false}};         // a failure is not remembered: the next call tries again
    const int sp = sbs ? 1 : 0;
    const void* fn = sp ? (const void*)gemm24_kernel<HAS_RES, true, TT> : (const void*)gemm24_kernel<HAS_RES, false, TT>;
    if (!attr_set[sp].load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, GmLds<TT>::TOTAL24);
        if (attr != hipSuccess) return attr;
        attr_set[sp].store(true, std::memory_order_release);
    }
    if (sp) hipLaunchKernelGGL((gemm24_kernel<HAS_RES, true, TT>), grid, dim3(256), GmLds<TT>::TOTAL24, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    else hipLaunchKernelGGL((gemm24_kernel<HAS_RES, false, TT>), grid, dim3(256), GmLds<TT>::TOTAL24, st, p, X, T, Y, y_fp32, xsal, cfix, sbs, part);
    return hipGetLastError();
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// Measurement aid: the rate at which one wavefront per SIMD issues the matrix instructions of the kernels above (and
// their 32x32 forms) on independent accumulators, alone or with V vector instructions after each.  (The scheduling
// fences keep every accumulator updated in place: left to itself the compiler picks another destination register for
// half of them, at four register copies and a no-op per instruction, and the 16x16x32 form looks a third slower than
// it is.)
// ------------------------------------------------------------------------------------------------
namespace {
template <int KIND, int V, bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int steps, float4_t* __restrict__ sink) {
    typedef float float16_t __attribute__((ext_vector_type(16)));
    constexpr bool WIDE = KIND >= 2;                    // 32x32 tiles: 8 accumulators of 16 registers, else 32 of 4
    float4_t acc[32];
    float16_t accw[8];
#pragma unroll
    for (int q = 0; q < 32; q++) acc[q] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int q = 0; q < 8; q++)
#pragma unroll
        for (int e = 0; e < 16; e++) accw[q][e] = 0.0f;
    const uint32_t seed = threadIdx.x * 0x9E3779B9u + blockIdx.x;
    uint32_t w[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        w[j] = 0x3C003C00u ^ ((seed >> j) & 0x00010001u);      // fp16 values next to 1.0
        if (RANDOM) {
            // every operand bit random (sign, mantissa, exponent 13..15: magnitudes in [0.25, 2)): the matrix pipes run
            // slower on operands like these than on the near-constant ones above (measured; presumably a power limit)
            uint32_t h = (seed + (uint32_t)j * 0x85EBCA6Bu) * 0xC2B2AE35u;
            h ^= h >> 15; h *= 0x27D4EB2Fu; h ^= h >> 13;
            const uint32_t e0 = 13u + (h & 3u) % 3u, e1 = 13u + ((h >> 2) & 3u) % 3u;
            w[j] = (h & 0x83FF83FFu) | (e0 << 10) | (e1 << 26);
        }
    }
    const uint4 av4 = make_uint4(w[0], w[1], w[2], w[3]);
    const half8_t av = __builtin_bit_cast(half8_t, av4);
    const half8_t bv = __builtin_bit_cast(half8_t, make_uint4(w[4], w[5], w[6], w[7]));
    typedef uint32_t u8v __attribute__((ext_vector_type(8)));
    const u8v bv8 = {w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7]};
    const half16_t bw = __builtin_bit_cast(half16_t, bv8);
    uint32_t x[8];                                      // eight independent chains of vector instructions
#pragma unroll
    for (int j = 0; j < 8; j++) x[j] = seed * (uint32_t)(2 * j + 3);
    const uint32_t sel = 0x05040100u + (blockIdx.x & 1u);
    for (int it = 0; it < steps; it++) {
#pragma unroll
        for (int q = 0; q < 32; q++) {
            if (KIND == 0) acc[q] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc[q], 0, 0, 0);
            else if (KIND == 1) acc[q] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(av, bw, acc[q], 0x44444444, 0, 0);
            else if (KIND == 2) accw[q % 8] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, bv, accw[q % 8], 0, 0, 0);
            else accw[q % 8] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(av, bw, accw[q % 8], 0x44444444, 0, 0);
            __builtin_amdgcn_sched_barrier(0);          // the vector instructions stay behind their matrix instruction
#pragma unroll
            for (int v = 0; v < V; v++) {
                const int j = (q * V + v) % 8;
                x[j] = perm(x[j], x[(j + 1) % 8], sel);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float4_t t = {0.0f, 0.0f, 0.0f, 0.0f};
    if (WIDE) {
#pragma unroll
        for (int q = 0; q < 8; q++)
#pragma unroll
            for (int e = 0; e < 16; e++) t[e % 4] += accw[q][e];
    } else {
#pragma unroll
        for (int q = 0; q < 32; q++) t += acc[q];
    }
    uint32_t xx = 0u;
#pragma unroll
    for (int j = 0; j < 8; j++) xx ^= x[j];
    t[0] += (float)(xx & 1u);
    sink[blockIdx.x * 256 + threadIdx.x] = t;
}
}  // namespace

extern "C" int stb_tiled_probe_mfma(int kind, int valu, int steps, int n_workgroups, void* sink, void* stream, int* hip_err) {
    if (kind < 0 || kind > 7) return STB_EINVAL;
    const dim3 grid(n_workgroups), wg(256);
    const hipStream_t st = (hipStream_t)stream;
    float4_t* out = (float4_t*)sink;
    const bool random = kind >= 4;
    kind &= 3;
#define STB_PROBE(K, V) { if (random) hipLaunchKernelGGL((probe_mfma_kernel<K, V, true>), grid, wg, 0, st, steps, out); \
                          else hipLaunchKernelGGL((probe_mfma_kernel<K, V, false>), grid, wg, 0, st, steps, out); }
#define STB_PROBE_KIND(K) \
    if (kind == K && valu == 0) STB_PROBE(K, 0) \
    else if (kind == K && valu == 2) STB_PROBE(K, 2) \
    else if (kind == K && valu == 3) STB_PROBE(K, 3) \
    else if (kind == K && valu == 5) STB_PROBE(K, 5) \
    else if (kind == K && valu == 8) STB_PROBE(K, 8)
    STB_PROBE_KIND(0)
    else STB_PROBE_KIND(1)
    else STB_PROBE_KIND(2)
    else STB_PROBE_KIND(3)
    else return STB_EINVAL;
#undef STB_PROBE_KIND
#undef STB_PROBE
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}

static int64_t round_up256(int64_t v) { return (v + 255) / 256 * 256; }
static int cfix_of(const stb_layout_t* L) { return (L->max_sal_half + 7) / 8; }

// K split: with fewer than 200 workgroups in the (token tile, row group) grid the superblocks are dealt to up to 16
// groups of workgroups, each of which leaves an fp32 partial tile in the workspace; a second kernel adds them in order.
// Returns the number of superblocks per group (0: no split) and the number of groups.
static int gemm_split(const stb_layout_t* L, int T, int tok, int* groups) {
    const int64_t base = (int64_t)((T + tok - 1) / tok) * ((L->n_row_tiles + GM_ROWT - 1) / GM_ROWT);
    *groups = 1;
    if (base >= 200 || L->n_super < 2) return 0;
    int S = (int)((256 + base - 1) / base);
    S = S > 16 ? 16 : S;
    S = S > L->n_super ? L->n_super : S;
    if (S < 2) return 0;
    const int sbs = (L->n_super + S - 1) / S;
    *groups = (L->n_super + sbs - 1) / sbs;
    return *groups > 1 ? sbs : 0;
}
static int64_t gather_bytes(const stb_layout_t* L, int T) { return round_up256((int64_t)T * L->n_super * 2 * cfix_of(L) * 32 * 2); }

extern "C" int64_t stb_tiled_gemm_workspace(const stb_layout_t* L, int T) {
    // the gathered salient columns of X, then the partial tiles of a K split (both token-tile sizes give the same
    // number of groups or fewer for the larger one: take the larger need)
    int g0 = 1, g1 = 1;
    const int s0 = gemm_split(L, T, GmLds<GM_TT>::TOK, &g0), s1 = gemm_split(L, T, GmLds<GM_TT24>::TOK, &g1);
    const int gmax = (s0 ? g0 : 0) > (s1 ? g1 : 0) ? (s0 ? g0 : 0) : (s1 ? g1 : 0);
    return gather_bytes(L, T) + round_up256((int64_t)gmax * T * L->cfg.n_out * 4);
}

extern "C" int stb_tiled_gemm(const stb_layout_t* L, const void* X, int T, void* Y, int y_fp32, void* workspace,
                              int64_t workspace_bytes, void* stream, int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    const TiledPlanes p = make_tiled(L);
    const int cfix = cfix_of(L);
    const bool res = p.res_words > 0 && cfix > 0;
    const hipStream_t st = (hipStream_t)stream;
    const int64_t need = stb_tiled_gemm_workspace(L, T);
    if (need > 0) {
        if (!workspace) return STB_ENULL;
        if (workspace_bytes < need) return STB_EINVAL;
        if ((uintptr_t)workspace % 256) return STB_EALIGN;
    }
    if (res) {
        const int64_t pieces = (int64_t)T * p.nsb * 2 * cfix * 4;
        hipLaunchKernelGGL(gemm_gather_kernel, dim3((unsigned)((pieces + 255) / 256)), dim3(256), 0, st, p,
                           (const __half*)X, T, (__half*)workspace, cfix);
    }
    // stb_set_kernel_override: 1 keeps 2:4 layers on the dense-instruction kernel (16x16x32 form), 2 runs its 32x32x16
    // form on any layer, 3 runs 2:4 layers on the 16x16x64 form of the sparse instruction instead of the 32x32x32 one,
    // 4 runs any layer on the shared-expansion kernel: the tests use them to run every kernel on every case it can
    // take.
    const int which = stb_kernel_override(2);
    const int n8 = stb_tiled_slots(&L->cfg);             // slots per 8 columns in the planes (4 or 6)
    const __half* xh = (const __half*)X;
    const __half* xs = (const __half*)workspace;
    hipError_t e;
    // override 4: the kernel that shares the expanded operands through LDS (any layer; measured slower than the
    // kernels below, see stb_gemm_shared.hpp)
    const bool is24 = L->cfg.N == 2 && L->cfg.M == 4;
    if (which == 4) {
        if (n8 == 4) e = res ? launch_gemm_shared<4, true>(st, p, xh, T, Y, y_fp32, xs, cfix) : launch_gemm_shared<4, false>(st, p, xh, T, Y, y_fp32, xs, cfix);
        else e = res ? launch_gemm_shared<6, true>(st, p, xh, T, Y, y_fp32, xs, cfix) : launch_gemm_shared<6, false>(st, p, xh, T, Y, y_fp32, xs, cfix);
        *hip_err = (int)e;
        return e == hipSuccess ? STB_OK : STB_EHIP;
    }
    const bool sparse_ok = is24 && which != 1 && which != 2;
    const bool narrow = which != 2;
    const bool sparse32 = sparse_ok && which != 3;
    // up to GM_SMALL_TOK tokens: the instantiations with half as many token tiles per workgroup (half the matrix
    // instructions on padding; 2:4 layers take the 16x16x64 form, whose pipeline is written for any tile count)
    const bool small = which == 0 && T <= GM_SMALL_TOK;
    const int tok = small ? GM_SMALL_TOK : sparse_ok ? GmLds<GM_TT24>::TOK : GmLds<GM_TT>::TOK;      // tokens per workgroup of the kernel that runs
    int groups = 1;
    const int sbs = gemm_split(L, T, tok, &groups);
    float* part = sbs ? (float*)((char*)workspace + gather_bytes(L, T)) : nullptr;
    const dim3 grid((T + tok - 1) / tok, (p.nrt + GM_ROWT - 1) / GM_ROWT, groups);
    if (small && sparse_ok) e = res ? launch_gemm24<true, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm24<false, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (small && n8 == 4) e = res ? launch_gemm<4, true, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm<4, false, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (small) e = res ? launch_gemm<6, true, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm<6, false, GM_SMALL_TT>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (sparse32) e = res ? launch_gemm24_wide<true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm24_wide<false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (sparse_ok) e = res ? launch_gemm24<true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm24<false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (narrow && n8 == 4) e = res ? launch_gemm<4, true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm<4, false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (narrow) e = res ? launch_gemm<6, true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm<6, false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else if (n8 == 4) e = res ? launch_gemm_wide<4, true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm_wide<4, false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    else e = res ? launch_gemm_wide<6, true>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part) : launch_gemm_wide<6, false>(grid, st, p, xh, T, Y, y_fp32, xs, cfix, sbs, part);
    if (e == hipSuccess && sbs) {
        const int64_t count = (int64_t)T * p.n;
        hipLaunchKernelGGL(gemm_splitk_reduce_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, part, groups, count, Y, y_fp32);
        e = hipGetLastError();
    }
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}
