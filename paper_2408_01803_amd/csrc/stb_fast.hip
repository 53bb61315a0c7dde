// Decode GEMV and verification dequantiser for the tiled device order (STB_KIND_TILED), gfx950.
// The expansion of packed bits into matrix-core operands is in stb_tiled.hpp.
#include "stb_tiled.hpp"

#include <atomic>
#include <cstdlib>

using namespace stbt;

#ifndef STB_VARIANT
#define STB_VARIANT 0
#endif
#define STB_GEMV_PHASE 6
#define STB_GEMV_RESW 6144        // uint32 words of LDS for the res_sign words of a workgroup's row tiles
#ifndef STB_LUT_AHEAD
#define STB_LUT_AHEAD 2
#endif


namespace {

// ------------------------------------------------------------------------------------------------
// stb_dequant on the tiled order: one wavefront per tile, lane (i, g) writes the 128 columns of its
// (row, block), half by half, with the same expansion code the product kernels use.  Salient weights are
// reassembled as f32(s*alpha_o + t*alpha_r) from the two fp16 terms with one fp32 addition.
// ------------------------------------------------------------------------------------------------
template <int N8>
__global__ __launch_bounds__(64) void dequant_tiled_kernel(TiledPlanes p, float* __restrict__ out) {
    __shared__ ScatterLds lut;
    build_luts<N8>(&lut);
    __syncthreads();
    const int rt = blockIdx.x / p.nsb, sb = blockIdx.x % p.nsb;
    const int lane = threadIdx.x, i = lane & 15, g = lane >> 4;
    const int q = 4 * sb + g, row = rt * 16 + i;
    if (row >= p.n || q >= p.nb) return;
    uint32_t ord = p.res_words ? p.sal_prefix[q] : 0u;      // index of the block's first salient column
    float* o = out + (int64_t)row * p.k + (int64_t)q * 128;
    for (int half = 0; half < 2; half++) {
        const LaneOffsets lo = lane_offsets<N8>(lane, half);
        HalfData<N8> d;
        load_half<N8>(p, (int64_t)rt * p.nsb + sb, lo, half, d);
        const uint32_t TL = perm(d.sc.y, d.sc.x, 0x06040200u), TH = perm(d.sc.y, d.sc.x, 0x07050301u);
        const float ar = __half2float(__ushort_as_half((unsigned short)d.ar));
#pragma unroll
        for (int t = 0; t < 8; t++) {
            uint32_t e[4];
            expand_group<N8>(d, TL, TH, t, lut_fetch<N8>(d, t, &lut, lane & 7), e);
            const half8_t a = as_half8(e);
            const uint32_t mb = (d.m[t >> 2] >> (8 * (t & 3))) & 0xFFu;
            const uint32_t salb = p.res_words ? (p.sal_bitmap[4 * q + 2 * half + (t >> 2)] >> (8 * (t & 3))) & 0xFFu : 0u;
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
            float* dst = o + 64 * half + 8 * t;
            *reinterpret_cast<float4*>(dst) = make_float4(vals[0], vals[1], vals[2], vals[3]);
            *reinterpret_cast<float4*>(dst + 4) = make_float4(vals[4], vals[5], vals[6], vals[7]);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Decode GEMV (App. C: the memory-bound regime), the kernel with thin wavefronts.  stb_gemv uses it when the LDS
// areas of the fat-wavefront kernel (stb_gemv24.hip) do not fit, and the tests run it on every tiled case.
//
// Workgroup (gr, ks) of the grid owns SPS superblocks of the columns (column split ks) and 16 / (2*SPS) row
// streams of R 16-row tiles; a wavefront works on one half block (64 columns of each of the 4 blocks) of one
// superblock of one row stream.  Everything that depends on the columns only -- the 8 B operands holding x for
// the wavefront's 4 x 64 columns, the salient-column selectors and the gathered x of the salient columns -- is
// loaded once (through LDS when it fits) and stays in registers while the wavefront streams its R half tiles of
// packed weights, three in flight.  Partial products go to LDS ([wavefront][tile][256] fp32) and are summed in a
// fixed order at the end of every phase.  With several column splits each writes its partial sums to the
// workspace, takes a ticket, and the last split to finish a row group adds the partial sums in split order and
// writes y.  Four wavefronts share a SIMD (at most 128 VGPRs each).
// ------------------------------------------------------------------------------------------------
struct ResInv {
    ResSel sel;
    uint32_t xs[4];     // x at the 8 salient columns of the record (B operand)
    uint32_t ord;       // index of the record's first entry in a res_sign row
};

// xblk = x of batch row min(i, B - 1) at the first column of block q (any valid address if the lane has no
// x to supply); live = the lane supplies x (i < B and q < nb).  All loads are unconditional so that they
// issue back to back; entries that do not exist read column 0 and are zeroed afterwards.
__device__ inline ResInv load_res_inv(const TiledPlanes& p, int q, int half, int c, const unsigned short* __restrict__ xblk,
                                      bool live) {
    const uint32_t* rec = p.sal_tab + (((int64_t)q * 2 + half) * p.sal_chunks + c) * 12;
    const uint4 a = *reinterpret_cast<const uint4*>(rec);
    const uint4 pv = *reinterpret_cast<const uint4*>(rec + 8);
    ResInv r;
    r.sel.sel0 = a.x; r.sel.sel1 = a.y; r.sel.bit0 = a.z; r.sel.bit1 = a.w;
    r.ord = rec[4];
    const uint32_t pw[4] = {pv.x, pv.y, pv.z, pv.w};
    uint32_t h[8];
#pragma unroll
    for (int e = 0; e < 8; e++) {
        const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
        h[e] = xblk[pos & 127u];
        if (!(live && pos < 128u)) h[e] = 0u;
    }
#pragma unroll
    for (int v = 0; v < 4; v++) r.xs[v] = h[2 * v] | (h[2 * v + 1] << 16);
    return r;
}

template <int N8, bool HAS_RES, bool STAGED>
__global__ __launch_bounds__(1024) void gemv_stream_kernel(TiledPlanes p, const __half* __restrict__ x, int B,
                                                            void* __restrict__ y, int y_fp32, int R, int SPS,
                                                            float* __restrict__ ws_part, uint32_t* __restrict__ ws_count) {
    __shared__ ScatterLds lut;
    __shared__ uint32_t ticket;
    __shared__ __attribute__((aligned(16))) uint32_t recs[STAGED && HAS_RES ? 64 * 12 : 4];   // first salient-column record of each (block, half) of the split
    __shared__ __attribute__((aligned(16))) uint32_t resw[STAGED && HAS_RES ? STB_GEMV_RESW : 4];   // res_sign words of the workgroup's row tiles
    extern __shared__ __attribute__((aligned(16))) float part[];                  // [16][PH][256]; before the first product: the staged x
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 15, g = lane >> 4;
    const int gr = blockIdx.x, ks = blockIdx.y, S = gridDim.y;
    // Column split ks covers the SPS superblocks ks*SPS .. ks*SPS + SPS - 1; 2*SPS wavefronts (one per half
    // block) form a row stream, and the 16 wavefronts of the workgroup hold RS = 16 / (2*SPS) row streams of R
    // tiles each (SPS = 8: one stream, all of a 4096-column slice; SPS = 2: four streams on 1024 columns, which
    // keeps the x traffic of a workgroup small when B is large).
    const int WS = 2 * SPS, RS = 16 / WS;
    const int rs = wave / WS, within = wave - rs * WS;
    const int sb = ks * SPS + (within >> 1), half = within & 1;
    const int r0 = (gr * RS + rs) * R;
    const int r1 = r0 + R < p.nrt ? r0 + R : p.nrt;
    const int rl = r1 - 1;
    const bool active = rs < RS && sb < p.nsb && r0 < p.nrt;      // uniform per wavefront
    constexpr bool RES_GLOBAL = HAS_RES && !STAGED;  // the streaming loop loads res_sign words itself
    constexpr int L = TileLoads<RES_GLOBAL>::count;
    constexpr int PH = STB_GEMV_PHASE;               // half tiles a wavefront streams between two reductions
    const int Wa = 2 * (p.nsb - ks * SPS < SPS ? p.nsb - ks * SPS : SPS);   // wavefronts of a row stream that have work
    const int q = 4 * sb + g;

    LaneOffsets lo = lane_offsets<N8>(lane, half);
    auto tile_of = [&](int rt) { return (int64_t)rt * p.nsb + sb; };
    auto clamp = [&](int rt) { return rt < rl ? rt : rl; };

    // ---- prologue.  A compute unit takes a vector memory instruction only every dozen cycles or so, whatever
    //      its width (measured), so with three tiles per wavefront the number of load instructions decides the
    //      start-up time.  STAGED: the workgroup brings its slice of x and the salient-column records into LDS
    //      with a few full-width loads (B * SPS / 16 per wavefront) and every wavefront takes its B operands, its
    //      record and the x of its salient columns from there; the alternative is 19 narrow loads per
    //      wavefront.  The staged x lies where the partial products go later; it is only used when it fits. ----
    TileRegs<N8> t0, t1, t2;
    uint4_t xr[8];
    ResInv inv;
    int nch = 0, rsh = 0;
    const bool live = active && i < B && q < p.nb;
    const __half* xblk = x + (int64_t)(i < B ? i : B - 1) * p.k + (int64_t)(active && q < p.nb ? q : 0) * 128;
    if constexpr (STAGED) {
        const int per_row = SPS * 64;                               // 16-byte pieces of one batch row of the slice
        const int total = B * per_row;                              // at most 6 * 1024 (checked by the launcher)
        const int xstride = SPS * 1024 + 16;                        // bytes per staged row; the skew spreads rows over banks
        const uint32_t sps_magic = (65536u + (uint32_t)SPS - 1u) / (uint32_t)SPS;    // v / SPS = (v * magic) >> 16 for v < 2^10
        char* xs = reinterpret_cast<char*>(part);
        uint4_t sx0, sx1, sx2, sx3, sx4, sx5;
        uint4_t sr = {0u, 0u, 0u, 0u};
        const int n_u = (total + 1023) >> 10;                       // staging loads per thread: uniform, at most 6
        // piece u of this thread: destination in LDS (-1: none) and whether it lies inside x (columns past k and
        // pieces past the slice load x[0] instead and store zeros, so that a wavefront issues n_u loads on every path)
        auto piece = [&](int u, int& dst, bool& inside) -> const __half* {
            const int pc = (int)threadIdx.x + 1024 * u;
            const int b = (int)(((uint32_t)(pc >> 6) * sps_magic) >> 16), c16 = pc - b * per_row;
            const int col = ks * SPS * 512 + c16 * 8;
            dst = pc < total ? b * xstride + c16 * 16 : -1;
            inside = pc < total && col < p.k;
            return inside ? x + (int64_t)b * p.k + col : x;
        };
        int d0, d1, d2, d3, d4, d5;
        bool in0, in1, in2, in3, in4, in5;
#define STB_STAGE_LOAD(u, reg, d, in) if (u < n_u) { const __half* src = piece(u, d, in); asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(reg) : "v"(src)); }
        STB_STAGE_LOAD(0, sx0, d0, in0) STB_STAGE_LOAD(1, sx1, d1, in1) STB_STAGE_LOAD(2, sx2, d2, in2)
        STB_STAGE_LOAD(3, sx3, d3, in3) STB_STAGE_LOAD(4, sx4, d4, in4) STB_STAGE_LOAD(5, sx5, d5, in5)
#undef STB_STAGE_LOAD
        // records: three 16-byte pieces each, taken by the last three wavefronts
        const int rt3 = (int)threadIdx.x - (1024 - 192);
        const int rI = rt3 >= 0 ? rt3 / 3 : -1, rpc = rt3 - rI * 3;          // record (block of the split, half), piece
        if (HAS_RES && rI >= 0 && ks * SPS + (rI >> 3) < p.nsb && (rI >> 3) < SPS) {
            const uint32_t* src = p.sal_tab + (((int64_t)(4 * ks * SPS) * 2 + rI) * p.sal_chunks) * 12 + 4 * rpc;
            asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(sr) : "v"(src));
        }
        // res_sign words of the workgroup's row tiles [g0, g1): one contiguous piece of the plane, at most two
        // 16-byte loads per thread (the launcher checks that it fits)
        const int g0 = gr * RS * R, g1 = g0 + RS * R < p.nrt ? g0 + RS * R : p.nrt;
        const int rpieces = HAS_RES ? (g1 - g0) * p.res_words * 4 : 0;
        const int n_rw = (rpieces + 1023) >> 10;
        uint4_t rw0 = {0u, 0u, 0u, 0u}, rw1 = {0u, 0u, 0u, 0u};
        {
            const uint4_t* src = reinterpret_cast<const uint4_t*>(p.res_sign + (int64_t)g0 * p.res_words * 16);
            const int t0i = (int)threadIdx.x, t1i = (int)threadIdx.x + 1024;
            if (n_rw > 0) { const uint4_t* a = src + (t0i < rpieces ? t0i : 0); asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rw0) : "v"(a)); }
            if (n_rw > 1) { const uint4_t* a = src + (t1i < rpieces ? t1i : 0); asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rw1) : "v"(a)); }
        }
        if (active) fetch_main<N8>(t0, p, tile_of(clamp(r0)), lo);
        build_luts<N8>(&lut);                            // arithmetic only: overlaps with the loads in flight
        // the staging loads are older than the five of the first tile (which a wavefront without work has not issued)
        if (!active) asm volatile("s_waitcnt vmcnt(0)");
        asm volatile("s_waitcnt vmcnt(5)" : "+v"(sx0), "+v"(sx1), "+v"(sx2), "+v"(sx3), "+v"(sx4), "+v"(sx5), "+v"(sr), "+v"(rw0), "+v"(rw1));
        if (HAS_RES) {
            if (n_rw > 0 && (int)threadIdx.x < rpieces) *reinterpret_cast<uint4_t*>(&resw[4 * threadIdx.x]) = rw0;
            if (n_rw > 1 && (int)threadIdx.x + 1024 < rpieces) *reinterpret_cast<uint4_t*>(&resw[4 * (threadIdx.x + 1024)]) = rw1;
        }
#define STB_STAGE_STORE(u, reg, d, in) if (u < n_u && d >= 0) *reinterpret_cast<uint4_t*>(xs + d) = in ? reg : uint4_t{0u, 0u, 0u, 0u};
        STB_STAGE_STORE(0, sx0, d0, in0) STB_STAGE_STORE(1, sx1, d1, in1) STB_STAGE_STORE(2, sx2, d2, in2)
        STB_STAGE_STORE(3, sx3, d3, in3) STB_STAGE_STORE(4, sx4, d4, in4) STB_STAGE_STORE(5, sx5, d5, in5)
#undef STB_STAGE_STORE
        if (HAS_RES && rI >= 0) *reinterpret_cast<uint4_t*>(&recs[rI * 12 + 4 * rpc]) = sr;
        __syncthreads();
        if (active) {
            const int ql = 4 * (sb - ks * SPS) + g;                   // block inside the split
            const char* xrow = xs + (i < B ? i : 0) * xstride + ql * 256;
#pragma unroll
            for (int t = 0; t < 8; t++) {
                xr[t] = *reinterpret_cast<const uint4_t*>(xrow + 128 * half + 16 * t);
                if (i >= B) xr[t] = uint4_t{0u, 0u, 0u, 0u};
            }
            if (HAS_RES) {
                const uint32_t* rec = &recs[(ql * 2 + half) * 12];
                const uint4_t ra = *reinterpret_cast<const uint4_t*>(rec);
                const uint2_t rb = *reinterpret_cast<const uint2_t*>(rec + 4);
                const uint4_t rp = *reinterpret_cast<const uint4_t*>(rec + 8);
                inv.sel.sel0 = ra.x; inv.sel.sel1 = ra.y; inv.sel.bit0 = ra.z; inv.sel.bit1 = ra.w;
                inv.ord = rb.x;
                nch = __builtin_amdgcn_readfirstlane((int)rb.y);
                rsh = (int)(inv.ord & 31u);
                const int wa = (int)(inv.ord >> 5) < p.res_words ? (int)(inv.ord >> 5) : p.res_words - 1;
                const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
                lo.ores0 = (uint32_t)(wa * 16 + i) * 4u;
                lo.ores1 = (uint32_t)(wb * 16 + i) * 4u;
                const uint32_t pw[4] = {rp.x, rp.y, rp.z, rp.w};
                uint32_t h[8];
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    h[e] = *reinterpret_cast<const unsigned short*>(xrow + 2 * (pos & 127u));
                    if (!(i < B && pos < 128u)) h[e] = 0u;
                }
#pragma unroll
                for (int v = 0; v < 4; v++) inv.xs[v] = h[2 * v] | (h[2 * v + 1] << 16);
            }
            fetch_res<N8, false>(t0, p, clamp(r0), lo);
            fetch_tile<N8, false>(t1, p, tile_of(clamp(r0 + 1)), clamp(r0 + 1), lo);
            fetch_tile<N8, false>(t2, p, tile_of(clamp(r0 + 2)), clamp(r0 + 2), lo);
        }
        __syncthreads();                                 // every wavefront has taken its x: the area may be overwritten
    } else {
        // ---- every load that does not depend on another one goes out first: the packed planes of the first
        //      tile, x for the wavefront's columns, the first record of the salient-column table, the expansion
        //      tables ----
        uint4_t rec_a = {0u, 0u, 0u, 0u}, rec_p = {0u, 0u, 0u, 0u};
        uint2_t rec_b = {0u, 0u};
        uint32_t h[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};      // x at the salient columns of the first record, one fp16 each
        if (active) {
            // Every load of the kernel's streaming part is an asm statement: their order, and with it the count
            // in each wait, is fixed, and the compiler (which does not see them) places no wait of its own that
            // would drain the prefetched tiles.
            if (HAS_RES) {                               // first: other loads depend on this record
                const uint32_t* rec = p.sal_tab + (((int64_t)q * 2 + half) * p.sal_chunks) * 12;
                asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(rec_a) : "v"(rec));
                asm volatile("global_load_dwordx2 %0, %1, off offset:16" : "=v"(rec_b) : "v"(rec));
                asm volatile("global_load_dwordx4 %0, %1, off offset:32" : "=v"(rec_p) : "v"(rec));
            }
            fetch_main<N8>(t0, p, tile_of(clamp(r0)), lo);
            // x: only the lanes that supply a batch row load (lane 0 always does, so the wavefront issues these
            // loads on every path and the wait counts below hold); the others keep zeros.  A load by all 64 lanes
            // would cost a full kilobyte of cache bandwidth per instruction, for B = 1 sixteen times the data.
            const __half* xh = xblk + 64 * half;
#pragma unroll
            for (int t = 0; t < 8; t++) xr[t] = uint4_t{0u, 0u, 0u, 0u};
            if (live) {
#pragma unroll
                for (int t = 0; t < 8; t++)
                    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "+v"(xr[t]) : "v"(xh), "n"(16 * t));
            }
        }
        build_luts<N8>(&lut);                            // arithmetic only: overlaps with the loads in flight

        // ---- the loads that depend on the table record (res_sign words of the first tile, x at the salient
        //      columns), then the second and third tile ----
        uint32_t pw[4] = {0u, 0u, 0u, 0u};
        if (active) {
            if (HAS_RES) {
                // the record has arrived once at most the 5 plane loads and 8 x loads behind it are outstanding
                asm volatile("s_waitcnt vmcnt(13)" : "+v"(rec_a), "+v"(rec_b), "+v"(rec_p));
                inv.sel.sel0 = rec_a.x; inv.sel.sel1 = rec_a.y; inv.sel.bit0 = rec_a.z; inv.sel.bit1 = rec_a.w;
                inv.ord = rec_b.x;
                nch = __builtin_amdgcn_readfirstlane((int)rec_b.y);
                rsh = (int)(inv.ord & 31u);
                const int wa = (int)(inv.ord >> 5) < p.res_words ? (int)(inv.ord >> 5) : p.res_words - 1;
                const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
                lo.ores0 = (uint32_t)(wa * 16 + i) * 4u;
                lo.ores1 = (uint32_t)(wb * 16 + i) * 4u;
                pw[0] = rec_p.x; pw[1] = rec_p.y; pw[2] = rec_p.z; pw[3] = rec_p.w;
                if (live) {
#pragma unroll
                    for (int e = 0; e < 8; e++) {
                        const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                        const __half* src = xblk + (pos & 127u);
                        asm volatile("global_load_ushort %0, %1, off" : "+v"(h[e]) : "v"(src));
                    }
                }
            }
            fetch_res<N8, HAS_RES>(t0, p, clamp(r0), lo);
            fetch_tile<N8, HAS_RES>(t1, p, tile_of(clamp(r0 + 1)), clamp(r0 + 1), lo);
            fetch_tile<N8, HAS_RES>(t2, p, tile_of(clamp(r0 + 2)), clamp(r0 + 2), lo);
        }
        __syncthreads();

        if (active) {
            // The first tile, x and the gathered x have arrived once only the 2 * L loads of the second and third
            // tile are outstanding: the wait counts of the loop hold from its first iteration.
            asm volatile("s_waitcnt vmcnt(%16)"
                         : "+v"(xr[0]), "+v"(xr[1]), "+v"(xr[2]), "+v"(xr[3]), "+v"(xr[4]), "+v"(xr[5]), "+v"(xr[6]), "+v"(xr[7]),
                           "+v"(h[0]), "+v"(h[1]), "+v"(h[2]), "+v"(h[3]), "+v"(h[4]), "+v"(h[5]), "+v"(h[6]), "+v"(h[7])
                         : "n"(2 * L));
            __builtin_amdgcn_sched_barrier(0);
            if (HAS_RES) {
#pragma unroll
                for (int e = 0; e < 8; e++) {
                    const uint32_t pos = (pw[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
                    h[e] = live && pos < 128u ? (h[e] & 0xFFFFu) : 0u;
                }
#pragma unroll
                for (int v = 0; v < 4; v++) inv.xs[v] = h[2 * v] | (h[2 * v + 1] << 16);
            }
        }

    }

    // D[row][b] of a tile: lane l holds b = l % 16, rows 4*(l / 16) + v.  Consecutive threads take consecutive rows.
    const int64_t n16 = (int64_t)p.nrt * 16;
    // v / B for 0 <= v < 2^27 and 2 <= B <= 16, as one multiply: with m = ceil(2^32 / B) the error v * (m*B - 2^32)
    // stays below 2^32 (m does not fit 32 bits for B = 1, which needs no division).
    const uint32_t b_magic = B > 1 ? (uint32_t)((0x100000000ull + (uint32_t)B - 1) / (uint32_t)B) : 0u;
    auto div_b = [&](int v) { return B > 1 ? (int)__umulhi((uint32_t)v, b_magic) : v; };
    // sum over the wavefronts of row stream rsq of the 16 x 16 block of phase slot j, element (b, r16)
    auto wg_sum = [&](int rsq, int j, int b, int r16) {
        const int l = b + 16 * (r16 >> 2), v = r16 & 3;
        const float* src = part + (int64_t)(rsq * WS * PH + j) * 256 + 64 * v + l;
        float t[16];
#pragma unroll
        for (int w = 0; w < 16; w++) t[w] = w < Wa ? src[w * PH * 256] : 0.0f;      // independent reads, fixed order of adds
        float s = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; w++) s += t[w];
        return s;
    };
    auto store_y = [&](int row, int b, float s) {
        if (b < B && row < p.n) {
            if (y_fp32) reinterpret_cast<float*>(y)[(int64_t)b * p.n + row] = -s;
            else reinterpret_cast<__half*>(y)[(int64_t)b * p.n + row] = __float2half(-s);
        }
    };

    const int wg_t0 = gr * RS * R;                   // first row tile of the workgroup (origin of resw)
    auto product = [&](const TileRegs<N8>& tr, int rt, int slot) {
        HalfData<N8> d;
        unpack_tile<N8>(tr, half, d);
        if constexpr (STAGED && HAS_RES) {           // lo.ores0 / ores1 are byte offsets inside the row tile's words
            const char* rbase = reinterpret_cast<const char*>(resw) + (int64_t)(rt - wg_t0) * p.res_words * 64;
            d.rlo = *reinterpret_cast<const uint32_t*>(rbase + lo.ores0);
            d.rhi = *reinterpret_cast<const uint32_t*>(rbase + lo.ores1);
        }
        const uint32_t TL = perm(d.sc.y, d.sc.x, 0x06040200u), TH = perm(d.sc.y, d.sc.x, 0x07050301u);
        float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        constexpr int D = STB_LUT_AHEAD;                             // table reads run D groups ahead
        uint4 gl[D];
#pragma unroll
        for (int t = 0; t < D; t++) gl[t] = lut_fetch<N8>(d, t, &lut, lane & 7);
#pragma unroll
        for (int t = 0; t < 8; t++) {
            const uint4 cur = gl[t % D];
            if (t + D < 8) gl[t % D] = lut_fetch<N8>(d, t + D, &lut, lane & 7);
            __builtin_amdgcn_sched_barrier(0);
            uint32_t o[4];
            expand_group<N8>(d, TL, TH, t, cur, o);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), __builtin_bit_cast(half8_t, xr[t]), acc, 0, 0, 0);
        }
        if (HAS_RES && nch > 0) {
            const uint32_t ar2 = d.ar | (d.ar << 16);
            const uint32_t rb = __builtin_amdgcn_alignbit(d.rhi, d.rlo, (uint32_t)rsh);
            uint32_t o[4];
            residual_chunk(d.m, rb, ar2, inv.sel, o);
            acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(inv.xs), acc, 0, 0, 0);
        }
        float* dst = part + ((int64_t)(wave * PH + slot) * 256 + lane);
#pragma unroll
        for (int v = 0; v < 4; v++) dst[64 * v] = acc[v];
    };

    // The R tiles are taken in phases of PH (a multiple of 3, so that the three tile buffers keep their roles):
    // the wavefronts stream PH half tiles each, the workgroup adds the partial products of the phase in a
    // fixed order and stores them, and the next phase reuses the LDS.  Prefetches run across phase boundaries.
    // (Summing through LDS float atomics instead, without phases, was measured three times slower.)
    // Three tiles are in flight per wavefront (four wavefronts share a SIMD): while tile rt is expanded, the
    // loads of rt + 1 and rt + 2 are outstanding.  A fetch past the last tile of the workgroup re-reads that tile (a
    // cache hit), which keeps the number of loads between a fetch and its wait the same on every path.
    for (int ph = 0; ph < R; ph += PH) {
        const int ph0 = r0 + ph;
        const int ph1 = ph0 + PH < r1 ? ph0 + PH : r1;
        if (active) {
            for (int rt = ph0; rt < ph1; rt += 3) {
                wait_tile<2 * L>(t0);
                product(t0, rt, rt - ph0);
                fetch_tile<N8, RES_GLOBAL>(t0, p, tile_of(clamp(rt + 3)), clamp(rt + 3), lo);
                wait_tile<2 * L>(t1);
                if (rt + 1 < ph1) product(t1, rt + 1, rt + 1 - ph0);
                fetch_tile<N8, RES_GLOBAL>(t1, p, tile_of(clamp(rt + 4)), clamp(rt + 4), lo);
                wait_tile<2 * L>(t2);
                if (rt + 2 < ph1) product(t2, rt + 2, rt + 2 - ph0);
                fetch_tile<N8, RES_GLOBAL>(t2, p, tile_of(clamp(rt + 5)), clamp(rt + 5), lo);
            }
            // Half blocks with more than 8 salient columns: the remaining records, outside the streaming loop
            // so that its load/wait pattern stays fixed.  Rare; every operand is re-read with ordinary loads
            // (the compiler's waits for them may also drain the prefetched tile: harmless).
            if (HAS_RES && nch > 1) {
                const int64_t rstride = (int64_t)p.res_words * 16;
                for (int rt = ph0; rt < ph1; rt++) {
                    HalfData<N8> d;
                    load_half<N8>(p, tile_of(rt), lo, half, d);
                    const uint32_t ar2 = d.ar | (d.ar << 16);
                    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
                    for (int c = 1; c < nch; c++) {
                        const ResInv rv = load_res_inv(p, q, half, c, reinterpret_cast<const unsigned short*>(xblk), live);
                        const int wa = (int)(rv.ord >> 5) < p.res_words ? (int)(rv.ord >> 5) : p.res_words - 1;
                        const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
                        const uint32_t rlo = p.res_sign[rt * rstride + (int64_t)wa * 16 + i];
                        const uint32_t rhi = p.res_sign[rt * rstride + (int64_t)wb * 16 + i];
                        uint32_t o[4];
                        residual_chunk(d.m, __builtin_amdgcn_alignbit(rhi, rlo, rv.ord & 31u), ar2, rv.sel, o);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(rv.xs), acc, 0, 0, 0);
                    }
                    float* dst = part + ((int64_t)(wave * PH + (rt - ph0)) * 256 + lane);
#pragma unroll
                    for (int v = 0; v < 4; v++) dst[64 * v] += acc[v];
                }
            }
        }
        __syncthreads();
        // outputs of this phase: (row stream, slot, b, row in tile), consecutive threads on consecutive rows
        const int total = RS * PH * B * 16;
        for (int o = threadIdx.x; o < total; o += blockDim.x) {
            const int r16 = o & 15, sj = div_b(o >> 4), b = (o >> 4) - sj * B, j = sj % PH, rsq = sj / PH;
            const int base = (gr * RS + rsq) * R;
            const int tile = base + ph + j;
            if (ph + j >= R || tile >= p.nrt) continue;
            const float s = wg_sum(rsq, j, b, r16);
            const int row = tile * 16 + r16;
            if (S == 1) store_y(row, b, s);
            else __hip_atomic_store(ws_part + ((int64_t)ks * 16 + b) * n16 + row, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (ph + PH < R) __syncthreads();            // the next phase overwrites the partial products
    }
    if (active) {
        wait_tile<0>(t0);                            // drain: no load may still target a register that is reused
        wait_tile<0>(t1);
        wait_tile<0>(t2);
    }
    if (S == 1) return;

    // ---- several column splits: the partial sums are in the workspace [split][16][n16]; take a ticket ----
    // The partial sums are written and read with agent-scope accesses (they go through to the level all
    // compute dies share), so no cache write-back or invalidate is needed around the ticket: the stores have
    // completed (vmcnt = 0, then the barrier) before thread 0 takes the ticket, and the last arrival issues
    // its loads after it has seen the ticket.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicInc(ws_count + gr, (uint32_t)(S - 1));    // wraps to 0 after S arrivals
    __syncthreads();
    if (ticket != (uint32_t)(S - 1)) return;
    const int g0 = gr * RS * R, g1 = g0 + RS * R < p.nrt ? g0 + RS * R : p.nrt;     // row tiles of this group
    const int total = (g1 - g0) * 16 * B;
    for (int o = threadIdx.x; o < total; o += blockDim.x) {
        const int r16 = o & 15, tb = div_b(o >> 4), b = (o >> 4) - tb * B, tile = g0 + tb;
        const int row = tile * 16 + r16;
        float t[4];
        float s = 0.0f;
        for (int c0 = 0; c0 < S; c0 += 4) {
#pragma unroll
            for (int u = 0; u < 4; u++)
                t[u] = c0 + u < S ? __hip_atomic_load(ws_part + ((int64_t)(c0 + u) * 16 + b) * n16 + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
#pragma unroll
            for (int u = 0; u < 4; u++) s += t[u];
        }
        store_y(row, b, s);
    }
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// launchers (internal ABI, see stb_internal.h)
// ------------------------------------------------------------------------------------------------
static int kept_per_8(const stb_layout_t* L) { return stb_tiled_slots(&L->cfg); }    // slots the planes hold per 8 columns

extern "C" int stb_tiled_supported(const stb_layout_t* L) { return stb_tiled_slots(&L->cfg) != 0; }

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

// Largest number of column splits the launcher below may choose for n_super superblocks.
static int max_splits(int n_super) { return (n_super + 1) / 2 + 3; }

extern "C" int64_t stb_tiled_gemv_workspace(int n_row_tiles, int n_super) {
    return round_up256(4 * (int64_t)n_row_tiles) + (int64_t)max_splits(n_super) * 16 * 16 * n_row_tiles * 4;
}

template <int N8, bool HAS_RES, bool STAGED>
static hipError_t launch_gemv_stream3(const TiledPlanes& p, const __half* x, int B, void* y, int y_fp32, int R, int SPS,
                                      dim3 grid, size_t lds, float* ws_part, uint32_t* ws_count, hipStream_t st) {
    static std::atomic<bool> attr_set{false};         // a failure is not remembered: the next call tries again
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t attr = hipFuncSetAttribute((const void*)gemv_stream_kernel<N8, HAS_RES, STAGED>, hipFuncAttributeMaxDynamicSharedMemorySize, 16 * STB_GEMV_PHASE * 1024);
        if (attr != hipSuccess) return attr;
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL((gemv_stream_kernel<N8, HAS_RES, STAGED>), grid, dim3(1024), lds, st, p, x, B, y, y_fp32, R, SPS, ws_part, ws_count);
    return hipGetLastError();
}

template <int N8, bool HAS_RES>
static hipError_t launch_gemv_stream(const TiledPlanes& p, const __half* x, int B, void* y, int y_fp32, int R, int SPS,
                                     dim3 grid, size_t lds, float* ws_part, uint32_t* ws_count, hipStream_t st) {
    // x is staged through LDS when the B rows of the split (SPS * 1024 + 16 bytes each) fit into the area of the
    // partial products
    // ... and the res_sign words of the workgroup's RS * R row tiles into their own area
    const int RS = 16 / (2 * SPS);
    const bool staged = (int64_t)B * (SPS * 1024 + 16) <= (int64_t)lds &&
                        (!HAS_RES || (int64_t)RS * R * p.res_words * 16 <= STB_GEMV_RESW);
    return staged ? launch_gemv_stream3<N8, HAS_RES, true>(p, x, B, y, y_fp32, R, SPS, grid, lds, ws_part, ws_count, st)
                  : launch_gemv_stream3<N8, HAS_RES, false>(p, x, B, y, y_fp32, R, SPS, grid, lds, ws_part, ws_count, st);
}

extern "C" int stb_tiled_gemv(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* workspace,
                              int64_t workspace_bytes, int64_t part_off, void* stream, int* hip_err) {
    if (!stb_tiled_supported(L)) return STB_EUNSUPPORTED;
    // stb_set_kernel_override can send every launch to the kernel below: the tests use it, because on ordinary
    // shapes the fat-wavefront kernel takes everything.
    const bool thin_only = stb_kernel_override(0) == 1;
    if (!thin_only && B <= 16) {                                    // the kernel with fat wavefronts, if its LDS areas fit
        const int rc = stb_tiled_gemv24(L, x, B, y, y_fp32, workspace, workspace_bytes, part_off, max_splits(L->n_super), stream, hip_err);
        if (rc != STB_EUNSUPPORTED) return rc;
    }
    const TiledPlanes p = make_tiled(L);
    constexpr int wg_target = 256;                                  // workgroups the launch aims for: one per compute unit
    // Superblocks per column split: at most 8 (a whole 4096-column slice per workgroup).  Narrower splits with
    // several row streams per workgroup come out of the search below when they balance the grid better.
    constexpr int sps0 = 8;
    // Among the split counts that fit, take the one with the fewest half tiles per compute unit (R tiles for each
    // wavefront with work, times the rounds the grid needs on 256 units); ties go to the fewest splits.
    int best_S = 0, best_R = 0, best_sps = 0;
    int64_t best_cost = 0;
    const int s_min = (p.nsb + sps0 - 1) / sps0;
    for (int S = s_min; S <= s_min + 3 && S <= max_splits(p.nsb) && S <= p.nsb; S++) {
        const int sps = (p.nsb + S - 1) / S;
        const int rs = 16 / (2 * sps);
        if (rs < 1 || (S - 1) * sps >= p.nsb) continue;            // a split must own at least one superblock
        const int groups = wg_target / S > 0 ? wg_target / S : 1;
        const int R = (p.nrt + rs * groups - 1) / (rs * groups);
        const int G = (p.nrt + rs * R - 1) / (rs * R);
        const int64_t cost = (int64_t)R * 2 * sps * rs * ((G * S + wg_target - 1) / wg_target);
        if (best_S == 0 || cost < best_cost) { best_cost = cost; best_S = S; best_R = R; best_sps = sps; }
    }
    if (best_S == 0) return STB_EINVAL;
    const int S = best_S, R = best_R, SPS = best_sps, RS = 16 / (2 * SPS);
    const int G = (p.nrt + RS * R - 1) / (RS * R);
    if (S > 1) {
        if (!workspace) return STB_ENULL;
        if (part_off < 0) part_off = round_up256(4 * (int64_t)p.nrt);
        if (part_off % 256 || part_off < 4 * (int64_t)p.nrt) return STB_EINVAL;
        if (workspace_bytes < part_off + (int64_t)S * 16 * 16 * p.nrt * 4) return STB_EINVAL;
        if ((uintptr_t)workspace % 256) return STB_EALIGN;
    }
    const size_t lds = (size_t)16 * STB_GEMV_PHASE * 256 * sizeof(float);   // + 32 KB of tables: 128 KB of LDS
    const dim3 grid(G, S);
    const hipStream_t st = (hipStream_t)stream;
    const __half* xh = (const __half*)x;
    uint32_t* cnt = (uint32_t*)workspace;
    float* part = S > 1 ? (float*)((char*)workspace + part_off) : nullptr;
    const bool res = p.res_words > 0;
    hipError_t e;
    if (kept_per_8(L) == 4)
        e = res ? launch_gemv_stream<4, true>(p, xh, B, y, y_fp32, R, SPS, grid, lds, part, cnt, st)
                : launch_gemv_stream<4, false>(p, xh, B, y, y_fp32, R, SPS, grid, lds, part, cnt, st);
    else
        e = res ? launch_gemv_stream<6, true>(p, xh, B, y, y_fp32, R, SPS, grid, lds, part, cnt, st)
                : launch_gemv_stream<6, false>(p, xh, B, y, y_fp32, R, SPS, grid, lds, part, cnt, st);
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}
