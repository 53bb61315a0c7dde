// Prefill GEMM with the expanded weights shared through LDS (included by stb_gemm.hip, inside its namespace).
//
// The other prefill kernels let every wavefront expand its own A operands: about 19 vector instructions per operand,
// used by 4 (32x32 form) or 8 (16x16 form) matrix instructions, and matrix and vector instructions share the SIMD's
// issue port -- that, not the matrix pipes, is what bounds them.  Here a workgroup owns 128 output rows x 256 tokens;
// each of its four wavefronts expands a quarter of the weight tile of the next K window, writes the fp16 operands to
// LDS, and all four read them back: an operand costs 20 vector instructions once per workgroup and one LDS read per
// use.  A wavefront computes 64 rows x 128 tokens (2 x 4 accumulator tiles of v_mfma_f32_32x32x16_f16) and needs 6
// operand reads for 8 matrix instructions.
//
// K runs in windows of one half block (64 columns of one 128-column block: K = 64, four steps of the matrix
// instruction), so that a token's share of a window is one whole 128-byte line of X.  A pass = the 4 windows of a
// (superblock, half block) plus, with salient columns, a residual window (Eq. 4: K = 32 = 8 salient columns per block,
// A from residual_chunk, B from the gathered columns that gemm_gather_kernel wrote to the workspace).
// Lane 16 g + i of wavefront w works on row i of row tile 2 w + g % 2 of the workgroup and on quarter g / 2 (32
// columns) of the window's half block: it loads the (row, block) records of all four blocks itself (the tiled order
// keeps a record's bytes per (row, block), so any lane can take any record) and uses one quarter of each.
// LDS:  three X window buffers (256 token rows x 128 bytes; the 16-byte piece t = 8-column group t of row r sits at
//       position t ^ ((r / 2) % 8): the 16 lanes that read one piece of 16 consecutive rows hit every bank once, and so
//       do the global -> LDS loads), two W window buffers (piece t of row r at (t * 128 + r) * 16), the scatter table
//       (4 copies).
// Pipeline, one barrier per window: during window j a wavefront issues the matrix instructions of window j, expands
// window j + 1 into the other W buffer and has the global -> LDS loads of windows j + 1 and j + 2 in flight.
// Every global load is an asm statement and every wait is written by hand (see GemmStage in stb_gemm.hip for why).

constexpr int GS_ROWT = 8;            // 16-row tiles per workgroup
constexpr int GS_TOK = 256;           // tokens per workgroup
struct GsLds {
    static constexpr int XB = 0, XBSZ = GS_TOK * 128;                 // X window buffers (three)
    static constexpr int WB = 3 * XBSZ, WBSZ = 128 * 8 * 16;          // W window buffers (two)
    static constexpr int LUT = WB + 2 * WBSZ;                         // scatter table, four copies
    static constexpr int TOTAL = LUT + 256 * 4 * 16;
    static constexpr int EPI = GS_TOK / 2 * 144;                      // epilogue: per wavefront 128 token rows of 144 bytes
};
static_assert(4 * GsLds::EPI <= GsLds::WB, "the epilogue's transpose areas lie on the X buffers");

template <int N8, bool HAS_RES>
__global__ __launch_bounds__(256) void gemm_shared_kernel(TiledPlanes p, const __half* __restrict__ X, int T,
                                                           void* __restrict__ Y, int y_fp32,
                                                           const __half* __restrict__ xsal, int cfix) {
    typedef GsLds G;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    uint4 (*const lut)[4] = reinterpret_cast<uint4 (*)[4]>(lds + G::LUT);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int i = lane & 15, g = lane >> 4, l31 = lane & 31, lh = lane >> 5;
    const int t0 = blockIdx.x * GS_TOK;
    const int rt0 = blockIdx.y * GS_ROWT;
    const int mh = wave & 1, th = wave >> 1;                         // the wavefront's 64 rows and 128 tokens of the tile
    const int nsh = p.nsb * 2;
    for (int mb = tid; mb < 256; mb += 256) {
        const uint4 v = scatter_entry<N8>((uint32_t)mb);
#pragma unroll
        for (int c = 0; c < 4; c++) lut[mb][c] = v;
    }

    float16_t acc[2][4];
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int tb = 0; tb < 4; tb++)
#pragma unroll
            for (int v = 0; v < 16; v++) acc[mb][tb][v] = 0.0f;

    // ---- addresses ----
    const uint32_t tok_last = (uint32_t)(T - 1 - t0), k2 = (uint32_t)p.k * 2u;
    const __half* const Xt = X + (int64_t)t0 * p.k;
    // X window -> LDS: load u (0..7) of wavefront w covers token rows 64 w + 8 u .. + 7; lane l = row l / 8 of them,
    // position l % 8, which holds piece (l % 8) ^ ((row / 2) % 8), (row / 2) % 8 = 4 (u % 2) + l / 16.  A row's eight
    // pieces are one 128-byte line of X.  Tokens past T are clamped to the last token (their outputs are never stored);
    // a piece past column k is clamped to the row's last 16 bytes (it meets zero weights).
    uint32_t pcol[2];
#pragma unroll
    for (int par = 0; par < 2; par++) pcol[par] = ((((uint32_t)lane & 7u) ^ (uint32_t)(4 * par + (lane >> 4))) & 7u) * 16u;
    uint32_t xrow[8];
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const uint32_t row = (uint32_t)(64 * wave + 8 * u + (lane >> 3));
        xrow[u] = __umul24(row < tok_last ? row : tok_last, k2);
    }
    // gathered salient columns -> LDS (rows of 64 bytes: piece b = block b at position b ^ ((r / 4) % 4)): load u
    // (0..3) of wavefront w covers rows 64 w + 16 u .. + 15; lane l = row l / 4 of them, position l % 4
    const int64_t E = (int64_t)p.nsb * 2 * cfix * 32;               // halves per token in xsal
    const __half* const xsal_t = xsal + (int64_t)t0 * E;
    uint32_t grow[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
        const uint32_t row = (uint32_t)(64 * wave + 16 * u + (lane >> 2));
        grow[u] = (row < tok_last ? row : tok_last) * (uint32_t)E * 2u + (((uint32_t)lane & 3u) ^ (((uint32_t)lane >> 4) & 3u)) * 16u;
    }
    // the wavefront's eight loads of a window go out two at a time (part 0..3): the four wavefronts share one path
    // to memory, and a burst of loads stalls them all
    auto load_x_part = [&](int sh, int blk, uint32_t xoff, int part) {
        const uint32_t wcol = (uint32_t)((sh >> 1) * 1024 + blk * 256 + (sh & 1) * 128);
        const uint32_t dst = lds0 + G::XB + xoff + wave * 8192;
#pragma unroll
        for (int u = 2 * part; u < 2 * part + 2; u++) {
            const uint32_t c = wcol + pcol[u & 1] < k2 - 16u ? wcol + pcol[u & 1] : k2 - 16u;
            load_to_lds(dst + u * 1024, xrow[u] + c, Xt);
        }
    };
    auto load_x = [&](int sh, int blk, uint32_t xoff) {
#pragma unroll
        for (int part = 0; part < 4; part++) load_x_part(sh, blk, xoff, part);
    };
    auto load_g_part = [&](int sh, int c, uint32_t xoff, int u) {
        load_to_lds(lds0 + G::XB + xoff + wave * 4096 + u * 1024, grow[u] + (uint32_t)(sh * cfix + c) * 64u, xsal_t);
    };
    auto load_g = [&](int sh, int c, uint32_t xoff) {
#pragma unroll
        for (int u = 0; u < 4; u++) load_g_part(sh, c, xoff, u);
    };
    // operand reads: A piece (2 s + lane / 32) of rows 64 mh + 32 mb + lane % 32; B piece (2 s + lane / 32) of token rows
    // 128 th + 32 tb + lane % 32
    const uint32_t ax = (uint32_t)(G::WB + (lh * 128 + 64 * mh + l31) * 16);
    uint32_t bx[4], gx[2];
#pragma unroll
    for (int s = 0; s < 4; s++) bx[s] = (uint32_t)(G::XB + (128 * th + l31) * 128 + (((2 * s + lh) ^ ((l31 >> 1) & 7))) * 16);
#pragma unroll
    for (int s = 0; s < 2; s++) gx[s] = (uint32_t)(G::XB + (128 * th + l31) * 64 + (((2 * s + lh) ^ ((l31 >> 2) & 3))) * 16);
    // operand writes: the lane's row (row tile 2 wave + g % 2, row i); normal pieces 4 (g / 2) + tq, residual pieces
    // (blocks) 2 (g / 2) + j
    const int q = g >> 1;
    const uint32_t wrow = (uint32_t)(G::WB + (16 * (2 * wave + (g & 1)) + i) * 16);
    const uint32_t wx = wrow + (uint32_t)q * 8192u, wr = wrow + (uint32_t)q * 4096u;

    // ---- records: the lane's row in each of the four blocks of the superblock ----
    auto row_tile = [&](int r) { const int rt = rt0 + 2 * wave + r; return rt < p.nrt ? rt : p.nrt - 1; };
    const uint32_t dtile = (g & 1) ? (uint32_t)((row_tile(1) - row_tile(0)) * p.nsb) : 0u;        // from the uniform tile to the lane's own
    auto fetch_record = [&](int sh, TileRegs<N8> (&tn)[4], int b) {
        const int64_t tile = (int64_t)__builtin_amdgcn_readfirstlane(row_tile(0) * p.nsb + (sh >> 1));
        LaneOffsets lo = lane_offsets<N8>(16 * b + i, sh & 1);
        lo.omask += dtile * (64u * 16u);
        lo.osign += dtile * (64u * 2u * N8);
        lo.oregion += dtile * (64u * 4u * N8);
        lo.o8 += dtile * (64u * 8u);
        lo.o2 += dtile * (64u * 2u);
        fetch_main<N8>(tn[b], p, tile, lo);
    };
    auto fetch_table = [&](int sh, uint4_t (&ran)[2], uint2_t (&rbn)[2]) {
        if (HAS_RES) {
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const uint32_t off = (uint32_t)(((4 * (sh >> 1) + 2 * q + j) * 2 + (sh & 1)) * p.sal_chunks) * 48u;
                asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(ran[j]) : "v"(off), "s"(p.sal_tab));
                asm volatile("global_load_dwordx2 %0, %1, %2 offset:16" : "=v"(rbn[j]) : "v"(off), "s"(p.sal_tab));
            }
        }
    };
    auto fetch_records = [&](int sh, TileRegs<N8> (&tn)[4], uint4_t (&ran)[2], uint2_t (&rbn)[2]) {
#pragma unroll
        for (int b = 0; b < 4; b++) fetch_record(sh, tn, b);
        fetch_table(sh, ran, rbn);
    };
    const uint32_t* const rsbase = p.res_sign + (int64_t)__builtin_amdgcn_readfirstlane(row_tile(0)) * p.res_words * 16;
    const uint32_t dres = (g & 1) ? (uint32_t)((row_tile(1) - row_tile(0)) * p.res_words) * 64u : 0u;
    // the two res_sign words of the lane's row that hold the bits of the record with first entry `ord`, for blocks 2 q + j
    auto fetch_res_words = [&](const uint2_t (&rbn)[2], uint32_t (&rlo)[2], uint32_t (&rhi)[2]) {
#pragma unroll
        for (int j = 0; j < 2; j++) {
            const uint32_t ord = rbn[j][0];
            const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
            const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
            const uint32_t oa = (uint32_t)(wa * 16 + i) * 4u + dres, ob = (uint32_t)(wb * 16 + i) * 4u + dres;
            asm volatile("global_load_dword %0, %1, %2" : "=v"(rlo[j]) : "v"(oa), "s"(rsbase));
            asm volatile("global_load_dword %0, %1, %2" : "=v"(rhi[j]) : "v"(ob), "s"(rsbase));
        }
    };
    // A record as the lane uses it: the scale tables, and its quarter (32 columns: column groups 0..3 of `v`) of the
    // mask, sign and id bits; `full` keeps the half block's whole mask and alpha_r for the residual operand.
    struct Quarter {
        HalfData<N8> v;
        uint32_t TL, TH, m0, m1;
    };
    auto make_quarter = [&](const HalfData<N8>& d, Quarter& o) {
        o.TL = perm(d.sc.y, d.sc.x, 0x06040200u);
        o.TH = perm(d.sc.y, d.sc.x, 0x07050301u);
        o.m0 = d.m[0]; o.m1 = d.m[1];
        o.v = d;
        o.v.m[0] = q ? d.m[1] : d.m[0];
        if (N8 == 4) {
            o.v.r[0] = q ? d.r[1] : d.r[0];
            o.v.s[0] = q ? d.s[0] >> 16 : d.s[0];
        } else {
            // ids: bits 48 q .. 48 q + 47 of the half record's 96; signs: bits 24 q .. 24 q + 23 of its 48
            o.v.r[0] = q ? __builtin_amdgcn_alignbit(d.r[2], d.r[1], 16) : d.r[0];
            o.v.r[1] = q ? d.r[2] >> 16 : d.r[1];
            o.v.r[2] = 0u;
            o.v.s[0] = q ? __builtin_amdgcn_alignbit(d.s[1], d.s[0], 24) : d.s[0];
            o.v.s[1] = 0u;
        }
    };

    // ---- the two halves of a window's work ----
    // operands of column group tq (8 columns) of the lane's quarter of a record -> W buffer, piece 4 q + tq; L = the
    // group's scatter selectors (read ahead of the arithmetic that uses them)
    auto lut_read = [&](const Quarter& d, int tq) { return lut[(d.v.m[0] >> (8 * tq)) & 0xFFu][lane & 3]; };
    auto expand_piece = [&](const Quarter& d, int tq, const uint4& L, uint32_t dst) {
        uint32_t o[4];
        expand_group<N8>(d.v, d.TL, d.TH, tq, L, o);
        *reinterpret_cast<uint4*>(lds + dst + tq * 2048) = make_uint4(o[0], o[1], o[2], o[3]);
    };
    // residual operand (8 salient columns) of the lane's row in one block -> W buffer
    auto residual_piece = [&](const Quarter& d, const uint4& ra, uint32_t ord, uint32_t rlo, uint32_t rhi, uint32_t dst) {
        ResSel sel;
        sel.sel0 = ra.x; sel.sel1 = ra.y; sel.bit0 = ra.z; sel.bit1 = ra.w;
        const uint32_t m[2] = {d.m0, d.m1};
        uint32_t o[4];
        residual_chunk(m, __builtin_amdgcn_alignbit(rhi, rlo, ord & 31u), d.v.ar | (d.v.ar << 16), sel, o);
        *reinterpret_cast<uint4*>(lds + dst) = make_uint4(o[0], o[1], o[2], o[3]);
    };
    // operands of step s of a window: A pieces of the two 32-row tiles, B pieces of the four 32-token tiles
    struct Ops { uint4 a[2], b[4]; };
    auto read_ops = [&](uint32_t a_addr, uint32_t b_addr, int b_stride, Ops& o) {
#pragma unroll
        for (int mb = 0; mb < 2; mb++) o.a[mb] = *reinterpret_cast<const uint4*>(lds + a_addr + mb * 512);
#pragma unroll
        for (int tb = 0; tb < 4; tb++) o.b[tb] = *reinterpret_cast<const uint4*>(lds + b_addr + tb * b_stride);
    };
    auto mfma8 = [&](const Ops& o) {
#pragma unroll
        for (int tb = 0; tb < 4; tb++)
#pragma unroll
            for (int mb = 0; mb < 2; mb++)
                acc[mb][tb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, o.a[mb]), __builtin_bit_cast(half8_t, o.b[tb]),
                                                                     acc[mb][tb], 0, 0, 0);
    };
    // A window of NS steps as a software pipeline: the operands of step s + 1 are read from LDS before the matrix
    // instructions of step s are issued, and the rest of the window's work rides in their shadow: `loads(s)` issues
    // the global loads that go with step s (the first ones right after the barrier, where they cover the latency of
    // the first operand reads), `work(s)` builds operands for the next window.  The scheduling fences keep the
    // compiler from sinking the reads down to their uses.
    auto window = [&](auto ns_, uint32_t a_addr, auto&& b_addr, int b_stride, auto&& loads, auto&& work) {
        constexpr int NS = decltype(ns_)::value;
        Ops o[2];
        read_ops(a_addr, b_addr(0), b_stride, o[0]);
        __builtin_amdgcn_sched_barrier(0);
        loads(0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < NS; st++) {
            if (st + 1 < NS) read_ops(a_addr + (st + 1) * 4096, b_addr(st + 1), b_stride, o[(st + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            mfma8(o[st & 1]);
            work(st);
            __builtin_amdgcn_sched_barrier(0);
            if (st + 1 < NS) loads(st + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // end of a window: the X loads of the next window have landed (at most K younger loads are still on their way),
    // this wavefront's operand writes are done, and so is everybody else
    auto end_window = [&](auto k_) {
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(decltype(k_)::value) : "memory");
        __syncthreads();
    };
    // the records of a pass, once they have arrived
    auto unpack_records = [&](TileRegs<N8> (&tn)[4], int half, Quarter (&hq)[4]) {
#pragma unroll
        for (int b = 0; b < 4; b++) {
            HalfData<N8> d;
            tn[b].rlo = 0u; tn[b].rhi = 0u;
            unpack_tile<N8>(tn[b], half, d);
            make_quarter(d, hq[b]);
        }
    };

    // ---- prologue: the first two windows, the records of the first pass, the operands of window 0 ----
    Quarter hd[4];
    uint4 ra[2] = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u)};
    uint2 rb[2] = {make_uint2(0u, 0u), make_uint2(0u, 0u)};
    uint32_t rlo[2] = {0u, 0u}, rhi[2] = {0u, 0u};
    load_x(0, 0, 0);
    load_x(0, 1, G::XBSZ);
    {
        TileRegs<N8> t0r[4];
        uint4_t ra0[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
        uint2_t rb0[2] = {{0u, 0u}, {0u, 0u}};
        fetch_records(0, t0r, ra0, rb0);
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(ra0[0]), "+v"(rb0[0]), "+v"(ra0[1]), "+v"(rb0[1]) : : "memory");
#pragma unroll
        for (int b = 0; b < 4; b++)
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t0r[b].m), "+v"(t0r[b].s), "+v"(t0r[b].r), "+v"(t0r[b].sc), "+v"(t0r[b].ar));
        unpack_records(t0r, 0, hd);
        if (HAS_RES) {
            uint32_t l0[2], h0[2];
            fetch_res_words(rb0, l0, h0);
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(l0[0]), "+v"(l0[1]), "+v"(h0[0]), "+v"(h0[1]) : : "memory");
#pragma unroll
            for (int j = 0; j < 2; j++) { rlo[j] = l0[j]; rhi[j] = h0[j]; }
        }
#pragma unroll
        for (int j = 0; j < 2; j++) {
            ra[j] = make_uint4(ra0[j].x, ra0[j].y, ra0[j].z, ra0[j].w);
            rb[j] = make_uint2(rb0[j].x, rb0[j].y);
        }
    }
    __syncthreads();                                                // the scatter table is complete
#pragma unroll
    for (int tq = 0; tq < 4; tq++) expand_piece(hd[0], tq, lut_read(hd[0], tq), wx);
    __syncthreads();

    // Window counter modulo 3 and 2: X buffer that is read (xr), X buffer that is loaded for the window after the next
    // (xl = the one read last), W buffer that is read (wb; the other one is written).
    uint32_t xr = 0u, xl = 2u * G::XBSZ, wb = 0u;
    auto rotate = [&]() {
        const uint32_t nx = xr + G::XBSZ;
        xl = xr;
        xr = nx == 3u * G::XBSZ ? 0u : nx;
        wb ^= (uint32_t)G::WBSZ;
    };
    // A normal window: matrix instructions of the window in (xr, wb); the operands of record d (the next window's
    // block) go to the other W buffer; `loads(s)` as in window().
    auto normal_window = [&](const Quarter& d, auto&& loads) {
        const uint32_t ww = wx + (wb ^ (uint32_t)G::WBSZ);
        uint4 L[4];
#pragma unroll
        for (int tq = 0; tq < 4; tq++) L[tq] = lut_read(d, tq);
        window(IntC<4>{}, ax + wb, [&](int st) { return bx[st] + xr; }, 4096, loads,
               [&](int st) { expand_piece(d, st, L[st], ww); });
    };

    // Global loads of a pass, in issue order (X loads of a window: 8, gathered columns: 4, records: NH + NC, res_sign
    // words: NRW); end_window<K>: K = the loads issued after the last X load of the window that comes next.
    //   window 0: at step s the record of block s of the next pass (after step 3 also its table records), then two
    //             of the X loads of window 2                                K = 8 + NH + NC (all of them)
    //   window 1: X of window 3                                             K = 8
    //   window 2: gathered columns (X of the next pass's window 0 without salient columns)      K = 4 (8)
    //   window 3: X of the next pass's window 0, then its res_sign words (X of its window 1)    K = 8 + NRW (8)
    //   window 4: X of the next pass's window 1        K = 8 (the res_sign words are waited for as well)
    constexpr int NH = 4 * TileLoads<false>::count, NC = HAS_RES ? 4 : 0, NRW = HAS_RES ? 4 : 0;
    for (int sh = 0; sh < nsh; sh++) {
        const int shn = sh + 1 < nsh ? sh + 1 : sh;                 // the last pass prefetches its own data again
        TileRegs<N8> tn[4];
        uint4_t ran[2] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};
        uint2_t rbn[2] = {{0u, 0u}, {0u, 0u}};
        Quarter hn[4];
        // window 0 (block 0): expands block 1
        normal_window(hd[1], [&](int st) {
            fetch_record(shn, tn, st);
            if (st == 3) fetch_table(shn, ran, rbn);
            load_x_part(sh, 2, xl, st);                             // (last: the window's X loads end with the window's youngest load)
        });
        end_window(IntC<8 + NH + NC>{});
        rotate();
        // window 1: expands block 2
        normal_window(hd[2], [&](int st) { load_x_part(sh, 3, xl, st); });
        end_window(IntC<8>{});
        rotate();
        if (HAS_RES) {
            // window 2: expands block 3
            normal_window(hd[3], [&](int st) { load_g_part(sh, 0, xl, st); });
            end_window(IntC<4>{});
            rotate();
            // the next pass's records have arrived (only the four loads above are younger)
            asm volatile("s_waitcnt vmcnt(4)" : "+v"(ran[0]), "+v"(rbn[0]), "+v"(ran[1]), "+v"(rbn[1]) : : "memory");
#pragma unroll
            for (int b = 0; b < 4; b++)
                asm volatile("s_waitcnt vmcnt(4)" : "+v"(tn[b].m), "+v"(tn[b].s), "+v"(tn[b].r), "+v"(tn[b].sc), "+v"(tn[b].ar));
            unpack_records(tn, shn & 1, hn);
            // window 3: expands the residual window (the lane's row in blocks 2 q and 2 q + 1)
            uint32_t rlon[2], rhin[2];
            {
                const uint32_t ww = wr + (wb ^ (uint32_t)G::WBSZ);
                window(IntC<4>{}, ax + wb, [&](int st) { return bx[st] + xr; }, 4096,
                       [&](int st) { load_x_part(shn, 0, xl, st); if (st == 3) fetch_res_words(rbn, rlon, rhin); },
                       [&](int st) { if (st < 2) residual_piece(q ? hd[2 + st] : hd[st], ra[st], rb[st].x, rlo[st], rhi[st], ww + st * 2048); });
            }
            end_window(IntC<8 + NRW>{});
            rotate();
            // window 4, the residual one (two steps: blocks 0, 1 and 2, 3): expands block 0 of the next pass
            {
                const uint32_t ww = wx + (wb ^ (uint32_t)G::WBSZ);
                uint4 L[4];
#pragma unroll
                for (int tq = 0; tq < 4; tq++) L[tq] = lut_read(hn[0], tq);
                window(IntC<2>{}, ax + wb, [&](int st) { return gx[st] + xr; }, 2048,
                       [&](int st) { load_x_part(shn, 1, xl, 2 * st); load_x_part(shn, 1, xl, 2 * st + 1); },
                       [&](int st) { expand_piece(hn[0], 2 * st, L[2 * st], ww); expand_piece(hn[0], 2 * st + 1, L[2 * st + 1], ww); });
            }
            // (also: the res_sign words of the next pass have arrived; they are carried into the next iteration)
            asm volatile("s_waitcnt vmcnt(8)" : "+v"(rlon[0]), "+v"(rlon[1]), "+v"(rhin[0]), "+v"(rhin[1]) : : "memory");
            __syncthreads();
            rotate();
#pragma unroll
            for (int j = 0; j < 2; j++) { rlo[j] = rlon[j]; rhi[j] = rhin[j]; }
        } else {
            // window 2: expands block 3
            normal_window(hd[3], [&](int st) { load_x_part(shn, 0, xl, st); });
            end_window(IntC<8>{});
            rotate();
#pragma unroll
            for (int b = 0; b < 4; b++)
                asm volatile("s_waitcnt vmcnt(8)" : "+v"(tn[b].m), "+v"(tn[b].s), "+v"(tn[b].r), "+v"(tn[b].sc), "+v"(tn[b].ar));
            unpack_records(tn, shn & 1, hn);
            // window 3: expands block 0 of the next pass
            normal_window(hn[0], [&](int st) { load_x_part(shn, 1, xl, st); });
            end_window(IntC<8>{});
            rotate();
        }
#pragma unroll
        for (int b = 0; b < 4; b++) hd[b] = hn[b];
#pragma unroll
        for (int j = 0; j < 2; j++) {
            ra[j] = make_uint4(ran[j].x, ran[j].y, ran[j].z, ran[j].w);
            rb[j] = make_uint2(rbn[j].x, rbn[j].y);
        }
    }
    // nothing may still be on its way to this workgroup's LDS from here on
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");

    // ---- half blocks with more than 8 salient columns: their further records, one at a time and without overlap
    //      (few: a record covers 8 of the 64 columns) ----
    if (HAS_RES && p.sal_chunks > 1) {
        const int64_t mytile0 = (int64_t)(row_tile(0) * p.nsb) + dtile;
        for (int sh0 = 0; sh0 < nsh; sh0 += 64) {
            const int shl = sh0 + lane < nsh ? sh0 + lane : nsh - 1;
            const uint32_t need_l = p.sal_tab[(((int64_t)(4 * (shl >> 1)) * 2 + (shl & 1)) * p.sal_chunks) * 12 + 5];
            uint64_t todo = __ballot(need_l > 1u && sh0 + lane < nsh);
            while (todo) {
                const int sh = sh0 + __builtin_ctzll(todo);
                todo &= todo - 1;
                const uint32_t* rec0[2];
                Quarter hx[2];
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    rec0[j] = p.sal_tab + (((int64_t)(4 * (sh >> 1) + 2 * q + j) * 2 + (sh & 1)) * p.sal_chunks) * 12;
                    HalfData<N8> d;
                    load_half<N8>(p, mytile0 + (sh >> 1), lane_offsets<N8>(16 * (2 * q + j) + i, sh & 1), sh & 1, d);
                    make_quarter(d, hx[j]);
                }
                const int nch = __builtin_amdgcn_readfirstlane((int)rec0[0][5]);       // the same for the four blocks
                for (int c = 1; c < nch; c++) {
                    __syncthreads();                             // every wavefront is done with the buffers
                    load_g(sh, c, 0);
#pragma unroll
                    for (int j = 0; j < 2; j++) {
                        const uint4 rc = *reinterpret_cast<const uint4*>(rec0[j] + c * 12);
                        const uint32_t ord = rec0[j][c * 12 + 4];
                        const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
                        const int wb2 = wa + 1 < p.res_words ? wa + 1 : wa;
                        const uint32_t* rs = reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(rsbase) + dres);
                        residual_piece(hx[j], rc, ord, rs[wa * 16 + i], rs[wb2 * 16 + i], wr + j * 2048);
                    }
                    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");
                    __syncthreads();
#pragma unroll
                    for (int st = 0; st < 2; st++) {
                        Ops o;
                        read_ops(ax + st * 4096, gx[st], 2048, o);
                        mfma8(o);
                    }
                }
            }
        }
    }
    __syncthreads();                                                // every wavefront is done with LDS

    // ---- epilogue: D lane l, register v = token l % 32, row 8 (v / 4) + 4 (l / 32) + v % 4 of the 32 x 32 tile ----
    const int rowb = rt0 * 16 + 64 * mh, tokb = t0 + 128 * th;
    const bool wide = !y_fp32 && (p.n & 7) == 0 && ((uintptr_t)Y & 15) == 0 && rowb + 64 <= p.n;      // uniform per wavefront
    if (wide) {
        // through LDS (the wavefront's own region; token rows of 144 bytes), so that a store writes 128-byte runs of Y
        char* const ep = lds + wave * G::EPI;
#pragma unroll
        for (int mb = 0; mb < 2; mb++)
#pragma unroll
            for (int tb = 0; tb < 4; tb++)
#pragma unroll
                for (int vq = 0; vq < 4; vq++) {
                    const __half2 lo = __floats2half2_rn(-acc[mb][tb][4 * vq + 0], -acc[mb][tb][4 * vq + 1]);
                    const __half2 hi = __floats2half2_rn(-acc[mb][tb][4 * vq + 2], -acc[mb][tb][4 * vq + 3]);
                    uint2 v;
                    v.x = __builtin_bit_cast(uint32_t, lo);
                    v.y = __builtin_bit_cast(uint32_t, hi);
                    *reinterpret_cast<uint2*>(ep + (32 * tb + l31) * 144 + (32 * mb + 8 * vq + 4 * lh) * 2) = v;
                }
        // (the wavefront reads back only what it wrote itself: LDS keeps a wavefront's accesses in order)
        __half* const Yh = reinterpret_cast<__half*>(Y);
#pragma unroll
        for (int it = 0; it < 16; it++) {
            const int tl = 8 * it + (lane >> 3), tok = tokb + tl;
            const uint4 v = *reinterpret_cast<const uint4*>(ep + tl * 144 + (lane & 7) * 16);
            if (tok < T) *reinterpret_cast<uint4*>(Yh + (int64_t)tok * p.n + rowb + (lane & 7) * 8) = v;
        }
        return;
    }
#pragma unroll
    for (int mb = 0; mb < 2; mb++)
#pragma unroll
        for (int tb = 0; tb < 4; tb++) {
            const int tok = tokb + 32 * tb + l31;
            if (tok >= T) continue;
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int row = rowb + 32 * mb + 8 * (v >> 2) + 4 * lh + (v & 3);
                if (row >= p.n) continue;
                const float val = -acc[mb][tb][v];
                if (y_fp32) reinterpret_cast<float*>(Y)[(int64_t)tok * p.n + row] = val;
                else reinterpret_cast<__half*>(Y)[(int64_t)tok * p.n + row] = __float2half(val);
            }
        }
}

template <int N8, bool HAS_RES>
hipError_t launch_gemm_shared(hipStream_t st, const TiledPlanes& p, const __half* X, int T, void* Y, int y_fp32,
                              const __half* xsal, int cfix) {
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute((const void*)gemm_shared_kernel<N8, HAS_RES>,
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, GsLds::TOTAL);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const dim3 grid((T + GS_TOK - 1) / GS_TOK, (p.nrt + GS_ROWT - 1) / GS_ROWT);
    hipLaunchKernelGGL((gemm_shared_kernel<N8, HAS_RES>), grid, dim3(256), GsLds::TOTAL, st, p, X, T, Y, y_fp32, xsal, cfix);
    return hipGetLastError();
}
