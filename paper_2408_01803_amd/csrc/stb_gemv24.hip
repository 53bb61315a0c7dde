// Decode GEMV for the tiled order (App. C: the memory-bound regime), one fat wavefront per superblock.
//
// 2:4 layers run on the sparse matrix-core instruction.  Every group of 4 columns keeps exactly 2 weights
// (Sec. 3.1), which is the operand form of v_smfmac_f32_16x16x64_f16: A holds the kept weights only (8 per lane
// for 16 columns), an index register says where inside its group of 4 each of them sits, and the instruction
// multiplies against 64 rows of B.  The kept weights come out of the packed planes in slot order -- the order the
// sign and id planes are stored in -- so the per-column scatter that the dense kernels need disappears, and with
// it their table in LDS.  Layers that keep 4 or 6 of 8 columns run the same kernel in a dense mode: 16 steps of 8
// columns on v_mfma_f32_16x16x32_f16 with the scatter table of stb_tiled.hpp.
//
// Operand layout of the sparse instruction (found by probing single-element operands on the device):
//   A  lane 16*g + i, element e (0..7): row i, uncompressed K = 16*g + 4*(e/2) + idx_e, idx_e = bits 2e+1:2e of
//      the 16-bit half of the index register that ABID selects (0: low, 1: high);
//   B  lane 16*g' + n, element j (0..15): column n, K = 32*(j/8) + 8*g' + j%8;
//   D  as v_mfma_f32_16x16x32_f16: lane 16*q + n holds rows 4*q + v, column n.
// The kernel maps K to columns so that lane group g reads block g of the superblock, as the tiled order stores
// it: step s (0..7) of a block covers its columns 16*s .. 16*s+15, K = 16*g + c <-> column 16*s + c of block g.
//
// Measured on the device: a SIMD issues one wavefront-wide vector instruction every 4 cycles however many
// wavefronts share it, so the kernel is bound by its instruction count.  It therefore runs two fat wavefronts per
// SIMD (a wavefront owns a whole superblock: 64 VGPRs of x) instead of four thin ones, which halves the
// per-wavefront set-up work a SIMD executes, and loads everything through few wide instructions.
// Layers with more than 8 superblocks are cut into column splits whose sums meet through the caller's workspace,
// or, at small batches, handled by the MULTI form of the kernel: a wavefront visits up to three superblocks per
// row tile and adds their products up itself.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>

#include <atomic>
#include <cstddef>

#include "stb_tiled.hpp"

using namespace stbt;


namespace {

typedef _Float16 half16_t __attribute__((ext_vector_type(16)));

constexpr int LDS24 = 160 * 1024 - 64; // dynamic LDS a workgroup may ask for (a few bytes are static)
constexpr int MAXV24 = 8;             // most superblocks a wavefront visits per row tile
constexpr int PHASE24 = 15;           // row tiles between two reductions (a multiple of 3: three tile buffers)

// Packed operands of one (row, block): mask, sign and id words of the two half blocks, scales, alpha_r.
struct Tile24 {
    uint2_t m0, m1;
    uint32_t s0, s1;
    uint2_t r0, r1;
    uint2_t sc;
    uint32_t ar;
    uint32_t et;                      // res_t word: residual sign bits of the first 16 salient columns of half 0 | half 1 << 16
};
constexpr int LMAIN24 = 8;            // load instructions per tile: packed planes ...
constexpr int LRES24 = 1;             // ... and the res_t word

// A vector-memory instruction that takes an SGPR written by a vector-ALU instruction less than five wait states
// earlier reads the old value (the hardware does not interlock this case).  The compiler pads its own loads, but it
// does not look into an asm statement -- and it restores spilled scalars with v_readlane right in front of their
// use.  So every asm statement with a scalar base starts with five wait states of its own.
#define STB24_SGPR_SETTLE "s_nop 4\n\t"

// The loads are asm statements with the plane base in SGPRs; wait24 names their destination registers.  Between
// a fetch and its wait the registers must not pass through a copy or a join of two definitions (the compiler
// does not know that the data arrives later).
// Byte offsets of the lane's records in tile 0 of each plane, counted from the lowest plane address of the layer
// (`image`): with them a tile's loads need one scalar base, and the tile's position goes into the 32-bit offsets
// (the launcher checks that the planes lie within 4 GiB of that address).
struct LaneOff24 {
    uint32_t m, s, r, c, a, t;        // mask, sign, region, scales, res_scale, res_t
};

// The loads of one tile, one asm statement: packed planes first, then (RES) the res_t word.
template <bool RES>
__device__ inline void fetch24(Tile24& d, const char* image, int tile, const LaneOff24& lo) {
    const uint32_t t10 = (uint32_t)tile << 10;
    const uint32_t vm = t10 + lo.m, vr = t10 + lo.r, vs = (t10 >> 1) + lo.s, vc = (t10 >> 1) + lo.c, va = (t10 >> 3) + lo.a;
    if constexpr (RES) {
        const uint32_t vt = (t10 >> 2) + lo.t;
        asm volatile(STB24_SGPR_SETTLE
                     "global_load_dwordx2 %0, %9, %15\n\t"
                     "global_load_dwordx2 %1, %9, %15 offset:512\n\t"
                     "global_load_dword %2, %10, %15\n\t"
                     "global_load_dword %3, %10, %15 offset:256\n\t"
                     "global_load_dwordx2 %4, %11, %15\n\t"
                     "global_load_dwordx2 %5, %11, %15 offset:512\n\t"
                     "global_load_dwordx2 %6, %12, %15\n\t"
                     "global_load_ushort %7, %13, %15\n\t"
                     "global_load_dword %8, %14, %15"
                     : "=&v"(d.m0), "=&v"(d.m1), "=&v"(d.s0), "=&v"(d.s1), "=&v"(d.r0), "=&v"(d.r1), "=&v"(d.sc), "=&v"(d.ar), "=&v"(d.et)
                     : "v"(vm), "v"(vs), "v"(vr), "v"(vc), "v"(va), "v"(vt), "s"(image));
    } else {
        asm volatile(STB24_SGPR_SETTLE
                     "global_load_dwordx2 %0, %8, %13\n\t"
                     "global_load_dwordx2 %1, %8, %13 offset:512\n\t"
                     "global_load_dword %2, %9, %13\n\t"
                     "global_load_dword %3, %9, %13 offset:256\n\t"
                     "global_load_dwordx2 %4, %10, %13\n\t"
                     "global_load_dwordx2 %5, %10, %13 offset:512\n\t"
                     "global_load_dwordx2 %6, %11, %13\n\t"
                     "global_load_ushort %7, %12, %13"
                     : "=&v"(d.m0), "=&v"(d.m1), "=&v"(d.s0), "=&v"(d.s1), "=&v"(d.r0), "=&v"(d.r1), "=&v"(d.sc), "=&v"(d.ar)
                     : "v"(vm), "v"(vs), "v"(vr), "v"(vc), "v"(va), "s"(image));
    }
}

// The res_t word of the lane's (row, block) in tile `tile` alone (lane records of 4 bytes).
template <typename T>
__device__ inline void fetch24_res(T& d, const char* image, int tile, const LaneOff24& lo) {
    const uint32_t v = ((uint32_t)tile << 8) + lo.t;
    asm volatile(STB24_SGPR_SETTLE "global_load_dword %0, %1, %2" : "=&v"(d.et) : "v"(v), "s"(image));
}

template <int K>
__device__ inline void wait24(Tile24& d) {
    asm volatile("s_waitcnt vmcnt(%9)"
                 : "+v"(d.m0), "+v"(d.m1), "+v"(d.s0), "+v"(d.s1), "+v"(d.r0), "+v"(d.r1), "+v"(d.sc), "+v"(d.ar),
                   "+v"(d.et)
                 : "n"(K));
}
// The same in two steps: the packed planes (the older loads of a tile), then the res_t word.
template <int K>
__device__ inline void wait24_main(Tile24& d) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(d.m0), "+v"(d.m1), "+v"(d.s0), "+v"(d.s1), "+v"(d.r0), "+v"(d.r1), "+v"(d.sc), "+v"(d.ar)
                 : "n"(K));
}
template <int K, typename T>
__device__ inline void wait24_res(T& d) {
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(d.et) : "n"(K));
}

// The same for 6:8 layers: 12 bytes of sign bits per block (not cut in halves), 12 bytes of ids per half block.
struct Tile68 {
    uint2_t m0, m1;
    uint3_t s;
    uint3_t r0, r1;
    uint2_t sc;
    uint32_t ar;
    uint32_t et;
};
constexpr int LMAIN68 = 7;

template <bool RES>
__device__ inline void fetch24(Tile68& d, const char* image, int tile, const LaneOff24& lo) {
    const uint32_t t10 = (uint32_t)tile << 10;
    const uint32_t vm = t10 + lo.m, vs = (uint32_t)tile * 768u + lo.s, vr = (uint32_t)tile * 1536u + lo.r;
    const uint32_t vc = (t10 >> 1) + lo.c, va = (t10 >> 3) + lo.a;
    if constexpr (RES) {
        const uint32_t vt = (t10 >> 2) + lo.t;
        asm volatile(STB24_SGPR_SETTLE
                     "global_load_dwordx2 %0, %8, %14\n\t"
                     "global_load_dwordx2 %1, %8, %14 offset:512\n\t"
                     "global_load_dwordx3 %2, %9, %14\n\t"
                     "global_load_dwordx3 %3, %10, %14\n\t"
                     "global_load_dwordx3 %4, %10, %14 offset:768\n\t"
                     "global_load_dwordx2 %5, %11, %14\n\t"
                     "global_load_ushort %6, %12, %14\n\t"
                     "global_load_dword %7, %13, %14"
                     : "=&v"(d.m0), "=&v"(d.m1), "=&v"(d.s), "=&v"(d.r0), "=&v"(d.r1), "=&v"(d.sc), "=&v"(d.ar), "=&v"(d.et)
                     : "v"(vm), "v"(vs), "v"(vr), "v"(vc), "v"(va), "v"(vt), "s"(image));
    } else {
        asm volatile(STB24_SGPR_SETTLE
                     "global_load_dwordx2 %0, %7, %12\n\t"
                     "global_load_dwordx2 %1, %7, %12 offset:512\n\t"
                     "global_load_dwordx3 %2, %8, %12\n\t"
                     "global_load_dwordx3 %3, %9, %12\n\t"
                     "global_load_dwordx3 %4, %9, %12 offset:768\n\t"
                     "global_load_dwordx2 %5, %10, %12\n\t"
                     "global_load_ushort %6, %11, %12"
                     : "=&v"(d.m0), "=&v"(d.m1), "=&v"(d.s), "=&v"(d.r0), "=&v"(d.r1), "=&v"(d.sc), "=&v"(d.ar)
                     : "v"(vm), "v"(vs), "v"(vr), "v"(vc), "v"(va), "s"(image));
    }
}

template <int K>
__device__ inline void wait24(Tile68& d) {
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(d.m0), "+v"(d.m1), "+v"(d.s), "+v"(d.r0), "+v"(d.r1), "+v"(d.sc), "+v"(d.ar),
                   "+v"(d.et)
                 : "n"(K));
}
template <int K>
__device__ inline void wait24_main(Tile68& d) {
    asm volatile("s_waitcnt vmcnt(%7)"
                 : "+v"(d.m0), "+v"(d.m1), "+v"(d.s), "+v"(d.r0), "+v"(d.r1), "+v"(d.sc), "+v"(d.ar)
                 : "n"(K));
}

// MODE of the kernel below: 2 = 2:4 layers on the sparse instruction; 4 / 6 = layers that keep 4 / 6 of 8 columns
// on the dense instruction with the scatter table of stb_tiled.hpp.
template <int MODE> struct TileOf { typedef Tile24 type; static constexpr int lmain = LMAIN24; };
template <> struct TileOf<6> { typedef Tile68 type; static constexpr int lmain = LMAIN68; };

// The mask, sign and id words of half h of a tile in the form the shared expansion takes them.
__device__ inline void half_of(const Tile24& t, int h, HalfData<4>& d) {
    d.m[0] = h == 0 ? t.m0[0] : t.m1[0]; d.m[1] = h == 0 ? t.m0[1] : t.m1[1];
    d.s[0] = h == 0 ? t.s0 : t.s1; d.s[1] = 0u;
    d.r[0] = h == 0 ? t.r0[0] : t.r1[0]; d.r[1] = h == 0 ? t.r0[1] : t.r1[1]; d.r[2] = 0u;
}
__device__ inline void half_of(const Tile68& t, int h, HalfData<6>& d) {
    d.m[0] = h == 0 ? t.m0[0] : t.m1[0]; d.m[1] = h == 0 ? t.m0[1] : t.m1[1];
    if (h == 0) { d.s[0] = t.s[0]; d.s[1] = t.s[1]; }                                   // bits 0..47
    else { d.s[0] = __builtin_amdgcn_alignbit(t.s[2], t.s[1], 16u); d.s[1] = t.s[2] >> 16; }   // bits 48..95
    d.r[0] = h == 0 ? t.r0[0] : t.r1[0]; d.r[1] = h == 0 ? t.r0[1] : t.r1[1]; d.r[2] = h == 0 ? t.r0[2] : t.r1[2];
}

// expand_group of stb_tiled.hpp with the constants in registers (K3 = 0x03030303, K4 = 0x04000400,
// KS = 0x80008000), so that every and-or is one compiler-scheduled instruction.
template <int N8>
__device__ inline void expand8(const HalfData<N8>& d, uint32_t TL, uint32_t TH, int t, const uint4& L,
                               uint32_t K3, uint32_t K4, uint32_t KS, uint32_t out[4]) {
    uint32_t W[3];
    if (N8 == 4) {
        const uint32_t rw = d.r[t >> 2], r2 = rw >> 2;
        const uint32_t b = t & 3;
        const uint32_t Z = perm(r2, rw, b | (b << 8) | ((4 + b) << 16) | ((4 + b) << 24));
        W[0] = perm(TH, TL, and_or_v(Z, K3, K4));
        W[1] = perm(TH, TL, and_or_v(Z >> 4, K3, K4));
        const uint32_t sw = d.s[0];
        const uint32_t sb = (t >> 1) & 3;
        const uint32_t X = perm(sw, sw, 0x000C000Cu | (sb << 8) | (sb << 24));     // halves = sign byte << 8
        const int base = 4 * (t & 1);
        W[0] = and_or_v(pk_shl(X, 7 - base, 6 - base), KS, W[0]);                   // scales are >= 0: their sign bit is clear
        W[1] = and_or_v(pk_shl(X, 5 - base, 4 - base), KS, W[1]);
        out[0] = perm(W[1], W[0], L.x);
        out[1] = perm(W[1], W[0], L.y);
        out[2] = perm(W[1], W[0], L.z);
        out[3] = perm(W[1], W[0], L.w);
    } else {
        const uint32_t v = window32<3>(d.r, 12 * t), v2 = v >> 2;
        const uint32_t Z = perm(v2, v, 0x04040000u);
        const uint32_t Z1 = perm(v2, v, 0x05050101u);
        W[0] = perm(TH, TL, and_or_v(Z, K3, K4));
        W[1] = perm(TH, TL, and_or_v(Z >> 4, K3, K4));
        W[2] = perm(TH, TL, and_or_v(Z1, K3, K4));
        const uint32_t sv = window32<2>(d.s, 6 * t);
        const uint32_t X = perm(sv, sv, 0x000C000Cu);                               // halves = (sign bits) << 8
        W[0] = and_or_v(pk_shl(X, 7, 6), KS, W[0]);
        W[1] = and_or_v(pk_shl(X, 5, 4), KS, W[1]);
        W[2] = and_or_v(pk_shl(X, 3, 2), KS, W[2]);
        out[0] = perm(W[1], W[0], L.x);
        out[1] = perm(W[1], W[0], L.y);
        out[2] = perm(W[2], W[1], L.z);
        out[3] = perm(W[2], W[1], L.w);
    }
}

// Index register for 32 columns: every mask nibble (two bits set) becomes the positions of its two kept
// weights, low one in bits 1:0, high one in bits 3:2.  (nibble >> 1) & 7 is 1..6 for the six valid nibbles
// and addresses an 8-byte table through v_perm_b32; a nibble of the zero padding maps to positions 0, 1.
__device__ inline uint32_t index_word(uint32_t m, uint32_t T0, uint32_t T1, uint32_t K7) {
    const uint32_t t = m >> 1;
    const uint32_t lo = perm(T1, T0, t & K7);                   // index nibbles of the low nibble of each byte
    const uint32_t hi = perm(T1, T0, (t >> 4) & K7);            // ... of the high nibbles
    return (hi << 4) | lo;
}

// One wavefront-wide global -> LDS load of 16 bytes per active lane: lane l's bytes land at LDS address m0 + 16 * l.
__device__ inline void load_to_lds24(uint32_t lds_addr, uint32_t voff, const void* base) {
    asm volatile("s_mov_b32 m0, %0\n\t" STB24_SGPR_SETTLE "global_load_lds_dwordx4 %1, %2" : : "s"(lds_addr), "v"(voff), "s"(base) : "memory", "m0");
}

struct Res24 {
    ResSel sel;
    uint32_t xs[4];     // x at the 8 salient columns of the record (B operand of the dense instruction)
};

// One layer of a launch: its planes, vectors, scratch and launch shape (see stb_tiled_gemv24_plan), and where its
// workgroups sit in the launch's grid.  A launch takes up to GROUP24_MAX layers (the matrices of a decoder layer that
// share their input, say): the grid is the layers' grids one after the other, and a workgroup finds its layer by its
// index.  The descriptors travel by value in the kernel arguments, so a launch needs no table in device memory and can
// be captured in a HIP graph.
struct Gemv24Layer {
    TiledPlanes p;
    const char* image;        // lowest address of the streamed planes; their offsets from it (all below 4 GiB):
    uint32_t off_mask, off_sign, off_region, off_scales, off_res_scale, off_res_t;
    const __half* x;
    void* y;
    float* ws_part;
    uint32_t* ws_count;
    int R, SPS, PHT, WREG, REC_OFF, PART_OFF, V, XS;
    int G, S;                 // workgroups along the rows, column splits: the layer owns G * S workgroups ...
    int block0;               // ... starting at this one
    int variant;              // MODE | HAS_RES << 3 | MULTI << 4
};
constexpr int GROUP24_MAX = 8;
struct Gemv24Group {
    int n_layers, B, y_fp32, pad;
    Gemv24Layer l[GROUP24_MAX];
};

// Dynamic LDS of a workgroup: [0, 16) the ticket of the column splits; dense modes: the scatter table (32 KB); then one
// region of WREG bytes per wavefront.
constexpr int LDS24_HEAD = 16;

template <int MODE, bool HAS_RES, bool MULTI>
__device__ __forceinline__ void gemv24_body(const Gemv24Layer& d, const int B, const int y_fp32, const int gr, const int ks,
                                            char* const dyn) {
    const TiledPlanes& p = d.p;
    const __half* __restrict__ const x = d.x;
    void* __restrict__ const y = d.y;
    const int R = d.R, SPS = d.SPS, PHT = d.PHT, WREG = d.WREG, REC_OFF = d.REC_OFF, PART_OFF = d.PART_OFF, XS = d.XS;
    float* __restrict__ const ws_part = d.ws_part;
    uint32_t* __restrict__ const ws_count = d.ws_count;
    uint32_t& ticket = *reinterpret_cast<uint32_t*>(dyn);
    const int V = MULTI ? d.V : 1;                               // visits per wavefront
    constexpr int N8 = MODE == 6 ? 6 : 4;
    typedef typename TileOf<MODE>::type Tile;
    ScatterLds* const lut = reinterpret_cast<ScatterLds*>(dyn + LDS24_HEAD);      // dense modes: the scatter table, eight copies
    // Each wavefront owns a region of LDS of WREG bytes: its slice of x ([row][1040 bytes], B rows and one of zeros),
    // its 16 salient-column records at REC_OFF, its partial products [PHT][256] fp32 at PART_OFF (with one visit
    // per wavefront: 0, on top of the x rows, which are in registers by then).  A wavefront stages all of it itself,
    // so nothing before the first reduction needs a barrier and every wavefront starts on its tiles as soon as its
    // data is there.
    // V > 1 (layers with more than 8 superblocks, small batches): a wavefront visits V superblocks, sb, sb + SPS, ..,
    // for every row tile and adds their products up in registers, so that no other workgroup holds a part of the
    // row's sum; it keeps V slices of x (XS bytes apart) and V record sets in LDS and takes the operands of a
    // visit from there before each product.
    char* const lds_base = dyn + LDS24_HEAD + (MODE == 2 ? 0 : (int)sizeof(ScatterLds));
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int i = lane & 15, g = lane >> 4;
    const int nthr = blockDim.x;                                  // at least 64 * SPS: one wavefront per superblock of the split
    const int S = d.S;
    const int sb = ks * SPS * V + wave;                           // superblock of the first visit
    const int r0 = gr * R;
    const int r1 = r0 + R < p.nrt ? r0 + R : p.nrt;
    const int rl = r1 - 1;
    const bool active = wave < SPS && sb < p.nsb;                 // uniform per wavefront (a launch of several layers has the widest layer's wavefronts)
    const int Wa = p.nsb - ks * SPS * V < SPS ? p.nsb - ks * SPS * V : SPS;   // wavefronts with work
    auto sb_of = [&](int v) { return sb + v * SPS < p.nsb ? sb + v * SPS : sb; };       // a visit past the last superblock re-reads the first
    auto tile_of = [&](int rt, int v = 0) { return rt * p.nsb + sb_of(v); };
    auto clamp = [&](int rt) { return rt < rl ? rt : rl; };
    const uint32_t o8 = (uint32_t)lane * 8u, o4 = (uint32_t)lane * 4u, o2 = (uint32_t)lane * 2u;
    constexpr int XROW = 1040;                                    // bytes per staged row; the 16-byte skew spreads rows over banks
    char* const wreg = lds_base + (int64_t)wave * WREG;
    float* const part = reinterpret_cast<float*>(wreg + PART_OFF);
    uint32_t* const recs = reinterpret_cast<uint32_t*>(wreg + REC_OFF);         // [visit][block g][half][record 0 / 1] x 12

    // the scatter table is built while the first loads are in flight (wavefronts without work build it right away);
    // arithmetic and LDS stores only, the barrier comes after the staging
    if constexpr (MODE != 2) { if (!active) build_luts<N8>(lut); }
    half16_t xr[8];                                              // MODE 2: B operands of the 8 steps of a block
    half8_t xd[16];                                              // dense modes: of the 16 steps
    Res24 inv[2];                                                // first record of the lane's block, per half
    ResSel sel2[2];                                              // second record (half blocks with 9..16 salient columns)
    uint32_t xs2[2][4];
    int nch0 = 0, nch1 = 0;
    Tile t0 = {}, t1 = {}, t2 = {};
    constexpr int LMAIN = TileOf<MODE>::lmain;
    constexpr int L = LMAIN + (HAS_RES ? LRES24 : 0);            // loads per tile in the streaming loop
    const char* const image = d.image;
    const uint32_t o12 = o4 * 3u;
    const LaneOff24 lo = {d.off_mask + o8, d.off_sign + (MODE == 6 ? o12 : o4), d.off_region + (MODE == 6 ? o12 : o8),
                          d.off_scales + o8, d.off_res_scale + o2, d.off_res_t + o4};
    auto fetch_res = [&](Tile& t, int rt, int v) {
        if constexpr (HAS_RES) fetch24_res(t, image, tile_of(__builtin_amdgcn_readfirstlane(rt), __builtin_amdgcn_readfirstlane(v)), lo);
    };
    auto fetch_tile = [&](Tile& t, int rt, int v) {
        fetch24<HAS_RES>(t, image, tile_of(__builtin_amdgcn_readfirstlane(rt), __builtin_amdgcn_readfirstlane(v)), lo);
    };
    if (MULTI && active) {
        // ---- several visits: the slices of x and the record sets go from global memory straight to LDS (no staging
        //      registers); rows of zeros, the zero pads behind the rows and the lanes past column k are stored first ----
        const uint4_t zero = {0u, 0u, 0u, 0u};
        for (int v = 0; v < V; v++) {
            const int sbv = sb + v * SPS;
            if (sbv >= p.nsb) break;
            char* slice = wreg + v * XS;
            if (sbv * 512 + 512 > p.k)
                for (int b = 0; b < B; b++) *reinterpret_cast<uint4_t*>(slice + b * XROW + lane * 16) = zero;
            if (B < 16) *reinterpret_cast<uint4_t*>(slice + B * XROW + lane * 16) = zero;
            if (HAS_RES && lane <= B && lane < 16) *reinterpret_cast<uint4_t*>(slice + lane * XROW + 1024) = zero;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" : : : "memory");
        const uint32_t lds_w = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)wreg;
        for (int v = 0; v < V; v++) {
            const int sbv = sb + v * SPS;
            if (sbv >= p.nsb) break;
            const int col = sbv * 512 + lane * 8;
            if (col < p.k)
                for (int b = 0; b < B; b++)
                    load_to_lds24(lds_w + v * XS + b * XROW, (uint32_t)(b * p.k + col) * 2u, x);
            if (HAS_RES && lane < 48) {
                const int rI = lane / 6, rc = (lane - 6 * rI) / 3, rpc = lane % 3;
                const uint32_t off = (uint32_t)((((sbv * 8 + rI) * p.sal_chunks + (rc < p.sal_chunks ? rc : 0)) * 12 + 4 * rpc) * 4);
                load_to_lds24(lds_w + REC_OFF + v * 768, off, p.sal_tab);
            }
        }
        fetch24<false>(t0, image, tile_of(clamp(r0)), lo);
        if constexpr (MODE != 2) build_luts<N8>(lut);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(LMAIN) : "memory");
        if (HAS_RES && lane < 48 && lane % 3 == 2) {
            // the pieces with the column positions become byte offsets inside a staged row (see below)
            const uint32_t g2 = (uint32_t)(lane / 12) * (128u * 0x00010001u);
            for (int v = 0; v < V; v++) {
                if (sb + v * SPS >= p.nsb) break;
                uint4_t sr = *reinterpret_cast<const uint4_t*>(&recs[v * 192 + 4 * lane]);
#pragma unroll
                for (int w = 0; w < 4; w++) {
                    const uint32_t none = sr[w] & 0x80008000u;
                    const uint32_t full = __umul24(none >> 15, 0xFFFFu);
                    sr[w] = ((((sr[w] & 0x007F007Fu) + g2) << 1) & ~full) | (none >> 5);
                }
                *reinterpret_cast<uint4_t*>(&recs[v * 192 + 4 * lane]) = sr;
            }
        }
    }
    if (!MULTI && active) {
        // ---- all loads go out before the first wait: lane l brings columns 8l .. 8l+7 of the superblock for every
        //      batch row (one 16-byte load per row), lanes 0..47 the 16-byte pieces of the (block, half) records, then
        //      the packed planes of the first row tile ----
        const int col = sb * 512 + lane * 8;
        const bool col_ok = col < p.k;
        const __half* xsrc = x + (col_ok ? col : 0);
        uint4_t sx0, sx1, sx2, sx3, sx4, sx5, sx6, sx7, sx8, sx9, sx10, sx11, sx12, sx13, sx14, sx15;
#define STB24_LOAD(u, reg) { const __half* a = xsrc + (int64_t)(u) * p.k; asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(reg) : "v"(a)); }
        // B loads per lane; the conditions are nested so that a small batch passes few of them
        STB24_LOAD(0, sx0)
        if (B > 1) STB24_LOAD(1, sx1)
        if (B > 2) { STB24_LOAD(2, sx2) if (B > 3) STB24_LOAD(3, sx3) }
        if (B > 4) { STB24_LOAD(4, sx4) if (B > 5) STB24_LOAD(5, sx5) if (B > 6) STB24_LOAD(6, sx6) if (B > 7) STB24_LOAD(7, sx7) }
        if (B > 8) {
            STB24_LOAD(8, sx8) if (B > 9) STB24_LOAD(9, sx9) if (B > 10) STB24_LOAD(10, sx10) if (B > 11) STB24_LOAD(11, sx11)
            if (B > 12) STB24_LOAD(12, sx12) if (B > 13) STB24_LOAD(13, sx13) if (B > 14) STB24_LOAD(14, sx14) if (B > 15) STB24_LOAD(15, sx15)
        }
#undef STB24_LOAD
        uint4_t sr = {0u, 0u, 0u, 0u};
        if (HAS_RES && lane < 48) {                  // (block, half) lane / 6, record (lane % 6) / 3 of it, 16-byte piece lane % 3
            const int rI = lane / 6, rc = (lane - 6 * rI) / 3, rpc = lane % 3;
            const uint32_t* src = p.sal_tab + (((int64_t)sb * 8 + rI) * p.sal_chunks + (rc < p.sal_chunks ? rc : 0)) * 12 + 4 * rpc;
            asm volatile("global_load_dwordx4 %0, %1, off" : "+v"(sr) : "v"(src));
        }
        fetch24<false>(t0, image, tile_of(clamp(r0)), lo);
        if constexpr (MODE != 2) build_luts<N8>(lut);
        // The second and third tile go out after the operands are in registers: a compute unit keeps a limited
        // number of loads in flight, and the other wavefront of the SIMD should get its first tile early too
        // (issuing them here instead was measured: no faster with one wavefront per SIMD, slower with two).
        // The staging loads are older than the LMAIN of the first tile.
        asm volatile("s_waitcnt vmcnt(%17)"
                     : "+v"(sx0), "+v"(sx1), "+v"(sx2), "+v"(sx3), "+v"(sx4), "+v"(sx5), "+v"(sx6), "+v"(sx7),
                       "+v"(sx8), "+v"(sx9), "+v"(sx10), "+v"(sx11), "+v"(sx12), "+v"(sx13), "+v"(sx14), "+v"(sx15),
                       "+v"(sr)
                     : "n"(LMAIN));
        {
            char* dst = wreg + lane * 16;
            const uint4_t zero = {0u, 0u, 0u, 0u};
#define STB24_STORE(u, reg) *reinterpret_cast<uint4_t*>(dst + (u) * XROW) = col_ok ? reg : zero;
            STB24_STORE(0, sx0)
            if (B > 1) STB24_STORE(1, sx1)
            if (B > 2) { STB24_STORE(2, sx2) if (B > 3) STB24_STORE(3, sx3) }
            if (B > 4) { STB24_STORE(4, sx4) if (B > 5) STB24_STORE(5, sx5) if (B > 6) STB24_STORE(6, sx6) if (B > 7) STB24_STORE(7, sx7) }
            if (B > 8) {
                STB24_STORE(8, sx8) if (B > 9) STB24_STORE(9, sx9) if (B > 10) STB24_STORE(10, sx10) if (B > 11) STB24_STORE(11, sx11)
                if (B > 12) STB24_STORE(12, sx12) if (B > 13) STB24_STORE(13, sx13) if (B > 14) STB24_STORE(14, sx14) if (B > 15) STB24_STORE(15, sx15)
            }
#undef STB24_STORE
            if (B < 16) *reinterpret_cast<uint4_t*>(dst + B * XROW) = zero;     // row B: zeros, read by the lanes without a batch row
            if (HAS_RES) {
                // the 16 bytes after each row's 1024: zeros, the target of the table entries that hold no column
                if (lane <= B && lane < 16) *reinterpret_cast<uint4_t*>(wreg + lane * XROW + 1024) = zero;
                if (lane < 48) {
                    if (lane % 3 == 2) {
                        // the piece with the 8 column positions (inside the block; 0xFFFF = no entry) becomes byte
                        // offsets inside a staged row: 2 * (128 * block + position), 1024 for no entry
                        // (two 16-bit fields per word, worked on in place: no field carries into the other)
                        const uint32_t g2 = (uint32_t)(lane / 12) * (128u * 0x00010001u);
#pragma unroll
                        for (int w = 0; w < 4; w++) {
                            const uint32_t none = sr[w] & 0x80008000u;                      // bit 15: no entry
                            const uint32_t full = __umul24(none >> 15, 0xFFFFu);            // 0xFFFF in such a field
                            sr[w] = ((((sr[w] & 0x007F007Fu) + g2) << 1) & ~full) | (none >> 5);
                        }
                    }
                    *reinterpret_cast<uint4_t*>(&recs[4 * lane]) = sr;     // [block][half][record 0 / 1] x 12
                }
            }
        }
    }
    if constexpr (MODE != 2) __syncthreads();       // the scatter table is complete (every wavefront comes here)
    // ---- the wavefront takes the B operands, the records and the x of the salient columns of visit v back from LDS
    //      (its own stores: LDS keeps a wavefront's accesses in order) ----
    auto visit_setup = [&](int v) {
        const char* const xsl = wreg + v * XS;
        const uint32_t* const recv = recs + v * 192;
        if constexpr (MODE == 2) {
            // B lane 16*g + n: elements 0..7 <-> block g/2, elements 8..15 <-> block 2 + g/2, columns 16*s + 8*(g%2) ..
            const char* xrow = xsl + (i < B ? i : B) * XROW + (g >> 1) * 256 + (g & 1) * 16;
#pragma unroll
            for (int s = 0; s < 8; s++) {
                const uint4_t lo = *reinterpret_cast<const uint4_t*>(xrow + 32 * s);
                const uint4_t hi = *reinterpret_cast<const uint4_t*>(xrow + 512 + 32 * s);
                typedef uint32_t uint8_vec __attribute__((ext_vector_type(8)));
                const uint8_vec v = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
                xr[s] = __builtin_bit_cast(half16_t, v);
            }
        } else {
            // B lane 16*g + n of step t: columns 8t .. 8t+7 of block g
            const char* xrow = xsl + (i < B ? i : B) * XROW + g * 256;
#pragma unroll
            for (int t = 0; t < 16; t++) xd[t] = __builtin_bit_cast(half8_t, *reinterpret_cast<const uint4_t*>(xrow + 16 * t));
        }
        if (HAS_RES) {
            const char* xrow0 = xsl + (i < B ? i : B) * XROW;               // the lane's staged row of x (or the zeros)
            auto gather = [&](const uint4_t& q, uint32_t out[4]) {          // x at the 8 byte offsets of a record
                const uint32_t qw[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
                for (int v = 0; v < 4; v++) {
                    const ushort2_t pr = {*reinterpret_cast<const unsigned short*>(xrow0 + (qw[v] & 0xFFFFu)),
                                          *reinterpret_cast<const unsigned short*>(xrow0 + (qw[v] >> 16))};
                    out[v] = __builtin_bit_cast(uint32_t, pr);
                }
            };
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const uint32_t* rec = &recv[(g * 2 + h) * 24];
                const uint4_t ra = *reinterpret_cast<const uint4_t*>(rec);
                const uint4_t rp = *reinterpret_cast<const uint4_t*>(rec + 8);
                inv[h].sel.sel0 = ra.x; inv[h].sel.sel1 = ra.y; inv[h].sel.bit0 = ra.z; inv[h].sel.bit1 = ra.w;
                const uint2_t rb = *reinterpret_cast<const uint2_t*>(rec + 4);
                const uint32_t ord = rb.x;
                const int nc = __builtin_amdgcn_readfirstlane((int)rb.y);
                if (h == 0) nch0 = nc; else nch1 = nc;
                gather(rp, inv[h].xs);
                if (nc > 1) {                        // the second record of the half block
                    const uint4_t rc = *reinterpret_cast<const uint4_t*>(rec + 12);
                    const uint4_t rq = *reinterpret_cast<const uint4_t*>(rec + 20);
                    sel2[h].sel0 = rc.x; sel2[h].sel1 = rc.y; sel2[h].bit0 = rc.z; sel2[h].bit1 = rc.w;
                    gather(rq, xs2[h]);
                }
            }
        }
    };
    // producer side of the three tile buffers.  Order of the products of a workgroup: phase by phase (PHT row tiles),
    // inside a phase visit by visit, inside a visit row tile by row tile -- so that a wavefront takes the operands of a
    // visit (64 registers of x, the gathered salient x) once per phase and visit, not once per product.
    int p_ph0 = r0, p_n = r1 - r0 < PHT ? r1 - r0 : PHT, p_i = 0, p_v = 0;
    auto advance = [&]() {
        if (++p_i == p_n) {
            p_i = 0;
            if (++p_v == V) { p_v = 0; p_ph0 += p_n; p_n = r1 - p_ph0 < PHT ? r1 - p_ph0 : PHT; }
        }
    };
    auto fetch_next = [&](Tile& t) {
        if (p_n > 0) {
            fetch_tile(t, p_ph0 + p_i, p_v);
            advance();
        } else {
            fetch_tile(t, rl, V - 1);                // past the end: the last one again (same number of loads on every path)
        }
    };
    if (active) {
        if (!MULTI) visit_setup(0);
        // with one visit the partial products overwrite the x rows: every read above must have returned
        __builtin_amdgcn_s_waitcnt(0xC07F);          // lgkmcnt(0)
        __builtin_amdgcn_sched_barrier(0);
        fetch_res(t0, clamp(r0), 0);
        if (p_n > 0) advance();                      // t0 holds (r0, visit 0)
        fetch_next(t1);
        fetch_next(t2);
    }

    // index table of index_word and the other constants, in VGPRs (a VOP3 instruction takes one constant)
    uint32_t T0 = 0x09080404u, T1 = 0x0E0E0D0Cu, K7 = 0x07070707u, K3 = 0x03030303u, K4 = 0x04000400u, KS = 0x80008000u;
    asm volatile("" : "+v"(T0), "+v"(T1), "+v"(K7), "+v"(K3), "+v"(K4), "+v"(KS));

    const int64_t n16 = (int64_t)p.nrt * 16;
    const uint32_t b_magic = B > 1 ? (uint32_t)((0x100000000ull + (uint32_t)B - 1) / (uint32_t)B) : 0u;
    auto div_b = [&](int v) { return B > 1 ? (int)__umulhi((uint32_t)v, b_magic) : v; };     // v / B, v < 2^27
    auto store_y = [&](int row, int b, float s) {
        if (b < B && row < p.n) {
            if (y_fp32) reinterpret_cast<float*>(y)[(int64_t)b * p.n + row] = -s;
            else reinterpret_cast<__half*>(y)[(int64_t)b * p.n + row] = __float2half(-s);
        }
    };

    // One (row tile, superblock): the steps over the block's columns (sparse: 8 of 16 columns; dense: 16 of 8), then
    // the residual term of the two halves.
    float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};         // sum over the visits of the current row tile
    auto product = [&](Tile& tr, int rt, int slot) {
        const uint32_t TL = perm(tr.sc[1], tr.sc[0], 0x06040200u), TH = perm(tr.sc[1], tr.sc[0], 0x07050301u);
        const uint32_t mw[4] = {tr.m0[0], tr.m0[1], tr.m1[0], tr.m1[1]};
        if constexpr (MODE == 2) {
            const uint32_t rw[4] = {tr.r0[0], tr.r0[1], tr.r1[0], tr.r1[1]};
            const uint32_t sw[2] = {tr.s0, tr.s1};
#pragma unroll
            for (int w = 0; w < 4; w++) {                 // 32 columns: two steps
                const uint32_t IDX = index_word(mw[w], T0, T1, K7);
                const uint32_t r2 = rw[w] >> 2;
#pragma unroll
                for (int u = 0; u < 2; u++) {
                    const int s = 2 * w + u;
                    uint32_t W[4];
#pragma unroll
                    for (int c = 0; c < 2; c++) {         // byte 2u + c of the id word: 4 kept weights
                        const uint32_t bb = 2 * u + c;
                        const uint32_t Z = perm(r2, rw[w], bb | (bb << 8) | ((4 + bb) << 16) | ((4 + bb) << 24));
                        W[2 * c] = perm(TH, TL, and_or_v(Z, K3, K4));
                        W[2 * c + 1] = perm(TH, TL, and_or_v(Z >> 4, K3, K4));
                    }
                    const uint32_t sbi = (uint32_t)(s & 3);   // byte of the half's sign word
                    const uint32_t X = perm(sw[w >> 1], sw[w >> 1], 0x000C000Cu | (sbi << 8) | (sbi << 24));
#pragma unroll
                    for (int q = 0; q < 4; q++) W[q] = and_or_v(pk_shl(X, 7 - 2 * q, 6 - 2 * q), KS, W[q]);
                    const half8_t a = as_half8(W);
                    if (u == 0) acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, xr[s], acc, (int)IDX, 0, 0);
                    else acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(a, xr[s], acc, (int)IDX, 0, 1);
                }
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                HalfData<N8> d;
                half_of(tr, h, d);
                constexpr int D = 4;                                  // table reads run D groups ahead
                uint4 gl[D];
#pragma unroll
                for (int t = 0; t < D; t++) gl[t] = lut_fetch<N8>(d, t, lut, lane & 7);
#pragma unroll
                for (int t = 0; t < 8; t++) {
                    const uint4 cur = gl[t % D];
                    if (t + D < 8) gl[t % D] = lut_fetch<N8>(d, t + D, lut, lane & 7);
                    uint32_t o[4];
                    expand8<N8>(d, TL, TH, t, cur, K3, K4, KS, o);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), xd[8 * h + t], acc, 0, 0, 0);
                }
            }
        }
        if (HAS_RES) {
            wait24_res<2 * L>(tr);                    // the tile's res_t word: younger than its packed planes
            const uint32_t ar1 = tr.ar & 0xFFFFu, ar2 = ar1 | (ar1 << 16);
#pragma unroll
            for (int h = 0; h < 2; h++) {
                if ((h == 0 ? nch0 : nch1) > 0) {
                    const uint32_t rb = h == 0 ? tr.et : tr.et >> 16;      // bits 0..7: first record, 8..15: second
                    uint32_t o[4];
                    residual_chunk(&mw[2 * h], rb, ar2, inv[h].sel, o);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(inv[h].xs), acc, 0, 0, 0);
                    if ((h == 0 ? nch0 : nch1) > 1) {    // entries 8..15: their bits follow in the same 32-bit window
                        residual_chunk(&mw[2 * h], rb >> 8, ar2, sel2[h], o);
                        acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(xs2[h]), acc, 0, 0, 0);
                    }
                }
            }
        }
    };
    auto store_partial = [&](int slot) {
        float* dst = part + (slot * 256 + lane);
#pragma unroll
        for (int v = 0; v < 4; v++) dst[64 * v] = acc[v];
        acc = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    };

    auto add_partial = [&](int slot) {
        float* dst = part + (slot * 256 + lane);
#pragma unroll
        for (int v = 0; v < 4; v++) dst[64 * v] += acc[v];
        acc = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
    };

    // Half blocks with more than 16 salient columns: the records after the second, outside the streaming loop (rare).
    auto extra_records = [&](int rt, int v) {
        const int64_t rstride = (int64_t)p.res_words * 16;
        const int q = 4 * sb_of(v) + g;
        const bool live = i < B && q < p.nb;
        const unsigned short* xg = reinterpret_cast<const unsigned short*>(x + (int64_t)(i < B ? i : B - 1) * p.k + (int64_t)(q < p.nb ? q : 0) * 128);
        float4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int h = 0; h < 2; h++) {
            const int nc = h == 0 ? nch0 : nch1;
            if (nc <= 2) continue;
            HalfData<N8> d;
            load_half<N8>(p, (int64_t)tile_of(rt, v), lane_offsets<N8>(lane, h), h, d);
            const uint32_t ar2 = d.ar | (d.ar << 16);
            for (int c = 2; c < nc; c++) {
                const uint32_t* rec = p.sal_tab + (((int64_t)q * 2 + h) * p.sal_chunks + c) * 12;
                ResSel sel;
                sel.sel0 = rec[0]; sel.sel1 = rec[1]; sel.bit0 = rec[2]; sel.bit1 = rec[3];
                const uint32_t ord = rec[4];
                uint32_t hx[8];
                for (int e = 0; e < 8; e++) {
                    const uint32_t pos = (rec[8 + (e >> 1)] >> (16 * (e & 1))) & 0xFFFFu;
                    hx[e] = live && pos < 128u ? (uint32_t)xg[pos & 127u] : 0u;
                }
                uint32_t xs4[4];
                for (int v = 0; v < 4; v++) xs4[v] = hx[2 * v] | (hx[2 * v + 1] << 16);
                const int wa = (int)(ord >> 5) < p.res_words ? (int)(ord >> 5) : p.res_words - 1;
                const int wb = wa + 1 < p.res_words ? wa + 1 : wa;
                const uint32_t rlo = p.res_sign[rt * rstride + (int64_t)wa * 16 + i];
                const uint32_t rhi = p.res_sign[rt * rstride + (int64_t)wb * 16 + i];
                uint32_t o[4];
                residual_chunk(d.m, __builtin_amdgcn_alignbit(rhi, rlo, ord & 31u), ar2, sel, o);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(o), as_half8(xs4), acc, 0, 0, 0);
            }
        }
        return acc;
    };

    // The R row tiles are taken in phases of PHT (a multiple of 3 unless it is R itself): the wavefronts stream
    // PHT tiles each, the workgroup adds the partial products in a fixed order and stores them.  Three tiles are
    // in flight per wavefront; a fetch past the last tile re-reads that tile, which keeps the number of loads
    // between a fetch and its wait the same on every path.
    for (int ph = 0; ph < R; ph += PHT) {
        const int ph0 = r0 + ph;
        const int ph1 = ph0 + PHT < r1 ? ph0 + PHT : r1;
        if (active) {
            // consumer side of the three tile buffers: the (visit, row tile) of the next product, in the producer's
            // order.  The first visit stores a row tile's product, the others add theirs to it (LDS adds: the sum over
            // the visits is taken in visit order, whatever the launch shape of other layers).  A step past the phase's
            // last product only keeps the fetches going.
            const int cn = ph1 - ph0;
            int ci = 0, cv = cn > 0 ? 0 : V;
            auto step = [&](Tile& t) {
                wait24_main<2 * L + (HAS_RES ? LRES24 : 0)>(t);
                if (cv < V) {
                    if (sb + cv * SPS < p.nsb) {
                        if (MULTI && ci == 0) visit_setup(cv);
                        product(t, ph0 + ci, ci);
                        if (MULTI && HAS_RES && (nch0 > 2 || nch1 > 2)) acc += extra_records(ph0 + ci, cv);
                        if (!MULTI || cv == 0) store_partial(ci);
                        else add_partial(ci);
                    }
                    if (++ci == cn) { ci = 0; ++cv; }
                }
                fetch_next(t);
            };
            while (cv < V) {
                step(t0);
                step(t1);
                step(t2);
            }
            if (!MULTI && HAS_RES && (nch0 > 2 || nch1 > 2))
                for (int rt = ph0; rt < ph1; rt++) {
                    const float4_t e = extra_records(rt, 0);
                    float* dst = part + ((rt - ph0) * 256 + lane);
#pragma unroll
                    for (int v = 0; v < 4; v++) dst[64 * v] += e[v];
                }
        }
        __syncthreads();
        // outputs of this phase: (slot, b, row in tile), consecutive threads on consecutive rows
        const int total = (ph1 > ph0 ? ph1 - ph0 : 0) * B * 16;
        for (int o = threadIdx.x; o < total; o += nthr) {
            const int r16 = o & 15, j = div_b(o >> 4), b = (o >> 4) - j * B;
            const int l = b + 16 * (r16 >> 2), v = r16 & 3;
            const char* src = lds_base + PART_OFF + (j * 256 + 64 * v + l) * 4;
            float t[8];
#pragma unroll
            for (int w = 0; w < 8; w++) t[w] = w < Wa ? *reinterpret_cast<const float*>(src + (int64_t)w * WREG) : 0.0f;   // fixed order of adds
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < 8; w++) s += t[w];
            const int row = (ph0 + j) * 16 + r16;
            if (S == 1) store_y(row, b, s);
            else __hip_atomic_store(ws_part + ((int64_t)ks * 16 + b) * n16 + row, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        if (ph + PHT < R) __syncthreads();           // the next phase overwrites the partial products
    }
    if (active) {
        wait24<0>(t0);                               // drain: no load may still target a register that is reused
        wait24<0>(t1);
        wait24<0>(t2);
    }
    if (S == 1) return;

    // ---- several column splits: the partial sums are in the workspace [split][16][n16]; take a ticket.  They are
    //      written and read with agent-scope accesses, so no cache write-back or invalidate is needed: the stores
    //      have completed (vmcnt = 0, then the barrier) before thread 0 takes the ticket, and the last arrival
    //      issues its loads after it has seen the ticket. ----
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) ticket = atomicInc(ws_count + gr, (uint32_t)(S - 1));    // wraps to 0 after S arrivals
    __syncthreads();
    if (ticket != (uint32_t)(S - 1)) return;
    const int total = (r1 - r0) * 16 * B;
    for (int o = threadIdx.x; o < total; o += nthr) {
        const int r16 = o & 15, tb = div_b(o >> 4), b = (o >> 4) - tb * B;
        const int row = (r0 + tb) * 16 + r16;
        float s = 0.0f;
        for (int c0 = 0; c0 < S; c0 += 4) {
            float t[4];
#pragma unroll
            for (int u = 0; u < 4; u++)
                t[u] = c0 + u < S ? __hip_atomic_load(ws_part + ((int64_t)(c0 + u) * 16 + b) * n16 + row, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.0f;
#pragma unroll
            for (int u = 0; u < 4; u++) s += t[u];
        }
        store_y(row, b, s);
    }
}

// The launch: workgroup b belongs to the layer whose range of workgroups holds b and runs that layer's variant of
// the body.  Every variant fits two wavefronts per SIMD, so putting them into one kernel costs no occupancy.
__global__ __launch_bounds__(512) void gemv24_group_kernel(const Gemv24Group a) {
    extern __shared__ __attribute__((aligned(16))) char dyn24[];
    int li = 0;
    for (int l = 1; l < a.n_layers; l++)
        if ((int)blockIdx.x >= a.l[l].block0) li = l;
    li = __builtin_amdgcn_readfirstlane(li);
    // the descriptor comes out of the kernel-argument segment with scalar loads (indexing the by-value argument would
    // make a private copy of it, and the plane pointers must sit in scalar registers)
    typedef const __attribute__((address_space(4))) char* kernarg_ptr;
    const kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    Gemv24Layer d;
    __builtin_memcpy(&d, ka + offsetof(Gemv24Group, l) + (size_t)li * sizeof(Gemv24Layer), sizeof(Gemv24Layer));
    const int local = (int)blockIdx.x - d.block0;
    const int ks = local / d.G, gr = local - ks * d.G;
    switch (d.variant) {
#define STB24_CASE(MODE, RES, MULTI) case (MODE | (RES ? 8 : 0) | (MULTI ? 16 : 0)): gemv24_body<MODE, RES, MULTI>(d, a.B, a.y_fp32, gr, ks, dyn24); break;
        STB24_CASE(2, false, false) STB24_CASE(2, true, false) STB24_CASE(2, false, true) STB24_CASE(2, true, true)
        STB24_CASE(4, false, false) STB24_CASE(4, true, false) STB24_CASE(4, false, true) STB24_CASE(4, true, true)
        STB24_CASE(6, false, false) STB24_CASE(6, true, false) STB24_CASE(6, false, true) STB24_CASE(6, true, true)
#undef STB24_CASE
        default: break;
    }
}

int64_t round_up256(int64_t v) { return (v + 255) / 256 * 256; }
// Largest number of column splits the plan may choose for n_super superblocks (the workspace is sized for it).
int max_splits24(int n_super) { return (n_super + 1) / 2 + 3; }

}  // namespace

// The launch shape of gemv24_kernel for a layer of nrt row tiles and nsb superblocks at batch B (mode 2: sparse
// instruction, 4 / 6: dense): out = {S column splits, R row tiles per workgroup, SPS wavefronts per workgroup, V visits
// per wavefront, bytes of LDS per wavefront, offset of its records, offset of its partial tiles}.  Pure host
// arithmetic (the tests check its invariants over many shapes).  STB_EUNSUPPORTED when nothing fits.
// The index words of a whole 2:4 layer, written out as the meta index E of App. C ([n][k/16] uint16): the same
// index_word() that feeds the sparse matrix instruction above, one thread per (row, block, half of 64 columns).
namespace {
__global__ __launch_bounds__(256) void meta_index_kernel(TiledPlanes p, uint16_t* __restrict__ E) {
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (id >= (int64_t)p.n * p.nb * 2) return;
    const int half = (int)(id & 1), b = (int)((id >> 1) % p.nb), row = (int)((id >> 1) / p.nb);
    const int64_t tile = (int64_t)(row >> 4) * p.nsb + (b >> 2);
    const int lane = 16 * (b & 3) + (row & 15);
    const uint2 m = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(p.mask) + tile * 1024 + 512 * half + lane * 8);
    const uint32_t T0 = 0x09080404u, T1 = 0x0E0E0D0Cu, K7 = 0x07070707u;
    const uint32_t w0 = index_word(m.x, T0, T1, K7), w1 = index_word(m.y, T0, T1, K7);
    *reinterpret_cast<uint2*>(E + (int64_t)row * (p.k / 16) + b * 8 + half * 4) = make_uint2(w0, w1);
}
}  // namespace

extern "C" int stb_tiled_meta_index(const stb_layout_t* L, void* E, void* stream, int* hip_err) {
    const TiledPlanes p = make_tiled(L);
    const int64_t threads = (int64_t)p.n * p.nb * 2;
    hipLaunchKernelGGL(meta_index_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, (hipStream_t)stream, p, (uint16_t*)E);
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}

extern "C" int stb_tiled_gemv24_plan(int nrt, int nsb, int B, int mode, int max_splits, int cus, int* out) {
    if (nrt < 1 || nsb < 1 || B < 1 || B > 16 || (mode != 2 && mode != 4 && mode != 6) || cus < 1 || cus > 256 || !out) return STB_EUNSUPPORTED;
    const int64_t lds_max = LDS24 - (mode == 2 ? 0 : 32768);
    // Column splits of SPS <= 8 wavefronts; a wavefront takes V superblocks (V = 1: its own; V = 2 .. 8: it visits
    // them one after the other, each visit over all row tiles of a phase); a workgroup owns R row tiles.  Among the
    // shapes whose LDS fits, take the one with the lowest estimated time, in ns: per (row tile, superblock) product
    // ~750 on the sparse instruction, ~1000 on the dense one; ~800 per visit for taking its operands from LDS;
    // R * V products for each of the ceil(SPS / 4) wavefronts of a SIMD, times the rounds the grid needs on `cus`
    // compute units (256 for a layer that has the chip to itself; a layer's share of them when several layers run as
    // one launch); adding the column splits up through the workspace costs ~3000 plus ~90 per split and batch row.
    // Ties go to the fewest splits.
    // LDS of one wavefront: per visit the x rows (B rows and one of zeros, 1040 bytes each) and 16 records; the PHT
    // partial tiles lie on top of the x rows when there is one visit, behind everything otherwise.
    const int xbytes = (B < 16 ? B + 1 : 16) * 1040;
    int S = 0, R = 0, SPS = 0, V = 0, wreg = 0, rec_off = 0, part_off = 0;
    int64_t best_cost = 0;
    // stb_set_kernel_override can restrict the choice to a number of visits where such a shape exists: the tests use it,
    // because small layers never choose several visits themselves.
    const int asked = stb_kernel_override(1), asked_s = stb_kernel_override(3);
    const int v_only = asked >= 1 && asked <= MAXV24 && nsb >= asked ? asked : 0;
    const int s_only = asked_s >= 1 && asked_s <= max_splits && asked_s * (v_only ? v_only : 1) <= nsb ? asked_s : 0;
    for (int pass = 0; pass < 2 && S == 0; pass++)             // second pass: a forced shape that does not exist is ignored
    for (int v = 1; v <= MAXV24; v++) {
        if (pass == 0 && v_only && v != v_only) continue;
        for (int s = (nsb + 8 * v - 1) / (8 * v); s <= max_splits && s * v <= nsb; s++) {
            if (pass == 0 && s_only && s != s_only) continue;
            const int sps = (nsb + s * v - 1) / (s * v);
            if (sps > 8 || (s - 1) * sps * v >= nsb) continue;   // a split must own at least one superblock
            if ((s * v - 1) * sps >= nsb) continue;              // ... and so must the last visit of the last split
            const int groups = cus / s > 0 ? cus / s : 1;
            const int r = (nrt + groups - 1) / groups, g = (nrt + r - 1) / r;
            const int pht = r < PHASE24 ? r : PHASE24;
            int w, ro, po;
            if (v == 1) {
                const int ar = xbytes > pht * 1024 ? xbytes : pht * 1024;
                ro = ar; po = 0; w = ar + 768;
            } else {
                ro = v * xbytes; po = ro + v * 768; w = po + pht * 1024;
            }
            if ((int64_t)sps * w > lds_max) continue;
            const int phases = (r + pht - 1) / pht;
            // two wavefronts of a SIMD take turns at its issue port; a lone one leaves it idle while it waits (measured:
            // 1.45 times the time per product)
            const int64_t per_wave = (int64_t)(mode == 2 ? 750 : 1000) * r * v + (v > 1 ? (int64_t)800 * v * phases : 0);
            const int64_t per_simd = sps <= 4 ? per_wave * 29 / 20 : per_wave * ((sps + 3) / 4);
            const int64_t cost = per_simd * ((g * s + cus - 1) / cus) + (s > 1 ? 3000 + (int64_t)90 * s * B : 0);
            if (S == 0 || cost < best_cost) { best_cost = cost; S = s; R = r; SPS = sps; V = v; wreg = w; rec_off = ro; part_off = po; }
        }
    }
    if (S == 0) return STB_EUNSUPPORTED;
    out[0] = S; out[1] = R; out[2] = SPS; out[3] = V; out[4] = wreg; out[5] = rec_off; out[6] = part_off;
    return STB_OK;
}

// Plans and launches one kernel over n_layers tiled layouts (1 .. GROUP24_MAX) at the same batch; layer l reads xs[l],
// writes ys[l] and keeps the arrival counters of its column splits at counters[l] (4 bytes per row tile, zero before
// and after) and their partial sums at partials[l] (partial_bytes[l] bytes).  Returns STB_EUNSUPPORTED, and launches
// nothing, when a layout is not 2:4 / 4:8 / 6:8 or a staging area would not fit, so that the caller can fall back to
// the general kernel layer by layer.
extern "C" int stb_tiled_gemv24_group(int n_layers, const stb_layout_t* const* Ls, const void* const* xs, int B,
                                      void* const* ys, int y_fp32, void* const* counters, void* const* partials,
                                      const int64_t* partial_bytes, void* stream, int* hip_err) {
    if (n_layers < 1 || n_layers > GROUP24_MAX || B < 1 || B > 16) return STB_EUNSUPPORTED;
    Gemv24Group a;
    a.n_layers = n_layers; a.B = B; a.y_fp32 = y_fp32; a.pad = 0;
    const int xbytes = (B < 16 ? B + 1 : 16) * 1040;
    int blocks = 0, sps_max = 1;
    int64_t lds = 0;
    // every layer gets a share of the 256 compute units in proportion to its work, so that the layers of a launch run
    // side by side and end together instead of each being cut for the whole chip (work of a (row tile, superblock):
    // the vector instructions its product issues, as counted on the three kinds of layer)
    int64_t work[GROUP24_MAX], total_work = 0;
    for (int l = 0; l < n_layers; l++) {
        const bool sparse = Ls[l]->cfg.M == 4 && Ls[l]->cfg.N == 2;
        const int per_tile = sparse ? 314 : stb_tiled_slots(&Ls[l]->cfg) == 6 ? 560 : 378;
        work[l] = (int64_t)Ls[l]->n_row_tiles * Ls[l]->n_super * per_tile;
        total_work += work[l];
    }
    for (int l = 0; l < n_layers; l++) {
        const stb_layout_t* L = Ls[l];
        int cus = n_layers == 1 ? 256 : (int)((256 * work[l] + total_work / 2) / (total_work > 0 ? total_work : 1));
        cus = cus < 1 ? 1 : (cus > 256 ? 256 : cus);
        const int n8 = stb_tiled_slots(&L->cfg);          // slots per 8 columns in the planes
        if (n8 == 0) return STB_EUNSUPPORTED;
        const int mode = L->cfg.M == 4 && L->cfg.N == 2 ? 2 : n8;      // 2: sparse instruction; 4, 6: dense with the scatter table
        if (mode != 2 && mode != 4 && mode != 6) return STB_EUNSUPPORTED;
        Gemv24Layer& d = a.l[l];
        d.p = make_tiled(L);
        {
            // one scalar base for the streamed planes: every byte of them must lie within 4 GiB of the lowest plane
            // (an image laid out by stb_tiled_sizes does unless it is larger than that)
            const bool has_t = L->cfg.n_salient > 0;
            const uintptr_t at[6] = {(uintptr_t)L->mask, (uintptr_t)L->sign, (uintptr_t)L->region, (uintptr_t)L->scales,
                                     (uintptr_t)L->res_scale, has_t ? (uintptr_t)L->res_t : (uintptr_t)L->mask};
            const int64_t size[6] = {L->mask_bytes, L->sign_bytes, L->region_bytes, L->scales_bytes, L->res_scale_bytes,
                                     has_t ? L->res_t_bytes : 0};
            uintptr_t low = at[0];
            for (int i = 1; i < 6; i++) low = at[i] < low ? at[i] : low;
            uint32_t off[6];
            for (int i = 0; i < 6; i++) {
                if (size[i] < 0 || (uint64_t)(at[i] - low) + (uint64_t)size[i] > 0xFFFFFFFFull) return STB_EUNSUPPORTED;
                off[i] = (uint32_t)(at[i] - low);
            }
            d.image = (const char*)low;
            d.off_mask = off[0]; d.off_sign = off[1]; d.off_region = off[2]; d.off_scales = off[3];
            d.off_res_scale = off[4]; d.off_res_t = off[5];
        }
        int plan[7];
        if (stb_tiled_gemv24_plan(d.p.nrt, d.p.nsb, B, mode, max_splits24(d.p.nsb), cus, plan) != STB_OK) return STB_EUNSUPPORTED;
        d.S = plan[0]; d.R = plan[1]; d.SPS = plan[2]; d.V = plan[3]; d.WREG = plan[4]; d.REC_OFF = plan[5]; d.PART_OFF = plan[6];
        d.XS = xbytes;
        d.G = (d.p.nrt + d.R - 1) / d.R;
        d.PHT = d.R < PHASE24 ? d.R : PHASE24;
        d.block0 = blocks;
        d.variant = mode | (d.p.res_words > 0 ? 8 : 0) | (d.V > 1 ? 16 : 0);
        d.x = (const __half*)xs[l];
        d.y = ys[l];
        d.ws_count = nullptr; d.ws_part = nullptr;
        if (d.S > 1) {
            if (!counters[l] || !partials[l]) return STB_ENULL;
            if (partial_bytes[l] < (int64_t)d.S * 16 * 16 * d.p.nrt * 4) return STB_EINVAL;
            if ((uintptr_t)counters[l] % 4 || (uintptr_t)partials[l] % 256) return STB_EALIGN;
            d.ws_count = (uint32_t*)counters[l];
            d.ws_part = (float*)partials[l];
        }
        blocks += d.G * d.S;
        if (d.SPS > sps_max) sps_max = d.SPS;
        const int64_t need = LDS24_HEAD + (mode == 2 ? 0 : (int64_t)sizeof(ScatterLds)) + (int64_t)d.SPS * d.WREG;
        if (need > lds) lds = need;
    }
    for (int l = n_layers; l < GROUP24_MAX; l++) a.l[l] = a.l[0];
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        const hipError_t e = hipFuncSetAttribute((const void*)gemv24_group_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, LDS24 + LDS24_HEAD);
        if (e != hipSuccess) { *hip_err = (int)e; return STB_EHIP; }
        attr_set.store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(gemv24_group_kernel, dim3(blocks), dim3(64 * sps_max), (size_t)lds, (hipStream_t)stream, a);
    const hipError_t e = hipGetLastError();
    *hip_err = (int)e;
    return e == hipSuccess ? STB_OK : STB_EHIP;
}

extern "C" int stb_tiled_gemv24(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* workspace,
                                int64_t workspace_bytes, int64_t ws_part_off, int max_splits, void* stream, int* hip_err) {
    (void)max_splits;
    if (ws_part_off < 0) ws_part_off = round_up256(4 * (int64_t)L->n_row_tiles);
    if (ws_part_off % 256 || ws_part_off < 4 * (int64_t)L->n_row_tiles) return STB_EINVAL;
    if (workspace && (uintptr_t)workspace % 256) return STB_EALIGN;
    void* cnt = workspace;
    void* part = workspace ? (char*)workspace + ws_part_off : nullptr;
    const int64_t part_bytes = workspace && workspace_bytes > ws_part_off ? workspace_bytes - ws_part_off : 0;
    return stb_tiled_gemv24_group(1, &L, &x, B, &y, y_fp32, &cnt, &part, &part_bytes, stream, hip_err);
}
