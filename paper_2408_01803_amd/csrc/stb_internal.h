// Declarations shared by the host and device translation units of libstb (not part of the public ABI).
#ifndef STB_INTERNAL_H
#define STB_INTERNAL_H
#include "stb.h"

// Slots per 8 columns that the tiled order stores sign bits and group ids for: 4 for layers that keep 3 or 4 of 8
// columns (2:4, 4:8, 3:8), 6 for 5 or 6 of 8 (5:8, 6:8, 3:4); 0 for every other N:M (those stay on the row-major
// kernels).  With 3 or 5 kept columns one slot per group is padding: the kept columns are numbered as if the lowest
// pruned column of the group were kept too, and the slot of that phantom column is never read.
static inline int stb_tiled_slots(const stb_cfg_t* c) {
    if (c->M < 1 || (8 * c->N) % c->M != 0) return 0;
    const int n8 = 8 * c->N / c->M;
    return n8 == 3 || n8 == 4 ? 4 : (n8 == 5 || n8 == 6 ? 6 : 0);
}
static inline int stb_tiled_padded(const stb_cfg_t* c) {
    const int t8 = stb_tiled_slots(c);
    return t8 != 0 && 8 * c->N / c->M != t8;
}

#ifdef __cplusplus
extern "C" {
#endif
// The kernel choices forced by stb_set_kernel_override (stb_device.hip): which = 0 decode kernel (0 automatic,
// 1 thin wavefronts), 1 superblock visits per wavefront of the decode kernel (0 automatic, 1 .. 8), 2 prefill kernel
// (0 automatic, 1 dense 16x16x32, 2 dense 32x32x16, 3 sparse 16x16x64), 3 column splits of the decode kernel (0 automatic).
int stb_kernel_override(int which);

// STB_OK iff the size fields agree with the closed form for L->cfg and every required plane pointer is
// set and 16-byte aligned.
int stb_layout_check(const stb_layout_t* L);

// Kernels for the tiled device order (stb_fast.hip).  Each returns a stb_status and stores the HIP error
// code of a failed launch in *hip_err.  stb_tiled_supported: 1 iff the fast kernels cover this N:M.
int stb_tiled_supported(const stb_layout_t* L);
int stb_tiled_dequant(const stb_layout_t* L, float* out, void* stream, int* hip_err);
// The workspace holds the arrival counters of the column splits (4 bytes per row tile, at its start) and their partial
// sums at byte offset part_off (a multiple of 256, at least 4 * n_row_tiles; -1 = directly behind the counters).
int stb_tiled_gemv(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* workspace,
                   int64_t workspace_bytes, int64_t part_off, void* stream, int* hip_err);
// Scratch bytes of the tiled decode kernels for L's shape.
int64_t stb_tiled_gemv_workspace(int n_row_tiles, int n_super);
// Decode kernel with one fat wavefront per superblock (stb_gemv24.hip): 2:4 layouts on the sparse matrix-core
// instruction, 4:8 / 6:8 (and 3:4) on the dense one.  Returns STB_EUNSUPPORTED, without launching anything, when
// its staging areas would not fit: the caller then runs the older kernel.  max_splits bounds the number of column splits (the workspace is sized for that many).
int stb_tiled_gemv24(const stb_layout_t* L, const void* x, int B, void* y, int y_fp32, void* workspace,
                     int64_t workspace_bytes, int64_t part_off, int max_splits, void* stream, int* hip_err);
// One launch of that kernel over up to 8 layers at the same batch (B <= 16); see stb_gemv24.hip.
int stb_tiled_gemv24_group(int n_layers, const stb_layout_t* const* Ls, const void* const* xs, int B, void* const* ys,
                           int y_fp32, void* const* counters, void* const* partials, const int64_t* partial_bytes,
                           void* stream, int* hip_err);
// The launch shape stb_tiled_gemv24 takes for a layer that may use `cus` (1..256) compute units (host arithmetic only;
// out[7] = S, R, SPS, V, LDS bytes per wavefront, record offset, partial-tile offset).
int stb_tiled_gemv24_plan(int nrt, int nsb, int B, int mode, int max_splits, int cus, int* out);
// The meta index of a tiled 2:4 layout, made by the decode kernel's own index function (stb_gemv24.hip).
int stb_tiled_meta_index(const stb_layout_t* L, void* E, void* stream, int* hip_err);
// Prefill kernel for the tiled order (stb_gemm.hip) and its scratch size for T tokens.
int stb_tiled_gemm(const stb_layout_t* L, const void* X, int T, void* Y, int y_fp32, void* workspace,
                   int64_t workspace_bytes, void* stream, int* hip_err);
int64_t stb_tiled_gemm_workspace(const stb_layout_t* L, int T);
// Host: the derived tables of the tiled order (padded bitmap and prefix, table of salient columns, maxima) from the
// row-major bitmap and prefix; the output arrays hold tl->salmap_bytes, tl->salprefix_bytes, tl->saltab_bytes.
int stb_host_tiled_tables(const stb_layout_t* tl, const uint32_t* bitmap, const uint32_t* prefix, uint32_t* bitmap_out,
                          uint32_t* prefix_out, uint32_t* sal_tab_out, int* max_block, int* max_half);
// stb_tile with both images in device memory (stb_pack.hip); sets dst->max_sal_block / max_sal_half; waits for the stream.
int stb_tile_gpu(const stb_layout_t* src, stb_layout_t* dst, void* stream, int* hip_err);
// The packer on the GPU (stb_pack.hip): `out` is a checked row-major layout bound to device memory, the workspace holds
// stb_pack_gpu_workspace() bytes.  Waits for the stream before it returns.
int64_t stb_pack_gpu_workspace(const stb_cfg_t* cfg, int per_block);
int stb_pack_gpu(const float* W, const float* xnorm, const uint32_t* sal_bitmap, const stb_layout_t* out, int per_block,
                 void* workspace, void* stream, int* hip_err);
// The block loop of Alg. 1 with its float64 working copy kept by an accelerator (stb_host.cpp runs the loop,
// stb_pack.hip provides the three calls for a GPU): `start` receives the initial n x k copy, `fetch` writes the current
// values of block q's columns into the host copy (row stride k), `update` applies the compensation of block q from its
// error matrix E (n x 128).  Each returns a stb_status.
typedef struct {
    void* ctx;
    int (*start)(void* ctx, const double* Wd_host);
    int (*fetch)(void* ctx, int q, double* Wd_host);
    int (*update)(void* ctx, int q, const double* E_host);
} stb_obc_accel_t;
int stb_pack_obc_with(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                      stb_layout_t* out, int32_t n_threads, const stb_obc_accel_t* accel);
int64_t stb_pack_obc_gpu_workspace(const stb_cfg_t* cfg);
int stb_pack_obc_gpu(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap, stb_layout_t* out,
                     int32_t n_threads, void* workspace, void* stream, int* hip_err);
// Issue-rate probe of the matrix instructions the prefill kernels use (stb_gemm.hip); see stb_probe_mfma in stb.h.
int stb_tiled_probe_mfma(int kind, int valu, int steps, int n_workgroups, void* sink, void* stream, int* hip_err);
#ifdef __cplusplus
}
#endif
#endif
