/*
 * stb.h -- C ABI of the structured-binary (STBLLM) matrix-product library for AMD MI355X (gfx950).
 *
 * The library computes the inference-time product  y = x . W_hat^T  where W_hat is a structured-binary
 * weight matrix: every output row keeps exactly N of each M consecutive input weights (Sec. 3.1 "N:M
 * Sparsity"), a kept weight is a sign (Eq. 1-2) times one of three per-(row, 128-column block) fp16 scales
 * chosen by a 2-bit group id (Sec. 3.4 "Non-Salient Part", Alg. 2 "Trisection": dense / intermediate /
 * sparse region), and kept weights in salient columns carry a second, residual sign and scale
 * (Eq. 4, Alg. 2 "Res_Approx").
 *
 * Conventions for every function:
 *   - returns STB_OK (0) or a negative stb_status; never throws, never allocates device memory, and does not
 *     synchronise the stream -- except the packing calls whose description says that they wait for it
 *     (stb_pack_device, stb_tile_device, stb_pack_obc_hybrid: what their kernels find is their return value);
 *   - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory of the current
 *     device; the caller owns every buffer, before and after the call;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream); device work is only
 *     enqueued on it.
 *
 * Packed format ("STB1").  All planes are little-endian; bit b of byte c of a row <-> index 8c + b;
 * padding bits and bytes are zero.  The r-th kept weight of a row (its "slot", counted over the whole
 * row in ascending column order) is r = g*N + rank-inside-group for M-group g, because every group
 * keeps exactly N.
 *
 *   plane             shape / stride                          content
 *   mask              n rows x k/8 bytes                      bit j = weight j of the row is kept
 *   sign              n rows x sign_stride bytes              bit r = 1 iff kept weight r is >= 0  (1 -> +1, 0 -> -1)
 *   region            n rows x region_stride bytes            2-bit field r = group id of kept weight r:
 *                                                             0 dense, 1 intermediate, 2 sparse, 3 salient
 *   res_sign          n rows x n_salient_pad/8 bytes          bit u <-> u-th salient column (ascending):
 *                                                             1 iff the weight is kept there and its residual sign is +1
 *   scales            fp16 [n][k/128][4]                      {dense, intermediate, sparse, alpha_o}
 *   res_scale         fp16 [n][k/128]                         alpha_r
 *   sal_bitmap        k/32 uint32                             bit j = column j is salient
 *   sal_block_prefix  (k/128 + 1) uint32                      number of salient columns before each block
 *
 *   sign_stride   = round_up(k*N/(8M), 16),  region_stride = round_up(k*N/(4M), 16),
 *   n_salient_pad = round_up(n_salient, 128)
 *   total_bytes   = n*(k/8 + sign_stride + region_stride + n_salient_pad/8 + 10*k/128) + k/8 + 4*(k/128 + 1)
 *
 * Dequantised weight (what every kernel multiplies by, and what stb_dequant / stb_unpack write):
 *   not kept                 ->  0
 *   kept, id in {0,1,2}      ->  s * f32(scales[row][block][id])
 *   kept, id = 3             ->  f32( s * f32(alpha_o) + t * f32(alpha_r) )        one fp32 addition
 */
#ifndef STB_H
#define STB_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STB_BLOCK 128          /* columns per scale block */
#define STB_MAX_BATCH 32       /* largest B accepted by stb_gemv */
#define STB_PLANE_ALIGN 256    /* alignment of every plane inside one image */

typedef enum stb_status {
    STB_OK = 0,
    STB_EINVAL = -1,      /* bad configuration or argument (M not 4 or 8, N outside 1..M, k % 128 != 0, B outside 1..32, T < 1, layout fields that do not match the closed form, n_salient != popcount of the bitmap) */
    STB_ENULL = -2,       /* a required pointer is NULL */
    STB_EALIGN = -3,      /* a plane pointer is not 16-byte aligned */
    STB_ENONFINITE = -4,  /* NaN or Inf in W or xnorm, or xnorm < 0 */
    STB_EHIP = -5,        /* a HIP call failed; the HIP error code is returned by stb_last_hip_error() */
    STB_EUNSUPPORTED = -6, /* valid request that this build has no kernel for */
    STB_ETOOBIG = -7      /* stb_gemv_static: the problem needs more scratch than the library's static device array holds */
} stb_status;

/* Problem description. block must be 128. region_mode: 0 = break-point search of Alg. 2
 * "NonSalientAwareQuant" (160 candidates, p2 = 2*p1), 1 = tertile split of the kept non-salient
 * magnitudes of each block. n_salient = number of set bits of the salient-column bitmap. */
typedef struct stb_cfg {
    int32_t n_out;        /* n: rows of W = output features */
    int32_t k_in;         /* k: columns of W = input features, multiple of 128 */
    int32_t N, M;         /* keep N of every M consecutive input weights; M in {4, 8}, 1 <= N <= M */
    int32_t block;        /* 128 */
    int32_t n_salient;    /* S */
    int32_t region_mode;  /* 0 | 1, only read by stb_pack */
} stb_cfg_t;

/* Sizes, offsets and plane pointers of one packed matrix.  stb_layout_sizes / stb_tiled_sizes fill
 * everything except the pointers; stb_layout_bind derives the pointers from one base address (host or
 * device).  A caller may also set the plane pointers by hand (each 16-byte aligned).
 *
 * kind = STB_KIND_ROWMAJOR: the planes exactly as described above ("STB1").
 * kind = STB_KIND_TILED: the device order read by the fast kernels, a byte permutation of STB1 plus zero
 * padding (3:8 and 5:8: a bit permutation, see "slots" below).  Rows are grouped in tiles of 16 and 128-column blocks in groups of 4 ("superblock", 512
 * columns); a tile record holds one 64-lane wavefront's operands, lane = 16*(block % 4) + (row % 16):
 *   mask      [row_tile][super][half][lane][8 bytes]    the mask bytes of (row, block), columns 64*half .. 64*half+63
 *   sign      [row_tile][super][lane][sign_stride]      sign bits of the block's 128*N/M kept weights
 *   region    [row_tile][super][lane][region_stride]    their 2-bit ids
 *             sign / region are cut into two halves like mask ([row_tile][super][half][lane][stride/2], the
 *             kept weights of columns 64*half ..) when their stride is a multiple of 8 bytes, so that each
 *             half is a whole number of 32-bit words (2:4 and 4:8: both; 6:8: region only)
 *             slots: layers that keep 3 or 5 of 8 columns are stored in the records of 4:8 / 6:8 (sign_stride 8 /
 *             12, region_stride 16 / 24), one slot per group of 8 columns left zero: the kept columns of a
 *             group take the slots they would have if the group's lowest pruned column were kept as well,
 *             so that the kernels of 4:8 and 6:8 read them unchanged (the mask byte tells them which slot is
 *             the unused one).  The tiled image of such a layer is 3.25 (5:8) or 2.25 (3:8) bits per weight
 *             of mask, sign and id planes, against 2.875 and 2.125 in STB1.
 *   scales    [row_tile][super][lane][4] fp16, res_scale [row_tile][super][lane] fp16
 *   res_sign  [row_tile][word][row % 16] uint32: the STB1 row strings cut into 32-bit words and transposed
 *             inside each row tile (res_stride / 4 words per row)
 *   sal_bitmap / sal_block_prefix as in STB1, padded to whole superblocks
 *   sal_tab   [block][half][sal_chunks] records of 12 uint32, a derived table like sal_block_prefix.  A block
 *             is cut in two halves of 64 columns; record c of a half covers entries 8c .. 8c+7 of the
 *             ascending list of the half's salient columns (entry e at column p_e of the block, 0..127):
 *               [0] [1]   v_perm_b32 selectors that gather, out of the half's 8 mask bytes, the byte holding
 *                         entries 0..3 / 4..7 ((p_e >> 3) & 7; 0x0C = zero if the entry does not exist)
 *               [2] [3]   one byte per entry: 1 << (p_e & 7), 0 if the entry does not exist
 *               [4]       index of the record's first entry among all salient columns of the layer (= its
 *                         bit in a res_sign row)
 *               [5]       largest number of records any of the four blocks of this superblock needs in this
 *                         half
 *               [6]       number of entries in this record (0..8)        [7] zero
 *               [8..11]   uint16 p_e of the 8 entries, 0xFFFF if the entry does not exist
 *   res_t     [row_tile][super][lane] uint32, a derived copy of res_sign bits in lane-record order (the decode kernel
 *             reads one word per tile and lane instead of four scattered ones): bit e (e < 16) = the res_sign bit of
 *             the e-th salient column of the half of columns 0..63 of (row, block), bit 16 + e = the same for the
 *             half of columns 64..127; bits of entries that do not exist are 0.  Entries past the 16th of a half
 *             are read from res_sign.
 * Rows >= n and blocks >= k/128 of the padding are all-zero (nothing kept). */
#define STB_KIND_ROWMAJOR 0
#define STB_KIND_TILED 1

typedef struct stb_layout {
    stb_cfg_t cfg;
    int32_t n_salient_pad;     /* round_up(S, 128), 0 if S = 0 */
    int32_t n_blocks;          /* k / 128 */
    int32_t kind;              /* STB_KIND_ROWMAJOR | STB_KIND_TILED */
    int32_t n_row_tiles;       /* tiled: ceil(n / 16), else 0 */
    int32_t n_super;           /* tiled: ceil(n_blocks / 4), else 0 */
    int32_t sal_chunks;        /* tiled: records per half block in sal_tab = ceil(min(S, 64) / 8), else 0 */
    int32_t max_sal_block;     /* tiled: largest number of salient columns in one block (set by stb_tile) */
    int32_t max_sal_half;      /* tiled: largest number of salient columns in one half block of 64 columns (set by stb_tile) */
    int64_t mask_stride, sign_stride, region_stride, res_stride;   /* bytes per row (row-major) or per lane record (tiled; res_stride stays per row) */
    int64_t mask_bytes, sign_bytes, region_bytes, res_bytes,
            scales_bytes, res_scale_bytes, salmap_bytes, salprefix_bytes, saltab_bytes;
    int64_t total_bytes;       /* sum of the planes of this layout; for STB_KIND_ROWMAJOR these are the "packed bytes" that throughput is quoted on */
    int64_t off_mask, off_sign, off_region, off_res, off_scales, off_res_scale,
            off_salmap, off_salprefix, off_saltab;                 /* offsets inside one image */
    int64_t image_bytes;       /* size of one allocation holding all planes at the offsets above */
    uint32_t *mask, *sign, *region, *res_sign, *sal_bitmap, *sal_block_prefix, *sal_tab;
    uint16_t *scales, *res_scale;
    int64_t res_t_bytes, off_res_t;   /* tiled, S > 0: the plane res_t (below), else 0 */
    uint32_t *res_t;
} stb_layout_t;

/* Closed-form sizes and image offsets for `cfg` (Sec. 3.4 "Average Bits" gives the payload: N/M sign bits
 * per weight, a second one on kept salient weights, 2-bit ids).  Pointers in `out` are set to NULL.
 * Errors: STB_ENULL, STB_EINVAL. */
int stb_layout_sizes(const stb_cfg_t* cfg, stb_layout_t* out);

/* Point the eight plane pointers at base + off_*.  `base` is host or device memory of at least
 * image_bytes bytes, 256-byte aligned.  Errors: STB_ENULL, STB_EALIGN. */
int stb_layout_bind(stb_layout_t* layout, void* base);

/* Sizes and image offsets of the tiled device order for `cfg` (kind = STB_KIND_TILED).  `n_salient` columns
 * may all fall into one half block, so sal_chunks is sized for that worst case.
 * Errors: STB_ENULL, STB_EINVAL. */
int stb_tiled_sizes(const stb_cfg_t* cfg, stb_layout_t* out);

/* Host-side permutation STB1 -> tiled order (and back).  Both layouts must describe the same cfg and
 * be bound to caller-allocated host memory; every byte of the destination is written.  stb_tile also fills
 * dst->max_sal_block and dst->max_sal_half.  stb_untile(stb_tile(x)) == x bit for bit.
 * Errors: STB_ENULL, STB_EINVAL (kind or cfg mismatch; at 3:8 and 5:8 also a group of 8 columns whose mask byte
 * does not keep exactly N), STB_EALIGN. */
int stb_tile(const stb_layout_t* src_rowmajor, stb_layout_t* dst_tiled);
int stb_untile(const stb_layout_t* src_tiled, stb_layout_t* dst_rowmajor);

/* stb_tile with both images in device memory (say, the output of stb_pack_device): same bytes as stb_tile, and
 * dst->max_sal_block / max_sal_half are set in the caller's struct.  The small tables that depend on the salient
 * bitmap alone are made on the host (the bitmap is copied there and the tables back), the planes are permuted by
 * kernels; the call waits for `stream` before it returns.  Errors: as stb_tile, and STB_EHIP. */
int stb_tile_device(const stb_layout_t* src_rowmajor_dev, stb_layout_t* dst_tiled_dev, void* stream);

/* Structured binarisation of one linear layer on the host (Alg. 1 without its Hessian steps: the salient
 * column set is an input and there is no error compensation between blocks; stb_pack_obc has them):
 *   Standardized Importance over the whole layer (Eq. 3) -> N:M mask (ties keep the lower column) ->
 *   per 128-column block: residual binarisation of kept salient weights per row (Eq. 4), break points
 *   over the kept non-salient weights of all rows (Alg. 2 "NonSalientAwareQuant", or tertiles), one scale
 *   per (row, block, region) (Eq. 6) -> bit planes.
 * W: host, n x k row-major fp32.  xnorm: host, k values >= 0 (L2 norm of each input feature).
 * sal_bitmap: host, k/32 words.  out: layout from stb_layout_sizes bound to caller-allocated host memory;
 * every byte of every plane is written.  n_threads <= 0 picks the hardware concurrency.
 * The result is bit-for-bit reproducible and independent of n_threads.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_ENONFINITE. */
int stb_pack(const float* W, const float* xnorm, const uint32_t* sal_bitmap, stb_layout_t* out,
             int32_t n_threads);

/* The factor H^c that Alg. 1 takes ("H = 2 X X^T", "H^c = Cholesky((H + lambda I)^-1)") from calibration
 * activations: H = 2 X^T X over the k input features, Hc = the upper-triangular factor with Hc^T Hc = (H + lambda I)^-1
 * (the triangle whose entries right of a diagonal block the compensation step reads), computed as the inverse of the
 * upper-triangular R with R R^T = H + lambda I.  Float64 throughout, every entry one sum in a fixed order: reproducible
 * bit for bit and independent of n_threads; it agrees with a LAPACK inverse-then-Cholesky to rounding, not bit for bit.
 * X: host, r x k row-major fp32 (r samples).  lambda >= 0.  Hc: host, k x k row-major float64, fully overwritten
 * (zeros below the diagonal); it serves as the working array: the only other storage is a float64 copy of X.  xnorm (may be NULL):
 * host, k floats, the L2 norm of each feature over the samples (the xnorm of stb_pack and stb_salient_columns).
 * Cost: (r + k / 3) k^2 multiply-adds on the host.
 * Errors: STB_ENULL, STB_EINVAL, STB_ENONFINITE (NaN/Inf in X, or H + lambda I not positive definite in floating
 * point: more samples or a larger lambda are needed). */
int stb_hessian_factor(const float* X, int32_t r, int32_t k, double lambda, double* Hc, float* xnorm,
                       int32_t n_threads);

/* Alg. 1 with its block loop: blocks of 128 columns from left to right, on a float64 working copy of W,
 *   Standardized Importance (Eq. 3) of the block's slice alone (row sums, column sums, mean and deviation over the
 *   n x 128 slice) -> N:M mask -> residual binarisation, break points and scales as in stb_pack -> B, the block as
 *   inference dequantises it -> E = (W_block - B) with column j divided by Hc[j][j] ->
 *   W[:, later columns] -= E . Hc[block rows, later columns], each output's 128 terms added in ascending column
 *   order, one multiplication and one addition per term.
 * Hc: host, k x k row-major float64, the upper-triangular Cholesky factor of (H + lambda I)^-1 with H = 2 X^T X
 * over the calibration activations (Hc^T Hc = (H + lambda I)^-1); only the diagonal and the part right of each
 * diagonal block are read.  Hc == NULL skips the compensation: the result is stb_pack with the per-block
 * Standardized Importance of Alg. 1 in place of the whole-layer one.  The salient column set is an input.
 * All other arguments, the output and its reproducibility are those of stb_pack.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_ENONFINITE (also a zero, NaN or Inf on Hc's diagonal). */
int stb_pack_obc(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                 stb_layout_t* out, int32_t n_threads);

/* stb_pack_obc with the compensation step on the GPU (the rest of the block loop stays on the host): the float64
 * working copy of W and the factor live in the device workspace, the host quantises block after block, sends the
 * block's error matrix E (n x 128) and fetches the next block's columns; the update
 *   W[:, later columns] -= E . Hc[block rows, later columns]
 * runs as a kernel with the arithmetic stb_pack_obc states (per output the 128 terms in ascending column order, one
 * multiplication and one addition per term), so the packed bytes equal those of stb_pack_obc bit for bit.  The
 * update is n k^2 / 2 float64 multiply-adds in all, the largest part of the block loop's arithmetic.
 * W, Hc, xnorm, sal_bitmap, out: host, as for stb_pack_obc (Hc == NULL: the call is stb_pack_obc without a factor and
 * the workspace is not used).  workspace: device, 256-byte aligned, stb_pack_obc_hybrid_workspace_bytes(cfg) bytes
 * (8 n k + 8 k^2 + 1024 n, rounded up).  The call copies between host and device on `stream` and waits for it.
 * Errors: as stb_pack_obc, plus STB_EHIP, STB_EUNSUPPORTED (more than 524280 rows). */
int64_t stb_pack_obc_hybrid_workspace_bytes(const stb_cfg_t* cfg);
int stb_pack_obc_hybrid(const float* W, const double* Hc, const float* xnorm, const uint32_t* sal_bitmap,
                        stb_layout_t* out, int32_t n_threads, void* workspace, int64_t workspace_bytes, void* stream);

/* stb_pack on the GPU (Eq. 1-6, Sec. 3.1, Alg. 2 as in stb_pack): weights, feature norms and the salient bitmap in
 * device memory in, the STB1 planes in device memory out, bit for bit what stb_pack writes for the same inputs.  Every
 * float64 sum is taken in the order stb_pack takes it (a row's columns from left to right, the rows from the top
 * down, one thread per sum); rows, columns, blocks and the break-point candidates of Alg. 2 run side by side.
 * W: device, n x k row-major fp32, 16-byte aligned.  xnorm: device, k values >= 0.  sal_bitmap: device, k/32 words.
 * out: row-major layout (stb_layout_sizes) bound to device memory; every byte of every plane is written.
 * si_per_block: 0 = Standardized Importance over the whole layer (Eq. 3, as stb_pack); 1 = over each 128-column slice
 * (as Alg. 1 calls it; the result is that of stb_pack_obc without a factor).
 * workspace: device, at least stb_pack_device_workspace_bytes() bytes (< 0: a stb_status), 256-byte aligned.
 * The call enqueues its kernels on `stream` and waits for them: what the kernels find (a NaN, a bitmap that does not
 * hold cfg.n_salient columns) comes back as the status.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_ENONFINITE, STB_EHIP. */
int64_t stb_pack_device_workspace_bytes(const stb_cfg_t* cfg, int32_t si_per_block);
int stb_pack_device(const float* W, const float* xnorm, const uint32_t* sal_bitmap, const stb_layout_t* out,
                    int32_t si_per_block, void* workspace, int64_t workspace_bytes, void* stream);

/* Layer-wise N:M assignment (Sec. 3.3).  stb_layer_l2_norm: omega = the L2 norm of `count` host fp32 weights
 * (float64, sequential).  stb_layer_nm_assignment: for layers with norms omega[0 .. n_layers), alpha_i = omega_i /
 * sum(omega) (1 / n_layers each if the sum is 0) and N_i / M = alpha_i + (1 - alpha_i) * r_target; N_out[i] is the
 * nearest integer to M times that ratio (a half rounds up), kept inside 1..M (the paper gives the ratio, not the
 * rounding).  r_target in [0, 1].  Errors: STB_ENULL, STB_EINVAL, STB_ENONFINITE (NaN/Inf weight or norm, negative norm). */
int stb_layer_l2_norm(const float* W, int64_t count, double* omega);
int stb_layer_nm_assignment(const double* omega, int32_t n_layers, double r_target, int32_t M, int32_t* N_out);

/* The salient columns of a layer (Alg. 2 "Salient", called once per 128-column block as in Alg. 1), for use as the
 * sal_bitmap of stb_pack.  The Hessian of Alg. 1 (H = 2 X X^T, H^c = Cholesky((H + lambda I)^-1)) is taken as its
 * diagonal, which the feature norms give: the salient matrix is S_ij = w_ij^2 (2 xnorm_j^2 + lambda).  Per block:
 * candidates = the max_per_block columns with the largest column sums of S (ties: the lower column first); for
 * i = 1 .. max_per_block the first i candidates are binarised together and all other columns of the block together
 * (Eq. 1, one scale per row and group); the i with the smallest squared error is kept (the first such i).
 * W: host, n x k row-major fp32.  xnorm: host, k values >= 0.  lambda >= 0.  max_per_block in 0..128 (the paper
 * does not give the length of its top-k list).  sal_bitmap: host, k/32 words, fully overwritten.  n_selected
 * (may be NULL): the number of salient columns.  Sums are float64 and sequential: the result is reproducible bit
 * for bit.  Errors: STB_ENULL, STB_EINVAL, STB_ENONFINITE. */
int stb_salient_columns(const float* W, int32_t n, int32_t k, const float* xnorm, double lambda,
                        int32_t max_per_block, uint32_t* sal_bitmap, int32_t* n_selected);

/* The same selection with the factor of Alg. 1 itself, as Alg. 2 writes it: S_ij = w_ij^2 / (Hc[j][j])^2, the square of
 * the diagonal of the factor's diagonal block.  Hc: host, k x k row-major float64 (from stb_hessian_factor, say; only
 * its diagonal is read).  Everything else as stb_salient_columns.
 * Errors: STB_ENULL, STB_EINVAL, STB_ENONFINITE (also a zero, NaN or Inf on Hc's diagonal). */
int stb_salient_columns_hc(const float* W, int32_t n, int32_t k, const double* Hc, int32_t max_per_block,
                           uint32_t* sal_bitmap, int32_t* n_selected);

/* Host dequantisation of a packed matrix into dense fp32 (definition in the header comment).
 * host: layout bound to host memory.  W_hat: host, n x k row-major, fully overwritten.
 * Errors: STB_ENULL, STB_EINVAL (including a mask row that does not keep k*N/M weights). */
int stb_unpack(const stb_layout_t* host, float* W_hat);

/* The 2:4 group code of App. C ("D = A(E) x B + C": six bits per group of four columns), out of and into the mask
 * and sign planes of a row-major 2:4 layout on the host.
 *   E: host, [n][k/16] uint16, the meta index: the nibble at bits 4*(g % 4) of E[i][g / 4] belongs to group g of row
 *      i (columns 4g .. 4g+3); its low two bits are the position (0..3) of the first kept weight of the group, its
 *      high two bits the position of the second one (larger than the first).  The paper fixes the sizes (four index
 *      bits per group, a uint16 per four groups) but not the bit order: this is the order in which the structured-
 *      sparse matrix instructions take their index operand, and the word the 2:4 kernels here build in registers.
 *   V: host, [n][k/16] uint8, the values: bit 2*(g % 4) + j of V[i][g / 4] is the sign of the j-th kept weight of
 *      group g, 1 -> +1, 0 -> -1 (byte for byte the payload of the sign plane).
 * stb_code24_export reads the planes and writes every element of E and V; stb_code24_import checks all of E first
 * and then overwrites the mask and sign planes (padding bytes zero), leaving every other plane as it is.
 * Errors: STB_ENULL, STB_EINVAL (tiled kind; a group that does not keep exactly two weights; an index nibble
 * whose positions are equal or descending), STB_EALIGN, STB_EUNSUPPORTED (N:M other than 2:4). */
int stb_code24_export(const stb_layout_t* host, uint16_t* E, uint8_t* V);
int stb_code24_import(stb_layout_t* host, const uint16_t* E, const uint8_t* V);

/* The meta index E (as in stb_code24_export) of a tiled 2:4 layout in device memory, written by a HIP kernel with
 * the index function of the 2:4 kernels: what the structured-sparse matrix instruction is fed, laid out as the
 * paper's uint16 words.  E_dev: device, [n][k/16] uint16, 16-byte aligned, fully overwritten.  Asynchronous on
 * `stream`.  A padding group (nothing kept) never occurs inside [n][k]; a group that does not keep exactly two
 * weights gives an unspecified nibble (stb_code24_export checks, this does not).
 * Errors: STB_ENULL, STB_EINVAL (row-major kind), STB_EALIGN, STB_EUNSUPPORTED (N:M other than 2:4), STB_EHIP. */
int stb_code24_index(const stb_layout_t* dev, uint16_t* E_dev, void* stream);

/* Device dequantisation: same result as stb_unpack, bit for bit, written by a HIP kernel.
 * dev: layout (either kind) bound to device memory holding a copy of the packed image.  W_hat_dev: device,
 * n x k fp32.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_EHIP. */
int stb_dequant(const stb_layout_t* dev, float* W_hat_dev, void* stream);

/* Decode-time product (memory-bound regime, App. C "Theory Analysis": small N = batch):
 *   y[b][i] = sum_j x[b][j] * W_hat[i][j],  b < B <= 32.
 * dev: either kind; the tiled kind runs the wavefront-tiled matrix-core kernel (N:M in {2:4, 3:8, 4:8, 5:8, 6:8, 3:4}; it
 * assumes the stored scales are >= 0, as stb_pack writes them), the row-major kind a generic kernel for any
 * N:M.
 * x: device fp16 [B][k] row-major.  y: device [B][n] row-major, fp16 (y_fp32 = 0) or fp32 (y_fp32 = 1),
 * fully overwritten.  Accumulation is fp32.
 * workspace: device scratch of at least stb_gemv_workspace_bytes() bytes, 256-byte aligned (may be NULL when
 * that is 0).  It holds the partial sums and arrival counters of the column splits (used by most layers
 * with k > 4096; for smaller k the launcher may still split columns to balance the grid).  The
 * counters (its first 4 * ceil(n / 16) bytes) must be zero before the first call that uses the buffer; every
 * call leaves them zero.  Calls that share a workspace must not overlap in time.
 * B > 16: the decode kernel takes 16 rows of x per pass.  A tiled layer other than 2:4 runs instead as one pass of
 * the prefill kernel (the form of stb_gemm for up to 64 tokens: the weights are expanded once for all rows) when the
 * workspace is as large as stb_gemv_workspace_bytes(cfg, B) asks; with a smaller one (sized for B <= 16, say), on 2:4
 * layers and under stb_set_kernel_override it runs as two passes of the decode kernel.  Both ways meet the same
 * error bound; their results differ within rounding.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_EHIP. */
int stb_gemv(const stb_layout_t* dev, const void* x, int32_t B, void* y, int32_t y_fp32,
             void* workspace, int64_t workspace_bytes, void* stream);

/* stb_gemv for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same product, the decode kernels and (for B <= 16, 2:4 layers and any workspace
 * too small for stb_gemv's one-pass form) the same bits in y as stb_gemv -- B > 16 always runs as two passes here -- but the scratch of
 * the column splits lives in a device array that is part of the library's code object (STB_GEMV_STATIC_SCRATCH_BYTES
 * bytes on every GPU the library runs on, held until the process ends); the call allocates nothing and needs no set-up
 * call (the array's address on the current device is looked up at the first call there).
 * Limits: ceil(n / 16) <= 16384 row tiles, and 65536 + splits * 1024 * ceil(n / 16) bytes <= the array, where splits is
 * the number of column splits the launcher takes for the shape (1 for k <= 4096; the 70B-shaped layers of the
 * workloads need at most 4 MB); beyond that the call returns STB_ETOOBIG and launches nothing.
 * Every call on one GPU uses the same array: calls that overlap in time on one GPU (two streams, two threads) race.
 * The arrival counters at the start of the array are zero when the library is loaded and every call leaves them zero.
 * Errors: as stb_gemv, plus STB_ETOOBIG and STB_EUNSUPPORTED (device ordinal >= 64). */
#define STB_GEMV_STATIC_SCRATCH_BYTES (8 * 1024 * 1024)
int stb_gemv_static(const stb_layout_t* dev, const void* x, int32_t B, void* y, int32_t y_fp32, void* stream);

/* Scratch bytes stb_gemv needs for (cfg, B), for either kind of layout; negative stb_status on a bad
 * argument.  For B > 16 on N:M other than 2:4 this includes the scratch of the one-pass form (see stb_gemv), sized
 * for any placement of the salient columns. */
int64_t stb_gemv_workspace_bytes(const stb_cfg_t* cfg, int32_t B);

/* Several independent layers at the same B as one launch: the matrices of a decoder layer that share their input
 * (q, k and v; gate and up) or any other list.  Decode is bound by memory traffic (App. C "Theory Analysis", small
 * N), and a single layer of a few tens of MB is over before the memory system has ramped up; one launch over the
 * list streams all of them back to back.  Tiled layouts at 2:4, 3:8, 4:8, 5:8 or 6:8 run as one kernel per 8 layers whose grid is
 * the layers' grids one after the other (batches above 16 in two passes); any other list runs layer after layer.
 * dev, x, y: host arrays of n_layers pointers (x[l], y[l] as in stb_gemv; entries of x may be equal).  Every layer of
 * a launch gets a share of the compute units in proportion to its size, so its partial sums may be added in another
 * order than in a call of stb_gemv: results are reproducible bit for bit from call to call, within rounding of those
 * of single calls.
 * workspace: device scratch of at least stb_gemv_batched_workspace_bytes() bytes, 256-byte aligned; layer l owns its
 * own slice (the slices follow each other in the order of the list, each as large as round_up(stb_gemv_workspace_bytes
 * of the layer at a batch of 16 or less, 256)), whose first 4 * ceil(n / 16) bytes must be zero before the first call and are left zero.
 * Calls that share a workspace must not overlap in time.
 * Errors: as stb_gemv; nothing is launched unless every layer's arguments are valid. */
int stb_gemv_batched(int32_t n_layers, const stb_layout_t* const* dev, const void* const* x, int32_t B,
                     void* const* y, int32_t y_fp32, void* workspace, int64_t workspace_bytes, void* stream);

/* Scratch bytes stb_gemv_batched needs for the layers described by cfgs[0 .. n_layers) at batch B; negative
 * stb_status on a bad argument. */
int64_t stb_gemv_batched_workspace_bytes(int32_t n_layers, const stb_cfg_t* const* cfgs, int32_t B);

/* Prefill-time product (compute-bound regime, App. C: large N = batch x sequence length):
 *   Y[t][i] = sum_j X[t][j] * W_hat[i][j],  t < T.
 * The weights are dequantised to fp16 on the fly and contracted on the matrix cores with fp32 accumulation.
 * dev: the tiled kind runs the matrix-core kernel that expands the packed bits straight into MFMA operands
 * (N:M in {2:4, 3:8, 4:8, 5:8, 6:8, 3:4}; the residual term of the salient columns is a second, short contraction against
 * the gathered salient columns of X, which the call first writes to the workspace); the row-major kind runs a
 * generic kernel for any N:M (the two terms of a salient weight go through two contractions there too).
 * Tiled 2:4 layers run on the structured-sparse matrix instruction (kept weights plus an index word as the operand,
 * Sec. 3.1 / App. C; its 32x32x32 form).
 * When T and n are so small that a (128 tokens x 256 rows) tile per workgroup would leave most of the chip idle (fewer
 * than 200 workgroups), the 512-column superblocks are dealt to up to 16 groups of workgroups that each leave an fp32
 * partial tile in the workspace, and a second kernel adds the partial tiles in a fixed order: the result is
 * reproducible, and equal to the unsplit one up to fp32 summation order.
 * X: device fp16 [T][k], finite values (a padding column or token re-reads valid elements of X and meets zero
 * weights or an output that is never stored).  Y: device [T][n], fp16 or fp32, fully overwritten.  workspace: device scratch of at
 * least stb_gemm_workspace_bytes() bytes, 256-byte aligned (may be NULL when that is 0); it needs no
 * initialisation.  Calls that share a workspace must not overlap in time.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_EHIP. */
int stb_gemm(const stb_layout_t* dev, const void* X, int32_t T, void* Y, int32_t y_fp32,
             void* workspace, int64_t workspace_bytes, void* stream);

/* Scratch bytes stb_gemm needs for (layout, T): the size fields of `layout` are read (for the tiled kind
 * including max_sal_half, which stb_tile sets), its pointers are not.  Negative stb_status on a bad
 * argument. */
int64_t stb_gemm_workspace_bytes(const stb_layout_t* layout, int32_t T);

/* Measurement aid: reads `bytes` bytes (a multiple of 16, 16-byte aligned) of device memory with 128-bit loads
 * from every compute unit and writes one 32-bit checksum per workgroup to `sink` (device, at least 4096
 * bytes).  Timing it gives the streaming-read rate this GPU reaches on a buffer of that size, the practical
 * ceiling that the decode kernel's packed-weight GB/s is compared with.
 * Errors: STB_ENULL, STB_EINVAL, STB_EALIGN, STB_EHIP. */
int stb_probe_read(const void* src, int64_t bytes, void* sink, void* stream);

/* Measurement aid: `n_workgroups` workgroups of four wavefronts (one per SIMD) each issue `steps` x 32 matrix
 * instructions on independent accumulators, with `valu` (0, 2, 3, 5 or 8) vector instructions (v_perm_b32 on eight
 * independent registers) after each, in that order.
 * kind 0: v_mfma_f32_16x16x32_f16 (the dense prefill kernel's), kind 1: v_smfmac_f32_16x16x64_f16 (the 2:4 one's),
 * on 32 accumulators; kind 2: v_mfma_f32_32x32x16_f16, kind 3: v_smfmac_f32_32x32x32_f16, on 8 accumulators.  These
 * multiply operands that are all next to 1.0; kind 4..7 are the same four instructions on operands whose every bit is
 * random (magnitudes in [0.25, 2)), as weights and activations are: the matrix pipes issue those markedly slower.
 * Every thread writes 16 bytes to `sink` (device, 16-byte aligned, n_workgroups * 4096 bytes).  Timing it gives the
 * instruction rate this GPU sustains and how many vector instructions a matrix instruction hides: the practical
 * ceiling that the prefill kernels' TFLOP/s is compared with.
 * Errors: STB_ENULL, STB_EINVAL (kind outside 0..7, other valu, steps < 1, n_workgroups outside 1..65536), STB_EALIGN, STB_EHIP. */
int stb_probe_mfma(int32_t kind, int32_t valu, int32_t steps, int32_t n_workgroups, void* sink, void* stream);

/* Test hook: forces kernel choices that ordinary shapes would not reach, for every later call in this process (the
 * values are process-wide; set them while no other thread is inside stb_gemv / stb_gemm).
 *   gemv_kernel  0 automatic; 1 the tiled kind uses its older decode kernel with thin wavefronts, which otherwise
 *                only runs when the LDS areas of the default kernel do not fit
 *   gemv_visits  0 automatic; 1 .. 8: the default decode kernel takes that many superblocks per wavefront where the
 *                layer has as many and its staging areas fit (it chooses that by itself for wide layers at small
 *                batches)
 *   gemv_splits  0 automatic; 1 .. 64: the default decode kernel cuts the columns into that many splits where such a
 *                launch shape exists (otherwise the request is ignored)
 *   gemm_kernel  0 automatic; 1 keeps 2:4 layers on the dense-instruction prefill kernel (16x16x32 form); 2 runs any
 *                tiled layer on the 32x32x16 form of the dense kernel; 3 runs 2:4 layers on the 16x16x64 form of the
 *                sparse instruction; 4 runs any tiled layer on the kernel that shares the expanded operands of a
 *                workgroup through LDS
 * Errors: STB_EINVAL (a value outside the lists above; nothing is changed then). */
int stb_set_kernel_override(int32_t gemv_kernel, int32_t gemv_visits, int32_t gemv_splits, int32_t gemm_kernel);

/* Text for a status code (static storage). */
const char* stb_strerror(int status);

/* HIP error code of the last STB_EHIP on the calling thread (0 if none). */
int stb_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* STB_H */
