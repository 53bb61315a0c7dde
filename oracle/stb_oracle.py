"""Plain CPU oracle for structured-binary weights (STBLLM) and the product y = x . W_hat^T.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's CPU-baseline
leg.  It shares no code with the HIP library and never imports it.  Everything here is numpy in
float64 unless a stored format fixes another precision (fp16 scales, one fp32 add for salient weights).

What it follows (sections / equations / algorithms of the STBLLM paper):
  * si_magnitude, standardized_importance -- Sec. 3.2, Eq. 3 (Standardized Importance)
  * nm_mask                      -- Sec. 3.1 "N:M Sparsity", Alg. 1 step "Semi-Structured", Fig. 2(b)
  * binary                       -- Eq. 1-2, Alg. 2 "Binary" (alpha = l1 norm / count, sign(0) = +1)
  * residual_binary              -- Eq. 4, Alg. 2 "Res_Approx"
  * search_breakpoints           -- Alg. 2 "NonSalientAwareQuant", Eq. 5-6, ratio p2 = 2 p1 (App. A)
  * region_ids                   -- Alg. 2 "Trisection": sparse |w|>p2, intermediate p1<|w|<=p2, dense |w|<=p1
  * hessian_factor, pack_obc     -- Alg. 1 in full: H = 2 X^T X, H^c = Cholesky((H + lambda I)^-1), Standardized Importance
                                    on each 128-column slice, block-wise error compensation of the later columns
  * pack / unpack                -- the storage the paper accounts for in "Average Bits" (1 sign bit per
                                    kept weight, a second one on salient columns, 2-bit group id,
                                    per-block channel-wise scales) plus the N:M position mask
  * average_bits                 -- Sec. 3.4 "Average Bits": N_param * N / M, Table 1
  * layer_nm_assignment          -- Sec. 3.3 "Layer-wise N:M Assignment"
  * salient_columns              -- Alg. 2 "Salient" on a diagonal Hessian (Alg. 1: H = 2 X X^T, H^c = Cholesky((H + lambda I)^-1))
  * code24_encode / code24_decode -- App. C: the six-bit code of a 2:4 group (uint16 meta index E per four
                                    groups, uint8 of eight sign bits for the same 16 columns)
  * matmul                       -- the definition y = x . W_hat^T, evaluated in float64

Readings taken where the paper is silent are listed in the repository's design notes; the ones that
matter for the arithmetic are repeated next to the code below.

Canonical arithmetic (so that an independent implementation can reproduce the bytes exactly):
every sum is float64, sequential, in ascending index order (adding +0.0 for a non-member changes
nothing, so masked running sums are the same thing); mean = sum / count with one float64 divide;
fp16 storage = float64 -> float32 -> float16, round-to-nearest-even at each step.

Parity pins: see tests/test_oracle_pins.py.  Model quality (perplexity, zero-shot accuracy) is
"parity unpinned": it needs trained weights and datasets that do not exist here.
"""
from __future__ import annotations

import numpy as np

BLOCK = 128
DENSE, INTER, SPARSE, SALIENT = 0, 1, 2, 3
N_CANDIDATES = 160
RATIO = 2.0  # p2 = RATIO * p1


# ----------------------------------------------------------------------------------------------
# small helpers
# ----------------------------------------------------------------------------------------------
def pad_to(x: int, m: int) -> int:
    return (x + m - 1) // m * m


def to_f16(x) -> np.ndarray:
    """float64 -> float32 -> float16, round-to-nearest-even twice (the storage rule for scales)."""
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float16)


def seq_sum(v) -> float:
    """Sequential ascending-index float64 sum of a vector (running sum, last element)."""
    v = np.asarray(v, dtype=np.float64).ravel()
    if v.size == 0:
        return 0.0
    return float(np.cumsum(v)[-1])


def seq_rowsum(X) -> np.ndarray:
    """Sequential ascending-j float64 sum of each row."""
    X = np.asarray(X, dtype=np.float64)
    if X.shape[1] == 0:
        return np.zeros(X.shape[0], dtype=np.float64)
    return np.cumsum(X, axis=1)[:, -1].copy()


def seq_colsum(X) -> np.ndarray:
    """Sequential ascending-i float64 sum of each column."""
    X = np.asarray(X, dtype=np.float64)
    if X.shape[0] == 0:
        return np.zeros(X.shape[1], dtype=np.float64)
    return np.cumsum(X, axis=0)[-1, :].copy()


def sign_pm(w) -> np.ndarray:
    """sign(w) of Eq. 2: +1 for w >= 0, -1 otherwise (so a kept exact zero carries +alpha)."""
    return np.where(np.asarray(w) >= 0, 1.0, -1.0)


# ----------------------------------------------------------------------------------------------
# Standardized Importance, Eq. 3
# ----------------------------------------------------------------------------------------------
def si_magnitude(W) -> np.ndarray:
    """mu(|W_ij|) = |W_ij| / sum_j |W_ij|  +  |W_ij| / sum_i |W_ij|   (Eq. 3, right-hand part).

    A zero row (column) sum makes that term 0.
    """
    A = np.abs(np.asarray(W, dtype=np.float64))
    rs = seq_rowsum(A)
    cs = seq_colsum(A)
    mu = np.zeros_like(A)
    np.divide(A, rs[:, None], out=mu, where=(rs[:, None] > 0))
    t = np.zeros_like(A)
    np.divide(A, cs[None, :], out=t, where=(cs[None, :] > 0))
    mu += t
    return mu


def standardized_importance(W, xnorm) -> np.ndarray:
    """S_ij = sigma(mu(|W_ij|)) * ||X_:,j||_2  (Eq. 3).

    sigma(.) is the z-score over all n*k entries of the matrix mu (population standard deviation,
    a zero deviation is replaced by 1); xnorm_j is the L2 norm of input feature j.
    The formula is followed as printed: entries below the mean get a negative score, which a larger
    xnorm makes more negative.
    """
    mu = si_magnitude(W)
    n, k = mu.shape
    mean = seq_sum(seq_rowsum(mu)) / float(n * k)
    d = mu - mean
    var = seq_sum(seq_rowsum(d * d)) / float(n * k)
    sd = float(np.sqrt(var))
    if sd == 0.0:
        sd = 1.0
    return (d / sd) * np.asarray(xnorm, dtype=np.float64)[None, :]


# ----------------------------------------------------------------------------------------------
# N:M selection
# ----------------------------------------------------------------------------------------------
def nm_mask(S, N: int, M: int) -> np.ndarray:
    """Keep the N highest-scoring of every M consecutive input weights of each row.

    Equal scores: the lower column index is kept.  Returns a boolean (n, k) mask.
    """
    S = np.asarray(S, dtype=np.float64)
    n, k = S.shape
    assert k % M == 0 and 1 <= N <= M
    G = S.reshape(n, k // M, M)
    order = np.argsort(-G, axis=2, kind="stable")      # descending score, ties by ascending index
    keep = np.zeros((n, k // M, M), dtype=bool)
    np.put_along_axis(keep, order[:, :, :N], True, axis=2)
    return keep.reshape(n, k)


# ----------------------------------------------------------------------------------------------
# Binarisation, Eq. 1-2 and Eq. 4
# ----------------------------------------------------------------------------------------------
def binary(absw, member):
    """Per-row scale of Eq. 1 over the members of each row: alpha_i = sum_j |w_ij| / count_i.

    `absw` (n, c) float64 magnitudes, `member` (n, c) bool.  Rows without members get alpha 0.
    Returns (alpha float64 (n,), count int64 (n,)).
    """
    cnt = member.sum(axis=1).astype(np.int64)
    s = seq_rowsum(np.where(member, absw, 0.0))
    alpha = np.zeros(absw.shape[0], dtype=np.float64)
    np.divide(s, cnt, out=alpha, where=(cnt > 0))
    return alpha, cnt


def residual_binary(Wb, member):
    """Second-order binarisation of the salient weights of one column block (Eq. 4).

    B1 = alpha_o * sign(W); R = W - B1; B2 = alpha_r * sign(R); W ~ B1 + B2, per row over `member`.
    The residual is taken against the fp16-rounded alpha_o, i.e. against what inference will use.
    Returns (alpha_o fp16 (n,), alpha_r fp16 (n,), t bool (n, c) = residual sign is +1).
    """
    Wb = np.asarray(Wb, dtype=np.float64)
    alpha_o, _ = binary(np.abs(Wb), member)
    alpha_o16 = to_f16(alpha_o)
    R = Wb - alpha_o16.astype(np.float64)[:, None] * sign_pm(Wb)
    alpha_r, _ = binary(np.abs(R), member)
    return alpha_o16, to_f16(alpha_r), (R >= 0) & member


# ----------------------------------------------------------------------------------------------
# Non-salient regions: break-point search and trisection
# ----------------------------------------------------------------------------------------------
def region_ids(absw, p1: float, p2: float) -> np.ndarray:
    """Trisection: sparse (2) |w| > p2, intermediate (1) p1 < |w| <= p2, dense (0) |w| <= p1."""
    ids = np.zeros(absw.shape, dtype=np.uint8)
    ids[absw > p1] = INTER
    ids[absw > p2] = SPARSE
    return ids


def trisection_error(absw, member, p1: float, p2: float) -> float:
    """Eq. 5: squared error of binarising the three regions separately, each row with its own scale.

    ||W_r - alpha_r B_r||^2 summed over the regions equals sum (|w| - alpha_region(row))^2 over the
    members; rows are summed left to right, then the row totals top to bottom.
    """
    ids = region_ids(absw, p1, p2)
    alpha_at = np.zeros_like(absw)
    for r in (SPARSE, INTER, DENSE):
        m = member & (ids == r)
        alpha, _ = binary(absw, m)                       # Eq. 6: alpha = l1 norm / member count
        alpha_at = np.where(m, alpha[:, None], alpha_at)
    d = np.where(member, absw - alpha_at, 0.0)
    return seq_sum(seq_rowsum(d * d))


def candidate_grid() -> np.ndarray:
    return np.linspace(0.1, 0.9, N_CANDIDATES)


def search_breakpoints(Wb, member, return_errors: bool = False):
    """Alg. 2 "NonSalientAwareQuant" on one column block (all rows, non-salient kept weights).

    Scan 160 candidates p1 = c * max|w|, c in linspace(0.1, 0.9, 160), p2 = 2 * p1; skip a candidate
    when p2 > 0.9 * max|w|; keep the first strict minimum of the trisection error.
    """
    absw = np.abs(np.asarray(Wb, dtype=np.float64))
    mx = float(np.max(np.where(member, absw, 0.0))) if member.any() else 0.0
    best_e, best_p1, best_p2 = np.inf, 0.0, 0.0
    errors = {}
    for t, c in enumerate(candidate_grid()):
        p1 = float(c) * mx
        p2 = RATIO * p1
        if p2 > 0.9 * mx:
            continue
        e = trisection_error(absw, member, p1, p2)
        errors[t] = e
        if e < best_e:
            best_e, best_p1, best_p2 = e, p1, p2
    if return_errors:
        return best_p1, best_p2, errors
    return best_p1, best_p2


def tertile_breakpoints(Wb, member):
    """Break-points at the one-third and two-thirds order statistics of the members' magnitudes.

    With the m magnitudes sorted ascending a[0..m-1]: p1 = a[ceil(m/3) - 1], p2 = a[ceil(2m/3) - 1].
    """
    a = np.sort(np.abs(np.asarray(Wb, dtype=np.float64))[member])
    m = a.size
    if m == 0:
        return 0.0, 0.0
    return float(a[(m + 2) // 3 - 1]), float(a[(2 * m + 2) // 3 - 1])


# ----------------------------------------------------------------------------------------------
# Layout: closed forms
# ----------------------------------------------------------------------------------------------
def layout_sizes(n: int, k: int, N: int, M: int, S: int) -> dict:
    """Byte counts of the packed planes (closed form)."""
    assert k % BLOCK == 0 and k % M == 0
    nb = k // BLOCK
    slots = k * N // M
    S_pad = pad_to(S, 128) if S > 0 else 0
    d = dict(
        mask_stride=k // 8,
        sign_stride=pad_to(pad_to(slots, 8) // 8, 16),
        region_stride=pad_to(pad_to(2 * slots, 8) // 8, 16),
        res_stride=S_pad // 8,
        n_salient_pad=S_pad,
        n_blocks=nb,
    )
    d["mask_bytes"] = n * d["mask_stride"]
    d["sign_bytes"] = n * d["sign_stride"]
    d["region_bytes"] = n * d["region_stride"]
    d["res_bytes"] = n * d["res_stride"]
    d["scales_bytes"] = n * nb * 4 * 2
    d["res_scale_bytes"] = n * nb * 2
    d["salmap_bytes"] = k // 8
    d["salprefix_bytes"] = 4 * (nb + 1)
    d["total_bytes"] = (d["mask_bytes"] + d["sign_bytes"] + d["region_bytes"] + d["res_bytes"]
                        + d["scales_bytes"] + d["res_scale_bytes"] + d["salmap_bytes"]
                        + d["salprefix_bytes"])
    return d


def average_bits(r_salient: float, N: int, M: int) -> float:
    """Sec. 3.4: N_param = 2 r_salient + (1 - r_salient);  N_stbllm = N_param * N / M."""
    return (2.0 * r_salient + (1.0 - r_salient)) * N / M


# ----------------------------------------------------------------------------------------------
# Packing
# ----------------------------------------------------------------------------------------------
def _bits_to_bytes(bits, stride_bytes: int) -> np.ndarray:
    """(n, nbits) 0/1 -> (n, stride_bytes) uint8, bit b of byte c <-> index 8c + b, zero padded."""
    bits = np.asarray(bits, dtype=np.uint8)
    n, nbits = bits.shape
    full = np.zeros((n, stride_bytes * 8), dtype=np.uint8)
    full[:, :nbits] = bits
    return np.packbits(full, axis=1, bitorder="little")


def bitmap_to_bool(words, k: int) -> np.ndarray:
    b = np.unpackbits(np.ascontiguousarray(words, dtype="<u4").view(np.uint8), bitorder="little")
    return b[:k].astype(bool)


def pack(W, xnorm, sal_bitmap, N: int, M: int, region_mode: int = 0, return_debug: bool = False):
    """Structured-binarise W and emit the packed planes.

    Steps, per Alg. 1 without the Hessian parts (no calibration data exists here, so the salient
    column set is an input and there is no error compensation between blocks):
      1. Standardized Importance over the whole layer (Eq. 3)
      2. N:M mask from the scores
      3. per 128-column block: residual binarisation of the kept salient weights (per row),
         break-point search (mode 0) or tertile split (mode 1) over the kept non-salient weights of
         all rows, then trisection with one scale per (row, block, region)
      4. signs (Eq. 2) and the bit planes

    Planes (all little-endian; bit b of byte c <-> index 8c + b; padding is zero):
      mask      (n, k/8) bytes        bit j = weight j of the row is kept
      sign      (n, sign_stride)      bit r = 1 iff the r-th kept weight of the row is >= 0
      region    (n, region_stride)    2-bit field r = group id of the r-th kept weight
                                      (0 dense, 1 intermediate, 2 sparse, 3 salient)
      res_sign  (n, S_pad/8)          bit u <-> u-th salient column (ascending); 1 iff kept there and
                                      the residual sign is +1
      scales    fp16 (n, k/128, 4)    [dense, intermediate, sparse, alpha_o]
      res_scale fp16 (n, k/128)       alpha_r
      sal_bitmap (k/32 words)         bit j = column j is salient
      sal_block_prefix uint32 (k/128 + 1)   salient columns before each block
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    n, k = W.shape
    sal = bitmap_to_bool(sal_bitmap, k)
    S = int(sal.sum())
    L = layout_sizes(n, k, N, M, S)
    nb = L["n_blocks"]

    score = standardized_importance(W, xnorm)
    mask = nm_mask(score, N, M)
    del score

    W64 = W.astype(np.float64)
    ids = np.zeros((n, k), dtype=np.uint8)
    tpos = np.zeros((n, k), dtype=bool)
    scales = np.zeros((n, nb, 4), dtype=np.float16)
    res_scale = np.zeros((n, nb), dtype=np.float16)
    breakpoints = np.zeros((nb, 2), dtype=np.float64)

    for q in range(nb):
        c0, c1 = q * BLOCK, (q + 1) * BLOCK
        Wb = W64[:, c0:c1]
        absb = np.abs(Wb)
        kept_sal = mask[:, c0:c1] & sal[None, c0:c1]
        kept_ns = mask[:, c0:c1] & ~sal[None, c0:c1]

        a_o, a_r, t = residual_binary(Wb, kept_sal)
        scales[:, q, SALIENT] = a_o
        res_scale[:, q] = a_r
        tpos[:, c0:c1] = t

        if region_mode == 0:
            p1, p2 = search_breakpoints(Wb, kept_ns)
        elif region_mode == 1:
            p1, p2 = tertile_breakpoints(Wb, kept_ns)
        else:
            raise ValueError("region_mode must be 0 or 1")
        breakpoints[q] = (p1, p2)
        rid = region_ids(absb, p1, p2)
        for r in (DENSE, INTER, SPARSE):
            alpha, _ = binary(absb, kept_ns & (rid == r))
            scales[:, q, r] = to_f16(alpha)
        rid[kept_sal] = SALIENT
        ids[:, c0:c1] = rid

    slots = k * N // M
    sign_slots = (W >= 0)[mask].reshape(n, slots)
    id_slots = ids[mask].reshape(n, slots)
    id_bits = np.zeros((n, 2 * slots), dtype=np.uint8)
    id_bits[:, 0::2] = id_slots & 1
    id_bits[:, 1::2] = id_slots >> 1

    planes = dict(
        mask=np.packbits(mask, axis=1, bitorder="little"),
        sign=_bits_to_bytes(sign_slots, L["sign_stride"]),
        region=_bits_to_bytes(id_bits, L["region_stride"]),
        res_sign=(_bits_to_bytes((tpos & mask)[:, sal], L["res_stride"]) if S > 0
                  else np.zeros((n, 0), dtype=np.uint8)),
        scales=scales,
        res_scale=res_scale,
        sal_bitmap=np.ascontiguousarray(sal_bitmap, dtype="<u4").copy(),
        sal_block_prefix=np.concatenate(
            [[0], np.cumsum(sal.reshape(nb, BLOCK).sum(axis=1))]).astype("<u4"),
    )
    if return_debug:
        return planes, dict(mask=mask, ids=ids, tpos=tpos, breakpoints=breakpoints)
    return planes


def _emit_planes(n, k, N, M, mask, signpos, ids, tpos, scales, res_scale, sal_bitmap):
    """The bit planes of pack() from per-weight decisions (mask, sign >= 0, group id, residual sign) and the scales."""
    sal = bitmap_to_bool(sal_bitmap, k)
    S = int(sal.sum())
    L = layout_sizes(n, k, N, M, S)
    nb = L["n_blocks"]
    slots = k * N // M
    sign_slots = signpos[mask].reshape(n, slots)
    id_slots = ids[mask].reshape(n, slots)
    id_bits = np.zeros((n, 2 * slots), dtype=np.uint8)
    id_bits[:, 0::2] = id_slots & 1
    id_bits[:, 1::2] = id_slots >> 1
    return dict(
        mask=np.packbits(mask, axis=1, bitorder="little"),
        sign=_bits_to_bytes(sign_slots, L["sign_stride"]),
        region=_bits_to_bytes(id_bits, L["region_stride"]),
        res_sign=(_bits_to_bytes((tpos & mask)[:, sal], L["res_stride"]) if S > 0
                  else np.zeros((n, 0), dtype=np.uint8)),
        scales=scales,
        res_scale=res_scale,
        sal_bitmap=np.ascontiguousarray(sal_bitmap, dtype="<u4").copy(),
        sal_block_prefix=np.concatenate(
            [[0], np.cumsum(sal.reshape(nb, BLOCK).sum(axis=1))]).astype("<u4"),
    )


def hessian_factor(X, lam: float) -> np.ndarray:
    """H^c of Alg. 1 for calibration activations X (r samples x k input features):
    H = 2 X^T X (the Hessian of the layer's squared output error), H^c = the upper-triangular Cholesky factor of
    (H + lam I)^-1, i.e. H^c^T H^c = (H + lam I)^-1.

    Readings: the paper writes H = 2 X X^T for X in R^{r x d}; the Hessian over the d = k input features is meant.
    Its "Cholesky(.)" does not say which triangle: only the upper factor has non-zero entries H^c[b:b+beta, b+beta:]
    for the compensation step to use, so the upper one it is.
    """
    X = np.asarray(X, dtype=np.float64)
    k = X.shape[1]
    H = 2.0 * (X.T @ X) + float(lam) * np.eye(k)
    Hinv = np.linalg.inv(H)
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.ascontiguousarray(np.linalg.cholesky(Hinv).T)


def pack_obc(W, Hc, xnorm, sal_bitmap, N: int, M: int, region_mode: int = 0, return_debug: bool = False):
    """Alg. 1 as a whole: block after block (128 columns), on a float64 working copy of W:
      1. Standardized Importance of the block's slice (Alg. 1 calls it on W[:, b:b+beta]: sums, mean and deviation of
         Eq. 3 over the slice) and the N:M mask from it
      2. residual binarisation of the kept salient weights, break points and trisection of the kept non-salient ones,
         exactly as pack() does per block -> B, the dequantised block (what inference will multiply by)
      3. E = (W_block - B) / diag(H^c)_block  (column j of the error is divided by H^c[j, j])
      4. W[:, later columns] -= E . H^c[block, later columns]
    Hc: (k, k) upper-triangular factor from hessian_factor(), or None: then steps 3-4 are skipped, which leaves pack()
    with the per-block Standardized Importance of Alg. 1 instead of the whole-layer one of Eq. 3.
    The salient column set is an input, as in pack().

    Readings: "E <- (W - B) / H^c_{b:b+beta, b:b+beta}" divides column j by the diagonal entry H^c[j, j] (the scaling
    of a column's error in the optimal-brain-compression update that the comment in Alg. 1 names); the product of step
    4 is accumulated over the block's columns in ascending order, one multiply and one add per term.
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    n, k = W.shape
    sal = bitmap_to_bool(sal_bitmap, k)
    nb = k // BLOCK
    xn = np.asarray(xnorm, dtype=np.float32)
    Wd = W.astype(np.float64)
    mask = np.zeros((n, k), dtype=bool)
    signpos = np.zeros((n, k), dtype=bool)
    ids = np.zeros((n, k), dtype=np.uint8)
    tpos = np.zeros((n, k), dtype=bool)
    scales = np.zeros((n, nb, 4), dtype=np.float16)
    res_scale = np.zeros((n, nb), dtype=np.float16)
    for q in range(nb):
        c0, c1 = q * BLOCK, (q + 1) * BLOCK
        Wb = Wd[:, c0:c1].copy()
        absb = np.abs(Wb)
        mb = nm_mask(standardized_importance(Wb, xn[c0:c1]), N, M)
        kept_sal = mb & sal[None, c0:c1]
        kept_ns = mb & ~sal[None, c0:c1]
        a_o, a_r, t = residual_binary(Wb, kept_sal)
        if region_mode == 0:
            p1, p2 = search_breakpoints(Wb, kept_ns)
        elif region_mode == 1:
            p1, p2 = tertile_breakpoints(Wb, kept_ns)
        else:
            raise ValueError("region_mode must be 0 or 1")
        rid = region_ids(absb, p1, p2)
        for r in (DENSE, INTER, SPARSE):
            alpha, _ = binary(absb, kept_ns & (rid == r))
            scales[:, q, r] = to_f16(alpha)
        rid[kept_sal] = SALIENT
        scales[:, q, SALIENT] = a_o
        res_scale[:, q] = a_r
        mask[:, c0:c1] = mb
        signpos[:, c0:c1] = Wb >= 0
        ids[:, c0:c1] = rid
        tpos[:, c0:c1] = t
        if Hc is not None and c1 < k:
            # B: the dequantised block, with the stored (fp16) scales and the one fp32 addition of salient weights
            s = np.where(Wb >= 0, np.float32(1), np.float32(-1))
            a = np.take_along_axis(scales[:, q, :].astype(np.float32), rid.astype(np.int64), axis=1)
            B = (s * a).astype(np.float32)
            tt = np.where(t, np.float32(1), np.float32(-1))
            both = (s * a).astype(np.float32) + (tt * res_scale[:, q].astype(np.float32)[:, None]).astype(np.float32)
            B = np.where(kept_sal, both.astype(np.float32), B)
            B = np.where(mb, B, np.float32(0)).astype(np.float64)
            E = (Wb - B) / np.diag(Hc)[None, c0:c1]
            acc = np.zeros((n, k - c1), dtype=np.float64)
            for c in range(BLOCK):                      # ascending, one multiply and one add per term
                acc += E[:, c:c + 1] * Hc[c0 + c:c0 + c + 1, c1:]
            Wd[:, c1:] -= acc
    planes = _emit_planes(n, k, N, M, mask, signpos, ids, tpos, scales, res_scale, sal_bitmap)
    if return_debug:
        return planes, dict(mask=mask, ids=ids, tpos=tpos, W_final=Wd)
    return planes


# ----------------------------------------------------------------------------------------------
# Layer-wise N:M assignment, Sec. 3.3
# ----------------------------------------------------------------------------------------------
def layer_l2_norm(W) -> float:
    """omega of Sec. 3.3: the L2 norm of a layer's weights (float64, sequential sum of squares in row-major order)."""
    W = np.asarray(W, dtype=np.float64)
    return float(np.sqrt(seq_sum(W * W)))


def layer_nm_assignment(omegas, r_target: float, M: int = 8):
    """N_i of every layer for a target ratio (Sec. 3.3): alpha_i = omega_i / sum(omega),
    N_i / M = alpha_i + (1 - alpha_i) * r_target.

    Readings: the paper gives the ratio but not how it becomes an integer N: the nearest integer to M * ratio (a half
    rounds up), kept inside 1..M.  As printed, the ratio never falls below r_target (alpha_i >= 0), so the mean ratio
    over the layers lies above the target by the mean of alpha_i (1 - r_target); the text's example of layers below
    the target (3:8 around 4:8) does not follow from the formula, and the formula is what is implemented.
    Returns (N int64 (L,), ratio float64 (L,)).
    """
    om = np.asarray(omegas, dtype=np.float64)
    assert om.ndim == 1 and om.size >= 1 and (om >= 0).all() and 0.0 <= r_target <= 1.0 and M >= 1
    total = seq_sum(om)
    alpha = om / total if total > 0 else np.full(om.shape, 1.0 / om.size)
    ratio = alpha + (1.0 - alpha) * float(r_target)
    N = np.clip(np.floor(M * ratio + 0.5), 1, M).astype(np.int64)
    return N, ratio


# ----------------------------------------------------------------------------------------------
# Salient columns, Alg. 2 "Salient"
# ----------------------------------------------------------------------------------------------
def salient_columns(W, xnorm, lam: float, max_per_block: int) -> np.ndarray:
    """The salient columns of every 128-column block (Alg. 1 calls Salient once per block), as a (k,) bool vector.

    Reading: only the norms of the input features are known here, so the Hessian H = 2 X X^T is taken as its
    diagonal, 2 xnorm_j^2; then H^c = Cholesky((H + lam I)^-1) is diagonal with [H^c_jj]^2 = 1 / (2 xnorm_j^2 + lam)
    and the salient matrix S = W^2 / [H^c]^2 is w_ij^2 (2 xnorm_j^2 + lam).  The length of the top-k list is not
    given in the paper: `max_per_block` is an input.  "binary" is the per-row scale of Eq. 1 over the columns of the
    set (the reading taken everywhere else).
    Steps: column score = sum_i S_ij; candidates = the max_per_block columns of the block with the largest score
    (ties: the lower column first); for i = 1 .. len: binarise the first i candidates together and all other columns
    of the block together, e_i = ||W - B||^2; keep the first i with the smallest e_i.
    """
    xn = np.asarray(xnorm, dtype=np.float32).astype(np.float64)
    h = 2.0 * xn * xn + float(lam)
    return _salient_select(W, lambda Wb, b: (Wb * Wb) * h[None, b:b + BLOCK], max_per_block)


def salient_columns_hc(W, Hc, max_per_block: int) -> np.ndarray:
    """Salient(W, H^c) of Alg. 2 with the factor itself: the salient matrix of a block is W^2 divided by the square of
    the diagonal of H^c's diagonal block, S_ij = w_ij^2 / (H^c_jj)^2; everything after the scores is as in
    salient_columns().  Hc: (k, k) factor from hessian_factor() (only its diagonal is read)."""
    d = np.diagonal(np.asarray(Hc, dtype=np.float64)).copy()
    assert (d != 0).all()
    return _salient_select(W, lambda Wb, b: (Wb * Wb) / (d * d)[None, b:b + BLOCK], max_per_block)


def _salient_select(W, salient_matrix, max_per_block: int) -> np.ndarray:
    """The steps of Salient() after the salient matrix: column scores, candidates, the count with the least error."""
    W = np.asarray(W, dtype=np.float64)
    n, k = W.shape
    assert k % BLOCK == 0 and 0 <= max_per_block <= BLOCK
    out = np.zeros(k, dtype=bool)
    for b in range(0, k, BLOCK):
        Wb = W[:, b:b + BLOCK]
        score = seq_colsum(salient_matrix(Wb, b))
        order = np.argsort(-score, kind="stable")[:max_per_block]
        absw, sgn = np.abs(Wb), sign_pm(Wb)
        best, n_star = np.inf, 0
        for i in range(1, len(order) + 1):
            sal = np.zeros(BLOCK, dtype=bool)
            sal[order[:i]] = True
            member = np.broadcast_to(sal, (n, BLOCK))
            a1, _ = binary(absw, member)
            a2, _ = binary(absw, ~member)
            B = np.where(member, a1[:, None], a2[:, None]) * sgn
            e = seq_sum(seq_rowsum((Wb - B) * (Wb - B)))
            if e < best:
                best, n_star = e, i
        out[b + order[:n_star]] = True
    return out


# ----------------------------------------------------------------------------------------------
# The 2:4 group code of App. C
# ----------------------------------------------------------------------------------------------
def code24_encode(mask, sign_slots):
    """Meta index E and value bytes V of a 2:4 matrix (App. C, "D = A(E) x B + C").

    mask: (n, k) bool, exactly two kept weights in every group of four columns, k a multiple of 16.
    sign_slots: (n, k/2) 0/1, the sign of every kept weight in column order, 1 -> +1, 0 -> -1.
    E: (n, k/16) uint16; group g of a row owns the nibble at bits 4*(g % 4) of E[row, g // 4]; the low two bits
       are the position (0..3) of its first kept weight, the high two bits the position of its second one.
    V: (n, k/16) uint8; bit 2*(g % 4) + j = sign bit of the j-th kept weight of group g.
    (The paper fixes four index bits and two value bits per group, a uint16 / uint8 per four groups, and
    1 -> +1; the order of the bits inside them is the reading stated here.)
    """
    mask = np.asarray(mask, dtype=bool)
    n, k = mask.shape
    assert k % 16 == 0
    groups = mask.reshape(n, k // 4, 4)
    assert (groups.sum(axis=2) == 2).all(), "every group of four must keep exactly two weights"
    first = np.full((n, k // 4), -1, dtype=np.int64)
    second = np.full((n, k // 4), -1, dtype=np.int64)
    for j in range(4):                                   # positions in ascending order
        kept = groups[:, :, j]
        is_second = kept & (first >= 0)
        is_first = kept & (first < 0)
        first = np.where(is_first, j, first)
        second = np.where(is_second, j, second)
    nibble = (first | (second << 2)).reshape(n, k // 16, 4)
    E = np.zeros((n, k // 16), dtype=np.uint16)
    for g in range(4):
        E |= (nibble[:, :, g] << (4 * g)).astype(np.uint16)
    V = np.packbits(np.asarray(sign_slots, dtype=np.uint8).reshape(n, k // 2), axis=1, bitorder="little")
    return E, V


def code24_decode(E, V):
    """The dense ternary matrix (n, k) of -1 / 0 / +1 that (E, V) stand for."""
    E = np.asarray(E, dtype=np.uint16)
    V = np.asarray(V, dtype=np.uint8)
    n, k16 = E.shape
    A = np.zeros((n, k16 * 16), dtype=np.int8)
    for i in range(n):
        for c in range(k16):
            for g in range(4):
                nib = (int(E[i, c]) >> (4 * g)) & 15
                for j, pos in enumerate((nib & 3, nib >> 2)):
                    bit = (int(V[i, c]) >> (2 * g + j)) & 1
                    A[i, 16 * c + 4 * g + pos] = 1 if bit else -1
    return A


# ----------------------------------------------------------------------------------------------
# Dequantisation from the packed bytes, and the product
# ----------------------------------------------------------------------------------------------
def unpack(planes: dict, n: int, k: int, N: int, M: int) -> np.ndarray:
    """Dense fp32 W_hat decoded from the packed bytes alone.

      not kept                      -> 0
      kept, id in {0, 1, 2}         -> s * f32(scale[row, block, id])
      kept, id = 3 (salient column) -> f32( s * f32(alpha_o) + t * f32(alpha_r) )   (one fp32 add)
    """
    mask = np.unpackbits(planes["mask"], axis=1, bitorder="little")[:, :k].astype(bool)
    slots = k * N // M
    assert (mask.sum(axis=1) == slots).all(), "mask does not keep k*N/M weights in every row"
    rank = np.cumsum(mask, axis=1) - 1                       # slot of each kept weight in its row
    rank = np.where(mask, rank, 0)
    sign_bits = np.unpackbits(planes["sign"], axis=1, bitorder="little")
    reg_bits = np.unpackbits(planes["region"], axis=1, bitorder="little")
    rows = np.arange(n)[:, None]
    s = np.where(sign_bits[rows, rank] == 1, np.float32(1), np.float32(-1))
    rid = reg_bits[rows, 2 * rank] | (reg_bits[rows, 2 * rank + 1] << 1)

    sal = bitmap_to_bool(planes["sal_bitmap"], k)
    ordinal = np.cumsum(sal) - 1                             # index among salient columns
    blk = (np.arange(k) // BLOCK)[None, :]
    scales = planes["scales"].astype(np.float32)             # (n, nb, 4)
    a = scales[rows, blk, rid]                               # scale selected by the group id
    What = np.where(mask, s * a, np.float32(0)).astype(np.float32)

    if sal.any():
        res_bits = np.unpackbits(planes["res_sign"], axis=1, bitorder="little")
        tcol = np.zeros((n, k), dtype=np.uint8)
        tcol[:, sal] = res_bits[:, ordinal[sal]]
        t = np.where(tcol == 1, np.float32(1), np.float32(-1))
        a_r = planes["res_scale"].astype(np.float32)[rows, blk]
        is_sal = mask & (rid == SALIENT)
        both = (s * a).astype(np.float32) + (t * a_r).astype(np.float32)   # single fp32 rounding
        What = np.where(is_sal, both.astype(np.float32), What)
    return What


def matmul(x, What):
    """y = x . W_hat^T in float64 and the row bound sum_j |x_bj| |W_hat_ij| used by the tolerance."""
    x64 = np.asarray(x, dtype=np.float64)
    W64 = np.asarray(What, dtype=np.float64)
    return x64 @ W64.T, np.abs(x64) @ np.abs(W64).T
