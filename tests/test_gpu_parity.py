"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle.

Bars: packed bytes and dequantised fp32 weights bit-exact; outputs within
|y_gpu - y_oracle| <= 2e-3 * sum_j |x_j| |W_hat_ij| (and exactly 0 where that bound is 0).
"""
import contextlib
import hashlib
import json
import os
import sys

import numpy as np
import pytest

import paper_2408_01803_amd as S
from oracle import stb_oracle as O
from workloads import WORKLOADS, make_layer, make_x

pytestmark = pytest.mark.gpu

TOL = 2e-3
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "packed_digests.json")


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert os.path.exists(S.LIB_PATH), "libstb.so is missing: build it before running the GPU tests"
    assert torch.cuda.is_available(), "no GPU visible"
    torch.cuda.set_device(0)
    return torch


@contextlib.contextmanager
def forced(gemv_kernel=0, gemv_visits=0, gemv_splits=0, gemm_kernel=0):
    """Kernels that ordinary shapes would not reach, asked for through the library's test hook."""
    S.stb_set_kernel_override(gemv_kernel, gemv_visits, gemv_splits, gemm_kernel)
    try:
        yield
    finally:
        S.stb_set_kernel_override(0, 0, 0, 0)


GEMM_KERNELS = {"dense": S.GEMM_DENSE, "dense32": S.GEMM_DENSE32, "sparse16": S.GEMM_SPARSE16, "shared": S.GEMM_SHARED}


def _within_bound(y_gpu, y_ref, bound, what):
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    err = np.abs(y_gpu - y_ref)
    ok = err <= TOL * bound
    if not ok.all():
        idx = np.unravel_index(np.argmax(err - TOL * bound), err.shape)
        raise AssertionError(f"{what}: {int((~ok).sum())} outputs outside 2e-3 of the row bound; worst at {idx}: "
                             f"gpu {y_gpu[idx]} oracle {y_ref[idx]} bound {bound[idx]}")
    return float((err / np.maximum(bound, 1e-300)).max())


def _oracle_planes_from(pm):
    """The library's host image re-read as the oracle's plane dictionary (shapes restored)."""
    lay = pm.host_layout
    n, nb = lay.cfg.n_out, lay.n_blocks
    P = {}
    P["mask"] = pm.plane("mask").reshape(n, lay.mask_stride)
    P["sign"] = pm.plane("sign").reshape(n, lay.sign_stride)
    P["region"] = pm.plane("region").reshape(n, lay.region_stride)
    P["res_sign"] = pm.plane("res_sign").reshape(n, lay.res_stride)
    P["scales"] = pm.plane("scales").view(np.float16).reshape(n, nb, 4)
    P["res_scale"] = pm.plane("res_scale").view(np.float16).reshape(n, nb)
    P["sal_bitmap"] = pm.plane("sal_bitmap").view("<u4")
    P["sal_block_prefix"] = pm.plane("sal_block_prefix").view("<u4")
    return P


SMALL = [
    # n, k, N, M, mode, kind, seed: several 64-row / 128-column tiles with ragged tails
    (130, 640, 4, 8, 0, "x8", 101),
    (257, 1024, 2, 4, 0, "t3", 102),
    (200, 768, 6, 8, 1, "x8", 103),
    (96, 512, 5, 8, 0, "x8", 104),
    (64, 256, 8, 8, 0, "x8", 105),
    (5, 128, 1, 4, 1, "x8", 106),
    # crowded salient columns (optional 8th field = their number): about 9 and about 16 per half block of 64
    # columns, which takes the kernels through their second salient-column record and past it
    (48, 1024, 2, 4, 1, "x8", 108, 150),
    (64, 512, 2, 4, 0, "t3", 107, 130),
    (80, 512, 4, 8, 0, "x8", 109, 100),
    # more than 4096 columns: two column splits that meet through the workspace
    (40, 4608, 2, 4, 1, "t3", 110),
    # less than one tile in both directions
    (5, 128, 2, 4, 0, "x8", 111),
    (1, 128, 4, 8, 1, "x8", 112),
    (17, 256, 6, 8, 0, "t3", 113),
    # 3 and 5 kept of 8 (Sec. 3.3, Table 1): in the tiled order these use the slots of 4:8 / 6:8 with one unused per group
    (150, 896, 3, 8, 0, "x8", 114),
    (70, 1536, 5, 8, 1, "t3", 115, 120),
    (33, 4608, 3, 8, 0, "x8", 116),
]


def _tiled_ok(N, M):
    return (8 * N) % M == 0 and (8 * N // M) in (3, 4, 5, 6)


SMALL_KINDS = [(c, tiled) for c in SMALL for tiled in (False, True) if not tiled or _tiled_ok(c[2], c[3])]


def _pack_on_device(torch, W, xnorm, sal_bitmap, N, M, mode, per_block=False):
    """stb_pack_device on device copies of the inputs; returns the holder whose host image received the planes."""
    n, k = W.shape
    S_ = int(np.unpackbits(np.ascontiguousarray(sal_bitmap, dtype="<u4").view(np.uint8)).sum())
    pm = S.PackedMatrix(S.make_cfg(n, k, N, M, S_, mode))
    img = S.new_device_scratch(pm.host_layout.image_bytes)
    img.fill_(0xAB)                                   # every byte of every plane has to be written
    lay = pm.clone_layout_for(img.data_ptr(), False)
    ws = S.new_device_scratch(S.stb_pack_device_workspace_bytes(pm.cfg, per_block))
    ws.fill_(0xCD)
    Wd = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).cuda()
    xd = torch.from_numpy(np.ascontiguousarray(xnorm, dtype=np.float32)).cuda()
    sd = torch.from_numpy(np.ascontiguousarray(sal_bitmap, dtype="<u4").view(np.int32)).cuda()
    S.stb_pack_device(Wd, xd, sd, lay, per_block, ws)
    pm.host_image[:] = img.cpu().numpy()
    return pm


PACK_CASES = SMALL + [(300, 2048, 4, 8, 0, "x8", 117), (300, 1280, 6, 8, 1, "t3", 118), (77, 384, 3, 8, 1, "x8", 119)]


@pytest.mark.parametrize("case", PACK_CASES, ids=lambda c: f"{c[0]}x{c[1]}_{c[2]}of{c[3]}_m{c[4]}")
@pytest.mark.parametrize("per_block", [False, True], ids=["layer_si", "block_si"])
def test_device_packer_is_bit_exact_against_the_oracle(case, per_block, torch_cuda):
    n, k, N, M, mode, kind, seed, *rest = case
    _say(f"[case] device packer {n}x{k} {N}:{M} mode {mode} per_block {per_block}")
    L = make_layer(n, k, seed, kind, n_salient=rest[0] if rest else None)
    if per_block:
        ref = O.pack_obc(L["W"], None, L["xnorm"], L["sal_bitmap"], N, M, mode)
    else:
        ref = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    pm = _pack_on_device(torch_cuda, L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode, per_block)
    for name, v in ref.items():
        got = pm.plane(name)
        want = np.ascontiguousarray(v).view(np.uint8).ravel()
        assert got.shape == want.shape, name
        assert (got == want).all(), (name, int((got != want).sum()))


TILE_CASES = [c for c in PACK_CASES if _tiled_ok(c[2], c[3])]


@pytest.mark.parametrize("n,k,N,M,mode,seed", [(48, 384, 4, 8, 0, 61), (37, 640, 6, 8, 1, 62), (130, 1024, 2, 4, 0, 63),
                                                (19, 256, 5, 8, 0, 64), (300, 2048, 4, 8, 0, 65)])
def test_block_loop_packer_with_the_update_on_the_gpu_is_bit_exact(torch_cuda, n, k, N, M, mode, seed):
    """stb_pack_obc_hybrid (the compensation update of Alg. 1 as a kernel, the rest of the block loop on the host)
    against the oracle's pack_obc and against the all-host stb_pack_obc: the same bytes."""
    L = make_layer(n, k, seed, "x8")
    rng = np.random.default_rng(seed + 500)
    X = (rng.standard_normal((2 * k, k)) @ (np.eye(k) + 0.6 * rng.standard_normal((k, k)) / np.sqrt(k))).astype(np.float32)
    Hc, _ = S.stb_hessian_factor(X, 0.01 * float(np.mean(2.0 * np.sum(X.astype(np.float64) ** 2, axis=0))))
    _say(f"[step] stb_pack_obc_hybrid {n}x{k} {N}:{M} mode {mode}")
    pm = S.PackedMatrix.pack_obc_hybrid(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode, n_threads=3)
    host = S.PackedMatrix.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode, n_threads=3)
    assert (pm.host_image == host.host_image).all()
    if n * k <= 130 * 1024:                                # the oracle's block loop is slow
        ref = O.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode)
        assert (pm.unpack() == O.unpack(ref, n, k, N, M)).all()
    # without a factor the call is the host packer with per-block importance and touches no device memory
    plain = S.PackedMatrix.pack_obc_hybrid(L["W"], None, L["xnorm"], L["sal_bitmap"], N, M, mode)
    assert (plain.host_image == S.PackedMatrix.pack_obc(L["W"], None, L["xnorm"], L["sal_bitmap"], N, M, mode).host_image).all()


@pytest.mark.parametrize("case", TILE_CASES, ids=lambda c: f"{c[0]}x{c[1]}_{c[2]}of{c[3]}_m{c[4]}")
def test_pack_and_tile_on_the_device_feed_the_kernels(case, torch_cuda):
    """Weights in HBM -> stb_pack_device -> stb_tile_device -> stb_gemv, nothing through the host: the tiled image is
    the host's byte for byte, and the product agrees with the oracle."""
    torch = torch_cuda
    n, k, N, M, mode, kind, seed, *rest = case
    _say(f"[case] device pack + tile {n}x{k} {N}:{M}")
    L = make_layer(n, k, seed, kind, n_salient=rest[0] if rest else None)
    host = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    tl_host, timg_host = host.tiled()
    rimg = S.new_device_scratch(host.host_layout.image_bytes)
    rlay = host.clone_layout_for(rimg.data_ptr(), False)
    ws = S.new_device_scratch(S.stb_pack_device_workspace_bytes(host.cfg))
    S.stb_pack_device(torch.from_numpy(L["W"]).cuda(), torch.from_numpy(L["xnorm"]).cuda(),
                      torch.from_numpy(L["sal_bitmap"].view(np.int32)).cuda(), rlay, False, ws)
    timg = S.new_device_scratch(tl_host.image_bytes)
    timg.fill_(0xEE)
    tlay = S.stb_tiled_sizes(host.cfg)
    S.stb_layout_bind(tlay, timg.data_ptr())
    S.stb_tile_device(rlay, tlay)
    assert (tlay.max_sal_block, tlay.max_sal_half) == (tl_host.max_sal_block, tl_host.max_sal_half)
    got = timg.cpu().numpy()
    for name, off, size in S.PLANE_FIELDS + (("sal_tab", "off_saltab", "saltab_bytes"), ("res_t", "off_res_t", "res_t_bytes")):
        o, sz = getattr(tl_host, off), getattr(tl_host, size)
        assert (got[o:o + sz] == timg_host[o:o + sz]).all(), name
    What = O.unpack(O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode), n, k, N, M)
    for B in (1, 7):
        x = make_x(B, k, seed)
        y_ref, bound = O.matmul(x, What)
        xd = torch.from_numpy(x).cuda()
        yd = torch.empty((B, n), dtype=torch.float32, device="cuda")
        wsg = S.new_device_scratch(S.stb_gemv_workspace_bytes(host.cfg, B), zero=True)
        S.stb_gemv(tlay, xd, B, yd, True, wsg)
        torch.cuda.synchronize()
        _within_bound(yd.cpu().numpy(), y_ref, bound, f"gemv on the device-made image, B={B}")
    # the mismatch checks of stb_tile hold here too
    with pytest.raises(S.StbError) as e:
        S.stb_tile_device(tlay, tlay)
    assert e.value.status == S.STB_EINVAL


def test_device_packer_and_tiling_on_random_shapes(torch_cuda):
    """40 seeded random layers (any of the five ratios, 1 .. 1200 rows, up to 5000 columns, none / few / many / crowded
    salient columns, both region modes, both scopes of the importance): stb_pack_device and stb_tile_device give the
    host's planes byte for byte."""
    torch = torch_cuda
    rng = np.random.default_rng(20240801)
    for case in range(40):
        N, M = [(2, 4), (3, 8), (4, 8), (5, 8), (6, 8)][rng.integers(0, 5)]
        n = int(rng.integers(1, 1200))
        k = 128 * int(rng.integers(1, 40))
        nsal = int(rng.choice([0, max(1, k // 20), max(1, k // 6), min(k, 60)]))
        mode, per_block, seed = int(rng.integers(0, 2)), bool(rng.integers(0, 2)), int(rng.integers(0, 1 << 30))
        _say(f"[case {case}] device pack + tile n={n} k={k} {N}:{M} sal={nsal} mode={mode} per_block={per_block} seed={seed}")
        L = make_layer(n, k, seed, "x8", n_salient=nsal)
        if rng.integers(0, 3) == 0 and nsal >= 40:          # crowd the salient columns into the first two blocks
            cols = np.sort(rng.choice(min(k, 256), min(nsal, min(k, 256)), replace=False))
            bits = np.zeros(k, dtype=np.uint8)
            bits[cols] = 1
            L["sal_bitmap"] = np.packbits(bits, bitorder="little").view("<u4").copy()
        host = (S.PackedMatrix.pack_obc(L["W"], None, L["xnorm"], L["sal_bitmap"], N, M, mode) if per_block
                else S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode))
        tl_host, timg_host = host.tiled()
        rimg = S.new_device_scratch(host.host_layout.image_bytes)
        rlay = host.clone_layout_for(rimg.data_ptr(), False)
        ws = S.new_device_scratch(S.stb_pack_device_workspace_bytes(host.cfg, per_block))
        S.stb_pack_device(torch.from_numpy(L["W"]).cuda(), torch.from_numpy(L["xnorm"]).cuda(),
                          torch.from_numpy(L["sal_bitmap"].view(np.int32)).cuda(), rlay, per_block, ws)
        got = rimg.cpu().numpy()
        for name, off, size in S.PLANE_FIELDS:
            o, sz = getattr(host.host_layout, off), getattr(host.host_layout, size)
            assert (got[o:o + sz] == host.host_image[o:o + sz]).all(), (case, name)
        timg = S.new_device_scratch(tl_host.image_bytes)
        timg.fill_(0xEE)
        tlay = S.stb_tiled_sizes(host.cfg)
        S.stb_layout_bind(tlay, timg.data_ptr())
        S.stb_tile_device(rlay, tlay)
        assert (tlay.max_sal_block, tlay.max_sal_half) == (tl_host.max_sal_block, tl_host.max_sal_half)
        got = timg.cpu().numpy()
        for name, off, size in S.PLANE_FIELDS + (("sal_tab", "off_saltab", "saltab_bytes"), ("res_t", "off_res_t", "res_t_bytes")):
            o, sz = getattr(tl_host, off), getattr(tl_host, size)
            assert (got[o:o + sz] == timg_host[o:o + sz]).all(), (case, name)


def test_device_packer_edge_cases_and_errors(torch_cuda):
    torch = torch_cuda
    k = 256
    # all-zero weights (every score ties, every scale is 0), and a block whose columns are all salient
    Z = np.zeros((5, k), dtype=np.float32)
    none = np.zeros(k // 32, dtype=np.uint32)
    ones = np.ones(k, dtype=np.float32)
    pm = _pack_on_device(torch, Z, ones, none, 2, 4, 0)
    for name, v in O.pack(Z, ones, none, 2, 4, 0).items():
        assert (pm.plane(name) == np.ascontiguousarray(v).view(np.uint8).ravel()).all(), name
    L = make_layer(9, k, 23, n_salient=0)
    bm = np.zeros(k // 32, dtype=np.uint32)
    bm[4:8] = 0xFFFFFFFF
    xn = L["xnorm"].copy()
    xn[::7] = 0.0
    for mode in (0, 1):
        pm = _pack_on_device(torch, L["W"], xn, bm, 6, 8, mode)
        for name, v in O.pack(L["W"], xn, bm, 6, 8, mode).items():
            assert (pm.plane(name) == np.ascontiguousarray(v).view(np.uint8).ravel()).all(), (mode, name)
    # what the kernels find comes back as a status
    L = make_layer(20, k, 24)
    bad = L["W"].copy()
    bad[7, 130] = np.nan
    with pytest.raises(S.StbError) as e:
        _pack_on_device(torch, bad, L["xnorm"], L["sal_bitmap"], 4, 8, 0)
    assert e.value.status == S.STB_ENONFINITE
    xb = L["xnorm"].copy()
    xb[3] = -1.0
    with pytest.raises(S.StbError) as e:
        _pack_on_device(torch, L["W"], xb, L["sal_bitmap"], 4, 8, 0)
    assert e.value.status == S.STB_ENONFINITE
    # a bitmap that does not hold cfg.n_salient columns
    pm = S.PackedMatrix(S.make_cfg(20, k, 4, 8, 5, 0))
    img = S.new_device_scratch(pm.host_layout.image_bytes)
    lay = pm.clone_layout_for(img.data_ptr(), False)
    ws = S.new_device_scratch(S.stb_pack_device_workspace_bytes(pm.cfg))
    Wd = torch.from_numpy(L["W"]).cuda()
    xd = torch.from_numpy(L["xnorm"]).cuda()
    sd = torch.from_numpy(L["sal_bitmap"].view(np.int32)).cuda()
    with pytest.raises(S.StbError) as e:
        S.stb_pack_device(Wd, xd, sd, lay, False, ws)
    assert e.value.status == S.STB_EINVAL
    with pytest.raises(S.StbError) as e:
        S.stb_pack_device(Wd, xd, sd, lay, False, ws[256:])
    assert e.value.status == S.STB_EINVAL                     # workspace too small
    with pytest.raises(S.StbError) as e:
        S.stb_pack_device(Wd, xd, sd, lay, False, ws[8:])
    assert e.value.status == S.STB_EALIGN
    tl = S.stb_tiled_sizes(pm.cfg)
    timg = S.new_device_scratch(tl.image_bytes)
    S.stb_layout_bind(tl, timg.data_ptr())
    with pytest.raises(S.StbError) as e:
        S.stb_pack_device(Wd, xd, sd, tl, False, ws)
    assert e.value.status == S.STB_EINVAL                     # the packer writes the row-major order


@pytest.fixture(scope="module", params=SMALL_KINDS,
                ids=lambda c: f"{c[0][0]}x{c[0][1]}_{c[0][2]}of{c[0][3]}_m{c[0][4]}{'_s%d' % c[0][7] if len(c[0]) > 7 else ''}_{'tiled' if c[1] else 'rowmajor'}")
def small_case(request, torch_cuda):
    (n, k, N, M, mode, kind, seed, *rest), tiled = request.param
    _say(f"[case] small {request.param}")
    L = make_layer(n, k, seed, kind, n_salient=rest[0] if rest else None)
    ref = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    for name, v in ref.items():
        assert (pm.plane(name) == np.ascontiguousarray(v).view(np.uint8).ravel()).all(), name
    pm.to_device(tiled=tiled)
    What = O.unpack(ref, n, k, N, M)
    return dict(n=n, k=k, N=N, M=M, seed=seed, pm=pm, What=What, tiled=tiled, ref=ref)


def test_dequant_bit_exact_small(small_case, torch_cuda):
    torch = torch_cuda
    c = small_case
    out = torch.full((c["n"], c["k"]), float("nan"), dtype=torch.float32, device="cuda")
    _say("[step] stb_dequant")
    S.stb_dequant(c["pm"].dev_layout, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert (got.view(np.uint32) == c["What"].view(np.uint32)).all()


def test_index_words_of_the_sparse_kernels_are_the_meta_index_small(small_case, torch_cuda):
    """App. C: the uint16 meta index E.  The 2:4 kernels make their index operand from the mask bits in registers;
    the same function, run over the whole layer, must give the oracle's E bit for bit."""
    torch = torch_cuda
    c = small_case
    if not (c["tiled"] and (c["N"], c["M"]) == (2, 4)):
        E_dev = torch.zeros((c["n"], c["k"] // 16), dtype=torch.int16, device="cuda")
        with pytest.raises(S.StbError) as e:
            S.stb_code24_index(c["pm"].dev_layout, E_dev)
        assert e.value.status == (S.STB_EINVAL if not c["tiled"] else S.STB_EUNSUPPORTED)
        return
    n, k = c["n"], c["k"]
    mask = np.unpackbits(c["ref"]["mask"], axis=1, bitorder="little")[:, :k].astype(bool)
    slots = np.unpackbits(c["ref"]["sign"], axis=1, bitorder="little")[:, :k // 2]
    E_ref, V_ref = O.code24_encode(mask, slots)
    E_dev = torch.full((n, k // 16), -1, dtype=torch.int16, device="cuda")
    _say("[step] stb_code24_index")
    S.stb_code24_index(c["pm"].dev_layout, E_dev)
    torch.cuda.synchronize()
    assert (E_dev.cpu().numpy().view(np.uint16) == E_ref).all()
    # and the host export of the same layer agrees with both
    E_host, V_host = S.stb_code24_export(c["pm"].host_layout)
    assert (E_host == E_ref).all() and (V_host == V_ref).all()


@pytest.mark.parametrize("B", [1, 2, 3, 5, 8, 16, 31, 32])
@pytest.mark.parametrize("y_fp32", [False, True])
def test_gemv_small(small_case, torch_cuda, B, y_fp32):
    torch = torch_cuda
    c = small_case
    x = make_x(B, c["k"], c["seed"])
    y_ref, bound = O.matmul(x, c["What"])
    xd = torch.from_numpy(x).cuda()
    yd = torch.full((B, c["n"]), float("nan"), dtype=torch.float32 if y_fp32 else torch.float16, device="cuda")
    _say(f"[step] stb_gemv B={B} fp32={y_fp32}")
    S.stb_gemv(c["pm"].dev_layout, xd, B, yd, y_fp32, c["pm"].workspace)
    torch.cuda.synchronize()
    _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"gemv B={B}")
    if c["tiled"]:
        # the tiled order has two decode kernels; ordinary shapes all go to the one with fat wavefronts, so the
        # other one is asked for through the test hook
        yd.fill_(float("nan"))
        with forced(gemv_kernel=S.GEMV_THIN):
            _say(f"[step] stb_gemv B={B} fp32={y_fp32}, thin-wavefront kernel")
            S.stb_gemv(c["pm"].dev_layout, xd, B, yd, y_fp32, c["pm"].workspace)
            torch.cuda.synchronize()
        _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"gemv B={B} (thin-wavefront kernel)")
        # ... and small layers never choose several superblock visits per wavefront themselves
        for visits in (2, 3, 5, 8):
            if (c["k"] + 511) // 512 < visits or B > 16:
                continue
            yd.fill_(float("nan"))
            with forced(gemv_visits=visits):
                _say(f"[step] stb_gemv B={B} fp32={y_fp32}, {visits} visits per wavefront")
                S.stb_gemv(c["pm"].dev_layout, xd, B, yd, y_fp32, c["pm"].workspace)
                torch.cuda.synchronize()
            _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"gemv B={B} ({visits} visits per wavefront)")


def test_gemv_with_planes_more_than_4_gib_apart(torch_cuda):
    """The default decode kernel addresses the streamed planes of a layer from one scalar base with 32-bit offsets, so
    it takes a layout only if its planes lie within 4 GiB of each other; any other layout (planes bound one by one to
    separate allocations, say) must still give the product, through the kernel with 64-bit plane addresses."""
    torch = torch_cuda
    n, k, N, M = 130, 640, 4, 8
    L = make_layer(n, k, 77, "x8")
    What = O.unpack(O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 0), n, k, N, M)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 0)
    lay, img = pm.host_pair(True)
    far = (9 << 29)                                                   # 4.5 GiB, a multiple of the plane alignment
    big = torch.empty(far + 2 * lay.image_bytes + 4096, dtype=torch.uint8, device="cuda")
    off = (-big.data_ptr()) % 256
    near_view = big[off:off + lay.image_bytes]
    far_view = big[off + far:off + far + lay.image_bytes]
    near_view.copy_(torch.from_numpy(img))
    far_view.copy_(torch.from_numpy(img))
    dl = pm.clone_layout_for(far_view.data_ptr(), True)               # every plane in the far copy ...
    dl.mask = near_view.data_ptr() + dl.off_mask                      # ... except the mask plane
    assert abs(dl.mask - dl.sign) > (1 << 32)
    ws = pm.new_workspace()
    for B in (1, 7, 16):
        x = make_x(B, k, 78)
        y_ref, bound = O.matmul(x, What)
        xd = torch.from_numpy(x).cuda()
        yd = torch.full((B, n), float("nan"), dtype=torch.float32, device="cuda")
        _say(f"[step] stb_gemv B={B}, mask plane 4.5 GiB away from the other planes")
        S.stb_gemv(dl, xd, B, yd, True, ws)
        torch.cuda.synchronize()
        _within_bound(yd.cpu().numpy(), y_ref, bound, f"gemv B={B}, planes far apart")


@pytest.mark.parametrize("T", [1, 63, 64, 200, 333])
def test_gemm_small(small_case, torch_cuda, T):
    torch = torch_cuda
    c = small_case
    x = make_x(T, c["k"], c["seed"] + 1)
    y_ref, bound = O.matmul(x, c["What"])
    xd = torch.from_numpy(x).cuda()
    for y_fp32 in (False, True):
        yd = torch.full((T, c["n"]), float("nan"), dtype=torch.float32 if y_fp32 else torch.float16, device="cuda")
        _say(f"[step] stb_gemm T={T} fp32={y_fp32}")
        S.stb_gemm(c["pm"].dev_layout, xd, T, yd, y_fp32, c["pm"].new_gemm_workspace(T))
        torch.cuda.synchronize()
        _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"gemm T={T}")
        # The library picks one kernel per tiled layer (2:4: the sparse matrix instruction 32x32x32; otherwise the dense
        # 16x16x32 one); the others that can take the layer (the 32x32x16 form, the kernel that shares the expanded
        # operands through LDS, the dense one and the other sparse form on 2:4 layers) are asked for through the test
        # hook.
        others = []
        if c["tiled"]:
            others += ["dense32", "shared"]
            if (c["N"], c["M"]) == (2, 4):
                others += ["dense", "sparse16"]
        for which in others:
            yd.fill_(float("nan"))
            with forced(gemm_kernel=GEMM_KERNELS[which]):
                _say(f"[step] stb_gemm T={T} fp32={y_fp32}, kernel asked for: {which}")
                S.stb_gemm(c["pm"].dev_layout, xd, T, yd, y_fp32, c["pm"].new_gemm_workspace(T))
                torch.cuda.synchronize()
            _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"gemm T={T} (kernel asked for: {which})")


@pytest.mark.parametrize("N,M", [(4, 8), (2, 4), (6, 8)])
def test_gemm_with_a_k_split_is_reproducible_and_matches_the_oracle(N, M, torch_cuda):
    # few tokens on a wide layer: the superblocks are dealt to groups of workgroups whose fp32 partial tiles a second
    # kernel adds in a fixed order (9 superblocks here, the last group is ragged)
    torch = torch_cuda
    n, k, T = 300, 4608, 70
    _say(f"[case] gemm K split {n}x{k} {N}:{M} T={T}")
    L = make_layer(n, k, 120 + N, "x8")
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 0).to_device(tiled=True)
    What = O.unpack(_oracle_planes_from(pm), n, k, N, M)
    x = make_x(T, k, 121)
    y_ref, bound = O.matmul(x, What)
    xd = torch.from_numpy(x).cuda()
    ws = pm.new_gemm_workspace(T)
    assert ws is not None and ws.numel() >= 2 * T * n * 4          # room for at least two partial tiles
    outs = []
    for y_fp32 in (False, True, True):
        ws.fill_(0x7F)                                                 # the workspace needs no initialisation
        yd = torch.full((T, n), float("nan"), dtype=torch.float32 if y_fp32 else torch.float16, device="cuda")
        S.stb_gemm(pm.dev_layout, xd, T, yd, y_fp32, ws)
        torch.cuda.synchronize()
        outs.append(yd.cpu().numpy())
        _within_bound(outs[-1], y_ref, bound, f"gemm K split fp32={y_fp32}")
    assert (outs[1].view(np.uint32) == outs[2].view(np.uint32)).all()


def test_zero_activations_and_zero_weights(torch_cuda):
    torch = torch_cuda
    n, k = 70, 256
    L = make_layer(n, k, 7)
    pm = S.PackedMatrix.pack(np.zeros((n, k), np.float32), L["xnorm"], L["sal_bitmap"], 4, 8, 0).to_device()
    xd = torch.from_numpy(make_x(4, k, 7)).cuda()
    yd = torch.full((4, n), float("nan"), dtype=torch.float16, device="cuda")
    S.stb_gemv(pm.dev_layout, xd, 4, yd, False, pm.workspace)
    torch.cuda.synchronize()
    assert (yd.cpu().numpy() == 0).all()
    pm2 = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 4, 8, 0).to_device()
    yd = torch.full((4, n), float("nan"), dtype=torch.float32, device="cuda")
    S.stb_gemv(pm2.dev_layout, torch.zeros_like(xd), 4, yd, True, pm2.workspace)
    torch.cuda.synchronize()
    assert (yd.cpu().numpy() == 0).all()


def test_probe_mfma_runs_and_rejects_bad_arguments(torch_cuda):
    torch = torch_cuda
    sink = torch.zeros(4 * 4096, dtype=torch.uint8, device="cuda")
    for kind in range(8):
        for valu in (0, 2, 3, 5, 8):
            S.stb_probe_mfma(kind, valu, 3, 4, sink)
    torch.cuda.synchronize()
    # (the last launch, random operands of magnitude below 2 on zeroed accumulators: every sum is finite)
    out = sink.view(torch.float32).cpu().numpy()
    assert np.isfinite(out).all()
    for bad in ((8, 0, 3, 4), (-1, 0, 3, 4), (0, 1, 3, 4), (2, 4, 3, 4), (0, 0, 0, 4), (0, 0, 3, 0)):
        with pytest.raises(S.StbError) as e:
            S.stb_probe_mfma(*bad, sink)
        assert e.value.status == S.STB_EINVAL


def test_device_entry_points_reject_bad_arguments(torch_cuda):
    torch = torch_cuda
    L = make_layer(16, 128, 9)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 0).to_device()
    xd = torch.zeros((33, 128), dtype=torch.float16, device="cuda")
    yd = torch.zeros((33, 16), dtype=torch.float16, device="cuda")
    for B in (0, 33, -1):
        with pytest.raises(S.StbError) as e:
            S.stb_gemv(pm.dev_layout, xd, B, yd)
        assert e.value.status == S.STB_EINVAL
    with pytest.raises(S.StbError) as e:
        S.stb_gemm(pm.dev_layout, xd, 0, yd)
    assert e.value.status == S.STB_EINVAL
    unbound = S.stb_layout_sizes(pm.cfg)
    with pytest.raises(S.StbError) as e:
        S.stb_gemv(unbound, xd, 1, yd)
    assert e.value.status == S.STB_ENULL


# --------------------------------------------------------------------------------------------------
# several layers in one launch
# --------------------------------------------------------------------------------------------------
def _bits(t):
    a = t.cpu().numpy()
    return a.view(np.uint32 if a.dtype == np.float32 else np.uint16)


@pytest.mark.parametrize("B", [1, 3, 16, 21])
def test_gemv_batched_is_one_launch_with_reproducible_bits(torch_cuda, B):
    """A list of layers that differ in everything (N:M, rows, columns, column splits, salient columns or none, a shared
    input vector) through stb_gemv_batched: against the oracle, and bit for bit against a second call (a layer's launch
    shape, and with it the order of its partial sums, depends on its share of the launch, not on timing)."""
    torch = torch_cuda
    shapes = [(130, 1024, 6, 8, 1, 0.05), (40, 1024, 6, 8, 0, 0.05), (257, 4608, 2, 4, 0, 0.05), (64, 512, 4, 8, 0, 0.0),
              (17, 9728, 4, 8, 1, 0.02), (5, 128, 2, 4, 0, 0.05), (100, 1024, 4, 8, 0, 0.1), (33, 640, 6, 8, 1, 0.0),
              (48, 1024, 2, 4, 1, 0.15), (96, 512, 5, 8, 0, 0.05)]
    layers = []
    xs_by_k = {}
    for j, (n, k, N, M, mode, frac) in enumerate(shapes):
        L = make_layer(n, k, 300 + j, "x8", n_salient=int(frac * k))
        What = O.unpack(O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode), n, k, N, M)
        pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode).to_device(tiled=_tiled_ok(N, M))
        if k not in xs_by_k:
            x = make_x(B, k, 300 + k)
            xs_by_k[k] = (x, torch.from_numpy(x).cuda())
        layers.append(dict(n=n, k=k, pm=pm, What=What))
    for sel, what in ((range(9), "nine tiled layers: two launches"), (range(3), "three layers"), (range(10), "a row-major layer in the list"),
                      ([4], "one layer")):
        sel = list(sel)
        for y_fp32 in (False, True):
            dt = torch.float32 if y_fp32 else torch.float16
            ys = [torch.full((B, layers[j]["n"]), float("nan"), dtype=dt, device="cuda") for j in sel]
            ws = S.new_device_scratch(S.stb_gemv_batched_workspace_bytes([layers[j]["pm"].cfg for j in sel], B), zero=True)
            first = None
            for rnd in range(2):                       # twice on the same workspace: the counters are left zero
                for yb in ys:
                    yb.fill_(float("nan"))
                _say(f"[step] stb_gemv_batched B={B} fp32={y_fp32}: {what}, call {rnd}")
                S.stb_gemv_batched([layers[j]["pm"].dev_layout for j in sel], [xs_by_k[layers[j]["k"]][1] for j in sel], B, ys,
                                   y_fp32, ws)
                torch.cuda.synchronize()
                for j, yb in zip(sel, ys):
                    ly = layers[j]
                    y_ref, bound = O.matmul(xs_by_k[ly["k"]][0], ly["What"])
                    _within_bound(yb.float().cpu().numpy(), y_ref, bound, f"batched gemv layer {j} B={B}")
                bits = [_bits(yb).copy() for yb in ys]
                if first is None:
                    first = bits
                else:
                    assert all((a == b).all() for a, b in zip(first, bits)), "two identical calls gave different bits"
            if len(sel) == 1:                          # a list of one layer is the single call
                ly = layers[sel[0]]
                y1 = torch.full((B, ly["n"]), float("nan"), dtype=dt, device="cuda")
                # (with a workspace sized for 16 rows: above 16 rows stb_gemv then runs the decode kernel twice, as the
                #  batched call does, instead of one pass of the prefill kernel)
                ws1 = S.new_device_scratch(S.stb_gemv_workspace_bytes(ly["pm"].cfg, min(B, 16)), zero=True)
                S.stb_gemv(ly["pm"].dev_layout, xs_by_k[ly["k"]][1], B, y1, y_fp32, ws1)
                torch.cuda.synchronize()
                assert (_bits(ys[0]) == _bits(y1)).all()


def test_decode_calls_captured_in_a_hip_graph_replay_with_the_eager_bits(torch_cuda):
    # stb_gemv / stb_gemv_batched / stb_gemv_static enqueue kernels only (no memset, no allocation, no synchronisation),
    # so a serving loop may capture them once and replay: every replay, with eager work and synchronisations between
    # the replays, must give the bits of the eager calls (the arrival counters of the column splits return to zero
    # by themselves)
    torch = torch_cuda
    specs = [(200, 4608, 2, 4, 131), (96, 4608, 4, 8, 132), (130, 1024, 6, 8, 133)]
    B = 3
    pms, xs, refs = [], [], []
    for n, k, N, M, seed in specs:
        L = make_layer(n, k, seed, "x8")
        pms.append(S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 0).to_device(tiled=True))
        xs.append(torch.from_numpy(make_x(B, k, seed)).cuda())
    ws = S.new_device_scratch(S.stb_gemv_batched_workspace_bytes([pm.cfg for pm in pms], B), zero=True)
    ws1 = pms[0].new_workspace()

    def step(ys, y_single, y_static):
        S.stb_gemv_batched([pm.dev_layout for pm in pms], xs, B, ys, True, ws)
        S.stb_gemv(pms[0].dev_layout, xs[0], B, y_single, True, ws1)
        S.stb_gemv_static(pms[0].dev_layout, xs[0], B, y_static, True)

    def fresh():
        return ([torch.full((B, pm.cfg.n_out), float("nan"), dtype=torch.float32, device="cuda") for pm in pms],
                torch.full((B, pms[0].cfg.n_out), float("nan"), dtype=torch.float32, device="cuda"),
                torch.full((B, pms[0].cfg.n_out), float("nan"), dtype=torch.float32, device="cuda"))

    eager = fresh()
    step(*eager)
    torch.cuda.synchronize()
    want = [t.cpu().numpy().copy() for t in eager[0]] + [eager[1].cpu().numpy().copy(), eager[2].cpu().numpy().copy()]
    assert all(np.isfinite(w).all() for w in want)
    outs = fresh()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            step(*outs)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        for t in outs[0] + [outs[1], outs[2]]:
            t.fill_(float("nan"))
        scratch = fresh()
        step(*scratch)                                   # eager work of the program itself between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in outs[0]] + [outs[1].cpu().numpy(), outs[2].cpu().numpy()]
        for a, b in zip(got, want):
            assert (a.view(np.uint32) == b.view(np.uint32)).all(), f"replay {replay}"


def test_gemv_batched_rejects_bad_arguments(torch_cuda):
    torch = torch_cuda
    L = make_layer(40, 4608, 9)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 1).to_device(tiled=True)
    xd = torch.zeros((1, 4608), dtype=torch.float16, device="cuda")
    yd = torch.zeros((1, 40), dtype=torch.float16, device="cuda")
    need = S.stb_gemv_batched_workspace_bytes([pm.cfg, pm.cfg], 1)
    assert need == 2 * S.stb_gemv_batched_workspace_bytes([pm.cfg], 1) and need % 256 == 0
    small = S.new_device_scratch(need - 256, zero=True)
    with pytest.raises(S.StbError) as e:
        S.stb_gemv_batched([pm.dev_layout, pm.dev_layout], [xd, xd], 1, [yd, yd], False, small)
    assert e.value.status == S.STB_EINVAL
    with pytest.raises(S.StbError) as e:
        S.stb_gemv_batched([pm.dev_layout], [xd], 33, [yd], False, small)
    assert e.value.status == S.STB_EINVAL


def test_decode_is_bitwise_reproducible_across_launch_shapes(torch_cuda):
    """The reduction order of the decode kernels is fixed (wavefronts in order inside a workgroup, column splits in
    order through the workspace): repeated calls give identical bits, and so do calls whose workgroups run in another
    order because other layers share the launch."""
    torch = torch_cuda
    n, k, B = 200, 9728, 5
    L = make_layer(n, k, 77, "t3")
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 0).to_device(tiled=True)
    L2 = make_layer(64, k, 78)
    pm2 = S.PackedMatrix.pack(L2["W"], L2["xnorm"], L2["sal_bitmap"], 4, 8, 0).to_device(tiled=True)
    xd = torch.from_numpy(make_x(B, k, 77)).cuda()
    outs = []
    for rep in range(3):
        y = torch.full((B, n), float("nan"), dtype=torch.float32, device="cuda")
        S.stb_gemv(pm.dev_layout, xd, B, y, True, pm.workspace)
        torch.cuda.synchronize()
        outs.append(_bits(y))
    for o in outs[1:]:
        assert (o == outs[0]).all()
    # as one of three layers of a launch: its workgroups run among the others', and twice gives the same bits; the two
    # copies of the other layer in the launch agree with each other
    ws = S.new_device_scratch(S.stb_gemv_batched_workspace_bytes([pm2.cfg, pm.cfg, pm2.cfg], B), zero=True)
    grouped = []
    for rep in range(2):
        y = torch.full((B, n), float("nan"), dtype=torch.float32, device="cuda")
        ya, yb = (torch.full((B, 64), float("nan"), dtype=torch.float32, device="cuda") for _ in range(2))
        S.stb_gemv_batched([pm2.dev_layout, pm.dev_layout, pm2.dev_layout], [xd, xd, xd], B, [ya, y, yb], True, ws)
        torch.cuda.synchronize()
        grouped.append(_bits(y).copy())
        assert (_bits(ya) == _bits(yb)).all()
    assert (grouped[0] == grouped[1]).all()


# --------------------------------------------------------------------------------------------------
# random shapes: every kernel that can take a layer, on shapes nobody chose by hand
# --------------------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_shapes_through_every_kernel(seed, torch_cuda):
    torch = torch_cuda
    rng = np.random.default_rng(seed)
    for case in range(6):
        N, M = [(2, 4), (4, 8), (6, 8), (2, 4)][rng.integers(0, 4)]
        n = int(rng.integers(1, 500))
        k = 128 * int(rng.integers(1, 44))
        n_sal = int(rng.choice([0, max(1, k // 20), max(1, k // 8), min(k, 40)]))
        mode = int(rng.integers(0, 2))
        lseed = int(rng.integers(0, 1 << 30))
        _say(f"[case] random {seed}/{case}: n={n} k={k} {N}:{M} salient={n_sal} mode={mode} seed={lseed}")
        L = make_layer(n, k, lseed, "x8", n_salient=n_sal)
        What = O.unpack(O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode), n, k, N, M)
        pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode).to_device(tiled=True)

        def run(hook, call):
            with forced(**hook):
                call()
                torch.cuda.synchronize()

        for B in sorted({int(b) for b in rng.integers(1, 33, 2)}):
            x = make_x(B, k, lseed + B)
            y_ref, bound = O.matmul(x, What)
            xd = torch.from_numpy(x).cuda()
            asks = [{}, dict(gemv_kernel=S.GEMV_THIN)]
            asks += [dict(gemv_visits=v) for v in (2, 3, 4, 7) if (k + 511) // 512 >= v and B <= 16]
            for hook in asks:
                yd = torch.full((B, n), float("nan"), dtype=torch.float16, device="cuda")
                _say(f"[step] stb_gemv B={B} {hook}")
                run(hook, lambda: S.stb_gemv(pm.dev_layout, xd, B, yd, False, pm.workspace))
                _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"random gemv B={B} {hook}")
        for T in sorted({int(t) for t in rng.integers(1, 300, 2)}):
            x = make_x(T, k, lseed + 1000 + T)
            y_ref, bound = O.matmul(x, What)
            xd = torch.from_numpy(x).cuda()
            for value in [None, "dense32", "shared"] + (["dense", "sparse16"] if (N, M) == (2, 4) else []):
                yd = torch.full((T, n), float("nan"), dtype=torch.float16, device="cuda")
                _say(f"[step] stb_gemm T={T} kernel asked for: {value}")
                run(dict(gemm_kernel=GEMM_KERNELS[value]) if value else {},
                    lambda: S.stb_gemm(pm.dev_layout, xd, T, yd, False, pm.new_gemm_workspace(T)))
                _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"random gemm T={T} kernel={value}")


# --------------------------------------------------------------------------------------------------
# a stack of layers at the N:8 that the layer-wise assignment gives each of them (Sec. 3.3)
# --------------------------------------------------------------------------------------------------
def test_layer_wise_assignment_feeds_the_kernels(torch_cuda):
    torch = torch_cuda
    shapes = [(96, 512), (64, 384), (130, 256), (48, 1024), (80, 640)]
    scales = [0.2, 1.0, 3.0, 0.5, 9.0]
    layers = [make_layer(n, k, 70 + i) for i, (n, k) in enumerate(shapes)]
    for L, c in zip(layers, scales):
        L["W"] = (L["W"] * np.float32(c)).astype(np.float32)
    om = [S.stb_layer_l2_norm(L["W"]) for L in layers]
    N = S.stb_layer_nm_assignment(om, 0.375, 8)                 # target 3:8
    assert N.tolist() == O.layer_nm_assignment([O.layer_l2_norm(L["W"]) for L in layers], 0.375, 8)[0].tolist()
    assert len(set(N.tolist())) >= 3, N                         # the stack really is mixed
    _say(f"[case] layer-wise assignment: N of 8 = {N.tolist()}")
    for (n, k), L, Ni in zip(shapes, layers, N.tolist()):
        sal = S.stb_salient_columns(L["W"], L["xnorm"], 0.01, 16)
        assert (O.bitmap_to_bool(sal, k) == O.salient_columns(L["W"], L["xnorm"], 0.01, 16)).all()
        ref = O.pack(L["W"], L["xnorm"], sal, Ni, 8, 0)
        What = O.unpack(ref, n, k, Ni, 8)
        pm = S.PackedMatrix.pack(L["W"], L["xnorm"], sal, Ni, 8, 0).to_device(tiled=_tiled_ok(Ni, 8))
        for B in (1, 7):
            x = make_x(B, k, 7 * Ni + B)
            y_ref, bound = O.matmul(x, What)
            yd = torch.full((B, n), float("nan"), dtype=torch.float16, device="cuda")
            _say(f"[step] stb_gemv {n}x{k} {Ni}:8 B={B}")
            S.stb_gemv(pm.dev_layout, torch.from_numpy(x).cuda(), B, yd, False, pm.workspace)
            torch.cuda.synchronize()
            _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"assigned {Ni}:8 gemv B={B}")
        T = 70
        x = make_x(T, k, 11 * Ni)
        y_ref, bound = O.matmul(x, What)
        yd = torch.full((T, n), float("nan"), dtype=torch.float16, device="cuda")
        _say(f"[step] stb_gemm {n}x{k} {Ni}:8 T={T}")
        S.stb_gemm(pm.dev_layout, torch.from_numpy(x).cuda(), T, yd, False, pm.new_gemm_workspace(T))
        torch.cuda.synchronize()
        _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"assigned {Ni}:8 gemm T={T}")


# --------------------------------------------------------------------------------------------------
# full-size workloads
# --------------------------------------------------------------------------------------------------
def _layer_key(cfg, spec):
    return (f"cfg{cfg}_{spec.name}_{spec.n}x{spec.k}_{spec.N}of{spec.M}"
            f"_mode{spec.region_mode}_{spec.salient_kind}_seed{spec.seed}")


FULL = [(cfg, i) for cfg, wl in WORKLOADS.items() for i in range(len(wl["layers"]))]


@pytest.mark.parametrize("cfg,idx", FULL, ids=lambda v: str(v))
def test_full_size_layer(cfg, idx, torch_cuda):
    """One layer of a workload at full size: the library's packed planes against the oracle's digests,
    GPU dequantisation against the oracle's decode of those bytes, then every decode batch and prefill
    length of the workload against the oracle's float64 product (prefill: on sampled tokens)."""
    torch = torch_cuda
    wl = WORKLOADS[cfg]
    spec = wl["layers"][idx]
    key = _layer_key(cfg, spec)
    _say(f"[case] full {key}")
    digests = json.load(open(GOLDEN)) if os.path.exists(GOLDEN) else {}
    L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
    if key not in digests:
        pytest.skip(f"no oracle digest stored for {key}")
    for name, _, _ in S.PLANE_FIELDS:
        assert hashlib.sha256(pm.plane(name).tobytes()).hexdigest() == digests[key][name], name
    assert pm.packed_bytes == digests[key]["total_bytes"]
    _say("[step] packed planes match the oracle digests")
    _say("[step] stb_pack_device")
    import time
    t0 = time.time()
    dp = _pack_on_device(torch, L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
    _say(f"       {time.time() - t0:.2f} s with the copies to and from the device")
    for name, _, _ in S.PLANE_FIELDS:
        assert hashlib.sha256(dp.plane(name).tobytes()).hexdigest() == digests[key][name], ("device packer", name)
    del L, dp
    torch.cuda.empty_cache()
    _say("[step] the device packer's planes match the oracle digests")

    What = O.unpack(_oracle_planes_from(pm), spec.n, spec.k, spec.N, spec.M)
    tiled = _tiled_ok(spec.N, spec.M)
    row_major = S.PackedMatrix.__new__(S.PackedMatrix)
    row_major.__dict__.update(pm.__dict__)
    row_major.to_device(tiled=False)
    if tiled:
        pm.to_device(tiled=True)
    else:
        pm = row_major
    if tiled:
        _say("[step] stb_tile_device")
        tl_host, timg_host = pm.tiled()
        timg = S.new_device_scratch(tl_host.image_bytes)
        tlay = S.stb_tiled_sizes(pm.cfg)
        S.stb_layout_bind(tlay, timg.data_ptr())
        S.stb_tile_device(row_major.dev_layout, tlay)
        assert (tlay.max_sal_block, tlay.max_sal_half) == (tl_host.max_sal_block, tl_host.max_sal_half)
        got = timg.cpu().numpy()
        for name, off, size in S.PLANE_FIELDS + (("sal_tab", "off_saltab", "saltab_bytes"), ("res_t", "off_res_t", "res_t_bytes")):
            o, sz = getattr(tl_host, off), getattr(tl_host, size)
            assert (got[o:o + sz] == timg_host[o:o + sz]).all(), ("device tiling", name)
        del timg, got
        torch.cuda.empty_cache()
    for which, holder in (("row-major", row_major), ("tiled", pm if tiled else None)):
        if holder is None:
            continue
        out = torch.empty((spec.n, spec.k), dtype=torch.float32, device="cuda")
        _say(f"[step] stb_dequant {which}")
        S.stb_dequant(holder.dev_layout, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        del out
        assert (got.view(np.uint32) == What.view(np.uint32)).all(), which
        del got

    W64 = What.astype(np.float64)
    A64 = np.abs(W64)
    for B in wl["decode_batches"]:
        x = make_x(B, spec.k, spec.seed)
        x64 = x.astype(np.float64)
        y_ref, bound = x64 @ W64.T, np.abs(x64) @ A64.T
        xd = torch.from_numpy(x).cuda()
        yd = torch.full((B, spec.n), float("nan"), dtype=torch.float16, device="cuda")
        _say(f"[step] stb_gemv B={B}")
        S.stb_gemv(pm.dev_layout, xd, B, yd, False, pm.workspace)
        torch.cuda.synchronize()
        worst = _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"{key} gemv B={B}")
        _say(f"       worst error / bound = {worst:.2e}")
        if tiled and (cfg, idx) in ((2, 1), (5, 4), (3, 2)) and B <= 16:
            # the decode kernels and launch shapes that the library does not pick for this layer, at full size: the
            # thin-wavefront kernel, several superblock visits per wavefront, other numbers of column splits
            nsb = (spec.k + 511) // 512
            hooks = [dict(gemv_kernel=S.GEMV_THIN)] + [dict(gemv_visits=v) for v in (2, 3, 5) if v <= nsb]
            hooks += [dict(gemv_visits=1, gemv_splits=sp) for sp in (2, 4, 7) if sp <= nsb]
            for hook in hooks:
                yd.fill_(float("nan"))
                with forced(**hook):
                    S.stb_gemv(pm.dev_layout, xd, B, yd, False, pm.workspace)
                    torch.cuda.synchronize()
                worst = _within_bound(yd.float().cpu().numpy(), y_ref, bound, f"{key} gemv B={B} {hook}")
                _say(f"       {hook}: worst error / bound = {worst:.2e}")
    for T in wl["prefill_tokens"]:
        x = make_x(T, spec.k, spec.seed)
        # one token out of every tile of 16 (every workgroup and every matrix-instruction tile of every prefill kernel
        # is compared), plus the edges
        rng = np.random.default_rng(spec.seed + T)
        rows = np.unique(np.concatenate([[0, 1, 63, 64, T - 65, T - 2, T - 1], 16 * np.arange(T // 16) + rng.integers(0, 16, T // 16)]))
        x64 = x[rows].astype(np.float64)
        y_ref, bound = x64 @ W64.T, np.abs(x64) @ A64.T
        xd = torch.from_numpy(x).cuda()
        yd = torch.full((T, spec.n), float("nan"), dtype=torch.float16, device="cuda")
        _say(f"[step] stb_gemm T={T}")
        for which, holder in (("row-major", row_major), ("tiled", pm if tiled else None)):
            if holder is None:
                continue
            yd.fill_(float("nan"))
            S.stb_gemm(holder.dev_layout, xd, T, yd, False, holder.new_gemm_workspace(T))
            torch.cuda.synchronize()
            y = yd.float().cpu().numpy()
            assert np.isfinite(y).all()
            worst = _within_bound(y[rows], y_ref, bound, f"{key} gemm T={T} {which}")
            _say(f"       {which}: worst error / bound on {len(rows)} sampled tokens = {worst:.2e}")
        if tiled:
            # the prefill kernels that the library does not pick by itself, on the same tokens
            for asked in ["dense32", "shared"] + (["dense", "sparse16"] if (spec.N, spec.M) == (2, 4) else []):
                yd.fill_(float("nan"))
                with forced(gemm_kernel=GEMM_KERNELS[asked]):
                    S.stb_gemm(pm.dev_layout, xd, T, yd, False, pm.new_gemm_workspace(T))
                    torch.cuda.synchronize()
                y = yd.float().cpu().numpy()
                assert np.isfinite(y).all()
                worst = _within_bound(y[rows], y_ref, bound, f"{key} gemm T={T} tiled, kernel asked for: {asked}")
                _say(f"       tiled, {asked}: worst error / bound = {worst:.2e}")
