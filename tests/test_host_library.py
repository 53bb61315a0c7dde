"""CPU tests of libstb's host side: exports, closed-form layout, error codes, and the packer / host
dequantiser against the oracle, bit for bit, on shapes that span several blocks and ragged row counts.
No GPU call is made here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2408_01803_amd as S
from oracle import stb_oracle as O
from workloads import make_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _oracle_bytes(P):
    return {name: np.ascontiguousarray(v).view(np.uint8).ravel() for name, v in P.items()}


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "stb.h")).read()
    declared = set(re.findall(r"\b(stb_[a-z_0-9]+)\s*\(", header))
    declared -= {"stb_status"}
    assert declared == set(S.EXPORTS)
    lib = C.CDLL(S.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("n,k,N,M,S_", [(4096, 4096, 4, 8, 204), (11008, 4096, 2, 4, 204),
                                         (13824, 5120, 6, 8, 256), (28672, 8192, 4, 8, 409),
                                         (8192, 28672, 2, 4, 1433), (7, 128, 5, 8, 0)])
def test_layout_sizes_match_the_oracle_closed_form(n, k, N, M, S_):
    lay = S.stb_layout_sizes(S.make_cfg(n, k, N, M, S_))
    ref = O.layout_sizes(n, k, N, M, S_)
    for f in ("mask_stride", "sign_stride", "region_stride", "res_stride", "mask_bytes", "sign_bytes",
              "region_bytes", "res_bytes", "scales_bytes", "res_scale_bytes", "salmap_bytes",
              "salprefix_bytes", "total_bytes", "n_salient_pad", "n_blocks"):
        assert getattr(lay, f) == ref[f], f
    offs = [getattr(lay, o) for _, o, _ in S.PLANE_FIELDS]
    sizes = [getattr(lay, s) for _, _, s in S.PLANE_FIELDS]
    assert all(o % S.STB_PLANE_ALIGN == 0 for o in offs)
    assert all(offs[i] + sizes[i] <= offs[i + 1] for i in range(len(offs) - 1))
    assert offs[-1] + sizes[-1] <= lay.image_bytes


def test_error_codes():
    with pytest.raises(S.StbError) as e:
        S.stb_layout_sizes(S.make_cfg(16, 128, 3, 6, 0))
    assert e.value.status == S.STB_EINVAL
    for bad in (S.make_cfg(16, 100, 2, 4, 0), S.make_cfg(16, 128, 5, 4, 0), S.make_cfg(0, 128, 2, 4, 0),
                S.make_cfg(16, 128, 0, 4, 0), S.make_cfg(16, 128, 2, 4, 0, region_mode=2)):
        with pytest.raises(S.StbError) as e:
            S.stb_layout_sizes(bad)
        assert e.value.status == S.STB_EINVAL
    L = make_layer(8, 128, 3)
    # n_salient that does not match the bitmap
    pm = S.PackedMatrix(S.make_cfg(8, 128, 2, 4, 2))
    with pytest.raises(S.StbError) as e:
        S.stb_pack(L["W"], L["xnorm"], L["sal_bitmap"], pm.host_layout)
    assert e.value.status == S.STB_EINVAL
    W = L["W"].copy()
    W[3, 5] = np.nan
    with pytest.raises(S.StbError) as e:
        S.PackedMatrix.pack(W, L["xnorm"], L["sal_bitmap"], 2, 4)
    assert e.value.status == S.STB_ENONFINITE
    xn = L["xnorm"].copy()
    xn[0] = -1.0
    with pytest.raises(S.StbError) as e:
        S.PackedMatrix.pack(L["W"], xn, L["sal_bitmap"], 2, 4)
    assert e.value.status == S.STB_ENONFINITE
    # unbound layout -> NULL planes
    lay = S.stb_layout_sizes(S.make_cfg(8, 128, 2, 4, 6))
    with pytest.raises(S.StbError) as e:
        S.stb_unpack(lay)
    assert e.value.status == S.STB_ENULL
    # misaligned base
    buf = S.aligned_bytes(lay.image_bytes + 64)
    with pytest.raises(S.StbError) as e:
        S.stb_layout_bind(lay, buf.ctypes.data + 8)
    assert e.value.status == S.STB_EALIGN
    assert "NULL" in str(e.value) or "align" in str(e.value)


CASES = [
    # n, k, N, M, mode, salient kind, seed
    (64, 256, 4, 8, 0, "x8", 1),
    (48, 512, 2, 4, 0, "t3", 2),
    (40, 384, 6, 8, 1, "x8", 3),
    (33, 256, 5, 8, 0, "x8", 4),
    (16, 128, 8, 8, 0, "x8", 5),
    (130, 640, 4, 8, 1, "t3", 6),
    (17, 1024, 2, 4, 1, "x8", 7),
    (1, 128, 1, 4, 0, "x8", 8),
    (24, 384, 3, 8, 0, "x8", 10),
]


@pytest.mark.parametrize("n,k,N,M,mode,kind,seed", CASES)
def test_packer_and_host_dequant_are_bit_exact_against_the_oracle(n, k, N, M, mode, kind, seed):
    L = make_layer(n, k, seed, kind)
    P = _oracle_bytes(O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode))
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode, n_threads=3)
    for name, ref in P.items():
        got = pm.plane(name)
        assert got.shape == ref.shape, name
        assert (got == ref).all(), name
    assert pm.packed_bytes == sum(v.size for v in P.values())
    ref_planes = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    assert (pm.unpack() == O.unpack(ref_planes, n, k, N, M)).all()


def _calibration_factor(k, seed, mix=0.6):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((2 * k, k)) @ (np.eye(k) + mix * rng.standard_normal((k, k)) / np.sqrt(k))
    return X, O.hessian_factor(X, 0.01 * np.mean(np.diag(2.0 * X.T @ X)))


@pytest.mark.parametrize("n,k,N,M,mode,kind,seed", [c for c in CASES if c[1] > 128] + [(16, 128, 4, 8, 0, "x8", 9)])
@pytest.mark.parametrize("compensate", [True, False])
def test_block_loop_packer_is_bit_exact_against_the_oracle(n, k, N, M, mode, kind, seed, compensate):
    # Alg. 1 with its block loop: per-slice Standardized Importance, and (with a factor) the compensation of the
    # later columns, whose float64 sums must follow the stated order for every later decision to agree
    L = make_layer(n, k, seed, kind)
    Hc = _calibration_factor(k, seed + 500)[1] if compensate else None
    ref = O.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode)
    pm = S.PackedMatrix.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode, n_threads=3)
    for name, v in _oracle_bytes(ref).items():
        got = pm.plane(name)
        assert got.shape == v.shape, name
        assert (got == v).all(), name
    assert (pm.unpack() == O.unpack(ref, n, k, N, M)).all()
    one = S.PackedMatrix.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], N, M, mode, n_threads=1)
    assert (one.host_image == pm.host_image).all()


def test_block_loop_packer_lowers_the_output_error_and_checks_its_factor():
    n, k = 64, 768
    L = make_layer(n, k, 31, "x8")
    X, Hc = _calibration_factor(k, 32, mix=0.8)
    W = L["W"].astype(np.float64)
    plain = S.PackedMatrix.pack_obc(L["W"], None, L["xnorm"], L["sal_bitmap"], 4, 8).unpack()
    comp = S.PackedMatrix.pack_obc(L["W"], Hc, L["xnorm"], L["sal_bitmap"], 4, 8).unpack()
    assert np.linalg.norm(X @ (W - comp).T) < 0.97 * np.linalg.norm(X @ (W - plain).T)
    bad = Hc.copy()
    bad[5, 5] = 0.0
    with pytest.raises(S.StbError) as e:
        S.PackedMatrix.pack_obc(L["W"], bad, L["xnorm"], L["sal_bitmap"], 4, 8)
    assert e.value.status == S.STB_ENONFINITE
    bad[5, 5] = np.nan
    with pytest.raises(S.StbError):
        S.PackedMatrix.pack_obc(L["W"], bad, L["xnorm"], L["sal_bitmap"], 4, 8)


def test_packer_result_does_not_depend_on_thread_count():
    L = make_layer(96, 512, 17)
    a = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 4, 8, 0, n_threads=1)
    b = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 4, 8, 0, n_threads=7)
    assert (a.host_image == b.host_image).all()


def test_packer_edge_cases_zero_matrix_no_salient_and_all_salient_block():
    k = 256
    # all-zero weights: ties keep the first N of each group, kept zeros carry +scale = +0
    Z = np.zeros((4, k), dtype=np.float32)
    none = np.zeros(k // 32, dtype=np.uint32)
    pm = S.PackedMatrix.pack(Z, np.ones(k, dtype=np.float32), none, 2, 4, 0)
    ref = O.pack(Z, np.ones(k, dtype=np.float32), none, 2, 4, 0)
    for name, v in _oracle_bytes(ref).items():
        assert (pm.plane(name) == v).all(), name
    assert (pm.unpack() == 0).all()
    # a block whose 128 columns are all salient (no non-salient weight there), and zero xnorm entries
    L = make_layer(9, k, 23, n_salient=0)
    bm = np.zeros(k // 32, dtype=np.uint32)
    bm[4:8] = 0xFFFFFFFF
    xn = L["xnorm"].copy()
    xn[::7] = 0.0
    pm = S.PackedMatrix.pack(L["W"], xn, bm, 6, 8, 0)
    ref = O.pack(L["W"], xn, bm, 6, 8, 0)
    for name, v in _oracle_bytes(ref).items():
        assert (pm.plane(name) == v).all(), name
    assert (pm.unpack() == O.unpack(ref, 9, k, 6, 8)).all()


@pytest.mark.parametrize("n,k,N,M,mode,kind,seed", CASES)
def test_tile_untile_round_trip_is_a_byte_permutation(n, k, N, M, mode, kind, seed):
    L = make_layer(n, k, seed, kind)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, mode)
    tl, timg = pm.tiled()
    assert tl.kind == S.STB_KIND_TILED and tl.n_row_tiles == (n + 15) // 16 and tl.n_super == (k // 128 + 3) // 4
    # 3 or 5 kept of 8: the tiled order holds the sign bits and ids in the slots of 4 / 6 of 8, one slot per group unused
    padded = M == 8 and N in (3, 5)
    t8 = N + 1 if padded else None
    # same multiset of payload bytes: sorted bytes of each per-row plane agree up to zero padding
    for name, off, size in (("mask", "off_mask", "mask_bytes"), ("sign", "off_sign", "sign_bytes"),
                            ("region", "off_region", "region_bytes"), ("scales", "off_scales", "scales_bytes"),
                            ("res_scale", "off_res_scale", "res_scale_bytes")):
        if padded and name in ("sign", "region"):
            continue
        a = np.sort(pm.plane(name))
        b = np.sort(timg[getattr(tl, off):getattr(tl, off) + getattr(tl, size)])
        a, b = a[a != 0], b[b != 0]
        assert a.shape == b.shape and (a == b).all(), name
    back = S.PackedMatrix(pm.cfg)
    back.host_image[:] = 0xAB
    S.stb_untile(tl, back.host_layout)
    for name, _, _ in S.PLANE_FIELDS:
        assert (back.plane(name) == pm.plane(name)).all(), name
    # mask / sign / region: lane records [row_tile][super][lane = 16*(block % 4) + row % 16], cut into two halves
    # ([row_tile][super][half][lane]) when the record is a multiple of 8 bytes
    nrt, nsb, nb = tl.n_row_tiles, tl.n_super, k // 128
    planes_rm = {name: pm.plane(name).reshape(n, -1) for name in ("mask", "sign", "region")}
    sign_rec, region_rec = 16 * N // M, 32 * N // M
    if padded:
        # the same records written out slot by slot: the kept columns of a group of 8 are numbered together with the
        # group's lowest pruned column, which takes a slot that stays zero
        nb_ = k // 128
        mask_bits = np.unpackbits(planes_rm["mask"], axis=1, bitorder="little")[:, :k]
        sign_bits = np.unpackbits(planes_rm["sign"], axis=1, bitorder="little")
        reg_bits = np.unpackbits(planes_rm["region"], axis=1, bitorder="little")
        ps = np.zeros((n, nb_, 16 * t8), np.uint8)
        pr = np.zeros((n, nb_, 16 * t8, 2), np.uint8)
        for i in range(n):
            slot = 0
            for g in range(k // 8):
                kept = mask_bits[i, 8 * g:8 * g + 8].astype(bool)
                assert kept.sum() == N
                aug = kept.copy()
                aug[np.flatnonzero(~kept)[0]] = True
                for c in np.flatnonzero(kept):
                    t = t8 * (g % 16) + int(aug[:c].sum())
                    ps[i, g // 16, t] = sign_bits[i, slot]
                    pr[i, g // 16, t] = reg_bits[i, 2 * slot:2 * slot + 2]
                    slot += 1
        planes_rm["sign"] = np.packbits(ps.reshape(n, -1), axis=1, bitorder="little")
        planes_rm["region"] = np.packbits(pr.reshape(n, -1), axis=1, bitorder="little")
        sign_rec, region_rec = 2 * t8, 4 * t8
        assert tl.sign_stride == sign_rec and tl.region_stride == region_rec
    for name, off, size, rec in (("mask", "off_mask", "mask_bytes", 16), ("sign", "off_sign", "sign_bytes", sign_rec),
                                 ("region", "off_region", "region_bytes", region_rec)):
        t = timg[getattr(tl, off):getattr(tl, off) + getattr(tl, size)]
        if rec % 8 == 0:
            t = t.reshape(nrt, nsb, 2, 4, 16, rec // 2).transpose(0, 4, 1, 3, 2, 5)      # [rt][i][sb][g][half][bytes]
        else:
            t = t.reshape(nrt, nsb, 4, 16, rec).transpose(0, 3, 1, 2, 4)                 # [rt][i][sb][g][bytes]
        t = t.reshape(nrt * 16, nsb * 4, rec)
        rm = np.zeros((nrt * 16, nsb * 4, rec), np.uint8)
        rm[:n, :nb] = planes_rm[name][:, :nb * rec].reshape(n, nb, rec)
        assert (t == rm).all(), name
    # res_sign: the row strings cut into 32-bit words, transposed inside each 16-row tile
    if tl.res_bytes:
        words = tl.res_stride // 4
        t = timg[tl.off_res:tl.off_res + tl.res_bytes].view("<u4").reshape(tl.n_row_tiles, words, 16)
        rm = np.zeros((tl.n_row_tiles * 16, words), "<u4")
        rm[:n] = pm.plane("res_sign").view("<u4").reshape(n, words)
        assert (t.transpose(0, 2, 1).reshape(-1, words) == rm).all()
    # res_t: per (row, block) lane record, the res_sign bits of the first 16 salient columns of each half block
    if tl.res_bytes:
        assert tl.res_t_bytes == nrt * nsb * 64 * 4
        rt = timg[tl.off_res_t:tl.off_res_t + tl.res_t_bytes].view("<u4").reshape(nrt, nsb, 4, 16)
        rs_bits = np.unpackbits(pm.plane("res_sign").reshape(n, -1), axis=1, bitorder="little")
        sal_cols = [int(c) for c in L["sal_cols"]]
        want = np.zeros((nrt * 16, nsb * 4), np.uint32)
        for q in range(nb):
            for h in range(2):
                entries = [u for u, c in enumerate(sal_cols) if 128 * q + 64 * h <= c < 128 * q + 64 * h + 64][:16]
                for e, u in enumerate(entries):
                    want[:n, q] |= rs_bits[:, u].astype(np.uint32) << np.uint32(16 * h + e)
        assert (rt.transpose(0, 3, 1, 2).reshape(nrt * 16, nsb * 4) == want).all()
    else:
        assert tl.res_t_bytes == 0
    # sal_tab: per half block, records of 8 salient columns with the selectors that gather their mask bytes
    if len(L["sal_cols"]):
        C = tl.sal_chunks
        nbk = tl.n_super * 4
        rec = timg[tl.off_saltab:tl.off_saltab + tl.saltab_bytes].view("<u4").reshape(nbk, 2, C, 12)
        pos = rec[:, :, :, 8:12].copy().view("<u2").reshape(nbk, 2, C * 8).astype(np.int64)
        cols = [int(q) * 128 + int(p) for q in range(nbk) for h in range(2) for p in pos[q, h] if p != 0xFFFF]
        assert cols == L["sal_cols"].tolist()
        valid = pos != 0xFFFF
        assert ((pos >> 6) == np.arange(2)[None, :, None])[valid].all()          # entries lie in their half
        per_half = valid.sum(axis=2)
        assert tl.max_sal_block == per_half.sum(axis=1).max()
        assert (rec[:, :, :, 6] == valid.reshape(nbk, 2, C, 8).sum(axis=3)).all()
        need = ((per_half + 7) // 8).reshape(tl.n_super, 4, 2).max(axis=1)        # [superblock][half]
        assert (rec[:, :, :, 5] == np.repeat(need, 4, axis=0)[:, :, None]).all()
        # [4]: ordinal of the record's first entry among all salient columns
        first = np.concatenate([[0], np.cumsum(per_half.reshape(-1))[:-1]]).reshape(nbk, 2)
        assert (rec[:, :, :, 4] == first[:, :, None] + 8 * np.arange(C)[None, None, :]).all()
        sel = rec[:, :, :, 0:2].copy().view(np.uint8).reshape(nbk, 2, C, 8)
        bit = rec[:, :, :, 2:4].copy().view(np.uint8).reshape(nbk, 2, C, 8)
        p8 = pos.reshape(nbk, 2, C, 8)
        v8 = valid.reshape(nbk, 2, C, 8)
        assert (sel == np.where(v8, (p8 >> 3) & 7, 0x0C)).all()
        assert (bit == np.where(v8, 1 << (p8 & 7), 0)).all()


def test_tile_of_padded_slots_rejects_a_group_with_the_wrong_number_of_kept_columns():
    L = make_layer(16, 256, 5)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 5, 8)
    pm.plane("mask")[3] |= 0xFF
    with pytest.raises(S.StbError) as e:
        pm.tiled()
    assert e.value.status == S.STB_EINVAL


def test_tile_rejects_mismatched_layouts():
    L = make_layer(16, 128, 3)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4)
    other = S.stb_tiled_sizes(S.make_cfg(32, 128, 2, 4, pm.cfg.n_salient))
    img = S.aligned_bytes(other.image_bytes)
    S.stb_layout_bind(other, img.ctypes.data)
    with pytest.raises(S.StbError) as e:
        S.stb_tile(pm.host_layout, other)
    assert e.value.status == S.STB_EINVAL
    with pytest.raises(S.StbError) as e:
        S.stb_tile(pm.host_layout, pm.host_layout)
    assert e.value.status == S.STB_EINVAL


def test_decode_launch_plan_invariants():
    """The launch shape the decode kernel picks (host arithmetic, no GPU): over many layer shapes, batches and
    modes the column splits and superblock visits cover every superblock, no split and no last visit is empty, the
    LDS areas do not overlap and fit, and the split count stays inside what the workspace is sized for."""
    import ctypes as C
    lib = S.binding._lib()
    plan = lib.stb_tiled_gemv24_plan
    plan.argtypes = [C.c_int] * 6 + [C.POINTER(C.c_int)]
    plan.restype = C.c_int
    out = (C.c_int * 7)()
    LDS, PHASE = 160 * 1024 - 64, 15
    seen_multi = 0
    for mode in (2, 4, 6):
        lds_max = LDS - (0 if mode == 2 else 32768)
        for nsb in list(range(1, 60)) + [64, 100, 112]:
            max_splits = (nsb + 1) // 2 + 3            # the bound the workspace is sized for
            for nrt in (1, 2, 3, 16, 63, 256, 257, 320, 512, 688, 864, 1792, 4000):
                for B, cus in ((1, 256), (2, 256), (4, 256), (5, 256), (8, 256), (15, 256), (16, 256), (1, 25), (1, 128), (4, 1), (16, 77)):
                    rc = plan(nrt, nsb, B, mode, max_splits, cus, out)
                    if rc != 0:
                        continue
                    Sn, R, SPS, V, wreg, rec_off, part_off = list(out)
                    what = (mode, nsb, nrt, B, cus, list(out))
                    assert 1 <= SPS <= 8 and 1 <= V <= 8 and 1 <= Sn <= max_splits and R >= 1, what
                    assert Sn * SPS * V >= nsb, what                      # every superblock has a wavefront and a visit
                    assert (Sn - 1) * SPS * V < nsb, what                 # no empty split
                    assert (Sn * V - 1) * SPS < nsb, what                 # no empty last visit
                    assert R == -(-nrt // max(cus // Sn, 1)), what        # row tiles per workgroup: one round on the layer's units if it can be
                    pht = min(R, PHASE)
                    assert pht == R or pht % 3 == 0, what                 # phases end on a whole round of the three tile buffers
                    xbytes = (B + 1 if B < 16 else 16) * 1040
                    if V == 1:
                        assert part_off == 0 and rec_off >= max(xbytes, pht * 1024) and wreg == rec_off + 768, what
                    else:
                        assert rec_off == V * xbytes and part_off == rec_off + V * 768 and wreg == part_off + pht * 1024, what
                        seen_multi += 1
                    assert SPS * wreg <= lds_max, what
    assert seen_multi > 0
    # arguments outside the kernel's range are refused
    assert plan(16, 8, 17, 2, 7, 256, out) != 0 and plan(16, 8, 1, 5, 7, 256, out) != 0 and plan(0, 8, 1, 2, 7, 256, out) != 0
    assert plan(16, 8, 1, 2, 7, 0, out) != 0 and plan(16, 8, 1, 2, 7, 257, out) != 0


# ----------------------------------------------------------------------------------------------
# the 2:4 group code of App. C, out of and into the mask and sign planes
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,k,seed", [(33, 256, 41), (5, 128, 42), (70, 1024, 43)])
def test_code24_export_import_against_the_oracle(n, k, seed):
    L = make_layer(n, k, seed)
    ref, dbg = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 0, return_debug=True)
    slots = np.unpackbits(ref["sign"], axis=1, bitorder="little")[:, :k // 2]
    E_ref, V_ref = O.code24_encode(dbg["mask"], slots)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 0)
    E, V = S.stb_code24_export(pm.host_layout)
    assert E.dtype == np.uint16 and V.dtype == np.uint8
    assert (E == E_ref).all() and (V == V_ref).all()
    # what the code stands for is the signed mask of the dequantised matrix's kept positions
    assert ((O.code24_decode(E, V) != 0) == dbg["mask"]).all()
    # import into a copy whose mask and sign planes were wiped: every plane is back, byte for byte
    before = pm.host_image.copy()
    pm.plane("mask")[:] = 0xAA
    pm.plane("sign")[:] = 0x55
    S.stb_code24_import(pm.host_layout, E, V)
    assert (pm.host_image == before).all()


def test_code24_rejects_what_it_cannot_represent():
    L = make_layer(16, 128, 44)
    pm48 = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 4, 8, 0)
    E = np.zeros((16, 8), dtype=np.uint16)
    V = np.zeros((16, 8), dtype=np.uint8)
    lib = S.binding._lib()
    assert lib.stb_code24_export(C.byref(pm48.host_layout), E.ctypes.data, V.ctypes.data) == S.STB_EUNSUPPORTED
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], 2, 4, 0)
    assert lib.stb_code24_export(C.byref(pm.host_layout), None, V.ctypes.data) == S.STB_ENULL
    lay_t, _img = pm.tiled()
    assert lib.stb_code24_export(C.byref(lay_t), E.ctypes.data, V.ctypes.data) == S.STB_EINVAL
    E, V = S.stb_code24_export(pm.host_layout)
    before = pm.host_image.copy()
    for bad in (0b0000, 0b0101, 0b0110):          # equal positions (0, 0) and (1, 1), descending (2, 1)
        E2 = E.copy()
        E2[3, 5] = (E2[3, 5] & 0xFF0F) | (bad << 4)
        with pytest.raises(S.StbError) as e:
            S.stb_code24_import(pm.host_layout, E2, V)
        assert e.value.status == S.STB_EINVAL
        assert (pm.host_image == before).all()    # checked before anything is written
    # a mask group that keeps three weights cannot be exported
    pm.plane("mask")[0] |= 0x07
    assert lib.stb_code24_export(C.byref(pm.host_layout), E.ctypes.data, V.ctypes.data) == S.STB_EINVAL


# ----------------------------------------------------------------------------------------------
# salient columns (Alg. 2 "Salient")
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,k,seed,kind,max_per_block,lam", [
    (24, 256, 51, "x8", 20, 0.01), (7, 128, 52, "t3", 128, 0.0), (40, 384, 53, "x8", 16, 1.0),
    (64, 512, 54, "x8", 0, 0.5), (33, 1024, 55, "t3", 9, 0.01), (128, 256, 56, "x8", 40, 100.0)])
def test_salient_columns_bit_exact_against_the_oracle(n, k, seed, kind, max_per_block, lam):
    L = make_layer(n, k, seed, kind)
    ref = O.salient_columns(L["W"], L["xnorm"], lam, max_per_block)
    bm = S.stb_salient_columns(L["W"], L["xnorm"], lam, max_per_block)
    assert bm.dtype == np.uint32 and bm.shape == (k // 32,)
    assert (O.bitmap_to_bool(bm, k) == ref).all()
    # and the bitmap is what stb_pack takes
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], bm, 4, 8, 0)
    ref_planes = O.pack(L["W"], L["xnorm"], bm, 4, 8, 0)
    for name, v in _oracle_bytes(ref_planes).items():
        assert (pm.plane(name) == v).all(), name


def test_salient_columns_reject_bad_arguments():
    L = make_layer(8, 128, 57)
    lib = S.binding._lib()
    W = np.ascontiguousarray(L["W"], dtype=np.float32)
    xn = np.ascontiguousarray(L["xnorm"], dtype=np.float32)
    out = np.zeros(4, dtype=np.uint32)
    call = lambda w, n, k, x, lam, m, o: lib.stb_salient_columns(w, n, k, x, C.c_double(lam), m, o, None)
    assert call(None, 8, 128, xn.ctypes.data, 0.1, 4, out.ctypes.data) == S.STB_ENULL
    assert call(W.ctypes.data, 8, 100, xn.ctypes.data, 0.1, 4, out.ctypes.data) == S.STB_EINVAL
    assert call(W.ctypes.data, 8, 128, xn.ctypes.data, -1.0, 4, out.ctypes.data) == S.STB_EINVAL
    assert call(W.ctypes.data, 8, 128, xn.ctypes.data, 0.1, 129, out.ctypes.data) == S.STB_EINVAL
    bad = W.copy()
    bad[3, 7] = np.nan
    assert call(bad.ctypes.data, 8, 128, xn.ctypes.data, 0.1, 4, out.ctypes.data) == S.STB_ENONFINITE
    xb = xn.copy()
    xb[5] = -1.0
    assert call(W.ctypes.data, 8, 128, xb.ctypes.data, 0.1, 4, out.ctypes.data) == S.STB_ENONFINITE


# ----------------------------------------------------------------------------------------------
# layer-wise N:M assignment (Sec. 3.3)
# ----------------------------------------------------------------------------------------------
def test_layer_nm_assignment_against_the_oracle():
    # a synthetic stack of layers of different shapes and scales
    shapes = [(64, 256), (64, 256), (256, 64), (128, 128), (32, 512), (96, 384)]
    layers = [make_layer(n, k, 60 + i)["W"] * np.float32(1.0 + 0.7 * i) for i, (n, k) in enumerate(shapes)]
    om_ref = [O.layer_l2_norm(W) for W in layers]
    om = [S.stb_layer_l2_norm(W) for W in layers]
    assert om == om_ref                                     # bit for bit: same sequential float64 sum
    for R in (0.5, 0.25, 0.75, 0.0, 1.0):
        N_ref, _ = O.layer_nm_assignment(om_ref, R, 8)
        assert S.stb_layer_nm_assignment(om, R, 8).tolist() == N_ref.tolist()
    assert S.stb_layer_nm_assignment(om, 0.5, 4).tolist() == O.layer_nm_assignment(om_ref, 0.5, 4)[0].tolist()
    with pytest.raises(S.StbError) as e:
        S.stb_layer_nm_assignment(om, 1.5, 8)
    assert e.value.status == S.STB_EINVAL
    with pytest.raises(S.StbError) as e:
        S.stb_layer_nm_assignment([1.0, float("nan")], 0.5, 8)
    assert e.value.status == S.STB_ENONFINITE


def test_decode_workspace_sizes_for_batches_above_16():
    """Up to 16 rows the scratch is that of the decode kernel alone; above 16 rows a layer other than 2:4 may run as
    one pass of the prefill kernel, whose scratch sits behind the decode kernel's: the size asked for grows with the
    batch, never shrinks below the decode kernel's, and 2:4 layers (two decode passes) keep theirs."""
    for (n, k, N, M, sal) in ((5120, 13824, 6, 8, 691), (4096, 4096, 4, 8, 204), (130, 640, 5, 8, 0), (11008, 4096, 2, 4, 204)):
        cfg = S.make_cfg(n, k, N, M, sal)
        w1, w16, w17, w32 = (S.stb_gemv_workspace_bytes(cfg, B) for B in (1, 16, 17, 32))
        assert w1 == w16 >= 0
        if (N, M) == (2, 4):
            assert w17 == w32 == w16
        else:
            assert w16 < w17 <= w32
            assert w17 % 256 == 0 and w32 % 256 == 0
    cfg = S.make_cfg(4096, 4096, 4, 8, 0)
    for B in (0, 33):
        with pytest.raises(S.StbError):
            S.stb_gemv_workspace_bytes(cfg, B)


@pytest.mark.parametrize("k,r,seed", [(128, 300, 41), (384, 500, 42), (257, 257, 43)])
def test_hessian_factor_against_the_oracle_and_its_defining_identity(k, r, seed):
    """stb_hessian_factor (factorisation from the last column, then a triangular inverse) against the oracle's
    inverse-then-Cholesky: the factor with a positive diagonal is unique, so the two agree to rounding; and the
    identity that defines it, Hc^T Hc (H + lambda I) = I."""
    rng = np.random.default_rng(seed)
    X = (rng.standard_normal((r, k)) @ (np.eye(k) + 0.5 * rng.standard_normal((k, k)) / np.sqrt(k))).astype(np.float32)
    H = 2.0 * X.astype(np.float64).T @ X.astype(np.float64)
    lam = 0.01 * float(np.mean(np.diag(H)))
    Hc, xnorm = S.stb_hessian_factor(X, lam, n_threads=3)
    ref = O.hessian_factor(X, lam)
    assert (np.tril(Hc, -1) == 0.0).all() and (np.diag(Hc) > 0).all()
    assert np.abs(Hc - ref).max() <= 1e-9 * np.abs(ref).max()
    assert np.abs(Hc.T @ Hc @ (H + lam * np.eye(k)) - np.eye(k)).max() < 1e-8
    assert np.allclose(xnorm, np.sqrt(np.sum(X.astype(np.float64) ** 2, axis=0)), rtol=1e-6, atol=0)
    one, xn1 = S.stb_hessian_factor(X, lam, n_threads=1)
    assert (one.view(np.uint64) == Hc.view(np.uint64)).all() and (xn1 == xnorm).all()


def test_hessian_factor_closed_form_for_orthogonal_features_and_errors():
    # orthogonal features: H is diagonal and the factor is 1 / sqrt(2 |x_j|^2 + lambda) on the diagonal
    k = 128
    d = np.arange(1, k + 1, dtype=np.float32)
    X = np.diag(d)
    Hc, xnorm = S.stb_hessian_factor(X, 0.5)
    assert (Hc[~np.eye(k, dtype=bool)] == 0.0).all()
    assert np.allclose(np.diag(Hc), 1.0 / np.sqrt(2.0 * d.astype(np.float64) ** 2 + 0.5), rtol=1e-15)
    assert (xnorm == d).all()
    # fewer samples than features and no damping: not positive definite
    with pytest.raises(S.StbError) as e:
        S.stb_hessian_factor(np.ones((3, 128), dtype=np.float32), 0.0)
    assert e.value.status == S.STB_ENONFINITE
    bad = np.ones((4, 128), dtype=np.float32)
    bad[1, 5] = np.nan
    with pytest.raises(S.StbError) as e:
        S.stb_hessian_factor(bad, 1.0)
    assert e.value.status == S.STB_ENONFINITE
    with pytest.raises(S.StbError) as e:
        S.stb_hessian_factor(np.ones((4, 128), dtype=np.float32), -1.0)
    assert e.value.status == S.STB_EINVAL


def test_calibration_activations_to_packed_layer_inside_the_library():
    """X -> stb_hessian_factor (factor and feature norms) -> stb_salient_columns -> stb_pack_obc: the chain Alg. 1
    describes, with no step outside the library; the packed bytes equal the oracle's for the same factor array."""
    n, k, N, M = 48, 384, 4, 8
    L = make_layer(n, k, 77, "x8")
    rng = np.random.default_rng(78)
    X = (rng.standard_normal((2 * k, k)) @ (np.eye(k) + 0.6 * rng.standard_normal((k, k)) / np.sqrt(k))).astype(np.float32)
    lam = 0.01 * float(np.mean(2.0 * np.sum(X.astype(np.float64) ** 2, axis=0)))
    Hc, xnorm = S.stb_hessian_factor(X, lam)
    bitmap = S.stb_salient_columns_hc(L["W"], Hc, 8)
    assert (O.bitmap_to_bool(bitmap, k) == O.salient_columns_hc(L["W"], Hc, 8)).all() and bitmap.any()
    ref = O.pack_obc(L["W"], Hc, xnorm, bitmap, N, M, 0)
    pm = S.PackedMatrix.pack_obc(L["W"], Hc, xnorm, bitmap, N, M, 0)
    for name, v in _oracle_bytes(ref).items():
        assert (pm.plane(name) == v).all(), name
    assert (pm.unpack() == O.unpack(ref, n, k, N, M)).all()


@pytest.mark.parametrize("n,k,seed,max_per_block", [(48, 512, 91, 16), (7, 128, 92, 128), (130, 384, 93, 5)])
def test_salient_columns_from_the_factor_bit_exact_against_the_oracle(n, k, seed, max_per_block):
    L = make_layer(n, k, seed, "x8")
    rng = np.random.default_rng(seed)
    X = (rng.standard_normal((k + 50, k)) @ (np.eye(k) + 0.5 * rng.standard_normal((k, k)) / np.sqrt(k))).astype(np.float32)
    Hc, _ = S.stb_hessian_factor(X, 0.5)
    got = O.bitmap_to_bool(S.stb_salient_columns_hc(L["W"], Hc, max_per_block), k)
    assert (got == O.salient_columns_hc(L["W"], Hc, max_per_block)).all()
    bad = Hc.copy()
    bad[3, 3] = 0.0
    with pytest.raises(S.StbError) as e:
        S.stb_salient_columns_hc(L["W"], bad, max_per_block)
    assert e.value.status == S.STB_ENONFINITE
    with pytest.raises(S.StbError) as e:
        S.stb_salient_columns_hc(L["W"], Hc, 129)
    assert e.value.status == S.STB_EINVAL


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys, os
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
