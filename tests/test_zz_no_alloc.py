"""stb_gemv_static (the entry point that allocates nothing: its scratch is a device array inside the library) against
stb_gemv with a caller's workspace, through the C ABI: same bits, and both inside the oracle's tolerance.  Two calls in
a row share the array, the second on a smaller layer."""
import os
import sys

import numpy as np
import pytest

import paper_2408_01803_amd as S
from oracle import stb_oracle as O
from workloads import make_layer, make_x

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _layer(n, k, N, M, seed):
    L = make_layer(n, k, seed, "x8")
    ref = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 1)
    pm = S.PackedMatrix.pack(L["W"], L["xnorm"], L["sal_bitmap"], N, M, 1).to_device(tiled=True)
    return pm, O.unpack(ref, n, k, N, M)


def test_gemv_static_matches_gemv_on_two_calls_in_a_row():
    import torch
    assert os.path.exists(S.LIB_PATH) and torch.cuda.is_available()
    torch.cuda.set_device(0)
    # the first layer is wide enough for column splits (k > 4096), so the scratch array is really used; the second is
    # smaller in both directions and has a different number of row tiles
    cases = [(200, 9728, 2, 4, 901, 3), (72, 4608, 4, 8, 902, 16)]
    layers = [(_layer(n, k, N, M, seed), n, k, seed, B) for (n, k, N, M, seed, B) in cases]
    for rnd in range(2):                      # the whole sequence twice: the array keeps the last call's contents
        for (pm, What), n, k, seed, B in layers:
            x = make_x(B, k, seed)
            y_ref, bound = O.matmul(x, What)
            xd = torch.from_numpy(x).cuda()
            for y_fp32 in (True, False):
                dt = torch.float32 if y_fp32 else torch.float16
                y_ws = torch.full((B, n), float("nan"), dtype=dt, device="cuda")
                y_st = torch.full((B, n), float("nan"), dtype=dt, device="cuda")
                _say(f"[step] round {rnd}: stb_gemv / stb_gemv_static {n}x{k} B={B} fp32={y_fp32}")
                S.stb_gemv(pm.dev_layout, xd, B, y_ws, y_fp32, pm.workspace)
                S.stb_gemv_static(pm.dev_layout, xd, B, y_st, y_fp32)
                torch.cuda.synchronize()
                a, b = y_ws.cpu().numpy(), y_st.cpu().numpy()
                assert (a.view(np.uint32 if y_fp32 else np.uint16) == b.view(np.uint32 if y_fp32 else np.uint16)).all()
                err = np.abs(b.astype(np.float64) - y_ref)
                assert (err <= TOL * bound).all()


def test_gemv_static_rejects_what_does_not_fit():
    import torch
    torch.cuda.set_device(0)
    # 16384 row tiles is the limit of the counter area: a layout that claims more is turned away before any launch
    cfg = S.make_cfg(16 * 16385, 128, 2, 4, 0)
    lay = S.stb_tiled_sizes(cfg)
    xd = torch.zeros((1, 128), dtype=torch.float16, device="cuda")
    yd = torch.zeros((1, 16 * 16385), dtype=torch.float16, device="cuda")
    with pytest.raises(S.StbError) as e:
        S.stb_gemv_static(lay, xd, 1, yd)
    assert e.value.status == S.STB_ETOOBIG
