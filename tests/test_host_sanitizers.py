"""The host side of the library (packer, host dequantiser, tiling, the 2:4 group code, salient columns, layer-wise
assignment) under AddressSanitizer and UndefinedBehaviorSanitizer: stb_host.cpp is compiled on its own with
-fsanitize=address,undefined into a separate shared object and driven from a child process (the sanitizer runtime has
to be loaded before the interpreter's allocator is in use, hence LD_PRELOAD in the child only).  No GPU, no HIP."""
import os
import shutil
import subprocess
import sys
import textwrap

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2408_01803_amd", "csrc", "stb_host.cpp")

CHILD = textwrap.dedent('''
    import ctypes as C, sys
    import numpy as np
    sys.path.insert(0, %(root)r)
    import paper_2408_01803_amd.binding as B
    B.LIB_PATH = %(lib)r                      # the sanitized build holds the host entry points only
    lib = C.CDLL(B.LIB_PATH)
    P = C.POINTER
    lib.stb_layout_sizes.argtypes = [P(B.stb_cfg_t), P(B.stb_layout_t)]
    lib.stb_layout_bind.argtypes = [P(B.stb_layout_t), C.c_void_p]
    lib.stb_tiled_sizes.argtypes = [P(B.stb_cfg_t), P(B.stb_layout_t)]
    lib.stb_tile.argtypes = [P(B.stb_layout_t), P(B.stb_layout_t)]
    lib.stb_untile.argtypes = [P(B.stb_layout_t), P(B.stb_layout_t)]
    lib.stb_pack.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, P(B.stb_layout_t), C.c_int32]
    lib.stb_pack_obc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, P(B.stb_layout_t), C.c_int32]
    lib.stb_unpack.argtypes = [P(B.stb_layout_t), C.c_void_p]
    lib.stb_salient_columns.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_double, C.c_int32, C.c_void_p, P(C.c_int32)]
    lib.stb_layer_l2_norm.argtypes = [C.c_void_p, C.c_int64, P(C.c_double)]
    lib.stb_layer_nm_assignment.argtypes = [C.c_void_p, C.c_int32, C.c_double, C.c_int32, C.c_void_p]
    lib.stb_code24_export.argtypes = [P(B.stb_layout_t), C.c_void_p, C.c_void_p]
    lib.stb_code24_import.argtypes = [P(B.stb_layout_t), C.c_void_p, C.c_void_p]
    from workloads import make_layer

    def image(sizes_fn, cfg):
        lay = B.stb_layout_t()
        assert sizes_fn(C.byref(cfg), C.byref(lay)) == 0
        img = B.aligned_bytes(lay.image_bytes)
        assert lib.stb_layout_bind(C.byref(lay), C.c_void_p(img.ctypes.data)) == 0
        return lay, img

    cases = [(37, 640, 4, 8, 0, 33), (130, 1024, 2, 4, 1, 51), (5, 128, 1, 4, 0, 0), (64, 256, 8, 8, 1, 12),
             (17, 256, 6, 8, 0, 12), (96, 512, 5, 8, 1, 25), (48, 1024, 3, 8, 0, 150)]
    for n, k, N, M, mode, S_ in cases:
        L = make_layer(n, k, 500 + n, "x8", n_salient=S_)
        cfg = B.make_cfg(n, k, N, M, S_, mode)
        lay, img = image(lib.stb_layout_sizes, cfg)
        for threads in (1, 3):
            assert lib.stb_pack(L["W"].ctypes.data, L["xnorm"].ctypes.data, L["sal_bitmap"].ctypes.data, C.byref(lay), threads) == 0
        out = np.empty((n, k), dtype=np.float32)
        assert lib.stb_unpack(C.byref(lay), out.ctypes.data) == 0
        if k <= 640:                                   # the block loop of Alg. 1, with and without a factor
            Xc = np.random.default_rng(n).standard_normal((k + 7, k)).astype(np.float32)
            Hf = np.empty((k, k), dtype=np.float64)
            xn = np.empty(k, dtype=np.float32)
            lib.stb_hessian_factor.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_void_p, C.c_void_p, C.c_int32]
            assert lib.stb_hessian_factor(Xc.ctypes.data, k + 7, k, 0.5, Hf.ctypes.data, xn.ctypes.data, 3) == 0
            assert lib.stb_hessian_factor(Xc.ctypes.data, k + 7, k, 0.5, Hf.ctypes.data, None, 1) == 0
            assert np.isfinite(Hf).all() and (np.tril(Hf, -1) == 0).all()
            bm = np.zeros(k // 32, dtype=np.uint32)
            cnt = C.c_int32(0)
            lib.stb_salient_columns_hc.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, P(C.c_int32)]
            assert lib.stb_salient_columns_hc(L["W"].ctypes.data, n, k, Hf.ctypes.data, 9, bm.ctypes.data, C.byref(cnt)) == 0
            Hc = np.triu(0.02 * np.random.default_rng(n).standard_normal((k, k)), 1) + np.eye(k)
            for factor in (None, Hc.ctypes.data):
                assert lib.stb_pack_obc(L["W"].ctypes.data, factor, L["xnorm"].ctypes.data, L["sal_bitmap"].ctypes.data, C.byref(lay), 3) == 0
            assert lib.stb_unpack(C.byref(lay), out.ctypes.data) == 0
        assert np.isfinite(out).all()
        if (8 * N) %% M == 0 and 8 * N // M in (4, 6):
            tl, timg = image(lib.stb_tiled_sizes, cfg)
            assert lib.stb_tile(C.byref(lay), C.byref(tl)) == 0
            back, bimg = image(lib.stb_layout_sizes, cfg)
            assert lib.stb_untile(C.byref(tl), C.byref(back)) == 0
            assert (bimg == img).all()
        if (N, M) == (2, 4):
            E = np.empty((n, k // 16), dtype=np.uint16)
            V = np.empty((n, k // 16), dtype=np.uint8)
            assert lib.stb_code24_export(C.byref(lay), E.ctypes.data, V.ctypes.data) == 0
            assert lib.stb_code24_import(C.byref(lay), E.ctypes.data, V.ctypes.data) == 0
        sal = np.zeros(k // 32, dtype=np.uint32)
        cnt = C.c_int32(0)
        assert lib.stb_salient_columns(L["W"].ctypes.data, n, k, L["xnorm"].ctypes.data, 0.01, 12, sal.ctypes.data, C.byref(cnt)) == 0
        om = C.c_double(0)
        assert lib.stb_layer_l2_norm(L["W"].ctypes.data, L["W"].size, C.byref(om)) == 0
    oms = np.array([1.0, 2.0, 0.0, 5.5])
    Ns = np.zeros(4, dtype=np.int32)
    assert lib.stb_layer_nm_assignment(oms.ctypes.data, 4, 0.5, 8, Ns.ctypes.data) == 0
    # error paths: bad arguments must be turned away before any access
    bad = B.make_cfg(16, 100, 2, 4, 0)
    lay = B.stb_layout_t()
    assert lib.stb_layout_sizes(C.byref(bad), C.byref(lay)) != 0
    assert lib.stb_pack(None, None, None, C.byref(lay), 1) != 0
    assert lib.stb_pack_obc(None, None, None, None, C.byref(lay), 1) != 0
    maps = open("/proc/self/maps").read()
    assert "libasan" in maps and "libubsan" in maps, "the sanitizer runtimes are not loaded"
    print("SANITIZED_OK")
''')


def test_host_library_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    asan = subprocess.run([gxx, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    ubsan = subprocess.run([gxx, "-print-file-name=libubsan.so"], capture_output=True, text=True).stdout.strip()
    if not (os.path.isabs(asan) and os.path.exists(asan) and os.path.isabs(ubsan) and os.path.exists(ubsan)):
        pytest.skip("sanitizer runtimes are not installed")
    lib = str(tmp_path / "libstb_host_san.so")
    cmd = [gxx, "-O1", "-g", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off", "-pthread",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.dirname(SRC), SRC, "-o", lib]
    subprocess.run(cmd, check=True)
    env = dict(os.environ)
    preload = [asan, ubsan] + ([env["LD_PRELOAD"]] if env.get("LD_PRELOAD") else [])
    env["LD_PRELOAD"] = ":".join(preload)
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0:exitcode=23"       # (the interpreter itself leaks at exit)
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    r = subprocess.run([sys.executable, "-c", CHILD % dict(root=ROOT, lib=lib)], env=env, capture_output=True, text=True,
                       timeout=600)
    assert r.returncode == 0 and "SANITIZED_OK" in r.stdout, (r.returncode, r.stdout[-2000:], r.stderr[-4000:])
