"""Writes tests/golden/packed_digests.json: SHA-256 of every packed plane of every workload layer.

Calls only the CPU oracle (oracle/) and the seeded input generators (workloads/): no value in the
output comes from the HIP library.  The full-size parity tests compare the library's packer against
these digests, so the slow oracle packer does not have to run on the GPU machine.

    python tests/golden/make_golden.py [--jobs 4] [--only cfg1 cfg2 ...] [--cache DIR]

With --cache the oracle's planes are also saved as .npz files (useful to locate a mismatch).
"""
import argparse
import hashlib
import json
import multiprocessing as mp
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

PLANES = ("mask", "sign", "region", "res_sign", "scales", "res_scale", "sal_bitmap", "sal_block_prefix")
OUT = os.path.join(ROOT, "tests", "golden", "packed_digests.json")


def layer_key(cfg, spec):
    return (f"cfg{cfg}_{spec.name}_{spec.n}x{spec.k}_{spec.N}of{spec.M}"
            f"_mode{spec.region_mode}_{spec.salient_kind}_seed{spec.seed}")


def digest_planes(planes):
    out = {}
    for name in PLANES:
        out[name] = hashlib.sha256(np.ascontiguousarray(planes[name]).tobytes()).hexdigest()
    out["total_bytes"] = int(sum(np.ascontiguousarray(planes[name]).nbytes for name in PLANES))
    return out


def _work(args):
    cfg, spec, cache = args
    from oracle import stb_oracle as O
    from workloads import make_layer
    t0 = time.time()
    L = make_layer(spec.n, spec.k, spec.seed, spec.salient_kind)
    planes = O.pack(L["W"], L["xnorm"], L["sal_bitmap"], spec.N, spec.M, spec.region_mode)
    key = layer_key(cfg, spec)
    if cache:
        os.makedirs(cache, exist_ok=True)
        np.savez(os.path.join(cache, key + ".npz"), **planes)
    d = digest_planes(planes)
    d["seconds"] = round(time.time() - t0, 1)
    return key, d


def main():
    from workloads import WORKLOADS
    ap = argparse.ArgumentParser()
    ap.add_argument("--jobs", type=int, default=4)
    ap.add_argument("--only", nargs="*", default=None)
    ap.add_argument("--cache", default=None)
    ap.add_argument("--force", action="store_true", help="recompute layers already in the output file")
    a = ap.parse_args()
    done = set() if a.force or not os.path.exists(OUT) else set(json.load(open(OUT)))
    tasks = []
    for cfg, wl in WORKLOADS.items():
        if a.only and f"cfg{cfg}" not in a.only:
            continue
        for spec in wl["layers"]:
            if layer_key(cfg, spec) not in done:
                tasks.append((cfg, spec, a.cache))
    tasks.sort(key=lambda t: -(t[1].n * t[1].k * (1 if t[1].region_mode == 0 else 0.05)))
    result = json.load(open(OUT)) if os.path.exists(OUT) else {}
    with mp.Pool(a.jobs, maxtasksperchild=1) as pool:
        for key, d in pool.imap_unordered(_work, tasks):
            result[key] = d
            print(key, d["seconds"], "s", flush=True)
            with open(OUT, "w") as f:
                json.dump(dict(sorted(result.items())), f, indent=1)


if __name__ == "__main__":
    main()
