#!/usr/bin/env python3
"""Writes tests/golden/config4_fused.npz: the float64 oracle's results for the full-size
trigram workload with on-the-fly weights (B=4, T=1000, V=64, hidden 512).

Calls only `oracle/` (one process per batch item; de and dW are sums over items) and takes
about five minutes on four cores.  Stored: D [4]; dW [512,65] whole; 4096 seeded samples each
of df and de with their flat indices; the largest magnitudes of df and de.
Run from the repository root:  python tests/golden/make_config4_fused.py
"""
import os
import sys
from concurrent.futures import ProcessPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                            # noqa: E402
from paper_2304_13134_amd import workloads               # noqa: E402

N_SAMPLES = 4096


def one_item(b):
    cfg = workloads.config(4)
    o = oracle.fused_forward_backward(cfg["f"][b:b + 1], cfg["e"], cfg["W"], cfg["lengths"][b:b + 1],
                                      2, round_h=True, grads=True)
    return float(o["D"][0]), o["df"][0], o["de"], o["dW"]


def main():
    oracle.build()
    cfg = workloads.config(4)
    B = cfg["f"].shape[0]
    with ProcessPoolExecutor(max_workers=min(B, os.cpu_count() or 1)) as ex:
        res = list(ex.map(one_item, range(B)))
    D = np.array([r[0] for r in res])
    df = np.stack([r[1] for r in res])
    de = sum(r[2] for r in res)
    dW = sum(r[3] for r in res)
    rng = np.random.default_rng(workloads.SEED_BASE + 404)
    idx_f = rng.choice(df.size, N_SAMPLES, replace=False)
    idx_e = rng.choice(de.size, N_SAMPLES, replace=False)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "config4_fused.npz")
    np.savez_compressed(out, D=D, dW=dW, idx_f=idx_f, df=df.ravel()[idx_f], idx_e=idx_e,
                        de=de.ravel()[idx_e], df_max=np.max(np.abs(df)), de_max=np.max(np.abs(de)))
    print("wrote", out, "D =", D)


if __name__ == "__main__":
    main()
