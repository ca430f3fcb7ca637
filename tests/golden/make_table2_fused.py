#!/usr/bin/env python3
"""Writes tests/golden/table2_fused.npz: the float64 oracle's results for the shape of the paper's
own benchmark (Table 2 of arXiv 2304.13134: 32 labels, context size 2 = 1057 states, shared-embedding
weight function with 512 hidden units, batch 16, 1024 frames, 256 output labels), synthetic inputs
from workloads.config(5).

Calls only `oracle/`, one process per batch item (de and dW are sums over items); the denominator
takes a few minutes per item.  Stored, for the globally normalised loss D - N: D [16], N [16],
the gradient's dW [512,33] whole, 4096 seeded samples each of df and de with their flat indices,
the largest magnitudes of df and de.
Run from the repository root:  python tests/golden/make_table2_fused.py
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
    cfg = workloads.config(5)
    oracle.set_threads(1)
    den = oracle.fused_forward_backward(cfg["f"][b:b + 1], cfg["e"], cfg["W"], cfg["lengths"][b:b + 1],
                                        2, round_h=True, grads=True)
    num = oracle.fused_numerator(cfg["f"][b:b + 1], cfg["e"], cfg["W"], cfg["lengths"][b:b + 1],
                                 cfg["refs"][b:b + 1], cfg["ref_lengths"][b:b + 1], 2, round_h=True)
    print("item", b, "D", den["D"][0], "N", num["N"][0], flush=True)
    return (float(den["D"][0]), float(num["N"][0]), den["df"][0] - num["df"][0],
            den["de"] - num["de"], den["dW"] - num["dW"])


def main():
    oracle.build()
    cfg = workloads.config(5)
    B = cfg["f"].shape[0]
    with ProcessPoolExecutor(max_workers=min(B, os.cpu_count() or 1)) as ex:
        res = list(ex.map(one_item, range(B)))
    D = np.array([r[0] for r in res])
    N = np.array([r[1] for r in res])
    df = np.stack([r[2] for r in res])
    de = sum(r[3] for r in res)
    dW = sum(r[4] for r in res)
    rng = np.random.default_rng(workloads.SEED_BASE + 505)
    idx_f = rng.choice(df.size, N_SAMPLES, replace=False)
    idx_e = rng.choice(de.size, N_SAMPLES, replace=False)
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "table2_fused.npz")
    np.savez_compressed(out, D=D, N=N, dW=dW, idx_f=idx_f, df=df.ravel()[idx_f], idx_e=idx_e,
                        de=de.ravel()[idx_e], df_max=np.max(np.abs(df)), de_max=np.max(np.abs(de)))
    print("wrote", out, "D =", D, "N =", N)


if __name__ == "__main__":
    main()
