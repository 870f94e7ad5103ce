#!/usr/bin/env python3
"""Writes tests/golden/cfg<k>_checkpoints.npz: the fp64 oracle's state of a workload at every
100-round checkpoint of its full run, for workloads whose oracle is too slow to run inside the
GPU test suite (config 4: about 0.2 s per round, 3000 rounds).

Calls only oracle/ and rfast_workloads/ (never the HIP library).  Per checkpoint: the integer
state in full (counters, stamps), x and z of every node on a fixed sample of coordinates, and of
the full vectors the per-node norms and their projections on eight seeded +-1 vectors, so that an
error anywhere in a vector moves a stored number.

    python tests/golden/make_checkpoints.py --config 4            # about ten minutes on one core
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

N_PROJ = 8


def sample_coords(p, count=96, seed=2307):
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, p])))
    pick = g.choice(p, size=min(count, p), replace=False)
    return np.unique(np.concatenate([pick, np.arange(min(16, p)), np.arange(max(p - 16, 0), p)])).astype(np.int64)


def projection_signs(p, seed=11617):
    """[N_PROJ][p] of +-1, as int8."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, p])))
    return (2 * g.integers(0, 2, size=(N_PROJ, p), dtype=np.int8) - 1).astype(np.int8)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--rounds", type=int, default=0, help="0: the full run of the workload")
    ap.add_argument("--every", type=int, default=100)
    ap.add_argument("--out", default="")
    args = ap.parse_args()
    from oracle.from_workload import make_oracle
    from rfast_workloads import configs
    w = configs.CONFIGS[args.config]()
    rounds = args.rounds or w.rounds
    orc = make_oracle(w)
    coords = sample_coords(w.p)
    signs = projection_signs(w.p).astype(np.float64)
    out = {k: [] for k in ("round", "t", "tau_v", "tau_rho", "x_s", "z_s", "x_norm", "z_norm", "g_norm", "x_proj", "z_proj")}
    t0 = time.time()
    for r in range(rounds):
        q = w.sched.round(r)
        orc.round(q.active, q.delay_R, q.delay_C, q.drop_R, q.drop_C, w.gamma, q.batch_idx)
        if (r + 1) % args.every == 0 or r + 1 == rounds:
            sl = orc.slots()
            out["round"].append(r + 1)
            out["t"].append(np.asarray(sl["t"], np.int32))
            out["tau_v"].append(np.asarray(sl["tau_v"], np.int32))
            out["tau_rho"].append(np.asarray(sl["tau_rho"], np.int32))
            out["x_s"].append(orc.x[:, coords].astype(np.float32))
            out["z_s"].append(orc.z[:, coords].astype(np.float32))
            out["x_norm"].append(np.linalg.norm(orc.x, axis=1))
            out["z_norm"].append(np.linalg.norm(orc.z, axis=1))
            out["g_norm"].append(np.linalg.norm(orc.g, axis=1))
            out["x_proj"].append(orc.x @ signs.T)
            out["z_proj"].append(orc.z @ signs.T)
            print(f"round {r + 1}: checkpoint, {time.time() - t0:.0f} s", flush=True)
        elif (r + 1) % 10 == 0:
            print(f"round {r + 1}: {time.time() - t0:.0f} s", flush=True)
    path = args.out or os.path.join(ROOT, "tests", "golden", f"cfg{args.config}_checkpoints.npz")
    np.savez_compressed(path, workload=np.array(w.name), coords=coords, **{k: np.stack(v) for k, v in out.items()})
    print("wrote", path, os.path.getsize(path), "bytes")


if __name__ == "__main__":
    main()
