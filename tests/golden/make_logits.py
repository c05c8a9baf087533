"""Writes the stored oracle logits that the full-size GPU parity tests compare against.

Only `oracle/` (the plain CPU definition of the merged model, Section 3.3 / Fig. 1(c)) and `mt_synth/` (seeded
inputs and weights, no arithmetic of the method) are used: no value in these files ever comes from the HIP
library.  The oracle takes minutes to hours for these sizes, which is why its results are stored instead of being
recomputed inside a test.

    python tests/golden/make_logits.py [workload ...]      # default: every workload below

Files (float32, C order), one per workload, beside this script:
    oracle_logits_base.npy     [128][32][16]  batches 0..127 of `base`  (4096 sequences, B = 32, S = 128)
    oracle_logits_hetero.npy   [1][64][16]    batch 0 of `hetero`       (B = 64, S = 128)
    oracle_logits_latency.npy  [1][8][16]     batch 0 of `latency`      (B = 8,  S = 64; smaller B are its prefixes)
    oracle_logits_large.npy    [1][128][16]   batch 0 of `large`        (B = 128, S = 256)
A finished batch is kept in `<file>.partial.npy` so that an interrupted run resumes where it stopped.
"""
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import mt_synth as ms  # noqa: E402
import oracle  # noqa: E402

# workload -> number of batches (batch_index 0..n-1 of the workload's own input seed, its own batch size)
PLAN = {"hetero": 1, "latency": 1, "large": 1, "base": 128}


def path_of(name: str) -> str:
    return os.path.join(HERE, f"oracle_logits_{name}.npy")


def make(name: str, n_batches: int) -> None:
    spec = ms.get_config(name)
    out_path = path_of(name)
    part_path = out_path[:-4] + ".partial.npy"
    out = np.full((n_batches, spec.batch, spec.n_logits), np.nan, dtype=np.float32)
    if os.path.exists(part_path):
        old = np.load(part_path)
        if old.shape == out.shape:
            out = old
    trunk, _ = ms.make_trunk_params(spec)
    tasks = [ms.make_task_params(spec, t)[0] for t in range(spec.n_tasks)]
    orc = oracle.Oracle(spec, trunk, tasks)
    t0 = time.time()
    for bi in range(n_batches):
        if np.isfinite(out[bi]).all():
            continue
        ids, mask, _ = ms.make_inputs(spec, batch_index=bi)
        out[bi] = orc.mt_forward(ids, mask)
        np.save(part_path, out)
        print(f"{name}: batch {bi + 1}/{n_batches} done, {time.time() - t0:.0f} s", flush=True)
    assert np.isfinite(out).all()
    np.save(out_path, out)
    if os.path.exists(part_path):
        os.remove(part_path)
    print(f"{name}: wrote {out_path} {out.shape}", flush=True)


if __name__ == "__main__":
    names = sys.argv[1:] or list(PLAN)
    for nm in names:
        make(nm, PLAN[nm])
