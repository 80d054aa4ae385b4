"""Writes the stored oracle values for the full-size parity tests.

For one configuration it runs the CPU oracle's scoring (float64) over every scored row of every model
at the configuration's full size and stores logp, lse and entropy as float32, together with
fingerprints of the seeded inputs they belong to.  It calls nothing but `oracle/` and `workloads/`.

    python tests/golden/make_fullsize_golden.py 1        # every scored row; about 12 minutes on 8 cores
    python tests/golden/make_fullsize_golden.py 4 4096   # a seeded sample of 4096 scored rows per model
    python tests/golden/make_fullsize_golden.py 4 0 4    # every scored row, four worker processes
    python tests/golden/make_fullsize_golden.py 4r3 4096 2  # configuration 4 with three fixed rounds (245 760 tokens), a sample

The optional third argument runs the oracle in that many worker processes, each on its own blocks of
rows (the oracle's element-wise passes are single-threaded; its matrix product is a library call).

With a sample size the file also holds `rows_m`, the sorted row indices (within the model's stream)
that were evaluated: the first and last 256 scored rows plus a seeded draw from the rest; the other
entries of logp/lse/entropy stay zero.

The full-size tests use these values to build old log-probs (oracle log-prob + generator noise) and to
evaluate sampled rows of dH and dW, none of which the CPU could afford to recompute inside a test.
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads as wl                      # noqa: E402
from oracle import umas_oracle as orc       # noqa: E402


def fingerprint(t):
    """Cheap identity of the generated tensors: a few sums that any change of the generator moves."""
    return np.array([float(t["H"][:64].astype(np.float64).sum()), float(t["W"][:64].astype(np.float64).sum()),
                     float(t["ids"].astype(np.int64).sum()), float(t["noise"].astype(np.float64).sum())])


def sample_rows(rows, n_sample, seed):
    """First and last 256 scored rows (tile edges, ragged tail) plus a seeded draw from the rest."""
    if n_sample <= 0 or n_sample >= len(rows):
        return rows
    edge = min(256, n_sample // 4)
    mid = rows[edge:len(rows) - edge]
    pick = np.random.default_rng([seed, 977]).choice(len(mid), size=n_sample - 2 * edge, replace=False)
    return np.sort(np.concatenate([rows[:edge], mid[pick], rows[len(rows) - edge:]]))


_T = None


def _score_block(rr):
    a, b, c = orc.score(_T["H"], _T["W"], _T["ids"], rr)
    return rr, a[rr].astype(np.float32), b[rr].astype(np.float32), c[rr].astype(np.float32)


def main(name, n_sample=0, procs=1):
    """name: a configuration number, or `4r3` for configuration 4 with every trajectory running three rounds."""
    global _T
    cfg = int(name.split("r")[0])
    w = wl.make_workload(cfg, fixed_rounds=int(name.split("r")[1])) if "r" in name else wl.make_workload(cfg)
    st = orc.route(w.n_models, w.role_to_model, w.traj_turn_off, w.turn_role, w.turn_tok_off, w.tok_mask)
    out = {}
    for m in range(w.n_models):
        t = w.model_tensors(m)
        ra, re = int(st["model_rowsel_off"][m]), int(st["model_rowsel_off"][m + 1])
        rows = sample_rows(st["rowsel"][ra:re], n_sample, 1000 * cfg + m)
        if len(rows) < re - ra:
            out[f"rows_{m}"] = rows.astype(np.int64)
        n = len(t["ids"])
        logp, lse, ent = np.zeros(n, np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32)
        t0 = time.time()
        step = 2048
        blocks = [rows[c0:c0 + step] for c0 in range(0, len(rows), step)]
        _T = t
        if procs > 1:
            import multiprocessing as mp
            from threadpoolctl import threadpool_limits
            with threadpool_limits(limits=max(1, (os.cpu_count() or 1) // procs)):
                with mp.get_context("fork").Pool(procs) as pool:      # the workers inherit the tensors
                    results = pool.imap(_score_block, blocks)
                    done = 0
                    for rr, a, b, c in results:
                        logp[rr], lse[rr], ent[rr] = a, b, c
                        done += len(rr)
                        print(f"cfg {cfg} model {m}: {done}/{len(rows)} rows, {time.time() - t0:.0f} s", flush=True)
        else:
            for rr in blocks:
                _, a, b, c = _score_block(rr)
                logp[rr], lse[rr], ent[rr] = a, b, c
                print(f"cfg {cfg} model {m}: {rr[-1]}/{len(rows)} rows, {time.time() - t0:.0f} s", flush=True)
        out[f"logp_{m}"], out[f"lse_{m}"], out[f"entropy_{m}"] = logp, lse, ent
        out[f"fingerprint_{m}"] = fingerprint(t)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"fullsize_cfg{name}.npz")
    np.savez_compressed(path, **out)
    print("wrote", path)


if __name__ == "__main__":
    main(sys.argv[1], int(sys.argv[2]) if len(sys.argv) > 2 else 0, int(sys.argv[3]) if len(sys.argv) > 3 else 1)
