"""Writes the stored oracle references for the large workloads (configs 2-5).

Calls only the CPU oracle and the seeded input generator; nothing here comes
from the HIP path.  For each workload it stores the loss, the log-sum-exp of
every row, and exact dX rows / dW rows for a fixed sample of rows and
vocabulary ids (full fp64 oracle arithmetic; stored as float32, which costs
6e-8 relative, far below the parity tolerance).

    python tests/golden/make_golden.py [config ...]      # default: 2 3 4 5
    python tests/golden/make_golden.py rmsnorm3          # RMSNorm in front of config 3
"""
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402
from oracle import flce_oracle  # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))
N_ROWS, N_VOCAB = 32, 32


def sample_indices(w):
    g = np.random.default_rng(12345 + w.seed)
    ign = np.nonzero(w.targets == w.ignore_index)[0]
    val = np.nonzero(w.targets != w.ignore_index)[0]
    rows = [0, w.BT - 1, 255, 256, w.BT // 2 - 1, w.BT // 2]        # tile and chunk edges
    rows += list(ign[:3])                                          # ignored rows give zeros
    rows += list(g.choice(val, N_ROWS, replace=False))
    rows = np.array(sorted(set(int(r) for r in rows))[:N_ROWS + 4], dtype=np.int64)
    counts = np.bincount(w.targets[val], minlength=w.V)
    hot = list(np.argsort(-counts)[:6])                            # most frequent targets
    cold = list(np.nonzero(counts == 0)[0][:6])                    # never a target
    vocab = [0, w.V - 1, 255, 256] + hot + cold
    vocab += list(g.choice(w.V, N_VOCAB, replace=False))
    vocab = np.array(sorted(set(int(v) for v in vocab))[:N_VOCAB + 8], dtype=np.int64)
    return rows, vocab


RMSNORM_EPS = 1e-5


def rmsnorm_reference(idx):
    """RMSNorm + projection + cross entropy on workload idx: loss, dgamma (needs the
    whole dX), dh for the sampled rows, dW for the sampled vocabulary ids."""
    t0 = time.time()
    w = workloads.make_config(idx)
    h, gamma = workloads.make_rmsnorm_inputs(w)
    rows, vocab = sample_indices(w)
    r = flce_oracle.rmsnorm_flce(h.astype(np.float64), gamma.astype(np.float64), RMSNORM_EPS,
                                 w.W.astype(np.float64), w.targets, w.ignore_index, vocab=vocab)
    out = os.path.join(HERE, f"rmsnorm_config{idx}_{w.name}.npz")
    np.savez_compressed(out, loss=np.float64(r.loss), rows=rows, vocab=vocab, eps=np.float64(RMSNORM_EPS),
                        dh_rows=r.dh[rows].astype(np.float32), dW_rows=r.dW.astype(np.float32),
                        dgamma=r.dgamma.astype(np.float32),
                        dh_absmax=np.float64(np.abs(r.dh).max()), checksum=workloads.checksum(w),
                        h_sum=np.float64(h.astype(np.float64).sum()), gamma_sum=np.float64(gamma.sum()))
    print(f"rmsnorm config {idx}: loss={r.loss:.12f} -> {out} ({os.path.getsize(out) / 1e6:.2f} MB, "
          f"{time.time() - t0:.0f} s)", flush=True)


def main(argv):
    if argv and argv[0].startswith("rmsnorm"):
        return rmsnorm_reference(int(argv[0][len("rmsnorm"):]))
    configs = [int(a) for a in argv] or [2, 3, 4, 5]
    for idx in configs:
        t0 = time.time()
        w = workloads.make_config(idx)
        rows, vocab = sample_indices(w)
        r = flce_oracle.flce(w.X, w.W, w.targets, w.ignore_index, rows=rows, vocab=vocab)
        out = os.path.join(HERE, f"config{idx}_{w.name}.npz")
        np.savez_compressed(out, loss=np.float64(r.loss), lse=r.lse, rows=rows, vocab=vocab,
                            dX_rows=r.dX.astype(np.float32), dW_rows=r.dW.astype(np.float32),
                            dX_absmax_sample=np.float64(np.abs(r.dX).max()),
                            dW_absmax_sample=np.float64(np.abs(r.dW).max()),
                            n_valid=np.int64(w.n_valid), checksum=workloads.checksum(w),
                            shape=np.array([w.BT, w.H, w.V], dtype=np.int64))
        print(f"config {idx} {w.name}: loss={r.loss:.12f} n_valid={w.n_valid} "
              f"-> {out} ({os.path.getsize(out) / 1e6:.2f} MB, {time.time() - t0:.0f} s)", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
