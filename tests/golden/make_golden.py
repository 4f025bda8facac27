"""Writes the stored oracle references for the large workloads (configs 2-5).

Calls only the CPU oracle and the seeded input generator; nothing here comes
from the HIP path.  The oracle is run IN FULL (every dX row, every dW row, fp64)
and the file keeps what a GPU test can check against without redoing 1e13 fp64
flops:

  loss, lse            the loss and the log-sum-exp of every row
  rows, dX_q/dX_scale  exact dX rows: one random row out of every 256 rows of the
                       batch (every tile row of the dX product), the rows on both
                       sides of every multiple of 256 in the list of rows that have
                       a target (first and last row of a chunk of such rows,
                       whatever multiple of 256 the chunk size is), tile and batch
                       edges, three ignored rows
  vocab, dW_q/dW_scale exact dW rows: one random vocabulary id out of every 256
                       (every tile row of the dW product), the most frequent
                       targets, ids that are never a target, tile and table edges
  *_blk_sum, *_blk_sq  sum and sum of squares of every 256 x 256 block of dX, dW
  *_proj, *_norm       for EVERY row of dX and dW: its dot product with a fixed
                       vector of +-1 (`signs`) and its Euclidean norm

Sampled rows are stored as int16 with one fp64 scale per row (value = q * scale,
scale = max|row| / 32767): the quantisation error is at most scale / 2, i.e.
1.6e-5 of the row's largest entry; the tests subtract it from their tolerance.

    python tests/golden/make_golden.py [config ...]      # default: 2 3 4 5
    python tests/golden/make_golden.py rmsnorm3          # RMSNorm in front of config 3
    python tests/golden/make_golden.py multihead3        # two different heads at config 3
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
TILE = 256
RMSNORM_EPS = 1e-5
MULTIHEAD_SEQ = 2048          # sequence length behind the second head's shifted targets
MULTIHEAD_WEIGHTS = (1.0, 0.8)


def sample_rows(targets, ignore_index, BT, seed):
    """Row sample for dX (see the module docstring)."""
    g = np.random.default_rng(12345 + seed)
    ign = np.nonzero(targets == ignore_index)[0]
    val = np.nonzero(targets != ignore_index)[0]
    rows = [0, BT - 1, TILE - 1, TILE, BT // 2 - 1, BT // 2]
    rows += [int(r) for r in ign[:3]]
    for r0 in range(0, BT, TILE):                         # every tile row of the batch
        rows.append(int(g.integers(r0, min(r0 + TILE, BT))))
    for k in range(TILE, len(val), TILE):                 # chunk edges among the rows that have a target
        rows += [int(val[k - 1]), int(val[k])]
    if len(val):
        rows += [int(val[0]), int(val[-1])]
    return np.array(sorted(set(r for r in rows if 0 <= r < BT)), dtype=np.int64)


def sample_vocab(targets, ignore_index, V, seed):
    """Vocabulary sample for dW (see the module docstring)."""
    g = np.random.default_rng(54321 + seed)
    val = targets[targets != ignore_index]
    counts = np.bincount(val, minlength=V)
    vocab = [0, V - 1, TILE - 1, TILE]
    vocab += [int(v) for v in np.argsort(-counts, kind="stable")[:6]]      # most frequent targets
    vocab += [int(v) for v in np.nonzero(counts == 0)[0][:6]]              # never a target
    for v0 in range(0, V, TILE):                          # every tile row of the vocabulary
        vocab.append(int(g.integers(v0, min(v0 + TILE, V))))
    return np.array(sorted(set(v for v in vocab if 0 <= v < V)), dtype=np.int64)


def quantise_rows(a):
    """int16 codes and per-row scales: a ~= q * scale[:, None], |error| <= scale / 2."""
    amax = np.abs(a).max(axis=1)
    scale = np.where(amax > 0, amax / 32767.0, 1.0)
    q = np.rint(a / scale[:, None]).astype(np.int16)
    return q, scale


def block_stats(a):
    """Sum and sum of squares of every TILE x TILE block (ragged edges allowed)."""
    R, C = a.shape
    nr, nc = (R + TILE - 1) // TILE, (C + TILE - 1) // TILE
    s = np.zeros((nr, nc))
    q = np.zeros((nr, nc))
    for i in range(nr):
        blk = a[i * TILE:(i + 1) * TILE]
        for j in range(nc):
            b = blk[:, j * TILE:(j + 1) * TILE]
            s[i, j] = b.sum()
            q[i, j] = (b * b).sum()
    return s, q


def signs_vector(H, seed):
    return np.where(np.random.default_rng(777 + seed).random(H) < 0.5, -1.0, 1.0)


def whole_matrix_fields(prefix, a, signs):
    """The fields that cover every element of a full gradient matrix."""
    s, q = block_stats(a)
    return {f"{prefix}_blk_sum": s, f"{prefix}_blk_sq": q,
            f"{prefix}_proj": a @ signs, f"{prefix}_norm": np.sqrt((a * a).sum(axis=1)),
            f"{prefix}_absmax": np.float64(np.abs(a).max())}


def sampled_fields(prefix, a, index):
    q, scale = quantise_rows(a[index])
    return {f"{prefix}_q": q, f"{prefix}_scale": scale}


def config_reference(idx):
    t0 = time.time()
    w = workloads.make_config(idx)
    rows = sample_rows(w.targets, w.ignore_index, w.BT, w.seed)
    vocab = sample_vocab(w.targets, w.ignore_index, w.V, w.seed)
    signs = signs_vector(w.H, w.seed)
    r = flce_oracle.flce(w.X, w.W, w.targets, w.ignore_index)
    out = os.path.join(HERE, f"config{idx}_{w.name}.npz")
    np.savez_compressed(out, loss=np.float64(r.loss), lse=r.lse, rows=rows, vocab=vocab,
                        signs=signs.astype(np.int8), n_valid=np.int64(w.n_valid),
                        checksum=workloads.checksum(w),
                        shape=np.array([w.BT, w.H, w.V], dtype=np.int64),
                        **sampled_fields("dX", r.dX, rows), **sampled_fields("dW", r.dW, vocab),
                        **whole_matrix_fields("dX", r.dX, signs),
                        **whole_matrix_fields("dW", r.dW, signs))
    print(f"config {idx} {w.name}: loss={r.loss:.12f} n_valid={w.n_valid} rows={len(rows)} "
          f"vocab={len(vocab)} -> {out} ({os.path.getsize(out) / 1e6:.2f} MB, {time.time() - t0:.0f} s)",
          flush=True)


def rmsnorm_reference(idx):
    """RMSNorm + projection + cross entropy on workload idx."""
    t0 = time.time()
    w = workloads.make_config(idx)
    h, gamma = workloads.make_rmsnorm_inputs(w)
    rows = sample_rows(w.targets, w.ignore_index, w.BT, w.seed)
    vocab = sample_vocab(w.targets, w.ignore_index, w.V, w.seed)
    signs = signs_vector(w.H, w.seed)
    r = flce_oracle.rmsnorm_flce(h.astype(np.float64), gamma.astype(np.float64), RMSNORM_EPS,
                                 w.W.astype(np.float64), w.targets, w.ignore_index)
    out = os.path.join(HERE, f"rmsnorm_config{idx}_{w.name}.npz")
    np.savez_compressed(out, loss=np.float64(r.loss), rows=rows, vocab=vocab, eps=np.float64(RMSNORM_EPS),
                        signs=signs.astype(np.int8), dgamma=r.dgamma,
                        checksum=workloads.checksum(w),
                        h_sum=np.float64(h.astype(np.float64).sum()), gamma_sum=np.float64(gamma.sum()),
                        **sampled_fields("dh", r.dh, rows), **sampled_fields("dW", r.dW, vocab),
                        **whole_matrix_fields("dh", r.dh, signs),
                        **whole_matrix_fields("dW", r.dW, signs))
    print(f"rmsnorm config {idx}: loss={r.loss:.12f} -> {out} ({os.path.getsize(out) / 1e6:.2f} MB, "
          f"{time.time() - t0:.0f} s)", flush=True)


def multihead_reference(idx):
    """Two heads with different weights and targets on workload idx's hidden states: head 1
    has a weight of its own and looks one position further on inside 2048-token sequences."""
    t0 = time.time()
    c = workloads.CONFIGS[idx - 1]
    m = workloads.make_multihead(2, c["BT"], c["H"], c["V"], MULTIHEAD_SEQ, c["dtype"], c["targets"],
                                 c["ignore"], seed=workloads.BASE_SEED + idx)
    w = m.base
    assert workloads.checksum(w) == workloads.checksum(workloads.make_config(idx))
    weights = list(MULTIHEAD_WEIGHTS)
    signs = signs_vector(w.H, w.seed)
    r = flce_oracle.flce_multihead(w.X, m.Ws, m.targets, weights, w.ignore_index)
    rows = sorted(set(sample_rows(m.targets[0], w.ignore_index, w.BT, w.seed).tolist()) |
                  set(sample_rows(m.targets[1], w.ignore_index, w.BT, w.seed + 1).tolist()))
    rows = np.array(rows, dtype=np.int64)
    fields = dict(loss=np.float64(r.loss), head_losses=np.array(r.head_losses), rows=rows,
                  weights=np.array(weights), seq=np.int64(MULTIHEAD_SEQ), signs=signs.astype(np.int8),
                  checksum=workloads.checksum(w),
                  t1_sum=np.int64(m.targets[1].sum()), w1_sum=np.float64(m.Ws[1].astype(np.float64).sum()),
                  **sampled_fields("dX", r.dX, rows), **whole_matrix_fields("dX", r.dX, signs))
    for j in range(2):
        vocab = sample_vocab(m.targets[j], w.ignore_index, w.V, w.seed + j)
        fields[f"vocab{j}"] = vocab
        fields.update(sampled_fields(f"dW{j}", r.dWs[j], vocab))
        fields.update(whole_matrix_fields(f"dW{j}", r.dWs[j], signs))
    out = os.path.join(HERE, f"multihead2_config{idx}_{c['name']}.npz")
    np.savez_compressed(out, **fields)
    print(f"two heads on config {idx}: loss={r.loss:.12f} heads={r.head_losses} -> {out} "
          f"({os.path.getsize(out) / 1e6:.2f} MB, {time.time() - t0:.0f} s)", flush=True)


def main(argv):
    for a in (argv or ["2", "3", "4", "5"]):
        if a.startswith("rmsnorm"):
            rmsnorm_reference(int(a[len("rmsnorm"):]))
        elif a.startswith("multihead"):
            multihead_reference(int(a[len("multihead"):]))
        else:
            config_reference(int(a))


if __name__ == "__main__":
    main(sys.argv[1:])
