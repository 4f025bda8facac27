"""Pins for the CPU oracle: closed forms, invariants, finite differences,
special cases that reduce to a textbook or library routine.  None of these
re-uses the oracle's own formula; a dropped term, a wrong sign or index or a
transposed operand in oracle/flce_oracle.cpp fails at least one of them."""
import math

import numpy as np
import pytest
import torch

import workloads
from oracle import flce_oracle as oracle

IGN = -100


def _case(BT=6, H=5, V=7, seed=3, n_ign=1, w_std=0.7):
    g = np.random.default_rng(seed)
    X = g.standard_normal((BT, H))
    W = g.standard_normal((V, H)) * w_std
    t = g.integers(0, V, size=BT).astype(np.int64)
    for i in range(n_ign):
        t[(2 + 3 * i) % BT] = IGN
    return X, W, t


def test_gradients_match_central_finite_differences():
    # Pins dX, dW (every entry), the 1/N_valid factor and ignore handling
    # against the loss alone.
    X, W, t = _case()
    r = oracle.flce(X, W, t, IGN)
    eps = 1e-6

    def loss_at(Xp, Wp):
        return oracle.flce(Xp, Wp, t, IGN, want_dX=False, want_dW=False).loss

    fdX = np.zeros_like(X)
    for idx in np.ndindex(*X.shape):
        Xp, Xm = X.copy(), X.copy()
        Xp[idx] += eps
        Xm[idx] -= eps
        fdX[idx] = (loss_at(Xp, W) - loss_at(Xm, W)) / (2 * eps)
    fdW = np.zeros_like(W)
    for idx in np.ndindex(*W.shape):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += eps
        Wm[idx] -= eps
        fdW[idx] = (loss_at(X, Wp) - loss_at(X, Wm)) / (2 * eps)
    assert np.abs(fdX - r.dX).max() <= 1e-8 * max(1.0, np.abs(r.dX).max())
    assert np.abs(fdW - r.dW).max() <= 1e-8 * max(1.0, np.abs(r.dW).max())
    assert np.abs(r.dX).max() > 1e-3 and np.abs(r.dW).max() > 1e-3


@pytest.mark.parametrize("BT,H,V,n_ign", [(6, 5, 7, 1), (70, 33, 129, 9), (130, 16, 50, 0)])
def test_matches_library_cross_entropy_with_autograd(BT, H, V, n_ign):
    # The whole definition against a library routine: fp64 torch CPU
    # cross_entropy(X @ W.T) with ignore_index and mean reduction, plus autograd.
    X, W, t = _case(BT, H, V, seed=BT, n_ign=n_ign)
    r = oracle.flce(X, W, t, IGN, want_G=True)
    Xt = torch.tensor(X, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    Z = Xt @ Wt.T
    Z.retain_grad()
    loss = torch.nn.functional.cross_entropy(Z, torch.tensor(t), ignore_index=IGN, reduction="mean")
    loss.backward()
    assert abs(r.loss - loss.item()) <= 1e-13 * abs(loss.item())
    np.testing.assert_allclose(r.dX, Xt.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dW, Wt.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.G, Z.grad.numpy(), rtol=0, atol=1e-15)
    np.testing.assert_allclose(r.lse, torch.logsumexp(Z.detach(), dim=1).numpy(), rtol=1e-14)


def test_dlogit_rows_sum_to_zero_and_ignored_rows_are_zero():
    X, W, t = _case(40, 12, 300, seed=5, n_ign=7)
    r = oracle.flce(X, W, t, IGN, want_G=True)
    ign = t == IGN
    assert ign.sum() >= 5
    assert np.abs(r.G.sum(axis=1)).max() <= 1e-15 * 300
    assert (r.G[ign] == 0).all() and (r.dX[ign] == 0).all()
    assert np.abs(r.G[~ign]).max() > 0
    # consequence for the weight gradient: its rows sum to the zero vector
    assert np.abs(r.dW.sum(axis=0)).max() <= 1e-14


def test_zero_weight_closed_form():
    # W = 0: uniform softmax. loss = log V, dX = 0,
    # dW[v] = (1/N) sum_i (1/V - [t_i = v]) X_i over valid i.
    X, _, t = _case(30, 9, 17, seed=11, n_ign=4)
    V, H = 17, 9
    r = oracle.flce(X, np.zeros((V, H)), t, IGN)
    assert abs(r.loss - math.log(V)) <= 1e-15 * math.log(V) * 4
    assert (r.dX == 0).all()
    valid = t != IGN
    N = valid.sum()
    expect = np.tile(X[valid].sum(axis=0) / V, (V, 1))
    for i in np.nonzero(valid)[0]:
        expect[t[i]] -= X[i]
    expect /= N
    np.testing.assert_allclose(r.dW, expect, rtol=0, atol=1e-15)


def test_zero_hidden_closed_form():
    # X = 0: loss = log V, dW = 0, dX_i = (1/N)(mean_v W_v - W_{t_i}).
    _, W, t = _case(30, 9, 17, seed=12, n_ign=4)
    r = oracle.flce(np.zeros((30, 9)), W, t, IGN)
    assert abs(r.loss - math.log(17)) <= 1e-15 * 8
    assert (r.dW == 0).all()
    valid = t != IGN
    N = valid.sum()
    expect = np.zeros((30, 9))
    for i in np.nonzero(valid)[0]:
        expect[i] = (W.mean(axis=0) - W[t[i]]) / N
    np.testing.assert_allclose(r.dX, expect, rtol=0, atol=1e-15)


def test_two_classes_reduce_to_logistic_regression():
    # V = 2: loss_i = softplus(-(z_t - z_other)); dz_t = -sigmoid(-(z_t - z_other)).
    g = np.random.default_rng(8)
    X = g.standard_normal((11, 4))
    W = g.standard_normal((2, 4))
    t = g.integers(0, 2, size=11).astype(np.int64)
    r = oracle.flce(X, W, t, IGN, want_G=True)
    d = X @ (W[1] - W[0])
    margin = np.where(t == 1, d, -d)
    expect = np.mean(np.log1p(np.exp(-margin)))
    assert abs(r.loss - expect) <= 1e-14
    sig = 1.0 / (1.0 + np.exp(margin))
    np.testing.assert_allclose(r.G[np.arange(11), t], -sig / 11, rtol=0, atol=1e-15)


def test_shift_of_every_weight_row_leaves_loss_and_dlogits_unchanged():
    # Adding one vector c to all rows of W adds <x_i, c> to every logit of row i;
    # softmax does not see it.  A large c exercises the max subtraction.
    X, W, t = _case(20, 6, 31, seed=21, n_ign=3)
    c = np.full(6, 40.0)
    a = oracle.flce(X, W, t, IGN, want_G=True)
    b = oracle.flce(X, W + c, t, IGN, want_G=True)
    assert np.isfinite(b.loss) and abs(a.loss - b.loss) <= 1e-11
    np.testing.assert_allclose(a.G, b.G, rtol=0, atol=1e-13)
    # logits of several hundred must not overflow
    big = oracle.flce(X * 50, W * 20, t, IGN)
    assert np.isfinite(big.loss) and np.isfinite(big.dX).all() and np.isfinite(big.dW).all()


def test_rows_are_additive_so_any_chunking_gives_the_same_result():
    # Paper, FLCE paragraph: the weight gradient is a sum over rows, and a single
    # row is the special case of a chunk of size one.  Un-normalised results of
    # disjoint row sets must add up to the full result.
    X, W, t = _case(23, 7, 19, seed=30, n_ign=5)
    full = oracle.flce(X, W, t, IGN)
    N = (t != IGN).sum()
    for chunk in (1, 7, 23):
        loss_sum = 0.0
        dW = np.zeros_like(W)
        dX = np.zeros_like(X)
        for s in range(0, 23, chunk):
            sl = slice(s, s + chunk)
            n = (t[sl] != IGN).sum()
            part = oracle.flce(X[sl], W, t[sl], IGN)
            loss_sum += part.loss * n
            dW += part.dW * n
            dX[sl] = part.dX * n
        assert abs(loss_sum / N - full.loss) <= 1e-13
        np.testing.assert_allclose(dW / N, full.dW, rtol=0, atol=1e-14)
        np.testing.assert_allclose(dX / N, full.dX, rtol=0, atol=1e-14)


def test_selected_rows_and_vocab_equal_slices_of_the_full_result():
    w = workloads.make(150, 40, 333, "bf16", ignore=("iid", 0.2), seed=77)
    full = oracle.flce(w.X, w.W, w.targets, IGN)
    rows = np.array([0, 149, 63, 64, 65, 5])
    vocab = np.array([332, 0, 17, int(w.targets[w.targets >= 0][0])])
    part = oracle.flce(w.X, w.W, w.targets, IGN, rows=rows, vocab=vocab)
    assert part.loss == full.loss
    np.testing.assert_array_equal(part.dX, full.dX[rows])
    np.testing.assert_array_equal(part.dW, full.dW[vocab])
    np.testing.assert_array_equal(part.lse, full.lse)


def test_f32_held_inputs_equal_widened_inputs():
    w = workloads.make(70, 24, 100, "bf16", ignore=("iid", 0.1), seed=78)
    a = oracle.flce(w.X, w.W, w.targets, IGN)
    b = oracle.flce(w.X.astype(np.float64), w.W.astype(np.float64), w.targets, IGN)
    assert a.loss == b.loss
    np.testing.assert_array_equal(a.dX, b.dX)
    np.testing.assert_array_equal(a.dW, b.dW)


def test_standalone_cross_entropy_matches_library_and_flce_dlogits():
    X, W, t = _case(33, 8, 65, seed=40, n_ign=6)
    Z = X @ W.T
    loss, G, lse = oracle.cross_entropy(Z, t, IGN)
    Zt = torch.tensor(Z, requires_grad=True)
    ref = torch.nn.functional.cross_entropy(Zt, torch.tensor(t), ignore_index=IGN)
    ref.backward()
    assert abs(loss - ref.item()) <= 1e-14
    np.testing.assert_allclose(G, Zt.grad.numpy(), rtol=0, atol=1e-15)
    r = oracle.flce(X, W, t, IGN, want_G=True)
    np.testing.assert_allclose(G, r.G, rtol=0, atol=1e-15)


def test_no_valid_row_gives_zero_loss_and_gradients():
    # A reading, not a pin: the paper does not say what an all-ignored batch gives.
    X, W, _ = _case(5, 4, 6)
    r = oracle.flce(X, W, np.full(5, IGN, dtype=np.int64), IGN)
    assert r.loss == 0.0 and (r.dX == 0).all() and (r.dW == 0).all()


def test_out_of_range_target_is_rejected():
    X, W, t = _case()
    t[0] = 7
    with pytest.raises(ValueError):
        oracle.flce(X, W, t, IGN)


def test_brute_force_single_row_by_hand():
    # One row, three classes, numbers small enough to do with math.* alone.
    X = np.array([[1.0, -2.0]])
    W = np.array([[0.5, 0.25], [-1.0, 0.0], [0.0, 1.5]])
    z = [0.5 - 0.5, -1.0, -3.0]
    e = [math.exp(v) for v in z]
    y = [v / sum(e) for v in e]
    r = oracle.flce(X, W, np.array([2]), IGN, want_G=True)
    assert abs(r.loss - (-math.log(y[2]))) <= 1e-15
    g = [y[0], y[1], y[2] - 1.0]
    np.testing.assert_allclose(r.G[0], g, atol=1e-16)
    dX = [sum(g[v] * W[v, h] for v in range(3)) for h in range(2)]
    np.testing.assert_allclose(r.dX[0], dX, atol=1e-16)
    for v in range(3):
        np.testing.assert_allclose(r.dW[v], [g[v] * 1.0, g[v] * -2.0], atol=1e-16)


# ---- several heads on shared hidden states (paper section 4.2, Medusa paragraph) ----

def _heads_case(n=3, BT=24, H=6, V=11, seq=8, seed=5):
    g = np.random.default_rng(seed)
    X = g.standard_normal((BT, H))
    Ws = [g.standard_normal((V, H)) * 0.6 for _ in range(n)]
    base = g.integers(0, V, size=BT).astype(np.int64)
    base[3] = IGN
    ts = [base]
    for j in range(1, n):       # head j looks j tokens further inside its sequence
        t = np.full(BT, IGN, dtype=np.int64)
        for s in range(0, BT, seq):
            t[s:s + seq - j] = base[s + j:s + seq]
        ts.append(t)
    return X, Ws, ts, [1.0, 0.8, 0.64][:n]


def test_multihead_matches_autograd_of_the_weighted_sum_of_library_losses():
    # dX must collect every head's contribution with its weight, dW_j only head
    # j's; each head divides by ITS OWN number of valid rows.
    X, Ws, ts, wts = _heads_case()
    r = oracle.flce_multihead(X, Ws, ts, wts, IGN)
    Xt = torch.tensor(X, requires_grad=True)
    Wt = [torch.tensor(W, requires_grad=True) for W in Ws]
    per_head = [torch.nn.functional.cross_entropy(Xt @ W.T, torch.tensor(t), ignore_index=IGN)
                for W, t in zip(Wt, ts)]
    total = sum(w * l for w, l in zip(wts, per_head))
    total.backward()
    assert abs(r.loss - total.item()) <= 1e-13 * abs(total.item())
    for mine, ref in zip(r.head_losses, per_head):
        assert abs(mine - ref.item()) <= 1e-13 * abs(ref.item())
    np.testing.assert_allclose(r.dX, Xt.grad.numpy(), rtol=0, atol=1e-14)
    for mine, ref in zip(r.dWs, Wt):
        np.testing.assert_allclose(mine, ref.grad.numpy(), rtol=0, atol=1e-14)
    # the heads see different numbers of valid rows, so a shared divisor would show
    assert len({int((t != IGN).sum()) for t in ts}) == len(ts)


def test_multihead_with_one_head_is_the_single_head_result():
    X, Ws, ts, _ = _heads_case(n=1)
    r1 = oracle.flce_multihead(X, Ws, ts, None, IGN)
    r0 = oracle.flce(X, Ws[0], ts[0], IGN)
    assert r1.loss == r0.loss and r1.head_losses == [r0.loss]
    assert np.array_equal(r1.dX, r0.dX) and np.array_equal(r1.dWs[0], r0.dW)


def test_multihead_same_head_twice_doubles_loss_and_dX_but_not_dW():
    X, Ws, ts, _ = _heads_case(n=1)
    r0 = oracle.flce(X, Ws[0], ts[0], IGN)
    r2 = oracle.flce_multihead(X, [Ws[0], Ws[0].copy()], [ts[0], ts[0]], None, IGN)
    assert abs(r2.loss - 2 * r0.loss) <= 1e-15 * abs(r0.loss)
    np.testing.assert_allclose(r2.dX, 2 * r0.dX, rtol=0, atol=1e-16)
    for d in r2.dWs:
        np.testing.assert_allclose(d, r0.dW, rtol=0, atol=0)


def test_multihead_workload_shifts_targets_inside_sequences():
    m = workloads.make_multihead(3, BT=40, H=8, V=50, seq=16, dtype="f32", seed=9)
    t0 = m.targets[0]
    for j in (1, 2):
        tj = m.targets[j]
        for s in range(0, 40, 16):
            e = min(s + 16, 40)
            assert (tj[e - j:e] == IGN).all()
            assert np.array_equal(tj[s:e - j], t0[s + j:e])
    assert m.weights == [1.0, 0.8, 0.8 ** 2]
    assert not np.array_equal(m.Ws[1], m.Ws[2]) and m.Ws[0] is m.base.W


# ---- RMSNorm in front of the projection (paper section 3.2, RMSNorm paragraph) ----

def _norm_case(BT=9, H=6, V=7, seed=21):
    g = np.random.default_rng(seed)
    h = g.standard_normal((BT, H)) * 1.7
    gamma = 1.0 + 0.3 * g.standard_normal(H)
    W = g.standard_normal((V, H)) * 0.5
    t = g.integers(0, V, size=BT).astype(np.int64)
    t[4] = IGN
    return h, gamma, W, t


@pytest.mark.parametrize("eps", [1e-6, 0.5])
def test_rmsnorm_flce_matches_autograd_of_the_composed_definition(eps):
    # A large eps makes a wrong place of eps (outside the root, inside the mean) visible.
    h, gamma, W, t = _norm_case()
    r = oracle.rmsnorm_flce(h, gamma, eps, W, t, IGN)
    ht = torch.tensor(h, requires_grad=True)
    gt = torch.tensor(gamma, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    y = ht * torch.rsqrt(ht.pow(2).mean(dim=1, keepdim=True) + eps) * gt
    loss = torch.nn.functional.cross_entropy(y @ Wt.T, torch.tensor(t), ignore_index=IGN)
    loss.backward()
    assert abs(r.loss - loss.item()) <= 1e-13 * abs(loss.item())
    np.testing.assert_allclose(r.y, y.detach().numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dh, ht.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dgamma, gt.grad.numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dW, Wt.grad.numpy(), rtol=0, atol=1e-14)
    assert np.abs(r.dh).max() > 1e-3 and np.abs(r.dgamma).max() > 1e-3


def test_rmsnorm_gradients_match_finite_differences_of_the_loss():
    h, gamma, W, t = _norm_case(BT=5, H=4, V=5)
    eps, d = 1e-3, 1e-6
    r = oracle.rmsnorm_flce(h, gamma, eps, W, t, IGN)

    def loss_at(hp, gp):
        return oracle.rmsnorm_flce(hp, gp, eps, W, t, IGN, want_dh=False, want_dW=False).loss

    fd_h = np.zeros_like(h)
    for idx in np.ndindex(*h.shape):
        hp, hm = h.copy(), h.copy()
        hp[idx] += d
        hm[idx] -= d
        fd_h[idx] = (loss_at(hp, gamma) - loss_at(hm, gamma)) / (2 * d)
    fd_g = np.zeros_like(gamma)
    for j in range(gamma.size):
        gp, gm = gamma.copy(), gamma.copy()
        gp[j] += d
        gm[j] -= d
        fd_g[j] = (loss_at(h, gp) - loss_at(h, gm)) / (2 * d)
    assert np.abs(fd_h - r.dh).max() <= 1e-8 * max(1.0, np.abs(r.dh).max())
    assert np.abs(fd_g - r.dgamma).max() <= 1e-8 * max(1.0, np.abs(r.dgamma).max())


def test_rmsnorm_without_eps_is_scale_invariant_and_dh_is_orthogonal_to_h():
    # eps = 0: y does not change when a row of h is scaled, so the loss cannot change
    # along h: every row of dh is orthogonal to its row of h, and dh scales with 1/a.
    h, gamma, W, t = _norm_case()
    r1 = oracle.rmsnorm_flce(h, gamma, 0.0, W, t, IGN)
    r3 = oracle.rmsnorm_flce(3.0 * h, gamma, 0.0, W, t, IGN)
    assert abs(r1.loss - r3.loss) <= 1e-14
    np.testing.assert_allclose(r3.dh, r1.dh / 3.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(r3.dgamma, r1.dgamma, rtol=0, atol=1e-14)
    assert np.abs((r1.dh * h).sum(axis=1)).max() <= 1e-15
    # rows of y have mean square gamma-weighted 1: with gamma = 1, |y_i|^2 = n
    r = oracle.rmsnorm_flce(h, np.ones_like(gamma), 0.0, W, t, IGN, want_dh=False, want_dW=False)
    np.testing.assert_allclose((r.y ** 2).sum(axis=1), h.shape[1], rtol=1e-14)


def test_rmsnorm_of_unit_rms_rows_with_unit_gamma_is_the_plain_path():
    h, gamma, W, t = _norm_case()
    h = h / np.sqrt((h * h).mean(axis=1, keepdims=True))      # every row has RMS 1
    r = oracle.rmsnorm_flce(h, np.ones_like(gamma), 0.0, W, t, IGN)
    r0 = oracle.flce(h, W, t, IGN)
    assert abs(r.loss - r0.loss) <= 1e-14
    np.testing.assert_allclose(r.dW, r0.dW, rtol=0, atol=1e-14)
    np.testing.assert_allclose(r.dgamma, (r0.dX * h).sum(axis=0), rtol=0, atol=1e-14)
