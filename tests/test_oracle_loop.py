"""Pins for the multi-step loop oracle (CPU only).  The loop is the one-step
oracle applied repeatedly under a seed / bank-block schedule; what is pinned
here is the schedule and the bank algebra of Sec. 3.2 end to end."""
import math
from types import SimpleNamespace

import numpy as np
import pytest

from oracle import zo_loop
from oracle import zo_oracle as zo


def _problem(seed=0, d=24, hid=32, vocab=40, K=2, r=4, n_blocks=3, lens=(6, 6, 5, 5)):
    """Two linears and a head; K directions, candidates (+, -) per direction; the +/- sequences of a
    direction carry the same rows."""
    rng = np.random.default_rng(seed)
    seq_cand, rows, tg = [], [], []
    for i, ln in enumerate(lens):
        k = i % K
        x = rng.standard_normal((ln, d)); y = rng.integers(0, vocab, ln)
        for sgn in (0, 1):
            seq_cand.append(2 * k + sgn); rows.append(x); tg.append(y)
    lens2 = [len(x) for x in rows]
    cu = np.zeros(len(lens2) + 1, np.int32); cu[1:] = np.cumsum(lens2)
    cand_dir = np.repeat(np.arange(K), 2).astype(np.int32)
    cand_sign = np.tile([1.0, -1.0], K).astype(np.float32)
    batch = zo.Batch(cu, np.array(seq_cand, np.int32), cand_dir, cand_sign, np.zeros(K, np.uint64))
    R = n_blocks * K * r
    layers = []
    for i, (m, n) in enumerate([(hid, d), (d, hid)]):
        layers.append(SimpleNamespace(W=(rng.standard_normal((m, n)) / math.sqrt(n)).astype(np.float32),
                                      tensor_id=2 * i, act=1 if i == 0 else 0,
                                      P=np.zeros((m, R), np.float32), Vb=np.zeros((n, R), np.float32), R_used=R))
    head = (rng.standard_normal((vocab, d)) / math.sqrt(d)).astype(np.float32)
    return batch, np.concatenate(rows).astype(np.float32), layers, head, np.concatenate(tg).astype(np.int32), r


def test_schedule_reuses_v_over_an_interval_and_walks_the_blocks():
    K, r, nu, B = 3, 8, 4, 2
    seen_u = set()
    for t in range(nu * B):
        s = zo_loop.schedule(t, nu, B, K, r, 1000, 5000)
        assert s.interval == t // nu and s.block == s.interval % B and s.append == (t % nu == 0)
        assert list(s.seed_v) == [5000 + s.interval * K + j for j in range(K)]      # one V per interval
        assert not (set(s.seed_u.tolist()) & seen_u)                                  # a fresh U every step
        seen_u |= set(s.seed_u.tolist())
        assert list(s.col0) == [(s.block * K + j) * r for j in range(K)]
    blocks = [tuple(zo_loop.schedule(t, nu, B, K, r, 0, 0).col0) for t in range(0, nu * B, nu)]
    flat = sorted(c for b in blocks for c in b)
    assert flat == list(range(0, B * K * r, r))                                       # blocks tile the bank exactly
    assert zo_loop.schedule(nu * B, nu, B, K, r, 0, 0).block == 0                     # then wraps
    s = zo_loop.schedule(7, 2, 4, 1, 8, (1 << 64) - 3, 0)
    assert int(s.seed_u[0]) == ((1 << 64) - 3 + 7) % (1 << 64)                        # seeds wrap modulo 2^64


def test_bank_loop_equals_dense_weight_loop():
    """Eq. (layer-coupling), Eq. (combined-probe), Eq. (bank): keeping P_k per interval and probing
    W_0 + (P_k +- eps U_t) V_k^T is the same optimisation as updating dense weights.  Catches a V
    taken from the wrong interval, an update written to the wrong block, an open that does not reset
    the block, and a probe that ignores the bank."""
    batch, X, layers, head, tg, r = _problem()
    kw = dict(r=r, eps=1e-2, dtype="f32", reduction=0, steps=6, nu=2, lr=1e-2, base_u=77, base_v=991)
    outs, banks = zo_loop.run_loop(batch, X, layers, head, tg, n_blocks=3, **kw)
    outs_d, Ws = zo_loop.run_loop_dense(batch, X, layers, head, tg, **kw)
    moved = 0.0
    for t, (a, b) in enumerate(zip(outs, outs_d)):
        np.testing.assert_allclose(a["cand_loss"], b["cand_loss"], rtol=1e-6, err_msg="step %d" % t)
        np.testing.assert_allclose(a["proj_grad"], b["proj_grad"], rtol=1e-3, atol=1e-4, err_msg="step %d" % t)
    for l, bank, W in zip(layers, banks, Ws):
        W_eff = l.W.astype(np.float64) + bank.P.astype(np.float64) @ bank.Vb.astype(np.float64).T
        np.testing.assert_allclose(W_eff, W, rtol=0, atol=2e-6)
        moved = max(moved, np.abs(W - l.W).max())
    assert moved > 0.1                                   # the loop really moved the weights
    assert outs[-1]["cand_loss"][0] < outs[0]["cand_loss"][0] - 0.1   # and the loss went down


def test_planted_mistake_v_of_the_wrong_interval_is_caught(monkeypatch):
    batch, X, layers, head, tg, r = _problem()
    kw = dict(r=r, eps=1e-2, dtype="f32", reduction=0, steps=4, nu=2, lr=1e-2, base_u=77, base_v=991)
    outs_d, _ = zo_loop.run_loop_dense(batch, X, layers, head, tg, **kw)
    good = zo_loop.schedule

    def bad(step, nu, n_blocks, K, r, base_u, base_v):
        s = good(step, nu, n_blocks, K, r, base_u, base_v)
        s.seed_v = s.seed_v + np.uint64(step % nu)       # V changes inside the interval
        return s
    monkeypatch.setattr(zo_loop, "schedule", bad)
    outs, _ = zo_loop.run_loop(batch, X, layers, head, tg, n_blocks=3, **kw)
    monkeypatch.setattr(zo_loop, "schedule", good)
    assert not np.allclose(outs[-1]["cand_loss"], outs_d[-1]["cand_loss"], rtol=1e-6)


def test_bank_exhaustion_is_an_error_unless_wrapping_is_asked_for():
    batch, X, layers, head, tg, r = _problem(n_blocks=2)
    kw = dict(r=r, eps=1e-2, dtype="f32", reduction=0, nu=1, lr=0.1, base_u=1, base_v=2)
    with pytest.raises(ValueError):
        zo_loop.run_loop(batch, X, layers, head, tg, steps=3, n_blocks=2, **kw)
    outs, banks = zo_loop.run_loop(batch, X, layers, head, tg, steps=3, n_blocks=2, allow_wrap=True, **kw)
    # step 2 reopened block 0: it now holds exactly that step's update, block 1 still holds step 1's
    b2 = zo.Batch(batch.cu_seqlens, batch.seq_cand, batch.cand_dir, batch.cand_sign, outs[2]["schedule"].seed_u,
                  outs[2]["schedule"].seed_v)
    l = layers[0]
    U, V = zo.direction_factors(b2, 0, l.W.shape[0], l.W.shape[1], r, l.tensor_id, "f32")
    beta = -np.float32(0.1) * np.float32(outs[2]["proj_grad"][0]) * (np.float32(1) / np.float32(2))
    np.testing.assert_allclose(banks[0].P[:, 0:r], beta * U, rtol=1e-5, atol=1e-9)
    np.testing.assert_array_equal(banks[0].Vb[:, 0:r], V.astype(np.float32))


def test_separate_v_seed_changes_v_only():
    b = zo.Batch(np.array([0, 4], np.int32), np.array([0], np.int32), np.array([0], np.int32),
                 np.array([1.0], np.float32), np.array([5], np.uint64))
    U0, V0 = zo.direction_factors(b, 0, 12, 20, 4, 6, "f32")
    b.dir_seed_v = np.array([9], np.uint64)
    U1, V1 = zo.direction_factors(b, 0, 12, 20, 4, 6, "f32")
    assert np.array_equal(U0, U1) and not np.array_equal(V0, V1)
    b.dir_seed_v = np.array([5], np.uint64)
    assert np.array_equal(V0, zo.direction_factors(b, 0, 12, 20, 4, 6, "f32")[1])


def test_fold_moves_the_bank_into_the_base_without_changing_the_map():
    """Eq. (bank) read right to left: W_0 + P Vb^T folded into the base and an empty bank give the same
    centre forward.  Catches a transposed factor, columns beyond R_used leaking in, a bank left full."""
    rng = np.random.default_rng(4)
    m, n, R = 20, 28, 6
    W = rng.standard_normal((m, n))
    bank = zo.Bank(rng.standard_normal((m, R + 3)).astype(np.float32), rng.standard_normal((n, R + 3)).astype(np.float32), R)
    b = zo.Batch(np.array([0, 5], np.int32), np.array([0], np.int32), np.array([-1], np.int32),
                 np.array([0.0], np.float32), np.zeros(0, np.uint64))
    X = rng.standard_normal((5, n))
    Wn, empty = zo.fold_bank(W, bank, "f64")
    np.testing.assert_allclose(zo.probe_linear(b, X, Wn, 4, 1e-3, 0, empty, out_dtype="f64"),
                               zo.probe_linear(b, X, W, 4, 1e-3, 0, bank, out_dtype="f64"), rtol=1e-12)
    assert not empty.P.any() and not empty.Vb.any() and empty.R_used == R
    np.testing.assert_allclose(Wn - W, bank.P[:, :R].astype(np.float64) @ bank.Vb[:, :R].astype(np.float64).T, atol=1e-12)
    # rounding happens once, to the storage type: within half a bf16 ulp of the exact sum
    Wb = zo.fold_bank(W, bank, "bf16")[0]
    exact = W + bank.P[:, :R].astype(np.float64) @ bank.Vb[:, :R].astype(np.float64).T
    assert np.all(np.abs(Wb - exact) <= np.abs(exact) * 2.0 ** -8)
    assert np.array_equal(zo.fold_bank(Wb, zo.Bank(bank.P, bank.Vb, 0), "bf16")[0], Wb)   # empty bank: no change


def test_loop_with_fold_at_wrap_equals_dense_weight_loop():
    """Past nu * B steps the loop folds and goes on; nothing is lost relative to dense updates."""
    batch, X, layers, head, tg, r = _problem(n_blocks=2)
    kw = dict(r=r, eps=1e-2, dtype="f32", reduction=0, steps=7, nu=1, lr=1e-2, base_u=5, base_v=6)
    outs, banks, Ws = zo_loop.run_loop(batch, X, layers, head, tg, n_blocks=2, fold_at_wrap=True, **kw)
    outs_d, Wd = zo_loop.run_loop_dense(batch, X, layers, head, tg, **kw)
    for t, (a, b) in enumerate(zip(outs, outs_d)):
        np.testing.assert_allclose(a["cand_loss"], b["cand_loss"], rtol=2e-6, err_msg="step %d" % t)
    for W, bank, D in zip(Ws, banks, Wd):
        np.testing.assert_allclose(W.astype(np.float64) + bank.P.astype(np.float64) @ bank.Vb.astype(np.float64).T, D,
                                   atol=5e-6)
