"""Pins for the oracle's path functions (CPU only): invariants, closed forms,
reductions to library routines and brute force on tiny inputs.  Each test
says which mistake it is there to catch."""
import math

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import philox as px
from oracle import zo_oracle as zo


def _batch(lens, seq_cand, cand_dir, cand_sign, K):
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    return zo.Batch(cu, np.array(seq_cand, np.int32), np.array(cand_dir, np.int32),
                    np.array(cand_sign, np.float32), np.arange(K, dtype=np.uint64) + np.uint64(1234567))


def _small(seed=0, m=24, n=40, r=4, R=6, lens=(5, 3, 7, 4, 6, 2), K=2):
    rng = np.random.default_rng(seed)
    # candidates: 0:+d0 1:-d0 2:+d1 3:-d1 4:centre
    b = _batch(lens, [0, 1, -1, 4, 2, 3], [0, 0, 1, 1, -1], [1, -1, 1, -1, 0], K)
    T = b.n_tokens
    X = rng.standard_normal((T, n))
    W = rng.standard_normal((m, n)) / math.sqrt(n)
    bank = zo.Bank(rng.standard_normal((m, R + 2)) * 0.1, rng.standard_normal((n, R + 2)) * 0.1, R)
    return b, X, W, bank, m, n, r


def test_indices_brute_force():
    b = _batch([3, 0, 2, 0, 0, 4, 1], [0, 1, -1, 0, 1, 1, -1], [0, 0], [1, -1], 1)
    tok_seq, tok_cand = zo.batch_indices(b)
    want_seq, want_cand = [], []
    for s in range(b.n_seqs):
        for _ in range(b.cu_seqlens[s], b.cu_seqlens[s + 1]):
            want_seq.append(s); want_cand.append(int(b.seq_cand[s]))
    assert tok_seq.tolist() == want_seq and tok_cand.tolist() == want_cand
    assert tok_seq.dtype == np.int32 and tok_cand.dtype == np.int32


def test_factorised_equals_dense():
    """Sec. 3.2: the LoRA-style realisation (A = V^T, B = +-eps U, bank factors)
    is the same map as the mutated dense weight.  Catches a transposed factor,
    a wrong sign, a dropped eps or a dropped bank term in candidate_weight."""
    b, X, W, bank, m, n, r = _small()
    eps, tid = 1e-3, 4
    Y = zo.probe_linear(b, X, W, r, eps, tid, bank)
    tok_seq, tok_cand = zo.batch_indices(b)
    R = bank.R_used
    for t in range(b.n_tokens):
        c = tok_cand[t]
        y = X[t] @ W.T
        if c >= 0:
            y = y + (X[t] @ bank.Vb[:, :R]) @ bank.P[:, :R].T
            k, s = int(b.cand_dir[c]), float(b.cand_sign[c])
            if k >= 0 and s != 0:
                U = px.factor_matrix(int(b.dir_seed[k]), tid, m, r)
                V = px.factor_matrix(int(b.dir_seed[k]), tid + 1, n, r)
                y = y + s * eps * (X[t] @ V) @ U.T
        np.testing.assert_allclose(Y[t], y, rtol=1e-12, atol=1e-13)


def test_foreground_rows_equal_plain_gemm_bitwise():
    b, X, W, bank, m, n, r = _small()
    Y = zo.probe_linear(b, X, W, r, 1e-3, 0, bank)
    fg = np.nonzero(zo.batch_indices(b)[1] < 0)[0]
    assert len(fg) > 0
    assert np.array_equal(Y[fg], X[fg] @ W.T)


def test_special_cases_reduce():
    b, X, W, bank, m, n, r = _small()
    tok_cand = zo.batch_indices(b)[1]
    cen = np.nonzero(tok_cand == 4)[0]
    Weff = W + bank.P[:, :bank.R_used] @ bank.Vb[:, :bank.R_used].T
    # centre candidate sees the bank only (Eq. bank)
    np.testing.assert_allclose(zo.probe_linear(b, X, W, r, 1e-3, 0, bank)[cen], X[cen] @ Weff.T, rtol=1e-12)
    # eps = 0: every candidate row equals the centre
    Y0 = zo.probe_linear(b, X, W, r, 0.0, 0, bank)
    np.testing.assert_allclose(Y0[tok_cand >= 0], X[tok_cand >= 0] @ Weff.T, rtol=1e-12)
    # no bank: R_used = 0 and bank None agree
    a = zo.probe_linear(b, X, W, r, 1e-3, 0, None)
    c = zo.probe_linear(b, X, W, r, 1e-3, 0, zo.Bank(bank.P, bank.Vb, 0))
    assert np.array_equal(a, c)
    # columns beyond R_used are ignored
    bank2 = zo.Bank(bank.P.copy(), bank.Vb.copy(), bank.R_used)
    bank2.P[:, bank.R_used:] = 7.0
    assert np.array_equal(zo.probe_linear(b, X, W, r, 1e-3, 0, bank), zo.probe_linear(b, X, W, r, 1e-3, 0, bank2))


def test_zero_base_isolates_side_term():
    """W = 0, no bank: Y_+ - Y_- = 2 eps (X V) U^T on duplicated rows."""
    m, n, r, eps, tid = 12, 20, 4, 1e-3, 2
    b = _batch([6, 6], [0, 1], [0, 0], [1, -1], 1)
    rng = np.random.default_rng(1)
    x = rng.standard_normal((6, n))
    X = np.concatenate([x, x])
    Y = zo.probe_linear(b, X, np.zeros((m, n)), r, eps, tid)
    U = px.factor_matrix(int(b.dir_seed[0]), tid, m, r)
    V = px.factor_matrix(int(b.dir_seed[0]), tid + 1, n, r)
    np.testing.assert_allclose(Y[:6] - Y[6:], 2 * eps * (x @ V) @ U.T, rtol=1e-12)
    np.testing.assert_allclose(Y[:6], -Y[6:], rtol=1e-12)


def test_bias_activation_and_rounding_points():
    b, X, W, bank, m, n, r = _small()
    bias = np.linspace(-1, 1, m)
    pre = zo.probe_linear(b, X, W, r, 1e-3, 0, bank)
    post = zo.probe_linear(b, X, W, r, 1e-3, 0, bank, bias=bias, act=1)
    np.testing.assert_allclose(post, np.maximum(pre + bias, 0), rtol=1e-13)
    y32 = zo.probe_linear(b, X, W, r, 1e-3, 0, bank, out_dtype="f32")
    assert np.array_equal(y32, pre.astype(np.float32).astype(np.float64))
    y16 = zo.probe_linear(b, X, W, r, 1e-3, 0, bank, out_dtype="bf16")
    assert np.array_equal(y16, px.round_to_bf16(pre.astype(np.float32)).astype(np.float64))
    rows = np.array([7, 0, 20])
    np.testing.assert_allclose(zo.probe_linear(b, X, W, r, 1e-3, 0, bank, rows=rows), pre[rows], rtol=1e-13)


def test_spsa_on_quadratic_is_exact_directional_derivative():
    """Eq. 2 on L(W) = ||X W^T - Y*||_F^2 / (2T): the antithetic difference is
    exact for every eps and equals <(X W^T - Y*)^T X / T, U V^T>.  Catches a
    wrong sign or a missing 1/(2 eps) in estimate and a mis-scaled probe."""
    m, n, r, tid, T = 10, 16, 3, 6, 9
    rng = np.random.default_rng(5)
    x = rng.standard_normal((T, n)); W = rng.standard_normal((m, n)); Ystar = rng.standard_normal((T, m))
    b = _batch([T, T], [0, 1], [0, 0], [1, -1], 1)
    X = np.concatenate([x, x])
    U = px.factor_matrix(int(b.dir_seed[0]), tid, m, r)
    V = px.factor_matrix(int(b.dir_seed[0]), tid + 1, n, r)
    G = (x @ W.T - Ystar).T @ x / T
    want = float(np.sum(G * (U @ V.T)))
    for eps in (1e-3, 0.25):
        Y = zo.probe_linear(b, X, W, r, eps, tid)
        losses = np.array([np.sum((Y[:T] - Ystar) ** 2) / 2, np.sum((Y[T:] - Ystar) ** 2) / 2])
        _, g = zo.estimate(b, losses, np.array([T, T]), eps, reduction=0)
        np.testing.assert_allclose(g[0], want, rtol=1e-9)


def _nll_chain(eps, with_centre=True):
    m, n, r, V_, T = 16, 12, 4, 50, 20
    rng = np.random.default_rng(11)
    x = rng.standard_normal((T, n)); W = rng.standard_normal((m, n)) / math.sqrt(n)
    head = rng.standard_normal((V_, m)); y = rng.integers(0, V_, T)
    b = _batch([T, T, T], [0, 1, 2], [0, 0, -1], [1, -1, 0], 1)
    X = np.concatenate([x, x, x]); tg = np.concatenate([y, y, y])
    H = zo.probe_linear(b, X, W, r, eps, 0)
    _, _, cs, cc = zo.score(b, H, head, tg)
    loss, g = zo.estimate(b, cs, cc, eps)
    return loss, g


def test_antithetic_average_is_second_order():
    """(L_+ + L_-)/2 - L_0 = O(eps^2): halving eps divides it by 4."""
    d = []
    for eps in (4e-2, 2e-2, 1e-2):
        loss, _ = _nll_chain(eps)
        d.append((loss[0] + loss[1]) / 2 - loss[2])
    assert abs(d[0] / d[1] - 4) < 0.4 and abs(d[1] / d[2] - 4) < 0.4
    # and the two-point coefficient converges (its error is O(eps^2) too)
    g = [_nll_chain(e)[1][0] for e in (2e-2, 1e-2, 5e-3)]
    assert abs((g[0] - g[1]) / (g[1] - g[2]) - 4) < 0.5


def test_score_against_library_routines():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    T, d, V_ = 30, 8, 37
    H = rng.standard_normal((T, d)) * 3; Wh = rng.standard_normal((V_, d)); y = rng.integers(0, V_, T)
    y[[3, 17]] = -1
    nll = zo.token_nll(H, Wh, y)
    z = H @ Wh.T
    want = logsumexp(z, axis=1) - z[np.arange(T), np.where(y >= 0, y, 0)]
    want[y < 0] = 0
    np.testing.assert_allclose(nll, want, rtol=1e-12)
    ce = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.from_numpy(y.astype(np.int64)),
                                           ignore_index=-1, reduction="none").numpy()
    np.testing.assert_allclose(nll, ce, rtol=1e-12)


def test_score_closed_forms():
    rng = np.random.default_rng(4)
    T, d, V_ = 10, 6, 512
    H = rng.standard_normal((T, d)); y = rng.integers(0, V_, T)
    # zero head: uniform distribution, nll = ln V exactly
    np.testing.assert_allclose(zo.token_nll(H, np.zeros((V_, d)), y), math.log(V_), rtol=1e-14)
    # adding one vector to every head row shifts all logits of a token equally
    Wh = rng.standard_normal((V_, d))
    np.testing.assert_allclose(zo.token_nll(H, Wh + rng.standard_normal(d), y), zo.token_nll(H, Wh, y), rtol=1e-10)
    # a dominant target logit drives the nll to 0; large logits do not overflow
    Wd = np.zeros((V_, d)); Hd = np.zeros((T, d)); Hd[:, 0] = 1000.0
    Wd[7, 0] = 1.0
    assert np.all(zo.token_nll(Hd, Wd, np.full(T, 7)) < 1e-300)
    np.testing.assert_allclose(zo.token_nll(Hd, Wd, np.full(T, 8)), 1000.0, rtol=1e-12)


def test_score_reductions_brute_force():
    b, X, W, bank, m, n, r = _small()
    rng = np.random.default_rng(9)
    V_ = 33
    H = rng.standard_normal((b.n_tokens, m)); Wh = rng.standard_normal((V_, m))
    y = rng.integers(0, V_, b.n_tokens); y[::5] = -1
    tok, seq, cs, cc = zo.score(b, H, Wh, y)
    tok_seq, tok_cand = zo.batch_indices(b)
    want_seq = np.zeros(b.n_seqs); want_cs = np.zeros(b.n_cands); want_cc = np.zeros(b.n_cands, int)
    for t in range(b.n_tokens):
        if y[t] < 0:
            assert tok[t] == 0
            continue
        z = Wh @ H[t]
        nll = math.log(sum(math.exp(v - z.max()) for v in z)) + z.max() - z[y[t]]
        assert abs(tok[t] - nll) < 1e-11
        want_seq[tok_seq[t]] += nll
        if tok_cand[t] >= 0:
            want_cs[tok_cand[t]] += nll; want_cc[tok_cand[t]] += 1
    np.testing.assert_allclose(seq, want_seq, rtol=1e-12)
    np.testing.assert_allclose(cs, want_cs, rtol=1e-12)
    assert cc.tolist() == want_cc.tolist()
    assert seq[2] != 0 and cs.shape == (5,)       # the foreground sequence has a score, belongs to no candidate


def test_estimate_reductions_and_missing_pairs():
    b = _batch([1] * 4, [0, 1, 2, 3], [0, 0, 1, -1], [1, -1, 1, 0], 3)
    cs = np.array([10.0, 4.0, 9.0, 5.0]); cc = np.array([5, 2, 3, 0])
    loss, g = zo.estimate(b, cs, cc, 0.5, reduction=0)
    np.testing.assert_allclose(loss, [2.0, 2.0, 3.0, 5.0])
    np.testing.assert_allclose(g, [0.0, 0.0, 0.0])
    loss, g = zo.estimate(b, cs, cc, 0.5, reduction=1)
    np.testing.assert_allclose(loss, cs)
    np.testing.assert_allclose(g, [6.0, 0.0, 0.0])    # direction 1 lacks its '-' candidate, direction 2 has none


def test_lazy_accumulator_is_linear_and_matches_combined_probe():
    """Eq. layer-coupling / combined-probe: three accumulate steps with fresh U_t
    and one persistent V_k equal the dense sum of beta_t U_t V_k^T, and a probe
    whose direction reuses V_k sees W_0 + (P_k +- eps U_t) V_k^T."""
    m, n, r, tid = 14, 18, 4, 8
    rng = np.random.default_rng(21)
    W = rng.standard_normal((m, n)); x = rng.standard_normal((5, n))
    bank = zo.Bank(np.zeros((m, 8), np.float32), np.zeros((n, 8), np.float32), 0)
    seeds = [77, 78, 79]
    grads = [0.7, -1.3, 0.4]
    lr = 0.01
    # open the block with step 0 (its V becomes V_k), then accumulate two more U_t
    dense = np.zeros((m, n))
    Vk = px.factor_matrix(seeds[0], tid + 1, n, r)
    for t, (sd, g) in enumerate(zip(seeds, grads)):
        bt = _batch([5], [0], [0], [1], 1); bt.dir_seed = np.array([sd], np.uint64)
        bank = zo.bank_update(bank, bt, m, n, r, tid, [g], lr, col0=[4], dir_weight=[1.0], append=(t == 0))
        dense += (-np.float32(lr).astype(np.float64) * np.float32(g).astype(np.float64)) * px.factor_matrix(sd, tid, m, r) @ Vk.T
    assert bank.R_used == 8
    np.testing.assert_allclose(bank.Vb[:, 4:8], Vk.astype(np.float32), rtol=0)
    assert not bank.P[:, :4].any() and not bank.Vb[:, :4].any()
    # centre forward through the bank == forward through the dense accumulated update
    bc = _batch([5], [0], [-1], [0], 1)
    np.testing.assert_allclose(zo.probe_linear(bc, x, W, r, 1e-3, tid, bank), x @ (W + dense).T, rtol=1e-5, atol=1e-6)
    # probing with the seed that opened the block reproduces W_0 + (P_k + eps U) V_k^T
    bp = _batch([5], [0], [0], [1], 1); bp.dir_seed = np.array([seeds[0]], np.uint64)
    U0 = px.factor_matrix(seeds[0], tid, m, r)
    want = x @ (W + (bank.P[:, 4:8].astype(np.float64) + 1e-3 * U0) @ Vk.T).T
    np.testing.assert_allclose(zo.probe_linear(bp, x, W, r, 1e-3, tid, bank), want, rtol=1e-6, atol=1e-7)


def test_bank_update_defaults_and_overflow():
    m, n, r = 6, 5, 2
    b = _batch([1, 1], [0, 1], [0, 1], [1, 1], 2)
    bank = zo.Bank(np.ones((m, 4), np.float32), np.ones((n, 4), np.float32), 4)
    out = zo.bank_update(bank, b, m, n, r, 0, [2.0, -4.0], 0.5, col0=[0, 2])
    for k, g in enumerate([2.0, -4.0]):
        U = px.factor_matrix(int(b.dir_seed[k]), 0, m, r)
        np.testing.assert_allclose(out.P[:, 2 * k:2 * k + 2], 1 + (-0.5 * g / 2) * U, rtol=1e-6)
    assert np.array_equal(out.Vb, bank.Vb) and bank.P.min() == 1.0   # input untouched, Vb untouched when accumulating
    with pytest.raises(ValueError):
        zo.bank_update(bank, b, m, n, r, 0, [1.0, 1.0], 0.5, col0=[0, 3])


def test_planted_mistakes_are_caught(monkeypatch):
    """The pins bite: a sign error in the estimator, a dropped bank term and a
    swapped U/V stream each break a pinned property."""
    b, X, W, bank, m, n, r = _small()
    ref = zo.probe_linear(b, X, W, r, 1e-3, 0, bank)
    # swapped streams
    u_id, v_id = px.u_tensor_id, px.v_tensor_id
    monkeypatch.setattr(px, "u_tensor_id", v_id)
    monkeypatch.setattr(px, "v_tensor_id", u_id)
    assert not np.allclose(zo.probe_linear(b, X, W, r, 1e-3, 0, bank), ref, rtol=1e-9, atol=1e-9)
    monkeypatch.setattr(px, "u_tensor_id", u_id)
    monkeypatch.setattr(px, "v_tensor_id", v_id)
    assert np.array_equal(zo.probe_linear(b, X, W, r, 1e-3, 0, bank), ref)
    # dropped bank
    assert not np.allclose(zo.probe_linear(b, X, W, r, 1e-3, 0, None), ref, rtol=1e-6)
    # estimator sign
    bb = _batch([1, 1], [0, 1], [0, 0], [-1, 1], 1)
    _, g = zo.estimate(bb, np.array([1.0, 3.0]), np.array([1, 1]), 0.5)
    assert g[0] == 2.0


def test_es_estimate_is_a_normalised_reward_weighting():
    """Pins for the reward-normalised one-sided estimate: z has mean 0 and unit
    population variance, is unchanged by shifting or scaling the losses, skips
    directions without a positive candidate, and on a linear objective the
    weighted perturbation sum is a descent direction.  Catches a sign error
    (reward = +loss), a sample-std normalisation and a wrong eps scaling."""
    rng = np.random.default_rng(11)
    m, n, r, K, eps = 10, 14, 3, 6, 1e-2
    cand_dir = np.array(list(range(K - 1)) + [-1], np.int32)           # direction K-1 has no candidate; last = centre
    cand_sign = np.array([1.0] * (K - 1) + [0.0], np.float32)
    b = zo.Batch(np.array([0, 1], np.int32), np.array([0], np.int32), cand_dir, cand_sign,
                 np.arange(K, dtype=np.uint64) + np.uint64(77))
    G = rng.standard_normal((m, n))
    dirs = [zo.direction_factors(b, k, m, n, r, 0, "f32") for k in range(K)]
    # linear objective: L(W0 + eps U V^T) = L0 + eps <G, U V^T>
    L = np.array([3.0 + eps * np.sum(G * (U @ V.T)) for U, V in dirs[:K - 1]] + [3.0])
    cnt = np.ones(K, np.int64)
    loss, c = zo.estimate_es(b, L, cnt, eps, reduction=1)
    assert np.array_equal(loss, L) and c[K - 1] == 0.0
    z = -c[:K - 1] * eps
    assert abs(z.mean()) < 1e-12 and abs((z ** 2).mean() - 1.0) < 1e-12
    c2 = zo.estimate_es(b, 5.0 * L - 2.0, cnt, eps, reduction=1)[1]
    np.testing.assert_allclose(c2, c, rtol=1e-9)
    # beta_k = -lr c_k / K; the summed update must decrease the linear objective
    upd = sum((-1.0 * c[k] / K) * (dirs[k][0] @ dirs[k][1].T) for k in range(K - 1))
    assert np.sum(G * upd) < 0
    # mean reduction divides by the scored-token counts first
    cnt2 = np.array([2, 4, 1, 5, 3, 1])
    np.testing.assert_allclose(zo.estimate_es(b, L * cnt2, cnt2, eps, reduction=0)[1], c, rtol=1e-9)
    # equal rewards: nothing to prefer
    assert not zo.estimate_es(b, np.full(K, 2.0), cnt, eps, reduction=1)[1].any()
