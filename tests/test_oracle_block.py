"""Pins of the decoder-block oracle (CPU only).

Each test fixes oracle/zo_block.py against something other than itself: a
library routine on the special case both cover, a closed form, or an invariant
that a plausible mistake (wrong mask direction, a leak across packed
sequences, the wrong key/value head, a dropped scale, unbiased variance)
breaks.
"""
import types

import numpy as np
import pytest
import torch

from oracle import zo_block as zb
from oracle import zo_oracle as zo


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- normalisation

def test_layer_norm_matches_library_routine():
    g = _rng(0)
    x = g.normal(size=(7, 48)) * 3 + 1.5
    gamma = g.normal(size=48); beta = g.normal(size=48)
    want = torch.nn.functional.layer_norm(torch.tensor(x), (48,), torch.tensor(gamma), torch.tensor(beta), 1e-5)
    np.testing.assert_allclose(zb.layer_norm(x, gamma, beta, 1e-5), want.numpy(), rtol=1e-12, atol=1e-12)


def test_rms_norm_matches_library_routine():
    g = _rng(1)
    x = g.normal(size=(5, 64)) * 2
    gamma = g.normal(size=64)
    want = torch.nn.functional.rms_norm(torch.tensor(x), (64,), torch.tensor(gamma), 1e-6)
    np.testing.assert_allclose(zb.rms_norm(x, gamma, 1e-6), want.numpy(), rtol=1e-12, atol=1e-12)


def test_layer_norm_moments_and_shift_invariance():
    g = _rng(2)
    x = g.normal(size=(4, 256)) * 5
    y = zb.layer_norm(x, np.ones(256), None, 0.0)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-12)
    np.testing.assert_allclose((y ** 2).mean(axis=1), 1, rtol=1e-12)        # biased variance, not n-1
    np.testing.assert_allclose(zb.layer_norm(x + 17.0, np.ones(256), None, 0.0), y, atol=1e-10)


def test_rms_norm_scale_invariance_and_unit_rms():
    g = _rng(3)
    x = g.normal(size=(4, 128))
    y = zb.rms_norm(x, np.ones(128), 0.0)
    np.testing.assert_allclose((y ** 2).mean(axis=1), 1, rtol=1e-12)
    np.testing.assert_allclose(zb.rms_norm(-3.5 * x, np.ones(128), 0.0), -y, rtol=1e-12)
    # RMS norm does not remove the mean
    assert abs(zb.rms_norm(x + 4.0, np.ones(128), 0.0).mean()) > 0.5


def test_add_norm_sums_before_normalising():
    g = _rng(4)
    x = g.normal(size=(3, 32)); res = g.normal(size=(3, 32))
    gamma = g.normal(size=32); beta = g.normal(size=32)
    h, y = zb.add_norm(x, res, gamma, beta, zb.LAYER_NORM, 1e-5)
    np.testing.assert_allclose(h, x + res, rtol=0, atol=0)
    np.testing.assert_allclose(y, zb.layer_norm(x + res, gamma, beta, 1e-5), rtol=1e-14)
    h, y = zb.add_norm(x, None, gamma, None, zb.RMS_NORM, 1e-6)
    np.testing.assert_allclose(h, x, rtol=0, atol=0)
    np.testing.assert_allclose(y, zb.rms_norm(x, gamma, 1e-6), rtol=1e-14)


# ---------------------------------------------------------------- attention

def _qkv(seed, T, H, Hkv, dh):
    g = _rng(seed)
    return g.normal(size=(T, H * dh)), g.normal(size=(T, Hkv * dh)), g.normal(size=(T, Hkv * dh))


def test_attention_single_sequence_matches_library_routine():
    T, H, dh = 37, 3, 16
    q, k, v = _qkv(10, T, H, H, dh)
    got = zb.attention(q, k, v, [0, T], H, H, dh, dh ** -0.5)
    tq, tk, tv = (torch.tensor(a).reshape(T, H, dh).permute(1, 0, 2)[None] for a in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2)
    np.testing.assert_allclose(got, want.reshape(T, H * dh).numpy(), rtol=1e-10, atol=1e-12)


def test_attention_scale_is_applied():
    T, H, dh = 9, 2, 8
    q, k, v = _qkv(11, T, H, H, dh)
    got = zb.attention(q, k, v, [0, T], H, H, dh, 0.37)
    tq, tk, tv = (torch.tensor(a).reshape(T, H, dh).permute(1, 0, 2)[None] for a in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=0.37)[0]
    np.testing.assert_allclose(got, want.permute(1, 0, 2).reshape(T, H * dh).numpy(), rtol=1e-10, atol=1e-12)
    assert np.abs(got - zb.attention(q, k, v, [0, T], H, H, dh, 1.0)).max() > 1e-3


def test_attention_equal_keys_give_the_causal_prefix_mean():
    # all scores of a row are equal => uniform weights over rows 0..t of the sequence
    T, H, dh = 12, 2, 4
    g = _rng(12)
    q = g.normal(size=(T, H * dh))
    k = np.tile(g.normal(size=(1, H * dh)), (T, 1))
    v = g.normal(size=(T, H * dh))
    cu = [0, 5, 5, 12]
    got = zb.attention(q, k, v, cu, H, H, dh, 1.0)
    want = np.zeros_like(v)
    for a, b in ((0, 5), (5, 12)):
        want[a:b] = np.cumsum(v[a:b], axis=0) / np.arange(1, b - a + 1)[:, None]
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_attention_first_row_of_every_sequence_returns_its_own_value():
    T, H, dh = 20, 2, 8
    q, k, v = _qkv(13, T, H, H, dh)
    cu = np.array([0, 1, 4, 4, 11, 20])
    got = zb.attention(q, k, v, cu, H, H, dh, 0.5)
    for a in (0, 1, 4, 11):
        np.testing.assert_allclose(got[a], v[a], rtol=1e-13)


def test_attention_sharp_scores_select_past_keys_only():
    # orthogonal keys, query t aimed at key target[t] with a large gain: the output is that key's
    # value when it lies in the past (or present) and must not be when it lies in the future
    T, dh = 8, 8
    k = np.eye(T, dh)
    v = _rng(14).normal(size=(T, dh))
    target = np.array([0, 0, 2, 1, 7, 5, 3, 7])        # row 4 aims at a future key
    q = 200.0 * np.eye(T, dh)[target]
    got = zb.attention(q, k, v, [0, T], 1, 1, dh, 1.0)
    for t in range(T):
        if target[t] <= t:
            np.testing.assert_allclose(got[t], v[target[t]], atol=1e-12)
        else:
            assert np.abs(got[t] - v[target[t]]).max() > 0.1
            np.testing.assert_allclose(got[t], v[:t + 1].mean(axis=0), atol=1e-12)   # all visible scores are 0


def test_attention_packed_sequences_do_not_interact():
    H, dh = 2, 8
    lens = [3, 9, 1, 6]
    cu = np.concatenate([[0], np.cumsum(lens)])
    q, k, v = _qkv(15, int(cu[-1]), H, H, dh)
    packed = zb.attention(q, k, v, cu, H, H, dh, 0.3)
    for i in range(len(lens)):
        a, b = cu[i], cu[i + 1]
        alone = zb.attention(q[a:b], k[a:b], v[a:b], [0, b - a], H, H, dh, 0.3)
        np.testing.assert_allclose(packed[a:b], alone, rtol=1e-13, atol=1e-14)
    # changing another sequence's keys and values leaves a sequence's rows untouched
    k2, v2 = k.copy(), v.copy()
    k2[cu[1]:cu[2]] += 5; v2[cu[1]:cu[2]] -= 3
    again = zb.attention(q, k2, v2, cu, H, H, dh, 0.3)
    np.testing.assert_array_equal(again[:cu[1]], packed[:cu[1]])
    np.testing.assert_array_equal(again[cu[2]:], packed[cu[2]:])


def test_attention_grouped_heads_read_the_right_key_value_head():
    T, H, Hkv, dh = 6, 6, 2, 4
    q, k, _ = _qkv(16, T, H, Hkv, dh)
    # value head j is the constant j + 1: head h must output (h // 3) + 1 everywhere
    v = np.concatenate([np.full((T, dh), j + 1.0) for j in range(Hkv)], axis=1)
    got = zb.attention(q, k, v, [0, T], H, Hkv, dh, 1.0)
    for h in range(H):
        np.testing.assert_allclose(got[:, h * dh:(h + 1) * dh], h // 3 + 1.0, rtol=1e-13)
    # grouped == the same keys/values repeated per query head
    q, k, v = _qkv(17, T, H, Hkv, dh)
    rep = lambda a: np.concatenate([a[:, (h // 3) * dh:(h // 3 + 1) * dh] for h in range(H)], axis=1)
    np.testing.assert_allclose(zb.attention(q, k, v, [0, T], H, Hkv, dh, 0.5),
                               zb.attention(q, rep(k), rep(v), [0, T], H, H, dh, 0.5), rtol=1e-13)


def test_attention_output_is_a_convex_combination_of_visible_values():
    T, H, dh = 16, 1, 4
    q, k, v = _qkv(18, T, H, H, dh)
    got = zb.attention(q * 4, k, v, [0, T], H, H, dh, 1.0)
    for t in range(T):
        assert (got[t] <= v[:t + 1].max(axis=0) + 1e-12).all()
        assert (got[t] >= v[:t + 1].min(axis=0) - 1e-12).all()


# ---------------------------------------------------------------- whole block

def _layer(g, m, n, tid, act=0, bias=True, R=0):
    l = types.SimpleNamespace(W=g.normal(size=(m, n)) / np.sqrt(n), tensor_id=tid, act=act,
                              bias=g.normal(size=m) * 0.1 if bias else None, P=None, Vb=None, R_used=0)
    if R:
        l.P = (g.normal(size=(m, R)) * 0.05).astype(np.float32)
        l.Vb = (g.normal(size=(n, R)) * 0.05).astype(np.float32)
        l.R_used = R
    return l


def _block(seed, d, H, Hkv, dh, ffn, kind, R=0):
    g = _rng(seed)
    return types.SimpleNamespace(
        norm_kind=kind, norm_eps=1e-5, g1=1 + 0.1 * g.normal(size=d), g2=1 + 0.1 * g.normal(size=d),
        b1=0.1 * g.normal(size=d) if kind == zb.LAYER_NORM else None,
        b2=0.1 * g.normal(size=d) if kind == zb.LAYER_NORM else None,
        n_heads=H, n_kv_heads=Hkv, head_dim=dh, scale=dh ** -0.5,
        qkv=_layer(g, (H + 2 * Hkv) * dh, d, 10, R=R), o=_layer(g, d, H * dh, 12, R=R),
        fc1=_layer(g, ffn, d, 14, act=1, R=R), fc2=_layer(g, d, ffn, 16, R=R))


def _batch(lens, seq_cand, cand_dir, cand_sign, seeds):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return zo.Batch(cu, np.asarray(seq_cand, np.int32), np.asarray(cand_dir, np.int32),
                    np.asarray(cand_sign, np.float32), np.asarray(seeds, np.uint64))


@pytest.mark.parametrize("kind", [zb.LAYER_NORM, zb.RMS_NORM])
def test_block_foreground_equals_a_plain_torch_block(kind):
    # every sequence foreground => no candidate state: the block is an ordinary pre-norm decoder block,
    # rebuilt here from torch's own layer_norm / rms_norm / linear / scaled_dot_product_attention
    d, H, Hkv, dh, ffn = 32, 4, 2, 8, 64
    blk = _block(20 + kind, d, H, Hkv, dh, ffn, kind)
    lens = [5, 11]
    batch = _batch(lens, [-1, -1], [0, 0], [1, -1], [7])
    x = _rng(22).normal(size=(sum(lens), d))
    got = zb.block_forward(batch, x, blk, 4, 1e-3, "f32", "f64")["h2"]

    F = torch.nn.functional
    t = lambda a: None if a is None else torch.tensor(np.asarray(a, np.float64))
    norm = (lambda z, g, b: F.layer_norm(z, (d,), t(g), t(b), 1e-5)) if kind == zb.LAYER_NORM else \
           (lambda z, g, b: F.rms_norm(z, (d,), t(g), 1e-5))
    want = []
    for a, b in ((0, 5), (5, 16)):
        h0 = t(x[a:b])
        qkv = F.linear(norm(h0, blk.g1, blk.b1), t(blk.qkv.W), t(blk.qkv.bias))
        L = b - a
        q = qkv[:, :H * dh].reshape(L, H, dh).permute(1, 0, 2)[None]
        k = qkv[:, H * dh:(H + Hkv) * dh].reshape(L, Hkv, dh).permute(1, 0, 2)[None]
        v = qkv[:, (H + Hkv) * dh:].reshape(L, Hkv, dh).permute(1, 0, 2)[None]
        att = F.scaled_dot_product_attention(q, k, v, is_causal=True, enable_gqa=True)[0]
        att = att.permute(1, 0, 2).reshape(L, H * dh)
        h1 = h0 + F.linear(att, t(blk.o.W), t(blk.o.bias))
        f = F.relu(F.linear(norm(h1, blk.g2, blk.b2), t(blk.fc1.W), t(blk.fc1.bias)))
        want.append((h1 + F.linear(f, t(blk.fc2.W), t(blk.fc2.bias))).numpy())
    np.testing.assert_allclose(got, np.concatenate(want), rtol=1e-9, atol=1e-11)


def test_block_candidates_equal_the_block_with_mutated_weights():
    # a candidate's rows must equal an ordinary block whose four weights were overwritten by
    # W + P Vb^T + s eps U V^T (dense mutation), evaluated as an all-foreground batch
    d, H, Hkv, dh, ffn, r, eps = 32, 2, 1, 16, 48, 4, 1e-2
    blk = _block(30, d, H, Hkv, dh, ffn, zb.RMS_NORM, R=8)
    lens = [6, 6, 9]
    batch = _batch(lens, [0, 1, 2], [0, 0, -1], [1, -1, 0], [99])
    x = _rng(31).normal(size=(sum(lens), d))
    got = zb.block_forward(batch, x, blk, r, eps, "f32", "f64")["h2"]
    cu = batch.cu_seqlens
    for s, cand in enumerate([0, 1, 2]):
        mutated = types.SimpleNamespace(**vars(blk))
        for name in ("qkv", "o", "fc1", "fc2"):
            l = getattr(blk, name)
            Wc = zo.candidate_weight(l.W, batch, cand, r, eps, l.tensor_id, zo.Bank(l.P, l.Vb, l.R_used), "f32")
            setattr(mutated, name, types.SimpleNamespace(W=Wc, tensor_id=l.tensor_id, act=l.act, bias=l.bias,
                                                         P=None, Vb=None, R_used=0))
        a, b = int(cu[s]), int(cu[s + 1])
        fg = _batch([b - a], [-1], [0], [1], [99])
        want = zb.block_forward(fg, x[a:b], mutated, r, eps, "f32", "f64")["h2"]
        np.testing.assert_allclose(got[a:b], want, rtol=1e-10, atol=1e-12)
    # and the probe does move the output
    plus, minus = got[0:6], got[6:12]
    base = zb.block_forward(_batch([6], [0], [-1], [0], [99]), x[0:6], blk, r, eps, "f32", "f64")["h2"]
    assert np.abs(plus - base).max() > 1e-5
    # both candidate sequences see different inputs, so compare each with its own centre instead
    base2 = zb.block_forward(_batch([6], [0], [-1], [0], [99]), x[6:12], blk, r, eps, "f32", "f64")["h2"]
    assert np.abs(minus - base2).max() > 1e-5


# ---------------------------------------------------------------- whole model

def _model(seed, n_blocks, d, H, Hkv, dh, ffn, vocab, kind, R=0):
    g = _rng(seed)
    blocks = []
    for b in range(n_blocks):
        blk = _block(seed * 10 + b, d, H, Hkv, dh, ffn, kind, R=R)
        for i, name in enumerate(("qkv", "o", "fc1", "fc2")):
            getattr(blk, name).tensor_id = 2 * (4 * b + i)
        blocks.append(blk)
    final = (1 + 0.1 * g.normal(size=d), 0.1 * g.normal(size=d) if kind == zb.LAYER_NORM else None)
    head = g.normal(size=(vocab, d)) / np.sqrt(d)
    return blocks, final, head


def test_model_candidates_equal_the_model_with_mutated_weights():
    """Per-candidate losses of the factorised model = losses of an ordinary model whose eight probed
    weights were densely overwritten (Sec. 2.3: the two evaluations are algebraically the same)."""
    d, H, Hkv, dh, ffn, vocab, r, eps = 24, 2, 1, 12, 40, 50, 3, 1e-2
    blocks, final, head = _model(41, 2, d, H, Hkv, dh, ffn, vocab, zb.LAYER_NORM, R=4)
    lens = [7, 7, 5]
    batch = _batch(lens, [0, 1, 2], [0, 0, -1], [1, -1, 0], [1234])
    g = _rng(42)
    x = g.normal(size=(sum(lens), d)); x[7:14] = x[0:7]          # the +/- pair sees the same rows
    targets = g.integers(0, vocab, size=sum(lens)); targets[7:14] = targets[0:7]
    got = zb.model_forward(batch, x, blocks, final, head, targets, r, eps, "f32", 0, "f64")
    cu = batch.cu_seqlens
    for s, cand in enumerate([0, 1, 2]):
        mutated = []
        for blk in blocks:
            m = types.SimpleNamespace(**vars(blk))
            for name in ("qkv", "o", "fc1", "fc2"):
                l = getattr(blk, name)
                Wc = zo.candidate_weight(l.W, batch, cand, r, eps, l.tensor_id, zo.Bank(l.P, l.Vb, l.R_used), "f32")
                setattr(m, name, types.SimpleNamespace(W=Wc, tensor_id=l.tensor_id, act=l.act, bias=l.bias,
                                                       P=None, Vb=None, R_used=0))
            mutated.append(m)
        a, b = int(cu[s]), int(cu[s + 1])
        plain = _batch([b - a], [0], [-1], [0], [1234])      # one centre candidate without a bank
        want = zb.model_forward(plain, x[a:b], mutated, final, head, targets[a:b], r, eps, "f32", 0, "f64")
        np.testing.assert_allclose(got["cand_loss"][cand], want["cand_loss"][0], rtol=1e-10)
    # the estimate is the two-point difference of those losses
    np.testing.assert_allclose(got["proj_grad"][0], (got["cand_loss"][0] - got["cand_loss"][1]) / (2 * eps), rtol=1e-12)
    assert abs(got["proj_grad"][0]) > 1e-6


def test_model_antithetic_losses_average_to_the_centre_loss_to_second_order():
    d, H, Hkv, dh, ffn, vocab, r = 16, 2, 2, 8, 24, 30, 2
    blocks, final, head = _model(43, 2, d, H, Hkv, dh, ffn, vocab, zb.RMS_NORM)
    for blk in blocks:
        blk.fc1.act = 0      # no ReLU kinks: softmax, norms and the NLL keep the model smooth and nonlinear
    lens = [6, 6, 6]
    g = _rng(44)
    x = np.tile(g.normal(size=(6, d)), (3, 1))
    targets = np.tile(g.integers(0, vocab, size=6), 3)
    gaps = []
    for eps in (8e-3, 4e-3, 2e-3):
        batch = _batch(lens, [0, 1, 2], [0, 0, -1], [1, -1, 0], [77])
        out = zb.model_forward(batch, x, blocks, final, head, targets, r, eps, "f32", 0, "f64")
        gaps.append(0.5 * (out["cand_loss"][0] + out["cand_loss"][1]) - out["cand_loss"][2])
    assert abs(gaps[0]) > 1e-9
    np.testing.assert_allclose(gaps[0] / gaps[1], 4.0, rtol=0.15)
    np.testing.assert_allclose(gaps[1] / gaps[2], 4.0, rtol=0.15)


# ---------------------------------------------------------------- Qwen3-family pieces

def test_rope_is_a_complex_rotation_of_each_pair():
    """The pair (x[i], x[i + dh/2]) as a complex number is multiplied by exp(1j * p * theta^(-2i/dh))."""
    dh, H, T = 16, 2, 11
    g = _rng(60)
    q = g.normal(size=(T, H * dh)); k = g.normal(size=(T, dh))
    cu = [0, 4, 4, 11]
    theta = 10000.0
    gq, gk = zb.qk_norm_rope(q, k, cu, H, 1, dh, None, None, 0.0, theta)
    pos = np.array([0, 1, 2, 3, 0, 1, 2, 3, 4, 5, 6])
    freq = theta ** (-2.0 * np.arange(dh // 2) / dh)
    rot = np.exp(1j * pos[:, None] * freq[None, :])
    for x, got, heads in ((q, gq, H), (k, gk, 1)):
        for h in range(heads):
            z = (x[:, h * dh:h * dh + dh // 2] + 1j * x[:, h * dh + dh // 2:(h + 1) * dh]) * rot
            np.testing.assert_allclose(got[:, h * dh:h * dh + dh // 2], z.real, rtol=1e-12, atol=1e-13)
            np.testing.assert_allclose(got[:, h * dh + dh // 2:(h + 1) * dh], z.imag, rtol=1e-12, atol=1e-13)


def test_rope_identity_at_position_zero_norm_preservation_and_relative_positions():
    dh, T = 8, 9
    g = _rng(61)
    q = g.normal(size=(T, dh)); k = g.normal(size=(T, dh))
    gq, gk = zb.qk_norm_rope(q, k, [0, 3, 9], 1, 1, dh, None, None, 0.0, 500.0)
    np.testing.assert_array_equal(gq[[0, 3]], q[[0, 3]])                      # first row of each sequence
    np.testing.assert_allclose((gq ** 2).sum(1), (q ** 2).sum(1), rtol=1e-12)
    # <rope(a, p1), rope(b, p2)> depends on p1 - p2 only: the same two vectors at positions (1, 4) and (2, 5)
    a, b = g.normal(size=dh), g.normal(size=dh)
    rows = np.tile(a, (6, 1)); keys = np.tile(b, (6, 1))
    rq, rk = zb.qk_norm_rope(rows, keys, [0, 6], 1, 1, dh, None, None, 0.0, 500.0)
    np.testing.assert_allclose(rq[4] @ rk[1], rq[5] @ rk[2], rtol=1e-12)
    assert abs(rq[4] @ rk[1] - rq[4] @ rk[2]) > 1e-6


def test_qk_norm_matches_library_rms_norm_per_head():
    dh, H, Hkv, T = 16, 3, 1, 5
    g = _rng(62)
    q = g.normal(size=(T, H * dh)) * 3; k = g.normal(size=(T, Hkv * dh)) * 0.2
    gam_q, gam_k = 1 + 0.1 * g.normal(size=dh), 1 + 0.1 * g.normal(size=dh)
    gq, gk = zb.qk_norm_rope(q, k, [0, T], H, Hkv, dh, gam_q, gam_k, 1e-6, None)
    want_q = torch.nn.functional.rms_norm(torch.tensor(q).reshape(T, H, dh), (dh,), torch.tensor(gam_q), 1e-6)
    want_k = torch.nn.functional.rms_norm(torch.tensor(k).reshape(T, Hkv, dh), (dh,), torch.tensor(gam_k), 1e-6)
    np.testing.assert_allclose(gq, want_q.reshape(T, H * dh).numpy(), rtol=1e-12)
    np.testing.assert_allclose(gk, want_k.reshape(T, Hkv * dh).numpy(), rtol=1e-12)
    # the norm comes before the rotation: norm, then rotate == the function with both switched on
    both_q, both_k = zb.qk_norm_rope(q, k, [0, T], H, Hkv, dh, gam_q, gam_k, 1e-6, 1e4)
    rq, rk = zb.qk_norm_rope(gq, gk, [0, T], H, Hkv, dh, None, None, 0.0, 1e4)
    np.testing.assert_allclose(both_q, rq, rtol=1e-13)
    np.testing.assert_allclose(both_k, rk, rtol=1e-13)


def test_gated_activation_of_the_probe_linear_matches_library_silu():
    """act = 2: adjacent output features are (gate, up) pairs; the layer returns silu(gate) * up."""
    g = _rng(63)
    m, n, T = 24, 10, 7
    W = g.normal(size=(m, n)); bias = g.normal(size=m)
    batch = _batch([T], [-1], [0], [1], [5])
    X = g.normal(size=(T, n))
    pre = zo.probe_linear(batch, X, W, 2, 1e-3, 0, None, bias=bias, act=0)
    got = zo.probe_linear(batch, X, W, 2, 1e-3, 0, None, bias=bias, act=2)
    want = torch.nn.functional.silu(torch.tensor(pre[:, 0::2])) * torch.tensor(pre[:, 1::2])
    assert got.shape == (T, m // 2)
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-14)


def test_gated_rotary_block_foreground_equals_a_plain_torch_block():
    """The Qwen3 form of the block (RMS norms, per-head q/k norms, rotary embedding, grouped heads, gated
    MLP), all sequences foreground, against the same block rebuilt from torch functions."""
    d, H, Hkv, dh, F_, theta = 32, 4, 2, 8, 40, 1e4
    blk = _block(64, d, H, Hkv, dh, F_, zb.RMS_NORM)
    g = _rng(65)
    blk.fc1 = _layer(g, 2 * F_, d, 14, act=2, bias=False)     # rows 2j, 2j+1 = gate_j, up_j
    blk.fc2 = _layer(g, d, F_, 16, bias=False)
    blk.qkv.bias = blk.o.bias = None
    blk.gq, blk.gk, blk.rope_theta = 1 + 0.1 * g.normal(size=dh), 1 + 0.1 * g.normal(size=dh), theta
    lens = [6, 9]
    batch = _batch(lens, [-1, -1], [0, 0], [1, -1], [7])
    x = g.normal(size=(sum(lens), d))
    got = zb.block_forward(batch, x, blk, 4, 1e-3, "f32", "f64")["h2"]
    F = torch.nn.functional
    t = lambda a: torch.tensor(np.asarray(a, np.float64))

    def rope(z):                       # z [L, heads, dh]
        L = z.shape[0]
        freq = theta ** (-2.0 * torch.arange(dh // 2, dtype=torch.float64) / dh)
        ang = torch.arange(L, dtype=torch.float64)[:, None] * freq[None, :]
        cos, sin = torch.cos(ang)[:, None, :], torch.sin(ang)[:, None, :]
        a, b = z[..., :dh // 2], z[..., dh // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)
    want = []
    for lo, hi in ((0, 6), (6, 15)):
        h0 = t(x[lo:hi]); L = hi - lo
        qkv = F.linear(F.rms_norm(h0, (d,), t(blk.g1), blk.norm_eps), t(blk.qkv.W))
        q = rope(F.rms_norm(qkv[:, :H * dh].reshape(L, H, dh), (dh,), t(blk.gq), blk.norm_eps))
        k = rope(F.rms_norm(qkv[:, H * dh:(H + Hkv) * dh].reshape(L, Hkv, dh), (dh,), t(blk.gk), blk.norm_eps))
        v = qkv[:, (H + Hkv) * dh:].reshape(L, Hkv, dh)
        att = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None], v.permute(1, 0, 2)[None],
                                             is_causal=True, enable_gqa=True)[0].permute(1, 0, 2).reshape(L, H * dh)
        h1 = h0 + F.linear(att, t(blk.o.W))
        gu = F.linear(F.rms_norm(h1, (d,), t(blk.g2), blk.norm_eps), t(blk.fc1.W))
        want.append((h1 + F.linear(F.silu(gu[:, 0::2]) * gu[:, 1::2], t(blk.fc2.W))).numpy())
    np.testing.assert_allclose(got, np.concatenate(want), rtol=1e-9, atol=1e-11)
