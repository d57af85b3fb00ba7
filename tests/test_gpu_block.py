"""GPU parity of what joins the probe linears of a decoder block (residual sum +
normalisation, packed causal attention) and of a whole block, against the CPU
oracle.  Tolerances as for the rest of the path: fp32 rel 1e-5, bf16 storage
with fp32 accumulation rel 2e-2 (rel means |got - want| <= rtol * max(|want|,
rms(want))); sums of two stored values are exact up to the storage rounding and
are compared bit for bit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import zo_block as ob
from oracle import zo_oracle as zo
from paper_2605_28760_amd import binding as zb
from paper_2605_28760_amd import workloads as wl
from paper_2605_28760_amd.runner import DeviceBatch, DeviceBlock, DeviceModel, DeviceWorkload
from zo_testlib import assert_close, oracle_batch, to_np

DEV = "cuda:0"


def _rng(seed):
    return np.random.default_rng(seed)


def _dev(a, dtype):
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32
    return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(DEV).to(tt)


def _vals(a, dtype):
    """The values the device holds for host array a."""
    return wl.as_bf16_values(a).astype(np.float64) if dtype == "bf16" else np.asarray(a, np.float32).astype(np.float64)


def _plain_batch(lens):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    S = len(lens)
    return DeviceBatch(cu, np.full(S, -1, np.int32), np.zeros(0, np.int32), np.zeros(0, np.float32),
                       np.zeros(0, np.uint64), DEV), cu


# ------------------------------------------------------------------ add + norm

def _run_add_norm(x, res, gamma, beta, kind, eps, dtype, want_sum=True, want_y=True, in_place=False, pad=0):
    T, d = x.shape
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32

    def padded(a):
        buf = torch.zeros((T, d + pad), device=DEV, dtype=tt)
        buf[:, :d] = _dev(a, dtype)
        return buf
    X = padded(x)
    R = None if res is None else padded(res)
    H = (X if in_place else torch.full((T, d + pad), 7.0, device=DEV, dtype=tt)) if (want_sum and res is not None) else None
    Y = torch.full((T, d + pad), 7.0, device=DEV, dtype=tt) if want_y else None
    g = None if gamma is None else torch.from_numpy(np.asarray(gamma, np.float32)).to(DEV)
    b = None if beta is None else torch.from_numpy(np.asarray(beta, np.float32)).to(DEV)
    ld = lambda t: 0 if t is None else t.stride(0)
    zb.zo_add_norm(X, ld(X), R, ld(R), g, b, kind, eps, T, d, zb.ZO_BF16 if dtype == "bf16" else zb.ZO_F32,
                   H, ld(H), Y, ld(Y))
    torch.cuda.synchronize()
    if pad:
        for t in (H, Y):       # columns past d are never written
            if t is not None and not (in_place and t is H):
                assert (to_np(t[:, d:]) == 7.0).all()
    return (None if H is None else to_np(H[:, :d])), (None if Y is None else to_np(Y[:, :d]))


@pytest.mark.parametrize("dtype,d,pad", [("f32", 77, 3), ("f32", 1024, 0), ("bf16", 256, 0), ("bf16", 4096, 8),
                                         ("bf16", 5120, 0), ("bf16", 6144, 0), ("bf16", 8192, 0), ("bf16", 100, 2),
                                         ("bf16", 8200, 0)])
@pytest.mark.parametrize("kind", [ob.LAYER_NORM, ob.RMS_NORM])
def test_add_norm_matches_oracle(dtype, d, pad, kind):
    g = _rng(d * 10 + kind)
    T = 37
    x = g.normal(size=(T, d)) * 2 + 0.3
    res = g.normal(size=(T, d))
    gamma = 1 + 0.2 * g.normal(size=d)
    beta = 0.1 * g.normal(size=d) if kind == ob.LAYER_NORM else None
    eps = 1e-5
    rtol = 1e-5 if dtype == "f32" else 2e-2
    xv, rv = _vals(x, dtype), _vals(res, dtype)
    gv = np.asarray(gamma, np.float32).astype(np.float64)
    bv = None if beta is None else np.asarray(beta, np.float32).astype(np.float64)
    # with a residual
    want_h, want_y = ob.add_norm(xv, rv, gv, bv, kind, eps, dtype)
    got_h, got_y = _run_add_norm(x, res, gamma, beta, kind, eps, dtype, pad=pad)
    np.testing.assert_array_equal(got_h, want_h)
    assert_close(got_y, want_y, rtol, "y")
    # without one
    _, want_y0 = ob.add_norm(xv, None, gv, bv, kind, eps, dtype)
    _, got_y0 = _run_add_norm(x, None, gamma, beta, kind, eps, dtype, pad=pad)
    assert_close(got_y0, want_y0, rtol, "y (no residual)")
    # sum written over X itself; and the sum alone
    got_h2, got_y2 = _run_add_norm(x, res, gamma, beta, kind, eps, dtype, in_place=True, pad=pad)
    np.testing.assert_array_equal(got_h2, want_h)
    np.testing.assert_array_equal(got_y2, got_y)
    got_h3, none_y = _run_add_norm(x, res, None, None, kind, eps, dtype, want_y=False, pad=pad)
    assert none_y is None
    np.testing.assert_array_equal(got_h3, want_h)
    # normalised rows without storing the sum
    _, got_y4 = _run_add_norm(x, res, gamma, beta, kind, eps, dtype, want_sum=False, pad=pad)
    np.testing.assert_array_equal(got_y4, got_y)


def test_add_norm_moments_of_a_shifted_row():
    """A common offset of 30 standard deviations must not spoil the variance: the one-pass formula
    E[x^2] - E[x]^2 loses about 900 * 2^-24 of it in fp32, the two-pass moments do not."""
    g = _rng(5)
    d = 2048
    x = (g.normal(size=(8, d)) + 30.0).astype(np.float32)
    _, got = _run_add_norm(x, None, np.ones(d), np.zeros(d), ob.LAYER_NORM, 1e-5, "f32")
    _, want = ob.add_norm(x.astype(np.float64), None, np.ones(d), np.zeros(d), ob.LAYER_NORM, 1e-5, "f32")
    assert_close(got, want, 1e-5, "shifted rows")


# ------------------------------------------------------------------ attention

def _run_attention(q, k, v, lens, H, Hkv, dh, scale, dtype, fused=True):
    batch, cu = _plain_batch(lens)
    T = int(cu[-1])
    nq, nkv = H * dh, Hkv * dh
    tt = torch.bfloat16 if dtype == "bf16" else torch.float32
    zdt = zb.ZO_BF16 if dtype == "bf16" else zb.ZO_F32
    out = torch.full((T, nq + 8), 3.0, device=DEV, dtype=tt)
    if fused:    # q, k, v as column ranges of one projection output
        qkv = torch.cat([_dev(q, dtype), _dev(k, dtype), _dev(v, dtype)], dim=1).contiguous()
        Q, K, V = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:]
        lq = lk = lv = qkv.stride(0)
    else:
        Q, K, V = _dev(q, dtype), _dev(k, dtype), _dev(v, dtype)
        lq, lk, lv = nq, nkv, nkv
    zb.zo_attention(batch.struct, Q, lq, K, lk, V, lv, H, Hkv, dh, scale, zdt, out, out.stride(0))
    torch.cuda.synchronize()
    assert (to_np(out[:, nq:]) == 3.0).all()
    return to_np(out[:, :nq]), cu


ATT_CASES = [
    # lens, heads, kv heads
    ([1, 0, 130, 64, 257, 300, 128, 5], 2, 2),
    ([129, 63, 65, 1, 1, 512], 4, 1),
    ([700], 8, 2),
    ([33] * 9, 3, 3),
]


@pytest.mark.parametrize("lens,H,Hkv", ATT_CASES)
def test_attention_bf16_matches_oracle(lens, H, Hkv):
    dh = 128
    g = _rng(sum(lens) + H)
    T = sum(lens)
    q, k, v = g.normal(size=(T, H * dh)), g.normal(size=(T, Hkv * dh)), g.normal(size=(T, Hkv * dh))
    scale = dh ** -0.5
    got, cu = _run_attention(q, k, v, lens, H, Hkv, dh, scale, "bf16")
    want = ob.attention(_vals(q, "bf16"), _vals(k, "bf16"), _vals(v, "bf16"), cu, H, Hkv, dh, scale, "bf16")
    assert_close(got, want, 2e-2, "attention bf16")
    # peaked scores (larger scale): the weights concentrate on few keys
    got2, _ = _run_attention(q, k, v, lens, H, Hkv, dh, 0.5, "bf16", fused=False)
    want2 = ob.attention(_vals(q, "bf16"), _vals(k, "bf16"), _vals(v, "bf16"), cu, H, Hkv, dh, 0.5, "bf16")
    assert_close(got2, want2, 2e-2, "attention bf16, peaked")


@pytest.mark.parametrize("lens,H,Hkv,dh", [([1, 0, 70, 64, 130, 5], 2, 2, 64), ([50, 3, 200], 4, 2, 80),
                                            ([40, 41], 6, 1, 128), ([17], 1, 1, 256), ([9, 9], 2, 1, 24)])
def test_attention_fp32_matches_oracle(lens, H, Hkv, dh):
    g = _rng(sum(lens) + dh)
    T = sum(lens)
    q, k, v = g.normal(size=(T, H * dh)), g.normal(size=(T, Hkv * dh)), g.normal(size=(T, Hkv * dh))
    got, cu = _run_attention(q, k, v, lens, H, Hkv, dh, dh ** -0.5, "f32")
    want = ob.attention(_vals(q, "f32"), _vals(k, "f32"), _vals(v, "f32"), cu, H, Hkv, dh, dh ** -0.5, "f32")
    assert_close(got, want, 1e-5, "attention fp32")


def test_attention_bf16_closed_forms():
    """Equal keys => causal prefix mean of the values; first row of a sequence => its own value."""
    dh, H = 128, 2
    lens = [200, 1, 77]
    T = sum(lens)
    g = _rng(3)
    q = g.normal(size=(T, H * dh))
    k = np.tile(g.normal(size=(1, H * dh)), (T, 1))
    v = g.normal(size=(T, H * dh))
    got, cu = _run_attention(q, k, v, lens, H, H, dh, 1.0, "bf16")
    vv = _vals(v, "bf16")
    for a, b in zip(cu[:-1], cu[1:]):
        want = np.cumsum(vv[a:b], axis=0) / np.arange(1, b - a + 1)[:, None]
        assert_close(got[a:b], want, 2e-2, "prefix mean")
        np.testing.assert_array_equal(got[a], vv[a])


def test_attention_rows_do_not_depend_on_the_rest_of_the_batch():
    dh, H, Hkv = 128, 4, 2
    lens = [150, 3, 260, 64]
    T = sum(lens)
    g = _rng(4)
    q, k, v = g.normal(size=(T, H * dh)), g.normal(size=(T, Hkv * dh)), g.normal(size=(T, Hkv * dh))
    packed, cu = _run_attention(q, k, v, lens, H, Hkv, dh, dh ** -0.5, "bf16")
    again, _ = _run_attention(q, k, v, lens, H, Hkv, dh, dh ** -0.5, "bf16")
    np.testing.assert_array_equal(packed, again)
    for i in (0, 2, 3):
        a, b = cu[i], cu[i + 1]
        alone, _ = _run_attention(q[a:b], k[a:b], v[a:b], [b - a], H, Hkv, dh, dh ** -0.5, "bf16")
        np.testing.assert_array_equal(alone, packed[a:b])


def test_attention_empty_batches():
    batch, _ = _plain_batch([0, 0])
    dummy = torch.zeros((1, 128), device=DEV, dtype=torch.bfloat16)
    zb.zo_attention(batch.struct, dummy, 128, dummy, 128, dummy, 128, 1, 1, 128, 1.0, zb.ZO_BF16, dummy, 128)
    torch.cuda.synchronize()
    assert (to_np(dummy) == 0).all()


# ------------------------------------------------------------------ whole block

def _stagewise_block_parity(w, rtol):
    d = DeviceWorkload(w, DEV)
    blk = DeviceBlock(d)
    h2 = blk.forward()
    torch.cuda.synchronize()
    b = w.meta["block"]
    ob_batch = oracle_batch(w)
    nq, nkv = b.n_heads * b.head_dim, b.n_kv_heads * b.head_dim

    def lin(l, x):
        bank = None if l.P is None else zo.Bank(l.P, l.Vb, l.R_used)
        return zo.probe_linear(ob_batch, x, l.W, w.r, w.eps, l.tensor_id, bank, bias=l.bias, act=l.act,
                               factor_dtype=w.dtype, out_dtype=w.dtype)
    # every stage of the oracle is fed the device's own input of that stage
    got = dict(a1=to_np(blk.a1), qkv=to_np(d.Y[0]), att=to_np(blk.att), o=to_np(d.Y[1]), h1=to_np(blk.h1),
               a2=to_np(blk.a2), f1=to_np(d.Y[2]), f2=to_np(d.Y[3]), h2=to_np(h2))
    x = np.asarray(w.X, np.float64)
    _, a1 = ob.add_norm(x, None, b.g1, b.b1, b.norm_kind, b.norm_eps, w.dtype)
    assert_close(got["a1"], a1, rtol, "a1")
    qkv_want = lin(b.qkv, got["a1"])
    if b.gq is not None or b.rope_theta:     # the device applies both in place on the projection output
        q_, k_ = ob.qk_norm_rope(qkv_want[:, :nq], qkv_want[:, nq:nq + nkv], w.cu_seqlens, b.n_heads, b.n_kv_heads,
                                 b.head_dim, b.gq, b.gk, b.norm_eps, b.rope_theta, w.dtype)
        qkv_want = np.concatenate([q_, k_, qkv_want[:, nq + nkv:]], axis=1)
    assert_close(got["qkv"], qkv_want, 2 * rtol if b.gq is not None else rtol, "qkv")
    qkv = got["qkv"]
    att = ob.attention(qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:], w.cu_seqlens, b.n_heads, b.n_kv_heads,
                       b.head_dim, b.scale, w.dtype)
    assert_close(got["att"], att, rtol, "att")
    assert_close(got["o"], lin(b.o, got["att"]), rtol, "o")
    h1, a2 = ob.add_norm(x, got["o"], b.g2, b.b2, b.norm_kind, b.norm_eps, w.dtype)
    np.testing.assert_array_equal(got["h1"], h1)
    assert_close(got["a2"], a2, rtol, "a2")
    assert_close(got["f1"], lin(b.fc1, got["a2"]), rtol, "f1")
    assert_close(got["f2"], lin(b.fc2, got["f1"]), rtol, "f2")
    np.testing.assert_array_equal(got["h2"], zo._round_out(got["h1"].astype(np.float64) + got["f2"], w.dtype))
    return got


def _small_batch(lens, n_dirs, n_fg):
    ex_dir = np.arange(len(lens) - n_fg) % n_dirs
    return wl._pair_batch(lens[:len(lens) - n_fg], ex_dir, n_fg, lens[len(lens) - n_fg:])


@pytest.mark.parametrize("norm_kind,bias,Hkv", [(0, True, 2), (1, False, 1)])
def test_block_bf16_stage_by_stage_and_end_to_end(norm_kind, bias, Hkv):
    batch = _small_batch([70, 131, 9, 200, 40], 2, 1)
    w = wl.decoder_block("blk-small", 40 + norm_kind, "bf16", 256, 2, Hkv, 128, 512, norm_kind, bias, 8, 1e-3, 32, batch)
    got = _stagewise_block_parity(w, 2e-2)
    # end to end: the oracle's own chain of rounded intermediates.  Eight stages of bf16 storage
    # each contribute up to one rounding of their output, so the bound is a small multiple of 2e-2.
    want = ob.block_forward(oracle_batch(w), w.X, w.meta["block"], w.r, w.eps, "bf16")
    assert_close(got["h2"], want["h2"], 4e-2, "h2 end to end")
    assert_close(got["att"], want["att"], 4e-2, "att end to end")


def test_block_fp32_stage_by_stage_and_end_to_end():
    batch = _small_batch([33, 64, 5, 90], 1, 1)
    w = wl.decoder_block("blk-small-f32", 50, "f32", 96, 3, 1, 32, 160, 0, True, 4, 1e-3, 8, batch)
    got = _stagewise_block_parity(w, 1e-5)
    want = ob.block_forward(oracle_batch(w), w.X, w.meta["block"], w.r, w.eps, "f32")
    assert_close(got["h2"], want["h2"], 5e-5, "h2 end to end")     # eight chained fp32 stages


def test_block_foreground_rows_bit_identical():
    """Foreground sequences of a mixed batch must come out of the block exactly as from a batch
    in which every sequence is foreground (Sec. 5.4 and the mixed-batch correctness appendix)."""
    batch = _small_batch([70, 131, 9, 200, 140], 2, 2)
    w = wl.decoder_block("blk-mixed", 60, "bf16", 256, 2, 2, 128, 512, 0, True, 8, 1e-3, 32, batch)
    d = DeviceWorkload(w, DEV)
    mixed = to_np(DeviceBlock(d).forward())
    wf = wl.foreground_only(w)
    plain = to_np(DeviceBlock(DeviceWorkload(wf, DEV)).forward())
    torch.cuda.synchronize()
    fg_rows = np.concatenate([np.arange(w.cu_seqlens[s], w.cu_seqlens[s + 1]) for s in np.nonzero(w.seq_cand < 0)[0]])
    np.testing.assert_array_equal(mixed[fg_rows], plain[fg_rows])
    probe_rows = np.setdiff1d(np.arange(w.T), fg_rows)
    assert np.abs(mixed[probe_rows] - plain[probe_rows]).max() > 0


# ------------------------------------------------------------------ whole model

def _oracle_model(w):
    return ob.model_forward(oracle_batch(w), w.X, w.meta["blocks"], w.meta["final_norm"], w.head, w.targets,
                            w.r, w.eps, w.dtype, w.reduction)


def test_model_fp32_scoring_pass_and_estimate():
    """Two decoder blocks, final norm, LM head: per-candidate losses and the projected gradient of the
    whole model against the oracle (fp32: rel 1e-5 per op; losses abs 1e-3; gradient rel 5e-2)."""
    batch = wl._pair_batch([33, 64, 5, 90], [0, 1, 0, 1], 1, [20])
    w = wl.decoder_model("model-small-f32", 70, "f32", 2, 96, 3, 1, 32, 160, 211, 0, True, 4, 1e-3, 8, batch)
    d = DeviceWorkload(w, DEV)
    model = DeviceModel(d)
    model.step(update=False)
    torch.cuda.synchronize()
    want = _oracle_model(w)
    assert_close(to_np(model.final), want["final"], 1e-4, "final hidden")      # 17 chained fp32 stages
    assert_close(to_np(d.tok_nll), want["tok_nll"], 1e-4, "tok_nll", atol=1e-4)
    assert np.array_equal(to_np(d.cand_cnt), want["cand_cnt"])
    assert_close(to_np(d.cand_loss), want["cand_loss"], 0.0, "cand_loss", atol=1e-3)
    assert_close(to_np(d.proj_grad), want["proj_grad"], 5e-2, "proj_grad")
    assert np.abs(want["proj_grad"]).min() > 1e-4


def test_model_bf16_scoring_pass_updates_and_foreground_rows():
    batch = wl._pair_batch([70, 131, 9, 200], [0, 1, 0, 1], 1, [140])
    w = wl.decoder_model("model-small-bf16", 71, "bf16", 2, 256, 2, 1, 128, 512, 1000, 1, False, 8, 1e-3, 32, batch)
    d = DeviceWorkload(w, DEV)
    model = DeviceModel(d)
    model.step(update=False)
    torch.cuda.synchronize()
    want = _oracle_model(w)
    # seventeen stages of bf16 storage lie between the input and the scored rows: individual entries may
    # be off by two storage roundings (the bound of the single block, 4e-2), the mean losses by 1e-3
    assert_close(to_np(model.final), want["final"], 4e-2, "final hidden")
    assert_close(to_np(d.cand_loss), want["cand_loss"], 0.0, "cand_loss", atol=1e-3)
    # scoring and estimate on the device's own final rows: the tolerances of the scoring path
    tok = zo.token_nll(to_np(model.final), w.head, w.targets)
    assert_close(to_np(d.tok_nll), tok, 1e-4, "tok_nll of the device rows", atol=1e-3)
    loss, grad = zo.estimate(oracle_batch(w), to_np(d.cand_sum), to_np(d.cand_cnt), w.eps, w.reduction)
    assert_close(to_np(d.proj_grad), grad, 5e-2, "proj_grad from the device sums")
    # foreground rows: identical to a pass in which nothing is probed
    fg_rows = np.concatenate([np.arange(w.cu_seqlens[s], w.cu_seqlens[s + 1]) for s in np.nonzero(w.seq_cand < 0)[0]])
    mixed = to_np(model.final)[fg_rows]
    plain_model = DeviceModel(DeviceWorkload(wl.foreground_only(w), DEV))
    plain_model.forward()
    torch.cuda.synchronize()
    np.testing.assert_array_equal(mixed, to_np(plain_model.final)[fg_rows])
    # the lazy update of all eight layers moves every bank by beta * U of its own tensor
    before = [l.P.clone() for l in d.layers]
    model.step(lr=1e-2, update=True)
    torch.cuda.synchronize()
    pg = to_np(d.proj_grad)
    for i, l in enumerate(w.layers):
        new = zo.bank_update(zo.Bank(l.P, l.Vb, l.R_used), oracle_batch(w), l.m, l.n, w.r, l.tensor_id, pg, 1e-2,
                             np.arange(len(w.dir_seed)) * w.r, None, False, "bf16")
        assert_close(to_np(d.layers[i].P), new.P, 1e-5, "P of %s" % l.name, atol=1e-7)
        assert not torch.equal(before[i], d.layers[i].P)


# ------------------------------------------------------------------ Qwen3-family pieces

def _run_qk_norm_rope(q, k, lens, H, Hkv, dh, gq, gk, eps, theta, dtype):
    batch, cu = _plain_batch(lens)
    nq, nkv = H * dh, Hkv * dh
    qkv = torch.cat([_dev(q, dtype), _dev(k, dtype), torch.full((q.shape[0], 16), 5.0, device=DEV, dtype=_dev(q, dtype).dtype)],
                    dim=1).contiguous()
    up = lambda a: None if a is None else torch.from_numpy(np.asarray(a, np.float32)).to(DEV)
    zb.zo_qk_norm_rope(batch.struct, qkv[:, :nq], qkv.stride(0), qkv[:, nq:nq + nkv], qkv.stride(0), H, Hkv, dh,
                       up(gq), up(gk), eps, theta or 0.0, zb.ZO_BF16 if dtype == "bf16" else zb.ZO_F32)
    torch.cuda.synchronize()
    assert (to_np(qkv[:, nq + nkv:]) == 5.0).all()
    return to_np(qkv[:, :nq]), to_np(qkv[:, nq:nq + nkv]), cu


@pytest.mark.parametrize("dtype,H,Hkv,dh", [("bf16", 8, 2, 128), ("bf16", 5, 1, 128), ("bf16", 2, 2, 64), ("f32", 3, 1, 32),
                                            ("f32", 2, 2, 256), ("f32", 1, 1, 6)])
@pytest.mark.parametrize("norm,theta", [(True, 1e6), (False, 1e4), (True, None)])
def test_qk_norm_rope_matches_oracle(dtype, H, Hkv, dh, norm, theta):
    lens = [1, 0, 130, 7, 300]
    T = sum(lens)
    g = _rng(H * 100 + dh)
    q, k = g.normal(size=(T, H * dh)) * 2, g.normal(size=(T, Hkv * dh)) * 0.5
    gq = 1 + 0.2 * g.normal(size=dh) if norm else None
    gk = 1 + 0.2 * g.normal(size=dh) if norm else None
    got_q, got_k, cu = _run_qk_norm_rope(q, k, lens, H, Hkv, dh, gq, gk, 1e-6, theta, dtype)
    f32 = lambda a: None if a is None else np.asarray(a, np.float32).astype(np.float64)
    want_q, want_k = ob.qk_norm_rope(_vals(q, dtype), _vals(k, dtype), cu, H, Hkv, dh, f32(gq), f32(gk), 1e-6, theta, dtype)
    rtol = 1e-5 if dtype == "f32" else 2e-2
    assert_close(got_q, want_q, rtol, "q")
    assert_close(got_k, want_k, rtol, "k")
    if theta and not norm:      # first row of every sequence sits at position 0: untouched, bit for bit
        for a in (0, 1, 131, 138):
            np.testing.assert_array_equal(got_q[a], _vals(q, dtype)[a])


def test_qwen_form_block_bf16_and_fp32():
    """RMS norms, per-head q/k norms, rotary embedding, grouped heads, gated MLP: stage by stage and
    end to end, with candidates and a foreground sequence in the batch."""
    batch = _small_batch([70, 131, 9, 200, 40], 2, 1)
    w = wl.decoder_block("blk-qwen", 80, "bf16", 256, 4, 2, 128, 384, 1, False, 8, 1e-3, 32, batch, qwen=True)
    got = _stagewise_block_parity(w, 2e-2)
    want = ob.block_forward(oracle_batch(w), w.X, w.meta["block"], w.r, w.eps, "bf16")
    assert_close(got["h2"], want["h2"], 4e-2, "h2 end to end")
    batch = _small_batch([33, 64, 5, 90], 1, 1)
    w = wl.decoder_block("blk-qwen-f32", 81, "f32", 96, 3, 1, 32, 160, 1, False, 4, 1e-3, 8, batch, qwen=True)
    got = _stagewise_block_parity(w, 1e-5)
    want = ob.block_forward(oracle_batch(w), w.X, w.meta["block"], w.r, w.eps, "f32")
    assert_close(got["h2"], want["h2"], 5e-5, "h2 end to end (fp32)")


def test_model_step_replayed_from_a_graph_equals_eager_steps():
    """The whole-model step (Qwen3 form: norms, q/k norm + rotary, attention, gated MLP, head scoring,
    estimate, the update of all layers in one call) captured once and replayed, with unrelated eager
    work between the replays, against the same number of eager steps: bit for bit, banks included."""
    batch = wl._pair_batch([70, 131, 9, 200], [0, 1, 0, 1], 1, [40])
    def build():
        w = wl.decoder_model("model-graph", 72, "bf16", 2, 256, 2, 1, 128, 384, 777, 1, False, 8, 1e-3, 32, batch,
                             qwen=True)
        d = DeviceWorkload(w, DEV)
        return d, DeviceModel(d)
    d1, eager = build()
    snaps = []
    for _ in range(4):          # the graph side runs one warm-up step before the capture: 1 + 3 replays
        eager.step(lr=1e-2)
        torch.cuda.synchronize()
        snaps.append((eager.final.clone(), d1.cand_loss.clone(), d1.proj_grad.clone(), [l.P.clone() for l in d1.layers]))
    d2, graphed = build()
    graphed.capture(lr=1e-2)
    # the capture itself does not run the step: the state is that after the warm-up step
    assert all(torch.equal(a, l.P) for a, l in zip(snaps[0][3], d2.layers))
    for k in range(1, 4):
        graphed.replay()
        junk = torch.randn(1 << 16, device=DEV).sum()      # unrelated eager work between replays
        torch.cuda.synchronize()
        assert torch.isfinite(junk)
        assert torch.equal(graphed.final, snaps[k][0]), k
        assert torch.equal(d2.cand_loss, snaps[k][1]) and torch.equal(d2.proj_grad, snaps[k][2]), k
        assert all(torch.equal(a, l.P) for a, l in zip(snaps[k][3], d2.layers)), k
    assert not torch.equal(snaps[0][3][0], snaps[3][3][0])      # the banks did move from step to step
