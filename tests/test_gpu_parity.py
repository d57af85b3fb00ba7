"""GPU parity: the HIP path (through the C ABI) against the CPU oracle,
element by element, on seeded inputs that span several tiles and ragged tails.
Tolerances: integers bit-exact; fp32 outputs rel 1e-5; bf16-in / fp32-accumulate
outputs rel 2e-2; per-candidate mean loss abs 1e-3; projected gradient rel 5e-2
(rel means |got - want| <= rtol * max(|want|, rms(want)))."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from oracle import philox as px
from oracle import zo_oracle as zo
from paper_2605_28760_amd import binding as zb
from paper_2605_28760_amd import workloads as wl
from paper_2605_28760_amd.runner import DeviceWorkload, DeviceBatch
from zo_testlib import assert_close, oracle_batch, oracle_bank, oracle_chain, oracle_layer, to_np

DEV = "cuda:0"


def _sync():
    torch.cuda.synchronize()


# ---- integer streams and indices: bit-exact --------------------------------------------
@pytest.mark.parametrize("seed,tid,first,nblk", [
    (0, 0, 0, 1), (0x5EED0000, 3, 0, 4097), (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF, 0xFFFFFFFF - 10, 64),
    (0x0123456789ABCDEF, 8, (7 << 32) + 5, 1000)])
def test_philox_words_bit_exact(seed, tid, first, nblk):
    out = torch.empty((nblk, 4), device=DEV, dtype=torch.int32)
    zb.zo_philox_words(seed, tid, first, nblk, out); _sync()
    got = out.cpu().numpy().view(np.uint32)
    assert np.array_equal(got, px.factor_words(seed, tid, nblk, first_block=first))


@pytest.mark.parametrize("rows,r", [(1, 1), (5, 3), (1000, 2), (4096, 8), (777, 16), (300, 64)])
def test_factor_fill_matches_oracle(rows, r):
    seed, tid = 0x5EED0000 + rows, 6
    out = torch.empty((rows, r), device=DEV, dtype=torch.float32)
    zb.zo_factor_fill(seed, tid, rows, r, zb.ZO_F32, out); _sync()
    want = px.factor_matrix(seed, tid, rows, r, "f32")
    got = out.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - want) <= 1e-5 * np.abs(want) + 1e-6)        # the bar: rel 1e-5, abs 1e-6 near zero
    # far inside it: the radius is good to 1.4e-7 (relative) and the sine / cosine to 1.3e-7 (absolute) for
    # every uniform the generator can produce, the radius is at most sqrt(48 ln 2) = 5.77
    assert np.all(np.abs(got - want) <= 3e-7 * np.abs(want) + 8e-7)
    ob = torch.empty((rows, r), device=DEV, dtype=torch.bfloat16)
    zb.zo_factor_fill(seed, tid, rows, r, zb.ZO_BF16, ob); _sync()
    wantb = px.factor_matrix(seed, tid, rows, r, "bf16")
    gotb = ob.float().cpu().numpy().astype(np.float64)
    # the rounding decision is taken on fp32 values that may differ in the last bit:
    # at most one bf16 step apart, and only rarely
    assert np.all(np.abs(gotb - wantb) <= np.abs(wantb) * 2.0 ** -7 + 1e-30)
    assert np.mean(gotb == wantb) >= 0.999 or rows * r < 1000


def test_batch_index_bit_exact():
    rng = np.random.default_rng(0)
    lens = rng.integers(0, 40, size=300); lens[[0, 5, 6, 299]] = 0
    cu = np.zeros(301, np.int32); cu[1:] = np.cumsum(lens)
    seq_cand = rng.integers(-1, 6, size=300).astype(np.int32)
    b = zo.Batch(cu, seq_cand, np.array([0, 0, 1, 1, -1, 2], np.int32), np.array([1, -1, 1, -1, 0, 1], np.float32),
                 np.arange(3, dtype=np.uint64))
    db = DeviceBatch(b.cu_seqlens, b.seq_cand, b.cand_dir, b.cand_sign, b.dir_seed, DEV)
    ts = torch.empty(db.T, device=DEV, dtype=torch.int32); tc = torch.empty_like(ts)
    zb.zo_batch_index(db.struct, ts, tc); _sync()
    want_seq, want_cand = zo.batch_indices(b)
    assert np.array_equal(ts.cpu().numpy(), want_seq) and np.array_equal(tc.cpu().numpy(), want_cand)


# ---- config 1: fp32 end to end ------------------------------------------------------------
def test_config1_fp32_end_to_end():
    w = wl.tiny_fp32()
    d = DeviceWorkload(w, DEV)
    w_before = d.layers[0].W.clone()
    d.step(update=False); _sync()
    ref = oracle_chain(w)
    assert_close(to_np(d.Y[0]), ref["Y"][0].astype(np.float32), 1e-5, "Y")
    # scoring parity on the GPU's own activations, then end to end
    tok, seq, cs, cc = zo.score(oracle_batch(w), to_np(d.Y[0]), w.head, w.targets)
    assert_close(to_np(d.tok_nll), tok, 1e-5, "tok_nll")
    assert_close(to_np(d.seq_nll), seq, 1e-5, "seq_nll")
    assert np.array_equal(to_np(d.cand_cnt), ref["cand_cnt"])
    assert np.max(np.abs(to_np(d.cand_loss) - ref["cand_loss"])) <= 1e-3
    assert_close(to_np(d.proj_grad), ref["proj_grad"], 5e-2, "proj_grad")
    assert ref["proj_grad"][0] != 0
    assert torch.equal(w_before, d.layers[0].W)          # the base is never written


def test_fp32_ragged_with_bank_and_mixed_rows():
    w = wl.mixed_foreground(hidden=72, ffn=100, vocab=333, n_ex=5, n_fg=3, len_lo=1, len_hi=37, r=3, R=5, dtype="f32")
    d = DeviceWorkload(w, DEV)
    d.step(update=False); _sync()
    H = w.X
    for i in range(2):
        assert_close(to_np(d.Y[i]), oracle_layer(w, i, H), 1e-5, "Y%d" % i)
        H = to_np(d.Y[i])
    tok, seq, cs, cc = zo.score(oracle_batch(w), H, w.head, w.targets)
    assert_close(to_np(d.tok_nll), tok, 1e-5, "tok_nll")
    assert_close(to_np(d.cand_sum), cs, 1e-5, "cand_sum")
    assert np.array_equal(to_np(d.cand_cnt), cc)
    # foreground rows: bit-identical to an all-foreground call
    y_mixed = [y.clone() for y in d.Y]
    fg = wl.foreground_only(w)
    dfg = DeviceWorkload(fg, DEV)
    dfg.step(update=False); _sync()
    rows = torch.from_numpy(np.nonzero(zo.batch_indices(oracle_batch(w))[1] < 0)[0]).to(DEV)
    assert len(rows) > 0
    assert torch.equal(y_mixed[0][rows], dfg.Y[0][rows])


# ---- bf16 matrix-core path on reduced shapes (several tiles, ragged tails) -----------------
def _per_layer_parity(w, d, rtol=2e-2):
    H = w.X
    for i in range(len(w.layers)):
        x_in = w.layers[i].X if w.layers[i].X is not None else H
        want = oracle_layer(w, i, x_in, out_dtype=d.out_dtype)
        assert_close(to_np(d.Y[i]), want, rtol, "Y[%s]" % w.layers[i].name)
        H = to_np(d.Y[i])
    return H


def test_bf16_layer_set_with_bank():
    """Config-2 structure on reduced shapes: six independent linears, r = 8, bank R = 64."""
    w = wl.opt_layer_set(hidden=320, ffn=1280, n_ex=3, seq_len=111, r=8, R=64)
    d = DeviceWorkload(w, DEV)
    for i in range(len(w.layers)):
        d.probe_linear(i)
    _sync()
    _per_layer_parity(w, d)


def test_bf16_side_term_isolated_fp32_out():
    """Y_+ - Y_- on duplicated rows equals 2 eps (X V) U^T: checks the probe term
    itself to 2e-2 (on Y alone it hides behind the base GEMM)."""
    w = wl.opt_layer_set(hidden=256, ffn=512, n_ex=2, seq_len=150, r=8, R=0)
    d = DeviceWorkload(w, DEV, out_dtype="f32")
    L = 150
    for i in (0, 4, 5):
        l = w.layers[i]
        y = to_np(d.probe_linear(i)); _sync()
        U = px.factor_matrix(int(w.dir_seed[0]), l.tensor_id, l.m, w.r, "bf16")
        V = px.factor_matrix(int(w.dir_seed[0]), l.tensor_id + 1, l.n, w.r, "bf16")
        want = 2 * w.eps * (l.X[:L].astype(np.float64) @ V) @ U.T
        assert_close(y[:L] - y[L:2 * L], want, 2e-2, "side term of %s" % l.name, atol=2e-5)
        assert_close(y, oracle_layer(w, i, l.X, out_dtype="f32"), 2e-2, "Y fp32 out")


@pytest.mark.parametrize("builder,kw", [
    (wl.opt_scoring, dict(hidden=256, ffn=512, vocab=1000, n_ex=5, seq_len=77, r=8, R=64)),
    (wl.ragged_packed, dict(hidden=256, ffn=384, vocab=1187, n_ex=8, n_dirs=4, len_lo=1, len_hi=140, r=16, R=32)),
    (wl.mixed_foreground, dict(hidden=192, ffn=448, vocab=777, n_ex=6, n_fg=5, len_lo=3, len_hi=160, r=16, R=48)),
    (wl.ragged_packed, dict(hidden=128, ffn=256, vocab=300, n_ex=6, n_dirs=3, len_lo=1, len_hi=50, r=2, R=0)),
    (wl.ragged_packed, dict(hidden=128, ffn=256, vocab=300, n_ex=4, n_dirs=2, len_lo=1, len_hi=90, r=40, R=160)),
    (wl.mixed_foreground, dict(hidden=64, ffn=192, vocab=515, n_ex=3, n_fg=2, len_lo=60, len_hi=300, r=64, R=16)),
    # vocabularies that end exactly on a 256-row tile of the head kernel, and one row into the next tile
    (wl.opt_scoring, dict(hidden=256, ffn=512, vocab=768, n_ex=5, seq_len=77, r=8, R=64)),
    (wl.ragged_packed, dict(hidden=256, ffn=384, vocab=257, n_ex=8, n_dirs=4, len_lo=1, len_hi=140, r=16, R=32)),
])
def test_bf16_chain_parity(builder, kw):
    w = builder(**kw)
    d = DeviceWorkload(w, DEV)
    d.step(update=False); _sync()
    H = _per_layer_parity(w, d)
    b = oracle_batch(w)
    tok, seq, cs, cc = zo.score(b, H, w.head, w.targets)
    assert_close(to_np(d.tok_nll), tok, 1e-4, "tok_nll", atol=1e-4)
    assert_close(to_np(d.seq_nll), seq, 1e-4, "seq_nll", atol=1e-3)
    assert_close(to_np(d.cand_sum), cs, 1e-4, "cand_sum", atol=1e-3)
    assert np.array_equal(to_np(d.cand_cnt), cc)
    loss, grad = zo.estimate(b, cs, cc, w.eps, w.reduction)
    assert_close(to_np(d.cand_loss), loss, 1e-4, "cand_loss", atol=1e-3 if w.reduction == 0 else 1e-2)
    assert_close(to_np(d.proj_grad), grad, 5e-2, "proj_grad (same activations)")
    # end to end against the oracle's own chain
    ref = oracle_chain(w)
    if w.reduction == 0:
        assert np.max(np.abs(to_np(d.cand_loss) - ref["cand_loss"])) <= 1e-3
    assert_close(to_np(d.proj_grad), ref["proj_grad"], 5e-2, "proj_grad (end to end)")


def test_foreground_rows_bit_identical_and_base_immutable():
    """Mixed batch (config 5 structure): foreground rows of every layer and their
    token NLL equal, bit for bit, (i) the same batch with every sequence
    foreground and (ii) the foreground sequences run alone; W is never written."""
    w = wl.mixed_foreground(hidden=192, ffn=448, vocab=777, n_ex=6, n_fg=5, len_lo=3, len_hi=160, r=16, R=48)
    d = DeviceWorkload(w, DEV)
    w_sum = [l.W.view(torch.int16).to(torch.int64).sum().item() for l in d.layers]
    d.step(update=False); _sync()
    tok_cand = zo.batch_indices(oracle_batch(w))[1]
    rows = torch.from_numpy(np.nonzero(tok_cand < 0)[0]).to(DEV)
    assert 0 < len(rows) < d.batch.T
    mixed = [y[rows].clone() for y in d.Y] + [d.tok_nll[rows].clone()]
    fg_seqs = np.nonzero(w.seq_cand < 0)[0]
    mixed_seq = d.seq_nll[torch.from_numpy(fg_seqs).to(DEV)].clone()
    assert [l.W.view(torch.int16).to(torch.int64).sum().item() for l in d.layers] == w_sum

    allfg = DeviceWorkload(wl.foreground_only(w), DEV)
    allfg.step(update=False); _sync()
    for a, y in zip(mixed[:-1], allfg.Y):
        assert torch.equal(a, y[rows])
    assert torch.equal(mixed[-1], allfg.tok_nll[rows])

    alone = DeviceWorkload(wl.foreground_only(w, keep_only_foreground=True), DEV)
    alone.step(update=False); _sync()
    for a, y in zip(mixed[:-1], alone.Y):
        assert torch.equal(a, y)
    assert torch.equal(mixed[-1], alone.tok_nll)
    assert torch.equal(mixed_seq, alone.seq_nll)


def test_batch_invariance_and_determinism():
    """A sequence's activations and NLL do not depend on what else is in the
    batch or where it sits (the paper's sample-level batch-invariance check);
    two runs are bitwise equal (no atomics)."""
    w = wl.ragged_packed(hidden=256, ffn=384, vocab=1187, n_ex=8, n_dirs=4, len_lo=1, len_hi=140, r=16, R=32)
    d = DeviceWorkload(w, DEV)
    d.step(update=False); _sync()
    first = [y.clone() for y in d.Y] + [d.tok_nll.clone(), d.seq_nll.clone(), d.cand_sum.clone(), d.proj_grad.clone()]
    d.step(update=False); _sync()
    for a, b_ in zip(first, d.Y + [d.tok_nll, d.seq_nll, d.cand_sum, d.proj_grad]):
        assert torch.equal(a, b_)
    # reverse the sequence order
    import copy
    S = len(w.seq_cand)
    perm = np.arange(S)[::-1]
    lens = np.diff(w.cu_seqlens)
    w2 = copy.copy(w)
    rows = np.concatenate([np.arange(w.cu_seqlens[s], w.cu_seqlens[s + 1]) for s in perm])
    cu2 = np.zeros(S + 1, np.int32); cu2[1:] = np.cumsum(lens[perm])
    w2.cu_seqlens, w2.seq_cand, w2.X, w2.targets = cu2, w.seq_cand[perm].copy(), w.X[rows], w.targets[rows]
    d2 = DeviceWorkload(w2, DEV)
    d2.step(update=False); _sync()
    rows_t = torch.from_numpy(rows).to(DEV)
    for a, b_ in zip(first[:2], d2.Y):
        assert torch.equal(a[rows_t], b_)
    assert torch.equal(first[2][rows_t], d2.tok_nll)
    assert torch.equal(first[3][torch.from_numpy(perm.copy()).to(DEV)], d2.seq_nll)


def test_side_term_does_not_depend_on_the_rest_of_the_batch():
    """Input widths of 1024 and 2048 make the side-down pass sum several K ranges per row.  How a row's
    side term is summed must depend on the width alone: a subset of the sequences, packed in another
    order (fewer rows, fewer work items), must reproduce the shared sequences bit for bit."""
    w = wl.ragged_packed(hidden=1024, ffn=2048, vocab=1187, n_ex=10, n_dirs=5, len_lo=1, len_hi=300, r=16, R=32)
    d = DeviceWorkload(w, DEV)
    d.step(update=False); _sync()
    keep = np.array([7, 6, 18, 19, 2, 3, 11], np.int64)
    sub = wl.subset_sequences(w, keep)
    assert sub.T < w.T // 2
    d2 = DeviceWorkload(sub, DEV)
    d2.step(update=False); _sync()
    rows_t = torch.from_numpy(sub.meta["rows"]).to(DEV)
    for a, b_ in zip(d.Y, d2.Y):
        assert torch.equal(a[rows_t], b_)
    assert torch.equal(d.tok_nll[rows_t], d2.tok_nll)
    assert torch.equal(d.seq_nll[torch.from_numpy(keep).to(DEV)], d2.seq_nll)
    # and against the oracle, so that the shared bits are the right ones
    H = _per_layer_parity(sub, d2)
    tok = zo.token_nll(H, sub.head, sub.targets)
    assert_close(to_np(d2.tok_nll), tok, 1e-4, "tok_nll of the subset", atol=1e-4)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_bank_update_parity(dtype):
    m, n, r, K, R_cap = 300, 200, 4, 3, 16
    rng = np.random.default_rng(5)
    P = (rng.standard_normal((m, R_cap)) * 0.01).astype(np.float32)
    Vb = (rng.standard_normal((n, R_cap)) * 0.01).astype(np.float32)
    seeds = np.array([11, 12, 13], np.uint64)
    b = zo.Batch(np.array([0, 1], np.int32), np.array([0], np.int32), np.array([0], np.int32), np.array([1.0], np.float32), seeds)
    grads = np.array([0.5, -2.0, 1.25], np.float32)
    Pd, Vd = torch.from_numpy(P).to(DEV), torch.from_numpy(Vb).to(DEV)
    bank = zb.make_bank(R_cap, 12, Pd, Vd)
    g = torch.from_numpy(grads).to(DEV)
    sd = torch.from_numpy(seeds.view(np.int64)).to(DEV)
    dt = zb.ZO_BF16 if dtype == "bf16" else zb.ZO_F32
    # accumulate into three existing blocks with default weights 1/K
    zb.zo_bank_update(bank, m, n, r, K, sd, 4, g, 0.1, None, np.array([0, 4, 8], np.int32), 0, dt); _sync()
    want = zo.bank_update(zo.Bank(P, Vb, 12), b, m, n, r, 4, grads, 0.1, [0, 4, 8], factor_dtype=dtype)
    assert_close(Pd.cpu().numpy(), want.P, 1e-5, "P accumulate")
    assert torch.equal(Vd.cpu(), torch.from_numpy(Vb)) and bank.R_used == 12
    # open a new block with explicit weights
    wts = torch.tensor([2.0], device=DEV)
    zb.zo_bank_update(bank, m, n, r, 1, sd[2:], 4, g[2:], 0.1, wts, np.array([12], np.int32), 1, dt); _sync()
    b1 = zo.Batch(b.cu_seqlens, b.seq_cand, b.cand_dir, b.cand_sign, seeds[2:])
    want2 = zo.bank_update(want, b1, m, n, r, 4, grads[2:], 0.1, [12], dir_weight=[2.0], append=True, factor_dtype=dtype)
    assert bank.R_used == 16 == want2.R_used
    assert_close(Pd.cpu().numpy(), want2.P, 1e-5, "P append")
    tol = 1e-5 if dtype == "f32" else 2.0 ** -7
    assert np.all(np.abs(Vd.cpu().numpy().astype(np.float64) - want2.Vb) <= tol * np.abs(want2.Vb) + 1e-6)
    with pytest.raises(zb.ZoError) as e:
        zb.zo_bank_update(bank, m, n, r, 1, sd, 4, g, 0.1, None, np.array([14], np.int32), 1, dt)
    assert e.value.status == zb.ZO_ERR_BANK_FULL


def test_bank_update_at_rank_128():
    """The lazy update with a block of 128 columns per direction (rank continuum), append then accumulate."""
    m, n, r, R_cap = 150, 90, 128, 256
    seeds = np.array([21, 22], np.uint64)
    b = zo.Batch(np.array([0, 1], np.int32), np.array([0], np.int32), np.array([0], np.int32), np.array([1.0], np.float32), seeds)
    grads = np.array([0.75, -1.5], np.float32)
    Pd = torch.zeros((m, R_cap), device=DEV); Vd = torch.zeros((n, R_cap), device=DEV)
    bank = zb.make_bank(R_cap, 0, Pd, Vd)
    g = torch.from_numpy(grads).to(DEV); sd = torch.from_numpy(seeds.view(np.int64)).to(DEV)
    col0 = np.array([0, 128], np.int32)
    zb.zo_bank_update(bank, m, n, r, 2, sd, 8, g, 0.2, None, col0, 1, zb.ZO_BF16); _sync()
    want = zo.bank_update(zo.Bank(np.zeros((m, R_cap), np.float32), np.zeros((n, R_cap), np.float32), 0), b, m, n, r, 8, grads, 0.2,
                          [0, 128], append=True, factor_dtype="bf16")
    assert bank.R_used == 256 == want.R_used
    zb.zo_bank_update(bank, m, n, r, 2, sd, 8, g, 0.1, None, col0, 0, zb.ZO_BF16); _sync()
    want = zo.bank_update(want, b, m, n, r, 8, grads, 0.1, [0, 128], factor_dtype="bf16")
    # U and V are rounded to bf16 from fp32 normals that may differ from the oracle's in the last bit: an entry
    # may land one bf16 step away, rarely; everything else agrees to fp32 accuracy
    gotP, gotV = Pd.cpu().numpy().astype(np.float64), Vd.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(gotP - want.P) <= 2.0 ** -7 * np.abs(want.P) + 1e-6)
    assert np.mean(np.abs(gotP - want.P) <= 1e-5 * np.abs(want.P) + 1e-7) >= 0.999
    assert np.all(np.abs(gotV - want.Vb) <= 2.0 ** -7 * np.abs(want.Vb) + 1e-6)


def test_bank_update_of_many_layers_in_one_call_equals_the_per_layer_updates():
    """zo_bank_update_multi over 50 layers of mixed shapes (more than one launch holds), accumulate and
    append, against zo_bank_update layer by layer: bit for bit, including the columns left alone."""
    rng = np.random.default_rng(77)
    r, K, R_cap = 4, 3, 24
    shapes = [(int(rng.integers(1, 300)), int(rng.integers(1, 300))) for _ in range(50)]
    seeds = torch.from_numpy((np.arange(K, dtype=np.uint64) + np.uint64(4242)).view(np.int64)).to(DEV)
    seeds_v = torch.from_numpy((np.arange(K, dtype=np.uint64) + np.uint64(777)).view(np.int64)).to(DEV)
    pg = torch.from_numpy(rng.standard_normal(K).astype(np.float32)).to(DEV)
    wts = torch.from_numpy(rng.random(K).astype(np.float32)).to(DEV)
    for append, col0 in ((1, [8, 0, 16]), (0, [16, 8, 0])):
        col0 = np.array(col0, np.int32)
        P0 = [torch.from_numpy(rng.standard_normal((m, R_cap)).astype(np.float32)).to(DEV) for m, n in shapes]
        V0 = [torch.from_numpy(rng.standard_normal((n, R_cap)).astype(np.float32)).to(DEV) for m, n in shapes]
        Pa, Va = [p.clone() for p in P0], [v.clone() for v in V0]
        Pb, Vb = [p.clone() for p in P0], [v.clone() for v in V0]
        used = 0 if append else R_cap
        singles = [zb.make_bank(R_cap, used, Pa[i], Va[i]) for i in range(len(shapes))]
        for i, (m, n) in enumerate(shapes):
            zb.zo_bank_update(singles[i], m, n, r, K, seeds, 2 * i, pg, 0.5, wts, col0, append, zb.ZO_BF16, dir_seed_v=seeds_v)
        arr = zb.make_layer_banks([(zb.make_bank(R_cap, used, Pb[i], Vb[i]), m, n, 2 * i) for i, (m, n) in enumerate(shapes)])
        zb.zo_bank_update_multi(arr, r, K, seeds, seeds_v, pg, 0.5, wts, col0, append, zb.ZO_BF16)
        _sync()
        for i in range(len(shapes)):
            assert torch.equal(Pa[i], Pb[i]) and torch.equal(Va[i], Vb[i]), i
            assert arr[i].bank.R_used == singles[i].R_used == (20 if append else R_cap)
            assert not torch.equal(Pa[i], P0[i])
            assert torch.equal(Pa[i][:, 20:], P0[i][:, 20:])


def test_lazy_update_then_probe_matches_oracle():
    """One full step with update, then a second forward: the bank the GPU wrote
    must act in the next probe exactly as the oracle's updated bank does."""
    w = wl.opt_scoring(hidden=256, ffn=512, vocab=1000, n_ex=4, seq_len=70, r=8, R=64)
    d = DeviceWorkload(w, DEV)
    d.step(lr=1e-3, update=True); _sync()
    grads = to_np(d.proj_grad)
    ob = oracle_batch(w)
    import copy
    w2 = copy.copy(w)
    w2.layers = [copy.copy(l) for l in w.layers]
    for l in w2.layers:
        nb = zo.bank_update(oracle_bank(l), ob, l.m, l.n, w.r, l.tensor_id, grads, 1e-3, [0], factor_dtype="bf16")
        l.P, l.Vb = nb.P, nb.Vb
    for i, l in enumerate(w2.layers):
        assert_close(d.layers[i].P.cpu().numpy(), l.P, 1e-5, "P after update")
    d.step(update=False); _sync()
    _per_layer_parity(w2, d)


def test_no_candidates_and_empty_batches():
    w = wl.opt_scoring(hidden=128, ffn=256, vocab=300, n_ex=2, seq_len=40, r=8, R=16)
    fg = wl.foreground_only(w)
    d = DeviceWorkload(fg, DEV)
    d.step(update=False); _sync()
    H = _per_layer_parity(fg, d)
    assert np.all(to_np(d.cand_cnt) == 0) and np.all(to_np(d.cand_sum) == 0) and np.all(to_np(d.proj_grad) == 0)
    tok, seq, _, _ = zo.score(oracle_batch(fg), H, fg.head, fg.targets)
    assert_close(to_np(d.seq_nll), seq, 1e-4, "foreground seq_nll", atol=1e-3)
    # unscored rows (negative targets) and an empty sequence in the middle
    import copy
    w3 = copy.copy(w)
    w3.targets = w.targets.copy(); w3.targets[::3] = -1
    cu = w.cu_seqlens.copy()
    w3.cu_seqlens = np.concatenate([cu[:2], cu[1:]]).astype(np.int32)       # duplicate an offset: empty sequence 1
    w3.seq_cand = np.concatenate([w.seq_cand[:1], [1], w.seq_cand[1:]]).astype(np.int32)
    d3 = DeviceWorkload(w3, DEV)
    d3.step(update=False); _sync()
    H3 = _per_layer_parity(w3, d3)
    tok, seq, cs, cc = zo.score(oracle_batch(w3), H3, w3.head, w3.targets)
    assert np.array_equal(to_np(d3.cand_cnt), cc) and to_np(d3.seq_nll)[1] == 0
    assert_close(to_np(d3.tok_nll), tok, 1e-4, "tok_nll with unscored rows", atol=1e-4)
    assert np.all(to_np(d3.tok_nll)[::3] == 0)


def _score_with_targets(d, w, targets):
    d.targets.copy_(torch.from_numpy(np.ascontiguousarray(targets, np.int32)))
    d.score(); _sync()
    return [to_np(x).copy() for x in (d.tok_nll, d.seq_nll, d.cand_sum, d.cand_cnt)]


def test_scoring_only_active_tokens():
    """Only tokens with a target get logits (Sec. 3.3, active-token scoring): the head runs over a
    device-built list of them.  Every pattern must match the oracle, and a scored token's NLL must not
    depend on which other tokens are scored."""
    w = wl.opt_scoring(hidden=128, ffn=256, vocab=777, n_ex=5, seq_len=150, r=8, R=16)   # T = 1500: 6 token tiles
    d = DeviceWorkload(w, DEV)
    d.step(update=False); _sync()
    H = to_np(d.Y[-1])
    full_tok = to_np(d.tok_nll).copy()
    ob = oracle_batch(w)
    rng = np.random.default_rng(5)
    T, cu = w.T, w.cu_seqlens
    patterns = {}
    last16 = np.full(T, -1, np.int32)
    for s in range(len(cu) - 1):
        last16[cu[s + 1] - 16:cu[s + 1]] = w.targets[cu[s + 1] - 16:cu[s + 1]]
    patterns["last 16 of every sequence"] = last16
    patterns["random tenth"] = np.where(rng.random(T) < 0.1, w.targets, -1).astype(np.int32)
    patterns["none"] = np.full(T, -1, np.int32)
    one = np.full(T, -1, np.int32); one[T // 2] = w.targets[T // 2]
    patterns["a single token"] = one
    for n_on in (256, 257, 511):
        t = np.full(T, -1, np.int32)
        keep = np.sort(rng.choice(T, size=n_on, replace=False))
        t[keep] = w.targets[keep]
        patterns["%d tokens" % n_on] = t
    first_seq_off = w.targets.copy(); first_seq_off[cu[0]:cu[1]] = -1
    patterns["one sequence unscored"] = first_seq_off
    for name, tg in patterns.items():
        tok, seq, cs, cc = _score_with_targets(d, w, tg)
        otok, oseq, ocs, occ = zo.score(ob, H, w.head, tg)
        assert np.array_equal(cc, occ), name
        assert_close(tok, otok, 1e-4, "tok_nll, " + name, atol=1e-3)
        assert_close(seq, oseq, 1e-4, "seq_nll, " + name, atol=1e-3)
        assert_close(cs, ocs, 1e-4, "cand_sum, " + name, atol=1e-2)
        on = tg >= 0
        assert np.all(tok[~on] == 0)
        assert np.array_equal(tok[on], full_tok[on]), name   # same bits as when every token is scored


def test_es_style_one_sided_candidates():
    """N one-sided candidates around a centre (Sec. 2.2 and Sec. 5.3, the evolution-strategies shape): the probe path
    evaluates them like any other candidate table; zo_estimate_es turns the losses into normalised-reward
    coefficients.  Checked against the oracle on the GPU's own candidate sums and end to end."""
    import copy
    base = wl.opt_scoring(hidden=128, ffn=256, vocab=300, n_ex=9, seq_len=50, r=8, R=16)
    N = 5
    w = copy.copy(base)
    S = len(base.seq_cand)
    w.seq_cand = (np.arange(S) % (N + 1)).astype(np.int32)
    w.cand_dir = np.array(list(range(N)) + [-1], np.int32)
    w.cand_sign = np.array([1.0] * N + [0.0], np.float32)
    w.dir_seed = (np.arange(N, dtype=np.uint64) + np.uint64(4242))
    w.reduction = 0
    d = DeviceWorkload(w, DEV)
    for i in range(len(w.layers)):
        d.probe_linear(i)
    d.score()
    zb.zo_estimate_es(d.batch.struct, d.cand_sum, d.cand_cnt, float(w.eps), 0, d.cand_loss, d.proj_grad); _sync()
    _per_layer_parity(w, d)
    ob = oracle_batch(w)
    loss, coef = zo.estimate_es(ob, to_np(d.cand_sum), to_np(d.cand_cnt), w.eps, 0)
    assert_close(to_np(d.cand_loss), loss, 1e-6, "cand_loss")
    assert_close(to_np(d.proj_grad), coef, 1e-3, "normalised-reward coefficients", atol=1e-2)
    z = -to_np(d.proj_grad) * w.eps
    assert abs(z.mean()) < 1e-4 and abs((z ** 2).mean() - 1.0) < 1e-3
    # the two-point estimate has nothing to difference here: no direction has a negative candidate
    zb.zo_estimate(d.batch.struct, d.cand_sum, d.cand_cnt, float(w.eps), 0, d.cand_loss, d.proj_grad); _sync()
    assert not to_np(d.proj_grad).any()
    # end to end: the oracle chain's own candidate losses give the same preference order
    out = oracle_chain(w)
    _, coef_o = zo.estimate_es(ob, out["cand_sum"], out["cand_cnt"], w.eps, 0)
    zb.zo_estimate_es(d.batch.struct, d.cand_sum, d.cand_cnt, float(w.eps), 0, d.cand_loss, d.proj_grad); _sync()
    assert_close(to_np(d.cand_loss), out["cand_loss"], 1e-5, "cand_loss vs oracle chain", atol=1e-3)


def _single_layer(seed, lens, seq_cand, cand_dir, cand_sign, m, n, r, R, act=0, bias=False):
    """One bf16 probe linear with its own input on an arbitrary candidate table."""
    rng = np.random.default_rng(seed)
    cu = np.zeros(len(lens) + 1, np.int32); cu[1:] = np.cumsum(lens)
    T = int(cu[-1])
    K = (max(cand_dir) + 1) if len(cand_dir) and max(cand_dir) >= 0 else 0
    X = wl.as_bf16_values(rng.standard_normal((T, n)).astype(np.float32))
    W = wl.as_bf16_values((rng.standard_normal((m, n)) / np.sqrt(n)).astype(np.float32))
    P = (rng.standard_normal((m, R)) * 1e-2).astype(np.float32) if R else None
    Vb = (rng.standard_normal((n, R)) * 1e-2).astype(np.float32) if R else None
    layer = wl.Layer("odd", m, n, 6, W, act, P, Vb, R, X, (rng.standard_normal(m) * 0.3).astype(np.float32) if bias else None)
    return wl.Workload("odd-shapes", 9, "bf16", r, 1e-3, cu, np.array(seq_cand, np.int32),
                       np.array(cand_dir, np.int32), np.array(cand_sign, np.float32),
                       (np.arange(K, dtype=np.uint64) + np.uint64(991 + seed)), [layer], False)


@pytest.mark.parametrize("case", range(17))
def test_bf16_probe_linear_odd_shapes(case):
    """Shapes that leave ragged tails in every tile dimension of the matrix-core kernel (out features
    not a multiple of 16, 128 or 256; one token; token counts just past a tile; many short sequences of
    different directions inside one token tile; ranks 1 and 64; a bank wider than one side-down pass;
    input widths whose 64-column steps do not divide evenly among the side-down pass's k ranges; bias with
    ReLU; the gated activation with and without bias, with out-feature counts that end inside a wave's
    128-feature strip and inside a 16-feature block; rank 64 with a bank of 528 columns, which takes
    five side-down passes over the input; the ranks of the rank continuum, 128 next to a bank, 200 and 512,
    whose direction columns take further passes of 8, 4, 2 or 1 blocks of 16)."""
    cases = [
        dict(lens=[1], seq_cand=[0], cand_dir=[0], cand_sign=[1], m=8, n=64, r=1, R=0),
        dict(lens=[257, 3], seq_cand=[0, 1], cand_dir=[0, 0], cand_sign=[1, -1], m=200, n=128, r=5, R=16),
        dict(lens=[5] * 60, seq_cand=[i % 7 - 1 for i in range(60)], cand_dir=[0, 0, 1, 1, 2, -1],
             cand_sign=[1, -1, 1, -1, 1, 0], m=264, n=192, r=64, R=48, act=1),
        dict(lens=[130, 0, 0, 126, 1], seq_cand=[1, 0, -1, -1, 0], cand_dir=[0, 0], cand_sign=[1, -1], m=24, n=320, r=16, R=144),
        dict(lens=[300], seq_cand=[-1], cand_dir=[0], cand_sign=[1], m=136, n=64, r=8, R=32),
        dict(lens=[64, 64, 64, 64, 1], seq_cand=[0, 1, 2, 3, 4], cand_dir=[0, 0, 1, 1, -1], cand_sign=[1, -1, 1, -1, 0],
             m=520, n=256, r=17, R=0),
        dict(lens=[511], seq_cand=[2], cand_dir=[1, 1, 0], cand_sign=[-1, 1, 1], m=256, n=1024, r=33, R=136),
        dict(lens=[2, 254, 2], seq_cand=[0, -1, 1], cand_dir=[0, 0], cand_sign=[1, -1], m=1032, n=64, r=2, R=8),
        dict(lens=[70, 9], seq_cand=[0, 1], cand_dir=[0, 0], cand_sign=[1, -1], m=64, n=1344, r=33, R=136),
        dict(lens=[40, 0, 100, 65], seq_cand=[1, 0, -1, 2], cand_dir=[0, 1, -1], cand_sign=[1, -1, 0], m=48, n=1600, r=8, R=16),
        dict(lens=[200, 70], seq_cand=[0, 1], cand_dir=[0, 0], cand_sign=[1, -1], m=264, n=128, r=8, R=16, act=1, bias=True),
        dict(lens=[257, 3, 60], seq_cand=[0, 1, -1], cand_dir=[0, 0], cand_sign=[1, -1], m=528, n=128, r=8, R=16, act=2, bias=True),
        dict(lens=[130, 5], seq_cand=[1, 0], cand_dir=[0, 0], cand_sign=[1, -1], m=1072, n=64, r=4, R=0, act=2),
        dict(lens=[90, 40, 7], seq_cand=[0, -1, 1], cand_dir=[0, -1], cand_sign=[1, 0], m=40, n=576, r=64, R=528),
        dict(lens=[100, 60, 0, 33], seq_cand=[0, 1, 2, -1], cand_dir=[0, 0, 1], cand_sign=[1, -1, 1], m=264, n=256, r=128, R=32),
        dict(lens=[70, 130], seq_cand=[1, 0], cand_dir=[0, 0], cand_sign=[1, -1], m=136, n=320, r=200, R=0, act=1, bias=True),
        dict(lens=[258, 5], seq_cand=[0, 1], cand_dir=[0, 1], cand_sign=[1, -1], m=72, n=192, r=512, R=16),
    ]
    w = _single_layer(case, **cases[case])
    d = DeviceWorkload(w, DEV)
    d.probe_linear(0); _sync()
    _per_layer_parity(w, d)
    y32 = to_np(DeviceWorkload(w, DEV, out_dtype="f32").probe_linear(0))
    assert_close(y32, oracle_layer(w, 0, w.layers[0].X, out_dtype="f32"), 2e-2, "fp32 output")


@pytest.mark.parametrize("act,bias", [(0, False), (1, True), (2, True)])
def test_bf16_probe_linear_half_tiles_of_the_last_round(act, bias):
    """A tile count that leaves a last round of at most half the workgroups (322 tiles on 256 compute
    units: 66 left over) makes the matrix-core kernel cut those tiles into halves of 128 weight rows.
    The result must not depend on that: parity with the oracle, and the rows of the halved tiles
    bit-identical to a call over the last sequences alone, whose 130 tiles are all whole."""
    lens = [24576, 4000, 0, 4000, 4000, 4421]                      # 40997 rows: 161 token tiles x 2 weight-row tiles
    w = _single_layer(77, lens, seq_cand=[-1, 0, 1, 1, -1, 2], cand_dir=[0, 0, -1], cand_sign=[1, -1, 0],
                      m=512, n=64, r=8, R=16, act=act, bias=bias)
    d = DeviceWorkload(w, DEV)
    d.probe_linear(0); _sync()
    _per_layer_parity(w, d)
    tail = wl.subset_sequences(w, [1, 2, 3, 4, 5])                   # rows 24576 .. : token tiles 96 .. 160
    dt = DeviceWorkload(tail, DEV)
    dt.probe_linear(0); _sync()
    a, b = to_np(d.Y[0])[24576:], to_np(dt.Y[0])
    assert a.shape == b.shape and np.array_equal(a, b)
    # the same tiling with fp32 outputs (the halves' other epilogue)
    y32 = to_np(DeviceWorkload(w, DEV, out_dtype="f32").probe_linear(0))
    assert_close(y32, oracle_layer(w, 0, w.layers[0].X, out_dtype="f32"), 2e-2, "fp32 output of a tiling with halves")


def test_scoring_with_an_input_pitch_beyond_the_gather_window():
    """H spanning 2 GiB or more (here through a large row pitch) cannot be addressed through the
    scored-token list; the head then multiplies every row.  Same results, same rules for unscored rows."""
    T, d, V, ld = 4200, 128, 333, 1 << 18                  # 4200 rows x 512 KiB pitch = 2.05 GiB
    rng = np.random.default_rng(21)
    Hh = wl.as_bf16_values(rng.standard_normal((T, d)).astype(np.float32))
    Wh = wl.as_bf16_values((rng.standard_normal((V, d)) / np.sqrt(d)).astype(np.float32))
    tg = rng.integers(0, V, T).astype(np.int32)
    tg[::5] = -1
    big = torch.empty((T, ld), dtype=torch.bfloat16, device=DEV)
    big[:, :d] = torch.from_numpy(Hh).to(DEV).to(torch.bfloat16)
    W = torch.from_numpy(Wh).to(DEV).to(torch.bfloat16)
    lens = [1000, 1200, 0, 2000]
    cu = np.zeros(5, np.int32); cu[1:] = np.cumsum(lens)
    b = DeviceBatch(cu, np.array([0, 1, 0, -1], np.int32), np.array([0, 0], np.int32), np.array([1.0, -1.0], np.float32),
                    np.array([7], np.uint64), DEV)
    wsb = zb.zo_score_workspace_bytes(T, 4, V, d, zb.ZO_BF16)
    ws = torch.empty(wsb, dtype=torch.uint8, device=DEV)
    tok = torch.empty(T, device=DEV); seq = torch.empty(4, device=DEV)
    cs = torch.empty(2, device=DEV); cc = torch.empty(2, dtype=torch.int32, device=DEV)
    zb.zo_score(b.struct, big, ld, W, d, V, d, zb.ZO_BF16, torch.from_numpy(tg).to(DEV), tok, seq, cs, cc, ws, wsb); _sync()
    ob = zo.Batch(cu, np.array([0, 1, 0, -1], np.int32), np.array([0, 0], np.int32), np.array([1.0, -1.0], np.float32),
                  np.array([7], np.uint64))
    otok, oseq, ocs, occ = zo.score(ob, Hh, Wh, tg)
    assert_close(to_np(tok), otok, 1e-4, "tok_nll", atol=1e-4)
    assert_close(to_np(seq), oseq, 1e-4, "seq_nll", atol=1e-3)
    assert_close(to_np(cs), ocs, 1e-4, "cand_sum", atol=1e-3)
    assert np.array_equal(to_np(cc), occ) and np.all(to_np(tok)[::5] == 0)
