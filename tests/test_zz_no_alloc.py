"""zo_score_static, the entry point that allocates nothing (its scratch is a static device array of the
library), against zo_score with a caller workspace: two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2605_28760_amd import binding as zb
from paper_2605_28760_amd import workloads as wl
from paper_2605_28760_amd.runner import DeviceBatch

DEV = "cuda:0"


def _score_both(w, rng):
    """Scores random hidden rows of the workload's batch through both entry points; returns their outputs."""
    b = DeviceBatch(w.cu_seqlens, w.seq_cand, w.cand_dir, w.cand_sign, w.dir_seed, DEV)
    vocab, d = w.head.shape
    dt = zb.ZO_BF16 if w.dtype == "bf16" else zb.ZO_F32
    tt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    H = torch.from_numpy(rng.standard_normal((b.T, d)).astype(np.float32)).to(device=DEV, dtype=tt)
    head = torch.from_numpy(w.head).to(device=DEV, dtype=tt)
    targets = w.targets.copy()
    targets[::7] = -1                                   # some rows are not scored
    tg = torch.from_numpy(targets.astype(np.int32)).to(DEV)
    outs = []
    for static in (False, True):
        tok = torch.full((b.T,), -7.0, device=DEV)
        seq = torch.full((b.S,), -7.0, device=DEV)
        cs = torch.full((b.C,), -7.0, device=DEV)
        cc = torch.full((b.C,), -7, device=DEV, dtype=torch.int32)
        if static:
            zb.zo_score_static(b.struct, H, H.stride(0), head, head.stride(0), vocab, d, dt, tg, tok, seq, cs, cc)
        else:
            nbytes = zb.zo_score_workspace_bytes(b.T, b.S, vocab, d, dt)
            ws = torch.empty(max(nbytes, 256), device=DEV, dtype=torch.uint8)
            zb.zo_score(b.struct, H, H.stride(0), head, head.stride(0), vocab, d, dt, tg, tok, seq, cs, cc, ws, nbytes)
        torch.cuda.synchronize()
        outs.append((tok, seq, cs, cc))
    return outs


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_score_static_matches_score_on_two_calls_in_a_row(dtype):
    rng = np.random.default_rng(5)
    big = wl.ragged_packed(hidden=256, ffn=256, vocab=1187, n_ex=8, n_dirs=4, len_lo=1, len_hi=140, r=8, R=0, dtype=dtype)
    small = wl.mixed_foreground(hidden=128, ffn=128, vocab=515, n_ex=3, n_fg=2, len_lo=3, len_hi=60, r=8, R=0, dtype=dtype)
    assert small.T < big.T
    for w in (big, small):                              # the second call reuses the array the first one filled
        ref, got = _score_both(w, rng)
        for a, b_ in zip(ref, got):
            assert torch.equal(a, b_)                   # same kernels, same scratch layout: bit for bit
        assert float(got[0].max()) > 0


def test_score_static_rejects_what_does_not_fit():
    cap = zb.zo_score_static_capacity()
    w = wl.opt_scoring(hidden=64, ffn=64, vocab=64, n_ex=2, seq_len=8)
    b = DeviceBatch(w.cu_seqlens, w.seq_cand, w.cand_dir, w.cand_sign, w.dir_seed, DEV)
    T, vocab, d = b.T, 151936, 64
    assert zb.zo_score_workspace_bytes(1 << 16, b.S, vocab, d, zb.ZO_BF16) > cap
    big = zb.make_batch(1 << 16, b.cu, b.seq_cand, b.cand_dir, b.cand_sign, b.dir_seed, None, None, None,
                        n_seqs=b.S, n_cands=b.C, n_dirs=b.K)
    x = torch.zeros(64, device=DEV, dtype=torch.bfloat16)   # never read: the call is rejected before any launch
    i32 = torch.zeros(64, device=DEV, dtype=torch.int32)
    f32 = torch.zeros(64, device=DEV)
    with pytest.raises(zb.ZoError) as e:
        zb.zo_score_static(big, x, d, x, d, vocab, d, zb.ZO_BF16, i32, None, f32, f32, i32)
    assert e.value.status == zb.ZO_ERR_WORKSPACE and "static" in str(e.value)
