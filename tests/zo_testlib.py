"""Shared helpers of the GPU parity tests: tolerance rule, oracle-side chain."""
import numpy as np

from oracle import zo_oracle as zo


def assert_close(got, want, rtol, what="", atol=0.0):
    """|got - want| <= rtol * max(|want|, rms(want)) + atol, element by element."""
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if want.size == 0:
        return
    rms = float(np.sqrt(np.mean(want ** 2)))
    bound = rtol * np.maximum(np.abs(want), rms) + atol
    err = np.abs(got - want)
    bad = ~(err <= bound)          # catches NaN too
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err / np.maximum(bound, 1e-300), 0)), err.shape)
        raise AssertionError("%s: %d of %d outside rtol %g (worst at %s: got %r want %r, rms %g)"
                             % (what, int(bad.sum()), err.size, rtol, i, got[i], want[i], rms))


def oracle_batch(w):
    return zo.Batch(w.cu_seqlens, w.seq_cand, w.cand_dir, w.cand_sign, w.dir_seed)


def oracle_bank(layer):
    if layer.P is None:
        return None
    return zo.Bank(layer.P, layer.Vb, layer.R_used)


def oracle_layer(w, i, X, rows=None, out_dtype=None):
    l = w.layers[i]
    return zo.probe_linear(oracle_batch(w), X, l.W, w.r, w.eps, l.tensor_id, oracle_bank(l), bias=getattr(l, "bias", None), act=l.act,
                           factor_dtype=w.dtype, out_dtype=out_dtype or w.dtype, rows=rows)


def oracle_chain(w):
    """End-to-end oracle: layers in sequence (rounding at each declared dtype), scoring, estimate."""
    return zo.run_chain(oracle_batch(w), w.X, w.layers, w.head, w.targets, w.r, w.eps, w.dtype, w.reduction)


def to_np(t):
    import torch
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()
