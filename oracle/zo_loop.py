"""Oracle for the multi-step loop (plain definition, composed of the one-step oracle).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Sec. 3.2: a direction's V_k is reused over an interval I_k of nu steps while
U_t is drawn afresh every step; the interval's updates factorise as
    sum_{t in I_k} beta_t U_t V_k^T = P_k V_k^T          (Eq. layer-coupling)
so the execution layer keeps P_k, the active probes are
    W_t^{+-} = W_0 + (P_k +- eps U_t) V_k^T              (Eq. combined-probe)
and completed intervals stay in the bank, W_eff = W_0 + sum_k P_k V_k^T (Eq. bank).
With B bank blocks the reuse covers nu * B steps before the bank must be
folded or the run stops.

Readings (the paper fixes no numbering of seeds or blocks):
  * step t, interval i = t // nu; with K directions per step,
        U seed of direction j = base_u + t * K + j      (mod 2^64)
        V seed of direction j = base_v + i * K + j      (mod 2^64)
  * interval i owns bank block i mod B, i.e. the columns
        [ (block * K + j) * r , +r )  for direction j;
    the first step of an interval opens the block (P = beta U, Vb = V), the
    others accumulate into it.  Wrapping over a block that still holds an
    earlier interval discards that interval: run_loop refuses unless told to.

run_loop applies the one-step definition (zo_oracle.run_chain, then
zo_oracle.bank_update) step after step.  run_loop_dense is the same
optimisation written without any bank: it keeps the dense weights
W_eff = W_0 + sum beta_t U_t V^T explicitly; the two must agree (pinned in
tests/test_oracle_loop.py), which is Eq. (layer-coupling) and Eq.
(combined-probe) checked end to end.
"""
import copy
from types import SimpleNamespace

import numpy as np

from . import zo_oracle as zo

_MASK = (1 << 64) - 1


def schedule(step, nu, n_blocks, K, r, base_u, base_v):
    """Seeds, bank block and mode of step `step` (see the module docstring)."""
    interval = step // nu
    block = interval % n_blocks
    seed_u = np.array([(base_u + step * K + j) & _MASK for j in range(K)], dtype=np.uint64)
    seed_v = np.array([(base_v + interval * K + j) & _MASK for j in range(K)], dtype=np.uint64)
    col0 = np.array([(block * K + j) * r for j in range(K)], dtype=np.int32)
    return SimpleNamespace(step=step, interval=interval, block=block, append=(step % nu == 0),
                           seed_u=seed_u, seed_v=seed_v, col0=col0)


def run_loop(batch, X, layers, head, targets, r, eps, dtype, reduction, steps, nu, n_blocks, lr,
             base_u, base_v, first_step=0, allow_wrap=False, fold_at_wrap=False):
    """`steps` optimisation steps starting at step number `first_step`.

    layers: objects with W, tensor_id, act, P, Vb, R_used (the banks must have
    room for n_blocks * K * r columns; they are not modified: the final banks
    are returned).  Every step evaluates the candidates of `batch` with that
    step's seeds against the current banks, then updates every layer's bank.
    With fold_at_wrap, whenever the schedule is about to reopen block 0 over
    intervals still in the bank, every bank is first folded into its layer's
    base weights (rounded to `dtype`) and emptied: the run continues past
    nu * n_blocks steps and nothing is discarded.
    Returns (per-step list of run_chain outputs, final list of Bank); with
    fold_at_wrap the final base weights are a third element."""
    K = len(batch.dir_seed)
    layers = [copy.copy(l) for l in layers]
    banks = [zo.Bank(np.array(l.P, np.float32), np.array(l.Vb, np.float32), int(l.R_used)) for l in layers]
    outs = []
    for t in range(first_step, first_step + steps):
        sc = schedule(t, nu, n_blocks, K, r, base_u, base_v)
        if sc.interval >= n_blocks and sc.block == 0 and sc.append and fold_at_wrap:
            for i, l in enumerate(layers):
                l.W, banks[i] = zo.fold_bank(l.W, banks[i], dtype)
        elif sc.interval >= n_blocks and not allow_wrap and not fold_at_wrap:
            raise ValueError("bank exhausted after %d steps: fold it or stop" % (nu * n_blocks))
        b = zo.Batch(batch.cu_seqlens, batch.seq_cand, batch.cand_dir, batch.cand_sign, sc.seed_u, sc.seed_v)
        cur = []
        for l, bank in zip(layers, banks):
            c = copy.copy(l)
            c.P, c.Vb, c.R_used = bank.P, bank.Vb, bank.R_used
            cur.append(c)
        out = zo.run_chain(b, X, cur, head, targets, r, eps, dtype, reduction)
        out["schedule"] = sc
        outs.append(out)
        banks = [zo.bank_update(bank, b, l.W.shape[0], l.W.shape[1], r, l.tensor_id, out["proj_grad"], lr, sc.col0,
                                append=sc.append, factor_dtype=dtype)
                 for l, bank in zip(layers, banks)]
    if fold_at_wrap:
        return outs, banks, [l.W for l in layers]
    return outs, banks


def run_loop_dense(batch, X, layers, head, targets, r, eps, dtype, reduction, steps, nu, lr, base_u, base_v):
    """The same optimisation without a bank: every layer's dense weight is
    updated in place in fp64, W <- W + beta_t U_t V^T, and the candidates of a
    step are W +- eps U_t V^T.  Returns the per-step run_chain outputs and the
    final dense weights."""
    K = len(batch.dir_seed)
    Ws = [np.asarray(l.W, np.float64).copy() for l in layers]
    outs = []
    for t in range(steps):
        sc = schedule(t, nu, 1 << 30, K, r, base_u, base_v)
        b = zo.Batch(batch.cu_seqlens, batch.seq_cand, batch.cand_dir, batch.cand_sign, sc.seed_u, sc.seed_v)
        cur = []
        for l, W in zip(layers, Ws):
            c = copy.copy(l)
            c.W, c.P, c.Vb, c.R_used = W, None, None, 0
            cur.append(c)
        out = zo.run_chain(b, X, cur, head, targets, r, eps, dtype, reduction)
        outs.append(out)
        g = np.asarray(out["proj_grad"], np.float64)
        for i, l in enumerate(layers):
            m, n = Ws[i].shape
            for k in range(K):
                U, V = zo.direction_factors(b, k, m, n, r, l.tensor_id, dtype)
                Ws[i] += (-float(np.float32(lr)) * g[k] / K) * (U @ V.T)
    return outs, Ws
