"""Oracle for batched candidate-state evaluation (plain definition, fp64).

TEST INFRASTRUCTURE ONLY (see the package docstring).

What the path computes, by definition:

  * a packed batch of S sequences (cu_seqlens) where every sequence names the
    candidate state it is evaluated under (the ProbePlan of Sec. 2.2, Eq. 3);
  * candidate c = (direction k, sign s) sees the dense weight
        W_c = W_0 + s * eps * U_k V_k^T + P Vb^T
    (Sec. 3.2: the +-eps U V^T candidates, the combined probe, and the bank
    W_eff = W_0 + sum_k P_k V_k^T);  a centre candidate (s = 0 or k = -1) sees
    W_0 + P Vb^T;  a foreground sequence (candidate id -1) sees W_0 alone
    (Sec. 5.4 and the mixed-batch correctness appendix: foreground requests observe the
    immutable base);
  * every token row is multiplied by its candidate's dense weight, scored
    against an LM head by the ordinary negative log-likelihood, the scores
    are summed per sequence and per candidate, and the antithetic two-point
    estimator of Sec. 2.1 (Eq. 2) turns them into one projected-gradient
    coefficient per direction;
  * the lazy update of Sec. 3.2 adds beta_k U_k to the direction's column
    block of P (and, when a block is opened, stores V_k next to it);
  * folding writes W_0 + P Vb^T back into the base and empties the bank.

The factorised evaluation the GPU performs is algebraically identical to this
dense definition (Sec. 2.3), so the oracle *is* the definition: each W_c is
materialised and applied with numpy.matmul; logits are formed in full.

Pins: see tests/test_oracle_*.py.  Closed forms (quadratic loss => exact
directional derivative; zero head => ln V), invariants (factorised == dense,
antithetic symmetry O(eps^2), linearity of the lazy accumulator), reductions to
library routines (scipy logsumexp / torch cross_entropy) and brute-force index
loops.  No value printed in the paper exists for this path (it prints timings
and training curves only), so none is stored.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

from . import philox as _px


@dataclass
class Batch:
    """ProbePlan reduced to a candidate table (Sec. 2.2, Eq. 3).

    cu_seqlens [S+1]  packed row offsets, cu[0] = 0, non-decreasing
    seq_cand   [S]    candidate id of each sequence, -1 = foreground
    cand_dir   [C]    direction index of each candidate, -1 = centre
    cand_sign  [C]    +1, -1 or 0
    dir_seed   [K]    64-bit seed of each direction
    dir_seed_v [K]    optional separate seed of each direction's V (None: V uses
                      dir_seed too).  Sec. 3.2 reuses one V_k over an interval of
                      steps while U_t is drawn afresh: two seeds express that.
    """
    cu_seqlens: np.ndarray
    seq_cand: np.ndarray
    cand_dir: np.ndarray
    cand_sign: np.ndarray
    dir_seed: np.ndarray
    dir_seed_v: Optional[np.ndarray] = None

    @property
    def n_tokens(self):
        return int(self.cu_seqlens[-1])

    @property
    def n_seqs(self):
        return len(self.seq_cand)

    @property
    def n_cands(self):
        return len(self.cand_dir)

    @property
    def n_dirs(self):
        return len(self.dir_seed)


@dataclass
class Bank:
    """Persistent low-rank update bank (Sec. 3.2, Eq. bank): W_eff = W_0 + P Vb^T
    over the first R_used columns.  P [m, R_cap], Vb [n, R_cap]."""
    P: np.ndarray
    Vb: np.ndarray
    R_used: int


def batch_indices(batch: Batch):
    """Token -> sequence and token -> candidate maps of a packed batch.
    tok_seq[t] is the sequence whose half-open row range contains t."""
    cu = np.asarray(batch.cu_seqlens, dtype=np.int64)
    T = int(cu[-1])
    tok_seq = np.searchsorted(cu, np.arange(T, dtype=np.int64), side="right") - 1
    tok_cand = np.asarray(batch.seq_cand, dtype=np.int64)[tok_seq] if T else np.zeros(0, np.int64)
    return tok_seq.astype(np.int32), tok_cand.astype(np.int32)


def direction_factors(batch: Batch, k, m, n, r, tensor_id, factor_dtype):
    """U_k [m, r] and V_k [n, r] of direction k for the layer `tensor_id`."""
    seed_u = int(batch.dir_seed[k])
    seed_v = seed_u if batch.dir_seed_v is None else int(batch.dir_seed_v[k])
    U = _px.factor_matrix(seed_u, _px.u_tensor_id(tensor_id), m, r, factor_dtype)
    V = _px.factor_matrix(seed_v, _px.v_tensor_id(tensor_id), n, r, factor_dtype)
    return U, V


def candidate_weight(W, batch: Batch, cand, r, eps, tensor_id,
                     bank: Optional[Bank], factor_dtype):
    """Dense weight seen by candidate id `cand` (-1 = foreground), fp64 [m, n]."""
    W = np.asarray(W, dtype=np.float64)
    m, n = W.shape
    if cand < 0:
        return W
    Wc = W.copy()
    if bank is not None and bank.R_used > 0:
        R = bank.R_used
        Wc += np.asarray(bank.P, np.float64)[:, :R] @ np.asarray(bank.Vb, np.float64)[:, :R].T
    k = int(batch.cand_dir[cand])
    s = float(batch.cand_sign[cand])
    if k >= 0 and s != 0.0:
        U, V = direction_factors(batch, k, m, n, r, tensor_id, factor_dtype)
        Wc += (s * float(eps)) * (U @ V.T)
    return Wc


def _round_out(Y, out_dtype):
    if out_dtype == "f64":
        return Y
    Y32 = Y.astype(np.float32)
    if out_dtype == "bf16":
        Y32 = _px.round_to_bf16(Y32)
    elif out_dtype != "f32":
        raise ValueError(out_dtype)
    return Y32.astype(np.float64)


def probe_linear(batch: Batch, X, W, r, eps, tensor_id, bank: Optional[Bank] = None,
                 bias=None, act=0, factor_dtype="f32", out_dtype="f64", rows=None):
    """Y[t, :] = act(X[t, :] W_{cand(t)}^T + bias), rounded to out_dtype.  act 0 = none, 1 = ReLU,
    2 = gated SiLU: the m output features are (gate_j, up_j) pairs in adjacent rows of W and the
    result is silu(gate_j) * up_j, m/2 columns, silu(x) = x / (1 + exp(-x)).

    rows: optional index array restricting the computation to those token
    rows (the returned array then has len(rows) rows, in that order).
    """
    X = np.asarray(X)
    m = np.asarray(W).shape[0]
    _, tok_cand = batch_indices(batch)
    sel = np.arange(X.shape[0]) if rows is None else np.asarray(rows, dtype=np.int64)
    Y = np.zeros((len(sel), m), dtype=np.float64)
    cands_here = tok_cand[sel]
    for cand in np.unique(cands_here):
        Wc = candidate_weight(W, batch, int(cand), r, eps, tensor_id, bank, factor_dtype)
        pick = np.nonzero(cands_here == cand)[0]
        Y[pick] = np.asarray(X[sel[pick]], dtype=np.float64) @ Wc.T
    if bias is not None:
        Y += np.asarray(bias, dtype=np.float64)[None, :]
    if act == 1:
        Y = np.maximum(Y, 0.0)
    elif act == 2:
        # gated MLP: output features come in (gate, up) pairs; the layer returns m/2 columns
        gate, up = Y[:, 0::2], Y[:, 1::2]
        Y = gate / (1.0 + np.exp(-gate)) * up
    elif act != 0:
        raise ValueError(act)
    return _round_out(Y, out_dtype)


def token_nll(H, W_head, targets):
    """nll_t = log sum_v exp(z_tv) - z_t[y_t] with z_t = H_t W_head^T formed in
    full; rows with a negative target are not scored and return 0."""
    H = np.asarray(H, dtype=np.float64)
    Wh = np.asarray(W_head, dtype=np.float64)
    y = np.asarray(targets, dtype=np.int64)
    z = H @ Wh.T
    zmax = z.max(axis=1)
    lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
    safe = np.where(y >= 0, y, 0)
    picked = z[np.arange(len(y)), safe]
    return np.where(y >= 0, lse - picked, 0.0)


def score(batch: Batch, H, W_head, targets):
    """Per-token, per-sequence and per-candidate negative log-likelihood.

    Returns tok_nll [T], seq_nll [S] (sum over the sequence's scored tokens),
    cand_sum [C] (sum of seq_nll over the candidate's sequences) and cand_cnt
    [C] (number of scored tokens of the candidate).  Foreground sequences get a
    seq_nll but belong to no candidate.
    """
    cu = np.asarray(batch.cu_seqlens, dtype=np.int64)
    y = np.asarray(targets, dtype=np.int64)
    T, S, C = batch.n_tokens, batch.n_seqs, batch.n_cands
    tok = np.zeros(T, dtype=np.float64)
    seq = np.zeros(S, dtype=np.float64)
    csum = np.zeros(C, dtype=np.float64)
    ccnt = np.zeros(C, dtype=np.int64)
    for s in range(S):
        a, b = int(cu[s]), int(cu[s + 1])
        if b == a:
            continue
        tok[a:b] = token_nll(H[a:b], W_head, y[a:b])
        seq[s] = tok[a:b].sum()
        c = int(batch.seq_cand[s])
        if c >= 0:
            csum[c] += seq[s]
            ccnt[c] += int((y[a:b] >= 0).sum())
    return tok, seq, csum, ccnt.astype(np.int32)


def estimate(batch: Batch, cand_sum, cand_cnt, eps, reduction=0):
    """Candidate losses and the antithetic two-point coefficients (Eq. 2):
        c_k = (L(theta + eps d_k) - L(theta - eps d_k)) / (2 eps).
    reduction 0: L_c = cand_sum / max(cand_cnt, 1) (mean over scored tokens);
    reduction 1: L_c = cand_sum.  A direction that lacks its + or its -
    candidate gets coefficient 0."""
    cand_sum = np.asarray(cand_sum, dtype=np.float64)
    cand_cnt = np.asarray(cand_cnt, dtype=np.int64)
    if reduction == 0:
        loss = cand_sum / np.maximum(cand_cnt, 1)
    elif reduction == 1:
        loss = cand_sum.copy()
    else:
        raise ValueError(reduction)
    K = batch.n_dirs
    grad = np.zeros(K, dtype=np.float64)
    for k in range(K):
        plus = [c for c in range(batch.n_cands)
                if batch.cand_dir[c] == k and batch.cand_sign[c] > 0]
        minus = [c for c in range(batch.n_cands)
                 if batch.cand_dir[c] == k and batch.cand_sign[c] < 0]
        if plus and minus:
            grad[k] = (loss[plus[0]] - loss[minus[0]]) / (2.0 * float(eps))
    return loss, grad


def estimate_es(batch: Batch, cand_sum, cand_cnt, eps, reduction=0):
    """Reward-normalised one-sided estimate (the evolution-strategies shape of
    Sec. 2.2, Sec. 5.3 and the taxonomy appendix: N candidate evaluations around one centre,
    reward normalisation, a reward-weighted perturbation update).

    Direction k is represented by its lowest-numbered candidate with positive
    sign; its reward is minus that candidate's loss.  Over the N directions
    that have such a candidate,
        z_k = (R_k - mean R) / max(std R, 1e-8)      (population std)
    and the coefficient handed to the bank update is c_k = -z_k / eps, so that
    beta_k = -lr c_k / N = lr z_k / (N eps): the update lr / (N sigma) *
    sum_k z_k eps_k of evolution strategies with sigma = eps and
    eps_k = U_k V_k^T.  Directions without a positive candidate get 0.
    [Reading: the paper names the ingredients, not the formula; this is the
    standard normalised-reward form.]  Returns (cand_loss, coefficients)."""
    cand_sum = np.asarray(cand_sum, dtype=np.float64)
    cand_cnt = np.asarray(cand_cnt, dtype=np.int64)
    if reduction == 0:
        loss = cand_sum / np.maximum(cand_cnt, 1)
    elif reduction == 1:
        loss = cand_sum.copy()
    else:
        raise ValueError(reduction)
    K = batch.n_dirs
    rep = np.full(K, -1, dtype=np.int64)
    for k in range(K):
        plus = [c for c in range(batch.n_cands) if batch.cand_dir[c] == k and batch.cand_sign[c] > 0]
        if plus:
            rep[k] = plus[0]
    have = rep >= 0
    coef = np.zeros(K, dtype=np.float64)
    if have.any():
        R = -loss[rep[have]]
        z = (R - R.mean()) / max(R.std(), 1e-8)
        coef[have] = -z / float(eps)
    return loss, coef


def bank_update(bank: Bank, batch: Batch, m, n, r, tensor_id, proj_grad, lr,
                col0, dir_weight=None, append=False, factor_dtype="f32"):
    """Lazy update (Sec. 3.2, Eq. layer-coupling): with beta_k = -lr c_k w_k,
        P[:, col0_k : col0_k + r] += beta_k U_k           (accumulate)
    or, when a block is opened,
        P[:, block] = beta_k U_k,  Vb[:, block] = V_k,  R_used = max(R_used, col0_k + r).
    w_k defaults to 1/K.  Returns a new Bank (inputs are not modified); P and
    Vb are fp32 state, so the result is rounded to fp32."""
    P = np.asarray(bank.P, dtype=np.float64).copy()
    Vb = np.asarray(bank.Vb, dtype=np.float64).copy()
    R_used = int(bank.R_used)
    K = batch.n_dirs
    g = np.asarray(proj_grad, dtype=np.float32).astype(np.float64)
    w = (np.full(K, np.float32(1.0) / np.float32(K), dtype=np.float32) if dir_weight is None
         else np.asarray(dir_weight, dtype=np.float32)).astype(np.float64)
    for k in range(K):
        c0 = int(col0[k])
        if c0 < 0 or c0 + r > P.shape[1]:
            raise ValueError("bank full")
        U, V = direction_factors(batch, k, m, n, r, tensor_id, factor_dtype)
        beta = -float(np.float32(lr)) * g[k] * w[k]
        if append:
            P[:, c0:c0 + r] = beta * U
            Vb[:, c0:c0 + r] = V
            R_used = max(R_used, c0 + r)
        else:
            P[:, c0:c0 + r] += beta * U
    return Bank(P.astype(np.float32), Vb.astype(np.float32), R_used)


def fold_bank(W, bank: Bank, dtype):
    """Fold the bank into the base (Sec. 3.2: standalone runs may fold the
    external state; Eq. bank read right to left): W <- W_0 + P Vb^T over the
    columns in use, evaluated exactly and rounded once to the storage type of W.
    Returns the new W (fp32 array holding values of that type) and an emptied
    bank of the same shape."""
    R = int(bank.R_used)
    Wn = np.asarray(W, np.float64) + np.asarray(bank.P, np.float64)[:, :R] @ np.asarray(bank.Vb, np.float64)[:, :R].T
    Wn = _round_out(Wn, dtype)
    empty = Bank(np.zeros_like(np.asarray(bank.P, np.float32)), np.zeros_like(np.asarray(bank.Vb, np.float32)), R)
    return Wn, empty


def run_chain(batch: Batch, X, layers, head, targets, r, eps, dtype, reduction):
    """The whole path on one batch, in the order the definition gives it:
    probe linears in sequence (each output rounded to the declared storage
    dtype), head scoring, two-point estimate.

    layers: sequence of objects with attributes W, tensor_id, act, P, Vb, R_used
    (P None = no bank).  Returns a dict of every intermediate.
    """
    H = X
    Ys = []
    for l in layers:
        bank = None if l.P is None else Bank(l.P, l.Vb, l.R_used)
        H = probe_linear(batch, H, l.W, r, eps, l.tensor_id, bank, act=l.act,
                         factor_dtype=dtype, out_dtype=dtype)
        Ys.append(H)
    tok, seq, cs, cc = score(batch, H, head, targets)
    loss, grad = estimate(batch, cs, cc, eps, reduction)
    return dict(Y=Ys, tok_nll=tok, seq_nll=seq, cand_sum=cs, cand_cnt=cc, cand_loss=loss, proj_grad=grad)
