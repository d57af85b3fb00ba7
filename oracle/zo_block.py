"""Oracle for the decoder block that sits between the probe linears (fp64).

TEST INFRASTRUCTURE ONLY (see the package docstring).

A candidate's token-scoring forward pass (Sec. 2.2: a query is evaluated by a
teacher-forced scoring pass of the model under the candidate's weights) runs
whole decoder blocks, not isolated linear layers.  The probed tensors are the
block's linear layers (Sec. 3.2: the candidate state is a set of per-tensor
low-rank factors next to the frozen base); what joins them -- normalisation,
causal self-attention over each packed sequence (Sec. 3.1: variable-length
packing, rows of different sequences never interact) and the residual sums --
has no parameters that are perturbed and is identical for every candidate.
The paper does not spell these operations out; they are the standard
definitions of the model families it evaluates, written here directly:

  layer_norm   y = (x - mean(x)) / sqrt(var(x) + eps) * gamma + beta   (biased variance)
  rms_norm     y = x / sqrt(mean(x^2) + eps) * gamma
  attention    per sequence and head: softmax over keys j <= t of
               scale * <q_t, k_j>, applied to the values; query head h reads
               key/value head h // (n_heads / n_kv_heads)
  block        h1 = x  + Wo . attention(split(Wqkv . norm1(x)))
               h2 = h1 + W2 . act(W1 . norm2(h1))
               (pre-norm; every linear is a probe linear under the row's candidate)
  qk_norm_rope (Qwen3 family) per head: q, k <- rms_norm over the head dimension, then the
               rotary embedding: the pair (x[i], x[i + dh/2]) of a row at position p of its
               sequence is rotated by the angle p * theta^(-2i/dh)
  gated MLP    fc1 is the fused gate/up projection with activation 2 of the probe linear
               (silu(gate_j) * up_j over adjacent output features), fc2 maps the ffn columns back

Nothing here is blocked, fused or reordered: scores are formed in full per
sequence and head.  Pins: tests/test_oracle_block.py (library routines on
their common special cases, closed forms such as the causal prefix mean,
masking / packing / head-grouping invariants).
"""
import numpy as np

from . import zo_oracle as _zo

LAYER_NORM = 0
RMS_NORM = 1


def layer_norm(x, gamma, beta, eps):
    x = np.asarray(x, np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x - mu) / np.sqrt(var + eps) * np.asarray(gamma, np.float64)
    if beta is not None:
        y = y + np.asarray(beta, np.float64)
    return y


def rms_norm(x, gamma, eps):
    x = np.asarray(x, np.float64)
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gamma, np.float64)


def add_norm(x, res, gamma, beta, kind, eps, dtype="f64"):
    """h = x + res (res may be None), y = norm(h).  Both are rounded to the
    storage type `dtype`; the norm is taken of the rounded h, which is the
    value a later residual sum reads back."""
    h = np.asarray(x, np.float64)
    if res is not None:
        h = _zo._round_out(h + np.asarray(res, np.float64), dtype)
    if kind == LAYER_NORM:
        y = layer_norm(h, gamma, beta, eps)
    elif kind == RMS_NORM:
        y = rms_norm(h, gamma, eps)
    else:
        raise ValueError(kind)
    return h, _zo._round_out(y, dtype)


def attention(q, k, v, cu_seqlens, n_heads, n_kv_heads, head_dim, scale, dtype="f64"):
    """Causal self-attention over packed sequences.

    q [T, n_heads*head_dim], k and v [T, n_kv_heads*head_dim]; row t of sequence
    i attends to rows cu[i] .. t of the same sequence only."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    T = q.shape[0]
    if n_heads % n_kv_heads != 0:
        raise ValueError("n_heads must be a multiple of n_kv_heads")
    group = n_heads // n_kv_heads
    out = np.zeros((T, n_heads * head_dim), np.float64)
    cu = np.asarray(cu_seqlens, np.int64)
    for i in range(len(cu) - 1):
        a, b = int(cu[i]), int(cu[i + 1])
        L = b - a
        if L == 0:
            continue
        future = np.triu(np.ones((L, L), dtype=bool), 1)     # [t, j] True where j > t
        for h in range(n_heads):
            g = h // group
            qh = q[a:b, h * head_dim:(h + 1) * head_dim]
            kh = k[a:b, g * head_dim:(g + 1) * head_dim]
            vh = v[a:b, g * head_dim:(g + 1) * head_dim]
            s = float(scale) * (qh @ kh.T)
            s[future] = -np.inf
            s -= s.max(axis=1, keepdims=True)
            p = np.exp(s)
            p /= p.sum(axis=1, keepdims=True)
            out[a:b, h * head_dim:(h + 1) * head_dim] = p @ vh
    return _zo._round_out(out, dtype)


def qk_norm_rope(q, k, cu_seqlens, n_heads, n_kv_heads, head_dim, gamma_q, gamma_k, norm_eps, theta, dtype="f64"):
    """Per-head RMS norm (skipped when gamma_q is None) and rotary embedding (skipped when theta is
    None) of the packed query and key rows; a row's position is its offset in its own sequence."""
    q = np.asarray(q, np.float64).copy()
    k = np.asarray(k, np.float64).copy()
    T = q.shape[0]
    cu = np.asarray(cu_seqlens, np.int64)
    pos = np.zeros(T, np.float64)
    for i in range(len(cu) - 1):
        pos[cu[i]:cu[i + 1]] = np.arange(cu[i + 1] - cu[i])
    half = head_dim // 2
    if theta is not None:
        inv_freq = float(theta) ** (-2.0 * np.arange(half) / head_dim)
        ang = pos[:, None] * inv_freq[None, :]
        cos, sin = np.cos(ang), np.sin(ang)
    for x, heads, gamma in ((q, n_heads, gamma_q), (k, n_kv_heads, gamma_k)):
        for h in range(heads):
            v = x[:, h * head_dim:(h + 1) * head_dim]
            if gamma is not None:
                v = rms_norm(v, gamma, norm_eps)
            if theta is not None:
                a, b = v[:, :half], v[:, half:]
                v = np.concatenate([a * cos - b * sin, b * cos + a * sin], axis=1)
            x[:, h * head_dim:(h + 1) * head_dim] = v
    return _zo._round_out(q, dtype), _zo._round_out(k, dtype)


def block_forward(batch, x, blk, r, eps, dtype, store=None):
    """One pre-norm decoder block under the batch's candidate table.

    blk: object with attributes norm_kind, norm_eps, g1, b1, g2, b2 (b* None
    for RMS norm), n_heads, n_kv_heads, head_dim, scale and the four layers
    qkv, o, fc1, fc2 (each with W, bias, tensor_id, act, P, Vb, R_used).  Optional attributes
    select the Qwen3 form: gq, gk (per-head RMS norm gains of queries and keys), rope_theta (rotary
    embedding); a gated MLP is simply fc1.act == 2 (fused gate/up projection, half as many outputs).
    dtype is the type of the generated factors; every intermediate is rounded
    to the storage type `store` (default: dtype), as a kernel that writes it to
    memory does.  Returns a dict of all intermediates."""
    store = store or dtype
    def lin(l, inp):
        bank = None if l.P is None else _zo.Bank(l.P, l.Vb, l.R_used)
        return _zo.probe_linear(batch, inp, l.W, r, eps, l.tensor_id, bank, bias=getattr(l, "bias", None),
                                act=l.act, factor_dtype=dtype, out_dtype=store)
    nq = blk.n_heads * blk.head_dim
    nkv = blk.n_kv_heads * blk.head_dim
    _, a1 = add_norm(x, None, blk.g1, blk.b1, blk.norm_kind, blk.norm_eps, store)
    qkv = lin(blk.qkv, a1)
    q, k, v = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:nq + 2 * nkv]
    gq, theta = getattr(blk, "gq", None), getattr(blk, "rope_theta", None)
    if gq is not None or theta is not None:
        q, k = qk_norm_rope(q, k, batch.cu_seqlens, blk.n_heads, blk.n_kv_heads, blk.head_dim, gq,
                            getattr(blk, "gk", None), blk.norm_eps, theta, store)
    att = attention(q, k, v, batch.cu_seqlens, blk.n_heads, blk.n_kv_heads, blk.head_dim, blk.scale, store)
    o = lin(blk.o, att)
    h1, a2 = add_norm(x, o, blk.g2, blk.b2, blk.norm_kind, blk.norm_eps, store)
    f1 = lin(blk.fc1, a2)
    f2 = lin(blk.fc2, f1)
    h2 = _zo._round_out(np.asarray(h1, np.float64) + f2, store)
    return dict(a1=a1, qkv=qkv, q=q, k=k, att=att, o=o, h1=h1, a2=a2, f1=f1, f2=f2, h2=h2)


def model_forward(batch, x, blocks, final_norm, head, targets, r, eps, dtype, reduction, store=None):
    """Scoring pass of a whole model: the blocks in sequence, a final norm, LM-head scoring of
    every row under its candidate (the head itself is not perturbed) and the two-point estimate.
    final_norm = (gain, shift or None), of the same kind as the blocks' norms."""
    store = store or dtype
    h = x
    per_block = []
    for blk in blocks:
        out = block_forward(batch, h, blk, r, eps, dtype, store)
        per_block.append(out)
        h = out["h2"]
    last = blocks[-1]
    _, hn = add_norm(h, None, final_norm[0], final_norm[1], last.norm_kind, last.norm_eps, store)
    tok, seq, cs, cc = _zo.score(batch, hn, head, targets)
    loss, grad = _zo.estimate(batch, cs, cc, eps, reduction)
    return dict(blocks=per_block, final=hn, tok_nll=tok, seq_nll=seq, cand_sum=cs, cand_cnt=cc, cand_loss=loss,
                proj_grad=grad)
