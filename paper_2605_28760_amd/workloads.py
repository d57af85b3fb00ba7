"""Seeded synthetic inputs for the candidate-evaluation path.

This module holds *no arithmetic of the method*: it only draws random arrays
with the shapes, batch structure and value distributions of the paper's
workloads (OPT-13B and Qwen3-8B layer shapes, batch sizes 16 and 64,
eps = 1e-3, ranks 4/8/16, ragged packed batches, mixed foreground + probe
batches) and hands the same arrays to whoever asks.  The real inputs of the
paper (SST-2 prompts, trained OPT / Qwen3 weights) are not available; these
stand in for them.

Every array is drawn from numpy.random.default_rng([cfg, tag]) so a tensor
does not depend on which other tensors were drawn before it.  "bf16" data is
drawn in fp32 and rounded to the nearest bfloat16 here (torch does the
rounding); it is returned as fp32 arrays whose values are exactly
representable in bf16.
"""
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

# tags of the independent random streams
_TAG_X, _TAG_W, _TAG_HEAD, _TAG_TGT, _TAG_P, _TAG_VB, _TAG_LEN, _TAG_PERM, _TAG_BIAS, _TAG_NORM = range(10)


def _rng(cfg, tag, sub=0):
    return np.random.default_rng([int(cfg), int(tag), int(sub)])


def as_bf16_values(x):
    """Round an fp32 array to bf16 (nearest even) and return it as fp32."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).to(torch.float32).numpy()


def _normal(cfg, tag, sub, shape, std, dtype):
    a = _rng(cfg, tag, sub).standard_normal(shape, dtype=np.float32)
    a *= np.float32(std)
    return as_bf16_values(a) if dtype == "bf16" else a


@dataclass
class Layer:
    name: str
    m: int                      # out features
    n: int                      # in features
    tensor_id: int              # even id; U uses it, V uses tensor_id | 1
    W: np.ndarray               # [m, n]
    act: int = 0                # 0 none, 1 ReLU, 2 gated SiLU over (gate, up) row pairs: m/2 outputs
    P: Optional[np.ndarray] = None    # [m, R_cap] fp32
    Vb: Optional[np.ndarray] = None   # [n, R_cap] fp32
    R_used: int = 0
    X: Optional[np.ndarray] = None    # own input [T, n] when layers are timed separately
    bias: Optional[np.ndarray] = None  # fp32 [m]


@dataclass
class Workload:
    name: str
    cfg: int
    dtype: str                  # "f32" or "bf16": storage type of X, W, head, Y and of the factors
    r: int
    eps: float
    cu_seqlens: np.ndarray      # int32 [S+1]
    seq_cand: np.ndarray        # int32 [S]
    cand_dir: np.ndarray        # int32 [C]
    cand_sign: np.ndarray       # float32 [C]
    dir_seed: np.ndarray        # uint64 [K]
    layers: List[Layer] = field(default_factory=list)
    chain: bool = True          # True: X -> layers in sequence -> head; False: layers are independent
    X: Optional[np.ndarray] = None      # [T, n_0]
    head: Optional[np.ndarray] = None   # [vocab, d]
    targets: Optional[np.ndarray] = None  # int32 [T]
    reduction: int = 0          # 0 mean, 1 sum
    meta: Dict = field(default_factory=dict)

    @property
    def T(self):
        return int(self.cu_seqlens[-1])


def _seeds(cfg, K):
    return (np.uint64(0x5EED0000) + np.uint64(1000 * cfg) + np.arange(K, dtype=np.uint64)).astype(np.uint64)


def _pair_batch(lengths, ex_dir, n_fg=0, fg_lengths=(), perm=None):
    """Sequences: every example appears twice (+ then -, adjacent) under the
    two candidates of its direction; foreground sequences follow; an optional
    permutation reorders the sequences.  Returns the batch arrays and, per
    sequence, the example index it replicates (foreground examples are numbered
    after the probe examples)."""
    K = int(max(ex_dir)) + 1 if len(ex_dir) else 0
    cand_dir = np.repeat(np.arange(K, dtype=np.int32), 2)
    cand_sign = np.tile(np.array([1.0, -1.0], dtype=np.float32), K)
    seq_len, seq_cand, seq_ex = [], [], []
    for e, (L, d) in enumerate(zip(lengths, ex_dir)):
        for sgn in (0, 1):
            seq_len.append(int(L)); seq_cand.append(2 * int(d) + sgn); seq_ex.append(e)
    for j, L in enumerate(fg_lengths):
        seq_len.append(int(L)); seq_cand.append(-1); seq_ex.append(len(lengths) + j)
    seq_len = np.array(seq_len, dtype=np.int64)
    seq_cand = np.array(seq_cand, dtype=np.int32)
    seq_ex = np.array(seq_ex, dtype=np.int64)
    if perm is not None:
        seq_len, seq_cand, seq_ex = seq_len[perm], seq_cand[perm], seq_ex[perm]
    cu = np.zeros(len(seq_len) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(seq_len)
    return cu, seq_cand, cand_dir, cand_sign, seq_ex, seq_len


def _replicated_rows(cfg, tag, seq_ex, seq_len, width, std, dtype, integer_high=None):
    """Rows of every sequence are those of the example it replicates, so the +
    and - copies of an example carry identical data (the duplicated
    positive/negative slots mentioned in the paper's Limitations)."""
    n_ex = int(seq_ex.max()) + 1 if len(seq_ex) else 0
    ex_len = np.zeros(n_ex, dtype=np.int64)
    ex_len[seq_ex] = seq_len
    ex_off = np.concatenate([[0], np.cumsum(ex_len)])
    total = int(ex_off[-1])
    if integer_high is None:
        base = _normal(cfg, tag, 0, (total, width), std, dtype)
    else:
        base = _rng(cfg, tag).integers(0, integer_high, size=total, dtype=np.int64).astype(np.int32)
    idx = np.concatenate([np.arange(ex_off[e], ex_off[e] + L) for e, L in zip(seq_ex, seq_len)]) \
        if len(seq_ex) else np.zeros(0, np.int64)
    return base[idx]


def _bank(cfg, sub, m, n, R, std=1e-2):
    """Bank entries N(0, 1e-4) (variance), fp32, all R columns in use."""
    if R == 0:
        return None, None
    P = _normal(cfg, _TAG_P, sub, (m, R), std, "f32")
    Vb = _normal(cfg, _TAG_VB, sub, (n, R), std, "f32")
    return P, Vb


def tiny_fp32(d=256, vocab=512, n_ex=8, seq_len=32, r=4, eps=1e-3, cfg=0):
    """Config 1: fp32 probe linear + scoring head, one direction, candidates
    +, -, 0 (centre), every example replicated under the three candidates."""
    cand_dir = np.array([0, 0, -1], dtype=np.int32)
    cand_sign = np.array([1.0, -1.0, 0.0], dtype=np.float32)
    seq_cand = np.tile(np.arange(3, dtype=np.int32), n_ex)
    seq_ex = np.repeat(np.arange(n_ex), 3)
    seq_len_a = np.full(3 * n_ex, seq_len, dtype=np.int64)
    cu = np.zeros(3 * n_ex + 1, dtype=np.int32); cu[1:] = np.cumsum(seq_len_a)
    X = _replicated_rows(cfg, _TAG_X, seq_ex, seq_len_a, d, 1.0, "f32")
    tgt = _replicated_rows(cfg, _TAG_TGT, seq_ex, seq_len_a, 1, 0, "f32", integer_high=vocab)
    W = _normal(cfg, _TAG_W, 0, (d, d), d ** -0.5, "f32")
    head = _normal(cfg, _TAG_HEAD, 0, (vocab, d), d ** -0.5, "f32")
    return Workload("c1-tiny-fp32", cfg, "f32", r, eps, cu, seq_cand, cand_dir, cand_sign,
                    _seeds(cfg, 1), [Layer("proj", d, d, 0, W)], True, X, head, tgt, 0)


def opt_layer_set(hidden=5120, ffn=20480, n_ex=16, seq_len=256, r=8, eps=1e-3, R=64, cfg=1,
                  dtype="bf16"):
    """Config 2: the six probed linears of one OPT-13B-shaped block, each with
    its own input and its own bank; one direction, candidates + and -."""
    cu, seq_cand, cand_dir, cand_sign, seq_ex, seq_len_a = _pair_batch([seq_len] * n_ex, [0] * n_ex)
    shapes = [("q", hidden, hidden), ("k", hidden, hidden), ("v", hidden, hidden),
              ("o", hidden, hidden), ("fc1", ffn, hidden), ("fc2", hidden, ffn)]
    layers = []
    x_cache = {}
    for i, (nm, m, n) in enumerate(shapes):
        if n not in x_cache:
            x_cache[n] = _replicated_rows(cfg, _TAG_X, seq_ex, seq_len_a, n, 1.0, dtype) if n == hidden else \
                _replicated_rows(cfg, _TAG_X + 100, seq_ex, seq_len_a, n, 1.0, dtype)
        W = _normal(cfg, _TAG_W, i, (m, n), n ** -0.5, dtype)
        P, Vb = _bank(cfg, i, m, n, R)
        layers.append(Layer(nm, m, n, 2 * i, W, 0, P, Vb, R, x_cache[n]))
    return Workload("c2-opt13b-layers", cfg, dtype, r, eps, cu, seq_cand, cand_dir, cand_sign,
                    _seeds(cfg, 1), layers, False, None, None, None, 1)


def _chain(name, cfg, dtype, hidden, ffn, vocab, r, eps, R, batch, reduction):
    cu, seq_cand, cand_dir, cand_sign, seq_ex, seq_len_a = batch
    K = int(cand_dir.max()) + 1
    X = _replicated_rows(cfg, _TAG_X, seq_ex, seq_len_a, hidden, 1.0, dtype)
    tgt = _replicated_rows(cfg, _TAG_TGT, seq_ex, seq_len_a, 1, 0, "f32", integer_high=vocab)
    layers = []
    for i, (nm, m, n, act) in enumerate([("fc1", ffn, hidden, 1), ("fc2", hidden, ffn, 0)]):
        W = _normal(cfg, _TAG_W, i, (m, n), n ** -0.5, dtype)
        P, Vb = _bank(cfg, i, m, n, R)
        layers.append(Layer(nm, m, n, 2 * i, W, act, P, Vb, R))
    head = _normal(cfg, _TAG_HEAD, 0, (vocab, hidden), hidden ** -0.5, dtype)
    return Workload(name, cfg, dtype, r, eps, cu, seq_cand, cand_dir, cand_sign, _seeds(cfg, K),
                    layers, True, X, head, tgt, reduction)


def opt_scoring(hidden=5120, ffn=20480, vocab=50272, n_ex=64, seq_len=128, r=8, eps=1e-3, R=64,
                cfg=2, dtype="bf16"):
    """Config 3: fc1 -> ReLU -> fc2 -> LM head, batch 64 x {+,-}, summed NLL."""
    batch = _pair_batch([seq_len] * n_ex, [0] * n_ex)
    return _chain("c3-opt13b-scoring-b64", cfg, dtype, hidden, ffn, vocab, r, eps, R, batch, 1)


def ragged_packed(hidden=4096, ffn=12288, vocab=151936, n_ex=32, n_dirs=16, len_lo=16, len_hi=512,
                  r=16, eps=1e-3, R=128, cfg=3, dtype="bf16"):
    """Config 4: ragged packed batch on Qwen3-8B shapes: n_ex examples with
    lengths uniform in [len_lo, len_hi], each duplicated for the + and -
    candidate of one of n_dirs directions (examples dealt round-robin)."""
    lengths = _rng(cfg, _TAG_LEN).integers(len_lo, len_hi + 1, size=n_ex)
    ex_dir = np.arange(n_ex) % n_dirs
    batch = _pair_batch(lengths, ex_dir)
    return _chain("c4-qwen3-ragged", cfg, dtype, hidden, ffn, vocab, r, eps, R, batch, 0)


def mixed_foreground(hidden=4096, ffn=12288, vocab=151936, n_ex=24, n_fg=16, len_lo=64, len_hi=1024,
                     r=16, eps=1e-3, R=128, cfg=4, dtype="bf16"):
    """Config 5: n_ex probe examples x {+,-} (one direction each) plus n_fg
    foreground sequences (candidate id -1), lengths uniform in
    [len_lo, len_hi], sequence order shuffled so row tiles mix the kinds."""
    lengths = _rng(cfg, _TAG_LEN).integers(len_lo, len_hi + 1, size=n_ex + n_fg)
    perm = _rng(cfg, _TAG_PERM).permutation(2 * n_ex + n_fg)
    batch = _pair_batch(lengths[:n_ex], np.arange(n_ex), n_fg, lengths[n_ex:], perm)
    return _chain("c5-qwen3-mixed", cfg, dtype, hidden, ffn, vocab, r, eps, R, batch, 0)


def foreground_only(w: Workload, keep_only_foreground=False):
    """The same workload with every sequence made foreground (candidate id -1);
    with keep_only_foreground the probe sequences are dropped instead, keeping
    the foreground sequences in their original relative order."""
    import copy
    out = copy.copy(w)
    if not keep_only_foreground:
        out.seq_cand = np.full_like(w.seq_cand, -1)
        return out
    keep = np.nonzero(w.seq_cand < 0)[0]
    lens = np.diff(w.cu_seqlens)[keep]
    rows = np.concatenate([np.arange(w.cu_seqlens[s], w.cu_seqlens[s + 1]) for s in keep]) \
        if len(keep) else np.zeros(0, np.int64)
    cu = np.zeros(len(keep) + 1, dtype=np.int32); cu[1:] = np.cumsum(lens)
    out.cu_seqlens, out.seq_cand = cu, w.seq_cand[keep].copy()
    out.X = w.X[rows]; out.targets = w.targets[rows]
    out.meta = dict(w.meta, rows=rows)
    return out


def subset_sequences(w: Workload, seq_ids):
    """The workload restricted to the given sequences (kept in the given order);
    weights, banks, seeds and the candidate table are shared, not copied."""
    import copy
    seq_ids = np.asarray(seq_ids, dtype=np.int64)
    out = copy.copy(w)
    lens = np.diff(w.cu_seqlens)[seq_ids]
    rows = np.concatenate([np.arange(w.cu_seqlens[s], w.cu_seqlens[s + 1]) for s in seq_ids]) \
        if len(seq_ids) else np.zeros(0, np.int64)
    cu = np.zeros(len(seq_ids) + 1, dtype=np.int32); cu[1:] = np.cumsum(lens)
    out.cu_seqlens, out.seq_cand = cu, w.seq_cand[seq_ids].copy()
    if w.X is not None:
        out.X = w.X[rows]
    if w.targets is not None:
        out.targets = w.targets[rows]
    out.layers = []
    for l in w.layers:
        l2 = copy.copy(l)
        if l.X is not None:
            l2.X = l.X[rows]
        out.layers.append(l2)
    out.meta = dict(w.meta, rows=rows)
    return out


@dataclass
class Block:
    """Parameters of one pre-norm decoder block whose four linears (fused q/k/v
    projection, output projection, fc1, fc2) are probed.  The layers are also
    workload.layers[0..3], in that order."""
    norm_kind: int              # 0 layer norm, 1 RMS norm
    norm_eps: float
    g1: np.ndarray              # fp32 [hidden]
    b1: Optional[np.ndarray]
    g2: np.ndarray
    b2: Optional[np.ndarray]
    n_heads: int
    n_kv_heads: int
    head_dim: int
    scale: float
    qkv: Layer
    o: Layer
    fc1: Layer
    fc2: Layer
    # the Qwen3 form: per-head RMS-norm gains of queries and keys and the rotary base; its gated MLP
    # is fc1 with 2 * ffn output features ((gate_j, up_j) in adjacent rows) and activation 2
    gq: Optional[np.ndarray] = None
    gk: Optional[np.ndarray] = None
    rope_theta: Optional[float] = None


def _block_params(cfg, dtype, index, hidden, n_heads, n_kv_heads, head_dim, ffn, norm_kind, with_bias, R,
                  qwen=False):
    """Block number `index` of a model: its four layers (tensor ids 8*index .. 8*index + 6) and norms.
    qwen: per-head q/k norms, rotary embedding (base 1e6) and a gated MLP instead of fc1 -> ReLU -> fc2."""
    shapes = [("qkv", (n_heads + 2 * n_kv_heads) * head_dim, hidden, 0), ("o", hidden, n_heads * head_dim, 0),
              ("fc1", 2 * ffn if qwen else ffn, hidden, 2 if qwen else 1), ("fc2", hidden, ffn, 0)]
    layers = []
    for i, (nm, m, n, act) in enumerate(shapes):
        sub = 4 * index + i
        W = _normal(cfg, _TAG_W, sub, (m, n), n ** -0.5, dtype)
        P, Vb = _bank(cfg, sub, m, n, R)
        bias = _normal(cfg, _TAG_BIAS, sub, (m,), 0.1, "f32") if with_bias else None
        layers.append(Layer(nm if index == 0 else "%s.%d" % (nm, index), m, n, 2 * sub, W, act, P, Vb, R, None, bias))
    gains = [np.float32(1) + _normal(cfg, _TAG_NORM, 4 * index + j, (hidden,), 0.1, "f32") for j in range(2)]
    shifts = [_normal(cfg, _TAG_NORM, 4 * index + 2 + j, (hidden,), 0.1, "f32") if norm_kind == 0 else None
              for j in range(2)]
    blk = Block(norm_kind, 1e-5 if norm_kind == 0 else 1e-6, gains[0], shifts[0], gains[1], shifts[1],
                n_heads, n_kv_heads, head_dim, float(head_dim) ** -0.5, *layers)
    if qwen:
        blk.gq = np.float32(1) + _normal(cfg, _TAG_NORM, 1000 + 2 * index, (head_dim,), 0.1, "f32")
        blk.gk = np.float32(1) + _normal(cfg, _TAG_NORM, 1001 + 2 * index, (head_dim,), 0.1, "f32")
        blk.rope_theta = 1e6
    return blk


def decoder_block(name, cfg, dtype, hidden, n_heads, n_kv_heads, head_dim, ffn, norm_kind, with_bias, r, eps, R,
                  batch, qwen=False):
    """A decoder block on the given batch (the tuple _pair_batch returns): unit-variance input rows,
    weights N(0, 1/fan_in), norm gains around 1, small biases, banks as in the chain workloads."""
    cu, seq_cand, cand_dir, cand_sign, seq_ex, seq_len_a = batch
    K = int(cand_dir.max()) + 1
    X = _replicated_rows(cfg, _TAG_X, seq_ex, seq_len_a, hidden, 1.0, dtype)
    blk = _block_params(cfg, dtype, 0, hidden, n_heads, n_kv_heads, head_dim, ffn, norm_kind, with_bias, R, qwen)
    layers = [blk.qkv, blk.o, blk.fc1, blk.fc2]
    return Workload(name, cfg, dtype, r, eps, cu, seq_cand, cand_dir, cand_sign, _seeds(cfg, K), layers, False, X,
                    None, None, 1, {"block": blk})


def decoder_model(name, cfg, dtype, n_blocks, hidden, n_heads, n_kv_heads, head_dim, ffn, vocab, norm_kind,
                  with_bias, r, eps, R, batch, reduction=0, qwen=False):
    """n_blocks decoder blocks, a final norm and an LM head on the given batch: the teacher-forced scoring
    pass of a whole (randomly initialised) model.  workload.layers holds the 4 * n_blocks probed linears in
    execution order; meta["blocks"] their blocks; meta["final_norm"] = (gain, shift or None)."""
    cu, seq_cand, cand_dir, cand_sign, seq_ex, seq_len_a = batch
    K = int(cand_dir.max()) + 1
    X = _replicated_rows(cfg, _TAG_X, seq_ex, seq_len_a, hidden, 1.0, dtype)
    tgt = _replicated_rows(cfg, _TAG_TGT, seq_ex, seq_len_a, 1, 0, "f32", integer_high=vocab)
    blocks = [_block_params(cfg, dtype, b, hidden, n_heads, n_kv_heads, head_dim, ffn, norm_kind, with_bias, R, qwen)
              for b in range(n_blocks)]
    layers = [l for blk in blocks for l in (blk.qkv, blk.o, blk.fc1, blk.fc2)]
    gf = np.float32(1) + _normal(cfg, _TAG_NORM, 4 * n_blocks, (hidden,), 0.1, "f32")
    bf = _normal(cfg, _TAG_NORM, 4 * n_blocks + 1, (hidden,), 0.1, "f32") if norm_kind == 0 else None
    head = _normal(cfg, _TAG_HEAD, 0, (vocab, hidden), hidden ** -0.5, dtype)
    return Workload(name, cfg, dtype, r, eps, cu, seq_cand, cand_dir, cand_sign, _seeds(cfg, K), layers, False, X,
                    head, tgt, reduction, {"blocks": blocks, "final_norm": (gf, bf)})


def opt_block(hidden=5120, n_heads=40, head_dim=128, ffn=20480, n_ex=64, seq_len=128, r=8, eps=1e-3, R=64, cfg=5,
              dtype="bf16"):
    """One OPT-13B-shaped decoder block (layer norm, biases, 40 heads of 128) on the batch of config 3."""
    batch = _pair_batch([seq_len] * n_ex, [0] * n_ex)
    return decoder_block("b3-opt13b-block-b64", cfg, dtype, hidden, n_heads, n_heads, head_dim, ffn, 0, True, r, eps,
                         R, batch)


def qwen_block(hidden=4096, n_heads=32, n_kv_heads=8, head_dim=128, ffn=12288, n_ex=32, n_dirs=16, len_lo=16,
               len_hi=512, r=16, eps=1e-3, R=128, cfg=6, dtype="bf16"):
    """One Qwen3-8B-shaped decoder block (RMS norm, no biases, 32 query heads over 8 key/value heads,
    per-head q/k norms, rotary embedding, gated MLP with a fused 2 x 12288 gate/up projection) on the
    ragged batch of config 4."""
    lengths = _rng(cfg, _TAG_LEN).integers(len_lo, len_hi + 1, size=n_ex)
    batch = _pair_batch(lengths, np.arange(n_ex) % n_dirs)
    return decoder_block("b4-qwen3-block-ragged", cfg, dtype, hidden, n_heads, n_kv_heads, head_dim, ffn, 1, False,
                         r, eps, R, batch, qwen=True)


BUILDERS = {"c1": tiny_fp32, "c2": opt_layer_set, "c3": opt_scoring, "c4": ragged_packed,
            "c5": mixed_foreground, "b3": opt_block, "b4": qwen_block}
