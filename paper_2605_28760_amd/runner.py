"""Device-side driver for a synthetic workload: uploads the arrays once,
allocates outputs and workspaces with torch (device memory and streams only)
and sequences the C-ABI calls of one step:

    zo_probe_linear (per layer) -> zo_score -> zo_estimate -> zo_bank_update

Nothing is computed here; every number comes out of libzo.so.
"""
import numpy as np
import torch

from . import binding as zb


def _dt(dtype):
    return zb.ZO_BF16 if dtype == "bf16" else zb.ZO_F32


def _tt(dtype):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


class DeviceBatch:
    """Batch arrays on the device plus the zo_batch struct that points at them."""

    def __init__(self, cu_seqlens, seq_cand, cand_dir, cand_sign, dir_seed, device, host_mirrors=True,
                 dir_seed_v=None):
        self.host = dict(cu=np.ascontiguousarray(cu_seqlens, np.int32), seq_cand=np.ascontiguousarray(seq_cand, np.int32),
                         cand_dir=np.ascontiguousarray(cand_dir, np.int32))
        self.cu = torch.from_numpy(self.host["cu"]).to(device)
        self.seq_cand = torch.from_numpy(self.host["seq_cand"]).to(device)
        self.cand_dir = torch.from_numpy(self.host["cand_dir"]).to(device)
        self.cand_sign = torch.from_numpy(np.ascontiguousarray(cand_sign, np.float32)).to(device)
        # torch has no uint64 arithmetic; the seeds travel as the same 64 bits in an int64 tensor
        self.dir_seed = torch.from_numpy(np.ascontiguousarray(dir_seed, np.uint64).view(np.int64)).to(device)
        self.dir_seed_v = None if dir_seed_v is None else \
            torch.from_numpy(np.ascontiguousarray(dir_seed_v, np.uint64).view(np.int64)).to(device)
        self.T = int(self.host["cu"][-1])
        self.S, self.C, self.K = len(self.host["seq_cand"]), len(self.host["cand_dir"]), len(dir_seed)
        mir = self.host if host_mirrors else dict(cu=None, seq_cand=None, cand_dir=None)
        self.struct = zb.make_batch(self.T, self.cu, self.seq_cand, self.cand_dir, self.cand_sign, self.dir_seed,
                                    mir["cu"], mir["seq_cand"], mir["cand_dir"],
                                    n_seqs=self.S, n_cands=self.C, n_dirs=self.K, dir_seed_v=self.dir_seed_v)


class DeviceLayer:
    def __init__(self, layer, dtype, device):
        self.name, self.m, self.n, self.tensor_id, self.act = layer.name, layer.m, layer.n, layer.tensor_id, layer.act
        self.W = torch.from_numpy(layer.W).to(device=device, dtype=_tt(dtype)).contiguous()
        self.X = None if layer.X is None else torch.from_numpy(layer.X).to(device=device, dtype=_tt(dtype)).contiguous()
        bias = getattr(layer, "bias", None)
        self.bias = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, np.float32)).to(device)
        self.bank = None
        self.P = self.Vb = None
        if layer.P is not None:
            self.P = torch.from_numpy(layer.P).to(device).contiguous()
            self.Vb = torch.from_numpy(layer.Vb).to(device).contiguous()
            self.bank = zb.make_bank(layer.P.shape[1], layer.R_used, self.P, self.Vb)


class DeviceWorkload:
    def __init__(self, w, device="cuda:0", host_mirrors=True, out_dtype=None):
        self.w = w
        self.device = torch.device(device)
        self.dtype = w.dtype
        self.out_dtype = out_dtype or w.dtype
        self.batch = DeviceBatch(w.cu_seqlens, w.seq_cand, w.cand_dir, w.cand_sign, w.dir_seed, self.device, host_mirrors)
        self.layers = [DeviceLayer(l, w.dtype, self.device) for l in w.layers]
        self.X = None if w.X is None else torch.from_numpy(w.X).to(device=self.device, dtype=_tt(w.dtype)).contiguous()
        self.head = None if w.head is None else torch.from_numpy(w.head).to(device=self.device, dtype=_tt(w.dtype)).contiguous()
        self.targets = None if w.targets is None else torch.from_numpy(np.ascontiguousarray(w.targets, np.int32)).to(self.device)
        b = self.batch
        T = b.T
        # a gated layer (activation 2) returns one column per (gate, up) pair of output features
        self.Y = [torch.empty((T, l.m // 2 if l.act == 2 else l.m), device=self.device, dtype=_tt(self.out_dtype))
                  for l in self.layers]
        ws = 0
        for l in self.layers:
            R = l.bank.R_used if l.bank is not None else 0
            ws = max(ws, zb.zo_probe_linear_workspace_bytes(T, b.S, b.K, l.m, l.n, w.r, R, _dt(w.dtype)))
        if self.head is not None:
            ws = max(ws, zb.zo_score_workspace_bytes(T, b.S, self.head.shape[0], self.head.shape[1], _dt(w.dtype)))
        self.ws_bytes = ws
        self.ws = torch.empty(max(ws, 256), device=self.device, dtype=torch.uint8)
        self.tok_nll = torch.empty(T, device=self.device, dtype=torch.float32)
        self.seq_nll = torch.empty(b.S, device=self.device, dtype=torch.float32)
        self.cand_sum = torch.empty(b.C, device=self.device, dtype=torch.float32)
        self.cand_cnt = torch.empty(b.C, device=self.device, dtype=torch.int32)
        self.cand_loss = torch.empty(b.C, device=self.device, dtype=torch.float32)
        self.proj_grad = torch.empty(b.K, device=self.device, dtype=torch.float32)

    # -- single calls -------------------------------------------------------------------
    def probe_linear(self, i, X=None, stream=None, batch=None):
        l = self.layers[i]
        x = X if X is not None else (l.X if l.X is not None else (self.X if i == 0 else self.Y[i - 1]))
        y = self.Y[i]
        zb.zo_probe_linear((batch or self.batch).struct, x, x.stride(0), l.W, l.W.stride(0), l.bias, l.m, l.n,
                           _dt(self.dtype), self.w.r, float(self.w.eps), l.tensor_id, l.bank, l.act,
                           y, y.stride(0), _dt(self.out_dtype), self.ws, self.ws_bytes, stream)
        return y

    def score(self, H=None, stream=None, batch=None):
        h = H if H is not None else self.Y[-1]
        zb.zo_score((batch or self.batch).struct, h, h.stride(0), self.head, self.head.stride(0), self.head.shape[0],
                    self.head.shape[1], _dt(self.dtype), self.targets, self.tok_nll, self.seq_nll, self.cand_sum,
                    self.cand_cnt, self.ws, self.ws_bytes, stream)

    def estimate(self, stream=None):
        zb.zo_estimate(self.batch.struct, self.cand_sum, self.cand_cnt, float(self.w.eps), self.w.reduction,
                       self.cand_loss, self.proj_grad, stream)

    def bank_update(self, i, lr, col0, append=0, dir_weight=None, stream=None):
        """Updates the blocks of the first len(col0) directions."""
        l = self.layers[i]
        col0 = np.ascontiguousarray(col0, np.int32)
        zb.zo_bank_update(l.bank, l.m, l.n, self.w.r, len(col0), self.batch.dir_seed, l.tensor_id,
                          self.proj_grad, float(lr), dir_weight, col0, append, _dt(self.dtype), stream)

    def bank_update_all(self, lr, col0, append=0, dir_weight=None, stream=None):
        """The same update for every layer that has a bank, in shared launches (zo_bank_update_multi)."""
        col0 = np.ascontiguousarray(col0, np.int32)
        banked = [l for l in self.layers if l.bank is not None]
        arr = zb.make_layer_banks([(l.bank, l.m, l.n, l.tensor_id) for l in banked])
        zb.zo_bank_update_multi(arr, self.w.r, len(col0), self.batch.dir_seed, None, self.proj_grad, float(lr),
                                dir_weight, col0, append, _dt(self.dtype), stream)
        for l, e in zip(banked, arr):
            l.bank.R_used = e.bank.R_used

    # -- one pass of the whole path --------------------------------------------------------
    def step(self, lr=1e-7, update=True, stream=None):
        for i in range(len(self.layers)):
            self.probe_linear(i, stream=stream)
        if self.head is not None and self.w.chain:
            self.score(stream=stream)
            self.estimate(stream=stream)
            if update:
                for i, l in enumerate(self.layers):
                    if l.bank is not None and l.bank.R_used >= self.w.r * self.batch.K:
                        col0 = np.arange(self.batch.K, dtype=np.int32) * self.w.r
                        self.bank_update(i, lr, col0, 0, stream=stream)


class DeviceBlock:
    """One pre-norm decoder block on a DeviceWorkload whose layers base .. base+3 are its fused q/k/v
    projection, output projection, fc1 and fc2: sequences
    zo_add_norm -> zo_probe_linear(qkv) -> zo_attention -> zo_probe_linear(o) -> zo_add_norm ->
    zo_probe_linear(fc1) -> zo_probe_linear(fc2) -> zo_add_norm (sum only)."""

    def __init__(self, d, blk=None, base=0):
        self.d, self.base = d, base
        blk = blk if blk is not None else d.w.meta["block"]
        self.blk = blk
        dev, tt = d.device, _tt(d.dtype)
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(dev)
        self.g1, self.b1, self.g2, self.b2 = up(blk.g1), up(blk.b1), up(blk.g2), up(blk.b2)
        T, hidden = d.batch.T, d.layers[base].n
        self.hidden = hidden
        self.a1, self.h1, self.a2, self.h2 = (torch.empty((T, hidden), device=dev, dtype=tt) for _ in range(4))
        self.att = torch.empty((T, blk.n_heads * blk.head_dim), device=dev, dtype=tt)
        self.h0 = None   # block input when it arrives as a pending sum (allocated on first use)
        # the Qwen3 form
        self.gq, self.gk = up(getattr(blk, "gq", None)), up(getattr(blk, "gk", None))
        self.rope_theta = getattr(blk, "rope_theta", None)

    def add_norm(self, x, res, gamma, beta, hsum, y, stream=None):
        ld = lambda t: 0 if t is None else t.stride(0)
        zb.zo_add_norm(x, ld(x), res, ld(res), gamma, beta, self.blk.norm_kind, float(self.blk.norm_eps),
                       x.shape[0], x.shape[1], _dt(self.d.dtype), hsum, ld(hsum), y, ld(y), stream)

    def qk_norm_rope(self, qkv, stream=None, batch=None):
        """Per-head q/k norm and rotary embedding, in place on the projection output (Qwen3 form only)."""
        b = self.blk
        if self.gq is None and not self.rope_theta:
            return
        nq, nkv = b.n_heads * b.head_dim, b.n_kv_heads * b.head_dim
        zb.zo_qk_norm_rope((batch or self.d.batch).struct, qkv[:, :nq], qkv.stride(0), qkv[:, nq:nq + nkv],
                           qkv.stride(0), b.n_heads, b.n_kv_heads, b.head_dim, self.gq, self.gk, float(b.norm_eps),
                           float(self.rope_theta or 0.0), _dt(self.d.dtype), stream)

    def attention(self, qkv, out, stream=None, batch=None):
        b = self.blk
        nq, nkv = b.n_heads * b.head_dim, b.n_kv_heads * b.head_dim
        q, k, v = qkv[:, :nq], qkv[:, nq:nq + nkv], qkv[:, nq + nkv:]
        zb.zo_attention((batch or self.d.batch).struct, q, qkv.stride(0), k, qkv.stride(0), v, qkv.stride(0),
                        b.n_heads, b.n_kv_heads, b.head_dim, float(b.scale), _dt(self.d.dtype), out,
                        out.stride(0), stream)

    def forward(self, X=None, stream=None, res=None, last_sum=True):
        """Runs the block on X (default: the workload's input), or on X + res when res is given (the
        previous block's pending residual sum, fused into this block's first norm).  With last_sum the
        final residual sum is written to h2 and returned; without it the two terms (h1, fc2 output) are
        returned for the caller to fuse into its next call."""
        d, i0 = self.d, self.base
        x = d.X if X is None else X
        if res is None:
            self.add_norm(x, None, self.g1, self.b1, None, self.a1, stream)
        else:
            if self.h0 is None:
                self.h0 = torch.empty_like(self.h1)
            self.add_norm(x, res, self.g1, self.b1, self.h0, self.a1, stream)
            x = self.h0
        qkv = d.probe_linear(i0, self.a1, stream)
        self.qk_norm_rope(qkv, stream)
        self.attention(qkv, self.att, stream)
        o = d.probe_linear(i0 + 1, self.att, stream)
        self.add_norm(x, o, self.g2, self.b2, self.h1, self.a2, stream)
        f1 = d.probe_linear(i0 + 2, self.a2, stream)
        f2 = d.probe_linear(i0 + 3, f1, stream)
        if not last_sum:
            return self.h1, f2
        self.add_norm(self.h1, f2, None, None, self.h2, None, stream)
        return self.h2


class DeviceModel:
    """A stack of decoder blocks, a final norm and the LM head on a DeviceWorkload built from
    workloads.decoder_model: the teacher-forced scoring pass of a whole model under the batch's candidate
    table, followed by the estimate and the lazy update of every probed layer."""

    def __init__(self, d):
        self.d = d
        blocks = d.w.meta["blocks"]
        self.blocks = [DeviceBlock(d, blk, 4 * i) for i, blk in enumerate(blocks)]
        gf, bf = d.w.meta["final_norm"]
        up = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(d.device)
        self.gf, self.bf = up(gf), up(bf)
        self.final = torch.empty_like(self.blocks[0].h1)

    def forward(self, stream=None):
        """Every residual sum is fused into the norm that follows it: a block hands its two terms on."""
        x, res = self.d.X, None
        for blk in self.blocks:
            x, res = blk.forward(x, stream, res, last_sum=False)
        self.blocks[-1].add_norm(x, res, self.gf, self.bf, None, self.final, stream)
        self.d.score(self.final, stream)
        return self.final

    def step(self, lr=1e-7, update=True, stream=None):
        d = self.d
        self.forward(stream)
        d.estimate(stream)
        if update:
            d.bank_update_all(lr, np.arange(d.batch.K, dtype=np.int32) * d.w.r, 0, stream=stream)

    def capture(self, lr=1e-7, update=True):
        """Captures one step (scoring pass, estimate, updates) into a HIP graph after one eager warm-up
        step on a side stream, which configures the kernels; nothing in a step depends on the host.
        The warm-up step is a real step: with update it moves the banks."""
        side = torch.cuda.Stream(device=self.d.device)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step(lr, update, stream=side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.step(lr, update, stream=torch.cuda.current_stream())
        return self.graph

    def replay(self):
        self.graph.replay()


class LoopDriver:
    """The multi-step loop of Sec. 3.2 on one DeviceWorkload: per step, the device-resident schedule
    draws the seeds (U fresh every step, V once per interval of `nu` steps) and names the bank block,
    then probe linears, scoring, estimate and the scheduled bank update of every layer follow on one
    stream.  Nothing in a step depends on the host, so one captured HIP graph replays every step.

    The banks of all layers must hold n_blocks * K * r columns; reset() zeroes them."""

    def __init__(self, d, nu, n_blocks, lr, base_u, base_v):
        self.d, self.nu, self.n_blocks, self.lr = d, int(nu), int(n_blocks), float(lr)
        self.base_u, self.base_v = int(base_u), int(base_v)
        b = d.batch
        dev = d.device
        self.sched = torch.zeros(4, dtype=torch.int64, device=dev)          # one zo_sched (32 bytes)
        self.seed_u = torch.zeros(max(b.K, 1), dtype=torch.int64, device=dev)
        self.seed_v = torch.zeros(max(b.K, 1), dtype=torch.int64, device=dev)
        self.batch = DeviceBatch(b.host["cu"], b.host["seq_cand"], b.host["cand_dir"], b.cand_sign.cpu().numpy(),
                                 np.zeros(b.K, np.uint64), dev, dir_seed_v=np.zeros(b.K, np.uint64))
        # the batch struct points at the schedule's seed buffers
        self.batch.dir_seed, self.batch.dir_seed_v = self.seed_u, self.seed_v
        self.batch.struct = zb.make_batch(b.T, self.batch.cu, self.batch.seq_cand, self.batch.cand_dir,
                                          self.batch.cand_sign, self.seed_u, b.host["cu"], b.host["seq_cand"],
                                          b.host["cand_dir"], n_seqs=b.S, n_cands=b.C, n_dirs=b.K,
                                          dir_seed_v=self.seed_v)
        need = self.n_blocks * b.K * d.w.r
        for l in d.layers:
            if l.bank is None or l.bank.R_cap < need:
                raise ValueError("layer %s: the loop needs a bank of %d columns" % (l.name, need))
            l.bank.R_used = l.bank.R_cap
            need_ws = zb.zo_probe_linear_workspace_bytes(b.T, b.S, b.K, l.m, l.n, d.w.r, l.bank.R_used, _dt(d.dtype))
            if need_ws > d.ws_bytes:
                d.ws_bytes = need_ws
                d.ws = torch.empty(need_ws, device=dev, dtype=torch.uint8)
        self.graph = None

    def reset(self, first_step=0):
        """Zeroes every bank and restarts the schedule at step `first_step`."""
        for l in self.d.layers:
            l.P.zero_()
            l.Vb.zero_()
        self.sched.zero_()
        self.sched[0] = int(first_step)

    def step(self, stream=None):
        d, b = self.d, self.batch
        zb.zo_schedule_step(self.sched, self.nu, self.n_blocks, b.K, self.base_u, self.base_v, self.seed_u,
                            self.seed_v, stream)
        for i in range(len(d.layers)):
            d.probe_linear(i, stream=stream, batch=b)
        d.score(stream=stream, batch=b)
        zb.zo_estimate(b.struct, d.cand_sum, d.cand_cnt, float(d.w.eps), d.w.reduction, d.cand_loss, d.proj_grad,
                       stream)
        for l in d.layers:
            zb.zo_bank_update_scheduled(l.bank, l.m, l.n, d.w.r, b.K, self.seed_u, self.seed_v, l.tensor_id,
                                        d.proj_grad, self.lr, None, self.sched, self.n_blocks, _dt(d.dtype), stream)

    def fold(self, stream=None):
        """Folds every layer's bank into its base weights and empties it (the one place the base is written)."""
        for l in self.d.layers:
            zb.zo_fold_bank(l.bank, l.W, l.W.stride(0), l.m, l.n, _dt(self.d.dtype), stream)

    def capture(self):
        """Captures one step into a HIP graph (after one eager warm-up step, which configures the
        kernels; call reset() afterwards).  replay() then runs a step."""
        side = torch.cuda.Stream(device=self.d.device)
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            self.step(stream=side)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            self.step(stream=torch.cuda.current_stream())
        return self.graph

    def replay(self):
        self.graph.replay()

    def read_sched(self):
        raw = self.sched.cpu().numpy()
        return zb.zo_sched.from_buffer_copy(raw.tobytes())

