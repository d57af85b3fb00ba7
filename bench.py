"""Benchmark of the candidate-evaluation hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch that is
already resident in HBM: probe linears (factor generation, side-down
projection, MFMA GEMM with side state), fused LM-head scoring, two-point
estimate and lazy bank update.  The headline workload is the largest of the
chain configurations that fit one GPU: the mixed foreground + probe batch on
Qwen3-8B shapes (64 sequences of 64-1024 rows, 24 directions x {+,-} of rank
16, 16 foreground sequences, bank rank 128, vocabulary 151936).  The other
two chain configurations (the OPT-13B-shaped scoring chain at batch 64 and
the ragged Qwen3-shaped batch) are timed in the same run and reported as
nested sections, as are the six OPT-13B-shaped linears at 8192 rows.

Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# Bytes per launch of the dominant kernel that crossed the L2 <-> fabric boundary, from the rocprofv3
# --pmc FETCH_SIZE and WRITE_SIZE runs summarised in the named file under profiles/ (FETCH_SIZE scaled by the
# factor 2.000 a plain 1 GiB copy calibrates; WRITE_SIZE factor 1.000).  They are figures of those profile
# runs, not of this run: the line names their source next to them (null for a workload without such a run).
MEASURED_TRAFFIC = {"c3": (1.241e10, "profiles/hbm_bytes_bench_c5_c3.txt"),
                    "c4": (3.730e10, "profiles/hbm_bytes_bench_c5_c3.txt"),
                    "c5": (6.545e10, "profiles/hbm_bytes_bench_c5_c3.txt")}


def _cpu_baseline(w, budget_hint_s=20.0):
    """The oracle as it stands, timed on the host cores over a bounded sample
    (the first 32 sequences of c3, i.e. 16 +/- pairs: about 10 s on the 16 host cores of a GPU machine) of the same workload."""
    import numpy as np
    from oracle import zo_oracle as zo
    from paper_2605_28760_amd import workloads as wl
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        cores = os.cpu_count() or 1
    # about 10-20 s of host work: the full logits of the sample are formed in fp64, so the large-vocabulary
    # workloads take half as many sequences
    n_seq = 32 if w.head.shape[0] < 100000 else 16
    sub = wl.subset_sequences(w, list(range(n_seq)))
    t0 = time.perf_counter()
    out = zo.run_chain(zo.Batch(sub.cu_seqlens, sub.seq_cand, sub.cand_dir, sub.cand_sign, sub.dir_seed),
                       sub.X, sub.layers, sub.head, sub.targets, sub.r, sub.eps, sub.dtype, sub.reduction)
    dt = time.perf_counter() - t0
    return {"value": sub.T / dt, "unit": "candidate-tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d sequences (%d of %d rows) of the same workload, whole chain (dense W_c per candidate, full logits) in fp64 NumPy, %.1f s"
                      % (n_seq, sub.T, w.T, dt)}, out, sub


def _block_section(name, n_rep):
    """Secondary: one decoder block (norm -> fused q/k/v probe linear -> packed causal attention -> output
    probe linear -> residual + norm -> fc1 -> fc2 -> residual) at the model shapes of the main workload,
    timed per stage with events on the launch stream."""
    import numpy as np
    import torch
    from paper_2605_28760_amd import workloads as wl
    from paper_2605_28760_amd.runner import DeviceBlock, DeviceWorkload
    w = wl.BUILDERS[name]()
    d = DeviceWorkload(w, "cuda:0")
    blk = DeviceBlock(d)
    b = w.meta["block"]
    st = torch.cuda.current_stream()
    x = d.X
    stages = [
        ("norm1", lambda: blk.add_norm(x, None, blk.g1, blk.b1, None, blk.a1, st)),
        ("qkv", lambda: d.probe_linear(0, blk.a1, st)),
        ("qk_norm_rope", lambda: blk.qk_norm_rope(d.Y[0], st)),
        ("attention", lambda: blk.attention(d.Y[0], blk.att, st)),
        ("o", lambda: d.probe_linear(1, blk.att, st)),
        ("add_norm2", lambda: blk.add_norm(x, d.Y[1], blk.g2, blk.b2, blk.h1, blk.a2, st)),
        ("fc1", lambda: d.probe_linear(2, blk.a2, st)),
        ("fc2", lambda: d.probe_linear(3, d.Y[2], st)),
        ("residual", lambda: blk.add_norm(blk.h1, d.Y[3], None, None, blk.h2, None, st)),
    ]
    if not b.rope_theta and b.gq is None:
        stages.pop(2)
    def timed(fn):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(n_rep):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_rep
    blk.forward(stream=st)
    torch.cuda.synchronize()
    ms = {nm: timed(fn) for nm, fn in stages}
    block_ms = timed(lambda: blk.forward(stream=st))
    T, hid = w.T, blk.hidden
    lens = np.diff(w.cu_seqlens).astype(np.float64)
    att_flops = 4.0 * b.n_heads * b.head_dim * float((lens * (lens + 1) / 2).sum())   # causal half only
    att_bytes = 2.0 * T * (2 * b.n_heads + 2 * b.n_kv_heads) * b.head_dim              # q, k, v read, o written
    gemm_flops = sum(2.0 * T * l.m * l.n for l in w.layers)
    gemm_ms = ms["qkv"] + ms["o"] + ms["fc1"] + ms["fc2"]
    return {"workload": w.name, "rows": T, "hidden": hid, "heads": [b.n_heads, b.n_kv_heads, b.head_dim],
            "norm": "layer" if b.norm_kind == 0 else "rms", "qk_norm_rope": bool(b.rope_theta), "gated_mlp": b.fc1.act == 2,
            "block_ms": block_ms, "stage_ms": ms,
            "tokens_per_s": T / (block_ms * 1e-3),
            "attention": {"tflops_causal": att_flops / (ms["attention"] * 1e-3) / 1e12,
                          "gbs": att_bytes / (ms["attention"] * 1e-3) / 1e9,
                          "frac_hbm_peak": att_bytes / (ms["attention"] * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "norm_gbs": {"norm1": 2 * 2.0 * T * hid / (ms["norm1"] * 1e-3) / 1e9,
                         "add_norm2": 4 * 2.0 * T * hid / (ms["add_norm2"] * 1e-3) / 1e9,
                         "residual": 3 * 2.0 * T * hid / (ms["residual"] * 1e-3) / 1e9},
            "probe_linears_tflops": gemm_flops / (gemm_ms * 1e-3) / 1e12,
            "share_outside_probe_linears": 1.0 - gemm_ms / sum(ms.values())}


def _layer_set_section(n_rep):
    """Secondary: the six OPT-13B-shaped linears at 16 x 256 x {+,-} = 8192 rows (one direction of rank 8, bank of
    rank 64), each zo_probe_linear call timed alone on its own input, with the candidates and with every
    sequence foreground (the plain GEMM of the same shape)."""
    import numpy as np
    import torch
    from paper_2605_28760_amd import workloads as wl
    from paper_2605_28760_amd.runner import DeviceBatch, DeviceWorkload
    w = wl.BUILDERS["c2"]()
    d = DeviceWorkload(w, "cuda:0")
    st = torch.cuda.current_stream()
    fg = DeviceBatch(w.cu_seqlens, np.full_like(w.seq_cand, -1), w.cand_dir, w.cand_sign, w.dir_seed, "cuda:0")

    def timed(fn):
        for _ in range(5):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(n_rep):
            fn()
        e1.record(st)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_rep
    layers, total_ms, total_flops = {}, 0.0, 0.0
    for _ in range(60):   # the device sat idle while the host built the inputs: let its clocks settle first
        d.probe_linear(0, stream=st)
    for i, l in enumerate(w.layers):
        ms = timed(lambda: d.probe_linear(i, stream=st))
        plain = timed(lambda: d.probe_linear(i, stream=st, batch=fg))
        flops = 2.0 * w.T * l.m * l.n
        layers[l.name] = {"m": l.m, "n": l.n, "ms": ms, "tflops": flops / (ms * 1e-3) / 1e12,
                          "frac_mfma_peak": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, "plain_ms": plain}
        total_ms += ms
        total_flops += flops
    return {"workload": w.name, "rows": w.T, "r": w.r, "bank_rank": int(w.layers[0].R_used), "layers": layers,
            "all_six_ms": total_ms, "tflops": total_flops / (total_ms * 1e-3) / 1e12,
            "frac_mfma_peak": total_flops / (total_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "candidate_tokens_per_s_through_the_six": w.T / (total_ms * 1e-3)}


def _chain(name, steps, warmup, full, block, cpu_baseline):
    """Times one chain workload: `warmup` untimed steps, then `steps` steps bracketed by device
    synchronisation, with per-call HIP events on the launch stream.  `full` adds the secondary
    measurements (plain forward, active-token scoring, loop, 40-layer update, decoder block)."""
    import numpy as np
    import torch
    from paper_2605_28760_amd import binding as zb
    from paper_2605_28760_amd import workloads as wl
    from paper_2605_28760_amd.runner import DeviceBatch, DeviceWorkload, LoopDriver

    t_gen = time.perf_counter()
    w = wl.BUILDERS[name]()
    d = DeviceWorkload(w, "cuda:0")
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t_gen
    stream = torch.cuda.current_stream()
    T = w.T
    vocab, hid = w.head.shape
    # as many directions as the bank has blocks for (c4, c5 probe more directions per step than their banks hold)
    n_upd = min(d.batch.K, int(w.layers[0].R_used) // w.r)
    col0 = np.arange(n_upd, dtype=np.int32) * w.r
    n_layers = len(d.layers)
    names = [l.name for l in d.layers] + ["score", "estimate", "bank_update"]

    def step(events=None):
        def mark(i):
            if events is not None:
                events[i].record(stream)
        mark(0)
        for i in range(n_layers):
            d.probe_linear(i, stream=stream)
            mark(i + 1)
        d.score(stream=stream)
        mark(n_layers + 1)
        d.estimate(stream=stream)
        mark(n_layers + 2)
        if n_upd > 0:
            for i in range(n_layers):
                d.bank_update(i, 1e-7, col0, 0, stream=stream)
        mark(n_layers + 3)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    n_marks = n_layers + 4
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(n_marks)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        step(ev[k])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    seg = np.array([[ev[k][i].elapsed_time(ev[k][i + 1]) for i in range(n_marks - 1)] for k in range(steps)])
    breakdown = {n: float(v) for n, v in zip(names, np.median(seg, axis=0))}   # median over the timed steps
    ms_per_step = elapsed / steps * 1e3
    cand_rows = int(sum(int(w.cu_seqlens[s_ + 1] - w.cu_seqlens[s_]) for s_ in range(len(w.seq_cand)) if w.seq_cand[s_] >= 0))

    # dominant kernel: the fused head GEMM + log-sum-exp (zo_score; its merge kernels are < 1 % of it)
    head_flops = 2.0 * T * hid * vocab
    head_ms = breakdown["score"]
    achieved = head_flops / (head_ms * 1e-3) / 1e12
    traffic, traffic_source = MEASURED_TRAFFIC.get(name, (None, None))
    roofline = {"kernel": "k_head_score (zo_score)", "bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic,
                "traffic_source": traffic_source, "avg_ms": head_ms}
    layer_flops = {l.name: 2.0 * T * l.m * l.n for l in d.layers}
    calls = {n: {"ms": breakdown[n], "tflops": layer_flops[n] / (breakdown[n] * 1e-3) / 1e12,
                 "frac_mfma_peak": layer_flops[n] / (breakdown[n] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
             for n in layer_flops}
    total_flops = head_flops + sum(layer_flops.values())
    probe_ms = sum(breakdown[n] for n in layer_flops)
    out = {
        "value": T * steps / elapsed, "ms_per_step": ms_per_step,
        "config": {"workload": w.name, "rows": T, "sequences": int(len(w.seq_cand)), "candidates": int(len(w.cand_dir)),
                   "directions": int(len(w.dir_seed)), "r": w.r, "eps": w.eps,
                   "layers": [[l.name, l.m, l.n] for l in w.layers], "bank_rank": int(w.layers[0].R_used),
                   "vocab": int(vocab), "hidden": int(hid)},
        "roofline": roofline,
        # rows of sequences that carry a candidate (all rows unless the batch mixes in foreground sequences)
        "candidate_rows": cand_rows, "candidate_rows_per_s": cand_rows * steps / elapsed,
        "chain_tflops": total_flops / (ms_per_step * 1e-3) / 1e12,
        "chain_frac_mfma_peak": total_flops / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "breakdown_ms": breakdown, "breakdown_stat": "median over the timed steps",
        "probe_linear_calls": calls,
        "probe_linears_frac_mfma_peak": sum(layer_flops.values()) / (probe_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "input_setup_s": gen_s,
        # bytes the update step moves (P read + write per layer) against rewriting the dense weights
        # once per candidate state and restoring them (4 x read + write of every probed W)
        "state_transition_bytes": {
            "bank_update": int(sum(2 * l.m * w.r * 4 * n_upd for l in w.layers)),
            "dense_rewrite": int(sum(4 * 2 * l.m * l.n * 2 for l in w.layers))},
    }

    # The same forward with every sequence foreground (candidate id -1: plain base GEMMs and plain scoring),
    # for the probe / plain ratio; outside the timed region.
    fg = DeviceBatch(w.cu_seqlens, np.full_like(w.seq_cand, -1), w.cand_dir, w.cand_sign, w.dir_seed, "cuda:0")

    def forward(batch):
        for i in range(n_layers):
            d.probe_linear(i, stream=stream, batch=batch)
        d.score(stream=stream, batch=batch)

    def timed(fn, n):
        fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(n):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    n_sec = max(3, min(10, steps))
    plain_ms = timed(lambda: forward(fg), n_sec)
    probe_fwd_ms = timed(lambda: forward(None), n_sec)
    # the probe linears alone, with the candidates and all foreground: what the side state costs them
    def linears(batch):
        for i in range(n_layers):
            d.probe_linear(i, stream=stream, batch=batch)
    lin_plain_ms = timed(lambda: linears(fg), n_sec)
    lin_probe_ms = timed(lambda: linears(None), n_sec)
    out["probe_over_plain"] = {"probe_ms": probe_fwd_ms, "plain_ms": plain_ms, "ratio": probe_fwd_ms / plain_ms,
                               "linears_probe_ms": lin_probe_ms, "linears_plain_ms": lin_plain_ms,
                               "linears_ratio": lin_probe_ms / lin_plain_ms}
    # whole step over the same forward with every sequence foreground: the analogue of the paper's
    # native / matched-inference ratio
    out["native_over_matched"] = ms_per_step / plain_ms
    if not full:
        del d
        torch.cuda.empty_cache()
        return out, w

    # Scoring when only the last 16 tokens of every sequence carry a target (answer tokens): the head
    # multiplies only those rows.
    all_targets = d.targets.clone()
    tail = np.full(T, -1, np.int32)
    for s_ in range(len(w.seq_cand)):
        lo = max(int(w.cu_seqlens[s_]), int(w.cu_seqlens[s_ + 1]) - 16)
        tail[lo:w.cu_seqlens[s_ + 1]] = w.targets[lo:w.cu_seqlens[s_ + 1]]
    d.targets.copy_(torch.from_numpy(tail))
    active_ms = timed(lambda: d.score(stream=stream), n_sec)
    d.targets.copy_(all_targets)
    torch.cuda.synchronize()
    out["active_token_scoring"] = {"scored_rows": int((tail >= 0).sum()), "rows": T, "score_ms": active_ms}

    # The lazy update of 40 layers (20 copies of this workload's two layer shapes, one rank-r block per
    # direction, accumulate mode) as one multi-layer call against 40 single-layer calls.
    def bank_update_40():
        shapes = [(l.m, l.n) for l in w.layers] * 20
        R_cap = int(w.layers[0].R_used)
        Ps = [torch.zeros((m, R_cap), device="cuda:0") for m, _ in shapes]
        Vs = [torch.zeros((n, R_cap), device="cuda:0") for _, n in shapes]
        banks = [zb.make_bank(R_cap, R_cap, Ps[i], Vs[i]) for i in range(len(shapes))]
        arr = zb.make_layer_banks([(banks[i], m, n, 2 * i) for i, (m, n) in enumerate(shapes)])
        dt = zb.ZO_BF16

        def multi():
            zb.zo_bank_update_multi(arr, w.r, n_upd, d.batch.dir_seed, None, d.proj_grad, 1e-7, None, col0, 0, dt, stream)

        def single():
            for i, (m, n) in enumerate(shapes):
                zb.zo_bank_update(banks[i], m, n, w.r, n_upd, d.batch.dir_seed, 2 * i, d.proj_grad, 1e-7, None, col0, 0,
                                  dt, stream)
        nbytes = sum(2 * m * w.r * 4 * n_upd for m, _ in shapes)
        t_multi, t_single = timed(multi, n_sec), timed(single, n_sec)
        return {"layers": len(shapes), "bytes": int(nbytes), "multi_ms": t_multi, "per_layer_calls_ms": t_single,
                "multi_gbs": nbytes / (t_multi * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (t_multi * 1e-3) / 1e9 / PEAK_HBM_GBS}
    out["bank_update_40_layers"] = bank_update_40() if n_upd > 0 else None

    # The multi-step loop (device-resident seed / bank-block schedule + the whole step), eager launches
    # against replays of one captured HIP graph.  Run last: it zeroes the banks.
    loop_info = None
    n_blocks = int(w.layers[0].R_used) // (w.r * d.batch.K) if w.layers[0].P is not None else 0
    if n_blocks >= 1:
        loop = LoopDriver(d, nu=4, n_blocks=n_blocks, lr=1e-10, base_u=1, base_v=2)   # small enough for the losses to stay put

        def time_loop(fn, n):
            loop.reset()
            return timed(fn, n)
        eager_ms = time_loop(lambda: loop.step(stream=stream), n_sec)
        loop.capture()
        graph_ms = time_loop(loop.replay, n_sec)
        # fold the (tiny) accumulated bank into the base weights: the price of going past nu * n_blocks steps
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        loop.fold(stream=stream)
        e0.record(stream)
        loop.fold(stream=stream)
        e1.record(stream)
        torch.cuda.synchronize()
        loop_info = {"nu": 4, "n_blocks": n_blocks, "eager_ms_per_step": eager_ms, "graph_ms_per_step": graph_ms,
                     "fold_all_layers_ms": e0.elapsed_time(e1)}
    out["loop"] = loop_info
    del d
    torch.cuda.empty_cache()
    out["block"] = _block_section({"c3": "b3"}.get(name, "b4"), n_sec) if block else None
    if cpu_baseline:
        out["cpu_baseline"], _, _ = _cpu_baseline(w)
    return out, w


def _operand_data_section(n_rep=10):
    """The head kernel (zo_score, all rows foreground) on the OPT-13B and Qwen3-8B head shapes with operands of
    different content: the same launch, addresses and traffic, so a difference in time is the chip's clock
    answering the switching activity of the data (a power-limited kernel), not the kernel's schedule.  Beside
    it, as context on the same box and data, the vendor library's plain GEMM of the same contraction
    (torch.matmul, which also writes the T x V logits that the head kernel never materialises)."""
    import torch
    from paper_2605_28760_amd import binding as zb
    dev = "cuda:0"
    st = torch.cuda.current_stream()

    def avg_ms(fn):
        for _ in range(3): fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(n_rep): fn()
        e1.record(st); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n_rep

    out = {}
    for key, (T, d, V) in (("c3_head", (16384, 5120, 50272)), ("c5_head", (33451, 4096, 151936))):
        cu = torch.tensor([0, T], dtype=torch.int32, device=dev)
        fg = torch.tensor([-1], dtype=torch.int32, device=dev)
        b = zb.make_batch(T, cu, fg, fg, fg, fg, n_seqs=1, n_cands=0, n_dirs=0)
        g = torch.Generator(device=dev); g.manual_seed(7)
        tg = torch.randint(0, V, (T,), device=dev, dtype=torch.int32, generator=g)
        wsb = zb.zo_score_workspace_bytes(T, 1, V, d, zb.ZO_BF16)
        ws = torch.empty(wsb + 256, dtype=torch.uint8, device=dev)
        tok = torch.empty(T, device=dev); seq = torch.empty(1, device=dev)
        Hr = torch.randn(T, d, device=dev, generator=g).to(torch.bfloat16)
        Wr = (torch.randn(V, d, device=dev, generator=g) * d ** -0.5).to(torch.bfloat16)
        Hz, Wz = torch.zeros_like(Hr), torch.zeros_like(Wr)
        logits = torch.empty(T, V, dtype=torch.bfloat16, device=dev)
        flop = 2.0 * T * V * d
        sec = {"shape": [T, d, V]}
        for name, (H, W) in (("random", (Hr, Wr)), ("zeros", (Hz, Wz)), ("random_tokens_zero_weights", (Hr, Wz)),
                             ("random_again", (Hr, Wr))):
            ms = avg_ms(lambda: zb.zo_score(b, H, d, W, d, V, d, zb.ZO_BF16, tg, tok, seq, None, None, ws, wsb, st))
            sec[name] = {"ms": ms, "tflops": flop / ms / 1e9}
        for name, (H, W) in (("library_gemm_random", (Hr, Wr)), ("library_gemm_zeros", (Hz, Wz))):
            ms = avg_ms(lambda: torch.matmul(H, W.t(), out=logits))
            sec[name] = {"ms": ms, "tflops": flop / ms / 1e9}
        out[key] = sec
        del Hr, Wr, Hz, Wz, logits, ws
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c5", choices=["c3", "c4", "c5"],
                    help="the workload of the headline line (default: the largest chain configuration)")
    ap.add_argument("--nested", default="c3,c4",
                    help="comma-separated chain workloads also timed and reported as nested sections ('' for none)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-block", action="store_true", help="skip the decoder-block secondary measurement")
    ap.add_argument("--no-layer-set", action="store_true",
                    help="skip the secondary measurement of the six OPT-13B-shaped linears at 8192 rows")
    ap.add_argument("--operand-data", action="store_true",
                    help="also time the head kernel, and the library GEMM of the same contraction, on random, zero and half-zero "
                         "operands (is the clock power-bound?)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size kernel for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by sequences, one replica per GPU); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_28760_amd import binding as zb

    zb.lib()   # fails loudly if the HIP library is missing
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    main_res, _ = _chain(args.workload, args.steps, args.warmup, True, not args.no_block, not args.no_cpu_baseline)
    nested = {}
    for nm in [x for x in args.nested.split(",") if x and x != args.workload]:
        n_steps = max(5, min(args.steps, 30))
        res, _ = _chain(nm, n_steps, min(args.warmup, 5), False, False, False)
        res["steps"], res["warmup"] = n_steps, min(args.warmup, 5)
        nested[nm] = res
    layer_set_info = None if args.no_layer_set else _layer_set_section(max(3, min(30, args.steps)))

    result = {
        "metric": "candidate-tokens scored/sec (probe linear + LM-head scoring)",
        "value": main_res.pop("value"), "unit": "candidate-tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": main_res.pop("config"), "roofline": main_res.pop("roofline"),
    }
    cpu = main_res.pop("cpu_baseline", None)
    result.update(main_res)
    result["nested_workloads"] = nested
    result["layer_set"] = layer_set_info
    if args.operand_data:
        result["head_operand_data"] = _operand_data_section()
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result))


if __name__ == "__main__":
    main()
