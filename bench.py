#!/usr/bin/env python3
"""Benchmark of libburstattn on one MI355X.

One "step" is one pass of the whole hot path over one batch: device i's complete simulated ring
-- G forward steps with the fused online-softmax merge, the D = rowsum(dO o O) preprocess, and G
backward steps (dQ_i accumulated locally, dK_j / dV_j produced for every visiting shard) -- at the
real per-device shard shape with every KV shard resident in HBM.  The reported value is
unmasked-FLOP throughput: visible (q, k) pairs x (4 d forward + 10 d backward) / time.

Prints ONE JSON line.  Per-kernel durations are taken inside the timed region with HIP events on
the stream the kernels are launched on (torch's current stream).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA: 256 CU x 4 SIMD x 1024 flop/clk x 2.4 GHz

# HBM bytes per ring step of the dominant kernel from the FETCH_SIZE / WRITE_SIZE counter runs of this
# command (counter sums over the kernel's launches of a ring, divided by its steps, scaled by what the same
# counters read for the 1 GiB copy issued below; at shards beyond 65536 rows a step is several launches of
# the kernel, one per 32768-row range of the streamed axis).  Counters cannot be read from inside the
# process, so the figure is the profiled one: it is reported with the profile it came from and its date,
# and only for the workload that was profiled.
PROFILED_TRAFFIC = {
    2: {"bytes": 1.984e9, "profile": "profiles/bench_config2_pmc_hbm_traffic.md", "taken": "with the kernels and launch plan as committed (pipelined dK/dV, 32768-row ranges)"},
    5: {"bytes": 1.961e11, "profile": "profiles/bench_config5_pmc_hbm_traffic.md", "taken": "with the kernels and launch plan as committed (pipelined dK/dV, 32768-row ranges)"},
}
# --lm-head, default shape: bytes per call over all its launches (profiles/bench_lm_head_kernel_trace_and_counters.md)
PROFILED_LM_HEAD_TRAFFIC_BYTES = 2.73e10


def block_masked_pairs(bm, pos_q, pos_k, R, causal, window):
    """Visible pairs of a step under a local block mask (blocks of R local rows): per open block pair,
    the pairs that the mode and the window leave; a function of the offset between the two blocks' first
    positions, since every local block has the same position pattern (consecutive or G apart)."""
    import numpy as np
    memo, total = {}, 0
    rel_q, rel_k = pos_q[:R] - pos_q[0], pos_k[:R] - pos_k[0]
    for a, b in zip(*np.nonzero(bm)):
        off = int(pos_q[a * R] - pos_k[b * R])
        if off not in memo:
            diff = off + rel_q[:, None] - rel_k[None, :]
            ok = np.ones_like(diff, dtype=bool) if not causal else (diff >= 0) & ((diff < window) if window else True)
            memo[off] = int(ok.sum())
        total += memo[off]
    return total


def cpu_baseline(w, kind, dev_i, shards, sample_rows, seed, window=0, pattern=None, block_rows=0, block_tokens=0):
    """The fp64 oracle, untuned, on a bounded sample of the same workload: `sample_rows` query rows
    (evenly spaced over the chunk) of one (batch, head) against each of the whole KV shards in
    `shards`, forward step + D + backward step per shard.  Returns TFLOPS with the same
    unmasked-FLOP count."""
    import numpy as np
    from oracle import burst_oracle as oc
    from paper_2509_19836_amd import workloads as wl
    G, N, d = w.shards, w.seq, w.head_dim
    pos_fn = {"zigzag": oc.zigzag_positions, "full": oc.contiguous_positions, "causal": oc.contiguous_positions,
              "striped": oc.striped_positions,
              "block_striped": lambda i_, G_, N_: oc.block_striped_positions(i_, G_, N_, block_tokens)}[kind]
    qpos_all = pos_fn(dev_i, G, N)
    sel = np.linspace(0, qpos_all.size - 1, sample_rows).astype(np.int64)
    rng = np.random.Generator(np.random.PCG64(seed))
    draw = lambda n: wl.bf16_bits_to_f64(wl.f32_to_bf16_bits(rng.standard_normal((n, d), dtype=np.float32)))
    Q, dO = draw(sample_rows), draw(sample_rows)
    pairs, dt = 0, 0.0
    for shard_j in shards:
        kpos = pos_fn(shard_j, G, N)
        K, V = draw(kpos.size), draw(kpos.size)
        if pattern is None:
            vis = oc.visibility(qpos_all[sel], kpos, kind != "full", window)
        else:
            R = block_rows // G if kind in ("striped", "block_striped") else block_rows
            bm = wl.local_block_mask(pattern, qpos_all, kpos, R, block_rows)
            vis = oc.apply_block_mask(oc.visibility(qpos_all, kpos, kind != "full", window), bm, R, R)[sel]
        pairs += int(vis.sum())
        t0 = time.perf_counter()
        O, lse = oc.step_fwd(Q, K, V, w.scale, vis)
        D = oc.preprocess_bwd(dO, O)
        oc.step_bwd(Q, K, V, dO, lse, D, w.scale, vis)
        dt += time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": pairs * 14 * d / dt / 1e12, "unit": "TFLOPS", "cores": int(cores), "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": f"{sample_rows} evenly spaced query rows of one (batch, head) against {len(shards)} full "
                      f"{N // G}-row KV shards (device {dev_i} vs shards {list(shards)}, {kind}), forward step "
                      f"+ D + backward step per shard in fp64 numpy; {pairs} visible pairs"}


def lm_head_bench(args):
    """The second kernel family (fused LM head + cross-entropy, Alg. 3) on the per-device share of a
    128K-token sequence over 8 devices with a LLaMA-7B-sized head.  Not the headline metric: run with
    --lm-head.  One step = one burst_lm_head_loss call (forward and backward of every sequence tile)."""
    import numpy as np
    import torch
    from paper_2509_19836_amd import binding as lib, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    N, d, v, B_s = args.lm_tokens, 4096, args.vocab, args.tile_tokens
    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.BASE_SEED + 900)
    h = torch.randn(N, d, device="cuda", generator=gen).to(torch.bfloat16)
    w = (torch.randn(v, d, device="cuda", generator=gen) * (2.0 / d ** 0.5)).to(torch.bfloat16)
    y = torch.randint(0, v, (N,), device="cuda", generator=gen)
    loss = torch.empty(N, device="cuda", dtype=torch.float32)
    dh = torch.empty(N, d, device="cuda", dtype=torch.bfloat16)
    dw = torch.zeros(v, d, device="cuda", dtype=torch.float32)
    shp = lib.lm_head_shape(N, d, v, B_s, 1.0 / N)
    ws = torch.empty(lib.burst_lm_head_workspace_bytes(shp), dtype=torch.uint8, device="cuda")
    full = lambda: lib.burst_lm_head_loss(shp, h, w, y, loss, ws, d_h=dh, d_w=dw, accumulate_dw=True)
    fwd_only = lambda: lib.burst_lm_head_loss(shp, h, w, y, loss, ws)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    def timed(fn, reps):
        a, b = ev(), ev()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps, (time.perf_counter() - t0) / reps * 1e3
    for _ in range(args.warmup):
        full()
    ms, wall_ms = timed(full, args.steps)
    fwd_ms, _ = timed(fwd_only, args.steps)
    # a plain 1 GiB copy: the calibration of the HBM-traffic counters when this command runs under rocprofv3
    src = torch.empty(1 << 28, device="cuda", dtype=torch.float32)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst
    flops = 6.0 * N * d * v
    value = flops / (wall_ms * 1e-3) / 1e12
    out = {
        "metric": "LM head + cross-entropy fwd+bwd TFLOPS (6 N d v)", "value": round(value, 2), "unit": "TFLOPS",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(wall_ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"fused LM head + loss (Alg. 3): {N} tokens (a 128K sequence over 8 devices), d={d}, "
                               f"vocabulary {v}, sequence tiles of {B_s} tokens, dH bf16, dW fp32 accumulated",
                   "workspace_gib": round(ws.numel() / 2 ** 30, 3)},
        "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "forward_only_ms": round(fwd_ms, 3),
        "forward_only_tflops": round(2.0 * N * d * v / (fwd_ms * 1e-3) / 1e12, 2),
        "mean_loss": round(float(loss.mean()), 4),
        # the three GEMM kernels carry all the flops; the call also holds the HBM-bound per-token kernel,
        # so this is a lower bound of what the GEMM kernels reach (per-kernel times: profiles/)
        "roofline": {"bound": "mfma", "kernel": "lm_logits_kernel + lm_dh_kernel + lm_dw_kernel (whole call)",
                     "achieved": round(flops / (ms * 1e-3) / 1e12, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
                     "traffic": PROFILED_LM_HEAD_TRAFFIC_BYTES if (N, v, B_s) == (16384, 32000, 8192) else None},
    }
    if not args.no_cpu_baseline:
        from oracle import lm_head_oracle as lmo
        n_s = 8192
        Hb, Wb, Y = wl.lm_head_tensors(wl.BASE_SEED + 901, n_s, d, v)
        H64, W64 = wl.bf16_bits_to_f64(Hb), wl.bf16_bits_to_f64(Wb)
        t0 = time.perf_counter()
        lmo.lm_head_loss(H64, W64, Y, 1.0 / n_s)
        dt = time.perf_counter() - t0
        try:
            from threadpoolctl import threadpool_info
            cores = max([p_.get("num_threads", 1) for p_ in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        out["cpu_baseline"] = {"value": 6.0 * n_s * d * v / dt / 1e12, "unit": "TFLOPS", "cores": int(cores),
                               "kind": "oracle", "seconds": round(dt, 3),
                               "sample": f"{n_s} tokens against the whole {v}-word head, definition in fp64 numpy"}
    print(json.dumps(out))


class ClockSampler:
    """Shader clock as the kernel driver reports it (the starred level of pp_dpm_sclk in sysfs),
    sampled from a thread while the timed region runs.  None where the file cannot be read."""

    def __init__(self, period_s=0.05):
        import glob
        import threading
        self.paths = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
        self.period, self.samples, self._stop = period_s, [], threading.Event()
        self._thread = threading.Thread(target=self._run, daemon=True)

    def _read(self):
        best = None
        for path in self.paths:
            try:
                for line in open(path).read().splitlines():
                    if line.rstrip().endswith("*"):
                        mhz = int("".join(ch for ch in line.split(":")[1] if ch.isdigit()))
                        best = mhz if best is None else max(best, mhz)
            except (OSError, ValueError, IndexError):
                pass
        return best

    def _run(self):
        while not self._stop.is_set():
            v = self._read()
            if v is not None:
                self.samples.append(v)
            self._stop.wait(self.period)

    def __enter__(self):
        self._thread.start()
        return self

    def __exit__(self, *exc):
        self._stop.set()
        self._thread.join()

    def summary(self):
        if not self.samples:
            return None
        xs = sorted(self.samples)
        return {"source": "pp_dpm_sclk (sysfs), current level", "samples": len(xs), "min": xs[0],
                "median": xs[len(xs) // 2], "max": xs[-1]}


def run_ring(args, config, steps, warmup, sample_clock=False):
    """Device i's whole simulated ring of one workload, `steps` times; returns the measurements."""
    import torch
    from paper_2509_19836_amd import binding as lib, ring, workloads as wl
    w = wl.WORKLOADS[config]
    kind, G, N, i = args.partition or w.mask, w.shards, w.seq, args.device_index % w.shards
    n, d, B, Hq, Hkv = w.shard_tokens, w.head_dim, w.batch, w.q_heads, w.kv_heads

    gen = torch.Generator(device="cuda")
    gen.manual_seed(wl.BASE_SEED + 100 * config)

    def draw(heads):
        x = torch.randn(B, n, heads, d, device="cuda", dtype=torch.float32, generator=gen)
        if w.head_scale:
            x = x * torch.empty(B, 1, heads, 1, device="cuda").uniform_(0.5, 2.0, generator=gen)
        return x.to(torch.bfloat16)

    q_i, do_i = draw(Hq), draw(Hq)
    ks, vs = [draw(Hkv) for _ in range(G)], [draw(Hkv) for _ in range(G)]
    f32 = dict(device="cuda", dtype=torch.float32)
    o_acc = torch.empty(B, n, Hq, d, **f32)
    lse_acc = torch.empty(B, Hq, n, **f32)
    d_i = torch.empty(B, Hq, n, **f32)
    dq = torch.empty(B, n, Hq, d, **f32)
    dks = [torch.empty(B, n, Hkv, d, **f32) for _ in range(G)]
    dvs = [torch.empty(B, n, Hkv, d, **f32) for _ in range(G)]

    order = ring.ring_order(i, G)
    block_tokens = args.block_rows if args.block_density > 0 else args.block_tokens   # N_blk of the block-striped split
    masks = {j: ring.fill_mask(kind, i, j, G, N, args.window, block_tokens) for j in order}
    pairs = {j: lib.burst_attn_visible_pairs(masks[j]) for j in order}
    pattern, block_masks = None, []
    if args.block_density > 0:
        # global blocks of --block-rows tokens; a local row block is a whole global block under the splits that
        # keep consecutive tokens together, slice / stripe i of it (1/G of its rows) under the two balanced splits
        Rg = args.block_rows
        R = Rg // G if kind in ("striped", "block_striped") else Rg
        if R % 256:
            sys.exit(f"bench.py: local row blocks of {R} rows; the kernels need multiples of 256 (raise --block-rows)")
        pattern = wl.block_sparse_pattern(N // Rg, args.block_density, wl.BASE_SEED + 77)
        for j in order:
            pos_q, pos_k = ring.mask_positions(masks[j], "q"), ring.mask_positions(masks[j], "k")
            bm = wl.local_block_mask(pattern, pos_q, pos_k, R, Rg)
            block_masks.append(torch.from_numpy(bm).cuda())   # kept alive for the whole run
            lib.set_block_mask(masks[j], block_masks[-1], R, R)
            pairs[j] = block_masked_pairs(bm, pos_q, pos_k, R, kind != "full", args.window)
    shp = lib.shape(B, Hq, Hkv, d, n, n, w.scale)
    DQ, DKV = lib.BURST_ACC_DQ, lib.BURST_ACC_DK | lib.BURST_ACC_DV
    ev = lambda: torch.cuda.Event(enable_timing=True)
    spans = {"step_fwd": [], "step_bwd_dq": [], "step_bwd_dkdv": [], "preprocess_bwd": []}
    by_kind = {}   # (kernel, kind of ring step) -> durations; kinds: the shard's own chunk, an earlier one, a later one
    kind_of = lambda j: "diag" if j == i else ("j<i" if j < i else "j>i")

    def reset():   # outside the timed region
        o_acc.zero_()
        lse_acc.fill_(-float("inf"))
        dq.zero_()
        for t in dks + dvs:
            t.zero_()

    def one_ring(record):
        marks = []
        def span(name, j, fn):
            if record:
                a, b = ev(), ev()
                a.record(); fn(); b.record()
                marks.append((name, j, a, b))
            else:
                fn()
        for j in order:
            span("step_fwd", j, lambda: lib.burst_attn_step_fwd(shp, masks[j], q_i, ks[j], vs[j], o_acc=o_acc, lse_acc=lse_acc))
        span("preprocess_bwd", None, lambda: lib.burst_attn_preprocess_bwd(shp, o_acc, do_i, d_i))
        for j in order:
            # the two launches burst_attn_step_bwd makes for (dq, dk, dv), bracketed one by one
            span("step_bwd_dq", j, lambda: lib.burst_attn_step_bwd(shp, masks[j], q_i, ks[j], vs[j], do_i, lse_acc, d_i,
                                                                  dq=dq, accumulate_flags=DQ))
            span("step_bwd_dkdv", j, lambda: lib.burst_attn_step_bwd(shp, masks[j], q_i, ks[j], vs[j], do_i, lse_acc, d_i,
                                                                    dk=dks[j], dv=dvs[j], accumulate_flags=DKV))
        return marks

    # The running state and the gradient accumulators are initialised once; later rings keep
    # folding into them ("+=" and merge are the same work whatever the buffers hold).
    reset()
    for _ in range(warmup):
        one_ring(False)
    all_marks = []
    sampler = ClockSampler() if sample_clock else None
    torch.cuda.synchronize()
    if sampler:
        sampler.__enter__()
    t0 = time.perf_counter()
    for _ in range(steps):
        all_marks += one_ring(True)
    torch.cuda.synchronize()
    total_s = time.perf_counter() - t0
    if sampler:
        sampler.__exit__()
    for name, j, a, b in all_marks:
        ms = a.elapsed_time(b)
        spans[name].append(ms)
        if j is not None:
            by_kind.setdefault((name, kind_of(j)), []).append(ms)
    assert torch.isfinite(o_acc).all() and torch.isfinite(dq).all(), "non-finite result"

    # Outside the timed region: the standalone online-softmax merge (bound by HBM: it reads the running
    # O, reads the partial, writes the running O, all fp32), timed on this workload's buffers.
    o_part = torch.zeros(B, n, Hq, d, **f32)
    lse_part = torch.zeros(B, Hq, n, **f32)
    merge = lambda: lib.burst_attn_lse_merge(shp, o_acc, lse_acc, o_part, lse_part)
    merge()
    a, b = ev(), ev()
    a.record()
    for _ in range(5):
        merge()
    b.record()
    torch.cuda.synchronize()
    merge_ms = a.elapsed_time(b) / 5
    merge_bytes = B * n * Hq * (3 * d * 4 + 3 * 4)
    del o_part, lse_part

    ring_pairs = sum(pairs.values()) * B * Hq
    fl_fwd, fl_bwd = ring_pairs * 4 * d, ring_pairs * 10 * d
    ms_ring = total_s / steps * 1e3
    avg = {k: sum(v) / len(v) for k, v in spans.items() if v}
    fwd_ms, bwd_ms = avg["step_fwd"] * G, (avg["step_bwd_dq"] + avg["step_bwd_dkdv"]) * G
    # The kinds of ring step timed separately: TFLOPS of a whole step (fwd + dq + dkdv launches) from the
    # median duration of each launch, with that step's own visible-pair count.
    med = lambda v: sorted(v)[len(v) // 2]
    step_kinds = {}
    for kind_ in ("diag", "j<i", "j>i"):
        js = [j for j in order if kind_of(j) == kind_]
        if not js:
            continue
        f_ms, q_ms, kv_ms = (med(by_kind[(n_, kind_)]) for n_ in ("step_fwd", "step_bwd_dq", "step_bwd_dkdv"))
        step_pairs = pairs[js[0]] * B * Hq
        step_kinds[kind_] = {"steps_per_ring": len(js), "fwd_ms": round(f_ms, 4), "bwd_dq_ms": round(q_ms, 4),
                             "bwd_dkdv_ms": round(kv_ms, 4),
                             "fwd_tflops": round(step_pairs * 4 * d / (f_ms * 1e-3) / 1e12, 1),
                             "bwd_tflops": round(step_pairs * 10 * d / ((q_ms + kv_ms) * 1e-3) / 1e12, 1),
                             "fwd_bwd_tflops": round(step_pairs * 14 * d / ((f_ms + q_ms + kv_ms) * 1e-3) / 1e12, 1)}
    # D = rowsum(dO o O) is bound by HBM: it reads O (fp32) and dO (bf16) once and writes one float per row
    pre_bytes = B * n * Hq * (d * 6 + 4)
    return {
        "workload": w, "kind": kind, "device": i, "order": order, "pattern": pattern, "block_tokens": block_tokens,
        "pairs_per_step": {str(j): pairs[j] for j in order},
        "name": f"{w.name} (config {config}): device {i} of {G}, one full simulated ring = "
                f"{G} fwd steps + D + {G} bwd steps, B={B} Hq={Hq} Hkv={Hkv} d={d}, "
                f"Q chunk {n} x {G} KV chunks of {n}, mask {kind}"
                + (f" (blocks of {block_tokens} tokens)" if kind == "block_striped" else "")
                + (f", window {args.window}" if args.window else "")
                + (f", block-sparse pattern of density {args.block_density} over {args.block_rows}-token blocks"
                   if pattern is not None else ""),
        "value": (fl_fwd + fl_bwd) / (ms_ring * 1e-3) / 1e12, "ms_ring": ms_ring,
        "fwd_tflops": fl_fwd / (fwd_ms * 1e-3) / 1e12, "bwd_tflops": fl_bwd / (bwd_ms * 1e-3) / 1e12,
        "avg": avg, "min": {k: min(v) for k, v in spans.items() if v}, "step_kinds": step_kinds,
        "preprocess_bwd_gb_s": pre_bytes / (avg["preprocess_bwd"] * 1e-3) / 1e9,
        "lse_merge_gb_s": merge_bytes / (merge_ms * 1e-3) / 1e9, "lse_merge_ms": merge_ms,
        "per_launch_pairs": sum(pairs.values()) / G * B * Hq,
        "clock": sampler.summary() if sampler else None,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=5,
                    help="workload index (1-5) of the benchmark definition; 5 = the 128K-token-shard configuration "
                         "the target is stated on (1M tokens over 8 shards), also the largest that one GPU holds")
    ap.add_argument("--device-index", type=int, default=3, help="which simulated device's ring to run")
    ap.add_argument("--cpu-sample-rows", type=int, default=0,
                    help="query rows of the CPU-oracle sample (0: sized so that the sample holds about 5e8 pairs)")
    ap.add_argument("--window", type=int, default=0, help="sliding-window attention: window in tokens (0 = none); "
                                                           "not the headline metric, for the sparse rows")
    ap.add_argument("--partition", default=None, choices=["zigzag", "striped", "block_striped", "causal", "full"],
                    help="override the workload's partition / mask kind (block_striped: slice i of every block of "
                         "--block-tokens tokens, the split of block-wise sparse attention)")
    ap.add_argument("--block-tokens", type=int, default=4096, help="N_blk of --partition block_striped without a block pattern")
    ap.add_argument("--block-density", type=float, default=0.0,
                    help="block-wise sparse attention: fraction of open blocks of a seeded random pattern over "
                         "global token blocks, diagonal always open (0 = no block mask); not the headline metric")
    ap.add_argument("--block-rows", type=int, default=512, help="rows of a (square) block of that pattern")
    ap.add_argument("--cpu-shards", type=int, default=0, help="KV shards the CPU baseline sample covers (0: 2 for shards "
                                                              "of 65536 rows or more, else 4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-config2", action="store_true", help="skip the extra (untimed for the headline) config-2 ring")
    ap.add_argument("--lm-head", action="store_true", help="measure the fused LM head + loss (Alg. 3) instead of the ring")
    ap.add_argument("--lm-tokens", type=int, default=16384)
    ap.add_argument("--vocab", type=int, default=32000, help="--lm-head: vocabulary (32000: LLaMA-1/2, 128256: LLaMA-3)")
    ap.add_argument("--tile-tokens", type=int, default=8192, help="--lm-head: tokens per sequence tile (B_s)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build measures the per-device compute step on ONE GPU; the ring is simulated "
                 "in HBM and there is no multi-GPU path (--gpus must be 1)")

    if args.lm_head:
        return lm_head_bench(args)
    import torch
    from paper_2509_19836_amd import binding as lib, workloads as wl
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    m = run_ring(args, args.config, args.steps, args.warmup, sample_clock=True)
    w, d = m["workload"], m["workload"].head_dim
    torch.cuda.empty_cache()
    # The previous headline workload (config 2, 16384-token shards), so that rounds stay comparable: its own
    # timed rings, after the headline's region and outside it.
    extra = None
    plain = not args.window and not args.partition and m["pattern"] is None
    if args.config != 2 and not args.no_config2 and plain:
        m2 = run_ring(args, 2, 10, 2)
        extra = {"fwd_bwd_tflops": round(m2["value"], 2), "fwd_tflops": round(m2["fwd_tflops"], 2),
                 "bwd_tflops": round(m2["bwd_tflops"], 2), "ms_per_ring": round(m2["ms_ring"], 3), "rings_timed": 10,
                 "kernel_ms": {k: round(v, 4) for k, v in m2["avg"].items()}}
        torch.cuda.empty_cache()

    # Outside the timed region: (1) the matrix-core ceiling of this chip as clocked under load, with
    # constant and with random register operands (real attention tiles are bounded by the latter: the
    # chip lowers its clock when the MFMA inputs toggle); (2) one plain 1 GiB device copy, so that a
    # counter profile of this command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by.
    ev = lambda: torch.cuda.Event(enable_timing=True)
    ceiling = {}
    for name, rnd in (("constant_operands", 0), ("random_operands", 1)):
        lib.burst_attn_mfma_probe(rnd, 20000)
        a, b = ev(), ev()
        a.record()
        flops = lib.burst_attn_mfma_probe(rnd, 200000)
        b.record()
        torch.cuda.synchronize()
        ceiling[name] = flops / (a.elapsed_time(b) * 1e-3) / 1e12
    src = torch.empty(1 << 28, device="cuda", dtype=torch.float32)
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    del src, dst

    # roofline of the dominant kernel (key-stationary dK/dV kernel).  Of the 10 d flop per visible
    # pair of a backward step it is charged 6 d: dV (2 d), dK (2 d) and half of the S and dP GEMMs
    # (2 d) that both backward kernels recompute; the dQ kernel carries the other 4 d.
    avg, value = m["avg"], m["value"]
    dom_flops = m["per_launch_pairs"] * 6 * d
    achieved = dom_flops / (avg["step_bwd_dkdv"] * 1e-3) / 1e12
    profiled = PROFILED_TRAFFIC.get(args.config) if (m["device"] == 3 and plain) else None
    out = {
        "metric": "attention fwd+bwd TFLOPS per ring step (unmasked FLOPs)",
        "value": round(value, 2), "unit": "TFLOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(m["ms_ring"], 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": m["name"], "ring_steps_per_step": w.shards,
                   "ms_per_ring_step": round(m["ms_ring"] / w.shards, 3)},
        "pct_of_bf16_mfma_peak": round(100 * value / PEAK_BF16_TFLOPS, 2),
        "fwd_tflops": round(m["fwd_tflops"], 2),
        "bwd_tflops": round(m["bwd_tflops"], 2),
        "kernel_ms": {k: round(v, 4) for k, v in avg.items()},
        "kernel_ms_min": {k: round(v, 4) for k, v in m["min"].items()},
        "step_kinds": m["step_kinds"],
        "visible_pairs_per_ring_step": m["pairs_per_step"],
        "preprocess_bwd_gb_s": round(m["preprocess_bwd_gb_s"], 1),
        "lse_merge_gb_s": round(m["lse_merge_gb_s"], 1),
        "hbm_peak_gb_s": 8000.0,
        "shader_clock_mhz": m["clock"],
        "mfma_ceiling_tflops": {k: round(v, 1) for k, v in ceiling.items()},
        "pct_of_random_operand_mfma_ceiling": round(100 * value / ceiling["random_operands"], 2),
        "config2_llama7b_zigzag_128k": extra,
        "roofline": {"bound": "mfma", "kernel": "step_bwd_dkdv_kernel", "achieved": round(achieved, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": profiled["bytes"] if profiled else None,
                     "traffic_source": {k: profiled[k] for k in ("profile", "taken")} if profiled else None,
                     "issued_tflops": round(m["per_launch_pairs"] * 8 * d / (avg["step_bwd_dkdv"] * 1e-3) / 1e12, 2)},
    }
    if not args.no_cpu_baseline:
        big = w.shard_tokens >= 65536
        shards = args.cpu_shards or (2 if big else 4)
        rows = args.cpu_sample_rows or max(256, min(w.shard_tokens, int(5.4e8 / (0.5 * shards * w.shard_tokens))))
        order = m["order"]
        out["cpu_baseline"] = cpu_baseline(w, m["kind"], m["device"], order[1:1 + shards] or order[:1], rows,
                                           wl.BASE_SEED + 5, args.window, m["pattern"], args.block_rows, m["block_tokens"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
