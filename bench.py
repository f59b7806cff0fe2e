#!/usr/bin/env python3
"""Benchmark of the FedAttn attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: the attention of
all M Transformer blocks of a workload, block after block (one launch per block, as the
blocks of a model depend on each other), local blocks attending inside each participant's
segment (fedattn_prefill) and every H-th block running Phase II from the participants' own
K/V (fedattn_prefill_sync_local_kv: aggregation + global attention; the participants'
matrices lie back to back in HBM, so the aggregated matrix is read in place).  Inputs are
resident in HBM before the timed region; a step's launches are replayed from a HIP graph
(checked against the eager step first), so the timed region measures the GPU, not Python.

Legs (each with its own `roofline` object):
  cfg3        heterogeneous prefill, N = 8 uneven segments, the H sweep {1, 4, 8, 32} of the
              configuration in one step (4 x 32 launches); also reported per H.  HEADLINE:
              the largest single-GPU workload.
  cfg5        sparse-sync prefill, 16 x 4096 tokens, a quarter of the 64-token chunks exchanged.
  cfg2        Llama-3-8B shape, 4 x 512 tokens (the smallest bf16 workload; launch-dominated).
  decode      cfg4: 16 participants, 256 decoding steps x 32 blocks, every step replayed from
              its own graph (the cache lengths grow step by step), GB/s over the whole run.
  peaks       what this machine reaches on the bare resources (a streaming read of a block-step's size,
              an MFMA-only loop), so that every roofline also carries a fraction of a measured peak.

Prints ONE JSON line.  `value` is useful attention TFLOP/s of the headline workload
(4*D*Hq*visible pairs; masked pairs and softmax not counted).  `roofline` is for the
dominant kernel of the headline (the MFMA prefill kernel); `decode.roofline` for the
streaming decode kernels; `cpu_baseline` is the fp64 oracle timed on this machine's host
cores on a bounded sample of the headline workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import fedattn_inputs as fi  # noqa: E402
import paper_2511_02647_amd as fa  # noqa: E402
from paper_2511_02647_amd.planning import cost_report  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# Figures that only a profiler run can give (hardware counters), copied from the rocprofv3
# summaries under profiles/ (each summary names the command that produced it; the CPU test
# tests/test_bench_constants.py checks that the numbers here are the ones in those files).
#   traffic_bytes  HBM bytes per launch, FETCH_SIZE + WRITE_SIZE scaled by the same counters'
#                  reading for a plain copy kernel of known size (aggregate_kv_kernel)
#   mfma_util      SQ_VALU_MFMA_BUSY_CYCLES / (4 SIMDs x SQ_BUSY_CU_CYCLES): share of the cycles a
#                  busy CU's matrix pipes were busy
PMC = {
    "cfg3": {"source": "profiles/hbm_traffic_pmc.txt, profiles/prefill_pmc_counters.txt", "traffic_bytes": 551348019, "mfma_util": 0.573},
    "cfg3_H4": {"source": "profiles/hbm_traffic_pmc.txt, profiles/prefill_pmc_counters.txt", "traffic_bytes": 499010453, "mfma_util": 0.563},
    "cfg5": {"source": "profiles/hbm_traffic_pmc.txt, profiles/prefill_pmc_counters.txt", "traffic_bytes": 1165607648, "mfma_util": 0.517},
    "cfg2": {"source": "profiles/hbm_traffic_pmc.txt, profiles/prefill_pmc_counters.txt", "traffic_bytes": 42180837, "mfma_util": 0.289},
    "decode": {"source": "profiles/hbm_traffic_pmc.txt", "traffic_bytes": 82282004},
}

CFG3_SWEEP = (1, 4, 8, 32)


def log(msg: str) -> None:
    print("[bench] " + msg, file=sys.stderr, flush=True)


def to_dev_bf16(x: np.ndarray) -> torch.Tensor:
    bits = fi.bf16_bits(x).view(np.int16)
    return torch.from_numpy(bits).to("cuda").view(torch.bfloat16)


def visible_pairs(seg: np.ndarray, is_sync: bool, keep_tok=None) -> int:
    """Number of (query, key) pairs a causal block evaluates usefully (per head)."""
    lens = np.diff(seg).astype(np.int64)
    own = int((lens * (lens + 1) // 2).sum())
    if not is_sync:
        return own
    if keep_tok is None:
        L = int(seg[-1])
        return L * (L + 1) // 2
    kept_before = np.concatenate([[0], np.cumsum(keep_tok.astype(np.int64))])
    remote = sum(int(lens[n]) * int(kept_before[seg[n]]) for n in range(len(lens)))
    return own + remote


def keep_tokens(flags: np.ndarray, seg: np.ndarray, chunk_tokens: int) -> np.ndarray:
    """Per-token keep flags from per-chunk flags (for the useful-FLOP count only)."""
    out = np.zeros(int(seg[-1]), dtype=np.uint8)
    c = 0
    for n in range(len(seg) - 1):
        for t in range(int(seg[n]), int(seg[n + 1]), chunk_tokens):
            out[t:min(t + chunk_tokens, int(seg[n + 1]))] = flags[c]
            c += 1
    return out


DEVICE_WARMUP_S = 0.3


def device_warmup(fn, seconds: float = DEVICE_WARMUP_S) -> None:
    """Untimed work before a measurement: the GPU raises its clock over the first tenths of a
    second of sustained load, and a throughput figure should be the sustained one."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            fn()
        torch.cuda.synchronize()


def timed_replays(fns, steps: int, warmup: int):
    """`fns`: the graph replays that make up one step, in order.  Runs `warmup` untimed steps,
    then exactly `steps` timed ones between two synchronisations; every replay is also bracketed
    by HIP events on the stream it is launched on.  Returns (wall seconds per step,
    ms[steps][len(fns)] by events)."""
    def one():
        for f in fns:
            f()
    device_warmup(one)
    for _ in range(warmup):
        one()
    evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in fns]
           for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        for i, f in enumerate(fns):
            evs[s][i][0].record()
            f()
            evs[s][i][1].record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps
    ms = np.array([[a.elapsed_time(b) for a, b in row] for row in evs])
    return wall, ms


def capture(fn, check_tensor: torch.Tensor):
    """`fn`'s launches captured into a HIP graph; two replays are compared with the eager run."""
    check_tensor.zero_()
    fn()
    torch.cuda.synchronize()
    ref = check_tensor.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.synchronize()
    for rep in range(2):
        check_tensor.zero_()
        graph.replay()
        torch.cuda.synchronize()
        if not torch.equal(check_tensor, ref):
            raise RuntimeError("graph replay %d differs from the eager run" % rep)
    return graph


class PrefillBench:
    """Resident inputs of one prefill workload and the launches of a step at a given H."""

    def __init__(self, name: str, n_data_blocks: int | None = None):
        self.w = fi.workload(name)
        w = self.w
        self.seg = w.seg_offsets
        self.M = w.n_blocks
        nd = self.M if n_data_blocks is None else min(n_data_blocks, self.M)
        self.nd = nd
        t0 = time.time()
        with ThreadPoolExecutor(max_workers=8) as ex:
            blocks = list(ex.map(lambda b: fi.prefill_block(w, b), range(nd)))
        self.q = torch.stack([to_dev_bf16(b[0]) for b in blocks])
        self.k = torch.stack([to_dev_bf16(b[1]) for b in blocks])
        self.v = torch.stack([to_dev_bf16(b[2]) for b in blocks])
        del blocks
        self.out = torch.empty_like(self.q)
        self.keep = None
        self.ws = None
        self.keep_tok = None
        self.p = {}
        if w.chunk_tokens:
            rounds = max(1, self.M // max(w.sync_interval, 1))
            flags = [fi.keep_chunks(w, t) for t in range(rounds)]
            self.keep = [torch.from_numpy(f).to("cuda") for f in flags]
            self.keep_tok = [keep_tokens(f, self.seg, w.chunk_tokens) for f in flags]
            nbytes = fa.fedattn_workspace_bytes(self.params(w.sync_interval), fa.FEDATTN_OP_PREFILL, w.total_tokens,
                                                w.chunk_tokens)
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        log("%s: %d blocks (%d distinct input blocks resident, %.2f GB), inputs ready in %.1f s"
            % (name, self.M, nd, (2 * self.q.numel() + 2 * self.k.numel()) * 2 / 1e9, time.time() - t0))

    def params(self, H: int):
        w = self.w
        if H not in self.p:
            self.p[H] = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, H, torch.bfloat16)
        return self.p[H]

    def sync_flags(self, H: int):
        return [fa.fedattn_is_sync_block(H, b) for b in range(self.M)]

    def flops_blocks(self, H: int):
        w = self.w
        fl = 4 * w.head_dim * w.n_q_heads
        out = []
        for b, s in enumerate(self.sync_flags(H)):
            kt = self.keep_tok[(b // H) % len(self.keep_tok)] if (s and self.keep_tok is not None) else None
            out.append(float(fl * visible_pairs(self.seg, s, kt)))
        return out

    def run_block(self, H: int, b: int):
        d = b % self.nd
        p = self.params(H)
        seg, n = self.seg, self.w.n_participants
        if fa.fedattn_is_sync_block(H, b):
            # Phase II from the participants' own matrices (views of one tensor: back to back)
            kl = [self.k[d][seg[i]:seg[i + 1]] for i in range(n)]
            vl = [self.v[d][seg[i]:seg[i + 1]] for i in range(n)]
            kc = self.keep[(b // H) % len(self.keep)] if self.keep is not None else None
            fa.fedattn_prefill_sync_local_kv(p, self.q[d], kl, vl, self.out[d], seg, keep_chunks=kc,
                                             chunk_tokens=self.w.chunk_tokens if kc is not None else 0, workspace=self.ws)
        else:
            fa.fedattn_prefill(p, b, self.q[d], self.k[d], self.v[d], self.out[d], seg)

    def step(self, H: int, only=None):
        """All M blocks (only = None), or the local (False) / sync (True) ones alone."""
        for b, s in enumerate(self.sync_flags(H)):
            if only is None or only == s:
                self.run_block(H, b)

    def batched_upper_bound(self, H: int, steps: int):
        """All M blocks in one fedattn_prefill_blocks launch (no dependency between the blocks):
        what the kernel does when launch gaps and partly filled grids are taken away."""
        if self.nd != self.M or self.keep is not None:
            return None
        run = lambda: fa.fedattn_prefill_blocks(self.params(H), 0, self.M, self.q, self.k, self.v, self.out,
                                                self.q[0].numel(), self.k[0].numel(), self.seg)
        _, ms = timed_replays([run], steps, 2)
        return float(np.median(ms)) * 1e-3


def prefill_leg(pb: PrefillBench, H: int, ms_step: np.ndarray, pmc_key: str | None, steps_kind: int) -> dict:
    """Leg record for workload pb at sync interval H; ms_step: event times of the step's graph replays."""
    w = pb.w
    sync = pb.sync_flags(H)
    fl = pb.flops_blocks(H)
    fl_step = float(sum(fl))
    med = float(np.median(ms_step))
    tflops = fl_step / (med * 1e-3) / 1e12
    leg = {"workload": w.name, "sync_interval": H, "blocks": pb.M, "sync_blocks": int(sum(sync)),
           "tflop_per_step": fl_step / 1e12, "ms_per_step": med, "ms_min": float(ms_step.min()), "ms_max": float(ms_step.max()),
           "iterations": int(ms_step.size), "value": tflops, "unit": "TFLOP/s", "frac_of_bf16_peak": tflops / PEAK_BF16_TFLOPS}
    pmc = PMC.get(pmc_key or "", {})
    roof = {"bound": "mfma", "achieved": tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": tflops / PEAK_BF16_TFLOPS,
            "traffic": pmc.get("traffic_bytes"), "mfma_util": pmc.get("mfma_util"), "counters_from": pmc.get("source"),
            "kernel": "prefill_mfma_kernel<128, *, true>", "launches_per_step": pb.M,
            "flop_per_launch": fl_step / pb.M, "avg_launch_us": med * 1e3 / pb.M,
            "timing": "HIP events around the graph replay of the step's %d launches on the replay stream, median of %d "
                      "replays, divided by the launches (gaps between graph nodes included: the figure errs low)"
                      % (pb.M, ms_step.size)}
    # the two kinds of block on their own: graphs of the step's local launches and of its sync launches
    for kind, name in ((False, "local"), (True, "sync")):
        idx = [b for b in range(pb.M) if sync[b] == kind]
        if not idx:
            continue
        g = capture(lambda: pb.step(H, only=kind), pb.out)
        _, ms = timed_replays([g.replay], steps_kind, 1)
        us = float(np.median(ms)) * 1e3 / len(idx)
        roof["avg_%s_us" % name] = us
        roof["%s_tflops" % name] = float(np.mean([fl[b] for b in idx])) / (us * 1e-6) / 1e12
        del g
    leg["roofline"] = roof
    return leg


class DecodeBench:
    """cfg4: N participants, one query each per step, all M blocks of a step through
    fedattn_decode_blocks (one host call per step, every block with its own launches)."""

    def __init__(self, name: str = "cfg4_decode"):
        self.w = fi.workload(name)
        w = self.w
        self.M = w.n_blocks
        self.seg = w.seg_offsets
        t0 = time.time()
        with ThreadPoolExecutor(max_workers=8) as ex:
            caches = list(ex.map(lambda b: fi.decode_cache_block(w, b), range(self.M)))
        self.kc = torch.stack([to_dev_bf16(c[0]) for c in caches])
        self.vc = torch.stack([to_dev_bf16(c[1]) for c in caches])
        del caches
        self.nq = 4   # distinct query sets, cycled over the steps
        self.q = torch.stack([torch.stack([to_dev_bf16(fi.decode_query(w, s, b)) for b in range(self.M)])
                              for s in range(self.nq)])
        self.out = torch.empty_like(self.q[0])
        self.p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, w.sync_interval,
                                torch.bfloat16)
        nbytes = fa.fedattn_workspace_bytes(self.p, fa.FEDATTN_OP_DECODE, w.total_tokens)
        self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.ws_fused = None
        self.prompt = 1024
        self.sync = [fa.fedattn_is_sync_block(w.sync_interval, b) for b in range(self.M)]
        torch.cuda.synchronize()
        log("%s: %d blocks, caches resident (%.1f GB), inputs ready in %.1f s"
            % (name, self.M, 2 * self.kc.numel() * 2 / 1e9, time.time() - t0))

    def bytes_block_step(self, step: int) -> float:
        w = self.w
        rows = w.n_participants * (self.prompt + step + 1)
        return float(rows * w.n_kv_heads * w.head_dim * 2 * 2)

    def run_step(self, step: int, sync_override: int = -1, fused: bool = False):
        lens = np.full(self.w.n_participants, self.prompt + step + 1, dtype=np.int32)
        q = self.q[step % self.nq]
        if fused and self.ws_fused is None:   # one workspace slice per block in flight
            one = self.ws.numel()
            self.ws_fused = torch.empty(one + (self.M - 1) * ((one + 255) // 256 * 256), dtype=torch.uint8, device="cuda")
        fa.fedattn_decode_blocks(self.p, 0, self.M, q, self.kc, self.vc, self.out, q[0].numel(), self.kc[0].numel(),
                                 self.seg, lens, sync_override=sync_override,
                                 workspace=self.ws_fused if fused else self.ws, fused=fused)

    def graphs(self, steps, sync_override: int = -1, fused: bool = False):
        return [capture(lambda s=s: self.run_step(s, sync_override, fused), self.out) for s in steps]


def decode_leg(iterations: int, n_steps: int | None = None) -> dict:
    db = DecodeBench()
    w = db.w
    all_steps = list(range(w.decode_steps))
    if n_steps is not None and n_steps < w.decode_steps:   # profiler runs: evenly spread steps of the run
        all_steps = sorted(set(int(s) for s in np.linspace(0, w.decode_steps - 1, n_steps)))
    t0 = time.time()
    graphs = db.graphs(all_steps)
    log("decode: %d step graphs captured and checked in %.1f s" % (len(graphs), time.time() - t0))
    total_bytes = sum(db.bytes_block_step(s) * db.M for s in all_steps)

    def run_all():
        for g in graphs:
            g.replay()
    wall, ms = timed_replays([run_all], iterations, 1)
    med = float(np.median(ms))
    gbs = total_bytes / (med * 1e-3) / 1e9
    n_launch = len(all_steps) * db.M
    # the two kinds of block-step on their own, and the bound without launch effects, on 8 sampled steps
    sample = sorted(set(int(s) for s in np.linspace(0, w.decode_steps - 1, 8)))
    sample_bytes = sum(db.bytes_block_step(s) * db.M for s in sample)
    kinds = {}
    for name, override, fused in (("local", 0, False), ("sync", 1, False), ("blocks_fused", -1, True)):
        gs = db.graphs(sample, override, fused)
        _, m = timed_replays([lambda gs=gs: [g.replay() for g in gs]], max(5, iterations // 2), 1)
        kinds[name] = float(np.median(m))
        del gs
    rate = lambda ms_: float(sample_bytes / (ms_ * 1e-3) / 1e9)
    pmc = PMC["decode"]
    return {"workload": "%s: N = %d, prompt %d, %d decoding steps x %d blocks, H = %d" % (
                w.name, w.n_participants, db.prompt, w.decode_steps, db.M, w.sync_interval),
            "launch": "fedattn_decode_blocks: one host call per decoding step, every block with its own launches; each "
                      "step replayed from its own HIP graph, all %d steps in order per iteration" % len(all_steps),
            "steps_timed": len(all_steps), "blocks": db.M, "iterations": iterations,
            "gbytes_per_run": total_bytes / 1e9, "ms_per_run": med, "ms_per_run_wall": wall * 1e3,
            "ms_per_decode_step": med / len(all_steps), "value": gbs, "unit": "GB/s", "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
            "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "traffic": pmc.get("traffic_bytes"), "counters_from": pmc.get("source"),
                         "kernel": "decode_stream_kernel (+ decode_combine_kernel in sync blocks)",
                         "bytes_per_block_step": total_bytes / n_launch, "avg_block_step_us": med * 1e3 / n_launch,
                         "timing": "HIP events around %d graph replays (all steps of the run), median of %d runs, divided by "
                                   "the block-steps (gaps between launches included)" % (len(all_steps), iterations),
                         "local_GBps": rate(kinds["local"]), "sync_GBps": rate(kinds["sync"]),
                         "avg_local_us": kinds["local"] * 1e3 / (len(sample) * db.M),
                         "avg_sync_us": kinds["sync"] * 1e3 / (len(sample) * db.M),
                         "blocks_fused_GBps": rate(kinds["blocks_fused"]),
                         "kinds_measured_on_steps": sample}}


def measured_peaks() -> dict:
    """What this machine reaches on the bare resources, measured with the library's probe kernels in the
    same run: a streaming read of one decode block-step's size per launch (32 launches over
    distinct buffers per graph replay, like the blocks of a decoding step), contiguous and in
    the decode cache's layout, and an MFMA-only loop."""
    n_launch, per = 32, 75_530_240          # the mean block-step of the decode workload
    stride = (per + (1 << 20) - 1) >> 20 << 20
    buf = torch.zeros(n_launch * stride, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1 << 18, dtype=torch.float32, device="cuda")
    out = {}
    for pattern, name in ((0, "stream_contiguous"), (1, "stream_cache_layout")):
        moved = []

        def run():
            moved.clear()
            for b in range(n_launch):
                moved.append(fa.fedattn_probe_stream(buf[b * stride:b * stride + per], pattern, sink))
        g = capture(run, sink)
        _, ms = timed_replays([g.replay], 20, 2)
        us = float(np.median(ms)) * 1e3 / n_launch
        out[name] = {"GBps": moved[0] / us / 1e3, "bytes_per_launch": moved[0], "us_per_launch": us,
                     "frac_of_published_peak": moved[0] / us / 1e3 / PEAK_HBM_GBS}
        del g
    flops = []
    run = lambda: flops.append(fa.fedattn_probe_mfma(sink, 20000))
    _, ms = timed_replays([run], 5, 1)
    out["mfma_bf16_loop"] = {"TFLOPs": flops[-1] / (float(np.median(ms)) * 1e-3) / 1e12,
                             "frac_of_published_peak": flops[-1] / (float(np.median(ms)) * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    out["how"] = ("fedattn_probe_stream: %d launches of %.1f MB over distinct buffers per graph replay, median of 20 replays; "
                  "fedattn_probe_mfma: v_mfma_f32_32x32x16_bf16 on register operands, two wavefronts per SIMD" % (n_launch, per / 1e6))
    return out


def end_to_end_leg(steps: int) -> dict:
    """The end-to-end configuration: the 8-block mini-Transformer (d_model 2048, feed-forward 5632,
    16/4 heads of 128) through the FedAttn schedule on 16 x 4096 tokens, sparse exchange in the
    sync blocks.  One forward = 8 blocks; GEMMs go to the GEMM library, everything else runs in
    this library's kernels.  Reported beside the headline, not part of it."""
    from paper_2511_02647_amd.block import BlockBuffers, BlockWeights, block_forward
    w = fi.workload("cfg5_sparse_sync")
    d_model, hidden = 2048, 5632
    seg, T = w.seg_offsets, w.total_tokens
    p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, w.sync_interval, torch.bfloat16)
    buf = BlockBuffers(p, T, d_model, hidden, chunk_tokens=w.chunk_tokens)
    weights = []
    for b in range(w.n_blocks):
        wt = fi.block_weights(w, b, d_model, hidden)
        weights.append(BlockWeights(*(to_dev_bf16(wt[k]) for k in ("qkv", "o", "gate_up", "down"))))
    sync = [fa.fedattn_is_sync_block(w.sync_interval, b) for b in range(w.n_blocks)]
    keep = [torch.from_numpy(fi.keep_chunks(w, t)).to("cuda") for t in range(w.n_blocks // w.sync_interval)]
    x0 = torch.from_numpy(fi.hidden_input(w, d_model).astype(np.float32)).to("cuda")
    x = torch.empty_like(x0)

    def forward():
        x.copy_(x0)
        pending = None
        for b in range(w.n_blocks):
            kc = keep[b // w.sync_interval] if sync[b] else None
            pending = block_forward(p, b, x, weights[b], seg, buf, keep_chunks=kc,
                                    chunk_tokens=w.chunk_tokens if kc is not None else 0, pending=pending,
                                    defer_update=True)["pending"]
        fa.fedattn_residual_add(x, pending)

    _, ms = timed_replays([forward], steps, 1)
    sec = float(np.median(ms)) * 1e-3
    fl_attn = 0.0
    for b in range(w.n_blocks):
        kt = keep_tokens(fi.keep_chunks(w, b // w.sync_interval), seg, w.chunk_tokens) if sync[b] else None
        fl_attn += 4.0 * w.head_dim * w.n_q_heads * visible_pairs(seg, sync[b], kt)
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    fl_gemm = w.n_blocks * 2.0 * T * (d_model * (Hq + 2 * Hkv) * D + Hq * D * d_model + d_model * 2 * hidden + hidden * d_model)
    return {"workload": "cfg5 end to end: 8 blocks, d_model 2048, 16 x 4096 tokens, H = 2, 25 % of 64-token chunks exchanged",
            "ms_per_forward": sec * 1e3, "attention_tflop": fl_attn / 1e12, "gemm_tflop": fl_gemm / 1e12,
            "tflops_all": (fl_attn + fl_gemm) / sec / 1e12, "finite": bool(torch.isfinite(x).all().item())}


def cpu_baseline(w, H: int, budget_s: float = 12.0) -> dict:
    """The oracle, as it stands, on a bounded sample of the headline workload."""
    import oracle
    block = 3
    q, k, v = fi.prefill_block(w, block)
    seg = w.seg_offsets
    sync = oracle.is_sync_block(H, block)
    rows, heads = fi.sample_rows(seg, w.n_q_heads, 256, fi.DEFAULT_SEED, salt=77)
    rows, heads = rows[-256:], heads[-256:]

    def pairs(rs):
        owner = np.searchsorted(seg, rs, side="right") - 1
        return int(np.sum(rs + 1 - (0 if sync else seg[owner])))

    t0 = time.perf_counter()
    oracle.attend_rows(q, k, v, seg, rows, heads, is_sync=sync)
    dt = time.perf_counter() - t0
    rate = pairs(rows) / dt
    n_more = int(min(200000, max(256, budget_s * rate / max(1.0, pairs(rows) / len(rows)))))
    # batches of at most 200000 rows (the oracle returns fp64 rows: 0.2 GB a batch) until the budget is used
    dt, n_pairs, n_rows = 0.0, 0, 0
    for i in range(64):
        rows2, heads2 = fi.sample_rows(seg, w.n_q_heads, n_more, fi.DEFAULT_SEED, salt=78 + i)
        rows2, heads2 = rows2[-n_more:], heads2[-n_more:]
        t0 = time.perf_counter()
        oracle.attend_rows(q, k, v, seg, rows2, heads2, is_sync=sync)
        dt += time.perf_counter() - t0
        n_pairs += pairs(rows2)
        n_rows += len(rows2)
        if dt * (i + 2) / (i + 1) > budget_s:   # the next batch would pass the budget
            break
    flops = 4.0 * w.head_dim * n_pairs
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.n_threads(), "kind": "oracle",
            "sample": "%d random (row, head) pairs of block %d (%s at H = %d) of %s, fp64, %.1f s"
                      % (n_rows, block, "sync" if sync else "local", H, w.name, dt)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--legs", default="cfg3,cfg5,cfg2,decode,peaks",
                    help="comma-separated: cfg3 (the H sweep), cfg3_H1|H4|H8|H32 (one H), cfg5, cfg2, decode, peaks (streaming-read and "
                         "MFMA-only rates of this box); copy (a plain "
                         "copy of known size, the yardstick of the HBM-traffic counters)")
    ap.add_argument("--end-to-end", action="store_true",
                    help="also run the 8-block mini-Transformer of the end-to-end configuration (adds ~20 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-iterations", type=int, default=20, help="timed passes over the 256 decoding steps")
    ap.add_argument("--decode-steps", type=int, default=None,
                    help="time this many evenly spread decoding steps instead of all 256 (for profiler runs)")
    ap.add_argument("--data-blocks", type=int, default=None, help="distinct input blocks kept resident (large workloads)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (participants are segments of one batch); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    fa.load()
    legs_req = [x.strip() for x in args.legs.split(",") if x.strip()]
    legs = {}
    headline = None
    cpu = None
    cost = None

    cfg3_hs = []
    for name in legs_req:
        if name == "cfg3":
            cfg3_hs = list(CFG3_SWEEP)
        elif name.startswith("cfg3_H"):
            cfg3_hs.append(int(name[6:]))
    if cfg3_hs:
        pb = PrefillBench("cfg3_hetero_prefill", args.data_blocks or 4)
        graphs = [capture(lambda H=H: pb.step(H), pb.out) for H in cfg3_hs]
        wall, ms = timed_replays([g.replay for g in graphs], args.steps, args.warmup)
        fl_sweep = sum(sum(pb.flops_blocks(H)) for H in cfg3_hs)
        tflops = fl_sweep / wall / 1e12
        n_launch = pb.M * len(cfg3_hs)
        ev_ms = float(np.median(ms.sum(axis=1)))
        log("cfg3 H in %s: %.2f ms per step (events %.2f ms), %.1f useful TFLOP/s" % (cfg3_hs, wall * 1e3, ev_ms, tflops))
        for i, H in enumerate(cfg3_hs):
            legs["cfg3_H%d" % H] = prefill_leg(pb, H, ms[:, i], "cfg3_H%d" % H, max(3, args.steps // 4))
            log("  cfg3 H=%d: %.2f ms, %.1f TFLOP/s (%.1f%% of peak)" % (H, legs["cfg3_H%d" % H]["ms_per_step"],
                legs["cfg3_H%d" % H]["value"], 100 * legs["cfg3_H%d" % H]["frac_of_bf16_peak"]))
        pmc = PMC.get("cfg3" if cfg3_hs == list(CFG3_SWEEP) else "cfg3_H%d" % cfg3_hs[0], {})
        achieved = fl_sweep / (ev_ms * 1e-3) / 1e12
        headline = {
            "value": tflops, "ms_per_step": wall * 1e3,
            "config": {"workload": "cfg3_hetero_prefill: N = 8 participants, segment lengths %s (U[1024, 3072] from the seed), "
                                   "M = 32 blocks, 32/8 heads of 128, bf16; one step = the configuration's sweep H in %s, "
                                   "%d launches" % (list(pb.w.seg_lens), cfg3_hs, n_launch),
                       "participants": pb.w.n_participants, "seg_lens": [int(x) for x in pb.w.seg_lens], "blocks": pb.M,
                       "sync_intervals": cfg3_hs, "q_heads": pb.w.n_q_heads, "kv_heads": pb.w.n_kv_heads,
                       "head_dim": pb.w.head_dim, "tflop_per_step": fl_sweep / 1e12,
                       "launch": "one launch per block: fedattn_prefill (local blocks), fedattn_prefill_sync_local_kv (sync "
                                 "blocks, K/V read in place); each H's 32 launches replayed from a HIP graph",
                       "distinct_input_blocks": pb.nd, "untimed_device_warmup_s": DEVICE_WARMUP_S},
            "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                         "frac": achieved / PEAK_BF16_TFLOPS, "traffic": pmc.get("traffic_bytes"),
                         "mfma_util": pmc.get("mfma_util"), "counters_from": pmc.get("source"),
                         "kernel": "prefill_mfma_kernel<128, 1, true>", "launches_per_step": n_launch,
                         "flop_per_launch": fl_sweep / n_launch, "avg_launch_us": ev_ms * 1e3 / n_launch,
                         "timing": "HIP events around every graph replay of the timed steps on the replay stream, median over "
                                   "%d steps of the step's total, divided by its %d launches" % (args.steps, n_launch)}}
        Hc = 4 if 4 in cfg3_hs else cfg3_hs[0]
        cost = cost_report(pb.w.seg_lens, pb.sync_flags(Hc), pb.w.n_q_heads, pb.w.n_kv_heads, pb.w.head_dim).as_dict()
        cost["sync_interval"] = Hc
        if not args.no_cpu_baseline:
            cpu = cpu_baseline(pb.w, Hc)
            log("cpu oracle: %.5f TFLOP/s on %d threads" % (cpu["value"], cpu["cores"]))
        del graphs, pb
        torch.cuda.empty_cache()

    for name, wl, nd, steps, pmc_key in (("cfg5", "cfg5_sparse_sync", args.data_blocks or 4, args.steps, "cfg5"),
                                         ("cfg2", "cfg2_llama8b_prefill", None, max(args.steps, 100), "cfg2")):
        if name not in legs_req:
            continue
        pb = PrefillBench(wl, nd)
        H = pb.w.sync_interval
        g = capture(lambda: pb.step(H), pb.out)
        wall, ms = timed_replays([g.replay], steps, args.warmup)
        legs[name] = prefill_leg(pb, H, ms[:, 0], pmc_key, max(3, steps // 4))
        if name == "cfg2":
            b = pb.batched_upper_bound(H, 10)
            if b is not None:
                legs[name]["roofline"]["blocks_batched_ms"] = b * 1e3
                legs[name]["roofline"]["blocks_batched_tflops"] = sum(pb.flops_blocks(H)) / b / 1e12
        log("%s: %.3f ms per step, %.1f TFLOP/s (%.1f%% of peak)" % (name, legs[name]["ms_per_step"], legs[name]["value"],
                                                                     100 * legs[name]["frac_of_bf16_peak"]))
        if headline is None:
            headline = {"value": legs[name]["value"], "ms_per_step": wall * 1e3,
                        "config": {"workload": wl, "sync_interval": H}, "roofline": legs[name]["roofline"]}
            if not args.no_cpu_baseline and cpu is None:
                cpu = cpu_baseline(pb.w, H)
        del g, pb
        torch.cuda.empty_cache()

    if "copy" in legs_req:
        # a plain copy of known size (fedattn_aggregate_kv from separate allocations), the yardstick the
        # FETCH_SIZE / WRITE_SIZE counters of the other legs are scaled by; not part of a default run
        w = fi.workload("cfg3_hetero_prefill")
        p3 = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, 4, torch.bfloat16)
        seg = w.seg_offsets
        kl = [torch.randn(int(seg[i + 1] - seg[i]), w.n_kv_heads, w.head_dim, device="cuda").to(torch.bfloat16)
              for i in range(w.n_participants)]
        vl = [t.clone() for t in kl]
        kg = torch.empty(w.total_tokens, w.n_kv_heads, w.head_dim, dtype=torch.bfloat16, device="cuda")
        vg = torch.empty_like(kg)
        run = lambda: fa.fedattn_aggregate_kv(p3, kl, vl, seg, kg, vg)
        _, ms = timed_replays([run], args.steps, args.warmup)
        nbytes = 2 * kg.numel() * 2
        legs["copy"] = {"kernel": "aggregate_kv_kernel", "bytes_read": nbytes, "bytes_written": nbytes,
                        "us": float(np.median(ms)) * 1e3, "GBps": 2 * nbytes / (float(np.median(ms)) * 1e-3) / 1e9}
        log("copy: %d bytes in, %d bytes out, %.1f us" % (nbytes, nbytes, legs["copy"]["us"]))
        if headline is None:
            headline = {"value": legs["copy"]["GBps"], "ms_per_step": legs["copy"]["us"] * 1e-3, "unit": "GB/s",
                        "config": {"workload": "copy calibration"}, "roofline": None}

    decode = None
    if "decode" in legs_req:
        decode = decode_leg(args.decode_iterations, args.decode_steps)
        log("decode: %.0f GB/s over %d steps x %d blocks (%.1f%% of HBM peak; local block-steps %.0f, sync %.0f, "
            "blocks sharing launches %.0f GB/s)" % (decode["value"], decode["steps_timed"], decode["blocks"],
            100 * decode["frac_of_hbm_peak"], decode["roofline"]["local_GBps"], decode["roofline"]["sync_GBps"],
            decode["roofline"]["blocks_fused_GBps"]))
        torch.cuda.empty_cache()

    peaks = None
    if "peaks" in legs_req:
        peaks = measured_peaks()
        log("measured on this box: streaming read %.0f GB/s contiguous, %.0f GB/s in the decode cache's layout (%.1f MB per "
            "launch); MFMA-only loop %.0f TFLOP/s" % (peaks["stream_contiguous"]["GBps"], peaks["stream_cache_layout"]["GBps"],
                                                       peaks["stream_contiguous"]["bytes_per_launch"] / 1e6,
                                                       peaks["mfma_bf16_loop"]["TFLOPs"]))
        if decode is not None:
            decode["roofline"]["frac_of_measured_stream_in_cache_layout"] = decode["value"] / peaks["stream_cache_layout"]["GBps"]
        for leg in legs.values():
            if isinstance(leg, dict) and leg.get("roofline") and leg["roofline"].get("bound") == "mfma":
                leg["roofline"]["frac_of_measured_mfma_loop"] = leg["value"] / peaks["mfma_bf16_loop"]["TFLOPs"]
        if headline is not None and headline.get("roofline") and headline["roofline"].get("bound") == "mfma":
            headline["roofline"]["frac_of_measured_mfma_loop"] = headline["value"] / peaks["mfma_bf16_loop"]["TFLOPs"]
        torch.cuda.empty_cache()

    if headline is None and decode is not None:
        headline = {"value": decode["value"], "ms_per_step": decode["ms_per_run"], "config": {"workload": decode["workload"]},
                    "roofline": decode["roofline"], "unit": "GB/s"}
    if headline is None:
        print("bench.py: no leg selected", file=sys.stderr)
        return 2

    result = {"metric": "prefill attn TFLOP/s (% bf16 MFMA peak); decode HBM GB/s (% peak)",
              "value": headline["value"], "unit": headline.get("unit", "TFLOP/s"), "n_gpus": 1, "steps": args.steps,
              "warmup": args.warmup, "ms_per_step": headline["ms_per_step"], "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": headline["config"],
              "frac_of_bf16_peak": headline["value"] / PEAK_BF16_TFLOPS if headline.get("unit", "TFLOP/s") == "TFLOP/s" else None,
              "roofline": headline["roofline"], "legs": legs}
    if decode is not None:
        result["decode"] = decode
    if peaks is not None:
        result["measured_peaks"] = peaks
    if cost is not None:
        result["analytic_cost_per_participant"] = cost
    if cpu is not None:
        result["cpu_baseline"] = cpu
    if args.end_to_end:
        torch.cuda.empty_cache()
        result["end_to_end"] = end_to_end_leg(3)
        log("end to end: %.1f ms per 8-block forward (%.2f TFLOP attention + %.2f TFLOP GEMM -> %.0f TFLOP/s)"
            % (result["end_to_end"]["ms_per_forward"], result["end_to_end"]["attention_tflop"],
               result["end_to_end"]["gemm_tflop"], result["end_to_end"]["tflops_all"]))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
