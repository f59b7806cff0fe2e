#!/usr/bin/env python3
"""Benchmark of the FedAttn attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: the
attention of all M Transformer blocks of the workload, block after block (one
launch per block, as the blocks of a model depend on each other), local blocks
attending inside each participant's segment and every H-th block aggregating
the participants' K/V (fedattn_aggregate_kv) and attending over the global KV.
Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is useful attention TFLOP/s of the headline
prefill workload (4*D*Hq*visible pairs; masked pairs and softmax not counted).
`roofline` is for the dominant kernel (the MFMA prefill kernel), `decode`
carries the split-KV decode kernel's achieved HBM GB/s on the decode workload,
and `cpu_baseline` is the fp64 oracle timed on this machine's host cores on a
bounded sample of the same workload.
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

# HBM bytes per launch (fetched + written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled by the same counters' reading for the plain-copy kernel aggregate_kv_kernel
# (profiles/hbm_traffic_pmc_cfg2_prefill_cfg4_decode.txt).
MEASURED_TRAFFIC_BYTES = {
    "cfg2_llama8b_prefill": (24717 + 16384) * 1024.0,   # prefill_mfma_kernel, per block launch (24 local, 8 sync)
    # decode_stream_kernel (+ decode_combine_kernel in sync blocks), 24 local and 8 sync block-steps per step,
    # mean of the first and the last decoding step
    "cfg4_decode": (0.75 * (74295 + 2204) + 0.25 * (73720 + 8320 + 8781 + 128)) * 1024.0,
}


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


class PrefillBench:
    def __init__(self, name: str, n_data_blocks: int | None = None, H: int | None = None, aggregate: bool = True):
        self.w = fi.workload(name)
        w = self.w
        self.H = w.sync_interval if H is None else H
        self.seg = w.seg_offsets
        self.M = w.n_blocks
        self.aggregate = aggregate
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
        self.kg = torch.empty_like(self.k[0])
        self.vg = torch.empty_like(self.v[0])
        self.p = fa.make_params(w.n_participants, w.n_q_heads, w.n_kv_heads, w.head_dim, self.H, torch.bfloat16)
        self.keep = None
        self.ws = None
        self.keep_tok = None
        if w.chunk_tokens:
            flags = [fi.keep_chunks(w, t) for t in range(max(1, self.M // max(self.H, 1)))]
            self.keep = [torch.from_numpy(f).to("cuda") for f in flags]
            self.keep_tok = [keep_tokens(f, self.seg, w.chunk_tokens) for f in flags]
            nbytes = fa.fedattn_workspace_bytes(self.p, fa.FEDATTN_OP_PREFILL, w.total_tokens, w.chunk_tokens)
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        self.sync = [fa.fedattn_is_sync_block(self.H, b) for b in range(self.M)]
        fl = 4 * w.head_dim * w.n_q_heads
        self.flops_block = []
        for b in range(self.M):
            kt = None
            if self.sync[b] and self.keep_tok is not None:
                kt = self.keep_tok[(b // self.H) % len(self.keep_tok)]
            self.flops_block.append(fl * visible_pairs(self.seg, self.sync[b], kt))
        self.flops_step = float(sum(self.flops_block))
        torch.cuda.synchronize()
        log("%s: %d blocks (%d resident), H=%d, %d sync, %.1f GFLOP/step, inputs ready in %.1f s"
            % (name, self.M, nd, self.H, sum(self.sync), self.flops_step / 1e9, time.time() - t0))

    def local_views(self, d: int):
        seg = self.seg
        n = self.w.n_participants
        return ([self.k[d][seg[i]:seg[i + 1]] for i in range(n)], [self.v[d][seg[i]:seg[i + 1]] for i in range(n)])

    def run_block(self, b: int, ev=None):
        d = b % self.nd
        k, v = self.k[d], self.v[d]
        kc = None
        if self.sync[b]:
            if self.aggregate:
                kl, vl = self.local_views(d)
                fa.fedattn_aggregate_kv(self.p, kl, vl, self.seg, self.kg, self.vg)
                k, v = self.kg, self.vg
            if self.keep is not None:
                kc = self.keep[(b // self.H) % len(self.keep)]
        if ev is not None:
            ev[0].record()
        fa.fedattn_prefill(self.p, b, self.q[d], k, v, self.out[d], self.seg, keep_chunks=kc,
                           chunk_tokens=self.w.chunk_tokens, workspace=self.ws)
        if ev is not None:
            ev[1].record()

    def step(self):
        for b in range(self.M):
            self.run_block(b)

    def batched_upper_bound(self, steps: int):
        """All M blocks in one fedattn_prefill_blocks launch (no dependency between the blocks, no
        aggregation): what the kernel does when launch gaps and partly filled grids are taken away."""
        if self.nd != self.M or self.keep is not None:
            return None
        run = lambda: fa.fedattn_prefill_blocks(self.p, 0, self.M, self.q, self.k, self.v, self.out,
                                                self.q[0].numel(), self.k[0].numel(), self.seg)
        return time_region(run, steps, 2)

    def kernel_times(self, steps: int):
        """Average duration of the prefill kernel per block kind, HIP events around each launch."""
        evs = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                for _ in range(self.M)] for _ in range(steps)]
        device_warmup(self.step)
        # keep the GPU busy while the host enqueues: the launches then run back to back and an
        # event pair brackets the kernel, not the time the GPU waited for the host
        if self.nd == self.M and self.keep is None:
            for _ in range(max(1, steps * self.M // 20)):   # 0.7 ms of GPU work each; the host needs ~20 us per launch
                fa.fedattn_prefill_blocks(self.p, 0, self.M, self.q, self.k, self.v, self.out,
                                          self.q[0].numel(), self.k[0].numel(), self.seg)
        for s in range(steps):
            for b in range(self.M):
                self.run_block(b, evs[s][b])
        torch.cuda.synchronize()
        ms = np.array([[e[0].elapsed_time(e[1]) for e in row] for row in evs])  # [steps, M]
        return ms


class DecodeBench:
    """cfg4: N participants, one query each per step, all M blocks of a step through
    fedattn_decode_blocks (one host call per step, one launch pair per block)."""

    def __init__(self, name: str = "cfg4_decode", n_data_blocks: int | None = None):
        self.w = fi.workload(name)
        w = self.w
        self.M = w.n_blocks
        self.seg = w.seg_offsets
        nd = self.M if n_data_blocks is None else min(n_data_blocks, self.M)
        assert nd == self.M, "decode keeps one cache per block resident"
        t0 = time.time()
        with ThreadPoolExecutor(max_workers=8) as ex:
            caches = list(ex.map(lambda b: fi.decode_cache_block(w, b), range(nd)))
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

    def timed(self, steps, sync_override: int = -1, fused: bool = False) -> float:
        """GPU milliseconds for the given decode steps (HIP events around the whole run)."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        device_warmup(lambda: self.run_step(steps[0], sync_override, fused))
        e0.record()
        for s in steps:
            self.run_step(s, sync_override, fused)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)


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
        for b in range(w.n_blocks):
            kc = keep[b // w.sync_interval] if sync[b] else None
            block_forward(p, b, x, weights[b], seg, buf, keep_chunks=kc, chunk_tokens=w.chunk_tokens if kc is not None else 0)

    sec = time_region(forward, steps, 1)
    fl_attn = 0.0
    for b in range(w.n_blocks):
        kt = keep_tokens(fi.keep_chunks(w, b // w.sync_interval), seg, w.chunk_tokens) if sync[b] else None
        fl_attn += 4.0 * w.head_dim * w.n_q_heads * visible_pairs(seg, sync[b], kt)
    Hq, Hkv, D = w.n_q_heads, w.n_kv_heads, w.head_dim
    fl_gemm = w.n_blocks * 2.0 * T * (d_model * (Hq + 2 * Hkv) * D + Hq * D * d_model + d_model * 2 * hidden + hidden * d_model)
    return {"workload": "cfg5 end to end: 8 blocks, d_model 2048, 16 x 4096 tokens, H = 2, 25 % of 64-token chunks exchanged",
            "ms_per_forward": sec * 1e3, "attention_tflop": fl_attn / 1e12, "gemm_tflop": fl_gemm / 1e12,
            "tflops_all": (fl_attn + fl_gemm) / sec / 1e12, "finite": bool(torch.isfinite(x).all().item())}


DEVICE_WARMUP_S = 0.3


def device_warmup(fn, seconds: float = DEVICE_WARMUP_S) -> None:
    """Untimed work before a measurement: the GPU raises its clock over the first tenths of a
    second of sustained load (the headline step measured 0.90 ms right after idle and 0.84 ms
    from 0.2 s on), and a throughput figure should be the sustained one."""
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()


def time_region(fn, steps: int, warmup: int) -> float:
    device_warmup(fn)
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def capture_step(pb: "PrefillBench"):
    """One step (every launch of it) captured into a HIP graph, so that the timed region
    measures the GPU and not the Python loop around 40 launches of 20-50 us each.  The replay
    is checked against the eager step before it is used."""
    pb.step()
    torch.cuda.synchronize()
    ref = pb.out.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            pb.step()
    torch.cuda.synchronize()
    for rep in range(2):
        pb.out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        if not torch.equal(pb.out, ref):
            raise RuntimeError("graph replay %d of the step differs from the eager step" % rep)
    return graph


def cpu_baseline(pb: PrefillBench, budget_s: float = 12.0) -> dict:
    """The oracle, as it stands, on a bounded sample of the headline workload."""
    import oracle
    w = pb.w
    q, k, v = fi.prefill_block(w, 3)
    seg = pb.seg
    sync = oracle.is_sync_block(pb.H, 3)
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
            "sample": "%d random (row, head) pairs of block 3 (%s) of %s, fp64, %.1f s"
                      % (n_rows, "sync" if sync else "local", w.name, dt)}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2_llama8b_prefill",
                    choices=["cfg2_llama8b_prefill", "cfg3_hetero_prefill", "cfg5_sparse_sync"])
    ap.add_argument("--sync-interval", type=int, default=None, help="override H of the workload")
    ap.add_argument("--no-aggregate", action="store_true", help="skip fedattn_aggregate_kv in sync blocks")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode measurement")
    ap.add_argument("--no-graph", action="store_true", help="time the step launched from Python, not a graph replay")
    ap.add_argument("--end-to-end", action="store_true",
                    help="also run the 8-block mini-Transformer of the end-to-end configuration (adds ~20 s)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=8, help="decode steps timed (spread over the 256)")
    ap.add_argument("--data-blocks", type=int, default=None, help="distinct input blocks kept resident")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (participants are segments of one batch); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    fa.load()

    nd = args.data_blocks
    if nd is None and args.workload != "cfg2_llama8b_prefill":
        nd = 4   # 336 MB (cfg3) / 0.8 GB (cfg5) of inputs per block: keep a few distinct ones
    pb = PrefillBench(args.workload, nd, args.sync_interval, aggregate=not args.no_aggregate)
    for _ in range(2):
        pb.step()   # first launches set kernel attributes; keep that out of the capture
    sec_eager = time_region(pb.step, args.steps, args.warmup)
    if args.no_graph:
        sec = sec_eager
    else:
        graph = capture_step(pb)
        sec = time_region(graph.replay, args.steps, args.warmup)
    tflops = pb.flops_step / sec / 1e12
    log("%s: %.3f ms/step, %.1f useful TFLOP/s (%s; launched from Python: %.3f ms/step)"
        % (pb.w.name, sec * 1e3, tflops, "eager" if args.no_graph else "HIP graph replay", sec_eager * 1e3))

    # dominant kernel: HIP events around every prefill launch, same steps again
    ms = pb.kernel_times(min(args.steps, 10))
    kern_ms = ms.sum(axis=1).mean()
    achieved = pb.flops_step / (kern_ms * 1e-3) / 1e12
    sync_idx = [b for b in range(pb.M) if pb.sync[b]]
    loc_idx = [b for b in range(pb.M) if not pb.sync[b]]
    roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC_BYTES.get(pb.w.name),
            "kernel": "prefill_mfma_kernel<128>", "launches_per_step": pb.M,
            "avg_launch_us": float(ms.mean() * 1e3),
            "avg_local_us": float(ms[:, loc_idx].mean() * 1e3) if loc_idx else None,
            "avg_sync_us": float(ms[:, sync_idx].mean() * 1e3) if sync_idx else None,
            "local_tflops": (np.mean([pb.flops_block[b] for b in loc_idx]) / (ms[:, loc_idx].mean() * 1e-3) / 1e12)
            if loc_idx else None,
            "sync_tflops": (np.mean([pb.flops_block[b] for b in sync_idx]) / (ms[:, sync_idx].mean() * 1e-3) / 1e12)
            if sync_idx else None}
    log("prefill kernel: avg %.1f us/launch -> %.1f TFLOP/s (%.1f%% of bf16 MFMA peak)"
        % (roof["avg_launch_us"], achieved, 100 * roof["frac"]))

    batched = pb.batched_upper_bound(min(args.steps, 10))
    if batched is not None:
        roof["blocks_batched_tflops"] = pb.flops_step / batched / 1e12
        roof["blocks_batched_ms"] = batched * 1e3
        log("all %d blocks in one launch (upper bound, no block dependencies): %.3f ms, %.1f TFLOP/s"
            % (pb.M, batched * 1e3, roof["blocks_batched_tflops"]))

    # the paper's analytic cost figures for this plan (Section VII-A, evaluation metrics)
    cost = cost_report(pb.w.seg_lens, pb.sync, pb.w.n_q_heads, pb.w.n_kv_heads, pb.w.head_dim,
                       keep_fraction=pb.w.keep_fraction if pb.w.chunk_tokens else 1.0)

    result = {"metric": "prefill attn TFLOP/s (% bf16 MFMA peak); decode HBM GB/s (% peak)",
              "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
              "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
              "dtype": "bf16", "data": "synthetic",
              "config": {"workload": pb.w.name, "participants": pb.w.n_participants,
                         "seg_lens": [int(x) for x in pb.w.seg_lens], "blocks": pb.M, "sync_interval": pb.H,
                         "q_heads": pb.w.n_q_heads, "kv_heads": pb.w.n_kv_heads, "head_dim": pb.w.head_dim,
                         "launch": ("one fedattn_prefill per block, fedattn_aggregate_kv before each sync block"
                                    if pb.aggregate else "one fedattn_prefill per block")
                                   + ("" if args.no_graph else "; the step's launches replayed from a HIP graph"),
                         "ms_per_step_launched_from_python": sec_eager * 1e3,
                         "untimed_device_warmup_s": DEVICE_WARMUP_S},
              "frac_of_bf16_peak": tflops / PEAK_BF16_TFLOPS,
              "roofline": roof,
              "analytic_cost_per_participant": cost.as_dict()}

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(pb)
        log("cpu oracle: %.5f TFLOP/s on %d threads" % (result["cpu_baseline"]["value"], result["cpu_baseline"]["cores"]))
    del pb
    torch.cuda.empty_cache()

    if not args.no_decode:
        db = DecodeBench()
        steps = sorted(set(int(s) for s in np.linspace(0, db.w.decode_steps - 1, args.decode_steps)))
        device_warmup(lambda: db.run_step(steps[0]))
        t0 = time.perf_counter()
        for s in steps:
            db.run_step(s)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        total_bytes = sum(db.bytes_block_step(s) * db.M for s in steps)
        ms_all = db.timed(steps)
        ms_loc = db.timed(steps, 0)     # every block forced local: the local-block kernels alone
        ms_syn = db.timed(steps, 1)     # every block forced sync
        ms_fused = db.timed(steps, -1, fused=True)   # upper bound: the blocks of a kind share launches
        gbs = lambda ms: float(total_bytes / (ms * 1e-3) / 1e9)
        n_launch = len(steps) * db.M
        dec = {"workload": db.w.name, "steps_timed": steps, "blocks": db.M,
               "launch": "fedattn_decode_blocks: one host call per step; local blocks one launch each (chunks merged "
                         "in the streaming kernel), sync blocks a split-KV + combine launch pair",
               "end_to_end_GBps": total_bytes / wall / 1e9,
               "ms_per_decode_step": wall / len(steps) * 1e3,
               "roofline": {"bound": "hbm", "achieved": gbs(ms_all), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": gbs(ms_all) / PEAK_HBM_GBS, "traffic": MEASURED_TRAFFIC_BYTES.get(db.w.name),
                            "kernel": "decode_stream_kernel + decode_combine_kernel (per block-step, HIP events)",
                            "avg_block_step_us": ms_all * 1e3 / n_launch,
                            "local_GBps": gbs(ms_loc), "sync_GBps": gbs(ms_syn),
                            "avg_local_us": ms_loc * 1e3 / n_launch, "avg_sync_us": ms_syn * 1e3 / n_launch,
                            "blocks_fused_GBps": gbs(ms_fused), "blocks_fused_ms_per_step": ms_fused / len(steps)}}
        result["decode"] = dec
        log("decode: %.0f GB/s by events (all-local %.0f, all-sync %.0f), %.0f GB/s end to end; "
            "upper bound with the blocks of a kind sharing launches (no block dependencies): %.0f GB/s"
            % (dec["roofline"]["achieved"], dec["roofline"]["local_GBps"], dec["roofline"]["sync_GBps"],
               dec["end_to_end_GBps"], dec["roofline"]["blocks_fused_GBps"]))

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
