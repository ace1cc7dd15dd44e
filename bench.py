#!/usr/bin/env python3
"""Benchmark of the BFP KV-cache hot path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input, as a decoder
layer would run it: kvbfp_quantize_append of the new token's K/V rows (one per sequence) followed
by kvbfp_decode_attention over the packed cache.  Successive steps walk a ring of distinct layer
caches (>= 1 GB in total) so no byte is served from the last-level cache of a previous step.

Prints ONE JSON line: the metric is achieved HBM GB/s of decode attention + append, computed from
the ALGORITHMIC bytes of a step (packed cache rows read once per KV head, q read, output written,
new rows read and their packed form written) divided by the measured time per step.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2403_20137_amd import kvbfp, synth  # noqa: E402

HBM_PEAK_GBS = 8000.0
HEADLINE = "llama3_8b_gqa_32k"
ELT_BYTES = {"f32": 4, "f16": 2, "bf16": 2}


def algorithmic_bytes(w: synth.Workload, seq_after_append: int):
    """(decode bytes, append bytes) one step must move."""
    elt = ELT_BYTES[w.dtype]
    cache = w.batch * w.n_kv_heads * seq_after_append * w.row_pair_bytes()
    q_io = 2 * w.batch * w.n_q_heads * w.head_dim * elt
    n_elem = 2 * w.batch * w.n_kv_heads * w.head_dim                  # K and V rows of one new token
    append = n_elem * elt + n_elem * w.mant_bits // 8 + n_elem // w.block
    return cache + q_io, append


class LayerRing:
    """`n_layers` packed caches of one workload, filled by bulk quantize_append on the GPU."""

    def __init__(self, w: synth.Workload, n_layers: int, device="cuda", capacity_pad=0):
        self.w = w
        self.S_max = w.seq + 1                      # tokens per sequence after the step's append
        self.capacity = self.S_max + capacity_pad   # tokens a sequence's region can hold (layout.max_seq)
        self.layout = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch, self.capacity)
        kg = synth.outlier_gains(synth.BASE_SEED, synth.TID_K_GAIN, w.n_kv_heads, w.head_dim, w.outlier_count, w.outlier_gain)
        vg = synth.outlier_gains(synth.BASE_SEED, synth.TID_V_GAIN, w.n_kv_heads, w.head_dim, w.outlier_count, w.outlier_gain)
        self.k_gain, self.v_gain = kg, vg
        calib_k = synth.kv_rows(1, w.n_calib, w.n_kv_heads, w.head_dim, w.dtype, kg, synth.BASE_SEED, synth.TID_K_CALIB)[0]
        calib_v = synth.kv_rows(1, w.n_calib, w.n_kv_heads, w.head_dim, w.dtype, vg, synth.BASE_SEED, synth.TID_V_CALIB)[0]
        self.perm_k_host = kvbfp.calibrate_perm(calib_k)
        self.perm_v_host = kvbfp.calibrate_perm(calib_v)
        self.perm_k = torch.as_tensor(self.perm_k_host, device=device)
        self.perm_v = torch.as_tensor(self.perm_v_host, device=device)
        self.caches = []
        for layer in range(n_layers):
            cache = kvbfp.alloc_cache(self.layout, device)
            k = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, kg, synth.BASE_SEED + layer, synth.TID_K, device)
            v = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, vg, synth.BASE_SEED + layer, synth.TID_V, device)
            kvbfp.quantize_append(cache, k, v, pos0=0, perm_k=self.perm_k, perm_v=self.perm_v)
            torch.cuda.synchronize()
            if layer == 0:
                self.k0, self.v0 = k, v          # kept for the CPU-baseline sample
            del k, v
            self.caches.append(cache)
        self.q = synth.queries(w.batch, w.n_q_heads, w.head_dim, w.dtype, synth.BASE_SEED, synth.TID_Q, device)
        self.k_new = synth.kv_rows(w.batch, 1, w.n_kv_heads, w.head_dim, w.dtype, kg, synth.BASE_SEED, synth.TID_K_NEW, device)
        self.v_new = synth.kv_rows(w.batch, 1, w.n_kv_heads, w.head_dim, w.dtype, vg, synth.BASE_SEED, synth.TID_V_NEW, device)
        self.pos = torch.full((w.batch,), w.seq, dtype=torch.int32, device=device)
        self.seq_len = torch.full((w.batch,), w.seq + 1, dtype=torch.int32, device=device)
        self.fused = True
        self.out = torch.empty_like(self.q)
        need = kvbfp.decode_workspace_bytes(self.layout, w.n_q_heads, self.S_max)
        self.workspace = torch.empty((need,), dtype=torch.uint8, device=device)
        self.scale = float(np.float32(w.head_dim ** -0.5))

    def append(self, i):
        kvbfp.quantize_append(self.caches[i % len(self.caches)], self.k_new, self.v_new, pos_dev=self.pos,
                              perm_k=self.perm_k, perm_v=self.perm_v)

    def decode(self, i):
        kvbfp.decode_attention(self.caches[i % len(self.caches)], self.q, self.S_max, self.scale,
                               perm_k=self.perm_k, perm_v=self.perm_v, out=self.out, workspace=self.workspace)

    def step(self, i):
        """One decode step of a layer: the current token is cast and appended, then attention."""
        if self.fused:
            kvbfp.append_decode_attention(self.caches[i % len(self.caches)], self.k_new, self.v_new, self.q, self.S_max,
                                          self.scale, seq_len_dev=self.seq_len, perm_k=self.perm_k, perm_v=self.perm_v,
                                          out=self.out, workspace=self.workspace)
        else:
            self.append(i)
            self.decode(i)

    def split_pass_ring_us(self, n_launches, q_mant_bits=0):
        """The split pass launched n_launches times back to back over the ring (HIP events on the stream around
        the batch, inside the library): average (split us, combine us) per launch."""
        _, split_ms, combine_ms = kvbfp.decode_attention_profile_ring(
            self.caches, n_launches, self.q, self.S_max, self.scale, q_mant_bits, perm_k=self.perm_k, perm_v=self.perm_v,
            out=self.out, workspace=self.workspace)
        return split_ms * 1e3, combine_ms * 1e3

    def stream_read_us(self, i):
        """Plain read of exactly the cache bytes one decode call streams (no arithmetic): the machine's ceiling."""
        units = self.w.batch * self.w.n_kv_heads                      # three workgroups per compute unit, like the split pass
        return kvbfp.measure_stream_read(self.caches[i % len(self.caches)], self.S_max, max(1, 768 // units)) * 1e3

    def decode_kernels(self, i, q_mant_bits=0):
        """The same decode call with HIP events around each of its two kernels: (split us, combine us)."""
        _, split_ms, combine_ms = kvbfp.decode_attention_profile(
            self.caches[i % len(self.caches)], self.q, self.S_max, self.scale, q_mant_bits, perm_k=self.perm_k,
            perm_v=self.perm_v, out=self.out, workspace=self.workspace)
        return split_ms * 1e3, combine_ms * 1e3


def paged_split_us(ring: LayerRing, page=256, n_pools=4):
    """The workload's caches again as pools of pages of `page` tokens, every sequence's pages scattered over its
    pool by a seeded shuffle; split pass of kvbfp_decode_attention_paged, HIP events inside the call,
    cycling over pools that together exceed the last-level cache."""
    w = ring.w
    per_seq = (ring.S_max + page - 1) // page
    pool_layout = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch * per_seq, page)
    rng = np.random.default_rng(synth.BASE_SEED)
    pools = []
    for layer in range(n_pools):
        pool = kvbfp.alloc_cache(pool_layout, ring.q.device)
        table = torch.as_tensor(rng.permutation(w.batch * per_seq).reshape(w.batch, per_seq).astype(np.int32),
                                device=ring.q.device)
        k = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, ring.k_gain, synth.BASE_SEED + layer, synth.TID_K,
                          ring.q.device)
        v = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, ring.v_gain, synth.BASE_SEED + layer, synth.TID_V,
                          ring.q.device)
        kvbfp.quantize_append_paged(pool, table, k, v, pos0=0, perm_k=ring.perm_k, perm_v=ring.perm_v)
        kvbfp.quantize_append_paged(pool, table, ring.k_new, ring.v_new, pos_dev=ring.pos, perm_k=ring.perm_k,
                                    perm_v=ring.perm_v)
        torch.cuda.synchronize()
        del k, v
        pools.append((pool, table))
    us = []
    for i in range(12):
        pool, table = pools[i % n_pools]
        us.append(kvbfp.decode_attention_paged(pool, table, ring.q, ring.S_max, ring.scale, perm_k=ring.perm_k,
                                               perm_v=ring.perm_v, out=ring.out, profile=True)[1] * 1e3)
    return float(np.median(us[2:]))


def capture_steps_graph(ring: LayerRing, first: int, count: int):
    """One HIP graph holding `count` consecutive steps (append + decode each) over the ring of layer caches, the
    way a model's per-token graph holds its layers: a serving loop replays it instead of paying the launch
    gaps between separate kernels and between separate small graphs."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        for i in range(count):
            ring.step(first + i)
    torch.cuda.synchronize()
    return g


def time_graph_steps(ring: LayerRing, steps: int, warmup: int):
    """`warmup` steps replayed from one graph, then exactly `steps` steps from another, timed around one replay
    (its first replay, which also uploads the graph to the device, is part of the untimed warm-up)."""
    g_warm = capture_steps_graph(ring, 0, warmup) if warmup > 0 else None
    g_timed = capture_steps_graph(ring, warmup, steps)
    g_timed.replay()
    if g_warm is not None:
        g_warm.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    g_timed.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_graph_per_layer(ring: LayerRing, steps: int, warmup: int):
    """The same steps as one small graph per layer cache, one replay per step (a launch gap between steps)."""
    graphs = []
    for i in range(len(ring.caches)):
        graphs.append(capture_steps_graph(ring, i, 1))
    for i in range(warmup):
        graphs[i % len(graphs)].replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        graphs[(warmup + i) % len(graphs)].replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_steps(ring: LayerRing, steps: int, warmup: int):
    """Eager launches of the two separate calls, each bracketed by HIP events."""
    for i in range(warmup):
        ring.append(i)
        ring.decode(i)
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        ev[i][0].record()
        ring.append(warmup + i)
        ev[i][1].record()
        ring.decode(warmup + i)
        ev[i][2].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    app = np.array([e[0].elapsed_time(e[1]) for e in ev]) * 1e3      # us
    dec = np.array([e[1].elapsed_time(e[2]) for e in ev]) * 1e3
    return (t1 - t0) / steps, app, dec


def cpu_baseline(ring: LayerRing, budget_s=12.0):
    """The oracle, as it stands, on (batch, kv-head) units of layer 0 of the same workload."""
    from oracle import kvbfp_oracle as O
    w = ring.w
    G = w.group
    units = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)]
    t_attn = t_quant = 0.0
    n_done = 0
    q_host = synth.to_f32_numpy(ring.q)
    for (b, h) in units:
        kk = synth.to_f32_numpy(ring.k0[b:b + 1, :, h:h + 1])
        vv = synth.to_f32_numpy(ring.v0[b:b + 1, :, h:h + 1])
        t = time.perf_counter()
        km, ke = O.quantize_append(kk, w.block, w.mant_bits, w.seq, 0, perm=ring.perm_k_host[h:h + 1])
        vm, ve = O.quantize_append(vv, w.block, w.mant_bits, w.seq, 0, perm=ring.perm_v_host[h:h + 1])
        t_quant += time.perf_counter() - t
        t = time.perf_counter()
        O.decode_attention(km, ke, vm, ve, w.head_dim, w.block, w.mant_bits, q_host[b:b + 1, h * G:(h + 1) * G],
                           [w.seq], ring.scale, ring.perm_k_host[h:h + 1], ring.perm_v_host[h:h + 1])
        t_attn += time.perf_counter() - t
        n_done += 1
        if t_attn + t_quant > budget_s:
            break
    bytes_done = n_done * w.seq * w.row_pair_bytes()
    elems = n_done * 2 * w.seq * w.head_dim
    return {"value": bytes_done / t_attn / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%d of %d (batch, kv-head) units of %s, %d tokens each: decode attention %.2f s; "
                      "their cast to BFP %.2f s = %.4f Gelem/s" % (n_done, len(units), w.name, w.seq, t_attn,
                                                                   t_quant, elems / t_quant / 1e9),
            "quantize_gelem_s": elems / t_quant / 1e9,
            "host_logical_cores": os.cpu_count()}


def bulk_quantize_rate(device="cuda", reps=5):
    """Bulk prefill cast (32 layers x 8 KV heads x 4096 tokens, K and V) in Gelem/s."""
    w = synth.WORKLOADS["prefill_bulk"]
    kg = synth.outlier_gains(synth.BASE_SEED, synth.TID_K_GAIN, w.n_kv_heads, w.head_dim, w.outlier_count, w.outlier_gain)
    k = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, kg, synth.BASE_SEED, synth.TID_K, device)
    v = synth.kv_rows(w.batch, w.seq, w.n_kv_heads, w.head_dim, w.dtype, kg, synth.BASE_SEED, synth.TID_V, device)
    layout = kvbfp.make_layout(w.head_dim, w.block, w.mant_bits, w.n_kv_heads, w.batch, w.seq)
    cache = kvbfp.alloc_cache(layout, device)
    def rate(perm):
        kvbfp.quantize_append(cache, k, v, perm_k=perm, perm_v=perm)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            kvbfp.quantize_append(cache, k, v, perm_k=perm, perm_v=perm)
            b.record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev]) * 1e3

    us = rate(None)
    # the same cast with the channel gather done at append time (a seeded permutation per KV head)
    g = torch.Generator().manual_seed(synth.BASE_SEED)
    perm = torch.stack([torch.randperm(w.head_dim, generator=g) for _ in range(w.n_kv_heads)]).to(torch.int32).to(device)
    us_perm = rate(perm)
    elems = 2 * k.numel()
    bytes_ = elems * 2 + elems * w.mant_bits // 8 + elems // w.block
    # the way back (kvbfp_dequantize): the K plane of the same cache to bf16 rows, in cache order and un-permuted
    out = torch.empty_like(k)
    def back(perm):
        kvbfp.dequantize(cache, 0, 0, w.seq, perm=perm, out=out)
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in ev:
            a.record()
            kvbfp.dequantize(cache, 0, 0, w.seq, perm=perm, out=out)
            b.record()
        torch.cuda.synchronize()
        return np.array([a.elapsed_time(b) for a, b in ev]) * 1e3
    dq, dq_perm = back(None), back(perm)
    return {"workload": w.name, "elements": elems, "us_median": float(np.median(us)), "us_min": float(us.min()),
            "gelem_s": elems / np.median(us) / 1e3, "hbm_gb_s": bytes_ / np.median(us) / 1e3,
            "hbm_frac": bytes_ / np.median(us) / 1e3 / HBM_PEAK_GBS,
            "with_perm_us_median": float(np.median(us_perm)), "with_perm_gelem_s": elems / np.median(us_perm) / 1e3,
            "dequantize_k_elements": elems // 2, "dequantize_k_us_median": float(np.median(dq)),
            "dequantize_k_gelem_s": elems / 2 / np.median(dq) / 1e3,
            "dequantize_k_hbm_frac": bytes_ / 2 / np.median(dq) / 1e3 / HBM_PEAK_GBS,
            "dequantize_k_with_perm_us_median": float(np.median(dq_perm))}


def profile_counters():
    """Counters taken from the tracked rocprofv3 summaries (profiles/counters.json): HBM traffic of the split pass
    (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy) and its vector-ALU busy fraction.  Not measured by this run."""
    path = os.path.join(ROOT, "profiles", "counters.json")
    try:
        return json.load(open(path))
    except Exception:
        return {}


def workload_entry(name, steps, batches=5):
    """One workload: split pass (ring of caches, back-to-back launches), whole call, plain streaming read."""
    w = synth.WORKLOADS[name]
    n_layers = min(64, max(2, -(-1_100_000_000 // w.cache_bytes(w.seq + 1))))
    ring = LayerRing(w, n_layers)
    dec_bytes, _ = algorithmic_bytes(w, w.seq + 1)
    n = max(n_layers, min(steps, 32))
    ring.split_pass_ring_us(n)                                   # warm-up
    runs = np.array([ring.split_pass_ring_us(n) for _ in range(batches)])
    split, combine = runs[:, 0], runs[:, 1]
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(steps, 12))]
    for i, (e0, e1) in enumerate(ev):
        e0.record()
        ring.decode(i)
        e1.record()
    torch.cuda.synchronize()
    call = np.array([a.elapsed_time(b) for a, b in ev])[2:] * 1e3
    stream = np.array([ring.stream_read_us(i) for i in range(10)])[2:]
    # the same call captured 64 times (cycling over the ring) into one graph, as a model's per-token graph would hold it
    n_graph = max(n_layers, 64)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=torch.cuda.Stream()):
        for i in range(n_graph):
            ring.decode(i)
    torch.cuda.synchronize()
    in_graph = []
    for _ in range(4):
        t0 = time.perf_counter()
        g.replay()
        torch.cuda.synchronize()
        in_graph.append((time.perf_counter() - t0) / n_graph * 1e6)
    in_graph_us = float(np.median(in_graph[1:]))
    del g
    counters = profile_counters().get(name, {})
    entry = {"algorithmic_bytes": dec_bytes, "layer_caches_in_ring": n_layers,
             "split_pass_us_avg": float(split.mean()), "split_pass_us_min": float(split.min()),
             "combine_pass_us_avg": float(combine.mean()),
             "split_pass_gb_s": dec_bytes / float(split.mean()) / 1e3,
             "split_pass_frac_of_hbm_peak": dec_bytes / float(split.mean()) / 1e3 / HBM_PEAK_GBS,
             "whole_call_us_median": float(np.median(call)), "whole_call_us_min": float(call.min()),
             "whole_call_gb_s": dec_bytes / float(np.median(call)) / 1e3,
             "whole_call_frac_of_hbm_peak": dec_bytes / float(np.median(call)) / 1e3 / HBM_PEAK_GBS,
             "whole_call_us_in_graph": in_graph_us, "whole_call_in_graph_calls": n_graph,
             "whole_call_in_graph_frac_of_hbm_peak": dec_bytes / in_graph_us / 1e3 / HBM_PEAK_GBS,
             "stream_read_us_median": float(np.median(stream)),
             "stream_read_gb_s": dec_bytes / float(np.median(stream)) / 1e3,
             "valu_busy_from_profile": counters.get("valu_busy"), "hbm_traffic_bytes_from_profile": counters.get("traffic")}
    del ring
    torch.cuda.empty_cache()
    return entry


def device_info():
    """Name, compute units and current clocks of the GPU the numbers were taken on.  The clocks are read from
    the driver's sysfs files (the level marked '*' in pp_dpm_sclk / pp_dpm_mclk); no other program is started."""
    p = torch.cuda.get_device_properties(0)
    info = {"name": p.name, "compute_units": p.multi_processor_count}
    try:
        import glob
        clocks = {}
        for path in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
            for key, name in (("sclk", "pp_dpm_sclk"), ("mclk", "pp_dpm_mclk")):
                with open(os.path.join(os.path.dirname(path), name)) as f:
                    cur = [ln.split(":", 1)[1].replace("*", "").strip() for ln in f if "*" in ln]
                if cur:
                    clocks[key] = cur[0]
            if clocks:
                break
        if clocks:
            info["current_clocks"] = clocks
    except Exception:
        pass
    return info


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(synth.WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="distinct layer caches in the ring (0 = enough for >= 1 GB)")
    ap.add_argument("--capacity-pad", type=int, default=0,
                    help="tokens of spare capacity per sequence region beyond the workload's length")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true")
    ap.add_argument("--no-graph", action="store_true", help="time eager launches instead of graph replays")
    ap.add_argument("--separate-calls", action="store_true",
                    help="a step = quantize_append + decode_attention as two calls instead of append_decode_attention")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy a few times (known HBM bytes; used to scale "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); --gpus %d is not "
              "supported. value is one GPU's throughput." % args.gpus, file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    kvbfp.lib()     # fail loudly if the HIP library has not been built
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 5}))
        return

    w = synth.WORKLOADS[args.workload]
    n_layers = args.layers or max(2, -(-1_100_000_000 // w.cache_bytes(w.seq + 1)))
    n_layers = min(n_layers, 64)
    ring = LayerRing(w, n_layers, capacity_pad=args.capacity_pad)
    dec_bytes, app_bytes = algorithmic_bytes(w, w.seq + 1)
    ring.fused = not args.separate_calls
    eager_sec_per_step, app_us, dec_us = time_steps(ring, args.steps, args.warmup)
    if args.no_graph:
        for i in range(args.warmup):
            ring.step(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            ring.step(args.warmup + i)
        torch.cuda.synchronize()
        sec_per_step = (time.perf_counter() - t0) / args.steps
    else:
        # the same steps replayed from captured graphs: the timed region of `value`
        sec_per_step = time_graph_steps(ring, args.steps, args.warmup)
    value = (dec_bytes + app_bytes) / sec_per_step / 1e9

    # The kernel that streams the cache (split pass): `steps` launches back to back over the ring, HIP events on the
    # launch stream around the batch (inside the library), several batches; its average duration per launch.
    # Beside it: events around single launches (each interval then holds one launch latency), and a plain read of
    # the same bytes with no arithmetic -- what a read-only kernel of this size reaches on this machine.
    n_batch = max(n_layers, args.steps)
    ring.split_pass_ring_us(n_batch)
    batch_runs = np.array([ring.split_pass_ring_us(n_batch) for _ in range(6)])
    split_avg_us, combine_avg_us = float(batch_runs[:, 0].mean()), float(batch_runs[:, 1].mean())
    kern = np.array([ring.decode_kernels(args.warmup + i) for i in range(args.steps)])
    single_us = kern[:, 0]
    stream_us = np.array([ring.stream_read_us(i) for i in range(14)])[2:]
    counters = profile_counters().get(w.name, {})
    roofline = {"bound": "hbm", "achieved": dec_bytes / split_avg_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": dec_bytes / split_avg_us / 1e3 / HBM_PEAK_GBS, "traffic": counters.get("traffic"),
                "kernel": "decode attention split pass (the kernel that reads the packed cache)",
                "bytes_per_launch": dec_bytes, "avg_launch_us": split_avg_us,
                "launches_timed": int(6 * n_batch), "min_batch_avg_us": float(batch_runs[:, 0].min()),
                "single_launch_event_interval_us_median": float(np.median(single_us)),
                "combine_pass_avg_us": combine_avg_us,
                "whole_call_avg_us": float(dec_us.mean()),
                "whole_call_frac": dec_bytes / (float(dec_us.mean()) * 1e-6) / 1e9 / HBM_PEAK_GBS,
                "stream_read_us_median": float(np.median(stream_us)),
                "stream_read_gb_s": dec_bytes / float(np.median(stream_us)) / 1e3,
                "frac_of_stream_read": float(np.median(stream_us)) / split_avg_us,
                "valu_busy_from_profile": counters.get("valu_busy")}

    result = {
        "metric": "BFP-KV decode attention HBM GB/s (% of peak); quantize-append Gelem/s",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "seq": w.seq + 1, "block": w.block, "mant_bits": w.mant_bits,
                   "layer_caches_in_ring": n_layers, "ring_bytes": n_layers * w.cache_bytes(w.seq + 1),
                   "step": ("quantize_append(1 token/sequence) + decode_attention, two calls" if args.separate_calls else
                            "append_decode_attention: 1 token/sequence cast and appended, then attention, one call"),
                   "launch": ("eager" if args.no_graph else
                              "one captured graph of the timed steps over the ring (as a model's per-token graph holds its "
                              "layers), replayed once")},
        "pct_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS,
        "two_calls_eager_ms_per_step": eager_sec_per_step * 1e3,
        "graph_per_step_ms_per_step": None if args.no_graph else time_graph_per_layer(ring, args.steps, args.warmup) * 1e3,
        "append_us_median": float(np.median(app_us)), "decode_us_median": float(np.median(dec_us)),
        "roofline": roofline,
    }
    if not args.no_extra:
        def extra(key, fn):
            """Every extra figure stands for itself: a failure is reported under its own key, never hidden."""
            try:
                result[key] = fn()
            except Exception as e:
                result[key] = {"error": repr(e)}

        def query_bfp8():
            return float(np.median([ring.decode_kernels(i, q_mant_bits=8)[0] for i in range(min(args.steps, 20))]))

        def single_cache_hot():
            # the same call over ONE cache again and again: whatever of it stays in the 256 MB last-level
            # cache is not read from HBM, so this figure is LLC-assisted and not a bandwidth claim
            hot = []
            for _ in range(12):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                ring.decode(0)
                e1.record()
                hot.append((e0, e1))
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in hot][2:]) * 1e3)

        def four_query_tokens():
            # four query tokens per sequence (G * 4 virtual heads per kv-head) over the same caches
            q4 = torch.stack([ring.q] * 4, dim=1).contiguous()
            ws4 = torch.empty((kvbfp.decode_workspace_bytes(ring.layout, w.n_q_heads * 4, ring.S_max),), dtype=torch.uint8,
                              device=ring.q.device)
            out4 = torch.empty_like(q4)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(12)]
            for i, (e0, e1) in enumerate(ev):
                e0.record()
                kvbfp.decode_attention_multi(ring.caches[i % len(ring.caches)], q4, ring.S_max, ring.scale, perm_k=ring.perm_k,
                                             perm_v=ring.perm_v, out=out4, workspace=ws4)
                e1.record()
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in ev][2:]) * 1e3)

        def rotary_at_read():
            # the same caches read as if their keys had been stored before the rotary embedding: rotation at
            # read with the reordered parameters (Alg. 1 step 5), split pass only, HIP events inside the call
            theta = (10000.0 ** (-np.arange(w.head_dim // 2, dtype=np.float64) / (w.head_dim // 2))).astype(np.float32)
            rp = [torch.from_numpy(x).to(ring.q.device)
                  for x in kvbfp.permute_rope(theta, ring.perm_k_host, kvbfp.ROPE_PAIRS_HALF_SPLIT)]
            rope_us = [kvbfp.decode_attention_rope(ring.caches[i % len(ring.caches)], ring.q, ring.S_max, ring.scale, *rp,
                                                   perm_k=ring.perm_k, perm_v=ring.perm_v, out=ring.out,
                                                   workspace=ring.workspace, profile=True)[1] * 1e3 for i in range(8)]
            return float(np.median(rope_us[2:]))

        def general_pass_vector_alu():
            # the same cache through the general split pass (fp32 multiply-adds on the vector ALUs, no matrix cores):
            # what the matrix-core passes are measured against.  Reached the way a caller reaches it: exponent planes
            # that are not 16-byte aligned.
            c0 = ring.caches[0]
            moved = []
            for t in (c0.k_exp, c0.v_exp):
                buf = torch.zeros((t.numel() + 64,), dtype=torch.uint8, device=t.device)
                view = buf[1:1 + t.numel()].view(t.shape)
                view.copy_(t)
                moved.append(view)
            odd = kvbfp.Cache(c0.layout, c0.k_mant, moved[0], c0.v_mant, moved[1])
            us = [kvbfp.decode_attention_profile(odd, ring.q, ring.S_max, ring.scale, perm_k=ring.perm_k, perm_v=ring.perm_v,
                                                 out=ring.out, workspace=ring.workspace)[1] * 1e3 for _ in range(6)]
            return float(np.median(us[2:]))

        extra("decode_split_us_median_general_pass_vector_alu", general_pass_vector_alu)
        extra("decode_split_us_median_query_bfp8", query_bfp8)
        extra("decode_us_median_single_cache_llc_assisted", single_cache_hot)
        extra("decode_4_query_tokens_us_median", four_query_tokens)
        extra("decode_split_us_median_rotary_at_read", rotary_at_read)
        extra("decode_split_us_median_paged_256", lambda: paged_split_us(ring))
        extra("decode_split_us_median_paged_16", lambda: paged_split_us(ring, page=16))
        extra("quantize_append_bulk", bulk_quantize_rate)
    result["device"] = device_info()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(ring)
    if not args.no_extra:
        # the other workloads of the contract and the headline shapes at the other block sizes and at 8 bits, decode
        # attention only (the timed region of `value` is the headline's)
        del ring
        torch.cuda.empty_cache()
        result["workloads"] = {}
        for name in ("llama2_7b_4k", "batched_8k_p4", "batched_8k_p8", "long_128k", "gqa_32k_n64", "gqa_32k_n128", "gqa_32k_p8n16",
                     "gqa8_32k", "gqa_32k_b96"):
            if name == w.name:
                continue
            try:
                result["workloads"][name] = workload_entry(name, args.steps)
            except Exception as e:
                result["workloads"][name] = {"error": repr(e)}
    print(json.dumps(result, default=float))


if __name__ == "__main__":
    main()
