#!/usr/bin/env python3
"""Benchmark of the L2-norm KV-cache compression hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic batch of the
32k-context Llama-3-8B-shaped GQA workload (config C3): compress every layer's
cache once (key norms -> lowest-norm selection -> K/V compaction), then run 64
decode steps of single-query GQA attention over the compacted cache of all 32
layers.  The cache is static during decoding: no row is appended per decode
step (the streaming workload C5 is the one that appends and evicts).  Inputs
are resident in HBM before the timed region starts.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3]

Prints ONE JSON line: whole-path effective HBM GB/s (algorithmic bytes / wall
time), microseconds per decode step, the roofline of the dominant kernel
(decode attention) from HIP events on the launch stream, the CPU oracle timed
on a bounded sample of the same workload (one thread, and threads over heads on
the host cores this process may use), and -- in the default run -- one short
pass each of the 131k-token retrieval workload (C4) and the ragged streaming
workload (C5) under "other_workloads", each with a GPU-vs-oracle check of a
sample.
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
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import paper_2406_11430_amd as l2kv            # noqa: E402
from paper_2406_11430_amd import synth         # noqa: E402

HBM_PEAK_GBPS = 8000.0      # MI355X published HBM3E peak (8 TB/s): the figure every fraction here is taken of

# HBM bytes of ONE decode-attention launch at the C3 per-layer shape, from two
# rocprofv3 --pmc runs (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, factors from a
# plain 1 GiB copy in the same runs): profiles/hot_path_hbm_traffic_pmc.md.
# A constant from that offline profile, not something this run measures;
# reported only when the timed shape is that shape.
PROFILED_DECODE_TRAFFIC_BYTES = {("bf16", 4, 8, 32, 128, 16384): (263029 + 491) * 1024}


def host_threads():
    """Threads the CPU baseline may use: the cores this process is allowed on,
    at most 16 (the host share that goes with one GPU)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def device_facts(dev):
    """What the device reports about itself, printed next to the peak used."""
    p = torch.cuda.get_device_properties(dev)
    info = l2kv.l2kv_device_info()
    clock_khz, bus_bits = info["memory_clock_khz"], info["memory_bus_bits"]
    from_props = None
    if clock_khz and bus_bits:
        # HBM3E moves 4 bits per pin per reported memory clock (8 Gb/s per pin at 2000 MHz)
        from_props = round(4.0 * clock_khz * 1e3 * bus_bits / 8 / 1e9, 1)
    return {"name": p.name, "compute_units": info["compute_units"],
            "memory_GiB": round(p.total_memory / 2 ** 30, 1),
            "memory_clock_MHz": None if not clock_khz else round(clock_khz / 1e3, 1),
            "memory_bus_bits": bus_bits, "GBps_from_bus_bits_x_clock_x_4_per_clock": from_props,
            "peak_used_GBps": HBM_PEAK_GBPS}


# ----------------------------------------------------------------- byte model
def compress_bytes_per_layer(cfg, k):
    """Algorithmic HBM bytes of norms + select + compact for one layer."""
    n = cfg.B * cfg.Hkv
    row = cfg.D * cfg.elem_bytes
    norms = n * cfg.T * row + n * cfg.T * 4            # read K, write norms
    select = n * cfg.T * 4 + n * k * 4                 # read norms, write indices
    compact = n * k * 4 + 2 * n * k * row + 2 * n * k * row   # indices + kept K,V rows in, rows out
    return norms, select, compact


def decode_bytes_per_layer(cfg, k):
    """Algorithmic HBM bytes of one decode-attention call on one layer: Kc and
    Vc once per KV head (shared by the query group), plus Q in and O out."""
    n = cfg.B * cfg.Hkv
    row = cfg.D * cfg.elem_bytes
    return 2 * n * k * row + cfg.B * cfg.Hq * cfg.D * cfg.elem_bytes + cfg.B * cfg.Hq * cfg.D * 4


# ------------------------------------------------------------------- workload
class Workload:
    def __init__(self, cfg, dev, decode_splits=0):
        self.cfg, self.dev = cfg, dev
        self.decode_splits = decode_splits          # 0: the library's own choice
        L, B, Hkv, Hq, D, T = cfg.L, cfg.B, cfg.Hkv, cfg.Hq, cfg.D, cfg.T
        dt = synth.torch_dtype(cfg.dtype)
        self.k = l2kv.l2kv_keep_count(T, cfg.keep_ratio)
        self.K = torch.empty((L, B, Hkv, T, D), dtype=dt, device=dev)
        self.V = torch.empty_like(self.K)
        for layer in range(L):
            Kl, Vl = synth.make_layer(cfg, layer, device=dev)
            self.K[layer].copy_(Kl)
            self.V[layer].copy_(Vl)
            del Kl, Vl
        self.Q = torch.empty((cfg.decode_steps, L, B, Hq, D), dtype=dt, device=dev)
        for layer in range(L):
            for step in range(cfg.decode_steps):
                self.Q[step, layer].copy_(synth.make_query(cfg, layer, step, device=dev))
        self.norms = torch.empty((L, B, Hkv, T), dtype=torch.float32, device=dev)
        self.idx = torch.empty((L, B, Hkv, self.k), dtype=torch.int32, device=dev)
        self.cnt = torch.empty((L, B, Hkv), dtype=torch.int32, device=dev)
        self.Kc = torch.empty((L, B, Hkv, self.k, D), dtype=dt, device=dev)
        self.Vc = torch.empty_like(self.Kc)
        self.O = torch.empty((L, B, Hq, D), dtype=torch.float32, device=dev)
        self.sel_ws = torch.zeros(l2kv.l2kv_select_workspace_bytes(L * B * Hkv, T),
                                  dtype=torch.uint8, device=dev)
        self.dec_ws = torch.zeros(l2kv.l2kv_decode_workspace_bytes(B, Hq, self.k, D),
                                  dtype=torch.uint8, device=dev)
        # per-layer views made once, so the timed loop only marshals pointers
        self.Q_v = [[self.Q[s, l] for l in range(L)] for s in range(cfg.decode_steps)]
        self.Kc_v = [self.Kc[l] for l in range(L)]
        self.Vc_v = [self.Vc[l] for l in range(L)]
        self.O_v = [self.O[l] for l in range(L)]
        torch.cuda.synchronize()

    # -- the hot path: every call below is one C-ABI entry point ---------------
    def compress(self):
        l2kv.l2kv_norms(self.K, self.norms)
        l2kv.l2kv_select(self.norms, self.cfg.keep_ratio, self.idx, self.cnt, self.sel_ws)
        l2kv.l2kv_compact(self.K, self.V, self.idx, self.Kc, self.Vc)

    def decode_step(self, step):
        Qs, ws = self.Q_v[step], self.dec_ws
        if self.decode_splits:
            for layer in range(self.cfg.L):
                l2kv.l2kv_decode_attn_splits(Qs[layer], self.Kc_v[layer], self.Vc_v[layer], self.O_v[layer], ws,
                                             n_splits=self.decode_splits)
            return
        for layer in range(self.cfg.L):
            l2kv.l2kv_decode_attn(Qs[layer], self.Kc_v[layer], self.Vc_v[layer], self.O_v[layer], ws)

    def decode_all(self):
        for step in range(self.cfg.decode_steps):
            self.decode_step(step)

    def step(self):
        self.compress()
        self.decode_all()


# --------------------------------------------------------------- CPU baseline
def cpu_baseline(w: Workload, layers, dec_steps, threads):
    """Time the CPU oracle, as it stands, on a bounded sample: the full
    compression of `layers` layers plus `dec_steps` decode steps on each of
    them.  Two legs over the same sample: one thread (a whole layer per oracle
    call), and `threads` threads over the (sequence, KV head) pairs of a layer
    (the same oracle calls on one head each; ctypes releases the interpreter
    lock around them).  The one-thread leg also compares the GPU results of the
    sample with the oracle's."""
    import oracle
    cfg = w.cfg
    G = cfg.Hq // cfg.Hkv
    t_one = t_all = 0.0
    bytes_total = 0
    worst = 0.0
    idx_equal = rows_equal = True
    heads = [(b, h) for b in range(cfg.B) for h in range(cfg.Hkv)]
    for layer in layers:
        Kn = synth.as_numpy_bits(w.K[layer])
        Vn = synth.as_numpy_bits(w.V[layer])
        Qn = [synth.as_numpy_bits(w.Q[step, layer]) for step in range(dec_steps)]
        bytes_total += sum(compress_bytes_per_layer(cfg, w.k)) + dec_steps * decode_bytes_per_layer(cfg, w.k)
        # ---- one thread
        t0 = time.perf_counter()
        n32, _, idx, Kc, Vc = oracle.compress(Kn, Vn, cfg.dtype, cfg.keep_ratio)
        t_one += time.perf_counter() - t0
        idx_equal &= bool(np.array_equal(idx, w.idx[layer].cpu().numpy()))
        rows_equal &= bool(np.array_equal(Kc, synth.as_numpy_bits(w.Kc[layer])))
        rows_equal &= bool(np.array_equal(Vc, synth.as_numpy_bits(w.Vc[layer])))
        for step in range(dec_steps):
            t0 = time.perf_counter()
            want = oracle.decode_attn(Qn[step], Kc, Vc, cfg.dtype)
            t_one += time.perf_counter() - t0
            O = torch.empty((cfg.B, cfg.Hq, cfg.D), dtype=torch.float32, device=w.dev)
            l2kv.l2kv_decode_attn(w.Q[step, layer], w.Kc[layer], w.Vc[layer], O, w.dec_ws)
            worst = max(worst, float(np.abs(O.cpu().numpy() - want).max()))
        del n32, idx, Kc, Vc
        # ---- threads over heads
        if threads > 1:
            def one_head(bh):
                b, h = bh
                _, _, _, kc, vc = oracle.compress(Kn[b:b + 1, h:h + 1], Vn[b:b + 1, h:h + 1], cfg.dtype, cfg.keep_ratio)
                for step in range(dec_steps):
                    oracle.decode_attn(np.ascontiguousarray(Qn[step][b:b + 1, h * G:(h + 1) * G]), kc, vc, cfg.dtype)
            t0 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=threads) as pool:
                list(pool.map(one_head, heads))
            t_all += time.perf_counter() - t0
    sample = "%s: full compress of layer(s) %s + %d decode step(s) on each" % (cfg.name, list(layers), dec_steps)
    one = {
        "value": bytes_total / t_one / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
        "sample": "%s; %.1f s of CPU time" % (sample, t_one), "seconds": t_one,
        "gpu_vs_oracle_on_sample": {"kept_idx_equal": idx_equal, "compacted_rows_equal": rows_equal,
                                    "attn_max_abs_err": worst},
    }
    many = None
    if threads > 1:
        many = {"value": bytes_total / t_all / 1e9, "unit": "GB/s", "cores": threads, "kind": "oracle",
                "sample": "%s; threads over the %d (sequence, KV head) pairs of a layer; %.1f s wall" % (sample, len(heads), t_all),
                "seconds": t_all, "host_cpu_count": os.cpu_count()}
    return one, many


# ------------------------------------------------------- streaming workload (C5)
class StreamWorkload:
    """Ragged batch under streaming eviction: compress every prompt to keep_ratio,
    then per decode step append the new token of every sequence (all layers, one
    launch), attend layer by layer over the ragged slot cache, and evict down to
    keep_count(tokens seen, keep_ratio) (all layers, one launch)."""

    def __init__(self, cfg, dev):
        self.cfg, self.dev = cfg, dev
        L, Hkv, Hq, D, n_seq = cfg.L, cfg.Hkv, cfg.Hq, cfg.D, cfg.n_seq
        dt = synth.torch_dtype(cfg.dtype)
        P = L * Hkv
        lens = synth.stream_lengths(cfg).tolist()
        self.lens0 = lens
        kc = l2kv.l2kv_keep_count
        self.k0 = [kc(n, cfg.keep_ratio) for n in lens]
        # budget after decode step t (tokens seen = prompt + t + 1) and slot capacity
        self.budgets_host = [[kc(n + t + 1, cfg.keep_ratio) for n in lens] for t in range(cfg.decode_steps)]
        caps = [max([self.k0[s]] + [b[s] for b in self.budgets_host]) + 1 for s in range(n_seq)]
        off = lambda v: torch.tensor([0] + list(np.cumsum(v)), dtype=torch.int64, device=dev)   # noqa: E731
        self.in_off, self.out_off, self.slot_off = off(lens), off(self.k0), off(caps)
        self.total, self.total_kept, self.total_slots = sum(lens), sum(self.k0), sum(caps)
        self.max_len, self.max_kept, self.max_cap = max(lens), max(self.k0), max(caps)
        # The slot cache is the long-lived object: allocated first, its K and V halves in one
        # allocation.  (Where tensors lie in device memory matters on this GPU: a launch whose K and
        # V streams come from different thirds of the memory runs about 9 % slower,
        # profiles/placement_in_device_memory.md.)
        self.KVc = torch.zeros((2, P, self.total_slots, D), dtype=dt, device=dev)
        self.Kc, self.Vc = self.KVc[0], self.KVc[1]
        self.K = torch.empty((P, self.total, D), dtype=dt, device=dev)
        self.V = torch.empty_like(self.K)
        for layer in range(L):
            Kl, Vl = synth.make_ragged_layer(cfg, layer, device=dev)
            self.K[layer * Hkv:(layer + 1) * Hkv].copy_(Kl)
            self.V[layer * Hkv:(layer + 1) * Hkv].copy_(Vl)
            del Kl, Vl
        self.Knew = torch.empty((cfg.decode_steps, L, n_seq, Hkv, D), dtype=dt, device=dev)
        self.Vnew = torch.empty_like(self.Knew)
        self.Q = torch.empty((cfg.decode_steps, L, n_seq, Hq, D), dtype=dt, device=dev)
        for t in range(cfg.decode_steps):
            a, b, q = synth.make_stream_step(cfg, t, device=dev)
            self.Knew[t].copy_(a), self.Vnew[t].copy_(b), self.Q[t].copy_(q)
        self.norms = torch.empty((P, self.total), dtype=torch.float32, device=dev)
        self.idx = torch.empty((P, self.total_kept), dtype=torch.int32, device=dev)
        self.nc = torch.zeros((P, self.total_slots), dtype=torch.float32, device=dev)
        self.pc = torch.zeros((P, self.total_slots), dtype=torch.int32, device=dev)
        self.lens_init = torch.tensor(self.k0, dtype=torch.int32, device=dev)
        self.lensA = torch.empty_like(self.lens_init)
        self.lensB = torch.empty_like(self.lens_init)
        self.seq_order = torch.empty_like(self.lens_init)
        self.use_order = True                       # launch the sequences longest first
        self.budgets = torch.tensor(self.budgets_host, dtype=torch.int32, device=dev)
        self.tokens = torch.tensor([[n + t for n in lens] for t in range(cfg.decode_steps)],
                                   dtype=torch.int32, device=dev)
        self.O = torch.empty((L, n_seq, Hq, D), dtype=torch.float32, device=dev)
        self.ws = torch.zeros(l2kv.l2kv_decode_ragged_workspace_bytes(n_seq, Hq, self.max_cap, D),
                              dtype=torch.uint8, device=dev)
        self.Kc_v = [self.Kc[l * Hkv:(l + 1) * Hkv] for l in range(L)]
        self.Vc_v = [self.Vc[l * Hkv:(l + 1) * Hkv] for l in range(L)]
        self.Q_v = [[self.Q[t, l] for l in range(L)] for t in range(cfg.decode_steps)]
        self.O_v = [self.O[l] for l in range(L)]
        torch.cuda.synchronize()

    def compress(self):
        l2kv.l2kv_norms(self.K, self.norms)
        l2kv.l2kv_select_ragged(self.norms, self.in_off, self.out_off, self.max_len, self.idx)
        l2kv.l2kv_compact_ragged(self.K, self.V, self.norms, self.idx, self.in_off, self.out_off,
                                 self.max_kept, self.slot_off, self.Kc, self.Vc, self.nc, self.pc)
        self.lensA.copy_(self.lens_init)
        # longest-first launch order of the batch: set up once per compression, reused by every
        # decode step (all sequences grow alike, so it stays the length order)
        l2kv.l2kv_length_order(self.lensA, self.seq_order)

    def decode_step(self, t):
        l2kv.l2kv_stream_append(self.Knew[t], self.Vnew[t], self.tokens[t], self.slot_off, self.lensA,
                                self.lensB, self.Kc, self.Vc, self.nc, self.pc)
        Qs = self.Q_v[t]
        for layer in range(self.cfg.L):
            l2kv.l2kv_decode_attn_ragged(Qs[layer], self.Kc_v[layer], self.Vc_v[layer], self.lensB,
                                         self.slot_off, self.max_cap, self.O_v[layer], self.ws,
                                         seq_order=self.seq_order if self.use_order else None)
        l2kv.l2kv_stream_evict(self.slot_off, self.lensB, self.budgets[t], self.lensA, self.Kc, self.Vc,
                               self.nc, self.pc)

    def step(self):
        self.compress()
        for t in range(self.cfg.decode_steps):
            self.decode_step(t)

    # algorithmic bytes
    def compress_bytes(self):
        cfg = self.cfg
        P, row = cfg.L * cfg.Hkv, cfg.D * cfg.elem_bytes
        norms = P * self.total * (row + 4)
        select = P * (self.total * 4 + self.total_kept * 4)
        compact = P * self.total_kept * (4 + 2 * row + 2 * row + 4 + 4 + 4)   # idx, rows in/out, norm in/out, id
        return norms + select + compact

    def decode_bytes(self):
        """(attention bytes, append + evict bytes) summed over all decode steps."""
        cfg = self.cfg
        P, row = cfg.L * cfg.Hkv, cfg.D * cfg.elem_bytes
        attn = other = 0
        cur = list(self.k0)
        for t in range(cfg.decode_steps):
            after_append = [c + 1 for c in cur]
            attn += P * sum(after_append) * 2 * row + cfg.L * cfg.n_seq * cfg.Hq * cfg.D * (cfg.elem_bytes + 4)
            other += P * cfg.n_seq * (4 * row + 8)                               # append: rows in, rows out, norm, id
            evicted = [max(0, a - b) for a, b in zip(after_append, self.budgets_host[t])]
            other += P * sum(a * 8 * (1 if e else 0) + e * (4 * row + 16) for a, e in zip(after_append, evicted))
            cur = [min(a, b) for a, b in zip(after_append, self.budgets_host[t])]
        return attn, other


def stream_parity_sample(w: "StreamWorkload", n_heads=5, steps=4):
    """CPU baseline of the streaming workload: the oracle timed on a small sample, which doubles as
    a GPU-vs-oracle check.  Sampled (plane, sequence) heads of the streaming batch: the
    oracle compresses the sampled prompts and replays the first decode steps
    token by token (append, attend, evict to budget).  Kept token ids, slot
    contents and lengths must agree exactly; the attention error is returned."""
    import oracle
    cfg = w.cfg
    w.compress()
    torch.cuda.synchronize()
    lens = w.lens0
    rng = np.random.default_rng(55)
    P = cfg.L * cfg.Hkv
    samples = {(0, int(np.argmax(lens))), (P - 1, int(np.argmin(lens)))}
    while len(samples) < n_heads:
        samples.add((int(rng.integers(P)), int(rng.integers(cfg.n_seq))))
    in_off, out_off, slot_off = (t.cpu().numpy() for t in (w.in_off, w.out_off, w.slot_off))
    caps = np.diff(slot_off)
    heads, idx_equal = {}, True
    t_cpu = 0.0
    row = cfg.D * cfg.elem_bytes
    sample_bytes = 0                      # algorithmic bytes of what the oracle is timed on (same formulas as the GPU side)
    for (p, s) in sorted(samples):
        a, b = in_off[s], in_off[s + 1]
        sample_bytes += (b - a) * (row + 4) + (b - a) * 4 + w.k0[s] * 4 + w.k0[s] * (4 + 4 * row + 12)
        Kn, Vn = synth.as_numpy_bits(w.K[p, a:b]), synth.as_numpy_bits(w.V[p, a:b])
        t0 = time.perf_counter()
        n32, _ = oracle.norms(Kn[None], cfg.dtype)
        kept = oracle.select(n32, w.k0[s])[0]
        h = oracle.StreamHead(int(caps[s]), cfg.D, cfg.dtype)
        h.load(Kn[kept], Vn[kept], n32[0, kept], kept.astype(np.int32))
        t_cpu += time.perf_counter() - t0
        idx_equal &= bool(np.array_equal(w.idx[p, out_off[s]:out_off[s + 1]].cpu().numpy(), kept))
        heads[(p, s)] = h

    def slots_equal():
        ok = True
        lens_dev = w.lensA.cpu().numpy()
        for (p, s), h in heads.items():
            n, a = len(h), slot_off[s]
            ids, Kk, Vk, nk = h.kept()
            pc = w.pc[p, a:a + n].cpu().numpy()
            order = np.argsort(pc, kind="stable")
            ok &= int(lens_dev[s]) == n and bool(np.array_equal(pc[order], ids))
            ok &= bool(np.array_equal(synth.as_numpy_bits(w.Kc[p, a:a + n])[order], Kk))
            ok &= bool(np.array_equal(synth.as_numpy_bits(w.Vc[p, a:a + n])[order], Vk))
            ok &= bool(np.array_equal(w.nc[p, a:a + n].cpu().numpy()[order].view(np.uint32), nk.view(np.uint32)))
        return ok

    G, worst = cfg.Hq // cfg.Hkv, 0.0
    cache_equal = slots_equal()
    for t in range(min(steps, cfg.decode_steps)):
        w.decode_step(t)
        torch.cuda.synchronize()
        O = w.O.cpu().numpy()
        for (p, s), h in heads.items():
            layer, hk = p // cfg.Hkv, p % cfg.Hkv
            kn = synth.as_numpy_bits(w.Knew[t, layer, s, hk])
            vn = synth.as_numpy_bits(w.Vnew[t, layer, s, hk])
            qn = synth.as_numpy_bits(w.Q[t, layer, s, hk * G:(hk + 1) * G])
            sample_bytes += (len(h) + 1) * 2 * row + G * cfg.D * (cfg.elem_bytes + 4) + 4 * row + 8
            t0 = time.perf_counter()
            h.append(kn, vn, lens[s] + t)
            want = h.attend(qn)
            h.evict_to(w.budgets_host[t][s])
            t_cpu += time.perf_counter() - t0
            worst = max(worst, float(np.abs(O[layer, s, hk * G:(hk + 1) * G] - want).max()))
        cache_equal &= slots_equal()
    n_steps = min(steps, cfg.decode_steps)
    return {"value": sample_bytes / t_cpu / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
            "sample": "%s: %d sampled (plane, sequence) heads %s: prompt compression + %d decode steps (append, attend, "
                      "evict) replayed token by token; %.2f s of CPU time" % (cfg.name, len(samples), sorted(samples), n_steps, t_cpu),
            "seconds": t_cpu,
            "gpu_vs_oracle_on_sample": {"kept_idx_equal": idx_equal, "slot_cache_equal": cache_equal,
                                        "attn_max_abs_err": worst}}


def run_stream(cfg, dev, steps, warmup, overridden=False, use_order=True, parity=True):
    w = StreamWorkload(cfg, dev)
    w.use_order = use_order
    attn_bytes, other_bytes = w.decode_bytes()
    comp_bytes = w.compress_bytes()
    step_bytes = comp_bytes + attn_bytes + other_bytes
    for _ in range(warmup):
        w.step()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(steps):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        w.compress()
        e[1].record()
        for t in range(cfg.decode_steps):
            w.decode_step(t)
        e[2].record()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    comp_ms = float(np.median([e[0].elapsed_time(e[1]) for e in marks]))
    dec_ms = float(np.median([e[1].elapsed_time(e[2]) for e in marks]))
    value = step_bytes / (wall / steps) / 1e9
    achieved = (attn_bytes + other_bytes) / dec_ms / 1e6
    out = {
        "metric": "compress+decode effective HBM GB/s", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(wall * 1e3 / steps, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + (" (size overridden)" if overridden else ""), "layers": cfg.L,
                   "sequences": cfg.n_seq, "prompt_lengths": "uniform[%d, %d], seeded (sum %d)" % (cfg.len_lo, cfg.len_hi, w.total),
                   "kv_heads": cfg.Hkv, "q_heads": cfg.Hq, "head_dim": cfg.D, "keep_ratio": cfg.keep_ratio,
                   "decode_steps": cfg.decode_steps,
                   "step": "ragged compress of all prompts + decode_steps x (append one row per sequence, "
                           "layers x ragged attention, evict to keep_count(tokens seen))"},
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_decode_step": round(dec_ms * 1e3 / cfg.decode_steps, 2),
        "phases": {"compress": {"ms": round(comp_ms, 4), "GBps": round(comp_bytes / comp_ms / 1e6, 1)},
                   "decode": {"ms": round(dec_ms, 4), "GBps": round(achieved, 1)}},
        "roofline": {"kernel": "streaming decode step (append + ragged attention over all layers + evict)",
                     "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                     "bytes_per_decode_step": (attn_bytes + other_bytes) // cfg.decode_steps},
    }
    if parity:
        out["cpu_baseline"] = stream_parity_sample(w)
    del w
    torch.cuda.empty_cache()
    return out


def main_stream(args, dev):
    cfg = synth.STREAM_CONFIGS[args.workload]
    overridden = False
    if args.layers:
        cfg, overridden = cfg.scaled(L=args.layers), True
    if args.decode_steps:
        cfg, overridden = cfg.scaled(decode_steps=args.decode_steps), True
    out = run_stream(cfg, dev, args.steps, args.warmup, overridden, not args.no_seq_order,
                     parity=not args.no_cpu_baseline)
    out["device"] = device_facts(dev)
    print(json.dumps(out))


def main_placement(args, dev):
    """Where the cache lies in device memory changes what the memory system delivers.  This probe
    (not a benchmark line) fills the memory with 1 GiB cache tensors in allocation order and
    reports, per position: the read rate of the norm pass, that of the bare read
    (l2kv_read_probe), and the time of a C3-shaped decode
    launch (8 layers, B=4, 8 KV / 32 Q heads, 16384 rows, bf16) whose K and V are neighbours or a
    given number of GiB apart."""
    L, B, Hkv, Hq, n, D = 8, 4, 8, 32, 16384, 128
    dt = torch.bfloat16
    tensor_bytes = L * B * Hkv * n * D * 2                                  # 1 GiB
    Q = torch.randn((L, B, Hq, D), device=dev, dtype=dt)
    O = torch.empty((L, B, Hq, D), device=dev, dtype=torch.float32)
    ws = torch.zeros(l2kv.l2kv_decode_workspace_bytes(B, Hq, n, D), dtype=torch.uint8, device=dev)
    norms = torch.empty((L, B, Hkv, n), dtype=torch.float32, device=dev)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps                                      # ms

    def decode_us(Kc, Vc):
        def run():
            for layer in range(L):
                l2kv.l2kv_decode_attn(Q[layer], Kc[layer], Vc[layer], O[layer], ws)
        return round(timed(run, 4) * 1e3 / L, 2)

    free, total = torch.cuda.mem_get_info()
    count = int((free - (10 << 30)) // tensor_bytes)
    tensors = []
    for i in range(count):
        t = torch.empty((L, B, Hkv, n, D), dtype=dt, device=dev)
        t.view(torch.int16).fill_(1000 + i)
        tensors.append(t)
    for _ in range(20):                                                       # clocks up before the first figure
        decode_us(tensors[0], tensors[1])
    read = [round(tensor_bytes / timed(lambda t=t: l2kv.l2kv_norms(t, norms), 4) / 1e6) for t in tensors[::2]]
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    bare = [round(tensor_bytes / timed(lambda t=t: l2kv.l2kv_read_probe(t, sink), 4) / 1e6) for t in tensors[::2]]
    apart = args.placement_apart
    out = {
        "probe": "placement of the cache in device memory", "device_memory_GiB": round(total / 2**30, 1),
        "tensors_of_1GiB": count,
        "norm_pass_read_GBps_every_2nd_tensor": read,
        "bare_read_GBps_every_2nd_tensor": bare,
        "decode_us_per_launch_K_V_neighbours": [decode_us(tensors[i], tensors[i + 1]) for i in range(0, count - 1, 2)],
        "decode_us_per_launch_K_V_%dGiB_apart" % apart: [decode_us(tensors[i], tensors[i + apart])
                                                         for i in range(0, count - apart, 2)],
    }
    print(json.dumps(out))


def main_alr(args, dev):
    """Attention-loss analysis (Sec. 3, Eq. 5-7) at the shape of one layer of the
    chosen workload, repeated over `--layers` layers (default 4): discard ranks
    from the key norms, then losses and Y for one query per head."""
    cfg = synth.CONFIGS[args.workload]
    L = args.layers or 4
    B, Hkv, Hq, T, D = cfg.B, cfg.Hkv, cfg.Hq, cfg.T, cfg.D
    k = l2kv.l2kv_keep_count(T, cfg.keep_ratio)
    layers = [synth.make_layer(cfg, l, dev) for l in range(L)]
    queries = [synth.make_query(cfg, l, 0, dev) for l in range(L)]
    norms = torch.empty((B, Hkv, T), dtype=torch.float32, device=dev)
    rank = torch.empty((B, Hkv, T), dtype=torch.int32, device=dev)
    ws_r = torch.empty(l2kv.l2kv_norm_ranks_workspace_bytes(B * Hkv, T), dtype=torch.uint8, device=dev)
    ws_a = torch.empty(l2kv.l2kv_alr_workspace_bytes(B, Hq, T), dtype=torch.uint8, device=dev)
    out = [torch.empty((L, B, Hq), dtype=torch.float64, device=dev) for _ in range(3)]

    def one_pass(marks=None):
        for l in range(L):
            K = layers[l][0]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if marks is not None else None
            if e: e[0].record()
            l2kv.l2kv_norms(K, norms)
            if e: e[1].record()
            l2kv.l2kv_norm_ranks(norms, rank, ws_r)
            if e: e[2].record()
            l2kv.l2kv_alr(queries[l], K, rank, T - k, out[0][l], out[1][l], out[2][l], ws_a)
            if e:
                e[3].record()
                marks.append(e)

    for _ in range(args.warmup):
        one_pass()
    torch.cuda.synchronize()
    marks = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_pass(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in marks]).mean(axis=0)
    row = D * cfg.elem_bytes
    n = B * Hkv
    alr_bytes = n * T * row + 2 * B * Hq * T * 4 + n * T * 4      # K once, logits out and back in, ranks in
    Y, Lm, Lref = (o.cpu().numpy() for o in out)
    res = {
        "metric": "attention-loss analysis, query heads per second", "unit": "heads/s",
        "value": round(L * B * Hq * args.steps / wall, 1), "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall * 1e3 / args.steps, 3), "higher_is_better": True,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + " (attention-loss analysis, %d layers)" % L, "batch": B, "kv_heads": Hkv,
                   "q_heads": Hq, "head_dim": D, "cached_tokens": T, "dropped_pairs_m": T - k},
        "ms_per_layer": {"norms": round(float(ms[0]), 4), "norm_ranks": round(float(ms[1]), 4),
                         "alr": round(float(ms[2]), 4)},
        "alr_GBps": round(alr_bytes / ms[2] / 1e6, 1),
        "results": {"mean_Y_over_T": round(float(Y.mean()) / T, 6), "mean_loss": round(float(Lm.mean()), 6),
                    "mean_loss_ref": round(float(Lref.mean()), 6)},
    }
    print(json.dumps(res))


# ----------------------------------------------------------------------- main
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="C3", choices=sorted(synth.CONFIGS) + sorted(synth.STREAM_CONFIGS))
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debug)")
    ap.add_argument("--decode-steps", type=int, default=0, help="override decode steps (debug)")
    ap.add_argument("--cpu-layers", type=int, default=8)
    ap.add_argument("--cpu-decode-steps", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--decode-splits", type=int, default=0,
                    help="workgroups per KV head in decode attention (0 = the library's default plan); "
                         "for sweeps of the decomposition, not for the reported line")
    ap.add_argument("--no-seq-order", action="store_true",
                    help="streaming workloads: pass no stored launch order to the ragged attention calls "
                         "(the library then works one out per call; for comparisons)")
    ap.add_argument("--q-heads", type=int, default=0,
                    help="override the number of query heads (a multiple of the KV heads): other query-group "
                         "sizes at the workload's shape, for profiles")
    ap.add_argument("--one-call-slabs", default=None,
                    help="comma-separated slab sizes (heads; 0 = all at once) for the l2kv_compress timings; "
                         "'none' skips them (default: 0, one sequence's KV heads, one layer's heads)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default C3 run only: skip the short C4 and C5 passes reported under other_workloads")
    ap.add_argument("--alr", action="store_true",
                    help="time the attention-loss analysis (norm ranks + losses + Y) at the workload's "
                         "per-layer shape instead of the hot path")
    ap.add_argument("--placement-probe", action="store_true",
                    help="instead of the benchmark: read rate of the norm pass and time of a decode launch "
                         "against the position of the cache in device memory (fills the memory)")
    ap.add_argument("--placement-apart", type=int, default=100,
                    help="placement probe: distance in GiB between the K and the V tensor of its second decode map")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (torch) before the timed region: "
                         "the known-size kernel that scales the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
                 "(the path shards over KV heads with no exchange, but no multi-GPU "
                 "code is part of this build)" % args.gpus)
    if not torch.cuda.is_available():
        sys.exit("bench.py: no HIP device visible")
    l2kv.lib()                                   # fail loudly if the library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.placement_probe:
        return main_placement(args, dev)
    if args.workload in synth.STREAM_CONFIGS:
        return main_stream(args, dev)
    if args.alr:
        return main_alr(args, dev)
    cfg = synth.CONFIGS[args.workload]
    overridden = False
    if args.layers:
        cfg, overridden = cfg.scaled(L=args.layers), True
    if args.decode_steps:
        cfg, overridden = cfg.scaled(decode_steps=args.decode_steps), True
    if args.q_heads:
        cfg, overridden = cfg.scaled(Hq=args.q_heads), True
    slabs = None
    if args.one_call_slabs is not None:
        slabs = [] if args.one_call_slabs == "none" else [int(x) for x in args.one_call_slabs.split(",")]
    out = run_uniform(cfg, dev, args.steps, args.warmup, overridden, args.decode_splits, args.copy_probe,
                      0 if args.no_cpu_baseline else args.cpu_layers, args.cpu_decode_steps, slabs)
    out["device"] = device_facts(dev)
    if args.workload == "C3" and not overridden and not args.no_other_workloads:
        # one short pass each of the other two full-size workloads, same fields, so that their
        # figures come from the same run on the same box as the headline
        out["other_workloads"] = [
            run_uniform(synth.CONFIGS["C4"], dev, 2, 1, False, 0, False, 0 if args.no_cpu_baseline else 1, 1),
            run_stream(synth.STREAM_CONFIGS["C5"], dev, 1, 1, parity=not args.no_cpu_baseline),
        ]
    print(json.dumps(out))


def run_uniform(cfg, dev, steps, warmup, overridden, decode_splits, copy_probe, cpu_layers, cpu_decode_steps,
                one_call_slabs=None):
    w = Workload(cfg, dev, decode_splits)
    k = w.k
    nb, sb, cb = compress_bytes_per_layer(cfg, k)
    comp_bytes = (nb + sb + cb) * cfg.L
    dec_bytes_layer = decode_bytes_per_layer(cfg, k)
    dec_bytes = dec_bytes_layer * cfg.L * cfg.decode_steps
    step_bytes = comp_bytes + dec_bytes

    if copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        w.step()
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)     # noqa: E731
    marks = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        e = [ev() for _ in range(5)]
        e[0].record()
        l2kv.l2kv_norms(w.K, w.norms)
        e[1].record()
        l2kv.l2kv_select(w.norms, cfg.keep_ratio, w.idx, w.cnt, w.sel_ws)
        e[2].record()
        l2kv.l2kv_compact(w.K, w.V, w.idx, w.Kc, w.Vc)
        e[3].record()
        w.decode_all()
        e[4].record()
        marks.append(e)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in marks])  # [steps][4]
    norms_ms, select_ms, compact_ms, decode_ms = (float(x) for x in np.median(ms, axis=0))
    ms_per_step = wall * 1e3 / steps
    value = step_bytes / (wall / steps) / 1e9
    n_decode_launch = cfg.L * cfg.decode_steps
    us_per_layer_call = decode_ms * 1e3 / n_decode_launch
    achieved = dec_bytes_layer / (us_per_layer_call * 1e-6) / 1e9
    # the norm pass is this library's own pure read stream (it reads K once and writes 1.6 % of
    # that): what a read-only kernel reaches on this machine in this run
    read_stream = nb * cfg.L / norms_ms / 1e6
    # the bare read of the same K tensor (nothing computed, nothing stored): the ceiling of this
    # buffer on this machine in this run
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    probe_ms = []
    for _ in range(5):
        a, b = ev(), ev()
        a.record()
        l2kv.l2kv_read_probe(w.K, sink)
        b.record()
        torch.cuda.synchronize()
        probe_ms.append(a.elapsed_time(b))
    read_probe = w.K.numel() * w.K.element_size() / float(np.median(probe_ms[1:])) / 1e6

    out = {
        "metric": "compress+decode effective HBM GB/s",
        "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {
            "workload": cfg.name + (" (size overridden)" if overridden else ""),
            "layers": cfg.L, "batch": cfg.B, "kv_heads": cfg.Hkv, "q_heads": cfg.Hq,
            "head_dim": cfg.D, "cached_tokens": cfg.T, "keep_ratio": cfg.keep_ratio, "kept": k,
            "decode_steps": cfg.decode_steps,
            "step": "compress all layers once + decode_steps x layers decode-attention calls over the "
                    "static compacted cache (no row appended per decode step)",
            "decode_splits": decode_splits or "library default",
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "us_per_decode_step": round(decode_ms * 1e3 / cfg.decode_steps, 2),
        "us_per_decode_layer": round(us_per_layer_call, 3),
        "phase_times": "median over the timed steps (HIP events)",
        "phases": {
            "norms": {"ms": round(norms_ms, 4), "GBps": round(nb * cfg.L / norms_ms / 1e6, 1)},
            "select": {"ms": round(select_ms, 4), "GBps": round(sb * cfg.L / select_ms / 1e6, 1)},
            "compact": {"ms": round(compact_ms, 4), "GBps": round(cb * cfg.L / compact_ms / 1e6, 1)},
            "compress": {"ms": round(norms_ms + select_ms + compact_ms, 4),
                         "GBps": round(comp_bytes / (norms_ms + select_ms + compact_ms) / 1e6, 1)},
            "decode": {"ms": round(decode_ms, 4), "GBps": round(dec_bytes / decode_ms / 1e6, 1)},
        },
        "roofline": {
            "kernel": "decode attention (one l2kv_decode_attn call on one layer)",
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "read_stream_GBps": round(read_stream, 1),
            "pct_of_read_stream": round(100.0 * achieved / read_stream, 1),
            "read_stream": "the norm pass of the same run (reads K once and stores one float per row)",
            "read_probe_GBps": round(read_probe, 1),
            "pct_of_read_probe": round(100.0 * achieved / read_probe, 1),
            "read_probe": "l2kv_read_probe over the same K tensor after the timed steps: loads only, no store",
            "traffic": PROFILED_DECODE_TRAFFIC_BYTES.get((cfg.dtype, cfg.B, cfg.Hkv, cfg.Hq, cfg.D, k)),
            "traffic_unit": "bytes per launch; constant from an offline rocprofv3 --pmc profile "
                            "(profiles/hot_path_hbm_traffic_pmc.md), not measured by this run",
            "bytes_per_launch": dec_bytes_layer, "us_per_launch": round(us_per_layer_call, 3),
            "timing": "HIP events on the launch stream around all %d calls of each step" % n_decode_launch,
        },
    }
    # the compression step behind its single entry point, all heads at once and slab by slab
    # (slabs of one sequence's KV heads and of one layer's), a few repetitions each
    one_call = {}
    for slab in ((0, cfg.Hkv, cfg.B * cfg.Hkv) if one_call_slabs is None else one_call_slabs):
        ts = []
        for _ in range(3):
            a, b = ev(), ev()
            a.record()
            l2kv.l2kv_compress(w.K, w.V, cfg.keep_ratio, w.norms, w.idx, w.Kc, w.Vc, w.sel_ws, slab_heads=slab)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        one_call["slab_heads_%d" % slab] = {"ms": round(float(np.median(ts)), 4),
                                            "GBps": round(comp_bytes / float(np.median(ts)) / 1e6, 1)}
    out["phases"]["compress_one_call"] = one_call
    if cpu_layers > 0:
        layers = list(range(min(cpu_layers, cfg.L)))
        one, many = cpu_baseline(w, layers, min(cpu_decode_steps, cfg.decode_steps), host_threads())
        out["cpu_baseline"] = one
        if many is not None:
            out["cpu_baseline_all_cores"] = many
    del w
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
