#!/usr/bin/env python3
"""Benchmark of the decode hot path: constant-batch generation with continuous refill and in-flight
weight updates on one MI355X, on a synthetic workload shaped like the paper's long-form reasoning
generation (7B-shaped decoder, batch 256, 512-token prompts, log-normal generation lengths, weight
update from pinned host memory every 128 steps).

Prints ONE JSON line: generated tokens/s, the attention kernel's achieved HBM bandwidth against the
8 TB/s peak (HIP events recorded by the engine on its decode stream), and the CPU oracle timed on the
host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth  # noqa: E402

HBM_PEAK_GBS = 8000.0

WORKLOADS = {
    # name: model, batch, prompt, mean generation length, max generation length, swap period (steps)
    "7b": dict(model="7b", batch=256, prompt=512, mean=4096.0, gmax=16384, swap_every=128, pool_tokens=1_700_000),
    "1p5b": dict(model="1p5b", batch=64, prompt=256, mean=2048.0, gmax=8192, swap_every=256, pool_tokens=400_000),
    "tiny": dict(model="tiny", batch=4, prompt=16, mean=48.0, gmax=64, swap_every=32, pool_tokens=4 * 128),
    # 32B shape: two 65.5 GB weight buffers + 256 KiB of KV per token.  128 slots as the configuration asks; the
    # KV pool takes what is left of the 288 GB (pool_tokens = 0), which holds fewer tokens than 128 sequences at
    # the stationary context mix need, so refill is under admission control (see Workload.refill) and the batch
    # actually achieved is reported; total length lognormal(mean 6000), at most 16384
    "32b": dict(model="32b", batch=128, prompt=512, mean=5488.0, gmax=15872, swap_every=64, pool_tokens=0,
                host_staged=True, admission=True),
}


def _hip():
    return ctypes.CDLL("libamdhip64.so")


def device_weight_blob(eng, torch, seed, std=0.02, base=None, delta=0.0):
    """Synthetic weights generated on the device: matrices ~ N(0, std^2), gains 1 (or base + N(0, delta^2))."""
    n = eng.weight_nbytes() // 2
    g = torch.Generator(device="cuda").manual_seed(seed)
    blob = torch.empty(n, device="cuda", dtype=torch.bfloat16)
    step = 1 << 28
    for o in range(0, n, step):
        m = min(step, n - o)
        if base is None:
            blob[o:o + m] = (torch.randn(m, generator=g, device="cuda", dtype=torch.float32) * std).to(torch.bfloat16)
        else:
            blob[o:o + m] = (base[o:o + m].float() + torch.randn(m, generator=g, device="cuda", dtype=torch.float32) * delta).to(torch.bfloat16)
    if base is None:
        for name, off, (r, c) in eng.weight_layout():
            if c == 1:
                blob[off:off + r] = 1.0
    return blob


def host_staged_weights(eng, torch, seed, std=0.02, delta=1e-3):
    """For blobs too large to hold a spare copy in HBM or two copies in pinned memory (this host pins
    about 64 GiB): W is generated piecewise on the device into ONE pinned host buffer and loaded from
    there; the buffer is then overwritten, piece by piece, with W + N(0, delta^2), the blob every later
    update copies in.  Returns the pinned buffer."""
    n = eng.weight_nbytes() // 2
    host = torch.empty(n, dtype=torch.bfloat16, pin_memory=True)
    gains = [(off, r) for name, off, (r, c) in eng.weight_layout() if c == 1]
    step = 1 << 28
    for version in range(2):
        g = torch.Generator(device="cuda").manual_seed(seed)
        g2 = torch.Generator(device="cuda").manual_seed(seed + 1)
        for o in range(0, n, step):
            m = min(step, n - o)
            w = (torch.randn(m, generator=g, device="cuda", dtype=torch.float32) * std).to(torch.bfloat16)
            if version == 1:
                w = (w.float() + torch.randn(m, generator=g2, device="cuda", dtype=torch.float32) * delta).to(torch.bfloat16)
            host[o:o + m].copy_(w)
        torch.cuda.synchronize()
        for off, r in gains:
            host[off:off + r] = 1.0
        if version == 0:
            eng.load_weights(host.data_ptr(), eng.weight_nbytes())
    return host


def fill_kv_pool(eng, torch, seed):
    """N(0,1) bf16 values in every page, so that sequences admitted mid-flight attend over real data."""
    ptr, nbytes = eng.debug_kv_pool()
    hip = _hip()
    hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    g = torch.Generator(device="cuda").manual_seed(seed)
    chunk = 1 << 29
    off = 0
    while off < nbytes:
        m = min(chunk, nbytes - off)
        t = torch.randn(m // 2, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        torch.cuda.synchronize()
        rc = hip.hipMemcpy(ctypes.c_void_p(ptr + off), ctypes.c_void_p(t.data_ptr()), m, 3)  # device to device
        if rc != 0:
            raise RuntimeError(f"hipMemcpy failed: {rc}")
        off += m


class Workload:
    """Alg. 2's Actor loop around the engine: pop finished, refill to H, request a weight update every
    `swap_every` steps, generate next tokens."""

    def __init__(self, eng, spec, model, seed, batched_prefill=True, keep_history=False):
        self.eng, self.spec, self.model, self.batched_prefill = eng, spec, model, batched_prefill
        self.keep_history = keep_history
        self.rng = np.random.default_rng(seed)
        self.next_id = 0
        self.page_tokens = eng.cfg.kv_page_tokens or 128
        self.preempted = 0
        self.order = []                              # occupied slots, oldest admission first

    def preempt_youngest(self):
        """The pool ran dry although admission kept headroom: retire the sequence admitted last (it has
        the least work to lose).  Its tokens so far are dropped; counted in `preempted`."""
        slot = self.order.pop()
        self.eng.retire_sequence(slot)
        self.preempted += 1

    def _new_len(self):
        return int(synth.lognormal_lengths(self.rng, 1, self.spec["mean"], 1, self.spec["gmax"])[0])

    def admit_steady_state(self):
        """Fill every slot with a sequence at a random point of its life, drawn from the stationary law of
        constant-batch refill: a slot is busy for prompt + length - 1 steps when the prompt is read one
        token per step, for `length` steps when it is read in batched passes at admission."""
        B, P = self.spec["batch"], self.spec["prompt"]
        cand = synth.lognormal_lengths(self.rng, 200_000, self.spec["mean"], 1, self.spec["gmax"])
        first = P - 1 if self.batched_prefill else 0
        busy = cand + P - 1 - first
        g = self.rng.choice(cand, size=B, p=busy / busy.sum())
        for i in range(B):
            G = int(g[i])
            pos = int(self.rng.integers(first, P + G - 1))
            if not self._headroom_ok(pos + 1):
                break                                # the pool holds no more sequences at these ages
            prompt = synth.random_prompts(self.rng, 1, P, self.model.vocab)[0]
            slot = self.eng.debug_add_sequence_at(self.next_id, prompt, P, G, 1.0, pos, max(0, pos - (P - 1)),
                                                  int(self.rng.integers(0, self.model.vocab)))
            self.order.append(slot)
            if self.keep_history:   # tokens "read so far", so that the cache can be recomputed after an update
                hist = np.concatenate([prompt, self.rng.integers(0, self.model.vocab, max(0, pos - P))])[:pos]
                self.eng.debug_set_history(slot, hist)
            self.next_id += 1

    def _headroom_ok(self, extra_tokens):
        """Admission control for pools smaller than the batch's worst case: a sequence is admitted only if,
        after its prompt, the free pages still cover one more page for every sequence in flight plus a tenth
        of the pool (sequences keep growing; running dry would force a preemption)."""
        if not self.spec.get("admission"):
            return True
        st = self.eng.stats()
        page = self.page_tokens
        need = (extra_tokens + page - 1) // page + self.eng.num_active() + 1 + st["kv_pages_total"] // 10
        return st["kv_pages_free"] >= need

    def refill(self):
        P = self.spec["prompt"]
        while self.eng.num_active() < self.spec["batch"] and self._headroom_ok(P):
            prompt = synth.random_prompts(self.rng, 1, P, self.model.vocab)[0]
            slot = self.eng.add_sequence(self.next_id, prompt, self._new_len(), 1.0)
            self.order.append(slot)
            if self.batched_prefill == "background":
                self.eng.prefill_async(slot)
            elif self.batched_prefill:
                self.eng.prefill(slot)
            self.next_id += 1

    def step(self):
        try:
            out = self.eng.decode_step()
        except Exception as ex:                      # pool exhausted in spite of the headroom: preempt the youngest
            if getattr(ex, "code", None) != -3:
                raise
            self.preempt_youngest()
            out = self.eng.decode_step()
        if self.spec.get("admission") and self.eng.num_active() < self.spec["batch"]:
            self.refill()                            # pages freed earlier may admit a waiting sequence now
        fin = np.nonzero(out["finished"])[0]
        emitted = int(out["emitted"].sum())
        for i in fin:
            self.eng.retire_sequence(int(out["slot"][i]))
            self.order.remove(int(out["slot"][i]))
        if len(fin):
            self.refill()
        return emitted, out["step_ms"], out["swap_stall_ms"], out["weight_version"][0] if out["n"] else 0


def stream_ceiling(torch, pl, nontemporal=False):
    """Read bandwidth HBM delivers to a kernel that only reads (GB/s; ordinary or non-temporal loads),
    timed with events on torch's current stream, where the probe is launched."""
    buf = torch.empty(2 << 30, dtype=torch.uint8, device="cuda")
    buf.random_(0, 255)
    best = 0.0
    s = torch.cuda.current_stream()
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(s)
        n = pl.pl_debug_stream_read(buf.data_ptr(), buf.numel(), nontemporal, s.cuda_stream)
        b.record(s)
        torch.cuda.synchronize()
        best = max(best, n / (a.elapsed_time(b) * 1e-3) / 1e9)
    return best


PROFILE_OF = {"7b": "decode_step_7b_b256.md", "32b": "decode_step_32b_b128.md"}


def counter_traffic(workload, algorithmic_bytes):
    """HBM bytes one attention launch moved according to rocprofv3's counters: the committed summary of
    the counter runs states them as a multiple of the algorithmic bytes (a line `attn_traffic_ratio: x`);
    None where no such run was recorded."""
    path = os.path.join(ROOT, "profiles", PROFILE_OF.get(workload, ""))
    try:
        for line in open(path):
            if line.startswith("attn_traffic_ratio:"):
                return float(line.split(":")[1].split()[0]) * algorithmic_bytes
    except OSError:
        pass
    return None


def cpu_baseline_tiny():
    """The tiny configuration is small enough for the oracle to run the WHOLE workload: batch 4, 16-token
    prompts, 64 generated tokens each (4 x (16 + 64 - 1) slot-steps), one weight update landing at
    generated token 32, cache kept.  Timed on one thread and again with the BLAS library's default
    threads; generated tokens per second."""
    import threadpoolctl
    from oracle.engine import OracleEngine
    m = synth.CONFIGS["tiny"]
    master = synth.make_weights(m, seed=1235)
    w = [{k: synth.bf16_round(v).astype(np.float64) for k, v in ws.items()}
         for ws in (master, synth.perturb_weights(master, seed=1236))]
    prompts = synth.random_prompts(np.random.default_rng(77), 4, 16, m.vocab)

    def run():
        orc = OracleEngine(m, w[0], max_batch=4, seed=1)
        for i in range(4):
            orc.add_sequence(i, prompts[i], 64)
        t0 = time.perf_counter()
        emitted = 0
        for step in range(16 + 64 - 1):
            if step == 15 + 32:
                orc.swap_weights(w[1])
            emitted += sum(r.emitted for r in orc.decode_step())
        return emitted / (time.perf_counter() - t0)

    with threadpoolctl.threadpool_limits(1):
        single = run()
    multi = run()
    cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    return {"value": single, "unit": "tokens/s", "cores": 1, "kind": "oracle",
            "sample": "the whole tiny workload: 4 sequences x (16 prompt + 64 generated tokens), update at generated "
                      "token 32, float64, one thread",
            "all_cores": {"value": multi, "cores": int(cores)}}


def cpu_baseline(model, seconds_budget=20.0):
    """The CPU oracle as it stands, on the host cores: one layer + LM head of the workload's decoder
    for one decode step of sequences at the workload's mean context (float32), for about
    `seconds_budget` seconds, extrapolated linearly to all layers.  Reported in generated tokens/s."""
    from oracle import decoder
    m1 = model.with_layers(1)
    rng = np.random.default_rng(7)
    w = {}
    for name, shp in synth.weight_shapes(m1).items():
        if name == "embed":
            continue
        w[name] = np.ones(shp, np.float32) if len(shp) == 1 else (rng.standard_normal(shp, dtype=np.float32) * np.float32(0.02))
    w["embed"] = w["lm_head"]        # same shape; saves generating a second vocabulary-sized matrix
    rows, ctx = 64, 3900
    caches = []
    for _ in range(rows):
        c = decoder.Cache(m1, np.float32)
        c.k[0] = rng.standard_normal((ctx, m1.n_kv_heads, m1.head_dim), dtype=np.float32)
        c.v[0] = rng.standard_normal((ctx, m1.n_kv_heads, m1.head_dim), dtype=np.float32)
        caches.append(c)
    m0 = model.with_layers(0)
    # time the LM head alone (0 layers) and one layer + LM head; the difference is one layer
    t0 = time.perf_counter()
    heads = 0
    while heads < rows and (heads == 0 or time.perf_counter() - t0 < 0.25 * seconds_budget):
        decoder.step(m0, w, int(rng.integers(m1.vocab)), 0, decoder.Cache(m0, np.float32), np.float32)
        heads += 1
    t_head = (time.perf_counter() - t0) / heads
    t0 = time.perf_counter()
    done = 0
    while done < rows and (done == 0 or time.perf_counter() - t0 < 0.75 * seconds_budget):
        decoder.step(m1, w, int(rng.integers(m1.vocab)), ctx, caches[done], np.float32)
        done += 1
    t_one = (time.perf_counter() - t0) / done
    t_layer = max(t_one - t_head, 1e-9)
    per_token = t_head + model.n_layers * t_layer
    try:
        import threadpoolctl
        cores = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": 1.0 / per_token, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"1 layer + LM head, {done} sequences x {ctx} cached positions, float32, "
                      f"extrapolated to {model.n_layers} layers (one step = {per_token:.3f} s per sequence)"}


def batch_study(args):
    """Throughput against the number of sequences in flight (the shape of Fig. 2a), and the replay of a
    generation stage that is not refilled (Fig. 2b/2c: the batch decays as sequences finish).  Both use
    the workload's model shape and length law; prints one JSON line of its own."""
    import torch
    import paper_2509_19128_amd as pl

    spec = WORKLOADS[args.workload]
    model = synth.CONFIGS[spec["model"]]
    P, max_ctx = spec["prompt"], spec["prompt"] + spec["gmax"]
    rng = np.random.default_rng(4321)
    blob = None
    per_tok = 2 * model.n_layers * model.n_kv_heads * model.head_dim * 2

    def timed(B, contexts, steps=24, warmup=4):
        """tokens/s of decode steps for sequences at the given context lengths in an engine sized for B."""
        nonlocal blob
        ctxs = np.minimum(np.asarray(contexts, np.int64), max_ctx - steps - warmup - 2)
        pool = int(sum((int(c) + steps + warmup + 256) for c in ctxs)) + 1024
        eng = pl.Engine.from_model(model, max_batch=B, max_context=max_ctx, kv_pool_tokens=pool,
                                   n_weight_buffers=1, seed=99, device=0)
        if blob is None:
            blob = device_weight_blob(eng, torch, seed=1237)
            torch.cuda.synchronize()
        eng.load_weights(blob.data_ptr(), eng.weight_nbytes())
        fill_kv_pool(eng, torch, seed=7)
        for i, c in enumerate(ctxs):
            c = int(max(c, P - 1))
            eng.debug_add_sequence_at(i, rng.integers(0, model.vocab, P), P, max_ctx - P, 1.0, c, c - (P - 1),
                                      int(rng.integers(model.vocab)))
        for _ in range(warmup):
            eng.decode_step()
        s0 = eng.stats()
        t0 = time.perf_counter()
        for _ in range(steps):
            eng.decode_step()
        wall = time.perf_counter() - t0
        s1 = eng.stats()
        eng.close()
        toks = s1["tokens_emitted"] - s0["tokens_emitted"]
        return {"tokens_per_s": toks / wall, "ms_per_step": 1e3 * wall / steps,
                "gpu_ms_per_step": (s1["gpu_ms_total"] - s0["gpu_ms_total"]) / steps,
                "mean_context": float(np.mean(ctxs)), "hbm_GBs": (s1["algorithmic_bytes"] - s0["algorithmic_bytes"]) / wall / 1e9}

    # stationary context mix of the refilled batch (prompts already read): generation length drawn
    # length-biased, age uniform
    cand = synth.lognormal_lengths(rng, 200_000, spec["mean"], 1, spec["gmax"])
    sweep = []
    for B in [1, 2, 4, 8, 16, 32, 64, 128, 192, 256, 384, 512]:
        g = rng.choice(cand, size=B, p=cand / cand.sum())
        ctx = P - 1 + (rng.random(B) * g).astype(np.int64)
        r = timed(B, ctx)
        r["batch"] = B
        sweep.append(r)
        print(f"# batch {B}: {r['tokens_per_s']:.0f} tokens/s, {r['ms_per_step']:.2f} ms/step", file=sys.stderr, flush=True)
    # a stage that is not refilled: B sequences start together; after t steps those with length > t
    # are alive, all at context P - 1 + t
    B0 = spec["batch"]
    lens = synth.lognormal_lengths(rng, B0, spec["mean"], 1, spec["gmax"])
    decay, t = [], 0
    while True:
        alive = int((lens > t).sum())
        if alive == 0:
            break
        r = timed(B0, [P - 1 + t] * alive, steps=12, warmup=2)
        r.update(step=t, alive=alive)
        decay.append(r)
        print(f"# step {t}: {alive} alive, {r['tokens_per_s']:.0f} tokens/s", file=sys.stderr, flush=True)
        t += 1024
    total_tokens = int(lens.sum())
    # time of the whole stage from the sampled step times (trapezoid over the sampled points)
    ts = [d["step"] for d in decay] + [int(lens.max())]
    ms = [d["ms_per_step"] for d in decay] + [decay[-1]["ms_per_step"]]
    stage_s = sum(0.5 * (ms[i] + ms[i + 1]) * (ts[i + 1] - ts[i]) for i in range(len(ts) - 1)) / 1e3
    print(json.dumps({"study": "throughput against sequences in flight, and a generation stage without refill",
                      "workload": args.workload, "sweep": sweep, "decay": decay,
                      "decay_stage": {"sequences": B0, "tokens": total_tokens, "seconds": stage_s,
                                      "tokens_per_s": total_tokens / stage_s}}))


def is_ess_study(args):
    """The trainer-side reduction over one optimizer batch of recorded log-probs (Sec. 2.1): 1024 packed
    sequences with the workload's generation lengths; prints one JSON line of its own."""
    import torch
    import paper_2509_19128_amd as pl
    from oracle import importance

    spec = WORKLOADS["7b"]
    rng = np.random.default_rng(77)
    lens = synth.lognormal_lengths(rng, 1024, spec["mean"], 1, spec["gmax"])
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    n = int(off[-1])
    mu = (-rng.random(n) * 6).astype(np.float32)
    pi = (mu + rng.normal(0, 0.3, n)).astype(np.float32)
    d_pi, d_mu, d_off = (torch.from_numpy(x).cuda() for x in (pi, mu, off))
    w = torch.empty(n, device="cuda", dtype=torch.float32)
    sums = torch.empty((1024, 2), device="cuda", dtype=torch.float64)
    ess = torch.empty(1024, device="cuda", dtype=torch.float64)
    tot = torch.empty(3, device="cuda", dtype=torch.float64)
    s = torch.cuda.current_stream()
    call = lambda: pl.pl_is_ess(d_pi.data_ptr(), d_mu.data_ptr(), d_off.data_ptr(), 1024, 5.0, w.data_ptr(),
                                sums.data_ptr(), ess.data_ptr(), tot.data_ptr(), s.cuda_stream)
    for _ in range(args.warmup):
        call()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(s)
    for _ in range(args.steps):
        call()
    b.record(s)
    torch.cuda.synchronize()
    ms = a.elapsed_time(b) / args.steps
    nbytes = 12.0 * n + 8 * 1025 + 24 * 1024                      # 2 reads + 1 write per token, offsets, per-sequence outputs
    m = min(n, 400_000)                                           # oracle on a bounded sample of the same batch
    k = int(np.searchsorted(off, m, side="right")) - 1
    t0 = time.perf_counter()
    _, _, et = importance.packed_is_ess(pi[:off[k]], mu[:off[k]], off[:k + 1], 5.0)
    t_cpu = time.perf_counter() - t0
    print(json.dumps({"metric": "tokens/s through the truncated-importance-weight + ESS reduction", "value": n / (ms * 1e-3),
                      "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
                      "dtype": "f64", "data": "synthetic",
                      "config": {"workload": "1024 packed sequences, lognormal(4096, 0.75, max 16384) lengths", "tokens": n},
                      "ess_total": float(tot.cpu()[2]),
                      "roofline": {"bound": "hbm", "kernel": "is_seq_kernel (+ is_total_kernel)", "achieved": nbytes / (ms * 1e-3) / 1e9,
                                   "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None},
                      "cpu_baseline": {"value": int(off[k]) / t_cpu, "unit": "tokens/s", "cores": 1, "kind": "oracle",
                                       "sample": f"first {k} sequences ({int(off[k])} tokens) of the same batch"}}))


GEMM_CFG = [("32x256", 32, 256), ("64x256", 64, 256), ("128x256", 128, 256), ("64x128", 64, 128), ("128x128", 128, 128),
            ("256x128", 256, 128), ("64x64", 64, 64), ("128x64", 128, 64), ("32x128", 32, 128), ("128x64P", 128, 64),
            ("256x64P", 256, 64)]


def gemm_sweep(args):
    """Every tile configuration and K split of the GEMM kernel on the five products of one layer of the
    workload's decoder (rows = its batch), through pl_debug_gemm_cfg.  Weights are cold (each measurement
    walks 6-64 distinct copies of the matrix back to back, more bytes than any cache holds), the chip rests
    4 ms before each measurement (sustained MFMA load lowers the clock, which would favour whatever is
    measured first), the order is reshuffled every round; median of `--steps` rounds.  Prints one text table."""
    import random
    import torch
    import paper_2509_19128_amd as pl

    spec = WORKLOADS[args.workload]
    m = synth.CONFIGS[spec["model"]]
    M, d, F = spec["batch"], m.d_model, m.d_ffn
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    products = [("QKV", qd + 2 * kvd, d, 0), ("O", d, qd, 0), ("gate/up + SwiGLU", 2 * F, d, 1), ("down", d, F, 0),
                ("LM head", m.vocab, d, 0)]

    def valid(K, sp):
        total = K // 256
        return 1 <= sp <= total and (sp - 1) * ((total + sp - 1) // sp) < total

    print(f"# GEMM sweep, {args.workload} shape, M = {M} rows; us per launch (median of {args.steps} rounds), weights TB/s, TFLOP/s")
    for tag, N, K, mode in products:
        x = torch.randn(M, K, device="cuda").to(torch.bfloat16)
        w = (torch.randn(N, K, device="cuda") * 0.02).to(torch.bfloat16)
        wo = torch.from_numpy(pl.operand_order(w.view(torch.int16).cpu().numpy())).cuda()
        copies = int(min(64, max(6, -(-700_000_000 // (N * K * 2)))))
        wos = [wo] + [wo.clone() for _ in range(copies - 1)]
        wide = N >= 32768
        cands = []
        for cfg, (name, rows, cols) in enumerate(GEMM_CFG):
            rt = (M + rows - 1) // rows
            if (mode == 1 and name in ("64x64", "128x64", "32x128")) or rt > 4 or (rows >= 2 * M and rows > 32):
                continue
            for sp in ([1] if wide else [1, 2, 3, 4, 6, 8, 9, 12]):
                if not valid(K, sp) or ((N + cols - 1) // cols) * rt * sp > 4096:
                    continue
                for paired in ((False, True) if sp == 1 and rt > 1 else (False,)):
                    cands.append((cfg, sp, paired))
        spmax = max(c[1] for c in cands)
        ws = torch.empty(spmax * M * N, device="cuda", dtype=torch.float32)
        y = ws if mode == 0 else torch.zeros(M * N // 2, device="cuda", dtype=torch.bfloat16)
        yw = torch.empty(spmax * M * N, device="cuda", dtype=torch.float32) if mode == 0 else ws
        times, bad = {c: [] for c in cands}, set()
        for r in range(args.steps + 1):
            order = cands[:]
            random.Random(r).shuffle(order)
            for c in order:
                if c in bad:
                    continue
                cfg, sp, paired = c
                torch.cuda.synchronize()
                time.sleep(0.004)
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                try:
                    a.record()
                    for i in range(copies):
                        pl.pl_debug_gemm_cfg(cfg, x.data_ptr(), wos[i].data_ptr(), (yw if mode == 0 else y).data_ptr(), ws.data_ptr(),
                                             M, N, K, mode, sp, 0, N, paired, 0)
                    b.record()
                    torch.cuda.synchronize()
                except pl.PlError:
                    bad.add(c)
                    continue
                if r:
                    times[c].append(a.elapsed_time(b) * 1e3 / copies)
        res = sorted((float(np.median(times[c])), c) for c in cands if c not in bad)
        print(f"== {tag}: N {N}, K {K}, weights {N * K * 2 / 1e6:.1f} MB, {copies} copies walked")
        for t, (cfg, sp, paired) in res[:8]:
            print(f"   {GEMM_CFG[cfg][0]:8s} slices {sp:2d}{' paired' if paired else '       '}: {t:7.1f} us  {N * K * 2 / t / 1e6:5.2f} TB/s  {2 * M * N * K / t / 1e6:5.0f} TFLOP/s")
        sys.stdout.flush()
        del wos, wo, w, ws, y, yw
        torch.cuda.empty_cache()


def attention_microbench(args):
    """One decode-attention step over a paged bf16 cache: batch 512, 28 q / 4 kv heads, head_dim 128,
    contexts lognormal(4096) clipped to [128, 16384], q/K/V ~ N(0,1); median over `--steps` launches (the
    4 GB of K/V exceed every cache, so consecutive launches do not help each other).  One JSON line."""
    import torch
    import paper_2509_19128_amd as pl
    from oracle import decoder

    B, Hq, Hkv, hd, pt = 512, 28, 4, 128, 128
    ctx = synth.attention_microbench_lengths(1236).astype(np.int32)
    need = (ctx + pt - 1) // pt
    n_pages, pps = int(need.sum()) + 4, int(need.max())
    rng = np.random.default_rng(0)
    perm = rng.permutation(n_pages).astype(np.int32)
    table = np.zeros((B, pps), np.int32)
    k = 0
    for b in range(B):
        table[b, :need[b]] = perm[k:k + need[b]]
        k += need[b]
    pe = Hkv * 2 * pt * hd
    pool = torch.empty(n_pages * pe, device="cuda", dtype=torch.bfloat16)
    g = torch.Generator(device="cuda").manual_seed(5)
    for o in range(0, n_pages * pe, 1 << 28):
        m = min(1 << 28, n_pages * pe - o)
        pool[o:o + m] = torch.randn(m, generator=g, device="cuda").to(torch.bfloat16)
    q = torch.randn(B, Hq, hd, generator=g, device="cuda").to(torch.bfloat16)
    out = torch.zeros(B, Hq, hd, device="cuda", dtype=torch.bfloat16)
    ws = torch.empty(pl.pl_attention_workspace_bytes(B, Hq, Hkv, hd, int(ctx.max())), device="cuda", dtype=torch.uint8)
    tb, cl = torch.from_numpy(table).cuda(), torch.from_numpy(ctx).cuda()
    s = torch.cuda.current_stream()
    times = []
    for i in range(args.warmup + args.steps):
        a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(s)
        pl.pl_attention_decode(q.data_ptr(), pool.data_ptr(), tb.data_ptr(), cl.data_ptr(), out.data_ptr(), ws.data_ptr(),
                               B, Hq, Hkv, hd, pt, pps, int(ctx.max()), s.cuda_stream)
        e.record(s)
        torch.cuda.synchronize()
        if i >= args.warmup:
            times.append(a.elapsed_time(e))
    ms = float(np.median(times))
    nbytes = float(ctx.sum()) * Hkv * hd * 2 * 2
    # oracle on a bounded sample: the shortest sequences of the batch, one by one, float64
    order = np.argsort(ctx)[:8]
    t0 = time.perf_counter()
    toks = 0
    for b in order:
        c = int(ctx[b])
        K, V = rng.standard_normal((c, Hkv, hd)), rng.standard_normal((c, Hkv, hd))
        decoder.attend_one(rng.standard_normal((Hq, hd)), K, V)
        toks += c
    t_cpu = time.perf_counter() - t0
    print(json.dumps({"metric": "decode attention, K/V bytes per second", "value": nbytes / (ms * 1e-3) / 1e9, "unit": "GB/s",
                      "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True,
                      "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "decode-attention microbenchmark: batch 512, 28 q / 4 kv heads, head_dim 128, "
                                             "contexts lognormal(4096) in [128, 16384], 128-token pages", "mean_context": float(ctx.mean())},
                      "roofline": {"bound": "hbm", "kernel": "attn_worklist_kernel + attn_decode_kernel + attn_combine_kernel",
                                   "achieved": nbytes / (ms * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                   "frac": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": nbytes},
                      "cpu_baseline": {"value": toks * Hkv * hd * 4 / t_cpu / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                                       "sample": f"the 8 shortest sequences ({toks} cached tokens), float64, counted at 2 bytes per element"}}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--attn-microbench", action="store_true",
                    help="instead of the benchmark line: the decode-attention microbenchmark (batch 512, one step)")
    ap.add_argument("--is-ess", action="store_true",
                    help="instead of the benchmark line: time the importance-weight / ESS reduction on one optimizer batch")
    ap.add_argument("--gemm-sweep", action="store_true",
                    help="instead of the benchmark line: every GEMM tile configuration and K split on the workload's five products")
    ap.add_argument("--batch-study", action="store_true",
                    help="instead of the benchmark line: throughput against batch size and a replay of a stage without refill")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1024)
    ap.add_argument("--warmup", type=int, default=16)
    ap.add_argument("--workload", default="7b", choices=sorted(WORKLOADS))
    ap.add_argument("--prefill", default="background", choices=["background", "batched", "decode"],
                    help="how a refilled slot reads its prompt: batched passes on a stream of their own while the other "
                         "slots keep decoding, batched passes that block, or one token per decode step")
    ap.add_argument("--recompute-kv", action="store_true",
                    help="weight updates rebuild every sequence's KV cache under the new weights (Sec. 5.1 variant; slow)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not record per-kernel HIP events")
    ap.add_argument("--profile-every", type=int, default=8,
                    help="HIP events around the attention kernel on every N-th timed step (such a step launches its "
                         "kernels one by one; the others replay the captured graph); 1 = every step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="finish with three plain 1 GiB device copies (known traffic, for scaling rocprofv3 counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one engine replica on one GPU; data-parallel replicas are independent "
              "and are not launched here (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    if args.gemm_sweep:
        return gemm_sweep(args)
    if args.batch_study:
        return batch_study(args)
    if args.is_ess:
        return is_ess_study(args)
    if args.attn_microbench:
        return attention_microbench(args)

    import torch
    import paper_2509_19128_amd as pl

    spec = WORKLOADS[args.workload]
    model = synth.CONFIGS[spec["model"]]
    max_ctx = spec["prompt"] + spec["gmax"]
    eng = pl.Engine.from_model(model, max_batch=spec["batch"], max_context=max_ctx,
                               kv_pool_tokens=spec["pool_tokens"], n_weight_buffers=2, seed=1234 + 3, device=0)
    if spec.get("host_staged"):
        hw = host_staged_weights(eng, torch, seed=1237)
        host = [hw, hw]      # every update copies the same blob in: the copy and the flip are what is measured
        torch.cuda.empty_cache()
    else:
        w0 = device_weight_blob(eng, torch, seed=1237)
        torch.cuda.synchronize()
        eng.load_weights(w0.data_ptr(), eng.weight_nbytes())
        # the "next optimizer step" weights wait in pinned host memory, as a trainer's broadcast buffer would
        w1 = device_weight_blob(eng, torch, seed=1238, base=w0, delta=1e-3)
        host = [torch.empty(w0.numel(), dtype=torch.bfloat16, pin_memory=True) for _ in range(2)]
        host[0].copy_(w1)
        host[1].copy_(w0)
        torch.cuda.synchronize()
        del w0, w1
        torch.cuda.empty_cache()
    fill_kv_pool(eng, torch, seed=1239)

    wl = Workload(eng, spec, model, seed=1234 + 3, batched_prefill={"background": "background", "batched": True, "decode": False}[args.prefill],
                  keep_history=args.recompute_kv)
    wl.admit_steady_state()
    # The dominant kernel is timed live, with HIP events around it on the engine's decode stream, on every
    # `profile_every`-th step of the timed window: a step with events cannot replay its captured graph and pays
    # the launches (0.5-0.8 ms of host time at 7B), so the window keeps most steps the way the product runs them.
    prof_every = max(1, args.profile_every)
    eng.debug_set_profile(0)
    step_ms, stalls, flips, requests = [], [], [], []
    swaps_requested = 0

    def request_update(k):
        """Alg. 2: the trainer requests an update; the engine stages it while decoding goes on."""
        nonlocal swaps_requested
        try:
            eng.swap_weights(host[swaps_requested % 2].data_ptr(), eng.weight_nbytes(),
                             flags=pl.PL_SWAP_ASYNC | (pl.PL_SWAP_RECOMPUTE_KV if args.recompute_kv else 0))
            swaps_requested += 1
            requests.append(k)
        except pl.PlError as ex:
            if ex.code != pl.PL_E_BUSY:
                raise

    # Updates arrive every `swap_every` steps; where that cycle stands when the timed window opens is
    # arbitrary.  A window of at least one period takes the first request half a period in.  A shorter
    # window would otherwise contain no update at all, so its one request is issued during the warm-up, at
    # the step from which the staging copy (its duration predicted from a timed 256 MiB copy out of the same
    # pinned buffer) ends nearest the middle of the timed window: the window then holds steps that overlap
    # the copy, the flip, and steps after it (this charges the window one update per `steps` instead of
    # one per `swap_every`).  If the copy outlasts warm-up + window, the line says the window holds no flip.
    every = spec["swap_every"]
    short_window = bool(every) and args.steps < every
    copy_est = None
    if short_window:
        n_probe = min(host[0].numel(), 1 << 27)
        probe = torch.empty(n_probe, dtype=torch.bfloat16, device="cuda")
        probe.copy_(host[0][:n_probe], non_blocking=True)
        torch.cuda.synchronize()
        tp = time.perf_counter()
        probe.copy_(host[0][:n_probe], non_blocking=True)
        torch.cuda.synchronize()
        copy_est = (time.perf_counter() - tp) * host[0].numel() / n_probe
        del probe
    warm_wall = []
    for i in range(args.warmup):
        if short_window and not requests and i >= min(2, args.warmup - 1):
            # wall time of a step from the warm-up steps so far (the first one pays one-off start-up costs)
            est = float(np.mean(warm_wall[1:])) if len(warm_wall) > 1 else None
            lands = None if est is None else (copy_est - (args.warmup - i) * est) / (args.steps * est)
            if lands is None or lands >= 0.3 or i == args.warmup - 1:
                request_update(i - args.warmup)
        tw = time.perf_counter()
        wl.step()
        warm_wall.append(time.perf_counter() - tw)
    if short_window and not requests:
        request_update(0)
    # no device-wide synchronisation here: it would wait for the staging copy; every step has already
    # returned its tokens, so the decode stream is idle
    s0 = eng.stats()
    emitted = 0
    last_version = s0["active_version"]
    t0 = time.perf_counter()
    for k in range(args.steps):
        if every and not short_window and k % every == every // 2:
            request_update(k)
        if not args.no_profile:
            eng.debug_set_profile(1 if k % prof_every == 0 else 0)   # events around the attention kernel only
        e, ms, stall, ver = wl.step()
        emitted += e
        step_ms.append(ms)
        stalls.append(stall)
        if ver != last_version:
            flips.append(k)
            last_version = ver
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    s1 = eng.stats()

    # a short extra pass with events around every kernel group, for the time split only
    split = None
    if not args.no_profile:
        eng.debug_set_profile(2)
        a0 = eng.stats()
        for _ in range(16):
            wl.step()
        a1 = eng.stats()
        eng.debug_set_profile(0)
        split = {k: (a1[k] - a0[k]) / 16 for k in ("attn_ms", "gemm_ms", "sample_ms", "other_ms")}

    d = {k: s1[k] - s0[k] for k in ("steps", "tokens_emitted", "slot_steps", "gpu_ms_total", "algorithmic_bytes",
                                     "attn_ms", "gemm_ms", "sample_ms", "other_ms", "attn_launches", "attn_kv_bytes",
                                     "attn_shared_ms", "attn_shared_launches", "attn_shared_kv_bytes",
                                     "host_enqueue_ms", "host_wait_ms")}
    sm = np.asarray(step_ms)
    med = float(np.median(sm))
    # swap stall: the step that contains the flip against the median of the 16 surrounding steps (None if no
    # flip fell inside the timed window: nothing was measured then)
    stall_ms, stall_each = None, []
    for k in flips:
        lo, hi = max(0, k - 8), min(len(sm), k + 9)
        around = np.concatenate([sm[lo:k], sm[k + 1:hi]])
        if len(around):
            stall_each.append(float(sm[k] - np.median(around)) + float(stalls[k]))
            stall_ms = max(stall_ms or 0.0, stall_each[-1])
    # interference: decode steps that run while a staging copy is in flight (request .. flip) against the rest
    during = np.zeros(len(sm), bool)
    for rq in requests:
        fl = [f for f in flips if f >= rq]
        during[max(rq, 0):(fl[0] if fl else len(sm))] = True
    interference = float(sm[during].mean() - sm[~during].mean()) if during.any() and (~during).any() else None
    res = {
        "metric": "generated tokens/s/GPU at constant batch", "value": emitted / wall, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * wall / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload}-shaped decoder, constant batch {spec['batch']} with continuous refill, "
                               f"{spec['prompt']}-token prompts, lognormal(mean {spec['mean']:.0f}, sigma 0.75, max {spec['gmax']}) "
                               f"generation lengths, steady-state ages, weight update from pinned host every {spec['swap_every']} steps, "
                               "prompts read " + {"background": "in batched passes in the background, overlapped with decode steps",
                                                   "batched": "in batched passes at admission", "decode": "one token per step"}[args.prefill],
                   "mean_context": d["algorithmic_bytes"] and float((d["attn_kv_bytes"] / max(d["attn_launches"], 1)) /
                                                                    (4.0 * model.n_kv_heads * model.head_dim) / spec["batch"]),
                   "slot_utilisation": d["tokens_emitted"] / max(d["slot_steps"], 1),
                   "mean_batch": d["slot_steps"] / max(d["steps"], 1), "preempted": wl.preempted,
                   "kv_pool_tokens": s1["kv_pages_total"] * wl.page_tokens},
        "host_ms_per_step": {"enqueue": d["host_enqueue_ms"] / max(d["steps"], 1), "wait_for_gpu": d["host_wait_ms"] / max(d["steps"], 1),
                             "outside_the_engine": (1e3 * wall - d["host_enqueue_ms"] - d["host_wait_ms"]) / max(d["steps"], 1),
                             "gpu_mean": d["gpu_ms_total"] / max(d["steps"], 1)},
        "gpu_ms_per_step_median": med, "gpu_ms_per_step_p99": float(np.percentile(sm, 99)),
        "step_hbm": {"algorithmic_bytes_per_step": d["algorithmic_bytes"] / max(d["steps"], 1),
                     "achieved_GBs": d["algorithmic_bytes"] / max(d["gpu_ms_total"], 1e-9) / 1e6,
                     "frac_of_8TBs": d["algorithmic_bytes"] / max(d["gpu_ms_total"], 1e-9) / 1e6 / HBM_PEAK_GBS},
        "swap": {"requested": swaps_requested, "requested_at_steps": requests, "flips_at_steps": flips,
                 "window_contains_a_flip": bool(flips), "stall_ms": stall_ms,
                 # per flip; a flip step that also shares the GPU with a background prompt-reading pass shows that
                 # pass's slowdown here (a few ms), not a wait for the update
                 "stall_ms_per_flip": stall_each,
                 "steps_overlapping_a_copy": int(during.sum()), "interference_ms_per_overlapping_step": interference,
                 "copy_ms": s1["last_swap_copy_ms"], "blob_GB": eng.weight_nbytes() / 1e9,
                 "kv_cache": "recomputed at the flip" if args.recompute_kv else "kept",
                 "recompute_positions": s1["recompute_positions"] - s0["recompute_positions"],
                 "recompute_passes": s1["recompute_passes"] - s0["recompute_passes"],
                 "recompute_gpu_ms": s1["recompute_ms"] - s0["recompute_ms"]},
        "time_split_ms_per_step": split,
        "prefill": {"mode": args.prefill, "positions": s1["prefill_positions"] - s0["prefill_positions"],
                    "passes": s1["prefill_passes"] - s0["prefill_passes"], "gpu_ms": s1["prefill_ms"] - s0["prefill_ms"]},
    }
    res["hbm_read_stream_ceiling_GBs"] = stream_ceiling(torch, pl)
    res["hbm_read_stream_ceiling_nontemporal_GBs"] = stream_ceiling(torch, pl, nontemporal=True)
    if d["attn_launches"]:
        # The kernel's figure is taken from the launches that had the GPU to themselves; launches of steps that
        # shared it with a background prompt-reading pass or with the staging copy of an update are reported beside it.
        alone = d["attn_launches"] - d["attn_shared_launches"]
        if alone:
            per_launch_bytes = (d["attn_kv_bytes"] - d["attn_shared_kv_bytes"]) / alone
            per_launch_ms = (d["attn_ms"] - d["attn_shared_ms"]) / alone
        else:
            per_launch_bytes, per_launch_ms = d["attn_kv_bytes"] / d["attn_launches"], d["attn_ms"] / d["attn_launches"]
        ach = per_launch_bytes / per_launch_ms / 1e6
        res["roofline"] = {"bound": "hbm", "kernel": "attn_decode_kernel", "achieved": ach, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                           "launches": int(alone or d["attn_launches"]),
                           "timed_on": f"one timed step in {prof_every}" if prof_every > 1 else "every timed step",
                           "launches_beside_a_background_pass_or_copy": int(d["attn_shared_launches"]),
                           "achieved_beside_a_background_pass_or_copy": (d["attn_shared_kv_bytes"] / d["attn_shared_ms"] / 1e6
                                                                 if d["attn_shared_launches"] else None),
                           # HBM bytes per launch from the rocprofv3 counter runs of this same command
                           # (FETCH_SIZE and WRITE_SIZE, scaled on plain copies), as recorded in profiles/
                           "traffic": counter_traffic(args.workload, per_launch_bytes),
                           "bytes_per_launch": per_launch_bytes, "ms_per_launch": per_launch_ms}
    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_tiny() if args.workload == "tiny" else cpu_baseline(model)
    eng.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
