#!/usr/bin/env python3
"""Benchmark of the rollout hot path on one MI355X.

One step = what one decode step plus the scoring of the generated positions
costs on the hot path: append one token's K/V per sequence to the arena,
single-token decode attention over the paged cache, and the fused token
log-prob / actor-vs-reference KL over the full logit matrices.  Inputs are
synthetic, seeded, and resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is the algorithmic HBM traffic of a whole step
divided by the step time; the per-kernel figures (decode-attention GB/s and its
fraction of peak, log-prob/KL positions per second) are in `components`.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X, HBM3E
METRIC = "decode-attn HBM GB/s (% of MI355X peak) + logprob/KL tokens/sec, 1 GPU"


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by a plain
# 1 GiB copy) are kept, with the hash of the kernel sources they were taken on, in the lines
#   traffic <name> workload=<index> bytes=<n> sha256=<hash of the listed sources>
# of this summary; they hold only while the sources still hash to that value.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_cfg5_gqa70b_hbm_traffic.txt")
TRAFFIC_SOURCES = {
    "logprob_kl": ["logprob_kl.hip", "device_ops.h"],
    "decode_attn": ["attention.hip", "mfma_ops.h", "device_ops.h"],
    "prefill_attn": ["prefill.hip", "mfma_ops.h", "device_ops.h"],
}


def sources_hash(name):
    import hashlib
    h = hashlib.sha256()
    for f in TRAFFIC_SOURCES[name]:
        h.update(open(os.path.join(ROOT, "paper_2410_15651_amd", "csrc", f), "rb").read())
    return h.hexdigest()


def measured_traffic(name, cfg_index):
    """Counter-measured HBM bytes per launch from the profile summary, or None --
    said loudly on stderr -- when the kernel has changed since the counters were
    taken, or for a workload the summary does not cover."""
    try:
        lines = open(TRAFFIC_PROFILE).read().splitlines()
    except OSError:
        log(f"bench.py: {TRAFFIC_PROFILE} is missing: roofline traffic of {name} reported as null")
        return None
    for line in lines:
        f = line.split()
        if len(f) == 5 and f[0] == "traffic" and f[1] == name and f[2] == f"workload={cfg_index}":
            if f[4] == "sha256=" + sources_hash(name):
                return int(f[3].split("=")[1])
            log(f"bench.py: {name} has changed since its HBM counters were taken "
                f"({os.path.relpath(TRAFFIC_PROFILE, ROOT)}): roofline traffic reported as null; re-run the two "
                f"rocprofv3 --pmc commands named in that file and update its 'traffic' line")
            return None
    return None


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def attention_bytes(lens, cfg, eb=2):
    """Algorithmic bytes of one decode-attention call: K and V of every cached
    token once, q in and out out, page ids and lengths."""
    P = 16
    lens = lens.astype(np.int64)
    kv = 2 * lens.sum() * cfg.n_kv_heads * cfg.head_dim * eb
    qo = 2 * cfg.batch * cfg.n_q_heads * cfg.head_dim * eb
    ids = 4 * ((lens + P - 1) // P).sum() + 4 * cfg.batch
    return int(kv + qo + ids)


def logprob_bytes(n, vocab, lb):
    return int(n) * (2 * vocab * lb + 4 + 8)


def append_bytes(cfg, eb=2):
    return 2 * 2 * cfg.batch * cfg.n_kv_heads * cfg.head_dim * eb   # rows read + written, K and V


class Workload:
    """Inputs of one configuration, resident in HBM, in `n_sets` independent copies
    (own arena, own logits) that the steps rotate through, so that a small working
    set is not simply served from the 256 MB last-level cache."""

    def __init__(self, cfg, steps_total, n_sets, dev):
        import torch
        from paper_2410_15651_amd import binding as rb
        from paper_2410_15651_amd import workloads as wl
        self.cfg, self.rb, self.torch = cfg, rb, torch
        P = wl.PAGE_TOKENS
        self.lens = wl.seq_lengths(cfg)
        self.q, self.ks, self.vs = wl.qkv(cfg, self.lens, device=dev)
        extra = steps_total + 1
        self.mpps = cfg.max_pages_per_seq(extra)
        n_pages = int(((self.lens.astype(np.int64) + extra + P - 1) // P).sum()) + 8
        order = wl.free_order(cfg, n_pages)
        kw = dict(max_seqs=cfg.batch, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, n_pages=n_pages,
                  max_pages_per_seq=self.mpps, kv_dtype=wl.DTYPE_CODE[cfg.kv_dtype], initial_free_order=order)
        self.arena_bytes = rb.rlhf_kv_arena_bytes_required(**kw)
        self.sets = []
        for i in range(n_sets):
            buf = torch.empty(self.arena_bytes, dtype=torch.uint8, device=dev)
            arena = rb.rlhf_kv_arena_create(device_buffer=buf, device_buffer_bytes=self.arena_bytes, **kw)
            done = np.zeros(cfg.batch, dtype=np.int64)
            for ids, n_new in wl.fill_schedule(cfg, self.lens, hold_back=0):
                k_new = torch.cat([self.ks[b][done[b]:done[b] + n] for b, n in zip(ids, n_new)]).contiguous()
                v_new = torch.cat([self.vs[b][done[b]:done[b] + n] for b, n in zip(ids, n_new)]).contiguous()
                rb.rlhf_kv_arena_append(arena, ids, n_new, k_new, v_new)
                done[ids] += n_new
            if i == 0:
                actor, ref = wl.logits(cfg, device=dev)
            else:                      # same values, different memory
                actor, ref = self.sets[0]["actor"].clone(), self.sets[0]["ref"].clone()
            self.sets.append(dict(buf=buf, arena=arena, views=rb.rlhf_kv_arena_views(arena), actor=actor,
                                  ref=ref, appended=0))
        g = torch.Generator(device=dev)
        g.manual_seed(cfg.seed)
        self.step_k = (torch.randn(cfg.batch, cfg.n_kv_heads, cfg.head_dim, generator=g, device=dev)
                       * cfg.qkv_std).to(self.q.dtype)
        self.step_v = (torch.randn(cfg.batch, cfg.n_kv_heads, cfg.head_dim, generator=g, device=dev)
                       * cfg.qkv_std).to(self.q.dtype)
        self.tok_np = wl.tokens(cfg)
        self.tok = torch.from_numpy(self.tok_np).to(dev)
        n = cfg.n_positions
        self.logp = torch.empty(n, dtype=torch.float32, device=dev)
        self.kl = torch.empty(n, dtype=torch.float32, device=dev)
        self.params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, self.mpps,
                                     wl.DTYPE_CODE[cfg.kv_dtype], max_seq_len=cfg.len_hi + extra)
        self.ws = torch.empty(rb.rlhf_decode_attention_workspace_bytes(self.params), dtype=torch.uint8, device=dev)
        self.out = torch.empty(cfg.batch, cfg.n_q_heads, cfg.head_dim, dtype=self.q.dtype, device=dev)
        self.seq_ids = np.arange(cfg.batch, dtype=np.int32)
        self.ones = np.ones(cfg.batch, dtype=np.int32)
        torch.cuda.synchronize()

    def step(self, i, marks=None):
        rb, torch = self.rb, self.torch
        s = self.sets[i % len(self.sets)]
        k_arena, v_arena, d_table, d_lens = s["views"]
        e = [torch.cuda.Event(enable_timing=True) for _ in range(4)] if marks is not None else None
        if e:
            e[0].record()
        rb.rlhf_kv_arena_append(s["arena"], self.seq_ids, self.ones, self.step_k, self.step_v)
        s["appended"] += 1
        if e:
            e[1].record()
        rb.rlhf_decode_attention(self.params, self.q, k_arena, v_arena, d_table, d_lens, self.out, self.ws)
        if e:
            e[2].record()
        rb.rlhf_token_logprobs_kl(s["actor"], s["ref"], self.tok, self.logp, self.kl)
        if e:
            e[3].record()
            marks.append((e, attention_bytes(self.lens.astype(np.int64) + s["appended"], self.cfg)))

    def close(self):
        for s in self.sets:
            self.rb.rlhf_kv_arena_destroy(s["arena"])
        self.sets = []


def time_calls(torch, call, n_calls, n_batches=5, warmup=10):
    """Per-call time of call(i): `warmup` untimed calls, then `n_batches` batches of
    `n_calls` calls, each batch between two events on the stream the calls run on.
    Returns (median, min, max) over the batches, in seconds per call."""
    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    per_call = []
    k = warmup
    for _ in range(n_batches):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_calls):
            call(k)
            k += 1
        e1.record()
        torch.cuda.synchronize()
        per_call.append(e0.elapsed_time(e1) * 1e-3 / n_calls)
    return float(np.median(per_call)), float(min(per_call)), float(max(per_call))


def measure_kernels(wk, n_attn=100, n_logp=100):
    """Decode attention and log-prob/KL each timed on its own, back to back calls
    (time_calls): `cold` rotates through the workload's input sets, whose K/V and
    logits together exceed the last-level cache, `hot` stays on the first set."""
    rb, torch, cfg = wk.rb, wk.torch, wk.cfg
    n_sets = len(wk.sets)

    def attn(rotate):
        def call(i):
            s = wk.sets[i % n_sets if rotate else 0]
            k_arena, v_arena, d_table, d_lens = s["views"]
            rb.rlhf_decode_attention(wk.params, wk.q, k_arena, v_arena, d_table, d_lens, wk.out, wk.ws)
        return call

    def logp(rotate):
        def call(i):
            s = wk.sets[i % n_sets if rotate else 0]
            rb.rlhf_token_logprobs_kl(s["actor"], s["ref"], wk.tok, wk.logp, wk.kl)
        return call

    lb = 4 if cfg.logits_dtype == "f32" else 2
    b_attn = attention_bytes(wk.lens.astype(np.int64) + wk.sets[0]["appended"], cfg)
    b_logp = logprob_bytes(cfg.n_positions, cfg.vocab, lb)
    out = {"method": f"median (min..max) of 5 batches; a batch is {n_attn} back-to-back attention calls or "
                     f"{n_logp} log-prob/KL calls between two events, after 10 warm-up calls",
           "rotating_input_sets": n_sets}
    for name, fn, n, nbytes in (("decode_attn", attn, n_attn, b_attn), ("logprob_kl", logp, n_logp, b_logp)):
        for mode, rotate in (("cold", True), ("hot", False)):
            med, lo, hi = time_calls(torch, fn(rotate), n)
            out[f"{name}_{mode}_us"] = round(med * 1e6, 2)
            out[f"{name}_{mode}_us_min_max"] = [round(lo * 1e6, 2), round(hi * 1e6, 2)]
            out[f"{name}_{mode}_GBps"] = round(nbytes / med / 1e9, 1)
            out[f"{name}_{mode}_frac_of_peak"] = round(nbytes / med / 1e9 / HBM_PEAK_GBPS, 4)
    out["logprob_kl_cold_tokens_per_s"] = round(cfg.n_positions / (out["logprob_kl_cold_us"] * 1e-6), 1)
    kv = n_sets * 2 * int(wk.lens.sum()) * cfg.n_kv_heads * cfg.head_dim * 2
    lg = n_sets * 2 * cfg.n_positions * cfg.vocab * lb
    out["cold_means"] = (f"rotation over {n_sets} input set(s): {kv / 1e6:.0f} MB of K/V and {lg / 1e6:.0f} MB of logits "
                         f"between two uses of the same bytes" +
                         ("" if kv > 512e6 else "; K/V rotation stays under 512 MB (capped at 12 sets): partly cache-resident"))
    return out


def rotation_sets(cfg):
    """Copies needed so that the rotated K/V and the rotated logits each exceed
    512 MB (more than the last-level cache holds), capped at 12."""
    lb = 4 if cfg.logits_dtype == "f32" else 2
    kv = (cfg.len_lo + cfg.len_hi) / 2 * cfg.batch * cfg.n_kv_heads * cfg.head_dim * 2 * 2
    lg = 2 * cfg.n_positions * cfg.vocab * lb
    need = max(512e6 / kv, 512e6 / lg)
    return int(min(12, max(1, np.ceil(need))))


APPEND_CALLS = 10 + 5 * 100      # time_calls on the append: warm-up + five batches of a hundred


def measure(cfg, K, W, dev):
    """Times K steps after W warm-up steps, then each kernel on its own
    (measure_kernels); returns the numbers of one configuration."""
    import torch
    lb = 4 if cfg.logits_dtype == "f32" else 2
    n_sets = rotation_sets(cfg)
    t0 = time.time()
    wk = Workload(cfg, K + W + APPEND_CALLS, n_sets, dev)
    log(f"setup {time.time() - t0:.1f}s: cfg{cfg.index} {cfg.name}, {n_sets} rotating input set(s), K/V "
        f"{2 * wk.lens.sum() * cfg.n_kv_heads * cfg.head_dim * 2 / 1e9:.3f} GB, logits "
        f"{2 * cfg.n_positions * cfg.vocab * lb / 1e9:.2f} GB, arena reserved {wk.arena_bytes / 1e9:.3f} GB each")
    for i in range(W):
        wk.step(i)
    torch.cuda.synchronize()
    marks = []
    t_start = time.perf_counter()
    for i in range(K):
        wk.step(W + i, marks)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t_start
    t_append = np.array([m[0][0].elapsed_time(m[0][1]) for m in marks]) * 1e-3
    t_attn = np.array([m[0][1].elapsed_time(m[0][2]) for m in marks]) * 1e-3
    t_logp = np.array([m[0][2].elapsed_time(m[0][3]) for m in marks]) * 1e-3
    t_step = np.array([m[0][0].elapsed_time(m[0][3]) for m in marks]) * 1e-3
    kernels = measure_kernels(wk, n_logp=10 if 2 * cfg.n_positions * cfg.vocab * lb > 16e9 else 100)
    s0 = wk.sets[0]
    med, lo, hi = time_calls(torch, lambda i: wk.rb.rlhf_kv_arena_append(s0["arena"], wk.seq_ids, wk.ones, wk.step_k,
                                                                          wk.step_v), 100)
    kernels["append_us"] = round(med * 1e6, 2)
    kernels["append_us_min_max"] = [round(lo * 1e6, 2), round(hi * 1e6, 2)]
    b_attn = float(np.mean([m[1] for m in marks]))
    b_logp = logprob_bytes(cfg.n_positions, cfg.vocab, lb)
    b_step = b_attn + b_logp + append_bytes(cfg)
    kv_rotated = n_sets * 2 * wk.lens.sum() * cfg.n_kv_heads * cfg.head_dim * 2
    # next-token sampling for one decode step (batch rows of the vocabulary); outside the timed step
    rows = wk.sets[0]["actor"][:cfg.batch]
    toks = torch.empty(cfg.batch, dtype=torch.int32, device=dev)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    sample_ws = torch.empty(wk.rb.rlhf_sample_tokens_workspace_bytes(cfg.batch, cfg.vocab), dtype=torch.uint8,
                            device=dev)
    for it in range(3):
        wk.rb.rlhf_sample_tokens_split(rows, toks, 1.0, cfg.seed, sample_ws, it)
    e0.record()
    for it in range(20):
        wk.rb.rlhf_sample_tokens_split(rows, toks, 1.0, cfg.seed, sample_ws, 3 + it)
    e1.record()
    torch.cuda.synchronize()
    sample_us = e0.elapsed_time(e1) / 20 * 1e3
    for it in range(3):   # the same draw restricted to the 50 largest logits of each row
        wk.rb.rlhf_sample_tokens_topk(rows, toks, 1.0, 50, cfg.seed, it)
    e0.record()
    for it in range(20):
        wk.rb.rlhf_sample_tokens_topk(rows, toks, 1.0, 50, cfg.seed, 3 + it)
    e1.record()
    torch.cuda.synchronize()
    topk_us = e0.elapsed_time(e1) / 20 * 1e3
    res = dict(
        wk=wk, n_sets=n_sets, t_total=t_total, b_step=b_step, b_attn=b_attn, b_logp=b_logp, lb=lb,
        ms_per_step=t_total / K * 1e3, value=b_step / (t_total / K) / 1e9,
        attn_gbps=b_attn / t_attn.mean() / 1e9, logp_gbps=b_logp / t_logp.mean() / 1e9,
        attn_us=t_attn.mean() * 1e6, logp_us=t_logp.mean() * 1e6, append_us=t_append.mean() * 1e6,
        sample_us=sample_us, topk_us=topk_us, attn_cold=bool(kv_rotated > 512e6), kernels=kernels,
        per_step={"step_ms": [round(float(x) * 1e3, 4) for x in (t_step.min(), np.median(t_step), t_step.max())],
                  "decode_attn_us": [round(float(x) * 1e6, 2) for x in (t_attn.min(), np.median(t_attn), t_attn.max())],
                  "logprob_kl_us": [round(float(x) * 1e6, 2) for x in (t_logp.min(), np.median(t_logp), t_logp.max())],
                  "order": "min, median, max over the timed steps (events around every call of every step)"},
        stats=wk.rb.rlhf_kv_arena_stats(wk.sets[0]["arena"]))
    return res


MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f16": 2500.0}   # MI355X dense matrix-core peak


def measure_prefill(cfg, dev, reps=10, warmup=5):
    """The prefill step of the same configuration (outside the timed decode
    step): every sequence's prompt is appended to an empty arena in one call and
    its causal attention runs over the arena.  `warmup` untimed passes (the pass
    follows seconds of host-only work, after which the device takes a few passes
    to return to its working clock), then the median of `reps` passes.  Returns
    times and flop counts."""
    import torch
    from paper_2410_15651_amd import binding as rb
    from paper_2410_15651_amd import workloads as wl
    P = wl.PAGE_TOKENS
    lens = wl.prompt_lengths(cfg)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T = int(cu[-1])
    _, ks, vs = wl.qkv(cfg, lens, device=dev)
    k_new, v_new = torch.cat(ks).contiguous(), torch.cat(vs).contiguous()
    del ks, vs
    q = wl.query_rows(cfg, T, device=dev)
    out = torch.empty_like(q)
    cu_d = torch.from_numpy(cu).to(dev)
    mpps = int((lens.max() + P - 1) // P)
    n_pages = int(((lens.astype(np.int64) + P - 1) // P).sum()) + 8
    kw = dict(max_seqs=cfg.batch, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim, n_pages=n_pages,
              max_pages_per_seq=mpps, kv_dtype=wl.DTYPE_CODE[cfg.kv_dtype],
              initial_free_order=wl.free_order(cfg, n_pages))
    nbytes = rb.rlhf_kv_arena_bytes_required(**kw)
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    arena = rb.rlhf_kv_arena_create(device_buffer=buf, device_buffer_bytes=nbytes, **kw)
    k_arena, v_arena, d_table, d_lens = rb.rlhf_kv_arena_views(arena)
    params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, mpps,
                            wl.DTYPE_CODE[cfg.kv_dtype])
    ids = np.arange(cfg.batch, dtype=np.int32)
    max_q = int(lens.max())
    t_app, t_att = [], []
    for it in range(warmup + reps):
        rb.rlhf_kv_arena_reset(arena)
        e = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        e[0].record()
        rb.rlhf_kv_arena_append(arena, ids, lens, k_new, v_new)
        e[1].record()
        rb.rlhf_prefill_attention(params, q, cu_d, max_q, k_arena, v_arena, d_table, d_lens, out)
        e[2].record()
        torch.cuda.synchronize()
        if it >= warmup:
            t_app.append(e[0].elapsed_time(e[1]) * 1e-3)
            t_att.append(e[1].elapsed_time(e[2]) * 1e-3)
    rb.rlhf_kv_arena_destroy(arena)
    L = lens.astype(np.float64)
    flops = 4.0 * cfg.head_dim * cfg.n_q_heads * float((L * (L + 1) / 2).sum())   # q.K and P.V, causal
    return dict(rows=T, flops=flops, attn_s=float(np.median(t_att)), append_s=float(np.median(t_app)),
                attn_min_max_s=(float(min(t_att)), float(max(t_att))), lens_lo=int(lens.min()),
                lens_hi=int(lens.max()))


def read_ceiling(dev, gib=4, reps=5):
    """GB/s of a kernel that does nothing but read a buffer once with the
    library's streaming loads: the practical ceiling under the published peak."""
    import torch
    from paper_2410_15651_amd import binding as rb
    buf = torch.empty(gib << 30, dtype=torch.uint8, device=dev)
    buf.fill_(1)
    rb.rlhf_probe_stream_read(buf)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        rb.rlhf_probe_stream_read(buf)
    e1.record()
    torch.cuda.synchronize()
    return buf.numel() / (e0.elapsed_time(e1) / reps * 1e-3) / 1e9


def matrix_ceiling(dev, iterations=20000):
    """What a kernel of nothing but the prefill kernel's matrix instruction reaches, and the shader clock
    the device holds meanwhile, on N(0,1) bf16 operands (the workload's K/V/q distribution) and on zeros.
    The device lowers its clock under matrix load by an amount that depends on the operand data."""
    import torch
    from paper_2410_15651_amd import binding as rb
    n_wg = torch.cuda.get_device_properties(dev).multi_processor_count
    g = torch.Generator(device=dev)
    g.manual_seed(20241015)
    out = {}
    for name, ops in (("N01", torch.randn(1 << 20, generator=g, device=dev).to(torch.bfloat16)),
                      ("zeros", torch.zeros(1 << 20, dtype=torch.bfloat16, device=dev))):
        ticks = torch.zeros(3, dtype=torch.int64, device=dev)
        rb.rlhf_probe_matrix_rate(ops, 200, n_wg, ticks)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        rb.rlhf_probe_matrix_rate(ops, iterations, n_wg, ticks)
        e1.record()
        torch.cuda.synchronize()
        t = ticks.cpu().tolist()
        flops = n_wg * 12 * iterations * 8 * 32768.0
        out[name] = {"TFLOPs": round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1),
                     "shader_clock_MHz": round(t[1] / max(t[0], 1) * 100.0)}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload index 1..5 (default: the largest)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the short per-kernel summary of the other four configurations")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device-to-device copies first (a kernel of known "
                         "traffic, to scale hardware byte counters in a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: the library runs on ONE GPU; --gpus above 1 is not supported "
            "(no collectives or sharding are part of it).")
        sys.exit(2)

    import torch
    from paper_2410_15651_amd import binding as rb
    from paper_2410_15651_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the hot path has no CPU fallback.")
        sys.exit(1)
    rb.lib()                                   # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = wl.config(args.config)
    K, W = args.steps, args.warmup
    if args.calibrate_copy:
        src = torch.full((1 << 30,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ceiling = read_ceiling(dev)
    torch.cuda.empty_cache()
    m = measure(cfg, K, W, dev)
    wk, stats = m["wk"], m["stats"]
    n_pos = cfg.n_positions
    attn_kernel = ("attn_stream_kernel" if cfg.n_q_heads == cfg.n_kv_heads else "attn_stream_gqa_kernel")
    result = {
        "metric": METRIC, "value": round(m["value"], 1), "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(m["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"configs[{cfg.index - 1}] {cfg.name}: batch {cfg.batch}, {cfg.n_q_heads}q/"
                               f"{cfg.n_kv_heads}kv heads, head_dim {cfg.head_dim}, {cfg.kv_dtype} KV, cache "
                               f"lengths U[{cfg.len_lo},{cfg.len_hi}], 16-token pages "
                               f"{'shuffled' if cfg.shuffled_pages else 'in order'}; logprob/KL {n_pos} positions x "
                               f"vocab {cfg.vocab}, {cfg.logits_dtype} logits",
                   "step": "append 1 token/seq + decode attention + token logprob/KL",
                   "storage": f"{cfg.kv_dtype} K/V, {cfg.logits_dtype} logits; fp32 arithmetic", "hbm_peak_GBps": HBM_PEAK_GBPS,
                   "hbm_read_ceiling_GBps": round(ceiling, 1), "rotating_input_sets": m["n_sets"]},
        "components": {
            "decode_attn_GBps": round(m["attn_gbps"], 1),
            "decode_attn_frac_of_peak": round(m["attn_gbps"] / HBM_PEAK_GBPS, 4),
            "decode_attn_frac_of_read_ceiling": round(m["attn_gbps"] / ceiling, 4),
            "decode_attn_us": round(m["attn_us"], 2), "decode_attn_bytes": int(m["b_attn"]),
            "logprob_kl_tokens_per_s": round(n_pos / (m["logp_us"] * 1e-6), 1),
            "logprob_kl_GBps": round(m["logp_gbps"], 1),
            "logprob_kl_frac_of_peak": round(m["logp_gbps"] / HBM_PEAK_GBPS, 4),
            "logprob_kl_frac_of_read_ceiling": round(m["logp_gbps"] / ceiling, 4),
            "logprob_kl_us": round(m["logp_us"], 2), "append_us": round(m["append_us"], 2),
            "sample_tokens_us_per_decode_step": round(m["sample_us"], 2),
            "sample_tokens_Gelem_per_s": round(cfg.batch * cfg.vocab / m["sample_us"] / 1e3, 1),
            "sample_tokens_top50_us_per_decode_step": round(m["topk_us"], 2),
            "arena_reserved_bytes": stats["reserved_bytes"], "arena_allocated_bytes": stats["allocated_bytes"],
            "arena_driver_allocations_after_create": 0,
            "per_step_distribution": m["per_step"],
            "kernels_back_to_back": m["kernels"],
        },
        "roofline": {"kernel": "logprob_kl_kernel", "bound": "hbm", "achieved": round(m["logp_gbps"], 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(m["logp_gbps"] / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic("logprob_kl", cfg.index)},
        "roofline_decode_attn": {"kernel": attn_kernel + (" (one launch: the wavefront that completes a unit merges it)"
                                                          if cfg.n_q_heads == cfg.n_kv_heads else "+attn_merge_kernel"),
                                 "bound": "hbm",
                                 "achieved": round(m["attn_gbps"], 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                 "frac": round(m["attn_gbps"] / HBM_PEAK_GBPS, 4),
                                 "traffic": measured_traffic("decode_attn", cfg.index)},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, wk.lens, wk.q, wk.ks, wk.vs, wk.sets[0]["actor"],
                                              wk.sets[0]["ref"], wk.tok_np, m["b_step"], m["lb"], 2)
    wk.close()
    del wk, m
    torch.cuda.empty_cache()

    # the prefill step of the same workload: reported beside the decode step, not part of `value`
    pf = measure_prefill(cfg, dev)
    tfl = pf["flops"] / pf["attn_s"] / 1e12
    peak = MFMA_PEAK_TFLOPS[cfg.kv_dtype]
    result["components"].update({
        "prefill_attn_us": round(pf["attn_s"] * 1e6, 1), "prefill_attn_TFLOPs": round(tfl, 1),
        "prefill_attn_us_min_max": [round(x * 1e6, 1) for x in pf["attn_min_max_s"]],
        "prefill_method": "median of 10 passes after 5 warm-up passes",
        "prefill_append_us": round(pf["append_s"] * 1e6, 1), "prefill_rows": pf["rows"],
        "prefill_tokens_per_s": round(pf["rows"] / (pf["attn_s"] + pf["append_s"]), 1),
        "prefill_prompt_lengths": f"U[{max(1, cfg.len_lo // 2)},{max(1, cfg.len_hi // 2)}]"})
    result["roofline_prefill_attn"] = {
        "kernel": "prefill_attn_kernel", "bound": "mfma", "achieved": round(tfl, 1), "peak": peak,
        "unit": "TFLOP/s", "frac": round(tfl / peak, 4), "traffic": measured_traffic("prefill_attn", cfg.index),
        "flops": "4 * head_dim * q heads * sum L(L+1)/2: q.K and P.V of the causal triangle"}
    probe = matrix_ceiling(dev)
    result["roofline_prefill_attn"]["matrix_probe"] = {
        **probe, "what": "a loop of 32x32x16 bf16 matrix instructions alone, three wavefronts per SIMD on every "
                         "compute unit: the rate and the clock the device holds depend on the operand data",
        "achieved_frac_of_probe_on_N01": round(tfl / probe["N01"]["TFLOPs"], 4)}
    torch.cuda.empty_cache()

    if not args.no_other_configs:
        others = []
        for c in wl.CONFIGS:
            if c.index == cfg.index:
                continue
            o = measure(c, 10, 2, dev)
            kb = o["kernels"]
            others.append({
                "workload": f"configs[{c.index - 1}] {c.name}", "method": kb["method"],
                "rotating_input_sets": o["n_sets"], "cold_means": kb["cold_means"],
                **{k: v for k, v in kb.items() if k.startswith(("decode_attn_", "logprob_kl_", "append_"))},
                "sample_tokens_us": round(o["sample_us"], 2),
                "sample_tokens_top50_us": round(o["topk_us"], 2),
                "step_loop": {"steps": 10, "warmup": 2, "step_GBps": round(o["value"], 1),
                              "decode_attn_us": round(o["attn_us"], 2), "logprob_kl_us": round(o["logp_us"], 2),
                              "append_us": round(o["append_us"], 2),
                              "note": "mean of 10 steps with events around every call (includes the launch "
                                      "latency of a lone call)"}})
            o["wk"].close()
            del o
            torch.cuda.empty_cache()
            pf = measure_prefill(c, dev, reps=5, warmup=3)
            others[-1].update({"prefill_attn_us": round(pf["attn_s"] * 1e6, 1),
                               "prefill_attn_TFLOPs": round(pf["flops"] / pf["attn_s"] / 1e12, 1),
                               "prefill_append_us": round(pf["append_s"] * 1e6, 1), "prefill_rows": pf["rows"]})
            torch.cuda.empty_cache()
        result["other_configs"] = others
    print(json.dumps(result), flush=True)


def cpu_baseline(cfg, lens, q, ks, vs, actor, ref, tok_np, b_step, lb, eb):
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample
    of the same workload (every sequence's attention, a few ten thousand logit
    rows in chunks that fit host memory) and scaled to a whole step."""
    import torch
    import oracle
    from paper_2410_15651_amd import workloads as wl
    P = wl.PAGE_TOKENS
    oracle.build()
    rng = np.random.default_rng(cfg.seed)
    n_seq = cfg.batch
    seqs = np.arange(n_seq)
    # about 20 s of oracle time on 16 cores at the largest vocabulary; never more rows than there are
    n_rows = min(cfg.n_positions, max(256, int(98304 * 128256 / cfg.vocab)))
    rows = np.sort(rng.choice(cfg.n_positions, n_rows, replace=False))
    # attention sample: plain pages in logical order for the sampled sequences
    ks_h = [wl.to_storage(ks[b]) for b in seqs]
    vs_h = [wl.to_storage(vs[b]) for b in seqs]
    need = [(int(lens[b]) + P - 1) // P for b in seqs]
    table = np.full((n_seq, max(need)), -1, dtype=np.int32)
    nxt = 0
    for i, n in enumerate(need):
        table[i, :n] = np.arange(nxt, nxt + n)
        nxt += n
    kp, vp = wl.plain_pages(ks_h, vs_h, table, nxt)
    qh = wl.to_storage(q)[seqs]
    code = wl.DTYPE_CODE[cfg.kv_dtype]
    t = time.perf_counter()
    oracle.decode_attention(qh, kp, vp, table, lens[seqs], code)
    t_attn = time.perf_counter() - t
    del ks_h, vs_h, kp, vp
    t_logp = 0.0
    chunk = 8192
    for c0 in range(0, n_rows, chunk):
        sel = rows[c0:c0 + chunk]
        idx = torch.from_numpy(sel).to(actor.device)
        a_h = wl.to_storage(actor[idx])
        r_h = wl.to_storage(ref[idx])
        t = time.perf_counter()
        oracle.token_logprobs_kl(a_h, r_h, tok_np[sel], wl.DTYPE_CODE[cfg.logits_dtype])
        t_logp += time.perf_counter() - t
    est_step = t_attn * cfg.batch / n_seq + t_logp * cfg.n_positions / n_rows
    return {
        "value": round(b_step / est_step / 1e9, 4), "unit": "GB/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"all {n_seq} sequences (attention, {t_attn:.2f}s) and {n_rows} of "
                  f"{cfg.n_positions} logit rows (logprob/KL, {t_logp:.2f}s), scaled to one whole step "
                  f"({est_step:.1f}s estimated)",
        "logprob_kl_tokens_per_s": round(n_rows / t_logp, 1),
    }


if __name__ == "__main__":
    main()
