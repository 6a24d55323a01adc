"""The hot path end to end, the way an experience-generation step would drive it
(Section 2.1 of the paper: the actor generates responses, then actor and
reference score them):

    prompts -> arena (one bulk append)          rlhf_kv_arena_append
            -> causal attention of the prompts  rlhf_prefill_attention
    for every generated token:
            -> append this step's K/V rows      rlhf_kv_arena_append
            -> single-token decode attention    rlhf_decode_attention
            -> draw the next token              rlhf_sample_tokens_split, or rlhf_sample_tokens_topk
    scoring of the generated positions          rlhf_token_logprobs_kl_rewards
    phase boundary                              rlhf_kv_arena_reset

    python -m paper_2410_15651_amd.rollout_demo [config 1..5] [generated tokens] [batch] [top_k]

There is no model here: queries, keys, values and logits are seeded random
tensors of the configuration's shapes (one attention layer's worth), so the
script shows the calls, their order and their cost, not text.  It needs a GPU.
"""
from __future__ import annotations

import sys
import time

import numpy as np


def run(cfg_index: int = 2, gen_len: int = 32, batch: int | None = None, verbose: bool = True,
        top_k: int | None = None) -> dict:
    import torch
    from . import binding as rb
    from . import workloads as wl

    if not torch.cuda.is_available():
        raise RuntimeError("rollout_demo needs a GPU: the library has no CPU fallback")
    dev = "cuda:0"
    P = wl.PAGE_TOKENS
    cfg = wl.config(cfg_index)
    if batch is not None:
        cfg = wl.small_variant(cfg, batch=batch)
    B, Hq, Hkv, D, V = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.vocab
    code = wl.DTYPE_CODE[cfg.kv_dtype]
    tdt = wl.torch_dtype(cfg.kv_dtype)
    ldt = wl.torch_dtype(cfg.logits_dtype)
    g = torch.Generator(device=dev)
    g.manual_seed(cfg.seed)

    def rand(*shape, std=cfg.qkv_std, dtype=tdt):
        return (torch.randn(*shape, generator=g, device=dev) * std).to(dtype)

    prompts = wl.prompt_lengths(cfg)
    final = prompts.astype(np.int64) + gen_len
    mpps = int((final.max() + P - 1) // P)
    n_pages = int(((final + P - 1) // P).sum())
    kw = dict(max_seqs=B, n_kv_heads=Hkv, head_dim=D, n_pages=n_pages, max_pages_per_seq=mpps, kv_dtype=code,
              initial_free_order=wl.free_order(cfg, n_pages))
    nbytes = rb.rlhf_kv_arena_bytes_required(**kw)
    buf = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    arena = rb.rlhf_kv_arena_create(device_buffer=buf, device_buffer_bytes=nbytes, **kw)
    times = {}

    def timed(name, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        times.setdefault(name, []).append(e0.elapsed_time(e1) * 1e-3)

    try:
        k_arena, v_arena, d_table, d_lens = rb.rlhf_kv_arena_views(arena)
        params = rb.attn_params(B, Hq, Hkv, D, mpps, code, max_seq_len=int(final.max()))
        ws = torch.empty(rb.rlhf_decode_attention_workspace_bytes(params), dtype=torch.uint8, device=dev)
        sample_ws = torch.empty(rb.rlhf_sample_tokens_workspace_bytes(B, V), dtype=torch.uint8, device=dev)
        ids = np.arange(B, dtype=np.int32)
        ones = np.ones(B, dtype=np.int32)

        # ---- prompts: one append, one causal attention over the arena
        T = int(prompts.sum())
        cu = np.concatenate([[0], np.cumsum(prompts)]).astype(np.int32)
        k_p, v_p, q_p = rand(T, Hkv, D), rand(T, Hkv, D), rand(T, Hq, D)
        out_p = torch.empty_like(q_p)
        cu_d = torch.from_numpy(cu).to(dev)
        timed("prompt append", lambda: rb.rlhf_kv_arena_append(arena, ids, prompts, k_p, v_p))
        timed("prefill attention", lambda: rb.rlhf_prefill_attention(params, q_p, cu_d, int(prompts.max()),
                                                                     k_arena, v_arena, d_table, d_lens, out_p))
        del k_p, v_p, q_p, out_p

        # ---- generation: append, attend, draw, once per token
        out = torch.empty(B, Hq, D, dtype=tdt, device=dev)
        drawn = torch.empty(gen_len, B, dtype=torch.int32, device=dev)
        step_logp = torch.empty(gen_len, B, dtype=torch.float32, device=dev)
        t_host = time.perf_counter()
        for t in range(gen_len):
            k_t, v_t, q_t = rand(B, Hkv, D), rand(B, Hkv, D), rand(B, Hq, D)
            logits_t = rand(B, V, std=cfg.logits_std, dtype=ldt)          # stands in for the LM head
            timed("decode append", lambda: rb.rlhf_kv_arena_append(arena, ids, ones, k_t, v_t))
            timed("decode attention", lambda: rb.rlhf_decode_attention(params, q_t, k_arena, v_arena, d_table,
                                                                       d_lens, out, ws))
            if top_k:
                timed("sampling", lambda: rb.rlhf_sample_tokens_topk(logits_t, drawn[t], 1.0, top_k, cfg.seed,
                                                                     offset=t, logp_out=step_logp[t]))
            else:
                timed("sampling", lambda: rb.rlhf_sample_tokens_split(logits_t, drawn[t], 1.0, cfg.seed, sample_ws,
                                                                      offset=t, logp_out=step_logp[t]))
        t_host = time.perf_counter() - t_host

        # ---- scoring of the generated positions: actor vs reference
        N = B * gen_len
        actor = rand(N, V, std=cfg.logits_std, dtype=ldt)
        ref = (actor.float() + torch.randn(N, V, generator=g, device=dev) * 0.1).to(ldt)
        tok = drawn.t().contiguous().view(N)                              # sequence-major, like the logits rows
        logp = torch.empty(N, dtype=torch.float32, device=dev)
        kl, ref_logp, reward = torch.empty_like(logp), torch.empty_like(logp), torch.empty_like(logp)
        terminal = torch.zeros(N, dtype=torch.float32, device=dev)
        terminal[gen_len - 1::gen_len] = 1.0                              # a reward model's score at the last token
        timed("log-prob / KL / rewards",
              lambda: rb.rlhf_token_logprobs_kl_rewards(actor, ref, tok, logp, kl, 0.1, ref_logp_out=ref_logp,
                                                        reward_out=reward, terminal_scores=terminal))
        stats = rb.rlhf_kv_arena_stats(arena)
        table, lens, _ = rb.rlhf_kv_arena_host_state(arena, B, mpps)
        assert lens.tolist() == final.tolist()
        assert torch.isfinite(out.float()).all() and torch.isfinite(logp).all() and (kl >= -1e-5).all()
        assert ((tok >= 0) & (tok < V)).all()
        rb.rlhf_kv_arena_reset(arena)                                      # the phase boundary: every page free again
        after = rb.rlhf_kv_arena_stats(arena)
        assert after["pages_in_use"] == 0 and after["reserved_bytes"] == stats["reserved_bytes"]
        # a kernel's first call also loads its code: per-step figures are medians
        per_step = {k: float(np.median(v)) for k, v in times.items()}
        result = dict(config=cfg.name, batch=B, prompt_tokens=T, generated=N, seconds=per_step,
                      decode_step_us=1e6 * (per_step["decode append"] + per_step["decode attention"]
                                            + per_step["sampling"]),
                      host_loop_us_per_step=1e6 * t_host / gen_len,
                      arena_reserved_bytes=stats["reserved_bytes"], arena_allocated_bytes=stats["allocated_bytes"],
                      arena_live_token_bytes=stats["live_token_bytes"], mean_kl=float(kl.mean()),
                      mean_logp=float(logp.mean()), mean_reward=float(reward.mean()))
    finally:
        rb.rlhf_kv_arena_destroy(arena)
    if verbose:
        print(f"{cfg.name}: {B} sequences, prompts {int(prompts.min())}-{int(prompts.max())} tokens, "
              f"{gen_len} generated tokens each")
        for name, v in times.items():
            if len(v) > 1:
                print(f"  {name:26s} {1e6 * np.median(v):9.1f} us per step (median of {len(v)})")
            else:
                print(f"  {name:26s} {1e3 * v[0]:9.3f} ms (first call: includes loading the kernel)")
        print(f"  arena: reserved {result['arena_reserved_bytes'] / 2**20:.1f} MiB (constant), allocated at the end "
              f"{result['arena_allocated_bytes'] / 2**20:.1f} MiB, of which tokens "
              f"{result['arena_live_token_bytes'] / 2**20:.1f} MiB; after the reset 0 pages in use")
        print(f"  mean log-prob {result['mean_logp']:.3f}, mean KL {result['mean_kl']:.5f}, "
              f"mean reward {result['mean_reward']:.5f}")
    return result


if __name__ == "__main__":
    a = sys.argv[1:]
    run(int(a[0]) if len(a) > 0 else 2, int(a[1]) if len(a) > 1 else 32, int(a[2]) if len(a) > 2 and int(a[2]) else None,
        top_k=int(a[3]) if len(a) > 3 else None)
