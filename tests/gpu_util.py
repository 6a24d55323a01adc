"""Helpers for the GPU parity tests: drive the library through its C ABI and
hand the same stored values to the CPU oracle.  Not collected by pytest."""
from __future__ import annotations

import numpy as np
import torch

from oracle import ArenaModel
from paper_2410_15651_amd import binding as rb
from paper_2410_15651_amd import workloads as wl

P = wl.PAGE_TOKENS
DEV = "cuda:0"


class FilledArena:
    """An arena filled the way a rollout fills it: the prompt part in bulk (in
    interleaved page-sized rounds for the shuffled configurations), then one
    single-token append per sequence, so the attention call sees a real decode
    step's state.  A Python model of the bookkeeping is replayed alongside."""

    def __init__(self, cfg: wl.RolloutConfig, lens: np.ndarray, ks, vs, slack_pages: int = 3,
                 extra_tokens: int = 0):
        self.cfg = cfg
        self.lens = lens.astype(np.int32)
        need = int(((lens.astype(np.int64) + extra_tokens + P - 1) // P).sum())
        self.n_pages = need + slack_pages
        self.mpps = max(1, cfg.max_pages_per_seq(extra_tokens))
        self.order = wl.free_order(cfg, self.n_pages)
        kw = dict(max_seqs=cfg.batch, n_kv_heads=cfg.n_kv_heads, head_dim=cfg.head_dim,
                  n_pages=self.n_pages, max_pages_per_seq=self.mpps,
                  kv_dtype=wl.DTYPE_CODE[cfg.kv_dtype], initial_free_order=self.order)
        self.bytes = rb.rlhf_kv_arena_bytes_required(**kw)
        # every byte 0xFF: slots that are never written read as NaN in both 16-bit
        # formats, so a kernel that lets an unused slot reach its arithmetic shows up
        self.buffer = torch.full((self.bytes,), 0xFF, dtype=torch.uint8, device=DEV)
        self.handle = rb.rlhf_kv_arena_create(device_buffer=self.buffer, device_buffer_bytes=self.bytes, **kw)
        self.model = ArenaModel(cfg.batch, cfg.n_kv_heads, cfg.head_dim, P, self.n_pages, self.mpps,
                                initial_free_order=self.order)
        done = np.zeros(cfg.batch, dtype=np.int64)
        calls = wl.fill_schedule(cfg, lens, hold_back=1)
        last = (np.arange(cfg.batch, dtype=np.int32)[lens > 0], np.ones(int((lens > 0).sum()), dtype=np.int32))
        for ids, n_new in calls + [last]:
            if len(ids) == 0:
                continue
            k_new = torch.cat([ks[b][done[b]:done[b] + n] for b, n in zip(ids, n_new)]).contiguous()
            v_new = torch.cat([vs[b][done[b]:done[b] + n] for b, n in zip(ids, n_new)]).contiguous()
            rb.rlhf_kv_arena_append(self.handle, ids, n_new, k_new, v_new)
            self.model.append([int(i) for i in ids], [int(n) for n in n_new])
            for b, n in zip(ids, n_new):
                done[b] += n
        torch.cuda.synchronize()
        assert (done == lens).all()

    def views(self):
        return rb.rlhf_kv_arena_views(self.handle)

    def host_state(self):
        return rb.rlhf_kv_arena_host_state(self.handle, self.cfg.batch, self.mpps)

    def close(self):
        if self.handle:
            rb.rlhf_kv_arena_destroy(self.handle)
            self.handle = None


def run_attention(cfg, arena: FilledArena, q, out_dtype=None, max_seq_len=0, scale=0.0):
    k, v, table, lens = arena.views()
    code = wl.DTYPE_CODE[cfg.kv_dtype]
    params = rb.attn_params(cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, arena.mpps, code,
                            out_dtype=out_dtype, max_seq_len=max_seq_len, softmax_scale=scale)
    # scratch poisoned (NaN in every float): a merge that reads a partial nobody wrote shows up
    ws = torch.full((rb.rlhf_decode_attention_workspace_bytes(params),), 0xFF, dtype=torch.uint8, device=DEV)
    odt = torch.float32 if out_dtype == rb.RLHF_F32 else wl.torch_dtype(cfg.kv_dtype)
    out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=odt, device=DEV)
    rb.rlhf_decode_attention(params, q, k, v, table, lens, out, ws)
    torch.cuda.synchronize()
    return out


def oracle_attention(oracle, cfg, q, ks, vs, table, lens, n_pages, seqs=None, scale=None):
    """Oracle output for all sequences or for the listed ones (rows of the result
    follow `seqs`)."""
    seqs = list(range(cfg.batch)) if seqs is None else list(seqs)
    ks_h = [wl.to_storage(ks[b]) for b in seqs]
    vs_h = [wl.to_storage(vs[b]) for b in seqs]
    sub_table = table[seqs]
    kp, vp = wl.plain_pages(ks_h, vs_h, sub_table, n_pages)
    qh = wl.to_storage(q)[seqs]
    return oracle.decode_attention(qh, kp, vp, sub_table, lens[seqs], wl.DTYPE_CODE[cfg.kv_dtype],
                                   scale=scale)


def run_logprobs(actor, ref, tokens_np, vocab=None, stride=0):
    n = actor.shape[0]
    tok = torch.from_numpy(tokens_np).to(DEV)
    logp = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    kl = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    if vocab is None:
        rb.rlhf_token_logprobs_kl(actor, ref, tok, logp, kl)
    else:
        rb.rlhf_token_logprobs_kl(actor, ref, tok, logp, kl, n_positions=n, vocab=vocab,
                                  row_stride_elems=stride, logits_dtype=rb.dtype_code(actor.dtype))
    torch.cuda.synchronize()
    return logp.cpu().numpy().astype(np.float64), kl.cpu().numpy().astype(np.float64)
