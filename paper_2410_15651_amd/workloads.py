"""Seeded synthetic inputs for the rollout hot path.

This module only draws random numbers and arranges them; it contains none of
the method's arithmetic, and both the GPU tests and the CPU oracle's tests take
their inputs from it.

The paper measures OPT, GPT-2 and Llama-2 models on the RLHF frameworks'
default prompts (Section 3 "Workload and Setting"; Appendix C).  Neither the
weights nor the prompts are needed for a decode-attention or log-prob kernel:
their cost depends on shapes, dtypes and cache-length mix only.  The five
configurations below have those models' head counts, head sizes and
vocabularies; values are Gaussian, cache lengths are uniform integers on a
closed interval, sampled tokens are uniform over the vocabulary.

Lengths, tokens and page permutations come from a CPU generator (they drive
integer bookkeeping that must be identical everywhere); Q/K/V/logit values come
from a generator on the requested device and whoever needs them on the host
copies the actual values back.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import List, Optional, Tuple

import numpy as np
import torch

PAGE_TOKENS = 16
BASE_SEED = 241015

_TORCH_DTYPE = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}
DTYPE_CODE = {"f16": 0, "bf16": 1, "f32": 2}


@dataclass(frozen=True)
class RolloutConfig:
    name: str
    index: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    kv_dtype: str           # 'f16' | 'bf16'
    qkv_std: float
    len_lo: int
    len_hi: int             # inclusive
    shuffled_pages: bool
    gen_len: int            # generated positions per sequence (n_positions = batch * gen_len)
    vocab: int
    logits_dtype: str       # 'f32' | 'bf16'
    logits_std: float
    ref_noise_std: Optional[float]   # None: ref drawn independently like actor

    @property
    def n_positions(self) -> int:
        return self.batch * self.gen_len

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    def max_pages_per_seq(self, extra_tokens: int = 0) -> int:
        return (self.len_hi + extra_tokens + PAGE_TOKENS - 1) // PAGE_TOKENS


CONFIGS: List[RolloutConfig] = [
    RolloutConfig("opt125m", 1, 4, 12, 12, 64, "f16", 0.125, 1, 512, False,
                  256, 50272, "f32", 2.0, None),
    RolloutConfig("opt1.3b", 2, 16, 32, 32, 64, "bf16", 1.0, 256, 512, False,
                  256, 50272, "bf16", 3.0, None),
    RolloutConfig("llama7b", 3, 32, 32, 32, 128, "bf16", 1.0, 512, 1024, False,
                  512, 32000, "bf16", 3.0, 0.1),
    RolloutConfig("llama13b", 4, 64, 40, 40, 128, "bf16", 1.0, 1024, 2048, True,
                  512, 32000, "bf16", 3.0, 0.1),
    RolloutConfig("gqa70b", 5, 128, 64, 8, 128, "bf16", 1.0, 2048, 4096, True,
                  1024, 128256, "bf16", 3.0, None),
]


def config(index_or_name) -> RolloutConfig:
    for c in CONFIGS:
        if c.index == index_or_name or c.name == index_or_name:
            return c
    raise KeyError(index_or_name)


def small_variant(cfg: RolloutConfig, **kw) -> RolloutConfig:
    """A copy of a configuration with some fields replaced (test sizes)."""
    return replace(cfg, **kw)


def torch_dtype(name: str) -> torch.dtype:
    return _TORCH_DTYPE[name]


def _cpu_rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.default_rng([seed, stream])


def seq_lengths(cfg: RolloutConfig, seed: Optional[int] = None) -> np.ndarray:
    """Cache lengths, uniform integers on [len_lo, len_hi], int32 [batch]."""
    rng = _cpu_rng(cfg.seed if seed is None else seed, 1)
    return rng.integers(cfg.len_lo, cfg.len_hi + 1, size=cfg.batch, dtype=np.int64).astype(np.int32)


def free_order(cfg: RolloutConfig, n_pages: int, seed: Optional[int] = None) -> Optional[np.ndarray]:
    """Initial free-list order: a seeded permutation for the shuffled-page
    configurations, None (identity) otherwise."""
    if not cfg.shuffled_pages:
        return None
    rng = _cpu_rng(cfg.seed if seed is None else seed, 2)
    return rng.permutation(n_pages).astype(np.int32)


def fill_schedule(cfg: RolloutConfig, lens: np.ndarray, hold_back: int = 1
                  ) -> List[Tuple[np.ndarray, np.ndarray]]:
    """Append calls that bring every sequence to lens[b] - hold_back tokens.

    For shuffled-page configurations the sequences grow in interleaved rounds of
    one page each, so that consecutive logical pages of a sequence land on
    scattered physical pages; otherwise one bulk call.  Each entry is
    (seq_ids, n_new), int32 arrays.
    """
    target = np.maximum(lens.astype(np.int64) - hold_back, 0)
    ids = np.arange(cfg.batch, dtype=np.int32)
    if not cfg.shuffled_pages:
        return [(ids, target.astype(np.int32))]
    calls = []
    done = np.zeros_like(target)
    while (done < target).any():
        n = np.minimum(target - done, PAGE_TOKENS)
        keep = n > 0
        calls.append((ids[keep], n[keep].astype(np.int32)))
        done += n
    return calls


def _device_gen(device, seed: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed * 1000 + stream)
    return g


def qkv(cfg: RolloutConfig, lens: np.ndarray, device="cpu", seed: Optional[int] = None):
    """q [B,Hq,D]; k, v: lists of per-sequence tensors [L_b, Hkv, D]; all in the
    cache dtype, values N(0, qkv_std^2) rounded to that dtype."""
    seed = cfg.seed if seed is None else seed
    dt = torch_dtype(cfg.kv_dtype)
    g = _device_gen(device, seed, 3)
    q = (torch.randn(cfg.batch, cfg.n_q_heads, cfg.head_dim, generator=g, device=device,
                     dtype=torch.float32) * cfg.qkv_std).to(dt)
    ks, vs = [], []
    for b in range(cfg.batch):
        L = int(lens[b])
        kv = torch.randn(2, L, cfg.n_kv_heads, cfg.head_dim, generator=g, device=device,
                         dtype=torch.float32) * cfg.qkv_std
        ks.append(kv[0].to(dt))
        vs.append(kv[1].to(dt))
    return q, ks, vs


def prompt_lengths(cfg: RolloutConfig, seed: Optional[int] = None) -> np.ndarray:
    """Prompt lengths for the prefill step: uniform integers on [len_lo/2,
    len_hi/2] (at least 1) -- the prompt as half of the final cache, the other
    half being generated.  int32 [batch]."""
    rng = _cpu_rng(cfg.seed if seed is None else seed, 6)
    lo, hi = max(1, cfg.len_lo // 2), max(1, cfg.len_hi // 2)
    return rng.integers(lo, hi + 1, size=cfg.batch, dtype=np.int64).astype(np.int32)


def query_rows(cfg: RolloutConfig, n_rows: int, device="cpu", seed: Optional[int] = None) -> torch.Tensor:
    """Packed query rows [n_rows, Hq, D] in the cache dtype, N(0, qkv_std^2)."""
    seed = cfg.seed if seed is None else seed
    g = _device_gen(device, seed, 7)
    q = torch.randn(n_rows, cfg.n_q_heads, cfg.head_dim, generator=g, device=device, dtype=torch.float32)
    return (q * cfg.qkv_std).to(torch_dtype(cfg.kv_dtype))


def tokens(cfg: RolloutConfig, n_positions: Optional[int] = None, seed: Optional[int] = None
           ) -> np.ndarray:
    """Sampled token ids, uniform over the vocabulary, int32 [n_positions]."""
    rng = _cpu_rng(cfg.seed if seed is None else seed, 4)
    n = cfg.n_positions if n_positions is None else n_positions
    return rng.integers(0, cfg.vocab, size=n, dtype=np.int64).astype(np.int32)


def logits(cfg: RolloutConfig, n_positions: Optional[int] = None, device="cpu",
           seed: Optional[int] = None, chunk_rows: int = 4096):
    """(actor, ref) logits [n_positions, vocab] in the logits dtype.

    actor ~ N(0, logits_std^2).  ref is an independent draw from the same law,
    or, when ref_noise_std is set, the stored actor value plus N(0,
    ref_noise_std^2), rounded to the logits dtype.  Generated in row chunks so
    the fp32 staging never exceeds chunk_rows * vocab elements.
    """
    seed = cfg.seed if seed is None else seed
    n = cfg.n_positions if n_positions is None else n_positions
    dt = torch_dtype(cfg.logits_dtype)
    g = _device_gen(device, seed, 5)
    actor = torch.empty(n, cfg.vocab, device=device, dtype=dt)
    ref = torch.empty(n, cfg.vocab, device=device, dtype=dt)
    for r0 in range(0, n, chunk_rows):
        r1 = min(n, r0 + chunk_rows)
        a = torch.randn(r1 - r0, cfg.vocab, generator=g, device=device, dtype=torch.float32)
        a.mul_(cfg.logits_std)
        actor[r0:r1] = a.to(dt)
        r = torch.randn(r1 - r0, cfg.vocab, generator=g, device=device, dtype=torch.float32)
        if cfg.ref_noise_std is None:
            r.mul_(cfg.logits_std)
        else:
            r.mul_(cfg.ref_noise_std).add_(actor[r0:r1].float())
        ref[r0:r1] = r.to(dt)
        del a, r
    return actor, ref


def to_storage(t: torch.Tensor) -> np.ndarray:
    """Host copy of a tensor's stored values: float32 arrays as they are, 16-bit
    floating types as their raw uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    if t.dtype in (torch.float16, torch.bfloat16):
        return t.view(torch.int16).numpy().view(np.uint16)
    raise TypeError(t.dtype)


def plain_pages(ks, vs, page_table: np.ndarray, n_pages: int):
    """Lays per-sequence rows [L_b, Hkv, D] out as plain token-major pages
    [n_pages, Hkv, PAGE_TOKENS, D] following a page table (storage arrays in,
    storage arrays out; untouched slots are zero).  Pure data movement."""
    Hkv, D = ks[0].shape[1], ks[0].shape[2]
    kp = np.zeros((n_pages, Hkv, PAGE_TOKENS, D), dtype=ks[0].dtype)
    vp = np.zeros_like(kp)
    for b, (k, v) in enumerate(zip(ks, vs)):
        L = k.shape[0]
        for lp in range((L + PAGE_TOKENS - 1) // PAGE_TOKENS):
            t0, t1 = lp * PAGE_TOKENS, min(L, (lp + 1) * PAGE_TOKENS)
            page = int(page_table[b, lp])
            kp[page, :, : t1 - t0, :] = np.swapaxes(k[t0:t1], 0, 1)
            vp[page, :, : t1 - t0, :] = np.swapaxes(v[t0:t1], 0, 1)
    return kp, vp


# ---------------------------------------------------------------------------
# Allocation trace of one PPO iteration (Section 2.1: generation, then the
# actor / reference / critic / reward inferences, then actor and critic
# training).  Only tensor sizes and lifetimes are stated here -- the order in
# which a framework built on an eager tensor library asks its allocator for
# memory -- no allocator policy.  Events:
#   ("phase", name) | ("alloc", key, nbytes, kind) | ("free", key)
# kind is "kv" for the key/value cache of generation and "tensor" otherwise.
@dataclass(frozen=True)
class TraceShape:
    name: str
    n_layers: int
    hidden: int
    n_kv_heads: int
    head_dim: int
    vocab: int
    critic_layers: int
    critic_hidden: int
    batch: int
    prompt_len: int
    gen_len: int
    lora_rank: int = 128


TRACE_SHAPES = {
    # actor/reference OPT-1.3b-shaped, critic/reward OPT-350m-shaped, the paper's batch of 2 (Section 3)
    "opt1.3b_b2": TraceShape("opt1.3b_b2", 24, 2048, 32, 64, 50272, 24, 1024, 2, 256, 256),
    # the same models at a rollout batch of 32 (the other framework's setting in Section 3)
    "opt1.3b_b32": TraceShape("opt1.3b_b32", 24, 2048, 32, 64, 50272, 24, 1024, 32, 256, 256),
}


def ppo_iteration_trace(shape: TraceShape, iterations: int = 2, seed: int = BASE_SEED):
    """Events of `iterations` PPO iterations.  Prompts are padded to a length
    drawn per iteration from [prompt_len/2, prompt_len], so successive
    iterations ask for slightly different sizes, as real batches do."""
    rng = _cpu_rng(seed, 8)
    ev = []
    counter = [0]

    def alloc(nbytes, kind="tensor"):
        counter[0] += 1
        ev.append(("alloc", counter[0], int(nbytes), kind))
        return counter[0]

    def free(key):
        ev.append(("free", key))

    B, NL, Hd, V = shape.batch, shape.n_layers, shape.hidden, shape.vocab
    kv_row = shape.n_kv_heads * shape.head_dim * 2            # bytes of one token's K (or V) in one layer
    # persistent: LoRA adapters, their gradients and optimizer moments (fp32), actor and critic
    ev.append(("phase", "setup"))
    for layers, hid in ((NL, Hd), (shape.critic_layers, shape.critic_hidden)):
        for _ in range(layers):
            for _ in range(4):                                 # adapter, gradient, two moments
                alloc(2 * hid * shape.lora_rank * 4 * 4)       # four adapted projections, A and B halves
    for it in range(iterations):
        P0 = int(rng.integers(max(1, shape.prompt_len // 2), shape.prompt_len + 1))
        G = shape.gen_len
        S = P0 + G
        # ---- generation: the cache of every layer grows by concatenation each step
        ev.append(("phase", f"generation[{it}]"))
        cache = [(alloc(B * P0 * kv_row, "kv"), alloc(B * P0 * kv_row, "kv")) for _ in range(NL)]
        ids = alloc(B * S * 8)
        for t in range(1, G + 1):
            h = alloc(B * Hd * 2)
            for layer in range(NL):
                k_new, v_new = alloc(B * (P0 + t) * kv_row, "kv"), alloc(B * (P0 + t) * kv_row, "kv")
                free(cache[layer][0])
                free(cache[layer][1])
                cache[layer] = (k_new, v_new)
                h2 = alloc(B * Hd * 2)
                free(h)
                h = h2
            logits = alloc(B * V * 4)
            probs = alloc(B * V * 4)
            free(logits)
            free(probs)
            free(h)
        for k_c, v_c in cache:
            free(k_c)
            free(v_c)
        # ---- four inferences over the full sequences
        outputs = []
        for who, layers, hid, head in (("actor", NL, Hd, V), ("reference", NL, Hd, V),
                                       ("critic", shape.critic_layers, shape.critic_hidden, 1),
                                       ("reward", shape.critic_layers, shape.critic_hidden, 1)):
            ev.append(("phase", f"inference:{who}[{it}]"))
            h = alloc(B * S * hid * 2)
            for _ in range(layers):
                att = alloc(B * S * hid * 2 * 3)               # fused q, k, v projections
                h2 = alloc(B * S * hid * 2)
                mlp = alloc(B * S * hid * 4 * 2)
                free(att)
                free(h)
                free(mlp)
                h = h2
            out = alloc(B * S * head * 2)
            free(h)
            if head > 1:
                lsm = alloc(B * S * head * 4)                  # fp32 log-softmax
                free(out)
                out = alloc(B * S * 4)                         # gathered log-probs
                free(lsm)
            outputs.append(out)
        # ---- training: actor, then critic; activations kept for backward, freed in reverse
        for who, layers, hid, head in (("actor", NL, Hd, V), ("critic", shape.critic_layers, shape.critic_hidden, 1)):
            ev.append(("phase", f"training:{who}[{it}]"))
            saved = []
            h = alloc(B * S * hid * 2)
            for _ in range(layers):
                saved.append(alloc(B * S * hid * 2))            # checkpointed layer input
                tmp = alloc(B * S * hid * 4 * 2)
                free(tmp)
            out = alloc(B * S * head * 4)
            grad_out = alloc(B * S * head * 4)
            free(out)
            for s_ in reversed(saved):
                re1 = alloc(B * S * hid * 2 * 3)                # recomputation + gradient temporaries
                re2 = alloc(B * S * hid * 4 * 2)
                g = alloc(B * S * hid * 2)
                free(re1)
                free(re2)
                free(s_)
                free(g)
            free(grad_out)
            free(h)
        for o in outputs:
            free(o)
        free(ids)
    ev.append(("phase", "end"))
    return ev
