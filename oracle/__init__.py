"""fp64 CPU oracle for the rollout hot path -- TEST INFRASTRUCTURE ONLY.

Nothing in the product package imports this.  It exists so that tests, the
smoke check and the benchmark's CPU-baseline leg can compare the GPU library
with the plain definitions (see rollout_oracle.c for what each function
computes and which passage of the paper names the quantity).

`build()` compiles rollout_oracle.c with gcc into this directory; the wrappers
below marshal numpy arrays into it.  16-bit floating-point inputs are passed as
raw uint16 bit patterns together with a dtype code.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from .alloc_model import CachingAllocatorModel  # noqa: F401
from .arena_model import ArenaModel, ArenaModelError  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rollout_oracle.c")
_LIB = os.path.join(_HERE, "librollout_oracle.so")

F16, BF16, F32 = 0, 1, 2


def build(force: bool = False, src: str = _SRC, lib: str = _LIB) -> str:
    """Compile the C oracle (gcc, OpenMP) if it is missing or stale."""
    if (not force and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(src)):
        return lib
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
           "-fno-fast-math", "-Wall", "-Wextra", src, "-o", lib, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def _storage(arr: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if arr.dtype != want:
        raise TypeError(f"dtype code {dtype} needs a {want.__name__} array, got {arr.dtype}")
    return np.ascontiguousarray(arr)


class OracleLib:
    """The compiled oracle behind numpy wrappers.  The module-level functions use
    the in-tree build; tests that plant a mistake in a copy of the C source load
    that copy through this class."""

    F16, BF16, F32 = F16, BF16, F32

    def __init__(self, lib_path: str):
        lib = ctypes.CDLL(lib_path)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_decode_attention.restype = ctypes.c_int
        lib.oracle_decode_attention.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_double]
        lib.oracle_token_logprobs_kl.restype = ctypes.c_int
        lib.oracle_token_logprobs_kl.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int64, ctypes.c_int]
        lib.oracle_token_rewards.restype = ctypes.c_int
        lib.oracle_token_rewards.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int64, ctypes.c_int, ctypes.c_double, ctypes.c_int]
        lib.oracle_prefill_attention.restype = ctypes.c_int
        lib.oracle_prefill_attention.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_double]
        lib.oracle_philox4x32_10.restype = None
        lib.oracle_philox4x32_10.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_sample_tokens.restype = ctypes.c_int
        lib.oracle_sample_tokens.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
            ctypes.c_double, ctypes.c_uint64, ctypes.c_uint64]
        lib.oracle_sample_tokens_topk.restype = ctypes.c_int
        lib.oracle_sample_tokens_topk.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
            ctypes.c_double, ctypes.c_int, ctypes.c_uint64, ctypes.c_uint64]
        self._lib = lib

    def num_threads(self) -> int:
        return int(self._lib.oracle_num_threads())

    def decode_attention(self, q, k_pages, v_pages, page_table, seq_lens, dtype, scale=None,
                         return_weights=False):
        """q [B,Hq,D], k_pages/v_pages [n_pages,Hkv,P,D] (plain token-major pages),
        page_table [B,max_pages] int32, seq_lens [B] int32 -> out [B,Hq,D] float64."""
        q = _storage(q, dtype)
        k_pages = _storage(k_pages, dtype)
        v_pages = _storage(v_pages, dtype)
        B, Hq, D = q.shape
        n_pages, Hkv, P, D2 = k_pages.shape
        assert D2 == D and v_pages.shape == k_pages.shape
        page_table = np.ascontiguousarray(page_table, dtype=np.int32).reshape(B, -1)
        seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
        assert seq_lens.shape == (B,)
        max_pages = page_table.shape[1]
        used = (seq_lens.astype(np.int64) + P - 1) // P
        for b in range(B):
            row = page_table[b, :used[b]]
            if row.size and (row.min() < 0 or row.max() >= n_pages):
                raise ValueError("page table entry out of range")
        if scale is None:
            scale = 1.0 / np.sqrt(D)
        out = np.zeros((B, Hq, D), dtype=np.float64)
        weights = np.zeros((B, Hq, max_pages * P), dtype=np.float64) if return_weights else None
        rc = self._lib.oracle_decode_attention(
            q.ctypes.data, k_pages.ctypes.data, v_pages.ctypes.data,
            page_table.ctypes.data, seq_lens.ctypes.data, out.ctypes.data,
            weights.ctypes.data if return_weights else None,
            B, Hq, Hkv, D, P, max_pages, dtype, float(scale))
        if rc != 0:
            raise ValueError("oracle_decode_attention rejected its arguments")
        return (out, weights) if return_weights else out

    def token_logprobs_kl(self, actor, ref, tokens, dtype, vocab=None):
        """actor/ref [N,stride] rows (first `vocab` columns used), tokens [N] int32
        -> (logp [N], kl [N]) float64."""
        actor = _storage(actor, dtype)
        ref = _storage(ref, dtype)
        assert actor.shape == ref.shape and actor.ndim == 2
        N, stride = actor.shape
        V = stride if vocab is None else int(vocab)
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        assert tokens.shape == (N,)
        logp = np.zeros(N, dtype=np.float64)
        kl = np.zeros(N, dtype=np.float64)
        rc = self._lib.oracle_token_logprobs_kl(
            actor.ctypes.data, ref.ctypes.data, tokens.ctypes.data,
            logp.ctypes.data, kl.ctypes.data, N, V, stride, dtype)
        if rc != 0:
            raise ValueError("oracle_token_logprobs_kl rejected its arguments")
        return logp, kl


    def token_rewards(self, actor, ref, tokens, dtype, kl_coef, sampled_penalty, terminal=None,
                      vocab=None):
        """-> (ref_logp [N], reward [N]) float64; terminal [N] float64 or None."""
        actor = _storage(actor, dtype)
        ref = _storage(ref, dtype)
        assert actor.shape == ref.shape and actor.ndim == 2
        N, stride = actor.shape
        V = stride if vocab is None else int(vocab)
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        term = None if terminal is None else np.ascontiguousarray(terminal, dtype=np.float64)
        assert tokens.shape == (N,) and (term is None or term.shape == (N,))
        ref_logp = np.zeros(N, dtype=np.float64)
        reward = np.zeros(N, dtype=np.float64)
        rc = self._lib.oracle_token_rewards(
            actor.ctypes.data, ref.ctypes.data, tokens.ctypes.data,
            None if term is None else term.ctypes.data, ref_logp.ctypes.data, reward.ctypes.data,
            N, V, stride, dtype, float(kl_coef), int(bool(sampled_penalty)))
        if rc != 0:
            raise ValueError("oracle_token_rewards rejected its arguments")
        return ref_logp, reward


    def prefill_attention(self, q, cu_q, k_pages, v_pages, page_table, seq_lens, dtype, scale=None):
        """q [T,Hq,D] packed query rows, cu_q [B+1] int32 offsets (sequence b owns rows
        cu_q[b]:cu_q[b+1], the last tokens of its cache) -> out [T,Hq,D] float64."""
        q = _storage(q, dtype)
        k_pages = _storage(k_pages, dtype)
        v_pages = _storage(v_pages, dtype)
        T, Hq, D = q.shape
        n_pages, Hkv, P, D2 = k_pages.shape
        assert D2 == D and v_pages.shape == k_pages.shape
        cu_q = np.ascontiguousarray(cu_q, dtype=np.int32)
        B = cu_q.shape[0] - 1
        assert cu_q[0] == 0 and cu_q[-1] == T
        page_table = np.ascontiguousarray(page_table, dtype=np.int32).reshape(B, -1)
        seq_lens = np.ascontiguousarray(seq_lens, dtype=np.int32)
        assert seq_lens.shape == (B,)
        used = (seq_lens.astype(np.int64) + P - 1) // P
        for b in range(B):
            row = page_table[b, :used[b]]
            if row.size and (row.min() < 0 or row.max() >= n_pages):
                raise ValueError("page table entry out of range")
        if scale is None:
            scale = 1.0 / np.sqrt(D)
        out = np.zeros((T, Hq, D), dtype=np.float64)
        rc = self._lib.oracle_prefill_attention(
            q.ctypes.data, cu_q.ctypes.data, k_pages.ctypes.data, v_pages.ctypes.data,
            page_table.ctypes.data, seq_lens.ctypes.data, out.ctypes.data,
            B, Hq, Hkv, D, P, page_table.shape[1], dtype, float(scale))
        if rc != 0:
            raise ValueError("oracle_prefill_attention rejected its arguments")
        return out

    def philox4x32_10(self, ctr, key):
        c = np.ascontiguousarray(ctr, dtype=np.uint32)
        k = np.ascontiguousarray(key, dtype=np.uint32)
        assert c.shape == (4,) and k.shape == (2,)
        out = np.zeros(4, dtype=np.uint32)
        self._lib.oracle_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
        return out

    def sample_tokens(self, logits, dtype, temperature, seed, offset=0, vocab=None,
                      return_perturbed=False):
        """logits [N,stride] -> (tokens [N] int32, logp [N] float64[, perturbed [N,V]])."""
        logits = _storage(logits, dtype)
        assert logits.ndim == 2
        N, stride = logits.shape
        V = stride if vocab is None else int(vocab)
        tokens = np.zeros(N, dtype=np.int32)
        logp = np.zeros(N, dtype=np.float64)
        pert = np.zeros((N, V), dtype=np.float64) if return_perturbed else None
        rc = self._lib.oracle_sample_tokens(
            logits.ctypes.data, tokens.ctypes.data, logp.ctypes.data,
            pert.ctypes.data if return_perturbed else None, N, V, stride, dtype,
            float(temperature), int(seed), int(offset))
        if rc != 0:
            raise ValueError("oracle_sample_tokens rejected its arguments")
        return (tokens, logp, pert) if return_perturbed else (tokens, logp)


    def sample_tokens_topk(self, logits, dtype, temperature, top_k, seed, offset=0, vocab=None,
                           return_perturbed=False):
        """logits [N,stride] -> (tokens [N] int32, logp [N] float64, threshold [N] float64,
        count [N] int32[, perturbed [N,V] with -inf for removed entries])."""
        logits = _storage(logits, dtype)
        assert logits.ndim == 2
        N, stride = logits.shape
        V = stride if vocab is None else int(vocab)
        tokens = np.zeros(N, dtype=np.int32)
        logp = np.zeros(N, dtype=np.float64)
        tau = np.zeros(N, dtype=np.float64)
        count = np.zeros(N, dtype=np.int32)
        pert = np.zeros((N, V), dtype=np.float64) if return_perturbed else None
        rc = self._lib.oracle_sample_tokens_topk(
            logits.ctypes.data, tokens.ctypes.data, logp.ctypes.data,
            pert.ctypes.data if return_perturbed else None, tau.ctypes.data, count.ctypes.data,
            N, V, stride, dtype, float(temperature), int(top_k), int(seed), int(offset))
        if rc != 0:
            raise ValueError("oracle_sample_tokens_topk rejected its arguments")
        return (tokens, logp, tau, count, pert) if return_perturbed else (tokens, logp, tau, count)


_default = None


def _load() -> OracleLib:
    global _default
    if _default is None:
        _default = OracleLib(build())
    return _default


def num_threads() -> int:
    return _load().num_threads()


def decode_attention(*args, **kw):
    return _load().decode_attention(*args, **kw)


def token_logprobs_kl(*args, **kw):
    return _load().token_logprobs_kl(*args, **kw)


def token_rewards(*args, **kw):
    return _load().token_rewards(*args, **kw)


def prefill_attention(*args, **kw):
    return _load().prefill_attention(*args, **kw)


def philox4x32_10(*args, **kw):
    return _load().philox4x32_10(*args, **kw)


def sample_tokens(*args, **kw):
    return _load().sample_tokens(*args, **kw)


def sample_tokens_topk(*args, **kw):
    return _load().sample_tokens_topk(*args, **kw)


decode_attention.__doc__ = OracleLib.decode_attention.__doc__
token_logprobs_kl.__doc__ = OracleLib.token_logprobs_kl.__doc__
