"""ctypes binding of librlhf_rollout.so: the same entry points as
include/rlhf_rollout.h, with argument marshalling only.  Every step of the hot
path runs in the library's HIP kernels; there is no fallback of any kind -- if
the shared object is missing, loading raises.

Device buffers are passed as torch tensors (their data_ptr() is used) or as raw
integer addresses; host integer arrays as anything numpy can turn into int32.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

RLHF_OK, RLHF_ERR_INVALID, RLHF_ERR_OOM, RLHF_ERR_DEVICE, RLHF_ERR_UNSUPPORTED = 0, -1, -2, -3, -4
RLHF_F16, RLHF_BF16, RLHF_F32 = 0, 1, 2
RLHF_PAGE_TOKENS = 16
RLHF_ARENA_HOST_ONLY = 1
RLHF_PENALTY_FULL_KL, RLHF_PENALTY_SAMPLED = 0, 1

# RLHF_ROLLOUT_LIB names another build of the same library (same exports) to load instead.
LIB_PATH = os.environ.get("RLHF_ROLLOUT_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)),
                                                             "librlhf_rollout.so")

EXPORTS = [
    "rlhf_kv_arena_bytes_required", "rlhf_kv_arena_create", "rlhf_kv_arena_destroy",
    "rlhf_kv_arena_append", "rlhf_kv_arena_free_seq", "rlhf_kv_arena_fail_next_submissions",
    "rlhf_kv_arena_reset", "rlhf_kv_arena_stats",
    "rlhf_kv_arena_views", "rlhf_kv_arena_host_state", "rlhf_kv_arena_gather",
    "rlhf_decode_attention_workspace_bytes", "rlhf_decode_attention", "rlhf_decode_attention_static",
    "rlhf_token_logprobs_kl",
    "rlhf_token_logprobs_kl_rewards", "rlhf_sample_tokens", "rlhf_sample_tokens_workspace_bytes",
    "rlhf_sample_tokens_split", "rlhf_sample_tokens_topk", "rlhf_prefill_attention",
    "rlhf_prefill_attention_wg", "rlhf_probe_stream_read", "rlhf_probe_matrix_rate",
    "rlhf_last_error_string", "rlhf_version",
    "rlhf_alloc_sim_create", "rlhf_alloc_sim_destroy", "rlhf_alloc_sim_malloc", "rlhf_alloc_sim_free",
    "rlhf_alloc_sim_empty_cache", "rlhf_alloc_sim_stats",
]


class AllocSimStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in (
        "reserved_bytes", "allocated_bytes", "peak_reserved_bytes", "peak_allocated_bytes",
        "driver_allocations", "driver_frees", "last_fragmentation_bytes", "peak_fragmentation_bytes",
        "fragmentation_at_peak_reserved_bytes", "n_segments", "n_free_blocks")]


class RlhfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rlhf status {status}: {message}")
        self.status = status


class ArenaDesc(ctypes.Structure):
    _fields_ = [
        ("max_seqs", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("page_tokens", ctypes.c_int32), ("n_pages", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("kv_dtype", ctypes.c_int32), ("flags", ctypes.c_uint32),
        ("device_buffer", ctypes.c_void_p), ("device_buffer_bytes", ctypes.c_size_t),
        ("initial_free_order", ctypes.c_void_p),
    ]


class ArenaStats(ctypes.Structure):
    _fields_ = [
        ("reserved_bytes", ctypes.c_uint64), ("allocated_bytes", ctypes.c_uint64),
        ("live_token_bytes", ctypes.c_uint64), ("driver_allocations", ctypes.c_uint64),
        ("pages_free", ctypes.c_int32), ("pages_in_use", ctypes.c_int32),
        ("peak_pages_in_use", ctypes.c_int32), ("live_seqs", ctypes.c_int32),
    ]


class AttnParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_tokens", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("max_seq_len", ctypes.c_int32),
        ("qkv_dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
    ]


class RewardShaping(ctypes.Structure):
    _fields_ = [
        ("ref_logp_out", ctypes.c_void_p), ("reward_out", ctypes.c_void_p),
        ("terminal_scores", ctypes.c_void_p), ("kl_coef", ctypes.c_float), ("penalty", ctypes.c_int32),
        ("token_error_flag", ctypes.c_void_p),
    ]


_lib = None


def lib() -> ctypes.CDLL:
    """Loads the shared library on first use; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_15651_amd.build` "
                "(there is no fallback path)")
        # PyTorch carries its own copy of the HIP runtime.  Device memory comes from
        # torch, so its runtime must be the one this process uses: load it first,
        # and the library below binds to the runtime already present.  (Loaded the
        # other way round, two runtimes coexist and this one finds no device.)
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        P = ctypes.POINTER
        L.rlhf_kv_arena_bytes_required.argtypes = [P(ArenaDesc), P(sz)]
        L.rlhf_kv_arena_create.argtypes = [P(ArenaDesc), P(vp)]
        L.rlhf_kv_arena_destroy.argtypes = [vp]
        L.rlhf_kv_arena_append.argtypes = [vp, vp, vp, i32, vp, vp, vp]
        L.rlhf_kv_arena_free_seq.argtypes = [vp, i32, vp]
        L.rlhf_kv_arena_fail_next_submissions.argtypes = [vp, i32]
        L.rlhf_kv_arena_reset.argtypes = [vp, vp]
        L.rlhf_kv_arena_stats.argtypes = [vp, P(ArenaStats)]
        L.rlhf_kv_arena_views.argtypes = [vp, P(vp), P(vp), P(vp), P(vp)]
        L.rlhf_kv_arena_host_state.argtypes = [vp, P(vp), P(vp), P(vp), P(i32)]
        L.rlhf_kv_arena_gather.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.rlhf_decode_attention_workspace_bytes.argtypes = [P(AttnParams), P(sz)]
        L.rlhf_decode_attention.argtypes = [P(AttnParams), vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.rlhf_decode_attention_static.argtypes = [P(AttnParams), vp, vp, vp, vp, vp, vp, vp]
        L.rlhf_token_logprobs_kl.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32, vp]
        L.rlhf_token_logprobs_kl_rewards.argtypes = [vp, vp, vp, vp, vp, i64, i32, i64, i32,
                                                     P(RewardShaping), vp]
        L.rlhf_sample_tokens.argtypes = [vp, vp, vp, i64, i32, i64, i32, ctypes.c_float, ctypes.c_uint64,
                                         ctypes.c_uint64, vp]
        L.rlhf_sample_tokens_workspace_bytes.argtypes = [i64, i32, P(sz)]
        L.rlhf_sample_tokens_split.argtypes = [vp, vp, vp, i64, i32, i64, i32, ctypes.c_float, ctypes.c_uint64,
                                               ctypes.c_uint64, vp, sz, vp]
        L.rlhf_sample_tokens_topk.argtypes = [vp, vp, vp, i64, i32, i64, i32, ctypes.c_float, i32,
                                              ctypes.c_uint64, ctypes.c_uint64, vp]
        L.rlhf_prefill_attention.argtypes = [P(AttnParams), vp, vp, i32, vp, vp, vp, vp, vp, vp]
        L.rlhf_prefill_attention_wg.argtypes = [P(AttnParams), vp, vp, i32, vp, vp, vp, vp, vp, i32, vp]
        L.rlhf_probe_stream_read.argtypes = [vp, sz, vp, vp]
        L.rlhf_probe_matrix_rate.argtypes = [vp, sz, i32, i32, vp, vp]
        u64 = ctypes.c_uint64
        L.rlhf_alloc_sim_create.argtypes = [P(vp)]
        L.rlhf_alloc_sim_destroy.argtypes = [vp]
        L.rlhf_alloc_sim_malloc.argtypes = [vp, u64, P(u64)]
        L.rlhf_alloc_sim_free.argtypes = [vp, u64]
        L.rlhf_alloc_sim_empty_cache.argtypes = [vp]
        L.rlhf_alloc_sim_stats.argtypes = [vp, P(AllocSimStats)]
        L.rlhf_last_error_string.restype = ctypes.c_char_p
        L.rlhf_last_error_string.argtypes = []
        L.rlhf_version.argtypes = []
        for name in EXPORTS:
            if name != "rlhf_last_error_string":
                getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != RLHF_OK:
        raise RlhfError(status, lib().rlhf_last_error_string().decode())


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()          # torch tensor


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        if torch.cuda.is_available() and torch.cuda.is_initialized():
            return torch.cuda.current_stream().cuda_stream or None
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def dtype_code(torch_dtype) -> int:
    import torch
    return {torch.float16: RLHF_F16, torch.bfloat16: RLHF_BF16, torch.float32: RLHF_F32}[torch_dtype]


# ---------------------------------------------------------------- arena ----
def _desc(max_seqs, n_kv_heads, head_dim, n_pages, max_pages_per_seq, kv_dtype, flags=0,
          device_buffer=None, device_buffer_bytes=0, initial_free_order=None,
          page_tokens=RLHF_PAGE_TOKENS):
    order = None
    if initial_free_order is not None:
        order = _i32(initial_free_order)
        if order.shape != (n_pages,):
            raise RlhfError(RLHF_ERR_INVALID, "initial_free_order must have n_pages entries")
    d = ArenaDesc(max_seqs, n_kv_heads, head_dim, page_tokens, n_pages, max_pages_per_seq, kv_dtype,
                  flags, _ptr(device_buffer), device_buffer_bytes,
                  order.ctypes.data if order is not None else None)
    return d, order


def rlhf_kv_arena_bytes_required(**kw) -> int:
    d, _keep = _desc(**kw)
    out = ctypes.c_size_t()
    _check(lib().rlhf_kv_arena_bytes_required(ctypes.byref(d), ctypes.byref(out)))
    return out.value


def rlhf_kv_arena_create(**kw) -> int:
    """Keyword arguments are the fields of rlhf_kv_arena_desc; returns the handle."""
    d, _keep = _desc(**kw)
    h = ctypes.c_void_p()
    _check(lib().rlhf_kv_arena_create(ctypes.byref(d), ctypes.byref(h)))
    return h.value


def rlhf_kv_arena_destroy(arena: int) -> None:
    _check(lib().rlhf_kv_arena_destroy(arena))


def rlhf_kv_arena_append(arena: int, seq_ids: Sequence[int], n_new: Sequence[int], k_new=None,
                         v_new=None, stream=None) -> None:
    ids, cnt = _i32(seq_ids), _i32(n_new)
    if ids.shape != cnt.shape or ids.ndim != 1:
        raise RlhfError(RLHF_ERR_INVALID, "seq_ids and n_new must be 1-D and of equal length")
    _check(lib().rlhf_kv_arena_append(arena, ids.ctypes.data, cnt.ctypes.data, ids.shape[0],
                                      _ptr(k_new), _ptr(v_new), _stream(stream)))


def rlhf_kv_arena_free_seq(arena: int, seq_id: int, stream=None) -> None:
    _check(lib().rlhf_kv_arena_free_seq(arena, seq_id, _stream(stream)))


def rlhf_kv_arena_fail_next_submissions(arena: int, n_calls: int) -> None:
    _check(lib().rlhf_kv_arena_fail_next_submissions(arena, n_calls))


def rlhf_kv_arena_reset(arena: int, stream=None) -> None:
    _check(lib().rlhf_kv_arena_reset(arena, _stream(stream)))


def rlhf_kv_arena_stats(arena: int) -> dict:
    s = ArenaStats()
    _check(lib().rlhf_kv_arena_stats(arena, ctypes.byref(s)))
    return {name: int(getattr(s, name)) for name, _ in ArenaStats._fields_}


def rlhf_kv_arena_views(arena: int):
    """(k_arena, v_arena, page_table, seq_lens) device addresses."""
    k, v, t, l = (ctypes.c_void_p() for _ in range(4))
    _check(lib().rlhf_kv_arena_views(arena, ctypes.byref(k), ctypes.byref(v), ctypes.byref(t), ctypes.byref(l)))
    return k.value, v.value, t.value, l.value


def rlhf_kv_arena_host_state(arena: int, max_seqs: int, max_pages_per_seq: int):
    """Copies of the host mirrors: (page_table [max_seqs, max_pages_per_seq],
    seq_lens [max_seqs], free_list [pages_free])."""
    t, l, f = (ctypes.c_void_p() for _ in range(3))
    n = ctypes.c_int32()
    _check(lib().rlhf_kv_arena_host_state(arena, ctypes.byref(t), ctypes.byref(l), ctypes.byref(f),
                                          ctypes.byref(n)))

    def copy(addr, count):
        if count == 0:
            return np.zeros(0, dtype=np.int32)
        return np.ctypeslib.as_array(ctypes.cast(addr, ctypes.POINTER(ctypes.c_int32)), (count,)).copy()

    table = copy(t.value, max_seqs * max_pages_per_seq).reshape(max_seqs, max_pages_per_seq)
    return table, copy(l.value, max_seqs), copy(f.value, n.value)


def rlhf_kv_arena_gather(arena: int, seq_id: int, start: int, n: int, k_out, v_out, stream=None) -> None:
    _check(lib().rlhf_kv_arena_gather(arena, seq_id, start, n, _ptr(k_out), _ptr(v_out), _stream(stream)))


# ------------------------------------------------------------ attention ----
def attn_params(batch, n_q_heads, n_kv_heads, head_dim, max_pages_per_seq, qkv_dtype, out_dtype=None,
                max_seq_len=0, softmax_scale=0.0, page_tokens=RLHF_PAGE_TOKENS) -> AttnParams:
    return AttnParams(batch, n_q_heads, n_kv_heads, head_dim, page_tokens, max_pages_per_seq,
                      max_seq_len, qkv_dtype, qkv_dtype if out_dtype is None else out_dtype,
                      softmax_scale)


def rlhf_decode_attention_workspace_bytes(params: AttnParams) -> int:
    out = ctypes.c_size_t()
    _check(lib().rlhf_decode_attention_workspace_bytes(ctypes.byref(params), ctypes.byref(out)))
    return out.value


def rlhf_decode_attention_static(params: AttnParams, q, k_arena, v_arena, page_table, seq_lens, out,
                                 stream=None) -> None:
    _check(lib().rlhf_decode_attention_static(ctypes.byref(params), _ptr(q), _ptr(k_arena), _ptr(v_arena),
                                              _ptr(page_table), _ptr(seq_lens), _ptr(out), _stream(stream)))


def rlhf_decode_attention(params: AttnParams, q, k_arena, v_arena, page_table, seq_lens, out,
                          workspace, workspace_bytes: Optional[int] = None, stream=None) -> None:
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(lib().rlhf_decode_attention(ctypes.byref(params), _ptr(q), _ptr(k_arena), _ptr(v_arena),
                                       _ptr(page_table), _ptr(seq_lens), _ptr(out), _ptr(workspace),
                                       workspace_bytes, _stream(stream)))


def rlhf_prefill_attention(params: AttnParams, q, cu_q, max_q_len: int, k_arena, v_arena, page_table,
                           seq_lens, out, stream=None) -> None:
    _check(lib().rlhf_prefill_attention(ctypes.byref(params), _ptr(q), _ptr(cu_q), int(max_q_len),
                                        _ptr(k_arena), _ptr(v_arena), _ptr(page_table), _ptr(seq_lens),
                                        _ptr(out), _stream(stream)))


def rlhf_prefill_attention_wg(params: AttnParams, q, cu_q, max_q_len: int, k_arena, v_arena, page_table,
                              seq_lens, out, wavefronts_per_workgroup: int, stream=None) -> None:
    _check(lib().rlhf_prefill_attention_wg(ctypes.byref(params), _ptr(q), _ptr(cu_q), int(max_q_len),
                                           _ptr(k_arena), _ptr(v_arena), _ptr(page_table), _ptr(seq_lens),
                                           _ptr(out), int(wavefronts_per_workgroup), _stream(stream)))


# ----------------------------------------------------------- logprob/KL ----
def rlhf_token_logprobs_kl(actor_logits, ref_logits, tokens, logp_out, kl_out, n_positions=None,
                           vocab=None, row_stride_elems=0, logits_dtype=None, stream=None) -> None:
    if n_positions is None:
        n_positions = actor_logits.shape[0]
    if vocab is None:
        vocab = actor_logits.shape[1]
        row_stride_elems = actor_logits.stride(0)
    if logits_dtype is None:
        logits_dtype = dtype_code(actor_logits.dtype)
    _check(lib().rlhf_token_logprobs_kl(_ptr(actor_logits), _ptr(ref_logits), _ptr(tokens), _ptr(logp_out),
                                        _ptr(kl_out), n_positions, vocab, row_stride_elems, logits_dtype,
                                        _stream(stream)))


def rlhf_token_logprobs_kl_rewards(actor_logits, ref_logits, tokens, logp_out, kl_out, kl_coef,
                                   penalty=RLHF_PENALTY_FULL_KL, ref_logp_out=None, reward_out=None,
                                   terminal_scores=None, n_positions=None, vocab=None, row_stride_elems=0,
                                   logits_dtype=None, stream=None, token_error_flag=None) -> None:
    if n_positions is None:
        n_positions = actor_logits.shape[0]
    if vocab is None:
        vocab = actor_logits.shape[1]
        row_stride_elems = actor_logits.stride(0)
    if logits_dtype is None:
        logits_dtype = dtype_code(actor_logits.dtype)
    sh = RewardShaping(_ptr(ref_logp_out), _ptr(reward_out), _ptr(terminal_scores), kl_coef, penalty,
                       _ptr(token_error_flag))
    _check(lib().rlhf_token_logprobs_kl_rewards(_ptr(actor_logits), _ptr(ref_logits), _ptr(tokens),
                                                _ptr(logp_out), _ptr(kl_out), n_positions, vocab,
                                                row_stride_elems, logits_dtype, ctypes.byref(sh),
                                                _stream(stream)))


def rlhf_sample_tokens(logits, tokens_out, temperature, seed, offset=0, logp_out=None, n_rows=None,
                       vocab=None, row_stride_elems=0, logits_dtype=None, stream=None) -> None:
    if n_rows is None:
        n_rows = logits.shape[0]
    if vocab is None:
        vocab = logits.shape[1]
        row_stride_elems = logits.stride(0)
    if logits_dtype is None:
        logits_dtype = dtype_code(logits.dtype)
    _check(lib().rlhf_sample_tokens(_ptr(logits), _ptr(tokens_out), _ptr(logp_out), n_rows, vocab,
                                    row_stride_elems, logits_dtype, temperature, seed, offset,
                                    _stream(stream)))


def rlhf_sample_tokens_workspace_bytes(n_rows: int, vocab: int) -> int:
    out = ctypes.c_size_t()
    _check(lib().rlhf_sample_tokens_workspace_bytes(n_rows, vocab, ctypes.byref(out)))
    return out.value


def rlhf_sample_tokens_split(logits, tokens_out, temperature, seed, workspace, offset=0, logp_out=None,
                             n_rows=None, vocab=None, row_stride_elems=0, logits_dtype=None,
                             workspace_bytes=None, stream=None) -> None:
    if n_rows is None:
        n_rows = logits.shape[0]
    if vocab is None:
        vocab = logits.shape[1]
        row_stride_elems = logits.stride(0)
    if logits_dtype is None:
        logits_dtype = dtype_code(logits.dtype)
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(lib().rlhf_sample_tokens_split(_ptr(logits), _ptr(tokens_out), _ptr(logp_out), n_rows, vocab,
                                          row_stride_elems, logits_dtype, temperature, seed, offset,
                                          _ptr(workspace), workspace_bytes, _stream(stream)))


def rlhf_sample_tokens_topk(logits, tokens_out, temperature, top_k, seed, offset=0, logp_out=None, n_rows=None,
                            vocab=None, row_stride_elems=0, logits_dtype=None, stream=None) -> None:
    if n_rows is None:
        n_rows = logits.shape[0]
    if vocab is None:
        vocab = logits.shape[1]
        row_stride_elems = logits.stride(0)
    if logits_dtype is None:
        logits_dtype = dtype_code(logits.dtype)
    _check(lib().rlhf_sample_tokens_topk(_ptr(logits), _ptr(tokens_out), _ptr(logp_out), n_rows, vocab,
                                         row_stride_elems, logits_dtype, temperature, top_k, seed, offset,
                                         _stream(stream)))


def rlhf_probe_stream_read(buffer, nbytes=None, sink=None, stream=None) -> None:
    if nbytes is None:
        nbytes = buffer.numel() * buffer.element_size()
    _check(lib().rlhf_probe_stream_read(_ptr(buffer), nbytes, _ptr(sink), _stream(stream)))


def rlhf_probe_matrix_rate(operands, iterations, n_workgroups, ticks, nbytes=None, stream=None) -> None:
    if nbytes is None:
        nbytes = operands.numel() * operands.element_size()
    _check(lib().rlhf_probe_matrix_rate(_ptr(operands), nbytes, iterations, n_workgroups, _ptr(ticks),
                                        _stream(stream)))


def rlhf_last_error_string() -> str:
    return lib().rlhf_last_error_string().decode()


def rlhf_version() -> int:
    return lib().rlhf_version()


# ------------------------------------------------- allocator simulator ----
class AllocSim:
    """The library's caching-allocator simulator (include/rlhf_memtrace.h)."""

    def __init__(self):
        h = ctypes.c_void_p()
        _check(lib().rlhf_alloc_sim_create(ctypes.byref(h)))
        self._h = h

    def malloc(self, nbytes: int) -> int:
        out = ctypes.c_uint64()
        _check(lib().rlhf_alloc_sim_malloc(self._h, int(nbytes), ctypes.byref(out)))
        return out.value

    def free(self, handle: int) -> None:
        _check(lib().rlhf_alloc_sim_free(self._h, int(handle)))

    def empty_cache(self) -> None:
        _check(lib().rlhf_alloc_sim_empty_cache(self._h))

    def stats(self) -> dict:
        st = AllocSimStats()
        _check(lib().rlhf_alloc_sim_stats(self._h, ctypes.byref(st)))
        return {n: getattr(st, n) for n, _ in AllocSimStats._fields_}

    def close(self) -> None:
        if self._h:
            lib().rlhf_alloc_sim_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
