"""ctypes binding for libmemosight.so: argument marshalling only, same names as the C ABI.

Device tensors are passed as torch tensors (their data_ptr() is handed over), host control arrays
as sequences of ints.  There is no fallback: if the HIP library cannot be loaded, importing this
module fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
from typing import Optional, Sequence

# torch ships its own HIP runtime (same SONAME as the system one).  It is imported first so that
# the library below binds to that already-loaded copy: two HIP runtimes in one process do not share
# devices, streams or allocations.
import torch  # noqa: F401

from . import build as _build

MS_PAGE_SIZE = 16
MS_MAX_BATCH = 256
MS_MAX_QUERIES = 64
MS_F32, MS_BF16 = 0, 1
MS_OK, MS_ERR_INVALID, MS_ERR_OOM_PAGES, MS_ERR_RANGE = 0, -1, -2, -3
MS_ERR_HIP, MS_ERR_UNSUPPORTED, MS_ERR_WORKSPACE = -4, -5, -6
MS_PRE_ROTATED, MS_ROPE_APPLY = 0, 1


class MsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"memosight error {code}: {msg}")
        self.code = code


class ms_cache_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("n_q_heads", C.c_int), ("n_kv_heads", C.c_int),
                ("head_dim", C.c_int), ("page_size", C.c_int), ("n_pages", C.c_int),
                ("max_seqs", C.c_int), ("max_pages_per_seq", C.c_int), ("dtype", C.c_int),
                ("rope_base", C.c_float), ("pool", C.c_void_p), ("pool_bytes", C.c_size_t)]


def _load() -> C.CDLL:
    if not os.path.exists(_build.LIB):
        _build.build()
    return C.CDLL(_build.LIB)


lib = _load()

_P, _I, _IP, _SZ, _F = C.c_void_p, C.c_int, C.POINTER(C.c_int), C.c_size_t, C.c_float
_SIGS = {
    "ms_last_error": (C.c_char_p, []),
    "ms_pool_bytes": (_SZ, [C.POINTER(ms_cache_desc)]),
    "ms_cache_create": (_I, [C.POINTER(ms_cache_desc), C.POINTER(_P)]),
    "ms_cache_destroy": (_I, [_P]),
    "ms_seq_create": (_I, [_P, _IP]),
    "ms_seq_import": (_I, [_P, _I, _IP, _I, _IP, _P]),
    "ms_seq_free": (_I, [_P, _I]),
    "ms_append_kv": (_I, [_P, _I, _IP, _IP, _P, _P, _P, _I, _P]),
    "ms_commit_accepted": (_I, [_P, _I, _IP, _IP, _I, _P, _P, _P, _P]),
    "ms_commit_accepted_device": (_I, [_P, _I, _IP, _P, _I, _I, _P, _P, _P, _P, _P]),
    "ms_cache_sync": (_I, [_P]),
    "ms_step_positions_device": (_I, [_I, _P, _I, _I, _P, _P]),
    "ms_compact_segment": (_I, [_P, _I, _IP, _IP, _IP, _IP, _P, _P, _P, _I, _P, _SZ, _P]),
    "ms_compact_workspace_bytes": (_SZ, [_P, _I, _IP, _IP, _IP]),
    "ms_predict_verify_attention": (_I, [_P, _I, _I, _IP, _I, _I, _P, _P, _P, _P, _P, _F, _P, _P, _SZ, _P]),
    "ms_attention_workspace_bytes": (_SZ, [_P, _I, _I]),
    "ms_predict_verify_attention_static": (_I, [_P, _I, _I, _IP, _I, _I, _P, _P, _P, _P, _P, _F, _P, _P]),
    "ms_accept": (_I, [_I, _I, _P, _P, _P, _I, _P, _P, _P]),
    "ms_seq_len": (_I, [_P, _I, _IP]),
    "ms_seq_page_table": (_I, [_P, _I, _IP, _I, _IP]),
    "ms_free_page_count": (_I, [_P, _IP]),
    "ms_peak_pages": (_I, [_P, _IP]),
    "ms_launch_count": (_I, [_P, C.POINTER(C.c_longlong)]),
    "ms_check_integrity": (_I, [_P, _P]),
    "ms_attention_set_deterministic": (_I, [_P, _I]),
    "ms_attention_fault_injection": (_I, [_P, _I, _I, _P]),
    "ms_embed_rows": (_I, [_P, _I, _I, _P, _I, _P, _P]),
    "ms_add_rmsnorm": (_I, [_P, _P, _P, _F, _P, _I, _I, _P]),
    "ms_swiglu": (_I, [_P, _P, _I, _I, _P]),
    "ms_argmax_rows": (_I, [_P, _I, _I, C.c_long, _P, _P]),
    "ms_gemm_workspace_bytes": (_SZ, [_I, _I, _I, _I]),
    "ms_gemm_swiglu_bf16": (_I, [_P, _P, _I, _I, _I, _P, _P, _SZ, _P]),
    "ms_gemm_add_rmsnorm_workspace_bytes": (_SZ, [_I, _I, _I, _I]),
    "ms_gemm_add_rmsnorm_bf16": (_I, [_P, _P, _I, _I, _I, _I, _P, _P, _F, _P, _P, _SZ, _P]),
    "ms_lm_head_argmax_workspace_bytes": (_SZ, [_I, _I, _I]),
    "ms_lm_head_argmax_bf16": (_I, [_P, _P, _I, _I, _I, _P, _P, _SZ, _P]),
    "ms_gemm_bf16": (_I, [_P, _P, _P, _I, _I, _I, _I, C.POINTER(_P), _IP, _I, _P, _SZ, _P]),
    "ms_profile_attention": (_I, [_P, _I, _I, _I]),
    "ms_profile_read": (_I, [_P, C.POINTER(C.c_float), _I, _IP]),
    "ms_hbm_read_probe": (_I, [_P, C.c_size_t, _I, _P, _P, C.POINTER(C.c_size_t)]),
    "ms_ama_count": (_I, [_I, _I]),
    "ms_upl_positions": (_I, [_I, _I, _I, _IP, _I]),
    "ms_output_token_pid": (_I, [_I]),
    "ms_foresight_pids": (_I, [_I, _I, _IP, _I]),
    "ms_default_ctx_new": (_I, [_I, _I, _IP, _I]),
    "ms_step_positions": (_I, [_I, _IP, _I, _I, _IP]),
    "ms_per_position_layout": (_I, [_I, _I, _I, _IP, _IP, _I]),
    "ms_consecutive_memory_positions": (_I, [_I, _I, _IP, _I]),
    "ms_upl_positions_fixed": (_I, [_I, _I, _I, _IP, _I]),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args

EXPORTED = tuple(_SIGS)


def _check(rc: int) -> None:
    if rc != MS_OK:
        raise MsError(rc, lib.ms_last_error().decode())


def int_array(xs: Sequence[int]):
    """A C int array holding xs.  Pass the result instead of a list to skip the conversion on every call
    (sequence ids, for instance, are the same for all layers of a step)."""
    xs = [int(x) for x in xs]
    if not xs:
        raise ValueError("int_array needs at least one element")
    return (C.c_int * len(xs))(*xs)


def _ints(xs):
    if isinstance(xs, C.Array):                       # already marshalled (int_array)
        return xs
    if isinstance(xs, np.ndarray) and xs.dtype == np.int32 and xs.flags["C_CONTIGUOUS"] and xs.size > 0:
        return xs.ctypes.data_as(_IP)                 # read during the call only
    xs = [int(x) for x in xs]
    return (C.c_int * max(1, len(xs)))(*xs)


def _dev(t) -> Optional[int]:
    """Device address of a torch tensor (None stays NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous device tensor")
    return t.data_ptr()


_DESC = {}   # cache handle -> (n_layers, n_q_heads, n_kv_heads, head_dim, element size)


def _sized(cache, t, what: str, n_elems: int, elem_size: Optional[int] = None) -> Optional[int]:
    """Device address of a tensor that must hold at least n_elems elements.  The C functions take
    bare pointers and trust the sizes they are told, so the extents are checked here."""
    if t is None:
        return None
    want = _DESC[cache][4] if elem_size is None else elem_size
    if t.numel() < n_elems or t.element_size() != want:
        raise MsError(MS_ERR_INVALID, f"{what}: expected at least {n_elems} elements of {want} bytes, got "
                                      f"{t.numel()} of {t.element_size()}")
    return _dev(t)


def _stream(stream) -> Optional[int]:
    if type(stream) is int:                           # a raw hipStream_t value
        return stream or None
    if stream is None:
        if not torch.cuda.is_available():
            return None
        return torch.cuda.current_stream().cuda_stream or None
    return getattr(stream, "cuda_stream", stream) or None


def ms_last_error() -> str:
    return lib.ms_last_error().decode()


def make_desc(n_layers, n_q_heads, n_kv_heads, head_dim, n_pages, max_seqs, max_pages_per_seq, dtype,
              rope_base, pool=None) -> ms_cache_desc:
    d = ms_cache_desc(n_layers, n_q_heads, n_kv_heads, head_dim, MS_PAGE_SIZE, n_pages, max_seqs,
                      max_pages_per_seq, dtype, rope_base, None, 0)
    if pool is not None:
        d.pool = _dev(pool)
        d.pool_bytes = pool.numel() * pool.element_size()
    return d


def ms_pool_bytes(desc: ms_cache_desc) -> int:
    return lib.ms_pool_bytes(C.byref(desc))


def ms_cache_create(desc: ms_cache_desc) -> int:
    h = _P()
    _check(lib.ms_cache_create(C.byref(desc), C.byref(h)))
    _DESC[h.value] = (desc.n_layers, desc.n_q_heads, desc.n_kv_heads, desc.head_dim, 2 if desc.dtype == MS_BF16 else 4)
    return h.value


def ms_cache_destroy(cache: int) -> None:
    _check(lib.ms_cache_destroy(cache))
    _DESC.pop(cache, None)


def ms_seq_create(cache: int) -> int:
    s = C.c_int(-1)
    _check(lib.ms_seq_create(cache, C.byref(s)))
    return s.value


def ms_seq_import(cache: int, length: int, pages: Sequence[int], stream=None) -> int:
    s = C.c_int(-1)
    _check(lib.ms_seq_import(cache, length, _ints(pages), len(pages), C.byref(s), _stream(stream)))
    return s.value


def ms_seq_free(cache: int, seq_id: int) -> None:
    _check(lib.ms_seq_free(cache, seq_id))


def ms_append_kv(cache, seq_ids, n_tok, k, v, pos_ids, flags=MS_ROPE_APPLY, stream=None) -> None:
    L, _, hkv, d, _ = _DESC[cache]
    rows = sum(int(n) for n in n_tok)
    _check(lib.ms_append_kv(cache, len(seq_ids), _ints(seq_ids), _ints(n_tok),
                            _sized(cache, k, "k", L * rows * hkv * d), _sized(cache, v, "v", L * rows * hkv * d),
                            _sized(cache, pos_ids, "pos_ids", rows, 4), flags, _stream(stream)))


def ms_commit_accepted(cache, seq_ids, accept_len, n_q, k_new, v_new, pos_ids, stream=None) -> None:
    L, _, hkv, d, _ = _DESC[cache]
    n = L * len(seq_ids) * n_q * hkv * d
    _check(lib.ms_commit_accepted(cache, len(seq_ids), _ints(seq_ids), _ints(accept_len), n_q,
                                  _sized(cache, k_new, "k_new", n), _sized(cache, v_new, "v_new", n),
                                  _sized(cache, pos_ids, "pos_ids", len(seq_ids) * n_q, 4), _stream(stream)))


def ms_commit_accepted_device(cache, seq_ids, accept_len, n_q, n_max, k_new, v_new, pos_ids, first_pid=None, stream=None) -> None:
    """accept_len (and first_pid, if given): int32 device tensors [B]."""
    L, _, hkv, d, _ = _DESC[cache]
    B = len(seq_ids)
    n = L * B * n_q * hkv * d
    _check(lib.ms_commit_accepted_device(cache, B, _ints(seq_ids), _sized(cache, accept_len, "accept_len", B, 4), n_q, n_max,
                                         _sized(cache, k_new, "k_new", n), _sized(cache, v_new, "v_new", n),
                                         _sized(cache, pos_ids, "pos_ids", B * n_q, 4), _sized(cache, first_pid, "first_pid", B, 4),
                                         _stream(stream)))


def ms_cache_sync(cache) -> None:
    _check(lib.ms_cache_sync(cache))


def ms_step_positions_device(first_pid, n_verify: int, n_foresight: int, out, stream=None) -> None:
    """first_pid: int32 device tensor [B]; out: int32 device tensor [B, n_verify + n_foresight]."""
    B = first_pid.numel()
    _check(lib.ms_step_positions_device(B, _sized(None, first_pid, "first_pid", B, 4), n_verify, n_foresight,
                                        _sized(None, out, "out", B * (n_verify + n_foresight), 4), _stream(stream)))


def ms_compact_workspace_bytes(cache, seq_ids, seg_begin, seg_len) -> int:
    return lib.ms_compact_workspace_bytes(cache, len(seq_ids), _ints(seq_ids), _ints(seg_begin), _ints(seg_len))


def ms_compact_segment(cache, seq_ids, seg_begin, seg_len, n_mem, mem_k, mem_v, mem_pos,
                       flags=MS_ROPE_APPLY, workspace=None, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    L, _, hkv, d, _ = _DESC[cache]
    rows = sum(int(n) for n in n_mem)
    _check(lib.ms_compact_segment(cache, len(seq_ids), _ints(seq_ids), _ints(seg_begin), _ints(seg_len),
                                  _ints(n_mem), _sized(cache, mem_k, "mem_k", L * rows * hkv * d),
                                  _sized(cache, mem_v, "mem_v", L * rows * hkv * d),
                                  _sized(cache, mem_pos, "mem_pos", rows, 4), flags,
                                  _dev(workspace), ws_bytes, _stream(stream)))


def ms_attention_workspace_bytes(cache, B: int, n_q: int) -> int:
    return lib.ms_attention_workspace_bytes(cache, B, n_q)


def ms_predict_verify_attention(cache, layer, seq_ids, n_verify, n_foresight, q, k_new, v_new, pos_ids,
                                ctx_new, scale, out, workspace, stream=None) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _, hq, hkv, d, _ = _DESC[cache]
    rows = len(seq_ids) * (n_verify + n_foresight)
    _check(lib.ms_predict_verify_attention(cache, layer, len(seq_ids), _ints(seq_ids), n_verify, n_foresight,
                                           _sized(cache, q, "q", rows * hq * d), _sized(cache, k_new, "k_new", rows * hkv * d),
                                           _sized(cache, v_new, "v_new", rows * hkv * d), _sized(cache, pos_ids, "pos_ids", rows, 4),
                                           _sized(cache, ctx_new, "ctx_new", rows, 4), float(scale),
                                           _sized(cache, out, "out", rows * hq * d), _dev(workspace), ws_bytes,
                                           _stream(stream)))


MS_STATIC_SCRATCH_BYTES = 32 << 20


def ms_predict_verify_attention_static(cache, layer, seq_ids, n_verify, n_foresight, q, k_new, v_new, pos_ids,
                                       ctx_new, scale, out, stream=None) -> None:
    """ms_predict_verify_attention on the library's fixed workspace (no device allocation anywhere)."""
    _, hq, hkv, d, _ = _DESC[cache]
    rows = len(seq_ids) * (n_verify + n_foresight)
    _check(lib.ms_predict_verify_attention_static(cache, layer, len(seq_ids), _ints(seq_ids), n_verify, n_foresight,
                                                  _sized(cache, q, "q", rows * hq * d), _sized(cache, k_new, "k_new", rows * hkv * d),
                                                  _sized(cache, v_new, "v_new", rows * hkv * d), _sized(cache, pos_ids, "pos_ids", rows, 4),
                                                  _sized(cache, ctx_new, "ctx_new", rows, 4), float(scale),
                                                  _sized(cache, out, "out", rows * hq * d), _stream(stream)))


def ms_embed_rows(table, tokens, h_out, stream=None) -> None:
    vocab, hidden = table.shape
    n = tokens.numel()
    _check(lib.ms_embed_rows(_sized(None, table, "table", vocab * hidden, 2), vocab, hidden,
                             _sized(None, tokens, "tokens", n, 4), n, _sized(None, h_out, "h_out", n * hidden, 4),
                             _stream(stream)))


def ms_add_rmsnorm(h, delta, weight, eps: float, out, stream=None) -> None:
    n, hidden = h.shape
    _check(lib.ms_add_rmsnorm(_sized(None, h, "h", n * hidden, 4), _sized(None, delta, "delta", n * hidden, 2),
                              _sized(None, weight, "weight", hidden, 2), float(eps),
                              _sized(None, out, "out", n * hidden, 2), n, hidden, _stream(stream)))


def ms_swiglu(gate_up, out, stream=None) -> None:
    n, two_i = gate_up.shape
    inter = two_i // 2
    _check(lib.ms_swiglu(_sized(None, gate_up, "gate_up", n * 2 * inter, 2), _sized(None, out, "out", n * inter, 2),
                         n, inter, _stream(stream)))


def ms_argmax_rows(logits, vocab: int, out, stream=None) -> None:
    n, ld = logits.shape
    _check(lib.ms_argmax_rows(_sized(None, logits, "logits", n * ld, 2), n, vocab, ld,
                              _sized(None, out, "out", n, 4), _stream(stream)))


def ms_gemm_workspace_bytes(M: int, N: int, K: int, split_k: int) -> int:
    return lib.ms_gemm_workspace_bytes(M, N, K, split_k)


def ms_gemm_bf16(a, w, bias, outs, split_k: int = 1, workspace=None, stream=None) -> None:
    """outs: list of [M, n_i] bf16 tensors that take consecutive column ranges of the product."""
    M_, K = a.shape
    N = w.shape[0]
    cols = [0]
    for o in outs:
        cols.append(cols[-1] + o.shape[1])
    ptrs = (_P * len(outs))(*[_sized(None, o, "out", M_ * o.shape[1], 2) for o in outs])
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    if w.shape[1] != K or cols[-1] != N:
        raise MsError(MS_ERR_INVALID, "ms_gemm_bf16: shapes do not match")
    _check(lib.ms_gemm_bf16(_sized(None, a, "a", M_ * K, 2), _sized(None, w, "w", N * K, 2), _sized(None, bias, "bias", N, 2),
                            M_, N, K, len(outs), ptrs, _ints(cols), split_k, _dev(workspace), ws_bytes, _stream(stream)))


def ms_gemm_swiglu_bf16(a, w_gate_up, out, workspace=None, stream=None) -> None:
    """out[M, inter] = silu(a . Wg^T) * (a . Wu^T); w_gate_up [2 * inter, K] with gate and up rows
    interleaved in blocks of 32 (see interleave_gate_up)."""
    M_, K = a.shape
    inter = out.shape[1]
    if w_gate_up.shape[0] != 2 * inter or w_gate_up.shape[1] != K or out.shape[0] != M_:
        raise MsError(MS_ERR_INVALID, "ms_gemm_swiglu_bf16: shapes do not match")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.ms_gemm_swiglu_bf16(_sized(None, a, "a", M_ * K, 2), _sized(None, w_gate_up, "w_gate_up", 2 * inter * K, 2), M_, inter, K,
                                   _sized(None, out, "out", M_ * inter, 2), _dev(workspace), ws_bytes, _stream(stream)))


def ms_gemm_add_rmsnorm_workspace_bytes(M: int, N: int, K: int, split_k: int) -> int:
    return lib.ms_gemm_add_rmsnorm_workspace_bytes(M, N, K, split_k)


def ms_gemm_add_rmsnorm_bf16(a, w, h, norm_weight, eps: float, out, split_k: int = 1, workspace=None, stream=None) -> None:
    """h[M, N] (fp32, in place) += bf16(a . w^T); out = rmsnorm(h) * norm_weight (bf16)."""
    M_, K = a.shape
    N = w.shape[0]
    if w.shape[1] != K or tuple(h.shape) != (M_, N) or tuple(out.shape) != (M_, N) or norm_weight.numel() != N:
        raise MsError(MS_ERR_INVALID, "ms_gemm_add_rmsnorm_bf16: shapes do not match")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.ms_gemm_add_rmsnorm_bf16(_sized(None, a, "a", M_ * K, 2), _sized(None, w, "w", N * K, 2), M_, N, K, split_k,
                                        _sized(None, h, "h", M_ * N, 4), _sized(None, norm_weight, "norm_weight", N, 2), eps,
                                        _sized(None, out, "out", M_ * N, 2), _dev(workspace), ws_bytes, _stream(stream)))


def ms_lm_head_argmax_workspace_bytes(M: int, vocab: int, K: int) -> int:
    return lib.ms_lm_head_argmax_workspace_bytes(M, vocab, K)


def ms_lm_head_argmax_bf16(a, w, out, workspace, stream=None) -> None:
    """out[m] (int32) = greedy token of row m: argmax of a[m] . w[n] over n on the fp32 sums."""
    M_, K = a.shape
    vocab = w.shape[0]
    if w.shape[1] != K:
        raise MsError(MS_ERR_INVALID, "ms_lm_head_argmax_bf16: shapes do not match")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.ms_lm_head_argmax_bf16(_sized(None, a, "a", M_ * K, 2), _sized(None, w, "w", vocab * K, 2), M_, vocab, K,
                                      _sized(None, out, "out", M_, 4), _dev(workspace), ws_bytes, _stream(stream)))


def interleave_gate_up(w_gate, w_up):
    """The weight layout ms_gemm_swiglu_bf16 reads: blocks of 32 gate rows followed by the 32 up rows
    of the same outputs.  A one-off re-ordering of rows at load time (no arithmetic)."""
    inter, K = w_gate.shape
    if inter % 32 or w_up.shape != w_gate.shape:
        raise MsError(MS_ERR_INVALID, "interleave_gate_up: widths must match and be multiples of 32")
    return torch.stack([w_gate.view(inter // 32, 32, K), w_up.view(inter // 32, 32, K)], dim=1).reshape(2 * inter, K).contiguous()


def ms_attention_set_deterministic(cache, on: bool) -> None:
    _check(lib.ms_attention_set_deterministic(cache, 1 if on else 0))


def ms_attention_fault_injection(cache, poll_limit: int, published_bias: int, stream=None) -> None:
    _check(lib.ms_attention_fault_injection(cache, poll_limit, published_bias, _stream(stream)))


def ms_accept(B, n, draft, target, stop_ids, accept_len, next_token, stream=None) -> None:
    n_stop = 0 if stop_ids is None else stop_ids.numel()
    _check(lib.ms_accept(B, n, _sized(None, draft, "draft", B * n, 4), _sized(None, target, "target", B * n, 4),
                         _sized(None, stop_ids, "stop_ids", n_stop, 4), n_stop, _sized(None, accept_len, "accept_len", B, 4),
                         _sized(None, next_token, "next_token", B, 4), _stream(stream)))


def ms_seq_len(cache, seq_id: int) -> int:
    n = C.c_int(0)
    _check(lib.ms_seq_len(cache, seq_id, C.byref(n)))
    return n.value


def ms_seq_page_table(cache, seq_id: int):
    n = C.c_int(0)
    _check(lib.ms_seq_page_table(cache, seq_id, None, 0, C.byref(n)))
    buf = (C.c_int * max(1, n.value))()
    _check(lib.ms_seq_page_table(cache, seq_id, buf, n.value, C.byref(n)))
    return list(buf[:n.value])


def ms_free_page_count(cache) -> int:
    n = C.c_int(0)
    _check(lib.ms_free_page_count(cache, C.byref(n)))
    return n.value


def ms_peak_pages(cache) -> int:
    n = C.c_int(0)
    _check(lib.ms_peak_pages(cache, C.byref(n)))
    return n.value


def ms_launch_count(cache) -> int:
    n = C.c_longlong(0)
    _check(lib.ms_launch_count(cache, C.byref(n)))
    return n.value


def ms_check_integrity(cache, stream=None) -> None:
    _check(lib.ms_check_integrity(cache, _stream(stream)))


def ms_profile_attention(cache, capacity: int, stride: int = 1, span: int = 1) -> None:
    _check(lib.ms_profile_attention(cache, capacity, stride, span))


def ms_profile_read(cache, cap: int):
    buf = (C.c_float * max(1, cap))()
    n = C.c_int(0)
    _check(lib.ms_profile_read(cache, buf, cap, C.byref(n)))
    return list(buf[:min(n.value, cap)])


def ms_hbm_read_probe(src, non_temporal: bool, sink, stream=None):
    """Plain streaming read of the tensor `src` (device, contiguous); `sink`: device tensor of >= 8192 bytes.
    Returns the bytes read (the tensor's size rounded down to a multiple of 32 KiB)."""
    n = C.c_size_t(0)
    _check(lib.ms_hbm_read_probe(_dev(src), src.numel() * src.element_size(), 1 if non_temporal else 0, _dev(sink), _stream(stream), C.byref(n)))
    return n.value


def ms_ama_count(n_tokens: int, c: int) -> int:
    return lib.ms_ama_count(n_tokens, c)


def ms_upl_positions(first_pid: int, n_tokens: int, c: int):
    n = lib.ms_upl_positions(first_pid, n_tokens, c, None, 0)
    if n < 0:
        raise MsError(n, "bad arguments")
    buf = (C.c_int * max(1, n))()
    lib.ms_upl_positions(first_pid, n_tokens, c, buf, n)
    return list(buf[:n])


def ms_output_token_pid(last_pid: int) -> int:
    return lib.ms_output_token_pid(last_pid)


def ms_foresight_pids(last_prefix_pid: int, d: int):
    buf = (C.c_int * max(1, d))()
    n = lib.ms_foresight_pids(last_prefix_pid, d, buf, d)
    if n < 0:
        raise MsError(n, "bad arguments")
    return list(buf[:n])


def ms_default_ctx_new(n_verify: int, n_foresight: int):
    n = n_verify + n_foresight
    buf = (C.c_int * max(1, n))()
    r = lib.ms_default_ctx_new(n_verify, n_foresight, buf, n)
    if r < 0:
        raise MsError(r, "bad arguments")
    return list(buf[:n])


def ms_per_position_layout(first_pid: int, n_verify: int, d: int):
    n = lib.ms_per_position_layout(first_pid, n_verify, d, None, None, 0)
    if n < 0:
        raise MsError(n, "bad arguments")
    pos, ctx = (C.c_int * max(1, n))(), (C.c_int * max(1, n))()
    lib.ms_per_position_layout(first_pid, n_verify, d, pos, ctx, n)
    return list(pos[:n]), list(ctx[:n])


def ms_consecutive_memory_positions(last_pid: int, n_mem: int):
    buf = (C.c_int * max(1, n_mem))()
    n = lib.ms_consecutive_memory_positions(last_pid, n_mem, buf, max(0, n_mem))
    if n < 0:
        raise MsError(n, "bad arguments")
    return list(buf[:n])


def ms_upl_positions_fixed(first_pid: int, n_tokens: int, n_mem: int):
    buf = (C.c_int * max(1, n_mem))()
    n = lib.ms_upl_positions_fixed(first_pid, n_tokens, n_mem, buf, max(0, n_mem))
    if n < 0:
        raise MsError(n, "bad arguments")
    return list(buf[:n])


def ms_step_positions(first_pid, n_verify: int, n_foresight: int, out=None):
    """first_pid: int32 numpy array [B]; out: int32 numpy array [B, n_q] (e.g. a view of pinned
    memory), allocated when omitted.  Returns out."""
    first = np.ascontiguousarray(first_pid, dtype=np.int32)
    B, n_q = first.shape[0], n_verify + n_foresight
    if out is None:
        out = np.empty((B, n_q), dtype=np.int32)
    if out.dtype != np.int32 or out.size < B * n_q or not out.flags["C_CONTIGUOUS"]:
        raise MsError(MS_ERR_INVALID, "ms_step_positions: out must be a contiguous int32 array of B * n_q entries")
    r = lib.ms_step_positions(B, first.ctypes.data_as(_IP), n_verify, n_foresight, out.ctypes.data_as(_IP))
    if r < 0:
        raise MsError(r, "bad arguments")
    return out
