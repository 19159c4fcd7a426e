"""Thin ctypes binding over the C ABI in include/sv.h.

Argument marshalling only: every step of the path runs in the HIP kernels of
libsv.so.  PyTorch provides device memory and the stream.  There is no CPU
fallback: if the library has not been built, importing this module fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsv.so")

SV_F32, SV_BF16 = 0, 1
SV_BATCH_GREEDY, SV_PER_SEQUENCE = 0, 1
SV_OK = 0
SV_ERR_INVALID_ARG, SV_ERR_NULL, SV_ERR_DTYPE, SV_ERR_ALIGN = -1, -2, -3, -4
SV_ERR_WORKSPACE, SV_ERR_LAUNCH, SV_ERR_TOO_LARGE = -5, -6, -7
FLAG_BAD_ROW, FLAG_NEAR_TIE, FLAG_RESIDUAL_FALLBACK, FLAG_NEAR_CDF_EDGE, FLAG_BAD_TOKEN = 1, 2, 4, 8, 16
FLAG_NOT_COMPACT = 32
FLAG_NO_CHAIN = 64
SV_SUPPORT_MAX_CAP = 1024
SV_SELECT_MAX_KEYS = 8192
SV_MAX_K = 64

EXPORTS = ("sv_strerror", "sv_workspace_bytes", "sv_row_stats", "sv_accept_estimate",
           "sv_select_length", "sv_verify_sample", "sv_set_timing_events", "sv_accept_ratio",
           "sv_quantile_edges", "sv_profile_accumulate", "sv_profile_finalize", "sv_warp_cutoffs",
           "sv_row_stats_warped", "sv_verify_sample_warped",
           "sv_warp_compact", "sv_row_stats_sparse", "sv_verify_sample_sparse", "sv_uniforms",
           "sv_accept_ratio_sparse", "sv_verify_sample_static", "sv_accept_ratio_warped",
           "sv_warp_cutoffs_multi", "sv_warp_compact_multi", "sv_verify_sample_chained",
           "sv_verify_sample_warped_chained", "sv_estimate_select", "sv_repetition_penalty",
           "sv_repetition_penalty_multi")
SV_WARP_MAX_TENSORS = 8
SV_STATIC_SCRATCH_BYTES = 1 << 20
(SV_KERNEL_ROW_STATS, SV_KERNEL_ACCEPT_ESTIMATE, SV_KERNEL_SELECT_LENGTH, SV_KERNEL_VERIFY_ROWS,
 SV_KERNEL_VERIFY_MASS, SV_KERNEL_VERIFY_PICK, SV_KERNEL_COUNT) = range(7)

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python paper_2509_24328_amd/build.py` "
                      "(or __graft_entry__.build()); there is no fallback path")

lib = ctypes.CDLL(LIB_PATH)
_vp, _i, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
lib.sv_strerror.restype = ctypes.c_char_p
lib.sv_strerror.argtypes = [_i]
lib.sv_workspace_bytes.restype = _sz
lib.sv_workspace_bytes.argtypes = [_i, _i, _i, _i]
lib.sv_row_stats.restype = _i
lib.sv_row_stats.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz,
                             _vp]
lib.sv_accept_estimate.restype = _i
lib.sv_accept_estimate.argtypes = [_vp, _vp, _i, _vp, _i, _vp, _i, _vp, _vp, _vp, _vp]
lib.sv_select_length.restype = _i
lib.sv_select_length.argtypes = [_vp, _i, _i, _vp, _i, _i, _vp, _vp, _vp, _vp]
lib.sv_repetition_penalty.restype = _i
lib.sv_repetition_penalty.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _vp, _i, _vp, _i, ctypes.c_float, _vp]
lib.sv_repetition_penalty_multi.restype = _i
lib.sv_repetition_penalty_multi.argtypes = [_i, _vp, _vp, _vp, _i, _vp, _i, _i, _vp, _i, _vp, _i, ctypes.c_float, _vp]
lib.sv_estimate_select.restype = _i
lib.sv_estimate_select.argtypes = [_vp, _vp, _i, _i, _vp, _i, _vp, _i, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]
lib.sv_verify_sample.restype = _i
lib.sv_verify_sample.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_uint64,
                                 ctypes.c_uint32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
lib.sv_verify_sample_chained.restype = _i
lib.sv_verify_sample_chained.argtypes = lib.sv_verify_sample.argtypes
lib.sv_verify_sample_static.restype = _i
lib.sv_verify_sample_static.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, ctypes.c_uint64,
                                        ctypes.c_uint32, _vp, _vp, _vp, _vp, _vp]
lib.sv_accept_ratio.restype = _i
lib.sv_accept_ratio.argtypes = [_vp, _i, _vp, _vp, _i, _i, _i, _i, _vp, _vp, _vp, _sz, _vp]
lib.sv_accept_ratio_warped.restype = _i
lib.sv_accept_ratio_warped.argtypes = [_vp, _i, _vp, _vp, _i, _i, _i, _i, ctypes.c_float, _vp, ctypes.c_float, _vp,
                                       _vp, _vp, _vp, _sz, _vp]
lib.sv_quantile_edges.restype = _i
lib.sv_quantile_edges.argtypes = [_vp, _i, _i, ctypes.c_float, ctypes.c_float, _vp, _vp]
lib.sv_profile_accumulate.restype = _i
lib.sv_profile_accumulate.argtypes = [_vp, _vp, _vp, _i, _vp, _i, _vp, _i, _i, _vp, _vp, _vp]
lib.sv_profile_finalize.restype = _i
lib.sv_profile_finalize.argtypes = [_vp, _vp, _i, _i, _i, _vp, _vp, _vp]
lib.sv_warp_cutoffs.restype = _i
lib.sv_warp_cutoffs.argtypes = [_vp, _i, _i, _i, ctypes.c_float, _i, ctypes.c_float, _vp, _vp, _vp]
_f = ctypes.c_float
lib.sv_warp_cutoffs_multi.restype = _i
lib.sv_warp_cutoffs_multi.argtypes = [_i, _vp, _vp, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp]
lib.sv_warp_compact_multi.restype = _i
lib.sv_warp_compact_multi.argtypes = [_i, _vp, _vp, _i, _i, _vp, _vp, _vp, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.sv_row_stats_warped.restype = _i
lib.sv_row_stats_warped.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _f, _vp, _f, _vp,
                                    _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
lib.sv_verify_sample_warped.restype = _i
lib.sv_verify_sample_warped.argtypes = [_vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i, _f, _vp, _f, _vp,
                                        ctypes.c_uint64, ctypes.c_uint32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
lib.sv_verify_sample_warped_chained.restype = _i
lib.sv_verify_sample_warped_chained.argtypes = lib.sv_verify_sample_warped.argtypes
lib.sv_warp_compact.restype = _i
lib.sv_warp_compact.argtypes = [_vp, _i, _i, _i, _f, _i, _f, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.sv_row_stats_sparse.restype = _i
lib.sv_row_stats_sparse.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i, _vp, _i, _i, _i,
                                    _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.sv_verify_sample_sparse.restype = _i
lib.sv_verify_sample_sparse.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _vp, _vp, _i, _i, _i,
                                        ctypes.c_uint64, ctypes.c_uint32, _vp, _vp, _vp, _vp, _vp]
lib.sv_accept_ratio_sparse.restype = _i
lib.sv_accept_ratio_sparse.argtypes = [_vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _vp, _i, _i, _i, _vp, _vp, _vp]
lib.sv_uniforms.restype = _i
lib.sv_uniforms.argtypes = [ctypes.c_uint64, ctypes.c_uint32, _i, _i, _vp, _vp, _vp]
lib.sv_set_timing_events.restype = _i
lib.sv_set_timing_events.argtypes = [_i, _vp, _vp]


class SvError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(lib.sv_strerror(status).decode())


def _check(status):
    if status != SV_OK:
        raise SvError(status)


def _ptr(t):
    """Device address of a tensor (None -> NULL).  The C ABI takes plain pointers to
    dense row-major device memory, so anything else is refused here instead of being
    read as if it were."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("sv: tensors must be contiguous device tensors "
                         f"(got device={t.device}, contiguous={t.is_contiguous()})")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_tag(t):
    if t.dtype == torch.float32:
        return SV_F32
    if t.dtype == torch.bfloat16:
        return SV_BF16
    raise SvError(SV_ERR_DTYPE)


def sv_strerror(status):
    return lib.sv_strerror(status).decode()


def sv_workspace_bytes(B, k, V, dtype):
    return int(lib.sv_workspace_bytes(B, k, V, dtype))


def alloc_workspace(B, k, V, dtype, device="cuda"):
    n = max(sv_workspace_bytes(B, k, V, dtype), 256)
    return torch.empty(n, dtype=torch.uint8, device=device)


def sv_row_stats(z_d, z_c, x, lse_d, lse_c, S, A, kl=None, flags=None, ws=None, stream=None,
                 entropy_d=None, pd_x=None):
    B, k, V = z_d.shape
    _check(lib.sv_row_stats(_ptr(z_d), _ptr(z_c), _ptr(x), B, k, V, _dtype_tag(z_d),
                            _ptr(lse_d), _ptr(lse_c), _ptr(S), _ptr(A), _ptr(kl), _ptr(entropy_d),
                            _ptr(pd_x), _ptr(flags), _ptr(ws), 0 if ws is None else ws.numel(),
                            _stream(stream)))


def sv_accept_estimate(S, A, edges_s, edges_a, table, p_hat, edge_flag=None, stream=None):
    _check(lib.sv_accept_estimate(_ptr(S), _ptr(A), S.numel(), _ptr(edges_s), edges_s.numel() - 1,
                                  _ptr(edges_a), edges_a.numel() - 1, _ptr(table), _ptr(p_hat),
                                  _ptr(edge_flag), _stream(stream)))


def sv_select_length(p_hat, latency, mode, gamma, t_offsets, total_M, stream=None):
    B, k = p_hat.shape
    _check(lib.sv_select_length(_ptr(p_hat), B, k, _ptr(latency), latency.numel(), mode,
                                _ptr(gamma), _ptr(t_offsets), _ptr(total_M), _stream(stream)))


def sv_estimate_select(S, A, edges_s, edges_a, table, latency, mode, p_hat, gamma, t_offsets, total_M,
                       edge_flag=None, stream=None):
    B, k = S.shape
    _check(lib.sv_estimate_select(_ptr(S), _ptr(A), B, k, _ptr(edges_s), edges_s.numel() - 1, _ptr(edges_a),
                                  edges_a.numel() - 1, _ptr(table), _ptr(latency), latency.numel(), mode,
                                  _ptr(p_hat), _ptr(edge_flag), _ptr(gamma), _ptr(t_offsets), _ptr(total_M),
                                  _stream(stream)))


def sv_verify_sample(z_t, t_offsets, z_d, x, gamma, seed, step, out_tokens, n_accept, flags,
                     ratio=None, ws=None, stream=None):
    B, k, V = z_d.shape
    n_t_rows = z_t.shape[0] if t_offsets is not None else 0
    _check(lib.sv_verify_sample(_ptr(z_t), _ptr(t_offsets), n_t_rows, _ptr(z_d), _ptr(x), _ptr(gamma),
                                B, k, V, _dtype_tag(z_d), seed, step, _ptr(out_tokens), _ptr(n_accept),
                                _ptr(flags), _ptr(ratio), _ptr(ws), 0 if ws is None else ws.numel(),
                                _stream(stream)))


def sv_verify_sample_chained(z_t, t_offsets, z_d, x, gamma, seed, step, out_tokens, n_accept, flags,
                             ratio=None, ws=None, stream=None):
    B, k, V = z_d.shape
    n_t_rows = z_t.shape[0] if t_offsets is not None else 0
    _check(lib.sv_verify_sample_chained(_ptr(z_t), _ptr(t_offsets), n_t_rows, _ptr(z_d), _ptr(x), _ptr(gamma),
                                        B, k, V, _dtype_tag(z_d), seed, step, _ptr(out_tokens),
                                        _ptr(n_accept), _ptr(flags), _ptr(ratio), _ptr(ws),
                                        0 if ws is None else ws.numel(), _stream(stream)))


def sv_verify_sample_static(z_t, t_offsets, z_d, x, gamma, seed, step, out_tokens, n_accept, flags,
                            ratio=None, stream=None):
    B, k, V = z_d.shape
    n_t_rows = z_t.shape[0] if t_offsets is not None else 0
    _check(lib.sv_verify_sample_static(_ptr(z_t), _ptr(t_offsets), n_t_rows, _ptr(z_d), _ptr(x), _ptr(gamma),
                                       B, k, V, _dtype_tag(z_d), seed, step, _ptr(out_tokens), _ptr(n_accept),
                                       _ptr(flags), _ptr(ratio), _stream(stream)))


def sv_set_timing_events(kernel, start_event, stop_event):
    """start_event / stop_event: raw hipEvent_t handles (ints / c_void_p) or None."""
    _check(lib.sv_set_timing_events(kernel, start_event, stop_event))


def sv_accept_ratio(z_t, z_d, x, ratio, flags=None, ws=None, stream=None):
    B, k, V = z_d.shape
    _check(lib.sv_accept_ratio(_ptr(z_t), z_t.shape[1], _ptr(z_d), _ptr(x), B, k, V, _dtype_tag(z_d),
                               _ptr(ratio), _ptr(flags), _ptr(ws), 0 if ws is None else ws.numel(),
                               _stream(stream)))


def sv_accept_ratio_warped(z_t, z_d, x, temperature_t, cutoff_t, temperature_d, cutoff_d, ratio, flags=None,
                           ws=None, stream=None):
    B, k, V = z_d.shape
    _check(lib.sv_accept_ratio_warped(_ptr(z_t), z_t.shape[1], _ptr(z_d), _ptr(x), B, k, V, _dtype_tag(z_d),
                                      temperature_t, _ptr(cutoff_t), temperature_d, _ptr(cutoff_d),
                                      _ptr(ratio), _ptr(flags), _ptr(ws), 0 if ws is None else ws.numel(),
                                      _stream(stream)))


def sv_quantile_edges(values, n_bins, lo, hi, edges, stream=None):
    _check(lib.sv_quantile_edges(_ptr(values), values.numel(), n_bins, lo, hi, _ptr(edges), _stream(stream)))


def sv_profile_accumulate(S, A, ratio, edges_s, edges_a, n_x, counts, sum_x, stream=None):
    _check(lib.sv_profile_accumulate(_ptr(S), _ptr(A), _ptr(ratio), S.numel(), _ptr(edges_s),
                                     edges_s.numel() - 1, _ptr(edges_a), edges_a.numel() - 1, n_x,
                                     _ptr(counts), _ptr(sum_x), _stream(stream)))


def sv_profile_finalize(counts, sum_x, table, info, stream=None):
    n_s, n_a, n_x = counts.shape
    _check(lib.sv_profile_finalize(_ptr(counts), _ptr(sum_x), n_s, n_a, n_x, _ptr(table), _ptr(info),
                                   _stream(stream)))


def sv_warp_cutoffs(z, temperature, top_k, top_p, cutoff, flags=None, stream=None):
    V = z.shape[-1]
    rows = z.numel() // V
    _check(lib.sv_warp_cutoffs(_ptr(z), rows, V, _dtype_tag(z), temperature, top_k, top_p, _ptr(cutoff),
                               _ptr(flags), _stream(stream)))


def _host_ptrs(tensors):
    """Host array of the device addresses of `tensors` (None entries -> NULL)."""
    return (ctypes.c_void_p * len(tensors))(*[None if t is None else _ptr(t).value for t in tensors])


def _warp_lists(zs, temperature, top_k, top_p):
    n = len(zs)
    V = zs[0].shape[-1]
    tag = _dtype_tag(zs[0])
    if any(z.shape[-1] != V or _dtype_tag(z) != tag for z in zs):
        raise SvError(SV_ERR_INVALID_ARG)
    as_list = lambda v: list(v) if isinstance(v, (list, tuple)) else [v] * n
    rows = (ctypes.c_int * n)(*[z.numel() // V for z in zs])
    T = (ctypes.c_float * n)(*as_list(temperature))
    K = (ctypes.c_int * n)(*as_list(top_k))
    Pp = (ctypes.c_float * n)(*as_list(top_p))
    return n, V, tag, rows, T, K, Pp


def sv_warp_cutoffs_multi(zs, temperature, top_k, top_p, cutoffs, flags=None, stream=None):
    """zs, cutoffs (, flags): lists of tensors; temperature / top_k / top_p: one value or a list."""
    n, V, tag, rows, T, K, Pp = _warp_lists(zs, temperature, top_k, top_p)
    _check(lib.sv_warp_cutoffs_multi(n, _host_ptrs(zs), rows, V, tag, T, K, Pp, _host_ptrs(cutoffs),
                                     None if flags is None else _host_ptrs(flags), _stream(stream)))


def sv_warp_compact_multi(zs, temperature, top_k, top_p, sups, cutoffs=None, flags=None, stream=None):
    n, V, tag, rows, T, K, Pp = _warp_lists(zs, temperature, top_k, top_p)
    if any(s.cap != sups[0].cap or s.rows != z.numel() // V for s, z in zip(sups, zs)):
        raise SvError(SV_ERR_INVALID_ARG)
    _check(lib.sv_warp_compact_multi(n, _host_ptrs(zs), rows, V, tag, T, K, Pp, sups[0].cap,
                                     _host_ptrs([s.count for s in sups]), _host_ptrs([s.token for s in sups]),
                                     _host_ptrs([s.prob for s in sups]), _host_ptrs([s.lse for s in sups]),
                                     None if cutoffs is None else _host_ptrs(cutoffs),
                                     None if flags is None else _host_ptrs(flags), _stream(stream)))


def sv_row_stats_warped(z_d, z_c, x, temperature_d, cutoff_d, temperature_c, cutoff_c, lse_d, lse_c, S, A,
                        kl=None, flags=None, ws=None, stream=None, entropy_d=None, pd_x=None):
    B, k, V = z_d.shape
    _check(lib.sv_row_stats_warped(_ptr(z_d), _ptr(z_c), _ptr(x), B, k, V, _dtype_tag(z_d),
                                   temperature_d, _ptr(cutoff_d), temperature_c, _ptr(cutoff_c),
                                   _ptr(lse_d), _ptr(lse_c), _ptr(S), _ptr(A), _ptr(kl), _ptr(entropy_d),
                                   _ptr(pd_x), _ptr(flags), _ptr(ws), 0 if ws is None else ws.numel(),
                                   _stream(stream)))


def sv_verify_sample_warped(z_t, t_offsets, z_d, x, gamma, temperature_t, cutoff_t, temperature_d, cutoff_d,
                            seed, step, out_tokens, n_accept, flags, ratio=None, ws=None, stream=None):
    B, k, V = z_d.shape
    n_t_rows = z_t.shape[0] if t_offsets is not None else 0
    _check(lib.sv_verify_sample_warped(_ptr(z_t), _ptr(t_offsets), n_t_rows, _ptr(z_d), _ptr(x), _ptr(gamma),
                                       B, k, V, _dtype_tag(z_d), temperature_t, _ptr(cutoff_t),
                                       temperature_d, _ptr(cutoff_d), seed, step, _ptr(out_tokens),
                                       _ptr(n_accept), _ptr(flags), _ptr(ratio), _ptr(ws),
                                       0 if ws is None else ws.numel(), _stream(stream)))


def sv_verify_sample_warped_chained(z_t, t_offsets, z_d, x, gamma, temperature_t, cutoff_t, temperature_d,
                                    cutoff_d, seed, step, out_tokens, n_accept, flags, ratio=None, ws=None,
                                    stream=None):
    B, k, V = z_d.shape
    n_t_rows = z_t.shape[0] if t_offsets is not None else 0
    _check(lib.sv_verify_sample_warped_chained(_ptr(z_t), _ptr(t_offsets), n_t_rows, _ptr(z_d), _ptr(x),
                                               _ptr(gamma), B, k, V, _dtype_tag(z_d), temperature_t,
                                               _ptr(cutoff_t), temperature_d, _ptr(cutoff_d), seed, step,
                                               _ptr(out_tokens), _ptr(n_accept), _ptr(flags), _ptr(ratio),
                                               _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)))


def sv_repetition_penalty(z, history, penalty, x=None, row_offsets=None, B=None, rows_per_seq=None, stream=None):
    """In place.  z: dense [B, R, V]; or packed [n_rows, V] with row_offsets [B+1], B and rows_per_seq given."""
    if row_offsets is None:
        B, rows_per_seq, V = z.shape
        n_rows = 0
    else:
        n_rows, V = z.shape
    n_hist = 0 if history is None else history.shape[1]
    k = 0 if x is None else x.shape[1]
    _check(lib.sv_repetition_penalty(_ptr(z), _ptr(row_offsets), n_rows, B, rows_per_seq, V, _dtype_tag(z),
                                     _ptr(history), n_hist, _ptr(x), k, penalty, _stream(stream)))


def sv_repetition_penalty_multi(zs, history, penalty, x=None, row_offsets=None, B=None, rows_per_seq=None,
                                stream=None):
    """In place, several tensors of one batch in one launch.  zs: dense [B, R_t, V] tensors; a packed one
    ([n_rows, V]) needs its entry of row_offsets ([B+1]) and of rows_per_seq set, and B given."""
    n = len(zs)
    offs = [None] * n if row_offsets is None else list(row_offsets)
    rps = [None] * n if rows_per_seq is None else list(rows_per_seq)
    n_rows = []
    for t, z in enumerate(zs):
        if offs[t] is None:
            B, rps[t] = z.shape[0], z.shape[1]
            n_rows.append(0)
        else:
            n_rows.append(z.shape[0])
    V = zs[0].shape[-1]
    tag = _dtype_tag(zs[0])
    if any(z.shape[-1] != V or _dtype_tag(z) != tag for z in zs):
        raise SvError(SV_ERR_INVALID_ARG)
    n_hist = 0 if history is None else history.shape[1]
    k = 0 if x is None else x.shape[1]
    _check(lib.sv_repetition_penalty_multi(n, _host_ptrs(zs), _host_ptrs(offs), (ctypes.c_int * n)(*n_rows), B,
                                           (ctypes.c_int * n)(*rps), V, tag, _ptr(history), n_hist, _ptr(x), k,
                                           penalty, _stream(stream)))


class Supports:
    """Device buffers for the compacted supports of `rows` logit rows (sv_warp_compact)."""

    def __init__(self, rows, cap, device="cuda"):
        self.rows, self.cap = rows, cap
        self.count = torch.empty(rows, dtype=torch.int32, device=device)
        self.token = torch.empty((rows, cap), dtype=torch.int32, device=device)
        self.prob = torch.empty((rows, cap), dtype=torch.float64, device=device)
        self.lse = torch.empty(rows, dtype=torch.float32, device=device)


def sv_warp_compact(z, temperature, top_k, top_p, sup, cutoff=None, flags=None, stream=None):
    V = z.shape[-1]
    rows = z.numel() // V
    if rows != sup.rows:
        raise SvError(SV_ERR_INVALID_ARG)
    _check(lib.sv_warp_compact(_ptr(z), rows, V, _dtype_tag(z), temperature, top_k, top_p, sup.cap,
                               _ptr(sup.count), _ptr(sup.token), _ptr(sup.prob), _ptr(sup.lse), _ptr(cutoff),
                               _ptr(flags), _stream(stream)))


def sv_row_stats_sparse(sup_d, sup_c, x, V, lse_d, lse_c, S, A, kl=None, flags=None, stream=None,
                        entropy_d=None, pd_x=None):
    B, k = x.shape
    if sup_d.cap != sup_c.cap or sup_d.rows != B * k or sup_c.rows != B * k:
        raise SvError(SV_ERR_INVALID_ARG)
    _check(lib.sv_row_stats_sparse(_ptr(sup_d.count), _ptr(sup_d.token), _ptr(sup_d.prob), _ptr(sup_d.lse),
                                   _ptr(sup_c.count), _ptr(sup_c.token), _ptr(sup_c.prob), _ptr(sup_c.lse),
                                   sup_d.cap, _ptr(x), B, k, V, _ptr(lse_d), _ptr(lse_c), _ptr(S), _ptr(A),
                                   _ptr(kl), _ptr(entropy_d), _ptr(pd_x), _ptr(flags), _stream(stream)))


def sv_verify_sample_sparse(sup_t, t_offsets, sup_d, x, gamma, V, seed, step, out_tokens, n_accept, flags,
                            ratio=None, stream=None):
    B, k = x.shape
    if sup_t.cap != sup_d.cap or sup_d.rows != B * k or (t_offsets is None and sup_t.rows != B * (k + 1)):
        raise SvError(SV_ERR_INVALID_ARG)
    n_t_rows = sup_t.rows if t_offsets is not None else 0
    _check(lib.sv_verify_sample_sparse(_ptr(sup_t.count), _ptr(sup_t.token), _ptr(sup_t.prob), _ptr(t_offsets),
                                       n_t_rows, _ptr(sup_d.count), _ptr(sup_d.token), _ptr(sup_d.prob),
                                       sup_t.cap, _ptr(x), _ptr(gamma), B, k, V, seed, step, _ptr(out_tokens),
                                       _ptr(n_accept), _ptr(flags), _ptr(ratio), _stream(stream)))


def sv_uniforms(seed, step, u_accept, u_sample, stream=None):
    B, n_pos = u_accept.shape
    _check(lib.sv_uniforms(seed, step, B, n_pos, _ptr(u_accept), _ptr(u_sample), _stream(stream)))


def sv_accept_ratio_sparse(sup_t, sup_d, x, V, ratio, flags=None, stream=None):
    B, k = x.shape
    if sup_t.cap != sup_d.cap or sup_d.rows != B * k or sup_t.rows % B != 0 or sup_t.rows // B not in (k, k + 1):
        raise SvError(SV_ERR_INVALID_ARG)
    _check(lib.sv_accept_ratio_sparse(_ptr(sup_t.count), _ptr(sup_t.token), _ptr(sup_t.prob), sup_t.rows // B,
                                      _ptr(sup_d.count), _ptr(sup_d.token), _ptr(sup_d.prob), sup_t.cap, _ptr(x),
                                      B, k, V, _ptr(ratio), _ptr(flags), _stream(stream)))
