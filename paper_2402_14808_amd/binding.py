"""ctypes binding of librelayattn.so: argument marshalling only.

Every function mirrors one entry point of include/relay_attn.h and takes torch tensors
(device memory) where the C signature takes device pointers.  No arithmetic of the method
happens here; there is no fallback when the library is missing.
"""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librelayattn.so")

RA_OK = 0
RA_ERR_INVALID_ARG = 1
RA_ERR_UNSUPPORTED = 2
RA_ERR_WORKSPACE_TOO_SMALL = 3
RA_ERR_HIP = 4

EXPORTED = ("relay_attn_workspace_bytes", "relay_attn_decode_plan", "relay_attn_decode",
            "relay_attn_decode_append", "relay_attn_decode_multi", "relay_attn_system_fill",
            "relay_attn_system_cache_layout",
            "relay_attn_prefill", "paged_attn_decode_naive", "relay_attn_cache_append",
            "relay_attn_debug_validate", "relay_attn_debug_decode_phases", "relay_attn_debug_timeline",
            "relay_attn_decode_static", "relay_attn_static_scratch_bytes",
            "relay_attn_decode_grouped", "relay_attn_group_requests", "relay_attn_prefill_multi",
            "relay_attn_debug_stream_probe", "relay_attn_debug_launch_probe",
            "relay_attn_status_string", "relay_attn_abi_version")


class RAParams(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
        ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("sys_len", ctypes.c_int32), ("block_size", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("max_context_len", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
        ("q_stride_token", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("o_stride_token", ctypes.c_int64), ("o_stride_head", ctypes.c_int64),
        ("sys_stride_token", ctypes.c_int64), ("sys_stride_head", ctypes.c_int64),
        ("out_is_fp32", ctypes.c_int32), ("sys_chunk_tokens", ctypes.c_int32),
        ("ctx_part_tokens", ctypes.c_int32), ("reserved0", ctypes.c_int32),
    ]


class RAPrefix(ctypes.Structure):
    _fields_ = [("k_sys", ctypes.c_void_p), ("v_sys", ctypes.c_void_p), ("sys_len", ctypes.c_int32),
                ("first_request", ctypes.c_int32), ("num_requests", ctypes.c_int32)]


class RADecodePlan(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "sys_chunk_tokens", "num_sys_chunks", "num_sys_workgroups", "num_ctx_wavefronts",
        "min_tiles_per_ctx_wavefront", "num_ctx_slots", "max_blocks_per_span",
        "first_light_ctx_wavefront", "num_light_ctx_wavefronts", "sys_workgroup_tiles",
        "sys_tiles_total", "sys_rows_per_workgroup", "compute_units")]


class RAValidateReport(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "bad_context_lens", "bad_block_ids", "bad_query_lens", "first_bad_request")]


ABI_VERSION = 6      # the structures above mirror include/relay_attn.h at this version


class RelayAttnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (ra_status %d)" % (where, status_string(status), status))


_lib = None


def load() -> ctypes.CDLL:
    """Load the HIP library built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "librelayattn.so is not built: run `python -m paper_2402_14808_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    P, V, I32, SZ = ctypes.POINTER(RAParams), ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.relay_attn_workspace_bytes.restype = SZ
    lib.relay_attn_workspace_bytes.argtypes = [P, I32]
    lib.relay_attn_decode.restype = ctypes.c_int
    lib.relay_attn_decode.argtypes = [P, V, V, V, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_decode_append.restype = ctypes.c_int
    lib.relay_attn_decode_append.argtypes = [P, V, V, V, ctypes.c_int64, ctypes.c_int64, V, V, V, V, V, V,
                                             V, V, V, SZ, V]
    lib.relay_attn_debug_decode_phases.restype = ctypes.c_int
    lib.relay_attn_debug_decode_phases.argtypes = [P, I32, V, V, V, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_debug_timeline.restype = ctypes.c_int
    lib.relay_attn_debug_timeline.argtypes = [P, V, V, I32, I32, V, V, V, V, V, V, V, V, V, SZ, V, I32, V]
    lib.relay_attn_decode_static.restype = ctypes.c_int
    lib.relay_attn_decode_static.argtypes = [P, V, V, V, V, V, V, V, V, V, V]
    lib.relay_attn_debug_stream_probe.restype = ctypes.c_int
    lib.relay_attn_debug_stream_probe.argtypes = [V, SZ, I32, V, V]
    lib.relay_attn_debug_launch_probe.restype = ctypes.c_int
    lib.relay_attn_debug_launch_probe.argtypes = [V, I32, V]
    lib.relay_attn_static_scratch_bytes.restype = SZ
    lib.relay_attn_static_scratch_bytes.argtypes = []
    lib.relay_attn_decode_plan.restype = ctypes.c_int
    lib.relay_attn_decode_plan.argtypes = [P, ctypes.POINTER(RADecodePlan)]
    lib.relay_attn_decode_multi.restype = ctypes.c_int
    lib.relay_attn_decode_multi.argtypes = [P, I32, ctypes.POINTER(RAPrefix), V, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_decode_grouped.restype = ctypes.c_int
    lib.relay_attn_decode_grouped.argtypes = [P, I32, ctypes.POINTER(RAPrefix), V, V, V, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_group_requests.restype = ctypes.c_int
    lib.relay_attn_group_requests.argtypes = [ctypes.POINTER(ctypes.c_int32), I32, I32,
                                              ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32)]
    lib.relay_attn_prefill_multi.restype = ctypes.c_int
    lib.relay_attn_prefill_multi.argtypes = [P, I32, ctypes.POINTER(RAPrefix), ctypes.POINTER(ctypes.c_int32),
                                             V, V, I32, I32, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_system_cache_layout.restype = ctypes.c_int
    lib.relay_attn_system_cache_layout.argtypes = [P, ctypes.POINTER(ctypes.c_int64),
                                                   ctypes.POINTER(ctypes.c_int64),
                                                   ctypes.POINTER(ctypes.c_size_t)]
    lib.relay_attn_system_fill.restype = ctypes.c_int
    lib.relay_attn_system_fill.argtypes = [P, V, V, ctypes.c_int64, ctypes.c_int64, I32, I32, V, V, V]
    lib.relay_attn_prefill.restype = ctypes.c_int
    lib.relay_attn_prefill.argtypes = [P, V, V, I32, I32, V, V, V, V, V, V, V, V, V, SZ, V]
    lib.paged_attn_decode_naive.restype = ctypes.c_int
    lib.paged_attn_decode_naive.argtypes = [P, V, V, V, V, V, V, V, V, SZ, V]
    lib.relay_attn_cache_append.restype = ctypes.c_int
    lib.relay_attn_cache_append.argtypes = [P, V, V, ctypes.c_int64, ctypes.c_int64, V, I32, V, V, V, V, V]
    lib.relay_attn_debug_validate.restype = ctypes.c_int
    lib.relay_attn_debug_validate.argtypes = [P, V, V, V, I32, V, SZ, V, ctypes.POINTER(RAValidateReport)]
    lib.relay_attn_status_string.restype = ctypes.c_char_p
    lib.relay_attn_status_string.argtypes = [ctypes.c_int]
    lib.relay_attn_abi_version.restype = I32
    lib.relay_attn_abi_version.argtypes = []
    if lib.relay_attn_abi_version() != ABI_VERSION:
        raise RuntimeError("librelayattn.so has ABI version %d, this binding expects %d: rebuild it "
                           "(`python -m paper_2402_14808_amd.build`)"
                           % (lib.relay_attn_abi_version(), ABI_VERSION))
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().relay_attn_status_string(int(status)).decode()


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_params(q, out, k_sys, k_cache, block_tables, *, batch, softmax_scale,
                max_context_len=0, sys_chunk_tokens=0, ctx_part_tokens=0) -> RAParams:
    """Fill ra_params from tensor shapes/strides.  q/out: [tokens, Hq, d]; k_sys: [s, Hkv, d]
    (any token/head strides) or None; k_cache: [num_blocks, Hkv, block_size, d] contiguous."""
    import torch
    p = RAParams()
    p.batch = int(batch)
    p.num_q_heads, p.head_dim = int(q.shape[1]), int(q.shape[2])
    p.num_kv_heads = int(k_cache.shape[1])
    p.sys_len = 0 if k_sys is None else int(k_sys.shape[0])
    p.block_size = int(k_cache.shape[2])
    p.num_blocks = int(k_cache.shape[0])
    p.max_blocks_per_seq = int(block_tables.shape[1])
    p.max_context_len = int(max_context_len)
    p.softmax_scale = float(softmax_scale)
    p.q_stride_token, p.q_stride_head = int(q.stride(0)), int(q.stride(1))
    p.o_stride_token, p.o_stride_head = int(out.stride(0)), int(out.stride(1))
    if k_sys is not None and k_sys.shape[0] > 0:
        p.sys_stride_token, p.sys_stride_head = int(k_sys.stride(0)), int(k_sys.stride(1))
    else:
        p.sys_stride_token, p.sys_stride_head = p.num_kv_heads * p.head_dim, p.head_dim
    p.out_is_fp32 = 1 if out.dtype == torch.float32 else 0
    p.sys_chunk_tokens, p.ctx_part_tokens = int(sys_chunk_tokens), int(ctx_part_tokens)
    p.reserved0 = 0
    return p


def relay_attn_decode_plan(params: RAParams) -> RADecodePlan:
    plan = RADecodePlan()
    _check(load().relay_attn_decode_plan(ctypes.byref(params), ctypes.byref(plan)),
           "relay_attn_decode_plan")
    return plan


def relay_attn_workspace_bytes(params: RAParams, total_q: int) -> int:
    return int(load().relay_attn_workspace_bytes(ctypes.byref(params), int(total_q)))


def _check(status, where):
    if status != RA_OK:
        raise RelayAttnError(status, where)


def relay_attn_decode(params, q, k_sys, v_sys, k_cache, v_cache, block_tables, context_lens,
                      out, lse_out, workspace):
    st = load().relay_attn_decode(
        ctypes.byref(params), _ptr(q), _ptr(k_sys), _ptr(v_sys), _ptr(k_cache), _ptr(v_cache),
        _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_decode")


def relay_attn_decode_append(params, q, k_new, v_new, k_sys, v_sys, k_cache, v_cache, block_tables,
                             context_lens, out, lse_out, workspace):
    """k_new / v_new: [batch, Hkv, d] tensors (any token / head strides, d contiguous)."""
    assert k_new.stride() == v_new.stride() and k_new.stride(2) == 1
    st = load().relay_attn_decode_append(
        ctypes.byref(params), _ptr(q), _ptr(k_new), _ptr(v_new), int(k_new.stride(0)),
        int(k_new.stride(1)), _ptr(k_sys), _ptr(v_sys), _ptr(k_cache), _ptr(v_cache),
        _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_decode_append")


def relay_attn_debug_timeline(params, q, cu_seqlens_q, total_q, max_q_len, k_sys, v_sys, k_cache, v_cache,
                              block_tables, context_lens, out, lse_out, workspace, timeline):
    """timeline: int64 / uint64 device tensor of 2 * n values (n wavefronts recorded)."""
    st = load().relay_attn_debug_timeline(
        ctypes.byref(params), _ptr(q), _ptr(cu_seqlens_q), int(total_q), int(max_q_len), _ptr(k_sys),
        _ptr(v_sys), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(context_lens), _ptr(out),
        _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(timeline),
        timeline.numel() // 2, _stream())
    _check(st, "relay_attn_debug_timeline")


def relay_attn_decode_static(params, q, k_sys, v_sys, k_cache, v_cache, block_tables, context_lens,
                             out, lse_out):
    st = load().relay_attn_decode_static(
        ctypes.byref(params), _ptr(q), _ptr(k_sys), _ptr(v_sys), _ptr(k_cache), _ptr(v_cache),
        _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(lse_out), _stream())
    _check(st, "relay_attn_decode_static")


def relay_attn_debug_stream_probe(src, nbytes, nontemporal, sink):
    _check(load().relay_attn_debug_stream_probe(_ptr(src), int(nbytes), int(nontemporal), _ptr(sink),
                                                _stream()), "relay_attn_debug_stream_probe")


def relay_attn_debug_launch_probe(sink, count=1):
    _check(load().relay_attn_debug_launch_probe(_ptr(sink), int(count), _stream()),
           "relay_attn_debug_launch_probe")


def relay_attn_static_scratch_bytes() -> int:
    return int(load().relay_attn_static_scratch_bytes())


def relay_attn_debug_decode_phases(params, phases, q, k_sys, v_sys, k_cache, v_cache, block_tables,
                                   context_lens, out, lse_out, workspace):
    st = load().relay_attn_debug_decode_phases(
        ctypes.byref(params), int(phases), _ptr(q), _ptr(k_sys), _ptr(v_sys), _ptr(k_cache),
        _ptr(v_cache), _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(lse_out),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_debug_decode_phases")


def relay_attn_prefill(params, q, cu_seqlens_q, total_q, max_q_len, k_sys, v_sys, k_cache,
                       v_cache, block_tables, context_lens, out, lse_out, workspace):
    st = load().relay_attn_prefill(
        ctypes.byref(params), _ptr(q), _ptr(cu_seqlens_q), int(total_q), int(max_q_len),
        _ptr(k_sys), _ptr(v_sys), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
        _ptr(context_lens), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_prefill")


def relay_attn_prefill_multi(params, groups, group_tokens, q, cu_seqlens_q, total_q, max_q_len, k_cache,
                             v_cache, block_tables, context_lens, out, lse_out, workspace):
    """groups: as for make_prefixes; group_tokens: new tokens of each group (host ints)."""
    arr = make_prefixes(groups) if isinstance(groups, (list, tuple)) else groups
    toks = (ctypes.c_int32 * len(arr))(*[int(x) for x in group_tokens])
    st = load().relay_attn_prefill_multi(
        ctypes.byref(params), len(arr), arr, toks, _ptr(q), _ptr(cu_seqlens_q), int(total_q),
        int(max_q_len), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(context_lens),
        _ptr(out), _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(),
        _stream())
    _check(st, "relay_attn_prefill_multi")


def paged_attn_decode_naive(params, q, k_cache, v_cache, block_tables, context_lens, out,
                            lse_out, workspace):
    st = load().paged_attn_decode_naive(
        ctypes.byref(params), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
        _ptr(context_lens), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "paged_attn_decode_naive")


def relay_attn_cache_append(params, k_new, v_new, cu_seqlens_q, total_q, k_cache, v_cache,
                            block_tables, context_lens):
    """k_new / v_new: [total_q, Hkv, d] tensors (any token / head strides, d contiguous)."""
    assert k_new.stride() == v_new.stride() and k_new.stride(2) == 1
    st = load().relay_attn_cache_append(
        ctypes.byref(params), _ptr(k_new), _ptr(v_new), int(k_new.stride(0)), int(k_new.stride(1)),
        _ptr(cu_seqlens_q), int(total_q), _ptr(k_cache), _ptr(v_cache), _ptr(block_tables),
        _ptr(context_lens), _stream())
    _check(st, "relay_attn_cache_append")


def make_prefixes(groups):
    """groups: list of (k_sys, v_sys, first_request, num_requests); k_sys [s_i, Hkv, d] tensors
    that all have the strides recorded in params (or None for an empty prefix).  Returns the
    host array relay_attn_decode_multi takes; the caller keeps the tensors alive."""
    arr = (RAPrefix * len(groups))()
    for i, (ks, vs, first, count) in enumerate(groups):
        n = 0 if ks is None else int(ks.shape[0])
        arr[i].k_sys = ks.data_ptr() if n else None
        arr[i].v_sys = vs.data_ptr() if n else None
        arr[i].sys_len, arr[i].first_request, arr[i].num_requests = n, int(first), int(count)
    return arr


def relay_attn_decode_multi(params, groups, q, k_cache, v_cache, block_tables, context_lens, out,
                            lse_out, workspace):
    """groups: a list as for make_prefixes, or the array it returned."""
    arr = make_prefixes(groups) if isinstance(groups, (list, tuple)) else groups
    st = load().relay_attn_decode_multi(
        ctypes.byref(params), len(arr), arr, _ptr(q), _ptr(k_cache), _ptr(v_cache),
        _ptr(block_tables), _ptr(context_lens), _ptr(out), _ptr(lse_out), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_decode_multi")


def relay_attn_group_requests(sys_id, num_prefixes):
    """sys_id: a host sequence of ints.  Returns (request_order, num_requests) as lists."""
    n = len(sys_id)
    ids = (ctypes.c_int32 * max(n, 1))(*[int(x) for x in sys_id])
    order = (ctypes.c_int32 * max(n, 1))()
    counts = (ctypes.c_int32 * int(num_prefixes))()
    _check(load().relay_attn_group_requests(ids, n, int(num_prefixes), order, counts),
           "relay_attn_group_requests")
    return list(order[:n]), list(counts)


def relay_attn_decode_grouped(params, prefixes, sys_id, request_order, q, k_cache, v_cache,
                              block_tables, context_lens, out, lse_out, workspace):
    """prefixes: list of (k_sys, v_sys, num_requests) per application (k_sys None for an empty
    prefix); sys_id / request_order: int32 device tensors [batch]."""
    arr = make_prefixes([(k, v, 0, n) for k, v, n in prefixes])
    st = load().relay_attn_decode_grouped(
        ctypes.byref(params), len(arr), arr, _ptr(sys_id), _ptr(request_order), _ptr(q),
        _ptr(k_cache), _ptr(v_cache), _ptr(block_tables), _ptr(context_lens), _ptr(out),
        _ptr(lse_out), _ptr(workspace), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "relay_attn_decode_grouped")


def relay_attn_debug_validate(params, block_tables, context_lens, workspace, cu_seqlens_q=None,
                              total_q=None):
    """Range check of lengths and block ids on the device (synchronises).  Returns
    (status, RAValidateReport); does not raise when the contents are out of range."""
    rep = RAValidateReport()
    st = load().relay_attn_debug_validate(
        ctypes.byref(params), _ptr(block_tables), _ptr(context_lens), _ptr(cu_seqlens_q),
        int(params.batch if total_q is None else total_q), _ptr(workspace),
        int(workspace.numel() * workspace.element_size()), _stream(), ctypes.byref(rep))
    return int(st), rep


def relay_attn_system_cache_layout(sys_len, num_kv_heads, head_dim):
    """(stride_token, stride_head, bytes per buffer) of the recommended system-cache layout."""
    p = RAParams()
    p.sys_len, p.num_kv_heads, p.head_dim = int(sys_len), int(num_kv_heads), int(head_dim)
    st_tok, st_head, nbytes = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_size_t()
    st = load().relay_attn_system_cache_layout(ctypes.byref(p), ctypes.byref(st_tok),
                                               ctypes.byref(st_head), ctypes.byref(nbytes))
    _check(st, "relay_attn_system_cache_layout")
    return st_tok.value, st_head.value, nbytes.value


def system_cache_view(buffer, sys_len, num_kv_heads, head_dim):
    """[sys_len, Hkv, d] view with the recommended strides over a flat bf16 buffer of at least
    the recommended size (the caller allocates it; nothing is copied)."""
    st_tok, st_head, nbytes = relay_attn_system_cache_layout(sys_len, num_kv_heads, head_dim)
    assert buffer.numel() * buffer.element_size() >= nbytes and buffer.element_size() == 2
    return buffer.as_strided((int(sys_len), int(num_kv_heads), int(head_dim)), (st_tok, st_head, 1))


def relay_attn_system_fill(params, k_new, v_new, first_pos, k_sys, v_sys):
    """k_new/v_new: [n, Hkv, d] (any token/head strides) written to system positions
    first_pos .. first_pos+n-1."""
    st = load().relay_attn_system_fill(
        ctypes.byref(params), _ptr(k_new), _ptr(v_new), int(k_new.stride(0)), int(k_new.stride(1)),
        int(first_pos), int(k_new.shape[0]), _ptr(k_sys), _ptr(v_sys), _stream())
    _check(st, "relay_attn_system_fill")
