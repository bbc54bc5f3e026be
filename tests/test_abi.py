"""CPU-only checks of the C ABI: the library loads, exports every function the header
declares, and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2402_14808_amd as ra
from paper_2402_14808_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b([a-z_0-9]+)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = ra.load()
    declared = _declared_functions()
    assert set(binding.EXPORTED) <= set(declared)
    assert len(declared) >= 6
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_and_version():
    assert ra.load().relay_attn_abi_version() >= 1
    seen = {ra.status_string(i) for i in range(5)}
    assert len(seen) == 5 and "ok" in seen
    assert ra.status_string(99) == "unknown status"


def _params(**kw):
    p = ra.RAParams()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = 4, 8, 2, 128
    p.sys_len, p.block_size, p.num_blocks, p.max_blocks_per_seq = 256, 16, 64, 8
    p.max_context_len, p.softmax_scale = 100, 0.088
    p.q_stride_token, p.q_stride_head = 8 * 128, 128
    p.o_stride_token, p.o_stride_head = 8 * 128, 128
    p.sys_stride_token, p.sys_stride_head = 2 * 128, 128
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def test_workspace_bytes_grows_with_work_and_rejects_bad_params():
    small = ra.relay_attn_workspace_bytes(_params(), 4)
    assert small > 0 and small % 256 == 0
    assert ra.relay_attn_workspace_bytes(_params(sys_len=8192), 4) > small
    assert ra.relay_attn_workspace_bytes(_params(), 64) > small
    assert ra.relay_attn_workspace_bytes(_params(head_dim=96), 4) == 0
    assert ra.relay_attn_workspace_bytes(_params(num_kv_heads=3), 4) == 0
    assert ra.relay_attn_workspace_bytes(_params(batch=-1), 4) == 0


FAKE = 0x10000  # a non-null, 256-byte aligned address that is never dereferenced on the host


def _decode(p, q=FAKE, ks=FAKE, vs=FAKE, kc=FAKE, vc=FAKE, bt=FAKE, cl=FAKE, out=FAKE, lse=None,
            ws=FAKE, ws_bytes=1 << 40):
    lib = ra.load()
    V = ctypes.c_void_p
    return lib.relay_attn_decode(ctypes.byref(p), V(q), V(ks), V(vs), V(kc), V(vc), V(bt), V(cl),
                                 V(out), V(lse), V(ws), ws_bytes, None)


@pytest.mark.parametrize("kw,code", [
    (dict(head_dim=96), binding.RA_ERR_UNSUPPORTED),
    (dict(num_q_heads=18, num_kv_heads=2), binding.RA_ERR_UNSUPPORTED),    # group 9 (1 .. 8 are supported)
    (dict(num_q_heads=7), binding.RA_ERR_INVALID_ARG),                      # not divisible
    (dict(batch=-2), binding.RA_ERR_INVALID_ARG),
    (dict(sys_len=-1), binding.RA_ERR_INVALID_ARG),
    (dict(block_size=12), binding.RA_ERR_INVALID_ARG),
    (dict(q_stride_head=100), binding.RA_ERR_INVALID_ARG),                  # not a multiple of 8
    (dict(q_stride_head=64), binding.RA_ERR_INVALID_ARG),                   # rows overlap
    (dict(max_context_len=1000), binding.RA_ERR_INVALID_ARG),               # > table capacity
    (dict(sys_chunk_tokens=100), binding.RA_ERR_INVALID_ARG),
    (dict(ctx_part_tokens=64), binding.RA_ERR_INVALID_ARG),
    (dict(out_is_fp32=2), binding.RA_ERR_INVALID_ARG),
    (dict(softmax_scale=float("nan")), binding.RA_ERR_INVALID_ARG),
    (dict(reserved0=7), binding.RA_ERR_INVALID_ARG),
])
def test_decode_rejects_bad_scalars(kw, code):
    assert _decode(_params(**kw)) == code


def test_decode_rejects_bad_pointers_and_workspace():
    p = _params()
    assert _decode(p, q=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, out=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, ks=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, kc=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, bt=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, cl=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, q=FAKE + 2) == binding.RA_ERR_INVALID_ARG            # misaligned
    assert _decode(p, ws=None) == binding.RA_ERR_INVALID_ARG
    assert _decode(p, ws=FAKE + 16) == binding.RA_ERR_INVALID_ARG          # not 256-aligned
    need = ra.relay_attn_workspace_bytes(p, p.batch)
    assert _decode(p, ws_bytes=need - 1) == binding.RA_ERR_WORKSPACE_TOO_SMALL
    assert ra.load().relay_attn_decode(None, *([None] * 10), 0, None) == binding.RA_ERR_INVALID_ARG


def test_empty_batch_is_ok_without_any_launch():
    assert _decode(_params(batch=0)) == binding.RA_OK


def test_naive_rejects_system_prompt_and_prefill_rejects_inconsistent_counts():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()
    st = lib.paged_attn_decode_naive(ctypes.byref(p), V(FAKE), V(FAKE), V(FAKE), V(FAKE),
                                     V(FAKE), V(FAKE), None, V(FAKE), 1 << 40, None)
    assert st == binding.RA_ERR_INVALID_ARG
    st = lib.relay_attn_prefill(ctypes.byref(p), V(FAKE), None, 10, 5, V(FAKE), V(FAKE), V(FAKE),
                                V(FAKE), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE), 1 << 40, None)
    assert st == binding.RA_ERR_INVALID_ARG                                 # cu_seqlens_q null
    st = lib.relay_attn_prefill(ctypes.byref(p), V(FAKE), V(FAKE), 100, 5, V(FAKE), V(FAKE),
                                V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE),
                                1 << 40, None)
    assert st == binding.RA_ERR_INVALID_ARG                                 # 4 requests x 5 < 100


def test_decode_append_and_phase_entry_argument_checks():
    lib = ra.load()
    V, I64 = ctypes.c_void_p, ctypes.c_int64
    p = _params()

    def app(kn=FAKE, vn=FAKE, st=None, sh=None, ws_bytes=1 << 40, params=p):
        st = p.num_kv_heads * p.head_dim if st is None else st
        sh = p.head_dim if sh is None else sh
        return lib.relay_attn_decode_append(ctypes.byref(params), V(FAKE), V(kn), V(vn), I64(st), I64(sh),
                                            V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE),
                                            None, V(FAKE), ws_bytes, None)

    assert app(kn=None) == binding.RA_ERR_INVALID_ARG
    assert app(vn=FAKE + 2) == binding.RA_ERR_INVALID_ARG                   # misaligned
    assert app(st=-8) == binding.RA_ERR_INVALID_ARG
    assert app(sh=12) == binding.RA_ERR_INVALID_ARG                         # not a multiple of 8
    assert app(sh=64) == binding.RA_ERR_INVALID_ARG                         # heads overlap
    assert app(ws_bytes=16) == binding.RA_ERR_WORKSPACE_TOO_SMALL
    assert app(params=_params(batch=0)) == binding.RA_OK                    # nothing to do, no launch
    assert app(params=_params(head_dim=96)) == binding.RA_ERR_UNSUPPORTED
    for phases in (0, 4, -1):
        st = lib.relay_attn_debug_decode_phases(ctypes.byref(p), phases, *([V(FAKE)] * 8), None, V(FAKE),
                                                1 << 40, None)
        assert st == binding.RA_ERR_INVALID_ARG


def test_static_scratch_entry_argument_checks():
    lib = ra.load()
    V = ctypes.c_void_p
    assert ra.relay_attn_static_scratch_bytes() == 32 << 20
    assert lib.relay_attn_decode_static(None, *([None] * 10)) == binding.RA_ERR_INVALID_ARG
    p = _params(head_dim=96)
    assert lib.relay_attn_decode_static(ctypes.byref(p), *([V(FAKE)] * 8), None, None) == binding.RA_ERR_UNSUPPORTED
    p = _params(batch=0)
    assert lib.relay_attn_decode_static(ctypes.byref(p), *([V(FAKE)] * 8), None, None) == binding.RA_OK
    # a batch whose partials exceed the fixed array is refused before any HIP call
    p = _params(batch=1 << 16, num_q_heads=64, num_kv_heads=64)
    assert ra.relay_attn_workspace_bytes(p, p.batch) > ra.relay_attn_static_scratch_bytes()
    assert lib.relay_attn_decode_static(ctypes.byref(p), *([V(FAKE)] * 8), None, None) == \
        binding.RA_ERR_WORKSPACE_TOO_SMALL


def test_plan_reports_the_compute_unit_count():
    plan = ra.relay_attn_decode_plan(_params())
    assert plan.compute_units >= 1          # 256 on a machine without a GPU, the device's count with one


def test_binding_raises_with_status():
    with pytest.raises(ra.RelayAttnError) as e:
        binding._check(binding.RA_ERR_UNSUPPORTED, "x")
    assert e.value.status == binding.RA_ERR_UNSUPPORTED


def test_cache_append_argument_checks():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()

    def call(kn=FAKE, vn=FAKE, st=2 * 128, sh=128, cu=None, total=4, kc=FAKE, vc=FAKE, bt=FAKE, cl=FAKE):
        return lib.relay_attn_cache_append(ctypes.byref(p), V(kn), V(vn), st, sh, V(cu), total,
                                           V(kc), V(vc), V(bt), V(cl), None)
    assert call(kn=None) == binding.RA_ERR_INVALID_ARG
    assert call(kc=None) == binding.RA_ERR_INVALID_ARG
    assert call(bt=None) == binding.RA_ERR_INVALID_ARG
    assert call(st=100) == binding.RA_ERR_INVALID_ARG                 # stride not a multiple of 8
    assert call(sh=64) == binding.RA_ERR_INVALID_ARG                  # head rows overlap
    assert call(total=5) == binding.RA_ERR_INVALID_ARG                # decode: one token per request
    assert call(total=0, cu=FAKE) == binding.RA_OK                    # nothing to write
    assert call(kn=FAKE + 4) == binding.RA_ERR_INVALID_ARG            # misaligned


def test_decode_multi_checks_the_grouping_on_the_host():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()                                                     # batch 4, sys_len 256

    def call(groups, count=None, params=p, ws_bytes=1 << 40):
        arr = (ra.RAPrefix * max(len(groups), 1))()
        for i, (k, v, s, first, n) in enumerate(groups):
            arr[i].k_sys, arr[i].v_sys = k, v
            arr[i].sys_len, arr[i].first_request, arr[i].num_requests = s, first, n
        return lib.relay_attn_decode_multi(ctypes.byref(params), len(groups) if count is None else count,
                                           arr, V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE),
                                           V(FAKE), None, V(FAKE), ws_bytes, None)
    INV, UNS = binding.RA_ERR_INVALID_ARG, binding.RA_ERR_UNSUPPORTED
    assert call([(FAKE, FAKE, 256, 0, 4)], count=0) == INV
    assert call([(FAKE, FAKE, 256, 0, 3)]) == INV                     # request 3 in no group
    assert call([(FAKE, FAKE, 256, 0, 2), (FAKE, FAKE, 100, 3, 1)]) == INV      # gap
    assert call([(FAKE, FAKE, 256, 0, 3), (FAKE, FAKE, 100, 2, 2)]) == INV      # overlap
    assert call([(FAKE, FAKE, 128, 0, 2), (FAKE, FAKE, 100, 2, 2)]) == INV      # p.sys_len != longest
    assert call([(None, FAKE, 256, 0, 2), (FAKE, FAKE, 100, 2, 2)]) == INV
    assert call([(FAKE, FAKE + 2, 256, 0, 2), (FAKE, FAKE, 100, 2, 2)]) == INV  # misaligned
    assert call([(FAKE, FAKE, 256, 0, 2), (FAKE, FAKE, 100, 2, 0), (FAKE, FAKE, 9, 2, 2)]) == INV
    p33 = _params(batch=33, max_blocks_per_seq=8)
    assert call([(FAKE, FAKE, 256, i, 1) for i in range(33)], params=p33) == UNS  # more than 32 groups
    # a valid grouping gets as far as the workspace check: the size asked for without knowing the
    # grouping is enough for any grouping
    need = ra.relay_attn_workspace_bytes(p, p.batch)
    ok = [(FAKE, FAKE, 256, 0, 1), (None, None, 0, 1, 1), (FAKE, FAKE, 31, 2, 2)]
    assert call(ok, ws_bytes=need - 1) == binding.RA_ERR_WORKSPACE_TOO_SMALL
    assert call(ok, params=_params(batch=0)) == INV                   # groups must tile the batch


def test_prefill_multi_checks_groups_and_token_counts_on_the_host():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()                                                     # batch 4, sys_len 256

    def call(groups, toks, total_q=12, max_q=5, cu=FAKE, params=p, ws_bytes=1 << 40, count=None):
        arr = (ra.RAPrefix * max(len(groups), 1))()
        for i, (k, v, s, first, n) in enumerate(groups):
            arr[i].k_sys, arr[i].v_sys = k, v
            arr[i].sys_len, arr[i].first_request, arr[i].num_requests = s, first, n
        t = (ctypes.c_int32 * max(len(toks), 1))(*toks)
        return lib.relay_attn_prefill_multi(ctypes.byref(params), len(groups) if count is None else count,
                                            arr, t, V(FAKE), V(cu), total_q, max_q, V(FAKE), V(FAKE),
                                            V(FAKE), V(FAKE), V(FAKE), None, V(FAKE), ws_bytes, None)
    INV, UNS = binding.RA_ERR_INVALID_ARG, binding.RA_ERR_UNSUPPORTED
    two = [(FAKE, FAKE, 256, 0, 1), (FAKE, FAKE, 100, 1, 3)]
    assert call(two, [3, 9], count=0) == INV
    assert call(two, [3, 8]) == INV                                   # token counts do not add up
    assert call(two, [6, 6]) == INV                                   # 6 tokens in one request of <= 5
    assert call(two, [-1, 13]) == INV
    assert call(two, [3, 9], cu=None) == INV
    assert call(two, [3, 9], max_q=2) == INV                          # 4 requests of <= 2 tokens < 12
    assert call([(FAKE, FAKE, 256, 0, 1), (FAKE, FAKE, 100, 2, 2)], [3, 9]) == INV      # gap
    assert call([(FAKE, FAKE, 128, 0, 1), (FAKE, FAKE, 100, 1, 3)], [3, 9]) == INV      # p.sys_len != longest
    assert call([(FAKE, None, 256, 0, 1), (FAKE, FAKE, 100, 1, 3)], [3, 9]) == INV
    assert call([(FAKE + 2, FAKE, 256, 0, 1), (FAKE, FAKE, 100, 1, 3)], [3, 9]) == INV  # misaligned
    p33 = _params(batch=33, max_blocks_per_seq=8)
    assert call([(FAKE, FAKE, 256, i, 1) for i in range(33)], [1] * 33, total_q=33, params=p33) == UNS
    # a valid call gets as far as the workspace check
    ok = [(FAKE, FAKE, 256, 0, 1), (None, None, 0, 1, 1), (FAKE, FAKE, 31, 2, 2)]
    assert call(ok, [5, 0, 7], ws_bytes=16) == binding.RA_ERR_WORKSPACE_TOO_SMALL
    assert call(ok, [0, 0, 0], total_q=0, cu=None) == binding.RA_OK   # nothing to do, no launch


def test_group_requests_and_grouped_decode_checks():
    order, counts = ra.relay_attn_group_requests([2, 0, 2, 1, 0, 2], 4)
    assert order == [1, 4, 3, 0, 2, 5] and counts == [2, 1, 3, 0]
    assert ra.relay_attn_group_requests([], 3) == ([], [0, 0, 0])
    with pytest.raises(ra.RelayAttnError):
        ra.relay_attn_group_requests([0, 3], 3)                       # id out of range
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()                                                     # batch 4, sys_len 256

    def call(groups, sid=FAKE, order=FAKE, params=p):
        arr = (ra.RAPrefix * max(len(groups), 1))()
        for i, (k, v, s, n) in enumerate(groups):
            arr[i].k_sys, arr[i].v_sys, arr[i].sys_len, arr[i].num_requests = k, v, s, n
        return lib.relay_attn_decode_grouped(ctypes.byref(params), len(groups), arr, V(sid), V(order),
                                             V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE), V(FAKE), None,
                                             V(FAKE), 16, None)
    INV = binding.RA_ERR_INVALID_ARG
    ok = [(FAKE, FAKE, 256, 1), (FAKE, FAKE, 100, 0), (None, None, 0, 3)]
    assert call(ok) == binding.RA_ERR_WORKSPACE_TOO_SMALL             # everything else accepted
    assert call(ok, sid=None) == INV and call(ok, order=None) == INV
    assert call([(FAKE, FAKE, 256, 1), (FAKE, FAKE, 100, 2)]) == INV  # counts do not add up to the batch
    assert call([(FAKE, FAKE, 100, 4), (FAKE, FAKE, 256, 0)]) == INV  # longest used prefix != p.sys_len
    assert call([(FAKE, FAKE, 256, -1), (FAKE, FAKE, 100, 5)]) == INV
    assert call([(None, FAKE, 256, 4)]) == INV


def test_debug_timeline_argument_checks():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()

    def call(tl=FAKE, n=64, cu=None, total_q=None, max_q=1, ws_bytes=16):
        tq = p.batch if total_q is None else total_q
        return lib.relay_attn_debug_timeline(ctypes.byref(p), V(FAKE), V(cu), tq, max_q, V(FAKE), V(FAKE), V(FAKE),
                                             V(FAKE), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE), ws_bytes, V(tl), n,
                                             None)
    INV = binding.RA_ERR_INVALID_ARG
    assert call(tl=None) == INV and call(n=0) == INV and call(tl=FAKE + 4) == INV
    assert call(total_q=p.batch + 1) == INV and call(max_q=2) == INV      # decode: one token per request
    assert call() == binding.RA_ERR_WORKSPACE_TOO_SMALL                   # everything else accepted
    assert call(cu=FAKE, total_q=40, max_q=20) == binding.RA_ERR_WORKSPACE_TOO_SMALL


def test_system_cache_layout_is_host_arithmetic():
    """The recommended row stride is the smallest one >= the dense stride that is 384 mod 1024
    bytes; the buffer ends with the last row's data."""
    for s_len, Hkv, d in [(2048, 52, 128), (2048, 32, 128), (8192, 8, 128), (100, 5, 128), (1, 52, 64),
                          (7, 3, 64), (0, 52, 128)]:
        st_tok, st_head, nbytes = ra.relay_attn_system_cache_layout(s_len, Hkv, d)
        dense = Hkv * d
        assert st_head == d and st_tok >= dense and st_tok - dense < 512
        assert (st_tok * 2) % 1024 == 384 and st_tok % 8 == 0
        assert nbytes == (((s_len - 1) * st_tok + dense) * 2 if s_len else 0)
    assert ra.relay_attn_system_cache_layout(2048, 52, 128)[0] == 6848          # 13696 bytes
    lib = ra.load()
    p = _params()
    a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_size_t()
    INV = binding.RA_ERR_INVALID_ARG
    assert lib.relay_attn_system_cache_layout(None, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)) == INV
    assert lib.relay_attn_system_cache_layout(ctypes.byref(p), None, ctypes.byref(b), ctypes.byref(c)) == INV
    assert lib.relay_attn_system_cache_layout(ctypes.byref(_params(num_kv_heads=0)), ctypes.byref(a),
                                              ctypes.byref(b), ctypes.byref(c)) == INV
    # the strides it names are accepted by the entry points' checks
    p.sys_stride_token, p.sys_stride_head = ra.relay_attn_system_cache_layout(p.sys_len, p.num_kv_heads, p.head_dim)[:2]
    assert ra.relay_attn_workspace_bytes(p, p.batch) > 0


def test_system_fill_argument_checks():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()                                                     # sys_len 256

    def call(kn=FAKE, vn=FAKE, st=2 * 128, sh=128, first=0, n=256, ks=FAKE, vs=FAKE, params=p):
        return lib.relay_attn_system_fill(ctypes.byref(params), V(kn), V(vn), st, sh, first, n,
                                          V(ks), V(vs), None)
    INV = binding.RA_ERR_INVALID_ARG
    assert call(n=257) == INV and call(first=200, n=57) == INV and call(first=-1) == INV
    assert call(kn=None) == INV and call(vs=None) == INV and call(ks=FAKE + 8) == INV
    assert call(st=100) == INV and call(sh=64) == INV
    assert call(n=0, kn=None, ks=None) == binding.RA_OK               # nothing to write
    assert call(params=_params(head_dim=96)) == binding.RA_ERR_UNSUPPORTED


def test_debug_validate_argument_checks():
    lib = ra.load()
    V = ctypes.c_void_p
    p = _params()

    def call(bt=FAKE, cl=FAKE, cu=None, total_q=None, ws=FAKE, ws_bytes=256, params=p):
        tq = params.batch if total_q is None else total_q
        return lib.relay_attn_debug_validate(ctypes.byref(params), V(bt), V(cl), V(cu), tq, V(ws),
                                             ws_bytes, None, None)
    INV = binding.RA_ERR_INVALID_ARG
    assert lib.relay_attn_debug_validate(None, V(FAKE), V(FAKE), None, 0, V(FAKE), 256, None, None) == INV
    assert call(cl=None) == INV and call(bt=None) == INV
    assert call(total_q=p.batch + 1) == INV                 # decode: one query token per request
    assert call(ws=None) == INV and call(ws=FAKE + 16) == INV
    assert call(ws_bytes=255) == binding.RA_ERR_WORKSPACE_TOO_SMALL
    assert call(params=_params(head_dim=96)) == binding.RA_ERR_UNSUPPORTED
