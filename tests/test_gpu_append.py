"""GPU tests of relay_attn_cache_append (the cache write that precedes attention in Alg. 1):
byte-exact against the oracle's cache write, then decode on the appended cache against the oracle."""
import sys
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
import paper_2402_14808_amd as ra
import workloads as W
from gpu_util import DeviceCase

pytestmark = pytest.mark.gpu


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _cfg(**kw):
    base = dict(name="a", batch=6, num_q_heads=8, num_kv_heads=4, head_dim=128, sys_len=150,
                ctx_lo=1, ctx_hi=200, block_size=16, q_lo=1, q_hi=40)
    base.update(kw)
    return W.AttnConfig(**base)


def _expected_append(case, k_new, v_new, prefill):
    """Alg. 1's cache write as the oracle performs it."""
    return oracle.cache_append(case.k_cache, case.v_cache, case.block_tables, case.context_lens,
                               k_new, v_new, case.cu_seqlens_q if prefill else None)


@pytest.mark.parametrize("cfg,seed,prefill", [
    (_cfg(), 301, False),
    (_cfg(head_dim=64, block_size=8, num_kv_heads=2), 302, False),
    (_cfg(), 303, True),
    (_cfg(block_size=1, q_hi=9, ctx_hi=30), 304, True),
])
def test_append_is_byte_exact_and_feeds_attention(cfg, seed, prefill):
    case = W.make_case(cfg, seed, prefill=prefill, extra_context=prefill, poison_tails=False)
    _say("%s seed=%d prefill=%s" % (cfg, seed, prefill))
    rng = np.random.Generator(np.random.PCG64(seed + 1000))
    total_q = int(case.cu_seqlens_q[-1])
    Hkv, d = cfg.num_kv_heads, cfg.head_dim
    # the new rows arrive as a slice of a wider (fused projection) tensor
    wide = W.bf16_round(rng.standard_normal((total_q, 3 * Hkv, d), dtype=np.float32))
    k_new, v_new = wide[:, Hkv:2 * Hkv], wide[:, 2 * Hkv:]
    want_k, want_v = _expected_append(case, k_new, v_new, prefill)

    dc = DeviceCase(case)
    wide_d = torch.from_numpy(wide).to(dc.dev).to(torch.bfloat16)
    kd, vd = wide_d[:, Hkv:2 * Hkv], wide_d[:, 2 * Hkv:]
    assert kd.stride(0) == 3 * Hkv * d
    out = torch.empty_like(dc.q)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))
    ra.relay_attn_cache_append(p, kd, vd, dc.cu_seqlens_q if prefill else None, total_q,
                               dc.k_cache, dc.v_cache, dc.block_tables, dc.context_lens)
    torch.cuda.synchronize()
    got_k = dc.k_cache.float().cpu().numpy()
    got_v = dc.v_cache.float().cpu().numpy()
    assert np.array_equal(got_k, want_k) and np.array_equal(got_v, want_v)

    # attention over the appended cache equals the oracle on the expected cache
    appended = replace(case, k_cache=want_k, v_cache=want_v)
    if prefill:
        got, _ = dc.prefill()
        want, _, _ = oracle.prefill_attention(appended.q, appended.cu_seqlens_q, appended.k_sys,
                                              appended.v_sys, want_k, want_v, appended.block_tables,
                                              appended.context_lens, appended.scale)
    else:
        got, _ = dc.decode()
        want, _, _ = oracle.decode_attention(appended.q, appended.k_sys, appended.v_sys, want_k,
                                             want_v, appended.block_tables, appended.context_lens,
                                             appended.scale)
    assert np.abs(got - want).max() <= 2e-3


@pytest.mark.parametrize("head_major", [False, True, "padded"])
def test_system_fill_is_byte_exact(head_major):
    """relay_attn_system_fill writes a slice of a fused projection output into positions
    first .. first+n-1 of the system cache (token-major, head-major, or token-major with the
    padded rows relay_attn_system_cache_layout recommends) and nothing else."""
    s, Hkv, d, first, n = 70, 4, 128, 9, 50
    _say("system fill layout=%s" % {False: "token-major", True: "head-major"}.get(head_major, head_major))
    rng = np.random.Generator(np.random.PCG64(77))
    wide = W.bf16_round(rng.standard_normal((n, 3 * Hkv, d), dtype=np.float32))
    old_k = W.bf16_round(rng.standard_normal((s, Hkv, d), dtype=np.float32))
    old_v = W.bf16_round(rng.standard_normal((s, Hkv, d), dtype=np.float32))
    want_k, want_v = old_k.copy(), old_v.copy()
    want_k[first:first + n] = wide[:, Hkv:2 * Hkv]
    want_v[first:first + n] = wide[:, 2 * Hkv:]

    dev = torch.device("cuda:0")
    to = lambda a: torch.from_numpy(a).to(dev).to(torch.bfloat16)
    wide_d = to(wide)
    pad_bufs = []
    if head_major == "padded":
        nbytes = ra.relay_attn_system_cache_layout(s, Hkv, d)[2]
        for old in (old_k, old_v):
            buf = torch.full((nbytes // 2,), -7.0, dtype=torch.bfloat16, device=dev)
            view = ra.system_cache_view(buf, s, Hkv, d)
            view.copy_(to(old))
            pad_bufs.append((buf, view))
        ks, vs = pad_bufs[0][1], pad_bufs[1][1]
    elif head_major:
        ks = to(old_k.transpose(1, 0, 2).copy()).transpose(0, 1)     # [s, Hkv, d] view of [Hkv, s, d]
        vs = to(old_v.transpose(1, 0, 2).copy()).transpose(0, 1)
    else:
        ks, vs = to(old_k), to(old_v)
    p = ra.RAParams()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = 1, Hkv, Hkv, d
    p.sys_len, p.block_size, p.num_blocks, p.max_blocks_per_seq = s, 16, 1, 1
    p.softmax_scale = 1.0
    p.q_stride_token, p.q_stride_head = Hkv * d, d
    p.o_stride_token, p.o_stride_head = Hkv * d, d
    p.sys_stride_token, p.sys_stride_head = ks.stride(0), ks.stride(1)
    ra.relay_attn_system_fill(p, wide_d[:, Hkv:2 * Hkv], wide_d[:, 2 * Hkv:], first, ks, vs)
    torch.cuda.synchronize()
    assert np.array_equal(ks.float().cpu().numpy(), want_k)
    assert np.array_equal(vs.float().cpu().numpy(), want_v)
    for buf, view in pad_bufs:                               # the padding between the rows is untouched
        rows = buf[: (s - 1) * view.stride(0) + Hkv * d].float().cpu().numpy()
        full = np.full(s * view.stride(0), -7.0, np.float32)
        full[: rows.size] = rows
        assert (full.reshape(s, view.stride(0))[:, Hkv * d:] == -7.0).all()
    with pytest.raises(ra.RelayAttnError):
        ra.relay_attn_system_fill(p, wide_d[:, :Hkv], wide_d[:, :Hkv], s - n + 1, ks, vs)
