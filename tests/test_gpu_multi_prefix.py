"""GPU parity of relay_attn_decode_multi, relay_attn_decode_grouped and relay_attn_prefill_multi
(several shared system prompts in one batch, App. D) against the CPU oracle, which is simply run
once per group with that group's system prompt."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2402_14808_amd as ra
import workloads as W
from gpu_util import DeviceCase, _bf16

pytestmark = pytest.mark.gpu
TOL = 2e-3
LSE_TOL = 1e-3


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _cfg(**kw):
    base = dict(name="mp", batch=12, num_q_heads=4, num_kv_heads=4, head_dim=128, sys_len=0,
                ctx_lo=1, ctx_hi=300, block_size=16)
    base.update(kw)
    return W.AttnConfig(**base)


def _oracle(case, groups):
    B, Hq, d = case.q.shape
    out = np.zeros((B, Hq, d), np.float32)
    lse = np.zeros((B, Hq), np.float32)
    for first, n, ks, vs in groups:
        sl = slice(first, first + n)
        o, l, _ = oracle.decode_attention(case.q[sl], ks, vs, case.k_cache, case.v_cache,
                                          case.block_tables[sl], case.context_lens[sl], case.scale)
        out[sl], lse[sl] = o, l
    return out, lse


def _run(case, groups, **tuning):
    dc = DeviceCase(case)
    longest = max(g[2].shape[0] for g in groups)
    # all prefixes live in one allocation so that they share strides
    dev_groups, proto = [], None
    for first, n, ks, vs in groups:
        kd = _bf16(ks, dc.dev) if ks.shape[0] else None
        vd = _bf16(vs, dc.dev) if vs.shape[0] else None
        if kd is not None and kd.shape[0] == longest:
            proto = kd
        dev_groups.append((kd, vd, first, n))
    out, lse = dc._outputs(True)
    p = ra.make_params(dc.q, out, proto, dc.k_cache, dc.block_tables, batch=case.cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()),
                       **tuning)
    ws = dc._workspace(p, case.cfg.batch)
    ra.relay_attn_decode_multi(p, dev_groups, dc.q, dc.k_cache, dc.v_cache, dc.block_tables,
                               dc.context_lens, out, lse, ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


CASES = [
    (_cfg(), 301, (5, 7), (300, 300), {}),
    (_cfg(), 302, (5, 7), (130, 700), {}),                               # unequal lengths
    (_cfg(), 303, (3, 4, 5), (1, 257, 64), {"sys_chunk_tokens": 128}),    # unequal chunk counts
    (_cfg(), 304, (6, 6), (0, 200), {}),                                 # a group without prefix
    (_cfg(batch=40, num_q_heads=8, num_kv_heads=2), 305, (1, 30, 9), (500, 90, 1100),
     {"sys_chunk_tokens": 256}),                                         # G=4, several row tiles
    (_cfg(batch=16, head_dim=64, ctx_lo=0, ctx_hi=40), 306, (2,) * 8, tuple(range(40, 360, 40)), {}),
    (_cfg(batch=9), 307, (9,), (400,), {}),                               # one group == decode
    (W.AttnConfig("llama30b_2apps", 32, 52, 52, 128, 0, 128, 128), 308, (16, 16), (2048, 1024), {}),
]


@pytest.mark.parametrize("cfg,seed,sizes,lens,tuning", CASES,
                         ids=["c%d" % c[1] for c in CASES])
def test_multi_prefix_matches_oracle(cfg, seed, sizes, lens, tuning):
    case = W.make_case(cfg, seed)
    groups = W.make_prefix_groups(case, seed + 1000, sizes, lens)
    _say("%s seed=%d groups=%s lens=%s tuning=%s" % (cfg, seed, sizes, lens, tuning))
    got, lse = _run(case, groups, **tuning)
    want, wlse = _oracle(case, groups)
    assert np.isfinite(got).all()
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert err <= TOL and lerr <= LSE_TOL


def test_one_group_is_bitwise_relay_attn_decode():
    case = W.make_case(_cfg(batch=9, sys_len=400), 309)
    _say("one group vs relay_attn_decode, seed 309")
    a, la = DeviceCase(case).decode()
    b, lb = _run(case, [(0, 9, case.k_sys, case.v_sys)])
    assert np.array_equal(a, b) and np.array_equal(la, lb)


@pytest.mark.parametrize("cfg,seed,n_apps,lens", [
    (_cfg(batch=23), 320, 3, (300, 70, 520)),
    (_cfg(batch=40, num_q_heads=8, num_kv_heads=2), 321, 12, tuple(64 * (i % 5) + 33 for i in range(12))),
    (_cfg(batch=64, head_dim=64, ctx_lo=0, ctx_hi=60), 322, 32, tuple(40 + 9 * i for i in range(32))),
    (_cfg(batch=10), 323, 4, (0, 128, 0, 257)),            # applications without a prompt / without requests
])
def test_requests_of_an_application_anywhere_in_the_batch(cfg, seed, n_apps, lens):
    """relay_attn_decode_grouped: sys_id per request in any order, up to 32 applications; the oracle
    is run per request group with that application's prompt."""
    case = W.make_case(cfg, seed)
    rng = np.random.Generator(np.random.PCG64(seed + 7))
    sys_id = rng.integers(0, n_apps, cfg.batch)
    if seed == 323:
        sys_id[sys_id == 2] = 1                            # application 2 has no request
    shape = lambda s: (int(s), cfg.num_kv_heads, cfg.head_dim)
    apps = [(W.bf16_round(rng.standard_normal(shape(s), dtype=np.float32)),
             W.bf16_round(rng.standard_normal(shape(s), dtype=np.float32))) for s in lens]
    order, counts = ra.relay_attn_group_requests(sys_id.tolist(), n_apps)
    _say("%s seed=%d sys_id=%s counts=%s" % (cfg, seed, sys_id.tolist(), counts))
    assert sorted(order) == list(range(cfg.batch))
    dc = DeviceCase(case)
    longest = max(lens[i] for i in range(n_apps) if counts[i] > 0)
    dev_apps, proto = [], None
    for (ks, vs), n in zip(apps, counts):
        kd = _bf16(ks, dc.dev) if ks.shape[0] else None
        vd = _bf16(vs, dc.dev) if vs.shape[0] else None
        if kd is not None and kd.shape[0] == longest and n > 0:
            proto = kd
        dev_apps.append((kd, vd, n))
    out, lse = dc._outputs(True)
    p = ra.make_params(dc.q, out, proto, dc.k_cache, dc.block_tables, batch=cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))
    ws = dc._workspace(p, cfg.batch)
    sid_d = torch.tensor(sys_id.tolist(), dtype=torch.int32, device=dc.dev)
    ord_d = torch.tensor(order, dtype=torch.int32, device=dc.dev)
    ra.relay_attn_decode_grouped(p, dev_apps, sid_d, ord_d, dc.q, dc.k_cache, dc.v_cache,
                                 dc.block_tables, dc.context_lens, out, lse, ws)
    torch.cuda.synchronize()
    got, glse = out.cpu().numpy(), lse.cpu().numpy()
    assert np.isfinite(got).all()
    for a in range(n_apps):
        idx = np.nonzero(sys_id == a)[0]
        if len(idx) == 0:
            continue
        o, l, _ = oracle.decode_attention(case.q[idx], apps[a][0], apps[a][1], case.k_cache, case.v_cache,
                                          case.block_tables[idx], case.context_lens[idx], case.scale)
        assert np.abs(got[idx] - o).max() <= TOL and np.abs(glse[idx] - l).max() <= LSE_TOL


def _prefill_oracle(case, groups):
    """The prompt-phase oracle run once per request group with that group's system prompt; the
    packed token offsets are re-based to the group's first token."""
    cu = case.cu_seqlens_q.astype(np.int64)
    T, Hq, d = case.q.shape
    out = np.zeros((T, Hq, d), np.float32)
    lse = np.zeros((T, Hq), np.float32)
    for first, n, ks, vs in groups:
        t0, t1 = int(cu[first]), int(cu[first + n])
        o, l, _ = oracle.prefill_attention(case.q[t0:t1], cu[first:first + n + 1] - t0, ks, vs,
                                           case.k_cache, case.v_cache,
                                           case.block_tables[first:first + n],
                                           case.context_lens[first:first + n], case.scale)
        out[t0:t1], lse[t0:t1] = o, l
    return out, lse


def _run_prefill(case, groups, fp32_out=True, **tuning):
    dc = DeviceCase(case)
    cu = case.cu_seqlens_q
    longest = max(g[2].shape[0] for g in groups)
    dev_groups, toks, proto = [], [], None
    for first, n, ks, vs in groups:
        kd = _bf16(ks, dc.dev) if ks.shape[0] else None
        vd = _bf16(vs, dc.dev) if vs.shape[0] else None
        if kd is not None and kd.shape[0] == longest:
            proto = kd
        dev_groups.append((kd, vd, first, n))
        toks.append(int(cu[first + n] - cu[first]))
    out, lse = dc._outputs(fp32_out)
    total_q, max_q = int(cu[-1]), int(np.diff(cu).max())
    p = ra.make_params(dc.q, out, proto, dc.k_cache, dc.block_tables, batch=case.cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()),
                       **tuning)
    ws = dc._workspace(p, total_q)
    ra.relay_attn_prefill_multi(p, dev_groups, toks, dc.q, dc.cu_seqlens_q, total_q, max_q,
                                dc.k_cache, dc.v_cache, dc.block_tables, dc.context_lens, out, lse, ws)
    torch.cuda.synchronize()
    _run_prefill.last_workspace = ws
    return out.float().cpu().numpy(), lse.cpu().numpy()


def _pcfg(**kw):
    base = dict(name="mpp", batch=6, num_q_heads=4, num_kv_heads=4, head_dim=128, sys_len=0,
                ctx_lo=0, ctx_hi=150, block_size=16, q_lo=1, q_hi=70)
    base.update(kw)
    return W.AttnConfig(**base)


PREFILL_CASES = [
    (_pcfg(), 340, (3, 3), (200, 200), {}),
    (_pcfg(), 341, (2, 4), (70, 530), {}),                                # unequal lengths
    (_pcfg(), 342, (1, 2, 3), (1, 257, 64), {"sys_chunk_tokens": 128}),    # unequal chunk counts
    (_pcfg(), 343, (3, 3), (0, 300), {}),                                 # a group without prefix
    (_pcfg(), 344, (3, 3), (300, 0), {}),
    (_pcfg(batch=8, num_q_heads=8, num_kv_heads=2, head_dim=64, q_hi=140), 345, (1, 5, 2),
     (500, 90, 1100), {"sys_chunk_tokens": 256}),                         # G=4, several row blocks
    (_pcfg(batch=16, q_lo=1, q_hi=5), 346, (2,) * 8, tuple(range(40, 360, 40)), {}),
    (_pcfg(batch=4, q_lo=150, q_hi=300, ctx_hi=300, num_q_heads=2, num_kv_heads=1), 347, (1, 3),
     (333, 129), {"ctx_part_tokens": 128}),
]


@pytest.mark.parametrize("cfg,seed,sizes,lens,tuning", PREFILL_CASES,
                         ids=["p%d" % c[1] for c in PREFILL_CASES])
def test_multi_prefix_prefill_matches_oracle(cfg, seed, sizes, lens, tuning):
    """relay_attn_prefill_multi: consecutive request groups, each with a system prompt of its
    own (App. D), in the prompt phase."""
    case = W.make_case(cfg, seed, prefill=True, extra_context=True)
    groups = W.make_prefix_groups(case, seed + 1000, sizes, lens)
    _say("%s seed=%d groups=%s lens=%s m=%s tuning=%s" % (cfg, seed, sizes, lens,
                                                        np.diff(case.cu_seqlens_q), tuning))
    got, lse = _run_prefill(case, groups, **tuning)
    want, wlse = _prefill_oracle(case, groups)
    assert np.isfinite(got).all()
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert err <= TOL and lerr <= LSE_TOL


def test_one_group_prefill_is_bitwise_relay_attn_prefill():
    cfg = _pcfg(batch=3, sys_len=200)
    case = W.make_case(cfg, 348, prefill=True, extra_context=True)
    _say("one group vs relay_attn_prefill, seed 348")
    a, la = DeviceCase(case).prefill()
    b, lb = _run_prefill(case, [(0, 3, case.k_sys, case.v_sys)])
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_multi_prefix_prefill_bf16_out():
    case = W.make_case(_pcfg(), 349, prefill=True, extra_context=True)
    groups = W.make_prefix_groups(case, 1349, (4, 2), (130, 260))
    _say("bf16 outputs, seed 349")
    got, lse = _run_prefill(case, groups, fp32_out=False)
    want, wlse = _prefill_oracle(case, groups)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)   # one bf16 step of the value
    assert (np.abs(got - want) <= np.maximum(TOL, ulp)).all() and np.abs(lse - wlse).max() <= LSE_TOL


@pytest.mark.parametrize("cfg,seed,sizes,lens", [
    (_pcfg(q_lo=40, q_hi=120), 350, (2, 4), (300, 470)),
    (_pcfg(q_lo=40, q_hi=120, num_q_heads=8, num_kv_heads=2, head_dim=64), 351, (1, 2, 3), (0, 257, 64)),
    (_pcfg(batch=4, q_lo=100, q_hi=200), 352, (3, 1), (129, 0)),
])
def test_multi_prefix_prefill_in_one_launch(cfg, seed, sizes, lens):
    """Many new tokens per request and one-chunk prompts: the one-launch form of the prompt phase,
    with every group's items attending to that group's prefix (the workspace stays untouched)."""
    case = W.make_case(cfg, seed, prefill=True, extra_context=True)
    groups = W.make_prefix_groups(case, seed + 1000, sizes, lens)
    assert int(case.cu_seqlens_q[-1]) >= 32 * cfg.batch
    _say("%s seed=%d groups=%s lens=%s m=%s" % (cfg, seed, sizes, lens, np.diff(case.cu_seqlens_q)))
    got, lse = _run_prefill(case, groups)
    assert bool((_run_prefill.last_workspace == 0xFF).all()), "the one-launch form was expected"
    want, wlse = _prefill_oracle(case, groups)
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL
    got2, lse2 = _run_prefill(case, groups, ctx_part_tokens=4096)      # the split form, same inputs
    assert not bool((_run_prefill.last_workspace == 0xFF).all())
    assert np.abs(got2 - want).max() <= TOL and np.abs(lse2 - wlse).max() <= LSE_TOL
