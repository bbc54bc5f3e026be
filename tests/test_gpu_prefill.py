"""GPU parity tests of relay_attn_prefill (prompt phase) against the CPU oracle."""
import sys
from dataclasses import replace

import numpy as np
import pytest

import oracle
import workloads as W
from gpu_util import DeviceCase

pytestmark = pytest.mark.gpu
TOL = 2e-3
LSE_TOL = 1e-3


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _oracle(case, rows=None):
    out, lse, _ = oracle.prefill_attention(case.q, case.cu_seqlens_q, case.k_sys, case.v_sys,
                                           case.k_cache, case.v_cache, case.block_tables,
                                           case.context_lens, case.scale, rows=rows)
    return out, lse


def _cfg(**kw):
    base = dict(name="p", batch=3, num_q_heads=4, num_kv_heads=4, head_dim=128, sys_len=200,
                ctx_lo=0, ctx_hi=150, block_size=16, q_lo=1, q_hi=70)
    base.update(kw)
    return W.AttnConfig(**base)


@pytest.mark.parametrize("cfg,seed,extra,tuning", [
    (_cfg(), 201, False, {}),
    (_cfg(), 202, True, {}),
    (_cfg(head_dim=64, num_q_heads=8, num_kv_heads=2, sys_len=95), 203, True, {}),
    (_cfg(sys_len=0, q_hi=130), 204, True, {}),
    (_cfg(batch=5, q_lo=1, q_hi=3, sys_len=1030), 205, False, {"sys_chunk_tokens": 256}),
    (_cfg(q_lo=200, q_hi=300, ctx_hi=300, num_q_heads=2, num_kv_heads=1), 206, True,
     {"ctx_part_tokens": 128}),
])
def test_prefill_matches_oracle_small(cfg, seed, extra, tuning):
    case = W.make_case(cfg, seed, prefill=True, extra_context=extra)
    _say("%s seed=%d m=%s c=%s" % (cfg, seed, np.diff(case.cu_seqlens_q), case.context_lens))
    want, wlse = _oracle(case)
    for layout in ("dense", "padded"):                   # of the system cache
        got, lse = DeviceCase(case, sys_layout=layout).prefill(**tuning)
        err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
        _say("system cache %s: max-abs err %.3e lse err %.3e" % (layout, err, lerr))
        assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL


def test_prefill_row_equals_decode_of_truncated_context():
    """Row j of a prompt-phase call is the decode step of that token over the context truncated
    after it (bottom-right causal alignment): both run on the GPU here, and both are compared
    with the oracle."""
    cfg = _cfg(batch=2, q_lo=5, q_hi=9)
    case = W.make_case(cfg, 207, prefill=True, extra_context=True)
    got, lse = DeviceCase(case).prefill()
    want, _ = _oracle(case)
    assert np.abs(got - want).max() <= TOL
    cu = case.cu_seqlens_q
    for i in range(cfg.batch):
        m, c = int(cu[i + 1] - cu[i]), int(case.context_lens[i])
        for j in range(m):
            one = replace(case, cfg=replace(cfg, batch=1), q=case.q[cu[i] + j:cu[i] + j + 1],
                          block_tables=case.block_tables[i:i + 1],
                          context_lens=np.array([c - m + j + 1], np.int32),
                          cu_seqlens_q=np.array([0, 1], np.int32))
            dec, dlse = DeviceCase(one).decode()
            np.testing.assert_allclose(dec[0], got[cu[i] + j], atol=2e-5, rtol=0)
            np.testing.assert_allclose(dlse[0], lse[cu[i] + j], atol=2e-5, rtol=0)


def _edge_rows(case, G, n_random, seed):
    """(token, head) rows that a random sample can miss: the first and last new token of every
    request and the tokens on both sides of every boundary between 128-row blocks (a work item of
    the kernel owns 128 stacked rows: of a request in the split form, of the whole packed batch in
    the one-launch form), all heads; plus random rows."""
    cu = case.cu_seqlens_q
    Hq = case.q.shape[1]
    tokens = set()
    for i in range(len(cu) - 1):
        a, b = int(cu[i]), int(cu[i + 1])
        tokens.update((a, b - 1))
        for edge in range(128, (b - a) * G, 128):       # stacked row = token * G + head-in-group
            t = edge // G
            tokens.update(a + x for x in (t - 1, t) if 0 <= x < b - a)
    # (the one-launch form cuts the packed rows of the whole batch into blocks of 128 instead)
    for edge in range(128, int(cu[-1]) * G, 128):
        tokens.update(x for x in (edge // G - 1, edge // G) if 0 <= x < int(cu[-1]))
    rows = [(t, h) for t in sorted(tokens) for h in range(Hq)]
    rng = np.random.Generator(np.random.PCG64(seed))
    rows += list(zip(rng.integers(0, int(cu[-1]), n_random).tolist(), rng.integers(0, Hq, n_random).tolist()))
    return np.array(rows, dtype=np.int32)


def test_llama13b_prefill_edge_and_sampled_rows():
    case = W.make_case(W.LLAMA13B_PREFILL, 5000, prefill=True)
    rows = _edge_rows(case, 1, 512, 3)
    _say("%s total_q=%d, %d rows checked" % (case.cfg, case.cu_seqlens_q[-1], len(rows)))
    got, lse = DeviceCase(case, sys_layout="padded").prefill()
    want, wlse = _oracle(case, rows=rows)
    err = np.abs(got[rows[:, 0], rows[:, 1]] - want).max()
    _say("max-abs err %.3e" % err)
    assert np.isfinite(got).all() and err <= TOL
    assert np.abs(lse[rows[:, 0], rows[:, 1]] - wlse).max() <= LSE_TOL


def test_llama13b_prefill_bf16_output_and_cached_context():
    """The same shape with an already cached part in front of the new tokens (c_i > m_i) and the
    bf16 output the benchmark times."""
    cfg = replace(W.LLAMA13B_PREFILL, batch=6, ctx_lo=1, ctx_hi=700)
    case = W.make_case(cfg, 5001, prefill=True, extra_context=True)
    rows = _edge_rows(case, 1, 256, 4)
    _say("%s total_q=%d, %d rows checked" % (cfg, case.cu_seqlens_q[-1], len(rows)))
    got, lse = DeviceCase(case, sys_layout="padded").prefill(fp32_out=False)
    want, wlse = _oracle(case, rows=rows)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    assert np.isfinite(got).all()
    assert (np.abs(got[rows[:, 0], rows[:, 1]] - want) <= np.maximum(TOL, ulp)).all()
    assert np.abs(lse[rows[:, 0], rows[:, 1]] - wlse).max() <= LSE_TOL


@pytest.mark.parametrize("cfg,seed,factor,bound", [
    (_cfg(), 210, 16, 0),
    (_cfg(q_lo=100, q_hi=300, ctx_hi=300, num_q_heads=8, num_kv_heads=2), 211, 8, 0),
    (_cfg(batch=5, sys_len=0, q_hi=130, block_size=8), 212, 8, 1024),
])
def test_prefill_length_bound_far_above_the_real_lengths(cfg, seed, factor, bound):
    case = W.make_case(cfg, seed, prefill=True, extra_context=True)
    wide = np.full((case.block_tables.shape[0], case.block_tables.shape[1] * factor),
                   W.POISON_BLOCK, dtype=np.int32)
    wide[:, :case.block_tables.shape[1]] = case.block_tables
    case = replace(case, block_tables=wide)
    _say("%s seed=%d table width %d bound %d" % (cfg, seed, wide.shape[1], bound))
    got, lse = DeviceCase(case).prefill(max_context_len=bound)
    want, wlse = _oracle(case)
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e lse err %.3e" % (err, lerr))
    assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL


SINGLE_LAUNCH = [
    # blocks of 128 rows that span two to four requests, cached context in front of the new tokens
    (_cfg(batch=5, q_lo=20, q_hi=90, sys_len=300), 230, True),
    # G = 4 (32 tokens per block), head_dim 64
    (_cfg(batch=4, q_lo=40, q_hi=200, num_q_heads=8, num_kv_heads=2, head_dim=64, sys_len=95), 231, True),
    # no system prompt
    (_cfg(batch=3, q_lo=64, q_hi=130, sys_len=0), 232, True),
    # block size 1: a context part holds 256 positions, so longer contexts take several parts
    (_cfg(batch=2, q_lo=40, q_hi=70, ctx_lo=500, ctx_hi=700, block_size=1, num_q_heads=2, num_kv_heads=1), 233, True),
    # contexts that are exactly the new tokens (c_i = m_i)
    (_cfg(batch=3, q_lo=100, q_hi=300, sys_len=400, num_q_heads=2, num_kv_heads=2), 234, False),
    # one token of one request between long requests
    (_cfg(batch=6, q_lo=60, q_hi=61, sys_len=129), 235, True),
    # more than 64 requests (the block's first request is searched 64 requests at a time), G = 3
    (_cfg(batch=70, q_lo=32, q_hi=40, ctx_hi=40, sys_len=77, num_q_heads=3, num_kv_heads=1, head_dim=64), 236, True),
]


@pytest.mark.parametrize("cfg,seed,extra", SINGLE_LAUNCH, ids=["w%d" % c[1] for c in SINGLE_LAUNCH])
def test_prefill_single_launch_and_split_forms(cfg, seed, extra):
    """With many new tokens per request and an untuned decomposition the prompt phase is ONE launch
    whose items carry their rows through system prompt and contexts and write the output (the
    workspace stays untouched); a hand-set context part keeps the split form (system items, context
    items, fusion launch).  Both against the oracle."""
    case = W.make_case(cfg, seed, prefill=True, extra_context=extra)
    if seed == 235:                                  # squeeze request 2 down to a single new token
        m = np.diff(case.cu_seqlens_q).copy()
        keep = np.concatenate([np.arange(case.cu_seqlens_q[i], case.cu_seqlens_q[i] + (1 if i == 2 else m[i]))
                               for i in range(cfg.batch)])
        lens = case.context_lens.copy()
        lens[2] -= m[2] - 1
        m[2] = 1
        cu = np.zeros(cfg.batch + 1, np.int32)
        cu[1:] = np.cumsum(m)
        case = replace(case, q=case.q[keep], cu_seqlens_q=cu, context_lens=lens)
    total_q = int(case.cu_seqlens_q[-1])
    assert total_q >= 32 * cfg.batch
    _say("%s seed=%d m=%s c=%s" % (cfg, seed, np.diff(case.cu_seqlens_q), case.context_lens))
    want, wlse = _oracle(case)
    dc = DeviceCase(case, sys_layout="padded")
    got, lse = dc.prefill()
    assert bool((dc.last_workspace == 0xFF).all()), "the single-launch form was expected (workspace untouched)"
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("single launch: max-abs err %.3e lse err %.3e" % (err, lerr))
    assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL
    b16, _ = dc.prefill(fp32_out=False)
    assert np.array_equal(W.bf16_round(got), b16)
    got2, lse2 = dc.prefill(ctx_part_tokens=256 if cfg.block_size == 1 else 4096)
    assert not bool((dc.last_workspace == 0xFF).all()), "the split form was expected (partials in the workspace)"
    err2, lerr2 = np.abs(got2 - want).max(), np.abs(lse2 - wlse).max()
    _say("split form:    max-abs err %.3e lse err %.3e" % (err2, lerr2))
    assert err2 <= TOL and lerr2 <= LSE_TOL

