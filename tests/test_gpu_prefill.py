"""GPU parity tests of relay_attn_prefill (prompt phase) against the CPU oracle."""
import sys

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
    got, lse = DeviceCase(case).prefill(**tuning)
    want, wlse = _oracle(case)
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e lse err %.3e" % (err, lerr))
    assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL


def test_prefill_row_equals_decode_of_truncated_context():
    cfg = _cfg(batch=2, q_lo=5, q_hi=9)
    case = W.make_case(cfg, 207, prefill=True, extra_context=True)
    got, _ = DeviceCase(case).prefill()
    want, _ = _oracle(case)
    assert np.abs(got - want).max() <= TOL


def test_llama13b_prefill_sampled_rows():
    case = W.make_case(W.LLAMA13B_PREFILL, 5000, prefill=True)
    _say("%s total_q=%d" % (case.cfg, case.cu_seqlens_q[-1]))
    rng = np.random.Generator(np.random.PCG64(3))
    n_tok, Hq, _ = case.q.shape
    rows = np.stack([rng.integers(0, n_tok, 96), rng.integers(0, Hq, 96)], axis=1).astype(np.int32)
    got, lse = DeviceCase(case).prefill()
    want, wlse = _oracle(case, rows=rows)
    err = np.abs(got[rows[:, 0], rows[:, 1]] - want).max()
    _say("sampled rows max-abs err %.3e" % err)
    assert np.isfinite(got).all() and err <= TOL
    assert np.abs(lse[rows[:, 0], rows[:, 1]] - wlse).max() <= LSE_TOL
