"""relay_attn_debug_validate on the GPU: a clean case passes, planted out-of-range entries are
counted, and entries the attention kernels never read are not checked."""
import sys

import numpy as np
import pytest
import torch

import paper_2402_14808_amd as ra
import workloads as W
from gpu_util import DeviceCase

pytestmark = pytest.mark.gpu
OK, INVALID = ra.binding.RA_OK, ra.binding.RA_ERR_INVALID_ARG


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _setup(seed, **kw):
    base = dict(name="v", batch=9, num_q_heads=4, num_kv_heads=2, head_dim=64, sys_len=40,
                ctx_lo=1, ctx_hi=300, block_size=16)
    base.update(kw)
    case = W.make_case(W.AttnConfig(**base), seed)
    dc = DeviceCase(case)
    out, _ = dc._outputs(True)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=case.cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))
    ws = torch.empty(256, dtype=torch.uint8, device=dc.dev)
    return case, dc, p, ws


def test_clean_case_passes_and_poisoned_unused_slots_are_ignored():
    case, dc, p, ws = _setup(501)
    _say("clean case, seed 501")
    # the generator already puts a poison index in every unused table slot
    assert (case.block_tables == W.POISON_BLOCK).any()
    st, rep = ra.relay_attn_debug_validate(p, dc.block_tables, dc.context_lens, ws)
    assert st == OK
    assert (rep.bad_context_lens, rep.bad_block_ids, rep.bad_query_lens, rep.first_bad_request) == (0, 0, 0, -1)


def test_planted_violations_are_counted():
    case, dc, p, ws = _setup(502)
    _say("planted violations, seed 502")
    bt = dc.block_tables.clone()
    cl = dc.context_lens.clone()
    used = -(-case.context_lens // case.cfg.block_size)
    # request 5: two used slots out of range; request 2: negative length; request 7: too long
    bt[5, 0] = p.num_blocks
    bt[5, int(used[5]) - 1] = -1
    cl[2] = -3
    cl[7] = p.max_context_len + 1
    st, rep = ra.relay_attn_debug_validate(p, bt, cl, ws)
    assert st == INVALID
    assert rep.bad_block_ids == (2 if used[5] > 1 else 1)
    assert rep.bad_context_lens == 2 and rep.bad_query_lens == 0 and rep.first_bad_request == 2
    # the same workspace is reusable: a clean run afterwards reports nothing
    st, rep = ra.relay_attn_debug_validate(p, dc.block_tables, dc.context_lens, ws)
    assert st == OK and rep.first_bad_request == -1


def test_query_lengths_of_a_prompt_phase_batch():
    case, dc, p, ws = _setup(503, batch=4, ctx_lo=20, ctx_hi=100)
    _say("cu_seqlens_q checks, seed 503")
    lens = case.context_lens
    m = np.minimum(lens, [3, 20, 1, 7]).astype(np.int32)
    cu = np.zeros(5, np.int32)
    cu[1:] = np.cumsum(m)
    total = int(cu[-1])
    dev = dc.dev
    st, rep = ra.relay_attn_debug_validate(p, dc.block_tables, dc.context_lens, ws,
                                           cu_seqlens_q=torch.from_numpy(cu).to(dev), total_q=total)
    assert st == OK
    bad = cu.copy()
    bad[2] = bad[1] - 1                               # decreasing: requests 1 and 2 both see it
    st, rep = ra.relay_attn_debug_validate(p, dc.block_tables, dc.context_lens, ws,
                                           cu_seqlens_q=torch.from_numpy(bad).to(dev), total_q=total)
    assert st == INVALID and rep.bad_query_lens >= 1 and rep.first_bad_request == 1
    more = cu.copy()
    more[1:] += int(lens[0])                          # request 0 claims more new tokens than context
    st, rep = ra.relay_attn_debug_validate(p, dc.block_tables, dc.context_lens, ws,
                                           cu_seqlens_q=torch.from_numpy(more).to(dev),
                                           total_q=int(more[-1]))
    assert st == INVALID and rep.bad_query_lens == 1 and rep.first_bad_request == 0


def test_debug_timeline_records_every_wavefront_and_leaves_the_result_alone():
    """relay_attn_debug_timeline: the decode step's result is bitwise relay_attn_decode's, every
    wavefront of the partial-attention launch has a begin <= end from one clock, and entries
    beyond the launch stay untouched.  The same for the prompt phase."""
    case = W.make_case(W.AttnConfig("tl", 20, 8, 4, 128, 700, 1, 400, 16), 520)
    dc = DeviceCase(case)
    _say("timeline, decode, seed 520")
    want, wlse = dc.decode()
    plan = dc.last_plan
    n_waves = 4 * plan.num_sys_workgroups + plan.num_ctx_wavefronts
    out, lse = dc._outputs(True)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=case.cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))
    ws = dc._workspace(p, case.cfg.batch)
    tl = torch.zeros(2 * (n_waves + 8), dtype=torch.int64, device=dc.dev)
    ra.relay_attn_debug_timeline(p, dc.q, None, case.cfg.batch, 1, dc.k_sys, dc.v_sys, dc.k_cache, dc.v_cache,
                                 dc.block_tables, dc.context_lens, out, lse, ws, tl)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), want) and np.array_equal(lse.cpu().numpy(), wlse)
    t = tl.cpu().numpy().reshape(-1, 2)
    assert (t[:n_waves, 0] > 0).all() and (t[:n_waves, 1] >= t[:n_waves, 0]).all()
    assert (t[n_waves:] == 0).all()
    span_us = (t[:n_waves, 1].max() - t[:n_waves, 0].min()) / 100.0
    _say("%d wavefronts, launch span %.1f us" % (n_waves, span_us))
    assert 0 < span_us < 1000

    pcase = W.make_case(W.AttnConfig("tlp", 3, 4, 4, 128, 300, 0, 100, 16, q_lo=40, q_hi=90), 521, prefill=True,
                        extra_context=True)
    pdc = DeviceCase(pcase)
    _say("timeline, prompt phase, seed 521")
    pwant, pwlse = pdc.prefill()
    total_q, max_q = int(pcase.cu_seqlens_q[-1]), int(np.diff(pcase.cu_seqlens_q).max())
    out, lse = pdc._outputs(True)
    p = ra.make_params(pdc.q, out, pdc.k_sys, pdc.k_cache, pdc.block_tables, batch=3, softmax_scale=pcase.scale,
                       max_context_len=int(pcase.context_lens.max()))
    ws = pdc._workspace(p, total_q)
    tl = torch.zeros(2 * 4096, dtype=torch.int64, device=pdc.dev)
    ra.relay_attn_debug_timeline(p, pdc.q, pdc.cu_seqlens_q, total_q, max_q, pdc.k_sys, pdc.v_sys, pdc.k_cache,
                                 pdc.v_cache, pdc.block_tables, pdc.context_lens, out, lse, ws, tl)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), pwant) and np.array_equal(lse.cpu().numpy(), pwlse)
    t = tl.cpu().numpy().reshape(-1, 2)
    n = int((t[:, 0] > 0).sum())
    assert n > 0 and n % 4 == 0 and (t[:n, 1] >= t[:n, 0]).all() and (t[n:] == 0).all()
