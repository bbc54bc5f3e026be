"""Seeded random shapes through relay_attn_decode and relay_attn_prefill against the CPU oracle:
batch, head grouping, head_dim, prompt length, context range, block size and the two tuning
knobs are all drawn, so that combinations nobody listed by hand get exercised (plans with many
or few system chunks, many-rows system items, spans over several requests, tiny blocks)."""
import sys

import numpy as np
import pytest

import oracle
import paper_2402_14808_amd as ra
import workloads as W
from gpu_util import DeviceCase

pytestmark = pytest.mark.gpu
TOL = 2e-3
LSE_TOL = 1e-3


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _draw_decode(rng):
    G = int(rng.choice([1, 1, 2, 3, 4, 5, 6, 7, 8]))
    Hkv = int(rng.integers(1, 5))
    wide = rng.random() < 0.3                      # many stacked rows, short contexts
    batch = int(rng.integers(64, 320)) // G + 1 if wide else int(rng.integers(1, 48))
    sys_len = int(rng.choice([0, 1, 31, 32, 33, int(rng.integers(34, 600)), int(rng.integers(600, 3000))]))
    ctx_hi = int(rng.integers(1, 60)) if wide else int(rng.choice([1, 17, 64, 200, 700, 1500]))
    ctx_lo = int(rng.integers(0, ctx_hi + 1))
    cfg = W.AttnConfig("r", batch, G * Hkv, Hkv, int(rng.choice([64, 128])), sys_len, ctx_lo, ctx_hi,
                       block_size=int(rng.choice([1, 2, 4, 8, 16, 16, 32, 64, 128])))
    tuning = {}
    if sys_len > 0 and rng.random() < 0.4:
        tuning["sys_chunk_tokens"] = 32 * int(rng.integers(1, 24))
    if rng.random() < 0.3 and cfg.block_size >= 2:
        tuning["ctx_part_tokens"] = int(rng.choice([128, 256, 512]))
    return cfg, tuning


@pytest.mark.parametrize("seed", range(7000, 7036))
def test_random_decode_shape(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cfg, tuning = _draw_decode(rng)
    case = W.make_case(cfg, seed)
    layout = "padded" if seed % 2 else "dense"           # of the system cache
    _say("decode %s seed=%d tuning=%s system cache %s" % (cfg, seed, tuning, layout))
    dc = DeviceCase(case, sys_layout=layout)
    try:
        got, lse = dc.decode(**tuning)
    except ra.RelayAttnError as e:
        # a fixed span whose block ids cannot fit the per-wavefront table is refused, not truncated
        assert e.status == ra.binding.RA_ERR_UNSUPPORTED
        assert tuning.get("ctx_part_tokens", 0) / cfg.block_size > 255 - 1
        _say("fixed span refused as documented; drawn again without it")
        tuning.pop("ctx_part_tokens")
        got, lse = dc.decode(**tuning)
    pl = dc.last_plan
    _say("plan: %d system workgroups of %d rows, %d chunks of %d; %d context wavefronts, %d slots"
         % (pl.num_sys_workgroups, pl.sys_rows_per_workgroup, pl.num_sys_chunks, pl.sys_chunk_tokens,
            pl.num_ctx_wavefronts, pl.num_ctx_slots))
    want, wlse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache, case.v_cache,
                                            case.block_tables, case.context_lens, case.scale)
    assert np.isfinite(got).all()
    live = np.isfinite(wlse)                       # rows with no key at all: out 0, lse -inf
    assert np.array_equal(np.isfinite(lse), live)
    err = np.abs(got - want).max()
    lerr = np.abs(lse[live] - wlse[live]).max() if live.any() else 0.0
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert err <= TOL and lerr <= LSE_TOL


def _draw_prefill(rng):
    G = int(rng.choice([1, 2, 3, 4, 7]))
    Hkv = int(rng.integers(1, 4))
    q_hi = int(rng.choice([1, 5, 40, 150, 300]))
    q_lo = int(rng.integers(1, q_hi + 1))
    cfg = W.AttnConfig("rp", int(rng.integers(1, 7)), G * Hkv, Hkv, int(rng.choice([64, 128])),
                       int(rng.choice([0, 1, 33, int(rng.integers(34, 1500))])), 0, int(rng.choice([0, 50, 400])),
                       block_size=int(rng.choice([4, 8, 16, 32])), q_lo=q_lo, q_hi=q_hi)
    tuning = {}
    if cfg.sys_len > 0 and rng.random() < 0.4:
        tuning["sys_chunk_tokens"] = 128 * int(rng.integers(1, 6))
    if rng.random() < 0.3:
        tuning["ctx_part_tokens"] = int(rng.choice([128, 256]))
    return cfg, bool(rng.random() < 0.6), tuning


@pytest.mark.parametrize("seed", range(7100, 7116))
def test_random_prefill_shape(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    cfg, extra, tuning = _draw_prefill(rng)
    case = W.make_case(cfg, seed, prefill=True, extra_context=extra)
    _say("prefill %s seed=%d extra=%s tuning=%s m=%s c=%s"
         % (cfg, seed, extra, tuning, np.diff(case.cu_seqlens_q), case.context_lens))
    got, lse = DeviceCase(case, sys_layout="padded" if seed % 2 else "dense").prefill(**tuning)
    want, wlse, _ = oracle.prefill_attention(case.q, case.cu_seqlens_q, case.k_sys, case.v_sys,
                                             case.k_cache, case.v_cache, case.block_tables,
                                             case.context_lens, case.scale)
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e lse err %.3e" % (err, lerr))
    assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL


@pytest.mark.parametrize("seed", range(7200, 7212))
def test_random_multi_prefix_shape(seed):
    """Random groupings of a batch over up to 8 shared prefixes of random lengths (some empty)."""
    import torch
    from gpu_util import _bf16
    rng = np.random.Generator(np.random.PCG64(seed))
    G = int(rng.choice([1, 2, 4]))
    Hkv = int(rng.integers(1, 4))
    n_groups = int(rng.integers(1, 9))
    sizes = [int(rng.integers(1, 12)) for _ in range(n_groups)]
    lens = [int(rng.choice([0, 1, 33, int(rng.integers(34, 900))])) for _ in range(n_groups)]
    if max(lens) == 0:
        lens[0] = 77
    cfg = W.AttnConfig("rm", sum(sizes), G * Hkv, Hkv, int(rng.choice([64, 128])), 0, 0,
                       int(rng.choice([1, 40, 300])), block_size=int(rng.choice([4, 16, 32])))
    tuning = {"sys_chunk_tokens": 32 * int(rng.integers(1, 10))} if rng.random() < 0.4 else {}
    case = W.make_case(cfg, seed)
    groups = W.make_prefix_groups(case, seed + 1000, sizes, lens)
    _say("multi %s seed=%d groups=%s lens=%s tuning=%s" % (cfg, seed, sizes, lens, tuning))
    dc = DeviceCase(case)
    longest = max(g[2].shape[0] for g in groups)
    dev_groups, proto = [], None
    for first, n, ks, vs in groups:
        kd = _bf16(ks, dc.dev) if ks.shape[0] else None
        vd = _bf16(vs, dc.dev) if vs.shape[0] else None
        if kd is not None and kd.shape[0] == longest:
            proto = kd
        dev_groups.append((kd, vd, first, n))
    out, lse = dc._outputs(True)
    p = ra.make_params(dc.q, out, proto, dc.k_cache, dc.block_tables, batch=cfg.batch,
                       softmax_scale=case.scale, max_context_len=max(1, int(case.context_lens.max())),
                       **tuning)
    ws = dc._workspace(p, cfg.batch)
    ra.relay_attn_decode_multi(p, dev_groups, dc.q, dc.k_cache, dc.v_cache, dc.block_tables,
                               dc.context_lens, out, lse, ws)
    torch.cuda.synchronize()
    got, glse = out.cpu().numpy(), lse.cpu().numpy()
    B, Hq, d = case.q.shape
    want = np.zeros((B, Hq, d), np.float32)
    wlse = np.zeros((B, Hq), np.float32)
    for first, n, ks, vs in groups:
        sl = slice(first, first + n)
        o, l, _ = oracle.decode_attention(case.q[sl], ks, vs, case.k_cache, case.v_cache,
                                          case.block_tables[sl], case.context_lens[sl], case.scale)
        want[sl], wlse[sl] = o, l
    assert np.isfinite(got).all()
    live = np.isfinite(wlse)
    assert np.array_equal(np.isfinite(glse), live)
    err = np.abs(got - want).max()
    lerr = np.abs(glse[live] - wlse[live]).max() if live.any() else 0.0
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert err <= TOL and lerr <= LSE_TOL
