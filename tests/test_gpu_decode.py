"""GPU parity tests of relay_attn_decode / paged_attn_decode_naive against the CPU oracle.
Every call goes through the C ABI (ctypes binding).  Tolerance: max-abs 2e-3 on the fp32
output (bf16 inputs, fp32 accumulation); block-table handling must be bit-exact."""
import sys
from dataclasses import replace

import numpy as np
import pytest
import torch

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
    out, lse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables, case.context_lens,
                                          case.scale, rows=rows)
    return out, lse


def _cfg(**kw):
    base = dict(name="t", batch=5, num_q_heads=4, num_kv_heads=4, head_dim=128, sys_len=300,
                ctx_lo=1, ctx_hi=200, block_size=16)
    base.update(kw)
    return W.AttnConfig(**base)


def _check(case, tuning=None, tol=TOL, layouts=("dense",)):
    """layouts: the system-cache layouts to run (one oracle result serves all): "dense" is
    [s][Hkv][d], "padded" the row stride relay_attn_system_cache_layout recommends."""
    tuning = tuning or {}
    want, wlse = _oracle(case)
    for layout in layouts:
        _say("%s seed=%d tuning=%s system cache %s" % (case.cfg, case.seed, tuning, layout))
        got, lse = DeviceCase(case, sys_layout=layout).decode(**tuning)
        assert np.isfinite(got).all()
        err = np.abs(got - want).max()
        lerr = np.abs(lse - wlse).max()
        _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
        assert err <= tol and lerr <= LSE_TOL
    return got, lse


SMALL = [
    (W.TINY, 101, {}),
    (_cfg(), 102, {}),
    (_cfg(head_dim=64, sys_len=77, ctx_hi=90), 103, {}),
    (_cfg(num_q_heads=8, num_kv_heads=4, sys_len=129), 104, {}),                 # G=2
    (_cfg(num_q_heads=8, num_kv_heads=2, sys_len=1000, ctx_hi=700), 105, {}),    # G=4, multi-part
    (_cfg(num_q_heads=8, num_kv_heads=1, head_dim=64, sys_len=33, batch=7), 106, {}),  # G=8, M=56
    (_cfg(batch=37, num_q_heads=2, num_kv_heads=2, sys_len=515), 107, {}),       # two row tiles
    (_cfg(sys_len=0), 108, {}),
    (_cfg(sys_len=1, ctx_lo=1, ctx_hi=1), 109, {}),
    (_cfg(sys_len=4096, batch=3, ctx_hi=40), 110, {"sys_chunk_tokens": 1024}),
    (_cfg(sys_len=700, ctx_hi=600), 111, {"sys_chunk_tokens": 32, "ctx_part_tokens": 128}),
    (_cfg(sys_len=700, ctx_hi=600, block_size=8), 112, {"sys_chunk_tokens": 160}),
    (_cfg(sys_len=64, ctx_lo=500, ctx_hi=1500, block_size=32, batch=3), 113, {}),
    (_cfg(sys_len=257, block_size=1, ctx_hi=70), 114, {}),
    (_cfg(sys_len=257, block_size=128, ctx_hi=300), 115, {}),
    (_cfg(sys_len=900, ctx_hi=600, num_q_heads=8, num_kv_heads=4), 116, {}),
    (_cfg(sys_len=0, ctx_hi=300), 117, {}),
    (_cfg(sys_len=2500, ctx_hi=40, batch=40, num_q_heads=8, num_kv_heads=2), 118,
     {"sys_chunk_tokens": 512}),                                                                # M=160
    (_cfg(batch=70, num_q_heads=2, num_kv_heads=2, sys_len=515, ctx_hi=700), 145, {}),          # > 64 requests
    (_cfg(batch=150, num_q_heads=4, num_kv_heads=1, head_dim=64, sys_len=100, ctx_lo=0, ctx_hi=99), 146, {}),
    (_cfg(batch=16, head_dim=64, ctx_lo=0, ctx_hi=40, sys_len=320), 147, {}),                   # spans over several items
    (_cfg(batch=11, num_q_heads=6, num_kv_heads=2, sys_len=400, ctx_hi=300), 170, {}),          # G=3
    (_cfg(batch=9, num_q_heads=5, num_kv_heads=1, head_dim=64, sys_len=150, ctx_hi=90), 171, {}),   # G=5
    (_cfg(batch=50, num_q_heads=12, num_kv_heads=2, sys_len=1200, ctx_hi=64), 172, {}),         # G=6, many-rows items
    (_cfg(batch=13, num_q_heads=28, num_kv_heads=4, sys_len=257, ctx_hi=500), 173, {}),         # G=7 (28 / 4 heads)
]


@pytest.mark.parametrize("cfg,seed,tuning", SMALL)
def test_decode_matches_oracle_small(cfg, seed, tuning):
    _check(W.make_case(cfg, seed), tuning, layouts=("dense", "padded"))


# 256 or more stacked rows per kv head and a system part that outweighs the contexts: the system
# items are 128-row items of the many-rows kind inside the tile launch
MANY_ROWS = [
    (_cfg(batch=70, num_q_heads=8, num_kv_heads=2, sys_len=2100, ctx_hi=300), 148, {}),          # 280 rows, ragged block
    (_cfg(batch=33, num_q_heads=8, num_kv_heads=1, head_dim=64, sys_len=515, ctx_hi=90), 149,
     {"sys_chunk_tokens": 96}),                                                                  # G=8, odd chunk
    (_cfg(batch=256, num_q_heads=2, num_kv_heads=2, sys_len=1000, ctx_lo=0, ctx_hi=50), 150, {}),
    (_cfg(batch=64, num_q_heads=8, num_kv_heads=2, sys_len=100, ctx_hi=30), 151, {}),            # one chunk of 4 tiles
    (_cfg(batch=64, num_q_heads=16, num_kv_heads=4, sys_len=2100, ctx_hi=200), 152, {}),
    (_cfg(batch=40, num_q_heads=8, num_kv_heads=1, sys_len=4000, ctx_hi=500, block_size=8), 153, {}),   # 16 chunks
    # exactly one block of 128 stacked rows per kv head and a long prompt
    (_cfg(batch=128, num_q_heads=4, num_kv_heads=4, sys_len=32785, ctx_hi=100), 154, {}),
]


@pytest.mark.parametrize("cfg,seed,tuning", MANY_ROWS, ids=["c%d" % c[1] for c in MANY_ROWS])
def test_decode_with_many_rows_system_items(cfg, seed, tuning):
    case = W.make_case(cfg, seed)
    _say("%s seed=%d tuning=%s" % (cfg, seed, tuning))
    want, wlse = _oracle(case)
    for layout in ("dense", "padded"):
        dc = DeviceCase(case, sys_layout=layout)
        got, lse = dc.decode(**tuning)
        assert dc.last_plan.sys_rows_per_workgroup == 128, "the case no longer exercises the many-rows items"
        assert np.isfinite(got).all()
        err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
        _say("system cache %s: max-abs err %.3e  lse err %.3e  (%d system workgroups, %d chunks)"
             % (layout, err, lerr, dc.last_plan.num_sys_workgroups, dc.last_plan.num_sys_chunks))
        assert err <= TOL and lerr <= LSE_TOL


def test_llama7b_full():
    _check(W.make_case(W.LLAMA7B, 2000), layouts=("padded", "dense"))


@pytest.mark.parametrize("s", W.LLAMA30B_SWEEP)
def test_llama30b_full_rows(s):
    """Every point of the timed system-prompt sweep, every output row, in the launch
    configuration the benchmark times (max_context_len = the longest real context; the system
    cache in the padded layout), and with a dense system cache."""
    _check(W.make_case(W.llama30b(s), 3000 + s, poison_tails=s < 16384), layouts=("padded", "dense"))


def test_llama30b_bf16_output_at_the_headline_shape():
    case = W.make_case(W.llama30b(2048), 3001)
    _say("%s bf16 output" % (case.cfg,))
    dc = DeviceCase(case)
    b16, lse = dc.decode(fp32_out=False)
    f32, _ = dc.decode(fp32_out=True)
    want, wlse = _oracle(case)
    assert np.array_equal(W.bf16_round(f32), b16)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    assert (np.abs(b16 - want) <= np.maximum(TOL, ulp)).all()
    assert np.abs(lse - wlse).max() <= LSE_TOL


@pytest.mark.parametrize("b", [4, 8, 16])
def test_speedup_grid_corner_shapes(b):
    """Corners of the (batch, context, prompt) grid of the standalone-attention experiment
    (Sec. 3.4 "Theoretical Speedup"): 52 heads, context 256, batches below one row tile."""
    cfg = W.AttnConfig("grid_b%d_c256_s2048" % b, b, 52, 52, 128, 2048, 256, 256)
    _check(W.make_case(cfg, 3100 + b))
    cfg = W.AttnConfig("grid_b%d_c128_s512" % b, b, 52, 52, 128, 512, 128, 128)
    _check(W.make_case(cfg, 3200 + b))


def _widen_tables(case, factor):
    """Same batch with a block table `factor` times wider (poison in the unused slots), so that
    the table capacity is far above every real context length."""
    wide = np.full((case.block_tables.shape[0], case.block_tables.shape[1] * factor),
                   W.POISON_BLOCK, dtype=np.int32)
    wide[:, :case.block_tables.shape[1]] = case.block_tables
    return replace(case, block_tables=wide)


@pytest.mark.parametrize("cfg,seed,factor,bound", [
    (_cfg(), 190, 16, 0),                                                    # 0: table capacity
    (_cfg(batch=37, num_q_heads=8, num_kv_heads=2, sys_len=900, ctx_hi=300), 191, 8, 0),
    (_cfg(sys_len=0, ctx_hi=500, block_size=8), 192, 32, 0),
    (_cfg(batch=64, num_q_heads=8, num_kv_heads=2, sys_len=2100, ctx_hi=120), 193, 8, 0),   # many-rows items
    (_cfg(batch=9, ctx_lo=0, ctx_hi=64, sys_len=515), 194, 4, 256),          # an explicit loose bound
    (W.llama30b(2048), 195, 8, 0),
    (W.LLAMA7B, 196, 32, 4096),
])
def test_length_bound_far_above_the_real_lengths(cfg, seed, factor, bound):
    """The serving default: max_context_len = 0 (the table capacity) or a loose bound, 4 - 32
    times the real lengths.  The plan is then sized for contexts that do not exist: spans shrink
    to the floor, trailing wavefronts idle, unused slots are marked empty on the device."""
    case = _widen_tables(W.make_case(cfg, seed), factor)
    _say("%s seed=%d table width %d bound %d (real max %d)"
         % (cfg, seed, case.block_tables.shape[1], bound, case.context_lens.max()))
    got, lse = DeviceCase(case).decode(max_context_len=bound)
    want, wlse = _oracle(case)
    assert np.isfinite(got).all()
    err, lerr = np.abs(got - want).max(), np.abs(lse - wlse).max()
    _say("max-abs err %.3e  lse err %.3e" % (err, lerr))
    assert err <= TOL and lerr <= LSE_TOL


@pytest.mark.parametrize("cfg,seed,tuning", [
    # one context far longer than a wavefront's block-id table covers (256 blocks): the span cap
    # forces more context workgroups than the balance rule alone would give
    (_cfg(batch=2, num_q_heads=2, num_kv_heads=1, sys_len=100, ctx_lo=17000, ctx_hi=20000, block_size=16), 160, {}),
    (_cfg(batch=2, num_q_heads=4, num_kv_heads=1, head_dim=64, sys_len=0, ctx_lo=9000, ctx_hi=9000, block_size=1), 161, {}),
    (_cfg(batch=12, num_q_heads=2, num_kv_heads=2, sys_len=3000, ctx_lo=1, ctx_hi=6000, block_size=8), 162, {}),
], ids=["c160", "c161", "c162"])
def test_very_long_contexts(cfg, seed, tuning):
    _check(W.make_case(cfg, seed), tuning)


def test_llama3_8b_gqa_full_rows():
    _check(W.make_case(W.LLAMA3_8B_GQA, 4000), layouts=("padded", "dense"))


def test_llama3_8b_gqa_bf16_output_sampled_rows():
    case = W.make_case(W.LLAMA3_8B_GQA, 4001)
    _say("%s bf16 output" % (case.cfg,))
    rng = np.random.Generator(np.random.PCG64(2))
    rows = np.stack([rng.integers(0, 128, 256), rng.integers(0, 32, 256)], axis=1).astype(np.int32)
    got, lse = DeviceCase(case).decode(fp32_out=False)
    want, wlse = _oracle(case, rows=rows)
    g = got[rows[:, 0], rows[:, 1]]
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
    assert np.isfinite(got).all()
    assert (np.abs(g - want) <= np.maximum(TOL, ulp)).all()
    assert np.abs(lse[rows[:, 0], rows[:, 1]] - wlse).max() <= LSE_TOL


def test_block_placement_is_bit_exact_and_poison_is_never_read():
    case = W.make_case(_cfg(num_q_heads=8, num_kv_heads=4, sys_len=200, ctx_hi=500), 120)
    assert np.isnan(case.k_cache).any() and (case.block_tables == W.POISON_BLOCK).any()
    base, lse0 = _check(case)
    for seed, ident in ((7, False), (8, True)):
        other = W.repage(case, seed, identity=ident)
        _say("repage seed=%d identity=%s" % (seed, ident))
        got, lse = DeviceCase(other).decode()
        assert np.array_equal(got, base) and np.array_equal(lse, lse0)


def test_one_workspace_serves_calls_with_different_shapes():
    """A workspace holds nothing between calls: one buffer full of garbage serves calls with
    other batch sizes and prompt lengths."""
    cases = [W.make_case(_cfg(sys_len=700, batch=9, ctx_hi=300), 130),
             W.make_case(_cfg(sys_len=64, batch=3, num_q_heads=8, num_kv_heads=2, ctx_hi=600), 131),
             W.make_case(_cfg(sys_len=1500, batch=17, head_dim=64, ctx_hi=90), 132),
             W.make_case(_cfg(sys_len=700, batch=9, ctx_hi=300), 130)]
    shared = torch.full((64 << 20,), 0x5A, dtype=torch.uint8, device="cuda:0")
    for case in cases:
        _say("shared workspace: %s" % (case.cfg,))
        dc = DeviceCase(case)
        dc._workspace = lambda params, total_q: shared
        got, lse = dc.decode()
        want, wlse = _oracle(case)
        assert np.abs(got - want).max() <= TOL and np.abs(lse - wlse).max() <= LSE_TOL


def test_runs_are_bitwise_reproducible():
    case = W.make_case(_cfg(sys_len=900, ctx_hi=400, batch=9), 121)
    dc = DeviceCase(case)
    a, la = dc.decode()
    b, lb = dc.decode()
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_request_permutation_permutes_outputs():
    case = W.make_case(_cfg(batch=6), 122)
    base, lse0 = _check(case)
    perm = np.array([4, 2, 0, 5, 1, 3])
    other = replace(case, q=case.q[perm], block_tables=case.block_tables[perm],
                    context_lens=case.context_lens[perm])
    got, lse = DeviceCase(other).decode()
    np.testing.assert_allclose(got, base[perm], atol=1e-5, rtol=0)
    np.testing.assert_allclose(lse, lse0[perm], atol=1e-5, rtol=0)


def test_prefix_split_point_does_not_matter():
    cfg = _cfg(sys_len=320, ctx_lo=5, ctx_hi=90)
    case = W.make_case(cfg, 123)
    base, lse0 = _check(case)
    want, _ = _oracle(case)
    for moved in (1, 37, 320):
        keep = cfg.sys_len - moved
        ck, cv = [], []
        for i in range(cfg.batch):
            k, v = W.logical_context(case, i)
            ck.append(np.concatenate([case.k_sys[keep:], k]))
            cv.append(np.concatenate([case.v_sys[keep:], v]))
        other = W.from_dense(cfg, case.q, case.k_sys[:keep], case.v_sys[:keep], ck, cv, seed=9)
        _say("moved %d system tokens into every context" % moved)
        got, lse = DeviceCase(other).decode()
        assert np.abs(got - want).max() <= TOL
        np.testing.assert_allclose(got, base, atol=2e-4, rtol=0)
        np.testing.assert_allclose(lse, lse0, atol=1e-4, rtol=0)


def test_bf16_output_is_the_rounded_fp32_output():
    case = W.make_case(_cfg(sys_len=400), 124)
    dc = DeviceCase(case)
    f32, _ = dc.decode(fp32_out=True)
    b16, _ = dc.decode(fp32_out=False)
    assert np.array_equal(W.bf16_round(f32), b16)
    want, _ = _oracle(case)
    ulp = np.maximum(2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7), 0)
    assert (np.abs(b16 - want) <= np.maximum(TOL, ulp)).all()


def test_requests_without_context_and_fully_empty_rows():
    cfg = _cfg(sys_len=100)
    case = W.make_case(cfg, 125)
    lens = case.context_lens.copy()
    lens[[1, 3]] = 0
    other = replace(case, context_lens=lens)
    _check(other)
    empty = np.zeros((0, cfg.num_kv_heads, cfg.head_dim), np.float32)
    nosys = replace(other, k_sys=empty, v_sys=empty, cfg=replace(cfg, sys_len=0))
    got, lse = DeviceCase(nosys).decode()
    want, wlse = _oracle(nosys)
    assert np.all(got[[1, 3]] == 0) and np.all(np.isneginf(lse[[1, 3]]))
    assert np.all(np.isneginf(wlse[[1, 3]]))
    keep = [0, 2, 4]
    assert np.abs(got[keep] - want[keep]).max() <= TOL


def test_strided_inputs_and_head_major_system_cache():
    case = W.make_case(_cfg(num_q_heads=8, num_kv_heads=4, sys_len=210), 126)
    want, _ = _oracle(case)
    dc = DeviceCase(case)
    wide = torch.zeros(case.cfg.batch, 8, 256, dtype=torch.bfloat16, device=dc.dev)
    wide[:, :, 64:192] = dc.q
    dc.q = wide[:, :, 64:192]
    dc.k_sys = dc.k_sys.permute(1, 0, 2).contiguous().permute(1, 0, 2)   # [Hkv, s, d] storage
    dc.v_sys = dc.v_sys.permute(1, 0, 2).contiguous().permute(1, 0, 2)
    assert dc.k_sys.stride(0) == 128 and dc.q.stride(1) == 256
    got, _ = dc.decode()
    assert np.abs(got - want).max() <= TOL


def test_naive_paged_attention_matches_oracle_and_relay():
    cfg = _cfg(sys_len=256, ctx_hi=120, num_q_heads=8, num_kv_heads=4)
    case = W.make_case(cfg, 127)
    relay, rlse = _check(case)
    flat = W.with_system_pages(case)
    _say("naive per-request view: context lens %s" % flat.context_lens)
    want, wlse = _oracle(flat)
    got, lse = DeviceCase(flat).naive()
    assert np.abs(got - want).max() <= TOL and np.abs(lse - wlse).max() <= LSE_TOL
    np.testing.assert_allclose(got, relay, atol=2e-4, rtol=0)
    short = W.make_case(_cfg(sys_len=0, ctx_hi=100), 128)       # single part: direct output
    want, wlse = _oracle(short)
    for fp32 in (True, False):
        got, lse = DeviceCase(short).naive(fp32_out=fp32)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - 7)
        assert (np.abs(got - want) <= (TOL if fp32 else np.maximum(TOL, ulp))).all()
        assert np.abs(lse - wlse).max() <= LSE_TOL


@pytest.mark.parametrize("G,d", [(3, 128), (5, 64), (6, 128), (7, 64)])
def test_naive_paged_attention_group_sizes_that_are_not_powers_of_two(G, d):
    cfg = _cfg(sys_len=0, ctx_lo=1, ctx_hi=700, num_q_heads=2 * G, num_kv_heads=2, head_dim=d, batch=6)
    case = W.make_case(cfg, 180 + G)
    _say("%s seed=%d" % (cfg, 180 + G))
    want, wlse = _oracle(case)
    got, lse = DeviceCase(case).naive()
    assert np.isfinite(got).all()
    assert np.abs(got - want).max() <= TOL and np.abs(lse - wlse).max() <= LSE_TOL
