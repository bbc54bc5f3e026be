"""Pins for the CPU oracle: every expected value here comes from the paper's equations,
from mathematics, or from an independent library routine — never from the oracle itself
and never from the HIP path.  All of it runs without a GPU."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import oracle
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _decode(case, **kw):
    out, lse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables, case.context_lens,
                                          case.scale, **kw)
    return out, lse


def _small_cfg(**kw):
    base = dict(name="small", batch=3, num_q_heads=4, num_kv_heads=2, head_dim=16, sys_len=37,
                ctx_lo=1, ctx_hi=45, block_size=8)
    base.update(kw)
    return W.AttnConfig(**base)


# ---------------------------------------------------------------- worked example
def _parse_golden():
    consts = {"LN2": math.log(2.0), "LN3": math.log(3.0), "LN6": math.log(6.0)}
    vals = {}
    with open(os.path.join(GOLDEN, "eq4_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(":", 1)
            rows = [[consts.get(t, None) if t in consts else float(t) for t in r.split()]
                    for r in rest.split(";")]
            vals[key.strip()] = np.array(rows, dtype=np.float64)
    return vals


@pytest.mark.parametrize("qmul,scale", [(1.0, 1.0), (2.0, 0.5)])
def test_hand_worked_example(qmul, scale):
    g = _parse_golden()
    cfg = W.AttnConfig("worked", 1, 1, 1, 2, 2, 1, 1, block_size=4)
    q = (g["q"] * qmul).reshape(1, 1, 2)
    ks, vs = g["k_sys"].reshape(2, 1, 2), g["v_sys"].reshape(2, 1, 2)
    kc, vc = g["k_ctx"].reshape(1, 1, 2), g["v_ctx"].reshape(1, 1, 2)
    case = W.from_dense(cfg, q, ks, vs, [kc], [vc])
    out, lse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables, case.context_lens,
                                          scale)
    np.testing.assert_allclose(out[0, 0], g["out"][0], atol=1e-6)
    np.testing.assert_allclose(lse[0, 0], g["lse"][0, 0], atol=1e-6)
    # system part alone (no context visible) and context part alone (no system prompt)
    o_s, l_s, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables,
                                          np.zeros(1, np.int32), scale)
    np.testing.assert_allclose(o_s[0, 0], g["out_sys"][0], atol=1e-6)
    np.testing.assert_allclose(l_s[0, 0], g["lse_sys"][0, 0], atol=1e-6)
    empty = np.zeros((0, 1, 2), np.float32)
    o_c, l_c, _ = oracle.decode_attention(case.q, empty, empty, case.k_cache, case.v_cache,
                                          case.block_tables, case.context_lens, scale)
    np.testing.assert_allclose(o_c[0, 0], g["out_ctx"][0], atol=1e-6)
    np.testing.assert_allclose(l_c[0, 0], g["lse_ctx"][0, 0], atol=1e-6)
    alpha = 1.0 / (1.0 + math.exp(l_c[0, 0] - l_s[0, 0]))
    assert abs(alpha - g["alpha_sys"][0, 0]) < 1e-6


# ---------------------------------------------------------------- library routine
def _dense_reference(case, scale):
    """torch CPU scaled_dot_product_attention (fp64) on the gathered dense sequence, and
    scipy's logsumexp of the logits: library routines, independent of the oracle's C."""
    B, Hq, d = case.q.shape
    G = case.cfg.num_q_heads // case.cfg.num_kv_heads
    outs, lses = [], []
    for i in range(B):
        kc, vc = W.logical_context(case, i)
        k = np.concatenate([case.k_sys, kc], axis=0).astype(np.float64)   # [l, Hkv, d]
        v = np.concatenate([case.v_sys, vc], axis=0).astype(np.float64)
        k = np.repeat(k, G, axis=1).transpose(1, 0, 2)                    # [Hq, l, d]
        v = np.repeat(v, G, axis=1).transpose(1, 0, 2)
        qi = case.q[i].astype(np.float64)[:, None, :]                     # [Hq, 1, d]
        o = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qi), torch.from_numpy(k), torch.from_numpy(v), scale=scale)
        outs.append(o.numpy()[:, 0, :])
        logits = scale * np.einsum("hd,hld->hl", case.q[i].astype(np.float64), k)
        lses.append(scipy.special.logsumexp(logits, axis=1))
    return np.stack(outs), np.stack(lses)


@pytest.mark.parametrize("cfg,seed", [
    (W.TINY, 11),
    (_small_cfg(), 12),
    (_small_cfg(num_q_heads=6, num_kv_heads=2, head_dim=8, block_size=4), 13),
    (_small_cfg(num_kv_heads=1, sys_len=0), 14),
    (_small_cfg(num_kv_heads=4, sys_len=5, ctx_lo=1, ctx_hi=3), 15),
])
def test_matches_library_attention(cfg, seed):
    case = W.make_case(cfg, seed)
    out, lse = _decode(case)
    ref_o, ref_l = _dense_reference(case, case.scale)
    np.testing.assert_allclose(out, ref_o, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, ref_l, rtol=0, atol=1e-12)


def test_scale_is_applied_to_logits():
    case = W.make_case(_small_cfg(), 16)
    for scale in (1.0, 0.3):
        out, lse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                              case.v_cache, case.block_tables,
                                              case.context_lens, scale)
        ref_o, ref_l = _dense_reference(case, scale)
        np.testing.assert_allclose(out, ref_o, atol=1e-12)
        np.testing.assert_allclose(lse, ref_l, atol=1e-12)


# ---------------------------------------------------------------- closed forms
def test_zero_query_gives_mean_and_log_count():
    case = W.make_case(_small_cfg(), 21)
    case.q[:] = 0.0
    out, lse = _decode(case)
    G = 2
    for i in range(case.cfg.batch):
        kc, vc = W.logical_context(case, i)
        allv = np.concatenate([case.v_sys, vc], axis=0).astype(np.float64)
        for h in range(case.cfg.num_q_heads):
            np.testing.assert_allclose(out[i, h], allv[:, h // G].mean(axis=0), atol=1e-13)
            assert abs(lse[i, h] - math.log(allv.shape[0])) < 1e-13


def test_single_visible_position_returns_its_value():
    cfg = _small_cfg(sys_len=0, ctx_lo=1, ctx_hi=1)
    case = W.make_case(cfg, 22)
    out, lse = _decode(case)
    for i in range(cfg.batch):
        kc, vc = W.logical_context(case, i)
        for h in range(cfg.num_q_heads):
            np.testing.assert_allclose(out[i, h], vc[0, h // 2], atol=1e-14)
            z = case.scale * float(np.dot(case.q[i, h].astype(np.float64),
                                          kc[0, h // 2].astype(np.float64)))
            assert abs(lse[i, h] - z) < 1e-12


def test_dominant_key_selects_its_value():
    cfg = _small_cfg(num_q_heads=2, num_kv_heads=2)
    case = W.make_case(cfg, 23)
    # make system position 5 of every head collinear with the query of request 0 and huge
    for h in range(2):
        case.k_sys[5, h] = W.bf16_round(case.q[0, h] * 64.0)
    out, _ = _decode(case)
    for h in range(2):
        np.testing.assert_allclose(out[0, h], case.v_sys[5, h], atol=1e-9)


def test_equal_keys_give_uniform_weights():
    case = W.make_case(_small_cfg(num_q_heads=2, num_kv_heads=2, sys_len=9, ctx_lo=5, ctx_hi=5,
                                  block_size=8), 24, poison_tails=False)
    key = case.k_sys[0].copy()
    case.k_sys[:] = key[None]
    case.k_cache[:] = key[None, :, None, :]
    out, lse = _decode(case)
    for i in range(case.cfg.batch):
        _, vc = W.logical_context(case, i)
        allv = np.concatenate([case.v_sys, vc], axis=0).astype(np.float64)
        for h in range(2):
            np.testing.assert_allclose(out[i, h], allv[:, h].mean(axis=0), atol=1e-12)
            z = case.scale * float(np.dot(case.q[i, h].astype(np.float64), key[h].astype(np.float64)))
            assert abs(lse[i, h] - (z + math.log(14))) < 1e-12


def test_empty_sequence_is_zero_with_minus_infinity():
    cfg = _small_cfg(sys_len=0)
    case = W.make_case(cfg, 25)
    out, lse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables,
                                          np.zeros(cfg.batch, np.int32), case.scale)
    assert np.all(out == 0.0) and np.all(np.isneginf(lse))


# ---------------------------------------------------------------- invariances
def test_logit_shift_invariance():
    # adding a to every key adds scale*q.a to every logit: output unchanged, beta shifted
    case = W.make_case(_small_cfg(), 31, poison_tails=False)
    out0, lse0 = _decode(case)
    a = W.bf16_round(np.full((case.cfg.num_kv_heads, case.cfg.head_dim), 0.5, np.float32))
    a[:, ::2] = -0.25
    shifted = W.make_case(_small_cfg(), 31, poison_tails=False)
    shifted.k_sys = case.k_sys + a[None]
    shifted.k_cache = case.k_cache + a[None, :, None, :]
    out1, lse1 = _decode(shifted)
    np.testing.assert_allclose(out1, out0, atol=1e-12)
    G = 2
    for i in range(case.cfg.batch):
        for h in range(case.cfg.num_q_heads):
            delta = case.scale * float(np.dot(case.q[i, h].astype(np.float64), a[h // G].astype(np.float64)))
            assert abs((lse1[i, h] - lse0[i, h]) - delta) < 1e-12


def _relay_combine(o_sys, l_sys, o_ctx, l_ctx):
    """Relay fusion exactly as App. A / Alg. 1 write it."""
    with np.errstate(over="ignore"):
        alpha_sys = 1.0 / (1.0 + np.exp(l_ctx - l_sys))
    alpha_ctx = 1.0 - alpha_sys
    return o_ctx * alpha_ctx[..., None] + o_sys * alpha_sys[..., None], alpha_sys, alpha_ctx


def test_relay_fusion_is_exact_at_every_split_point():
    """Eq. 5-7 with Eq. 11: splitting the sequence at ANY position and recombining the two
    partial attentions with alpha reproduces full attention (Sec. 3.3 notes nothing assumes
    where the split falls)."""
    cfg = _small_cfg(batch=2, sys_len=13, ctx_lo=6, ctx_hi=6, block_size=4)
    case = W.make_case(cfg, 32)
    full, lse_full = _decode(case)
    empty = np.zeros((0, cfg.num_kv_heads, cfg.head_dim), np.float32)
    ctx = [W.logical_context(case, i) for i in range(cfg.batch)]
    for split in range(0, cfg.sys_len + 6 + 1):
        # "system" := first `split` positions of the full sequence (identical for all requests
        # only while split <= s, so beyond s each request is evaluated on its own)
        for i in range(cfg.batch):
            k_all = np.concatenate([case.k_sys, ctx[i][0]], axis=0)
            v_all = np.concatenate([case.v_sys, ctx[i][1]], axis=0)
            qi = case.q[i:i + 1]
            one = W.AttnConfig("one", 1, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                               split, 0, 0, block_size=4)
            left = W.from_dense(one, qi, k_all[:split], v_all[:split], [empty], [empty])
            right = W.from_dense(one, qi, empty, empty, [k_all[split:]], [v_all[split:]])
            o_l, l_l = _decode(left)
            o_r, l_r = _decode(right)
            if split == 0:
                assert np.all(np.isneginf(l_l))
            fused, a_s, a_c = _relay_combine(o_l, l_l, o_r, l_r)
            assert np.all((a_s >= 0) & (a_s <= 1)) and np.allclose(a_s + a_c, 1.0, atol=1e-15)
            np.testing.assert_allclose(fused[0], full[i], atol=1e-12)
            np.testing.assert_allclose(np.logaddexp(l_l, l_r)[0], lse_full[i], atol=1e-12)


def test_alpha_closed_form_for_zero_query():
    case = W.make_case(_small_cfg(), 33)
    case.q[:] = 0.0
    empty = np.zeros((0, case.cfg.num_kv_heads, case.cfg.head_dim), np.float32)
    _, l_sys, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables,
                                          np.zeros(case.cfg.batch, np.int32), case.scale)
    _, l_ctx, _ = oracle.decode_attention(case.q, empty, empty, case.k_cache, case.v_cache,
                                          case.block_tables, case.context_lens, case.scale)
    s = case.cfg.sys_len
    for i in range(case.cfg.batch):
        c = int(case.context_lens[i])
        alpha = 1.0 / (1.0 + np.exp(l_ctx[i] - l_sys[i]))
        np.testing.assert_allclose(alpha, s / (s + c), atol=1e-14)
        np.testing.assert_allclose(l_sys[i], math.log(s), atol=1e-14)
        np.testing.assert_allclose(l_ctx[i], math.log(c), atol=1e-14)


def test_moving_system_tokens_into_every_context_changes_nothing():
    cfg = _small_cfg(sys_len=20, ctx_lo=3, ctx_hi=17, block_size=4)
    case = W.make_case(cfg, 34)
    base, lse0 = _decode(case)
    for moved in (1, 7, 20):
        keep = cfg.sys_len - moved
        ctx_k, ctx_v = [], []
        for i in range(cfg.batch):
            kc, vc = W.logical_context(case, i)
            ctx_k.append(np.concatenate([case.k_sys[keep:], kc], axis=0))
            ctx_v.append(np.concatenate([case.v_sys[keep:], vc], axis=0))
        other = W.from_dense(cfg, case.q, case.k_sys[:keep], case.v_sys[:keep], ctx_k, ctx_v, seed=5)
        out, lse = _decode(other)
        np.testing.assert_allclose(out, base, atol=1e-12)
        np.testing.assert_allclose(lse, lse0, atol=1e-12)


def test_requests_are_independent_and_permute():
    cfg = _small_cfg(batch=5)
    case = W.make_case(cfg, 35)
    base, lse0 = _decode(case)
    perm = np.array([3, 0, 4, 1, 2])
    out, lse, _ = oracle.decode_attention(case.q[perm], case.k_sys, case.v_sys, case.k_cache,
                                          case.v_cache, case.block_tables[perm],
                                          case.context_lens[perm], case.scale)
    assert np.array_equal(out, base[perm]) and np.array_equal(lse, lse0[perm])


def test_system_token_order_does_not_matter():
    case = W.make_case(_small_cfg(), 36)
    base, lse0 = _decode(case)
    perm = np.random.Generator(np.random.PCG64(1)).permutation(case.cfg.sys_len)
    case.k_sys, case.v_sys = case.k_sys[perm], case.v_sys[perm]
    out, lse = _decode(case)
    np.testing.assert_allclose(out, base, atol=1e-13)
    np.testing.assert_allclose(lse, lse0, atol=1e-13)


def test_physical_block_placement_is_invisible():
    case = W.make_case(_small_cfg(), 37)
    base, lse0 = _decode(case)
    for seed, ident in ((1, False), (2, True)):
        other = W.repage(case, seed, identity=ident)
        assert not np.array_equal(other.block_tables, case.block_tables)
        out, lse = _decode(other)
        assert np.array_equal(out, base) and np.array_equal(lse, lse0)


def test_poison_slots_and_tails_are_never_read():
    case = W.make_case(_small_cfg(), 38, poison_tails=True)
    assert np.isnan(case.k_cache).any()
    assert (case.block_tables == W.POISON_BLOCK).any()
    out, lse = _decode(case)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    bad = case.block_tables.copy()
    bad[0, 0] = case.num_blocks          # first block of request 0 is out of range
    with pytest.raises(ValueError):
        oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache, case.v_cache,
                                bad, case.context_lens, case.scale)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    cfg = _small_cfg(num_q_heads=6, num_kv_heads=2)
    case = W.make_case(cfg, 39)
    base, lse0 = _decode(case)
    mha = W.make_case(cfg, 39)
    out, lse, _ = oracle.decode_attention(
        mha.q, np.repeat(mha.k_sys, 3, axis=1), np.repeat(mha.v_sys, 3, axis=1),
        np.repeat(mha.k_cache, 3, axis=1), np.repeat(mha.v_cache, 3, axis=1),
        mha.block_tables, mha.context_lens, mha.scale)
    assert np.array_equal(out, base) and np.array_equal(lse, lse0)


# ---------------------------------------------------------------- prompt phase
def test_prefill_rows_equal_truncated_decode_and_library_causal():
    cfg = _small_cfg(batch=3, q_lo=2, q_hi=9, ctx_lo=0, ctx_hi=11, sys_len=10, block_size=4)
    for extra in (False, True):
        case = W.make_case(cfg, 41 + extra, prefill=True, extra_context=extra)
        out, lse, _ = oracle.prefill_attention(case.q, case.cu_seqlens_q, case.k_sys, case.v_sys,
                                               case.k_cache, case.v_cache, case.block_tables,
                                               case.context_lens, case.scale)
        G = cfg.num_q_heads // cfg.num_kv_heads
        for i in range(cfg.batch):
            a, b = int(case.cu_seqlens_q[i]), int(case.cu_seqlens_q[i + 1])
            m, c = b - a, int(case.context_lens[i])
            kc, vc = W.logical_context(case, i)
            # library: causal mask aligned bottom-right, system columns always visible
            k = np.repeat(np.concatenate([case.k_sys, kc]).astype(np.float64), G, axis=1).transpose(1, 0, 2)
            v = np.repeat(np.concatenate([case.v_sys, vc]).astype(np.float64), G, axis=1).transpose(1, 0, 2)
            qi = case.q[a:b].astype(np.float64).transpose(1, 0, 2)
            mask = np.zeros((m, cfg.sys_len + c), dtype=bool)
            for j in range(m):
                mask[j, :cfg.sys_len + c - m + j + 1] = True
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(qi), torch.from_numpy(k), torch.from_numpy(v),
                attn_mask=torch.from_numpy(mask), scale=case.scale).numpy().transpose(1, 0, 2)
            np.testing.assert_allclose(out[a:b], ref, atol=1e-12)
            # each row is a decode step over the context truncated after that token
            for j in range(m):
                o1, l1, _ = oracle.decode_attention(
                    case.q[a + j:a + j + 1], case.k_sys, case.v_sys, case.k_cache, case.v_cache,
                    case.block_tables[i:i + 1], np.array([c - m + j + 1], np.int32), case.scale)
                assert np.array_equal(o1[0], out[a + j]) and np.array_equal(l1[0], lse[a + j])


# ---------------------------------------------------------------- cache write (Alg. 1)
def _parse_append_golden():
    vals = {}
    with open(os.path.join(GOLDEN, "cache_append_worked_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, rest = line.split(":", 1)
            vals[key.strip()] = [[int(t) for t in r.split()] for r in rest.split(";")]
    return vals


def test_cache_append_hand_worked_example():
    g = _parse_append_golden()
    bs, nb = g["block_size"][0][0], g["num_blocks"][0][0]
    tables = np.array(g["tables"], np.int32)
    l_new = np.array(g["l_new"][0], np.int32)
    counts = np.array(g["new_counts"][0])
    cu = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    blk, off = np.meshgrid(np.arange(nb), np.arange(bs), indexing="ij")
    k0 = -(100.0 * blk + off).astype(np.float32).reshape(nb, 1, bs, 1)
    v0 = k0 - 1000.0
    k_new = (1.0 + np.arange(cu[-1], dtype=np.float32)).reshape(-1, 1, 1)
    v_new = 0.5 - k_new
    k1, v1 = oracle.cache_append(k0, v0, tables, l_new, k_new, v_new, cu)
    want_k, want_v = k0.copy(), v0.copy()
    for t, (b, o) in enumerate(g["slots"]):
        want_k[b, 0, o, 0] = 1.0 + t
        want_v[b, 0, o, 0] = 0.5 - (1.0 + t)
    assert np.array_equal(k1, want_k) and np.array_equal(v1, want_v)
    assert np.array_equal(k0[..., 0, 0], -(100.0 * np.arange(nb))[:, None])   # inputs untouched


@pytest.mark.parametrize("prefill", [False, True])
def test_cache_append_then_attend_equals_attention_over_the_concatenation(prefill):
    """Alg. 1 writes the new K,V into the cache and then attends over [0, l_new): the result must
    equal library attention over the dense sequence [system ; old context ; new tokens] that is
    assembled here without any paging."""
    cfg = _small_cfg(batch=4, q_lo=1, q_hi=6, ctx_lo=0 if prefill else 1, ctx_hi=19, block_size=4,
                     sys_len=9)
    case = W.make_case(cfg, 51 + prefill, prefill=prefill, extra_context=True, poison_tails=False)
    rng = np.random.Generator(np.random.PCG64(77))
    cu = case.cu_seqlens_q
    total = int(cu[-1])
    Hkv, d, G = cfg.num_kv_heads, cfg.head_dim, cfg.num_q_heads // cfg.num_kv_heads
    k_new = W.bf16_round(rng.standard_normal((total, Hkv, d), dtype=np.float32))
    v_new = W.bf16_round(rng.standard_normal((total, Hkv, d), dtype=np.float32))
    k_old, v_old = case.k_cache.copy(), case.v_cache.copy()
    old_ctx = [W.logical_context(case, i) for i in range(cfg.batch)]
    k1, v1 = oracle.cache_append(k_old, v_old, case.block_tables, case.context_lens, k_new, v_new,
                                 cu if prefill else None)
    out, lse, _ = oracle.prefill_attention(case.q, cu, case.k_sys, case.v_sys, k1, v1,
                                           case.block_tables, case.context_lens, case.scale)
    changed = 0
    for i in range(cfg.batch):
        a, b = int(cu[i]), int(cu[i + 1])
        m, c = b - a, int(case.context_lens[i])
        kc = np.concatenate([old_ctx[i][0][:c - m], k_new[a:b]])
        vc = np.concatenate([old_ctx[i][1][:c - m], v_new[a:b]])
        k = np.repeat(np.concatenate([case.k_sys, kc]).astype(np.float64), G, axis=1).transpose(1, 0, 2)
        v = np.repeat(np.concatenate([case.v_sys, vc]).astype(np.float64), G, axis=1).transpose(1, 0, 2)
        qi = case.q[a:b].astype(np.float64).transpose(1, 0, 2)
        mask = np.zeros((m, cfg.sys_len + c), dtype=bool)
        for j in range(m):
            mask[j, :cfg.sys_len + c - m + j + 1] = True
        ref = torch.nn.functional.scaled_dot_product_attention(
            torch.from_numpy(qi), torch.from_numpy(k), torch.from_numpy(v),
            attn_mask=torch.from_numpy(mask), scale=case.scale).numpy().transpose(1, 0, 2)
        np.testing.assert_allclose(out[a:b], ref, atol=1e-12)
        changed += m
    # exactly the new positions changed, nothing else (K and V alike)
    diff_k = np.any(k1 != k_old, axis=(1, 3))
    diff_v = np.any(v1 != v_old, axis=(1, 3))
    assert diff_k.sum() == changed and diff_v.sum() == changed


def test_cache_append_rejects_bad_inputs():
    case = W.make_case(_small_cfg(batch=2, ctx_lo=3, ctx_hi=3), 53, poison_tails=False)
    new = np.zeros((2, 2, 16), np.float32)
    bad = case.block_tables.copy()
    bad[1, 0] = case.num_blocks
    with pytest.raises(ValueError):
        oracle.cache_append(case.k_cache, case.v_cache, bad, case.context_lens, new, new)
    with pytest.raises(ValueError):       # five new tokens in a context of three
        oracle.cache_append(case.k_cache, case.v_cache, case.block_tables, case.context_lens,
                            np.zeros((10, 2, 16), np.float32), np.zeros((10, 2, 16), np.float32),
                            np.array([0, 5, 10]))


def test_row_selection_matches_full_result():
    case = W.make_case(_small_cfg(), 42)
    full, lse = _decode(case)
    rows = np.array([[2, 3], [0, 0], [1, 2]], np.int32)
    out, l, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                        case.v_cache, case.block_tables, case.context_lens,
                                        case.scale, rows=rows)
    for r, (t, h) in enumerate(rows):
        assert np.array_equal(out[r], full[t, h]) and l[r] == lse[t, h]


def test_bf16_rounding_helper():
    x = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 1e-3, 65504.0], np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(W.bf16_round(x), want)
    rng = np.random.Generator(np.random.PCG64(3))
    y = rng.standard_normal(10000, dtype=np.float32)
    assert np.array_equal(W.bf16_round(y), torch.from_numpy(y).to(torch.bfloat16).float().numpy())
