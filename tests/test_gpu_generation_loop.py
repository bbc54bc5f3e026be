"""A generation loop on the GPU, checked against the oracle at every step (Alg. 1, generation
phase, repeated: write the new key/value into the paged cache, then attend over [0, l_new)).
Shapes follow the synthetic workloads of App. C: a shared system prompt, user prompts of a fixed
length already cached, then one new token per request and step."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2402_14808_amd as ra
import workloads as W

pytestmark = pytest.mark.gpu
TOL = 2e-3
LSE_TOL = 1e-3


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


def _bf16(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev).to(torch.bfloat16)


@pytest.mark.parametrize("name,B,H,Hkv,s,user_lo,user_hi,steps", [
    ("app_c_64_128", 32, 32, 32, 512, 64, 64, 6),          # (user, generation) = (64, 128), s = 512
    ("ragged_gqa", 9, 8, 2, 300, 1, 70, 5),
    ("no_system_prompt", 4, 4, 4, 0, 15, 17, 4),
])
@pytest.mark.parametrize("fused", [False, True])
def test_generation_loop_matches_oracle_at_every_step(name, B, H, Hkv, s, user_lo, user_hi, steps, fused):
    d, bs = 128, 16
    rng = np.random.Generator(np.random.PCG64(6000 + B))
    user = rng.integers(user_lo, user_hi, size=B, endpoint=True).astype(np.int32)
    final = user + steps
    tables, num_blocks = W.lay_out_blocks(rng, final, bs)
    normal = lambda *shape: W.bf16_round(rng.standard_normal(shape, dtype=np.float32))
    k_sys, v_sys = normal(s, Hkv, d), normal(s, Hkv, d)
    # the cache starts full of NaN: every position the loop reads must have been written
    k_cache = np.full((num_blocks, Hkv, bs, d), np.nan, np.float32)
    v_cache = np.full((num_blocks, Hkv, bs, d), np.nan, np.float32)
    cu = np.concatenate([[0], np.cumsum(user)]).astype(np.int32)
    k_cache, v_cache = oracle.cache_append(k_cache, v_cache, tables, user,
                                           normal(int(cu[-1]), Hkv, d), normal(int(cu[-1]), Hkv, d), cu)
    dev = torch.device("cuda:0")
    kc_d, vc_d = _bf16(k_cache, dev), _bf16(v_cache, dev)
    ks_d, vs_d = _bf16(k_sys, dev), _bf16(v_sys, dev)
    tables_d = torch.from_numpy(tables).to(dev)
    lens = user.copy()
    lens_d = torch.from_numpy(lens).to(dev)
    out = torch.empty(B, H, d, device=dev, dtype=torch.float32)
    lse = torch.empty(B, H, device=dev, dtype=torch.float32)
    q0 = _bf16(normal(B, H, d), dev)
    p = ra.make_params(q0, out, ks_d if s else None, kc_d, tables_d, batch=B, softmax_scale=d ** -0.5,
                       max_context_len=int(final.max()))
    ws = torch.full((ra.relay_attn_workspace_bytes(p, B),), 0xFF, dtype=torch.uint8, device=dev)
    for t in range(steps):
        q = normal(B, H, d)
        # the step's projections arrive as one fused [B, (q|k|v) heads, d] tensor
        k_new, v_new = normal(B, Hkv, d), normal(B, Hkv, d)
        lens = lens + 1
        k_cache, v_cache = oracle.cache_append(k_cache, v_cache, tables, lens, k_new, v_new)
        want, wlse, _ = oracle.decode_attention(q, k_sys, v_sys, k_cache, v_cache, tables, lens,
                                                d ** -0.5)
        _say("%s fused=%s step %d lens %d..%d" % (name, fused, t, lens.min(), lens.max()))
        q_d = _bf16(q, dev)
        kv_d = _bf16(np.concatenate([k_new, v_new], axis=1), dev)
        kn_d, vn_d = kv_d[:, :Hkv], kv_d[:, Hkv:]
        lens_d += 1
        out.fill_(float("nan"))
        if fused:
            ra.relay_attn_decode_append(p, q_d, kn_d, vn_d, ks_d, vs_d, kc_d, vc_d, tables_d, lens_d,
                                        out, lse, ws)
        else:
            ra.relay_attn_cache_append(p, kn_d, vn_d, None, B, kc_d, vc_d, tables_d, lens_d)
            ra.relay_attn_decode(p, q_d, ks_d, vs_d, kc_d, vc_d, tables_d, lens_d, out, lse, ws)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        err = np.abs(got - want).max()
        lerr = np.abs(lse.cpu().numpy() - wlse).max()
        _say("max-abs err %.3e lse err %.3e" % (err, lerr))
        assert np.isfinite(got).all() and err <= TOL and lerr <= LSE_TOL
        # the cache itself: byte-exact (NaN where nothing was written yet)
        assert np.array_equal(kc_d.float().cpu().numpy(), k_cache, equal_nan=True)
        assert np.array_equal(vc_d.float().cpu().numpy(), v_cache, equal_nan=True)
