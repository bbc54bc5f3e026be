"""relay_attn_decode_static (the entry point that allocates nothing and takes no workspace)
against relay_attn_decode on the same inputs: bit for bit, on two calls in a row that share the
library's fixed scratch array, the second one smaller; and both against the oracle."""
import ctypes
import sys

import numpy as np
import pytest
import torch

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


def _static(dc, fp32_out=True):
    c = dc.case
    out, lse = dc._outputs(fp32_out)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=c.cfg.batch,
                       softmax_scale=c.scale, max_context_len=int(c.context_lens.max()))
    assert ra.relay_attn_workspace_bytes(p, c.cfg.batch) <= ra.relay_attn_static_scratch_bytes()
    ra.relay_attn_decode_static(p, dc.q, dc.k_sys, dc.v_sys, dc.k_cache, dc.v_cache,
                                dc.block_tables, dc.context_lens, out, lse)
    torch.cuda.synchronize()
    return out.float().cpu().numpy(), lse.cpu().numpy()


def test_static_scratch_entry_matches_the_workspace_entry_twice_in_a_row():
    big = W.make_case(W.llama30b(2048), 7001)
    small = W.make_case(W.AttnConfig("small", 5, 8, 4, 128, 300, 1, 200), 7002)
    for case in (big, small):                       # the second call is the smaller one
        _say("%s seed=%d" % (case.cfg, case.seed))
        dc = DeviceCase(case)
        got, lse = _static(dc)
        ref, rlse = dc.decode()
        assert np.array_equal(got, ref) and np.array_equal(lse, rlse)
        want, wlse, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache,
                                                case.v_cache, case.block_tables,
                                                case.context_lens, case.scale)
        assert np.isfinite(got).all()
        assert np.abs(got - want).max() <= TOL and np.abs(lse - wlse).max() <= LSE_TOL
        b16, _ = _static(dc, fp32_out=False)
        assert np.array_equal(b16, W.bf16_round(ref))


def test_static_scratch_entry_rejects_what_does_not_fit():
    """A batch whose partials exceed the fixed array is refused on the host, before any launch."""
    dev = torch.device("cuda:0")
    B, Hq, Hkv, d = 4096, 32, 8, 128
    q = torch.zeros(B, Hq, d, dtype=torch.bfloat16, device=dev)
    out = torch.zeros_like(q)
    ks = torch.zeros(64, Hkv, d, dtype=torch.bfloat16, device=dev)
    kc = torch.zeros(B, Hkv, 16, d, dtype=torch.bfloat16, device=dev)
    bt = torch.arange(B, dtype=torch.int32, device=dev).view(B, 1)
    cl = torch.ones(B, dtype=torch.int32, device=dev)
    p = ra.make_params(q, out, ks, kc, bt, batch=B, softmax_scale=0.1)
    assert ra.relay_attn_workspace_bytes(p, B) > ra.relay_attn_static_scratch_bytes()
    with pytest.raises(ra.RelayAttnError) as e:
        ra.relay_attn_decode_static(p, q, ks, ks, kc, kc, bt, cl, out, None)
    assert e.value.status == ra.binding.RA_ERR_WORKSPACE_TOO_SMALL


def test_static_scratch_entry_under_graph_capture():
    """The callers the entry point is for: a step captured into a HIP graph (no allocation, no
    workspace to keep alive) and replayed with eager work in between; every replay equals the
    eager result of relay_attn_decode.  The scratch address is looked up by the eager call made
    before the capture."""
    case = W.make_case(W.AttnConfig("cap", 7, 8, 4, 128, 900, 5, 400), 7003)
    _say("%s seed=%d" % (case.cfg, case.seed))
    dc = DeviceCase(case)
    ref, rlse = dc.decode()
    out, lse = dc._outputs(True)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=case.cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))

    def step():
        ra.relay_attn_decode_static(p, dc.q, dc.k_sys, dc.v_sys, dc.k_cache, dc.v_cache,
                                    dc.block_tables, dc.context_lens, out, lse)
    step()
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), ref)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        _static(DeviceCase(W.make_case(W.AttnConfig("other", 3, 4, 4, 64, 100, 1, 50), 7004)))   # another user of the scratch
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), ref) and np.array_equal(lse.cpu().numpy(), rlse), replay
