"""The decode path inside a captured HIP graph: the library allocates nothing, records no memset
and never synchronises, so a step (cache append + both attention launches) can be captured once
and replayed.  Every replay is checked against the eager result, with eager work and
synchronisations between the replays."""
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


def _say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("cfg,seed", [
    (W.AttnConfig("g1", 6, 8, 4, 128, 700, 20, 300), 401),
    (W.llama30b(2048), 402),
])
def test_captured_decode_step_replays_to_the_eager_result(cfg, seed):
    case = W.make_case(cfg, seed)
    _say("%s seed=%d" % (cfg, seed))
    dc = DeviceCase(case)
    want, _, _ = oracle.decode_attention(case.q, case.k_sys, case.v_sys, case.k_cache, case.v_cache,
                                         case.block_tables, case.context_lens, case.scale,
                                         rows=None if cfg.batch * cfg.num_q_heads < 400 else
                                         np.stack([np.arange(64) % cfg.batch, np.arange(64) % cfg.num_q_heads], 1).astype(np.int32))
    out = torch.zeros(cfg.batch, cfg.num_q_heads, cfg.head_dim, device=dc.dev, dtype=torch.float32)
    lse = torch.zeros(cfg.batch, cfg.num_q_heads, device=dc.dev, dtype=torch.float32)
    p = ra.make_params(dc.q, out, dc.k_sys, dc.k_cache, dc.block_tables, batch=cfg.batch,
                       softmax_scale=case.scale, max_context_len=int(case.context_lens.max()))
    ws = dc._workspace(p, cfg.batch)

    def step():
        ra.relay_attn_decode(p, dc.q, dc.k_sys, dc.v_sys, dc.k_cache, dc.v_cache, dc.block_tables,
                             dc.context_lens, out, lse, ws)
    step()
    torch.cuda.synchronize()
    eager = out.cpu().numpy().copy()
    eager_lse = lse.cpu().numpy().copy()

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(4):
        out.fill_(float("nan"))                    # eager work between the replays
        lse.fill_(float("nan"))
        ws.fill_(0xFF)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.array_equal(got, eager) and np.array_equal(lse.cpu().numpy(), eager_lse), replay
    if want.ndim == 3:
        assert np.abs(eager - want).max() <= TOL
    else:
        rows = np.stack([np.arange(64) % cfg.batch, np.arange(64) % cfg.num_q_heads], 1)
        assert np.abs(eager[rows[:, 0], rows[:, 1]] - want).max() <= TOL
