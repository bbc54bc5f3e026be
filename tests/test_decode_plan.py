"""CPU checks of the decode work decomposition (host side of relay_attn_decode): the plan the
library reports is replayed here with the rule the header states for the context wavefronts, over
random context lengths, and must cover every 32-position tile of every context item exactly once
within the stated slot and block-table bounds."""
import numpy as np
import pytest

import paper_2402_14808_amd as ra


def _params(B, Hq, Hkv, s, max_ctx, bs=16, d=128, **kw):
    p = ra.RAParams()
    p.batch, p.num_q_heads, p.num_kv_heads, p.head_dim = B, Hq, Hkv, d
    p.sys_len, p.block_size, p.num_blocks = s, bs, 1 << 20
    p.max_blocks_per_seq = (max_ctx + bs - 1) // bs
    p.max_context_len, p.softmax_scale = max_ctx, 0.1
    p.q_stride_token, p.q_stride_head = Hq * d, d
    p.o_stride_token, p.o_stride_head = Hq * d, d
    p.sys_stride_token, p.sys_stride_head = Hkv * d, d
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _replay(plan, lens, Hkv, bs):
    """Returns {(req, g): [(slot, tile_begin, tile_end), ...]} following the header's rule."""
    tiles = np.maximum(1, (lens + 31) // 32)
    N = int(tiles.sum()) * Hkv
    W = plan.num_ctx_wavefronts
    floor = plan.min_tiles_per_ctx_wavefront
    cap = max(1, (plan.max_blocks_per_span - 1) * bs // 32)     # most tiles a span may have

    def class_len(i, per_wg, extra, fix):
        if fix:
            return fix
        q = per_wg + (1 if (i >> 2) < extra else 0)
        return (q >> 2) + (1 if (i & 3) < (q & 3) else 0)

    lb, nl = W, 0
    l_per_wg = l_fix = l_total = 0
    if plan.num_light_ctx_wavefronts and W > plan.num_light_ctx_wavefronts:
        lb, nl = plan.first_light_ctx_wavefront, plan.num_light_ctx_wavefronts
        per_unit = (plan.sys_tiles_total + N) // 256
        l4 = max(per_unit - plan.sys_workgroup_tiles, 0)
        if l4 // 4 >= floor:
            l_per_wg, l_total = l4, l4 * (nl // 4)
        else:
            l_fix = floor if 2 * (l4 // 4) >= floor else 0
            l_total = l_fix * nl
        if l_total > N:
            l_per_wg = l_fix = l_total = 0

    def share_heavy(n_waves):
        rest, n_wg = N - l_total, n_waves // 4
        per = rest // n_wg
        if per // 4 >= floor:
            return per, rest - per * n_wg, 0
        return per, 0, floor
    h_per_wg, h_extra, h_fix = share_heavy(W - nl if nl else W)
    if nl:
        most_l = l_fix if l_fix else (l_per_wg + 3) >> 2
        most_h = h_fix if h_fix else (h_per_wg + (1 if h_extra else 0) + 3) >> 2
        if most_l > cap or most_h > cap:
            lb, nl = W, 0
            l_per_wg = l_fix = l_total = 0
            h_per_wg, h_extra, h_fix = share_heavy(W)
    begins, at = [], 0
    for w in range(W):
        begins.append(at)
        if lb <= w < lb + nl:
            at += class_len(w - lb, l_per_wg, 0, l_fix)
        else:
            at += class_len(w if w < lb else w - nl, h_per_wg, h_extra, h_fix)
    begins.append(at)
    assert at >= N
    first = {}
    at = 0
    for r, T in enumerate(tiles):
        for g in range(Hkv):
            first[(r, g)] = at
            at += int(T)
    items = sorted(first, key=first.get)
    starts = np.array([first[i] for i in items])
    cover = {i: [] for i in items}
    import bisect

    order = [w for w in range(W) if begins[w + 1] > begins[w]]     # wavefronts that have a span
    number = {w: k for k, w in enumerate(order)}                    # slot numbers count those only
    starts_of = [begins[w] for w in order]

    def span_of(x):
        return bisect.bisect_right(starts_of, x) - 1
    for w in order:
        x0, x1 = begins[w], min(begins[w + 1], N)
        x = x0
        while x < x1:
            k = int(np.searchsorted(starts, x, side="right")) - 1
            item = items[k]
            T = int(tiles[item[0]])
            j = x - first[item]
            seg = min(x1 - x, T - j)
            slot = number[w] - span_of(first[item])
            cover[item].append((slot, j, j + seg))
            span_tokens = min(int(lens[item[0]]), 32 * (j + seg)) - 32 * j
            if span_tokens > 0:
                blocks = (32 * j + span_tokens - 1) // bs - (32 * j) // bs + 1
                assert blocks <= plan.max_blocks_per_span
            x += seg
    return cover, tiles


CASES = [
    # B, Hq, Hkv, s, max_ctx, bs, length distribution
    (32, 52, 52, 2048, 128, 16, "full"),
    (32, 52, 52, 16384, 128, 16, "full"),
    (32, 52, 52, 512, 256, 16, "uniform"),
    (128, 32, 8, 8192, 1024, 16, "uniform"),
    (5, 4, 4, 300, 200, 16, "uniform"),
    (7, 8, 1, 33, 90, 8, "uniform"),
    (3, 4, 4, 0, 5000, 16, "one_long"),
    (70, 2, 2, 515, 700, 16, "uniform"),
    (200, 8, 2, 1000, 3000, 1, "one_long"),
    (4, 4, 4, 256, 64, 16, "zeros"),
    (9, 16, 16, 4096, 32768, 32, "uniform"),
    # small blocks: a span may cover few tiles only (255 blocks), close to the average share
    (32, 4, 4, 1024, 3072, 1, "full"),
    (32, 8, 8, 2048, 6336, 4, "full"),
    (32, 8, 8, 2048, 6336, 4, "uniform"),
    (16, 8, 8, 4096, 1800, 1, "full"),
]


@pytest.mark.parametrize("B,Hq,Hkv,s,max_ctx,bs,dist", CASES)
@pytest.mark.parametrize("part", [0, 128, 512])
def test_context_stream_is_covered_exactly_once(B, Hq, Hkv, s, max_ctx, bs, dist, part):
    p = _params(B, Hq, Hkv, s, max_ctx, bs, ctx_part_tokens=part)
    try:
        plan = ra.relay_attn_decode_plan(p)
    except ra.RelayAttnError as e:
        # a fixed span that cannot fit the block-id table is refused, never truncated
        assert part * 1.0 / bs > plan_cap() - 1 and e.status == ra.binding.RA_ERR_UNSUPPORTED
        return
    assert plan.num_ctx_wavefronts % 4 == 0 and plan.num_ctx_wavefronts > 0
    assert plan.num_ctx_slots >= 2
    rng = np.random.Generator(np.random.PCG64(B * 1000 + s + part))
    for trial in range(3):
        if dist == "full":
            lens = np.full(B, max_ctx)
        elif dist == "uniform":
            lens = rng.integers(0, max_ctx, size=B, endpoint=True)
        elif dist == "zeros":
            lens = np.zeros(B, dtype=np.int64)
        else:
            lens = rng.integers(0, 40, size=B)
            lens[rng.integers(0, B)] = max_ctx
        cover, tiles = _replay(plan, lens, Hkv, bs)
        for (r, g), segs in cover.items():
            segs.sort()
            assert [sl for sl, _, _ in segs] == list(range(len(segs)))         # slots 0..n-1
            assert len(segs) <= plan.num_ctx_slots
            assert segs[0][1] == 0 and segs[-1][2] == tiles[r]
            for (_, _, e0), (_, b1, _) in zip(segs, segs[1:]):
                assert e0 == b1                                                 # contiguous


def plan_cap():
    return ra.relay_attn_decode_plan(_params(1, 1, 1, 0, 32)).max_blocks_per_span


def test_system_chunks_cover_the_prompt_and_fill_the_machine():
    for s in (1, 31, 512, 2048, 5000, 16384):
        p = _params(32, 52, 52, s, 128)
        plan = ra.relay_attn_decode_plan(p)
        assert plan.sys_chunk_tokens % 32 == 0
        assert (plan.num_sys_chunks - 1) * plan.sys_chunk_tokens < s <= plan.num_sys_chunks * plan.sys_chunk_tokens
        assert plan.num_sys_workgroups == 52 * plan.num_sys_chunks
        # the Llama-30B-shaped launches are one machine-full (512 resident workgroups) or less
        assert plan.num_sys_workgroups + plan.num_ctx_wavefronts // 4 <= 512
    # the workspace covers the partials of the plan
    p = _params(32, 52, 52, 2048, 128)
    plan = ra.relay_attn_decode_plan(p)
    rows = 32 * 52
    need = (plan.num_sys_chunks + plan.num_ctx_slots) * rows * (128 + 1) * 4
    assert ra.relay_attn_workspace_bytes(p, 32) >= need


def test_wide_grouped_query_batches_take_many_rows_system_items():
    # (B, Hq, Hkv, s, max_ctx) -> expected stacked rows per system workgroup
    for (B, Hq, Hkv, s, mc), want in (((128, 32, 8, 8192, 1024), 128),     # Llama-3-8B shape
                                      ((64, 32, 8, 8192, 1024), 128),
                                      ((32, 52, 52, 8192, 128), 32),        # one row tile per kv head
                                      ((256, 8, 8, 4096, 1024), 32),        # mostly context
                                      ((128, 32, 8, 512, 1024), 32),
                                      ((128, 32, 8, 0, 1024), 32)):
        p = _params(B, Hq, Hkv, s, mc)
        plan = ra.relay_attn_decode_plan(p)
        assert plan.sys_rows_per_workgroup == want, (B, Hq, Hkv, s, mc)
        if s == 0:
            assert plan.num_sys_workgroups == 0
            continue
        rows_per_head = B * Hq // Hkv
        blocks = -(-rows_per_head // plan.sys_rows_per_workgroup)
        assert plan.num_sys_workgroups == Hkv * blocks * plan.num_sys_chunks
        assert plan.sys_chunk_tokens % 32 == 0
        assert (plan.num_sys_chunks - 1) * plan.sys_chunk_tokens < s <= plan.num_sys_chunks * plan.sys_chunk_tokens
        assert plan.sys_workgroup_tiles == plan.sys_chunk_tokens // 32
        assert plan.sys_tiles_total == Hkv * blocks * -(-s // 32)
        need = (plan.num_sys_chunks + plan.num_ctx_slots) * B * Hq * (128 + 1) * 4
        assert ra.relay_attn_workspace_bytes(p, B) >= need
        if want == 128:
            assert plan.num_sys_chunks <= 16
            assert plan.num_sys_workgroups + plan.num_ctx_wavefronts // 4 <= 512


def test_workspace_covers_the_plan_for_random_parameters():
    rng = np.random.Generator(np.random.PCG64(99))
    for _ in range(300):
        G = int(rng.choice([1, 2, 3, 4, 7, 8]))
        Hkv = int(rng.integers(1, 9))
        B = int(rng.choice([1, 3, 8, 32, 64, 100, 128, 300]))
        s = int(rng.choice([0, 1, 100, 512, 2048, 5000, 16384, 40000]))
        mc = int(rng.choice([1, 40, 128, 1000, 4096, 20000]))
        bs = int(rng.choice([1, 8, 16, 128]))
        d = int(rng.choice([64, 128]))
        kw = {}
        if s and rng.random() < 0.3:
            kw["sys_chunk_tokens"] = 32 * int(rng.integers(1, 40))
        p = _params(B, G * Hkv, Hkv, s, mc, bs, d, **kw)
        try:
            plan = ra.relay_attn_decode_plan(p)
        except ra.RelayAttnError as e:
            assert e.status == ra.binding.RA_ERR_UNSUPPORTED
            continue
        rows = B * G * Hkv
        need = (plan.num_sys_chunks + plan.num_ctx_slots) * rows * (d + 1) * 4
        assert ra.relay_attn_workspace_bytes(p, B) >= need, (B, G, Hkv, s, mc, bs, d, kw)
        assert plan.num_ctx_slots >= 2 and plan.num_ctx_wavefronts % 4 == 0
        if s:
            assert (plan.num_sys_chunks - 1) * plan.sys_chunk_tokens < s <= plan.num_sys_chunks * plan.sys_chunk_tokens
