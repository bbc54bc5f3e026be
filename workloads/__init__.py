"""Seeded synthetic inputs shared by the oracle-side tests and the HIP-side tests.

This module holds none of the method's arithmetic: it draws random numbers,
rounds them once to bfloat16, and lays out paged caches and block tables.  It
imports neither the oracle nor the HIP package.

Recipe (stands in for the chatbot / few-shot workloads of Sec. 4.1, Table 1,
whose data are not needed for a standalone attention layer; only their shapes
matter): values are standard normal float32 from numpy's PCG64 seeded with the
given seed, rounded to bfloat16 (round-to-nearest-even) and stored as float32;
context lengths are uniform integers in [ctx_lo, ctx_hi]; physical cache
blocks are a random permutation of a pool with >= 10 % spare blocks; unused
block-table slots hold a poison index; in parity mode the unused tail of each
request's last block is filled with NaN.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace

import numpy as np

POISON_BLOCK = 0x7FFFFFF0  # never dereferenced by a correct implementation


@dataclass(frozen=True)
class AttnConfig:
    name: str
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    sys_len: int
    ctx_lo: int
    ctx_hi: int
    block_size: int = 16
    # prompt phase only: new query tokens per request, uniform in [q_lo, q_hi]
    q_lo: int = 1
    q_hi: int = 1

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)


# The workload shapes this build is measured and tested on.
TINY = AttnConfig("tiny", 4, 4, 4, 64, 256, 16, 64)
LLAMA7B = AttnConfig("llama7b", 32, 32, 32, 128, 2048, 128, 128)


def llama30b(sys_len: int) -> AttnConfig:
    return AttnConfig("llama30b_s%d" % sys_len, 32, 52, 52, 128, sys_len, 128, 128)


LLAMA30B_SWEEP = (512, 1024, 2048, 4096, 8192, 16384)
LLAMA3_8B_GQA = AttnConfig("llama3_8b_gqa", 128, 32, 8, 128, 8192, 64, 1024)
LLAMA13B_PREFILL = AttnConfig("llama13b_prefill", 16, 40, 40, 128, 4096, 64, 512,
                              q_lo=64, q_hi=512)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    out = (r & 0xFFFFFFFF).astype(np.uint32).view(np.float32)
    return np.where(np.isnan(x), x, out).astype(np.float32).reshape(x.shape)


def _normal_bf16(rng, shape):
    return bf16_round(rng.standard_normal(shape, dtype=np.float32))


@dataclass
class AttnCase:
    cfg: AttnConfig
    seed: int
    q: np.ndarray              # [n_tokens, Hq, d]  (decode: n_tokens == batch)
    k_sys: np.ndarray          # [s, Hkv, d]
    v_sys: np.ndarray
    k_cache: np.ndarray        # [num_blocks, Hkv, block_size, d]
    v_cache: np.ndarray
    block_tables: np.ndarray   # [batch, max_blocks] int32
    context_lens: np.ndarray   # [batch] int32 (includes the tokens being processed)
    cu_seqlens_q: np.ndarray   # [batch+1] int32 (decode: arange)

    @property
    def scale(self) -> float:
        return self.cfg.scale

    @property
    def num_blocks(self) -> int:
        return self.k_cache.shape[0]

    @property
    def max_blocks(self) -> int:
        return self.block_tables.shape[1]


def lay_out_blocks(rng, context_lens, block_size, spare=0.10, identity=False,
                   min_table_width=0):
    """Give each request ceil(c/bs) distinct physical blocks. Returns (tables, num_blocks)."""
    need = [(int(c) + block_size - 1) // block_size for c in context_lens]
    total = sum(need)
    pool = int(math.ceil(total * (1.0 + spare))) + 1
    order = np.arange(pool) if identity else rng.permutation(pool)
    width = max(max(need) if need else 0, 1, min_table_width)
    tables = np.full((len(need), width), POISON_BLOCK, dtype=np.int32)
    at = 0
    for i, n in enumerate(need):
        tables[i, :n] = order[at:at + n]
        at += n
    return tables, pool


def make_case(cfg: AttnConfig, seed: int, poison_tails: bool = True,
              identity_blocks: bool = False, prefill: bool = False,
              extra_context: bool = False) -> AttnCase:
    """Draw one batch.  Decode: one query token per request.  Prefill: q_lo..q_hi new
    tokens per request whose context is those tokens (plus, with extra_context, an
    already cached part of ctx_lo..ctx_hi more positions)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    B, Hq, Hkv, d, s, bs = (cfg.batch, cfg.num_q_heads, cfg.num_kv_heads, cfg.head_dim,
                            cfg.sys_len, cfg.block_size)
    if prefill:
        m = rng.integers(cfg.q_lo, cfg.q_hi, size=B, endpoint=True).astype(np.int32)
        ctx = m.copy()
        if extra_context:
            ctx = ctx + rng.integers(cfg.ctx_lo, cfg.ctx_hi, size=B, endpoint=True).astype(np.int32)
    else:
        m = np.ones(B, dtype=np.int32)
        ctx = rng.integers(cfg.ctx_lo, cfg.ctx_hi, size=B, endpoint=True).astype(np.int32)
    cu = np.zeros(B + 1, dtype=np.int32)
    cu[1:] = np.cumsum(m)
    q = _normal_bf16(rng, (int(cu[-1]), Hq, d))
    k_sys = _normal_bf16(rng, (s, Hkv, d))
    v_sys = _normal_bf16(rng, (s, Hkv, d))
    tables, num_blocks = lay_out_blocks(rng, ctx, bs, identity=identity_blocks)
    k_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    v_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    if poison_tails:
        for i in range(B):
            c = int(ctx[i])
            if c % bs:
                blk = tables[i, c // bs]
                k_cache[blk, :, c % bs:, :] = np.nan
                v_cache[blk, :, c % bs:, :] = np.nan
    return AttnCase(cfg, seed, q, k_sys, v_sys, k_cache, v_cache, tables, ctx, cu)


def logical_context(case: AttnCase, i: int):
    """Gather request i's context K and V as dense [c_i, Hkv, d] arrays."""
    c = int(case.context_lens[i])
    bs = case.cfg.block_size
    nb = (c + bs - 1) // bs
    blks = case.block_tables[i, :nb]
    Hkv, d = case.cfg.num_kv_heads, case.cfg.head_dim
    k = case.k_cache[blks].transpose(0, 2, 1, 3).reshape(nb * bs, Hkv, d)[:c]
    v = case.v_cache[blks].transpose(0, 2, 1, 3).reshape(nb * bs, Hkv, d)[:c]
    return k, v


def repage(case: AttnCase, seed: int, identity: bool = False) -> AttnCase:
    """Same logical contents, different physical block placement."""
    rng = np.random.Generator(np.random.PCG64(seed))
    bs = case.cfg.block_size
    tables, num_blocks = lay_out_blocks(rng, case.context_lens, bs, identity=identity,
                                        min_table_width=case.max_blocks)
    Hkv, d = case.cfg.num_kv_heads, case.cfg.head_dim
    k_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    v_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    for i in range(case.cfg.batch):
        c = int(case.context_lens[i])
        nb = (c + bs - 1) // bs
        # copy whole blocks, tails included, so that poison travels with them
        k_cache[tables[i, :nb]] = case.k_cache[case.block_tables[i, :nb]]
        v_cache[tables[i, :nb]] = case.v_cache[case.block_tables[i, :nb]]
    return replace(case, k_cache=k_cache, v_cache=v_cache, block_tables=tables)


def from_dense(cfg: AttnConfig, q, k_sys, v_sys, ctx_k, ctx_v, seed=0, cu_seqlens_q=None,
               poison_tails=True) -> AttnCase:
    """Build a paged case from dense per-request context arrays ctx_k[i], ctx_v[i] of shape
    [c_i, Hkv, d] (values must already be bfloat16-representable)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    bs = cfg.block_size
    B = len(ctx_k)
    ctx = np.array([k.shape[0] for k in ctx_k], dtype=np.int32)
    tables, num_blocks = lay_out_blocks(rng, ctx, bs)
    Hkv, d = cfg.num_kv_heads, cfg.head_dim
    k_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    v_cache = _normal_bf16(rng, (num_blocks, Hkv, bs, d))
    for i in range(B):
        c = int(ctx[i])
        for j in range(c):
            blk = tables[i, j // bs]
            k_cache[blk, :, j % bs, :] = ctx_k[i][j]
            v_cache[blk, :, j % bs, :] = ctx_v[i][j]
        if poison_tails and c % bs:
            blk = tables[i, c // bs]
            k_cache[blk, :, c % bs:, :] = np.nan
            v_cache[blk, :, c % bs:, :] = np.nan
    if cu_seqlens_q is None:
        cu_seqlens_q = np.arange(B + 1, dtype=np.int32)
    cfg2 = replace(cfg, batch=B, sys_len=int(np.asarray(k_sys).shape[0]))
    return AttnCase(cfg2, seed, np.ascontiguousarray(q, dtype=np.float32),
                    np.ascontiguousarray(k_sys, dtype=np.float32),
                    np.ascontiguousarray(v_sys, dtype=np.float32),
                    k_cache, v_cache, tables, ctx, np.asarray(cu_seqlens_q, dtype=np.int32))


def with_system_pages(case: AttnCase) -> AttnCase:
    """The per-request ("no relay") view of the same batch: the system key/values are
    stored once as shared cache pages and every request's block table lists them before
    its own blocks, so a per-request paged kernel re-reads them for each request.
    Needs sys_len to be a multiple of the block size.  The result has sys_len 0."""
    cfg = case.cfg
    bs, s = cfg.block_size, cfg.sys_len
    if s % bs:
        raise ValueError("system length must be a multiple of the block size")
    nsb = s // bs
    Hkv, d = cfg.num_kv_heads, cfg.head_dim
    sys_k = case.k_sys.reshape(nsb, bs, Hkv, d).transpose(0, 2, 1, 3)
    sys_v = case.v_sys.reshape(nsb, bs, Hkv, d).transpose(0, 2, 1, 3)
    nb0 = case.num_blocks
    k_cache = np.concatenate([case.k_cache, sys_k], axis=0)
    v_cache = np.concatenate([case.v_cache, sys_v], axis=0)
    B = cfg.batch
    tables = np.full((B, nsb + case.max_blocks), POISON_BLOCK, dtype=np.int32)
    tables[:, :nsb] = nb0 + np.arange(nsb, dtype=np.int32)[None, :]
    tables[:, nsb:] = case.block_tables
    empty = np.zeros((0, Hkv, d), dtype=np.float32)
    return replace(case, cfg=replace(cfg, sys_len=0), k_sys=empty, v_sys=empty,
                   k_cache=np.ascontiguousarray(k_cache), v_cache=np.ascontiguousarray(v_cache),
                   block_tables=tables,
                   context_lens=(case.context_lens + s).astype(np.int32))


def make_prefix_groups(case: AttnCase, seed: int, group_sizes, sys_lens):
    """Split the decode batch of `case` into consecutive groups that each have a system
    prompt of their own (the multi-application setting of App. D).  Returns a list of
    (first_request, num_requests, k_sys, v_sys) with k_sys/v_sys of shape [s_i, Hkv, d]."""
    assert sum(group_sizes) == case.cfg.batch and len(group_sizes) == len(sys_lens)
    rng = np.random.Generator(np.random.PCG64(seed))
    groups, first = [], 0
    for n, s in zip(group_sizes, sys_lens):
        shape = (int(s), case.cfg.num_kv_heads, case.cfg.head_dim)
        groups.append((first, int(n), _normal_bf16(rng, shape), _normal_bf16(rng, shape)))
        first += int(n)
    return groups
