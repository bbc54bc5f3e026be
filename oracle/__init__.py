"""TEST INFRASTRUCTURE — the CPU fp64 oracle for relay attention.

This package is what the HIP library is checked against; it is not part of the
product.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
may import it.  It imports nothing from the HIP package and shares no code
with it.

What it computes is the paper's definition of causal attention (Sec. 3.3,
Eq. 4) over the concatenated [system ; context] key/value sequence, in double
precision, plus the natural-log log-sum-exp of App. A (Eq. 12).  The split
("relay") form of Eq. 5-7 is never used here.

Parity pins (all in tests/test_oracle_pins.py, none of them calls back into
this package for its expected value):
  * a hand-derived worked example (tests/golden/eq4_worked_example.txt),
  * torch's CPU scaled_dot_product_attention in fp64 on the dense, gathered
    sequence, and scipy's logsumexp for beta,
  * closed forms (q = 0, one visible position, one dominant key, equal keys),
  * logit-shift invariance, exactness of the relay fusion (Eq. 7 with Eq. 11)
    at every split point, request / system-token permutation, physical block
    placement, GQA-by-duplication, prompt-phase rows against truncated decode.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_attn.so")

ORACLE_ERRORS = {
    -1: "bad argument",
    -2: "block-table entry outside the cache",
    -3: "out of memory",
}


def build(force: bool = False) -> str:
    """Compile attention_oracle.c with gcc (-O2, OpenMP) into a shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        f = lib.oracle_attention_rows
        f.restype = ctypes.c_int
        P = ctypes.c_void_p
        I = ctypes.c_int
        f.argtypes = [I, I, I, I, I, I, ctypes.c_double, P, P, P, P, P, P, P, I, I, P, I,
                      I, P, P, P, P, I, P]
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def attention_rows(q, token_request, token_visible, k_sys, v_sys, k_cache, v_cache,
                   block_tables, scale, rows=None, n_threads=0):
    """Eq. 4 for selected (token, head) rows.

    q [n_tokens, Hq, d]; k_sys/v_sys [s, Hkv, d]; k_cache/v_cache
    [num_blocks, Hkv, block_size, d]; block_tables [n_requests, max_blocks].
    `rows` is an int array [n_rows, 2] of (token, head) pairs, or None for all.
    Returns (out [n_rows, d] float64, lse [n_rows] float64, threads_used).
    """
    lib = _load()
    q = _f32(q)
    k_sys, v_sys = _f32(k_sys), _f32(v_sys)
    k_cache, v_cache = _f32(k_cache), _f32(v_cache)
    block_tables = _i32(block_tables)
    token_request, token_visible = _i32(token_request), _i32(token_visible)
    n_tokens, Hq, d = q.shape
    s, Hkv, d2 = k_sys.shape
    num_blocks, Hkv2, block_size, d3 = k_cache.shape
    assert v_sys.shape == k_sys.shape and v_cache.shape == k_cache.shape
    assert d2 == d and d3 == d and Hkv2 == Hkv
    n_requests, max_blocks = block_tables.shape
    assert token_request.shape == (n_tokens,) and token_visible.shape == (n_tokens,)
    if rows is None:
        tt, hh = np.meshgrid(np.arange(n_tokens), np.arange(Hq), indexing="ij")
        rows = np.stack([tt.ravel(), hh.ravel()], axis=1)
    rows = _i32(rows)
    n_rows = rows.shape[0]
    row_token = np.ascontiguousarray(rows[:, 0])
    row_head = np.ascontiguousarray(rows[:, 1])
    out = np.zeros((n_rows, d), dtype=np.float64)
    lse = np.zeros((n_rows,), dtype=np.float64)
    used = ctypes.c_int(0)

    def p(a):
        return a.ctypes.data_as(ctypes.c_void_p)

    rc = lib.oracle_attention_rows(
        n_tokens, n_requests, Hq, Hkv, d, s, float(scale), p(q), p(token_request),
        p(token_visible), p(k_sys), p(v_sys), p(k_cache), p(v_cache), num_blocks, block_size,
        p(block_tables), max_blocks, n_rows, p(row_token), p(row_head), p(out), p(lse),
        int(n_threads), ctypes.byref(used))
    if rc != 0:
        raise ValueError("oracle: " + ORACLE_ERRORS.get(rc, "error %d" % rc))
    return out, lse, used.value


def decode_attention(q, k_sys, v_sys, k_cache, v_cache, block_tables, context_lens, scale,
                     rows=None, n_threads=0):
    """One decode step (Alg. 1, generation phase): token i is request i and sees its
    whole context of context_lens[i] positions.  q [B, Hq, d].
    Returns (out, lse, threads): [B, Hq, d] and [B, Hq] when rows is None."""
    B, Hq, d = q.shape
    out, lse, used = attention_rows(q, np.arange(B), context_lens, k_sys, v_sys, k_cache,
                                    v_cache, block_tables, scale, rows, n_threads)
    if rows is None:
        out, lse = out.reshape(B, Hq, d), lse.reshape(B, Hq)
    return out, lse, used


def prefill_attention(q, cu_seqlens_q, k_sys, v_sys, k_cache, v_cache, block_tables,
                      context_lens, scale, rows=None, n_threads=0):
    """Prompt phase (Alg. 1 with more than one new token): request i owns packed query
    tokens cu_seqlens_q[i]..cu_seqlens_q[i+1]; its context of context_lens[i] positions
    ends with those m_i new tokens, and new token j sees context positions
    0..c_i-m_i+j.  q [total_q, Hq, d]."""
    cu = np.asarray(cu_seqlens_q, dtype=np.int64)
    total_q, Hq, d = q.shape
    req = np.zeros(total_q, dtype=np.int32)
    vis = np.zeros(total_q, dtype=np.int32)
    for i in range(len(cu) - 1):
        m = int(cu[i + 1] - cu[i])
        c = int(context_lens[i])
        if m > c:
            raise ValueError("request %d: more new tokens than context positions" % i)
        req[cu[i]:cu[i + 1]] = i
        vis[cu[i]:cu[i + 1]] = c - m + np.arange(m) + 1
    out, lse, used = attention_rows(q, req, vis, k_sys, v_sys, k_cache, v_cache,
                                    block_tables, scale, rows, n_threads)
    if rows is None:
        out, lse = out.reshape(total_q, Hq, d), lse.reshape(total_q, Hq)
    return out, lse, used


def cache_append(k_cache, v_cache, block_tables, context_lens, k_new, v_new, cu_seqlens_q=None):
    """The cache write that precedes attention in Alg. 1 ("kv_cache[.., l_cache:l_new] = k, v"),
    written out with plain indexing, one position at a time.

    context_lens[i] is l_new, the length AFTER the write; request i's m_i new tokens (one per
    request when cu_seqlens_q is None, else cu_seqlens_q[i+1] - cu_seqlens_q[i]) are therefore
    context positions l_cache = l_new - m_i .. l_new - 1.  Position p of request i lives in
    physical block block_tables[i][p // block_size] at offset p % block_size.
    k_new / v_new [total_new, Hkv, d].  Returns new (k_cache, v_cache); the inputs are not
    modified.  (No pin outside tests/test_oracle_pins.py is needed to read it: see there.)"""
    k_out = np.array(k_cache, dtype=np.float32, copy=True)
    v_out = np.array(v_cache, dtype=np.float32, copy=True)
    num_blocks, _, block_size, _ = k_out.shape
    n_req = len(context_lens)
    if cu_seqlens_q is None:
        cu_seqlens_q = np.arange(n_req + 1)
    for i in range(n_req):
        first_new = int(cu_seqlens_q[i])
        m = int(cu_seqlens_q[i + 1]) - first_new
        l_new = int(context_lens[i])
        l_cache = l_new - m
        if l_cache < 0:
            raise ValueError("request %d: more new tokens than context positions" % i)
        for j in range(m):
            p = l_cache + j
            blk = int(block_tables[i][p // block_size])
            if blk < 0 or blk >= num_blocks:
                raise ValueError("oracle: " + ORACLE_ERRORS[-2])
            k_out[blk, :, p % block_size, :] = k_new[first_new + j]
            v_out[blk, :, p % block_size, :] = v_new[first_new + j]
    return k_out, v_out
