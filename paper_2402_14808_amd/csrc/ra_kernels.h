// Launch interfaces between the host entry points (relay_attn.hip) and the
// kernel files.  Plain structs passed by value; all pointers are device pointers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ra {

// Partial results live in the caller's workspace: for partial p and output row
// r = token * Hq + head, part_o[(p * rows + r) * D + e] is the normalised partial
// attention output (fp32) and part_lse[p * rows + r] its log-sum-exp in the base-2
// domain (log2 of the sum of 2^(logit * scale * log2 e)); -inf marks an empty partial.

struct CtxArgs {                 // per-request paged decode attention, item = (request, kv head, part)
    const uint16_t *q, *k_cache, *v_cache;
    const int32_t *block_tables, *context_lens;
    const int32_t *cu_seqlens_q;  // null for decode (token i = request i)
    float *part_o, *part_lse;
    void *out;                   // direct mode only (single part, no system prompt)
    float *lse_out;
    int64_t q_stride_token, q_stride_head, o_stride_token, o_stride_head;
    int batch, n_tokens, Hq, Hkv, block_size_log2, max_blocks_per_seq, part_tokens, n_parts, rows;
    int direct, out_is_fp32;
    float scale_log2;
};

constexpr int kMaxPrefixes = 32;  // shared system prompts ("applications", App. D) in one batch

struct TileArgs {                // both partial attentions of a decode step in one launch
    const uint16_t *q, *k_cache, *v_cache;
    // Cache write fused into the launch (Alg. 1 writes the new key/value, then attends): when
    // k_new is not null, context position context_lens[i]-1 of (request i, kv head g) is taken
    // from k_new / v_new + i * new_stride_token + g * new_stride_head and stored to the caches
    // (which are then written through these same pointers).
    const uint16_t *k_new, *v_new;
    int64_t new_stride_token, new_stride_head;
    // Shared prefixes: the requests of prefix p are tokens pfx_first[p] .. +pfx_tokens[p]-1 and
    // attend to pfx_len[p] system positions at pfx_k[p] / pfx_v[p]; system work items of prefix p
    // are grid indices pfx_item_end[p-1] .. pfx_item_end[p]-1.  One prefix = the paper's setting.
    int n_prefixes;
    int pfx_item_end[kMaxPrefixes], pfx_first[kMaxPrefixes], pfx_tokens[kMaxPrefixes],
        pfx_len[kMaxPrefixes];
    const uint16_t *pfx_k[kMaxPrefixes], *pfx_v[kMaxPrefixes];
    // Requests of a prefix in any order (null: prefix p owns tokens pfx_first[p] .. +pfx_tokens[p]-1
    // themselves): req_order lists the requests prefix by prefix, and pfx_first[p] is where prefix
    // p's run begins in it.
    const int32_t *req_order;
    const int32_t *block_tables, *context_lens;
    float *part_o, *part_lse;    // partial p: system chunk p, or n_sys_chunks + context part
    int64_t q_stride_token, q_stride_head, sys_stride_token, sys_stride_head;
    int n_tokens, Hq, Hkv, G, sys_chunk, n_sys_chunks, n_sys_items, sys_read_once;
    // > 0: the system items are many-rows items (kv head, block of 128 stacked rows, chunk), this
    // many row blocks per kv head; 0: streaming items of 32 stacked rows
    int n_sys_rowblocks;
    // context wavefronts in the grid (a multiple of 4), the least tiles one of them takes, context
    // partial slots per row, upper bound on context_lens
    int ctx_waves, ctx_t_floor, n_ctx_slots, max_ctx;
    int ctx_t_cap;               // most tiles a span may have (its block ids must fit the LDS table)
    // context wavefronts that share a compute unit with a system workgroup (0: none known), the
    // tiles of such a system workgroup, and the tiles of all system workgroups together
    int ctx_light_begin, ctx_light_waves, sys_wg_tiles, sys_tiles_total;
    int block_size_log2, max_blocks_per_seq, rows;
    int sys_head_fastest;        // system item order: kv head varies fastest (token-major cache)
    float scale_log2;
    // Measurement aid: when not null, wavefront w of the launch (4 per workgroup) stores the
    // 100 MHz counter at its begin and its end in timeline[2w], timeline[2w+1] (w < timeline_waves).
    unsigned long long *timeline;
    int timeline_waves;
};

struct RowsArgs {                // many query rows per kv head: prompt phase, wide decode batches
    const uint16_t *q, *k_sys, *v_sys, *k_cache, *v_cache;
    const int32_t *block_tables, *context_lens;
    const int32_t *cu_seqlens_q;  // null when there are no context items
    float *part_o, *part_lse;
    // items that carry a block of rows through system prompt and context and write the output
    // themselves (prompt phase, one launch): `whole` != 0, and then
    void *out;
    float *lse_out;               // natural log; may be null
    int64_t o_stride_token, o_stride_head;
    int out_is_fp32, whole, batch;
    unsigned long long *timeline;  // as in TileArgs
    int timeline_waves;
    int64_t q_stride_token, q_stride_head, sys_stride_token, sys_stride_head;
    int n_tokens, Hq, Hkv, G, sys_len, sys_chunk, n_sys_chunks, n_sys_rowblocks, n_sys_items;
    int ctx_part, n_ctx_parts, n_ctx_rowblocks, n_ctx_items;
    int block_size_log2, max_blocks_per_seq, rows, sys_head_fastest;
    float scale_log2;
    // Several shared prefixes in the prompt phase (0 or 1: the fields above describe the only
    // one): prefix p owns the packed tokens pfx_tok0[p] .. +pfx_ntok[p]-1 (its requests are
    // consecutive), attends to pfx_len[p] positions at pfx_k[p] / pfx_v[p], and its system items
    // are launch indices pfx_item_end[p-1] .. pfx_item_end[p]-1.
    int n_prefixes;
    int pfx_item_end[kMaxPrefixes], pfx_tok0[kMaxPrefixes], pfx_ntok[kMaxPrefixes], pfx_len[kMaxPrefixes];
    const uint16_t *pfx_k[kMaxPrefixes], *pfx_v[kMaxPrefixes];
};

constexpr int kMaxPartBlocks = 256;   // block-table entries one context item may span

struct AppendArgs {              // cache append (Alg. 1: write the new K,V before attending)
    const uint16_t *k_new, *v_new;
    uint16_t *k_cache, *v_cache;
    const int32_t *block_tables, *context_lens, *cu_seqlens_q;
    int64_t new_stride_token, new_stride_head;
    int batch, total_q, Hkv, head_dim, block_size_log2, max_blocks_per_seq;
};

struct SysFillArgs {             // offline fill of the shared system cache (Sec. 3.3)
    const uint16_t *k_new, *v_new;
    uint16_t *k_sys, *v_sys;
    int64_t new_stride_token, new_stride_head, sys_stride_token, sys_stride_head;
    int first_pos, num_pos, Hkv, head_dim;
};

struct FuseArgs {                // relay fusion (Alg. 1; Eq. 11 generalised to n partials)
    const float *part_o, *part_lse;
    void *out;
    float *lse_out;
    int64_t o_stride_token, o_stride_head;
    int rows, Hq, n_partials, out_is_fp32;
    // several shared prefixes: rows of tokens below pfx_token_end[p] (and not below the previous
    // end) have only pfx_chunks[p] of the n_sys_chunks system partials
    int n_prefixes, n_sys_chunks, pfx_token_end[kMaxPrefixes], pfx_chunks[kMaxPrefixes];
    const int32_t *req_prefix;   // not null: the prefix of each token (requests in any order)
};

hipError_t launch_ctx_decode(const CtxArgs &a, int head_dim, int group, hipStream_t stream);
hipError_t launch_relay_rows(const RowsArgs &a, int head_dim, hipStream_t stream);
hipError_t launch_relay_tiles(const TileArgs &a, int head_dim, hipStream_t stream);
hipError_t launch_cache_append(const AppendArgs &a, hipStream_t stream);
hipError_t launch_system_fill(const SysFillArgs &a, hipStream_t stream);

struct ValidateArgs {            // device-side range check of lengths and block ids
    const int32_t *block_tables, *context_lens, *cu_seqlens_q;
    int32_t *counters;           // [4]: bad lengths, bad block ids, bad query lengths, first bad request
    int batch, total_q, num_blocks, block_size_log2, max_blocks_per_seq, max_len;
};
hipError_t launch_validate(const ValidateArgs &a, hipStream_t stream);
hipError_t launch_fuse(const FuseArgs &a, int head_dim, hipStream_t stream);
// measurement aids: read `bytes` of `src` once with coalesced 16-byte loads; launch nothing much
hipError_t launch_stream_probe(const void *src, size_t bytes, int nontemporal, void *sink,
                               hipStream_t stream);
hipError_t launch_empty_probe(void *sink, int count, hipStream_t stream);

}  // namespace ra
