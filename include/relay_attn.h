/*
 * relay_attn.h — C ABI of the MI355X (gfx950) relay-attention library.
 *
 * RelayAttention (arXiv 2402.14808, Sec. 3.3, Alg. 1) computes exact causal
 * attention for a batch of requests that all start with the same system
 * prompt, reading the system prompt's keys/values from device memory once per
 * batch instead of once per request:
 *
 *   system attention   every query of the batch against the shared system KV,
 *                      grouped into one matrix product per KV head
 *                      (Alg. 1 "system attention"; Eq. 7, first term);
 *   context attention  every query against its own request's paged KV
 *                      (Alg. 1 "context attention"; Eq. 7, second term);
 *   relay fusion       out = alpha_sys * o_sys + (1 - alpha_sys) * o_ctx with
 *                      alpha_sys = 1 / (1 + exp(lse_ctx - lse_sys))
 *                      (Alg. 1 "relay fusion"; App. A, Eq. 11-12).
 *
 * The result equals full attention over [system ; context] (Eq. 4-7).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers on the current HIP device unless a
 *     parameter says "host".  The library never allocates, frees or copies
 *     device memory and never synchronises: it validates the scalar arguments
 *     on the host, then enqueues kernels on `hip_stream` (a hipStream_t passed
 *     as void*; NULL is the default stream) and returns.  The one HIP query it
 *     makes outside a launch is the device's compute-unit count, read once per
 *     process and cached (256 is assumed where no device answers).
 *   - The caller owns every buffer.  Inputs are read only; only `out`,
 *     `lse_out` and `workspace` are written (and the caches by the entry points
 *     whose job is to write them).
 *   - Length bounds are promises, not checks.  max_context_len (and max_q_len
 *     in the prompt phase) size the launch; a request whose real length exceeds
 *     the bound is silently attended over its first max_context_len positions
 *     only (a stale bound gives a wrong answer and RA_OK).  Only
 *     relay_attn_debug_validate reports such a request.
 *   - 16-bit floating data are bfloat16.  The innermost (head_dim) index of q,
 *     out, k_sys, v_sys and the caches is contiguous; every row start must be
 *     16-byte aligned (base pointers 16-byte aligned, strides multiples of 8
 *     elements).
 *   - Errors are returned as ra_status, never thrown.  All argument checks
 *     happen before the first HIP call, so they behave the same on a machine
 *     without a GPU.  Contents of device arrays (block-table entries, context
 *     lengths) are trusted: an entry that points outside the cache is
 *     undefined behaviour, as with any paged-attention kernel.
 *
 * Paged context cache (the paper inherits it from PagedAttention, App. A, and
 * does not fix a layout; this is ours):
 *   k_cache, v_cache   [num_blocks][num_kv_heads][block_size][head_dim] bf16
 *   block_tables       [batch][max_blocks_per_seq] int32, row i lists the
 *                      physical blocks of request i in logical order; slots at
 *                      or beyond ceil(context_lens[i] / block_size) are never
 *                      read
 *   context_lens       [batch] int32, number of cached positions of request i
 *                      INCLUDING the token(s) being processed (Alg. 1 appends
 *                      the new key/value before attending).  Positions at or
 *                      beyond it in the last block are never read.
 * Shared system cache (Sec. 3.3 "Peripheral adaptations": kept apart from the
 * request caches and filled before serving):
 *   k_sys, v_sys       sys_len x num_kv_heads x head_dim bf16, addressed as
 *                      base + token * sys_stride_token + head * sys_stride_head
 * Query head h uses KV head h / (num_q_heads / num_kv_heads).
 */
#ifndef RELAY_ATTN_H
#define RELAY_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RA_OK = 0,
    RA_ERR_INVALID_ARG = 1,         /* null pointer, negative size, misalignment, ... */
    RA_ERR_UNSUPPORTED = 2,         /* head_dim not in {64,128}, Hq/Hkv above 8, ...   */
    RA_ERR_WORKSPACE_TOO_SMALL = 3,
    RA_ERR_HIP = 4                  /* a HIP call (launch) failed                       */
} ra_status;

typedef struct {
    int32_t batch;                /* B  >= 0 requests                                    */
    int32_t num_q_heads;          /* Hq >= 1                                             */
    int32_t num_kv_heads;         /* Hkv >= 1, divides Hq; Hq/Hkv in 1 .. 8                */
    int32_t head_dim;             /* 64 or 128                                           */
    int32_t sys_len;              /* s >= 0 shared system positions                      */
    int32_t block_size;           /* tokens per cache block: 8, 16, 32, ... (power of 2) */
    int32_t num_blocks;           /* blocks in k_cache / v_cache                         */
    int32_t max_blocks_per_seq;   /* row length of block_tables                          */
    int32_t max_context_len;      /* host-side upper bound on context_lens[i]; 0 means
                                     max_blocks_per_seq * block_size.  Lengths above it
                                     are truncated to it without an error (see above)   */
    float   softmax_scale;        /* multiplies every logit (the paper folds it into q) */
    int64_t q_stride_token, q_stride_head;      /* elements                              */
    int64_t o_stride_token, o_stride_head;      /* elements of the output type           */
    int64_t sys_stride_token, sys_stride_head;  /* elements                              */
    int32_t out_is_fp32;          /* 0: `out` is bf16 (round to nearest even); 1: fp32   */
    /* Tuning; 0 selects the built-in heuristic. */
    int32_t sys_chunk_tokens;     /* system positions per work item (multiple of 32)     */
    int32_t ctx_part_tokens;      /* context positions per wavefront span in decode, per
                                     work item elsewhere (multiple of 128)               */
    int32_t reserved0;            /* must be 0                                           */
} ra_params;

/*
 * Bytes of device workspace relay_attn_decode / relay_attn_prefill need for
 * `total_q` query tokens (decode: total_q = batch).  The workspace holds the
 * fp32 partial outputs and log-sum-exps of the system chunks and context parts
 * (the operands of the relay fusion, Eq. 7) between the partial-attention
 * launch and the fusion launch; it needs no initialisation and may be reused
 * by any later call that does not overlap in time.  Returns 0 if the
 * parameters are invalid.  Host only, no launch.
 */
size_t relay_attn_workspace_bytes(const ra_params *p, int32_t total_q);

/*
 * One decode step of one attention layer for a batch (Alg. 1 with one new
 * token per request; Eq. 7).
 *   q        [batch] tokens x Hq x head_dim bf16 (strided by q_stride_*)
 *   out      same shape, bf16 or fp32 per out_is_fp32 (strided by o_stride_*)
 *   lse_out  nullable; [batch][Hq] fp32, natural-log log-sum-exp of the scaled
 *            logits over all sys_len + context_lens[i] positions (Eq. 12)
 * A request with sys_len + context_lens[i] == 0 gets a zero output row and
 * lse = -inf.  workspace must be 256-byte aligned and at least
 * relay_attn_workspace_bytes(p, batch) bytes.
 */
ra_status relay_attn_decode(const ra_params *p,
                            const void *q,
                            const void *k_sys, const void *v_sys,
                            const void *k_cache, const void *v_cache,
                            const int32_t *block_tables, const int32_t *context_lens,
                            void *out, float *lse_out,
                            void *workspace, size_t workspace_bytes,
                            void *hip_stream);

/*
 * One decode step INCLUDING the cache write that precedes attention in Alg. 1
 * ("kv_cache[layer, :, l_cache:l_new] = k, v", then attention over [0, l_new)): the same result
 * as relay_attn_cache_append followed by relay_attn_decode, in the launches of the latter.
 *   k_new, v_new   [batch] tokens x Hkv x head_dim bf16, addressed as
 *                  base + token * new_stride_token + head * new_stride_head (elements)
 * context_lens[i] already counts the new token: its key/value belong at context position
 * context_lens[i] - 1.  The wavefront that attends over the last positions of (request i, kv
 * head g) takes that position from k_new / v_new instead of the cache and writes it to
 * k_cache / v_cache on the side; nothing else in the launch reads that cache row, and whatever
 * the row held before is never read.  A request with context_lens[i] == 0 has nothing to write.
 * On return of the stream's work the caches hold the new rows (byte-exact copies).
 */
ra_status relay_attn_decode_append(const ra_params *p,
                                   const void *q,
                                   const void *k_new, const void *v_new,
                                   int64_t new_stride_token, int64_t new_stride_head,
                                   const void *k_sys, const void *v_sys,
                                   void *k_cache, void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   void *out, float *lse_out,
                                   void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/*
 * relay_attn_decode for callers that cannot allocate and have no workspace to pass: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments minus
 * the workspace, same kernels, same result bit for bit.  The partial results live in a
 * fixed array inside the library's device code instead (relay_attn_static_scratch_bytes() =
 * 32 MiB; every GPU the library runs on holds its copy until the process ends; its address is
 * looked up on the first call on a device).  Nothing is allocated, freed or copied.
 *   - A call whose partials would not fit returns RA_ERR_WORKSPACE_TOO_SMALL before any launch
 *     (the need is relay_attn_workspace_bytes(p, batch): about 0.5 KiB x output rows x partials
 *     per row; the Llama-30B shape at batch 32 needs 7 MiB, the Llama-3-8B shape at batch 128
 *     28 MiB).
 *   - The array needs no clearing between calls: every slot a call reads it has written itself.
 *   - All calls on one GPU share the one array: calls that overlap in time on the same GPU
 *     (two streams, two threads) race and must not be made; use relay_attn_decode with a
 *     workspace per stream for that.
 */
ra_status relay_attn_decode_static(const ra_params *p,
                                   const void *q,
                                   const void *k_sys, const void *v_sys,
                                   const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   void *out, float *lse_out,
                                   void *hip_stream);
size_t relay_attn_static_scratch_bytes(void);

/*
 * Measurement aid, not for serving: relay_attn_decode restricted to some of its launches.
 * phases bit 0 = the partial-attention launch (system + context attention into the workspace),
 * bit 1 = the relay-fusion launch (workspace -> out); 3 is relay_attn_decode.  The benchmark
 * times the dominant kernel alone with it.
 */
ra_status relay_attn_debug_decode_phases(const ra_params *p, int32_t phases,
                                         const void *q,
                                         const void *k_sys, const void *v_sys,
                                         const void *k_cache, const void *v_cache,
                                         const int32_t *block_tables, const int32_t *context_lens,
                                         void *out, float *lse_out,
                                         void *workspace, size_t workspace_bytes,
                                         void *hip_stream);

/*
 * Measurement aid, not for serving: relay_attn_decode (cu_seqlens_q NULL, total_q = p->batch,
 * max_q_len = 1) or relay_attn_prefill, with the partial-attention launch recording when each
 * of its wavefronts began and ended: wavefront w of the launch (4 per workgroup, in grid order:
 * system workgroups first in a decode step, see relay_attn_decode_plan) writes the device's
 * 100 MHz real-time counter to timeline[2w] and timeline[2w+1] (DEVICE memory, 8-byte aligned,
 * room for 2 * timeline_wavefronts values; wavefronts beyond that are not recorded; entries of
 * wavefronts that do not exist stay as they were).  The result of the call is the ordinary one.
 */
ra_status relay_attn_debug_timeline(const ra_params *p,
                                    const void *q,
                                    const int32_t *cu_seqlens_q, int32_t total_q, int32_t max_q_len,
                                    const void *k_sys, const void *v_sys,
                                    const void *k_cache, const void *v_cache,
                                    const int32_t *block_tables, const int32_t *context_lens,
                                    void *out, float *lse_out,
                                    void *workspace, size_t workspace_bytes,
                                    uint64_t *timeline, int32_t timeline_wavefronts,
                                    void *hip_stream);

/*
 * The work decomposition relay_attn_decode would use for these parameters (host only, no HIP
 * call; for tuning and for tests of the decomposition).  The partial-attention launch consists of
 * num_sys_workgroups workgroups that each take one (kv head, sys_rows_per_workgroup stacked query
 * rows, sys_chunk_tokens system positions) item, and num_ctx_wavefronts wavefronts that share the
 * 32-position tiles of all context items: the tiles of the batch (N of them, an empty context
 * counts as one), in (request, kv head, position) order, are cut into one span of consecutive
 * tiles per wavefront.
 *   A class of wavefronts (n_wg workgroups of four) that shares R tiles does so as follows, with
 *   floor = min_tiles_per_ctx_wavefront: if (R / n_wg) / 4 >= floor (integer divisions), workgroup v
 *   of the class takes Q_v = R / n_wg + (v < R mod n_wg) consecutive tiles and its wavefront k
 *   takes Q_v / 4 + (k < Q_v mod 4) of them; otherwise every wavefront takes `floor` tiles and the
 *   last ones none.
 *   Without light wavefronts all wavefronts are one class and R = N.
 *   With light wavefronts (numbers first_light_ctx_wavefront .. + num_light_ctx_wavefronts - 1:
 *   the ones that share a compute unit with a system workgroup, which is known when the launch
 *   is exactly two workgroups per compute unit) every light workgroup takes
 *   L = (sys_tiles_total + N) / 256 - sys_workgroup_tiles tiles (0 if that is negative), split over
 *   its four wavefronts as above; if L / 4 < floor a light wavefront takes floor tiles when
 *   2 (L / 4) >= floor and none otherwise; none either if the light wavefronts together would
 *   exceed N.  The other ("heavy") wavefronts are a class that shares the rest, so that every
 *   compute unit ends up with about the same number of tiles.  Should a span of either class then
 *   exceed (max_blocks_per_span - 1) * block_size / 32 tiles, the split into light and heavy is
 *   dropped.  Wavefronts whose span is empty do not count when segments of an item are numbered.
 * Every output row then has num_sys_chunks + num_ctx_slots partial results for the relay fusion
 * (Eq. 7 in n-partial form); a context item never spans more than num_ctx_slots wavefronts, and a
 * wavefront's span inside one item never covers more than max_blocks_per_span cache blocks.
 *   sys_rows_per_workgroup is 32 (a row tile streams its chunk alone) or, for batches with many
 *   stacked rows B * num_q_heads / num_kv_heads per kv head (from 128 on, depending on how the
 *   system part compares with the context part) and one shared prefix, 128
 *   (four row tiles share every K/V tile through LDS; sys_workgroup_tiles and sys_tiles_total
 *   count the tiles such workgroups fetch).
 */
typedef struct {
    int32_t sys_chunk_tokens, num_sys_chunks, num_sys_workgroups;
    int32_t num_ctx_wavefronts, min_tiles_per_ctx_wavefront, num_ctx_slots;
    int32_t max_blocks_per_span;
    int32_t first_light_ctx_wavefront, num_light_ctx_wavefronts;
    int32_t sys_workgroup_tiles, sys_tiles_total;
    int32_t sys_rows_per_workgroup;
    int32_t compute_units;        /* of the current device (256 where none answers); the light /
                                     heavy split above is only used when this is 256 */
} ra_decode_plan;

ra_status relay_attn_decode_plan(const ra_params *p, ra_decode_plan *plan);

/*
 * Several shared prefixes in one batch (App. D, "multi-application hosting": requests are
 * tagged with an application and the scheduler batches requests of the same application
 * together).  The batch is a sequence of groups; group i is requests first_request ..
 * first_request + num_requests - 1 (the groups tile 0 .. batch-1 in order, at most 32 of them)
 * and shares the system cache k_sys / v_sys of sys_len positions (device pointers, same
 * strides p->sys_stride_* for all groups).  p->sys_len must equal the longest sys_len.
 * `prefixes` is a HOST array, read before the call returns.  Everything else as
 * relay_attn_decode; one group is exactly relay_attn_decode.
 */
typedef struct {
    const void *k_sys, *v_sys;    /* device */
    int32_t sys_len;
    int32_t first_request, num_requests;
} ra_prefix;

ra_status relay_attn_decode_multi(const ra_params *p,
                                  int32_t num_prefixes, const ra_prefix *prefixes,
                                  const void *q,
                                  const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  void *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * The same with the requests of an application anywhere in the batch (App. D tags every request
 * with its application; a scheduler need not sort the batch).
 *   prefixes       HOST array, entry i describes application i: k_sys, v_sys, sys_len as above and
 *                  num_requests = how many requests of this batch carry sys_id i (0 is allowed);
 *                  first_request is ignored.  At most 32 entries.
 *   sys_id         DEVICE [batch] int32: the application of each request, 0 .. num_prefixes-1
 *   request_order  DEVICE [batch] int32: the requests listed application by application (first the
 *                  requests with sys_id 0, in any order, then those with sys_id 1, ...)
 * The two arrays must agree with each other and with the counts; like block tables they are
 * taken on trust.  relay_attn_group_requests builds request_order and the counts from a host copy
 * of sys_id (host only, no HIP call; RA_ERR_INVALID_ARG for an id out of range).
 * p->sys_len must equal the longest sys_len among the applications that have requests.
 */
ra_status relay_attn_group_requests(const int32_t *sys_id, int32_t batch, int32_t num_prefixes,
                                    int32_t *request_order, int32_t *num_requests);

ra_status relay_attn_decode_grouped(const ra_params *p,
                                    int32_t num_prefixes, const ra_prefix *prefixes,
                                    const int32_t *sys_id, const int32_t *request_order,
                                    const void *q,
                                    const void *k_cache, const void *v_cache,
                                    const int32_t *block_tables, const int32_t *context_lens,
                                    void *out, float *lse_out,
                                    void *workspace, size_t workspace_bytes,
                                    void *hip_stream);

/*
 * Prompt phase (Alg. 1 with more than one new token per request; Sec. 3.3
 * notes the reformulation does not assume a single query token).
 *   q             [total_q] packed tokens x Hq x head_dim
 *   cu_seqlens_q  device, [batch+1] int32: request i owns query tokens
 *                 cu_seqlens_q[i] .. cu_seqlens_q[i+1]-1 (m_i of them)
 *   total_q       host copy of cu_seqlens_q[batch]
 *   max_q_len     host-side upper bound on m_i
 * The m_i new tokens are the LAST m_i positions of request i's context
 * (context_lens[i] >= m_i): new token j attends to all system positions and
 * to context positions 0 .. context_lens[i]-m_i+j (causal).  out / lse_out are
 * indexed by packed token.
 * The workspace is required as for the decode step (relay_attn_workspace_bytes(p, total_q)); a
 * call with at least 32 new tokens per request on average (4 when the system prompt has at most
 * 1024 positions), a system prompt that is one chunk of work and no hand-set p->sys_chunk_tokens / ctx_part_tokens runs as a single launch that does
 * not touch it (the relay fusion of Alg. 1 happens in the accumulators), other calls write
 * partials there and fuse them in a second launch.  The results agree within the tolerance, not
 * bit for bit, between the two forms.
 */
ra_status relay_attn_prefill(const ra_params *p,
                             const void *q,
                             const int32_t *cu_seqlens_q, int32_t total_q, int32_t max_q_len,
                             const void *k_sys, const void *v_sys,
                             const void *k_cache, const void *v_cache,
                             const int32_t *block_tables, const int32_t *context_lens,
                             void *out, float *lse_out,
                             void *workspace, size_t workspace_bytes,
                             void *hip_stream);

/*
 * The prompt phase with several shared prefixes (App. D): consecutive groups of requests as in
 * relay_attn_decode_multi (`prefixes`, HOST), and prefix_num_tokens (HOST, [num_prefixes]) = the
 * new query tokens of each group's requests together (cu_seqlens_q[first + n] - cu_seqlens_q[first];
 * they sum to total_q).  Everything else as relay_attn_prefill; one group is exactly that call.
 * Errors: RA_ERR_INVALID_ARG when the groups do not tile the batch in order, the counts do not sum
 * to total_q, a count exceeds num_requests * max_q_len, p->sys_len is not the longest prefix or a
 * prefix pointer is NULL / misaligned; RA_ERR_UNSUPPORTED above 32 groups.  Counts that disagree
 * with the device's cu_seqlens_q cannot be seen from the host: every access stays inside
 * [0, total_q), but tokens near a group border then attend to the neighbouring group's prefix.
 */
ra_status relay_attn_prefill_multi(const ra_params *p,
                                   int32_t num_prefixes, const ra_prefix *prefixes,
                                   const int32_t *prefix_num_tokens,
                                   const void *q,
                                   const int32_t *cu_seqlens_q, int32_t total_q, int32_t max_q_len,
                                   const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   void *out, float *lse_out,
                                   void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/*
 * The comparison path the paper measures against (Sec. 3.2, second
 * observation; Eq. 8): ordinary per-request paged decode attention with no
 * shared-prefix handling.  Each request's block table lists ALL its positions
 * (the caller puts the system prompt's pages first), so the system KV is read
 * once per request.  p->sys_len must be 0; k_sys / v_sys do not exist here.
 * Same workspace rule as relay_attn_decode.
 */
ra_status paged_attn_decode_naive(const ra_params *p,
                                  const void *q,
                                  const void *k_cache, const void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  void *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * The step that precedes attention in Alg. 1 ("kv_cache[layer, :, l_cache:l_new] = k, v"):
 * writes the keys/values of the new tokens into the paged context cache.
 *   k_new, v_new   [total_q] tokens x Hkv x head_dim bf16, addressed as
 *                  base + token * new_stride_token + head * new_stride_head (elements), so a
 *                  slice of a fused projection output can be passed as it is
 *   cu_seqlens_q   device, [batch+1], or NULL for one new token per request (decode:
 *                  total_q must equal batch)
 * context_lens[i] already counts the new tokens (the convention of every entry point here):
 * new token j of the m_i tokens of request i is written to context position
 * context_lens[i] - m_i + j, i.e. into block block_tables[i][pos / block_size] at offset
 * pos % block_size.  Only k_cache / v_cache are written; nothing is allocated.
 */
ra_status relay_attn_cache_append(const ra_params *p,
                                  const void *k_new, const void *v_new,
                                  int64_t new_stride_token, int64_t new_stride_head,
                                  const int32_t *cu_seqlens_q, int32_t total_q,
                                  void *k_cache, void *v_cache,
                                  const int32_t *block_tables, const int32_t *context_lens,
                                  void *hip_stream);

/*
 * The layout this library recommends for the shared system cache (Sec. 3.3, "Peripheral
 * adaptations": the system prompt's keys/values live in a cache of their own, filled once,
 * offline; so its layout is the serving system's to choose).  HOST arithmetic only, no HIP call.
 * Token-major rows [s][Hkv][d] whose stride is NOT a multiple of 1024 bytes: with the dense
 * stride Hkv * d * 2 (13312 bytes for 52 heads of 128) every row piece of one kv head starts at
 * the same offset inside a 1 KiB window, and the memory system served the heads at some offsets
 * 12 % slower than the others (measured on MI355X); with the row padded so that its stride is
 * 384 mod 1024 bytes the pieces of every head walk through all offsets and the decode step is 1 - 4 %
 * shorter.  The padding is never read.  Every entry point takes any strides (multiples of 8
 * elements, head_dim contiguous); this call only names good ones:
 *   *stride_token_out, *stride_head_out   elements, to be put into p->sys_stride_token / _head
 *   *bytes_out                            bytes of ONE of the two buffers (k_sys or v_sys) for
 *                                         p->sys_len positions (0 for an empty prompt)
 * Reads p->num_kv_heads, p->head_dim and p->sys_len only.  RA_ERR_INVALID_ARG for a NULL
 * argument or non-positive head counts / head_dim / negative sys_len.
 */
ra_status relay_attn_system_cache_layout(const ra_params *p,
                                         int64_t *stride_token_out, int64_t *stride_head_out,
                                         size_t *bytes_out);

/*
 * Fills positions first_pos .. first_pos + num_pos - 1 of the shared system cache (Sec. 3.3,
 * "Peripheral adaptations": the system prompt's keys/values are computed once, offline, and kept
 * in a cache of their own, not in the request caches).  k_new / v_new hold num_pos x Hkv x
 * head_dim bf16 rows addressed like relay_attn_cache_append's; the destination is addressed with
 * p->sys_stride_*.  first_pos + num_pos must not exceed p->sys_len.  Only k_sys / v_sys are
 * written.
 */
ra_status relay_attn_system_fill(const ra_params *p,
                                 const void *k_new, const void *v_new,
                                 int64_t new_stride_token, int64_t new_stride_head,
                                 int32_t first_pos, int32_t num_pos,
                                 void *k_sys, void *v_sys,
                                 void *hip_stream);

/*
 * Debug aid: checks on the device what the attention entry points take on trust, the CONTENTS
 * of the index arrays (Alg. 1 indexes the cache with them: an entry out of range is a read
 * out of bounds).  Unlike every other entry point it SYNCHRONISES the stream and copies 16
 * bytes to the host; it is not meant for the serving loop and cannot be captured in a graph.
 *   context_lens[i] must lie in 0 .. max_blocks_per_seq * block_size (and in 0 ..
 *   max_context_len when that is set);
 *   block_tables[i][j] must lie in 0 .. num_blocks-1 for the slots in use,
 *   j < ceil(context_lens[i] / block_size) (other slots are never read, and not checked);
 *   cu_seqlens_q (NULL for decode; device, [batch+1]) must start at 0, not decrease, end at
 *   total_q, and give no request more new tokens than context_lens[i].
 * Uses the first 256 bytes of `workspace` (device, 256-byte aligned).  `report` (host, may
 * be NULL) receives the counts.  Returns RA_OK when everything is in range,
 * RA_ERR_INVALID_ARG when something is not (or an argument is malformed), RA_ERR_HIP when a
 * HIP call fails.
 */
typedef struct {
    int32_t bad_context_lens;   /* requests whose length is out of range */
    int32_t bad_block_ids;      /* used block-table slots that are out of range */
    int32_t bad_query_lens;     /* requests whose cu_seqlens_q entries break the rules above */
    int32_t first_bad_request;  /* lowest request index with any violation, -1 if none */
} ra_validate_report;

ra_status relay_attn_debug_validate(const ra_params *p,
                                    const int32_t *block_tables, const int32_t *context_lens,
                                    const int32_t *cu_seqlens_q, int32_t total_q,
                                    void *workspace, size_t workspace_bytes,
                                    void *hip_stream, ra_validate_report *report);

/*
 * Measurement aids for the bandwidth roofline of the decode path (Sec. 3.1 - 3.2 argue that decode
 * attention is bound by memory traffic, so the yardstick is what the memory system delivers):
 *   relay_attn_debug_stream_probe  reads `bytes` (a multiple of 16) of `src` (device, 16-byte
 *       aligned) exactly once with coalesced 16-byte loads, 256 KiB per workgroup, ordinary
 *       (nontemporal = 0) or non-temporal (1), and does nothing with them; `sink` (device, 4
 *       bytes) is practically never written.
 *   relay_attn_debug_launch_probe  launches `count` empty one-workgroup kernels back to back from
 *       one host call: timed as a whole, the cost of a launch in a stream by itself.
 * Neither synchronises.
 */
ra_status relay_attn_debug_stream_probe(const void *src, size_t bytes, int32_t nontemporal,
                                        void *sink, void *hip_stream);
ra_status relay_attn_debug_launch_probe(void *sink, int32_t count, void *hip_stream);

/* Static, NUL-terminated description of a status code.  Host only. */
const char *relay_attn_status_string(ra_status status);

/* Library ABI version; bumped when a signature or ra_params changes. */
int32_t relay_attn_abi_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RELAY_ATTN_H */
