// Host side of the C ABI declared in include/relay_attn.h: argument validation (before any
// HIP call), work decomposition, workspace layout and kernel launches.  Nothing here
// allocates, and nothing but relay_attn_debug_validate copies or synchronises.
#include "../../include/relay_attn.h"

#include <hip/hip_runtime.h>

#include <mutex>

#include "ra_kernels.h"

// Scratch of relay_attn_decode_static: the partial results between the partial-attention launch
// and the fusion launch, for callers that can neither allocate a workspace nor pass one.  Every
// device the library runs on holds its own copy of this array until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress, never an address to pass on.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int32_t kAbiVersion = 6;
constexpr int kWholeMinTokens = 32;   // new tokens per request, on average, from which the prompt phase is one launch

struct Plan {
    int group;            // query heads per kv head
    int rows;             // total_q * Hq output rows
    int n_mtiles;         // 32-row tiles of stacked queries per kv head
    int sys_chunk;        // system positions per work item
    int n_sys_chunks;
    int ctx_part;         // context positions per work item (prompt phase, per-request kernel)
    int n_ctx_parts;      // context partial slots per row
    int ctx_wgs;          // decode: context workgroups (four wavefronts each) in the tile launch
    int ctx_t_floor;      // decode: least tiles per context wavefront, bounds the slots per row
    bool paired;          // decode: the launch is exactly two workgroups per compute unit
    bool unsupported;
    int max_ctx;
    int block_size_log2;
    bool rows_path;       // system part (and prefill context part) through the many-rows kernel
    bool rows_sys;        // decode: system items of the many-rows kind inside the tile launch
    int n_sys_rowblocks;  // 128-row blocks of stacked queries per kv head
    int n_ctx_rowblocks;  // prefill: 128-row blocks per (request, kv head)
    // partial p of row r: o at off_o + (p*rows + r)*d*4, lse at off_lse + (p*rows + r)*4;
    // partials 0..n_sys_chunks-1 are system chunks, the rest context parts
    size_t off_o, off_lse, bytes;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

ra_status check_params(const ra_params *p, int32_t total_q) {
    if (!p) return RA_ERR_INVALID_ARG;
    if (p->batch < 0 || total_q < 0 || p->num_q_heads < 1 || p->num_kv_heads < 1 ||
        p->sys_len < 0 || p->block_size < 1 || p->num_blocks < 0 || p->max_blocks_per_seq < 0 ||
        p->max_context_len < 0 || p->sys_chunk_tokens < 0 || p->ctx_part_tokens < 0 ||
        p->reserved0 != 0)
        return RA_ERR_INVALID_ARG;
    if (p->num_q_heads % p->num_kv_heads != 0) return RA_ERR_INVALID_ARG;
    if ((p->block_size & (p->block_size - 1)) != 0) return RA_ERR_INVALID_ARG;
    if (!(p->softmax_scale == p->softmax_scale)) return RA_ERR_INVALID_ARG;  // NaN
    if (p->out_is_fp32 != 0 && p->out_is_fp32 != 1) return RA_ERR_INVALID_ARG;
    const int64_t strides[] = {p->q_stride_token, p->q_stride_head, p->o_stride_token,
                               p->o_stride_head, p->sys_stride_token, p->sys_stride_head};
    for (int64_t s : strides)
        if (s < 0 || (s % 8) != 0) return RA_ERR_INVALID_ARG;
    if (p->sys_chunk_tokens % 32 != 0 || p->ctx_part_tokens % 128 != 0) return RA_ERR_INVALID_ARG;
    if ((int64_t)p->max_blocks_per_seq * p->block_size > INT32_MAX) return RA_ERR_INVALID_ARG;
    if (p->max_context_len > (int64_t)p->max_blocks_per_seq * p->block_size)
        return RA_ERR_INVALID_ARG;
    if (p->head_dim != 64 && p->head_dim != 128) return RA_ERR_UNSUPPORTED;
    const int g = p->num_q_heads / p->num_kv_heads;
    if (g < 1 || g > 8) return RA_ERR_UNSUPPORTED;
    if ((int64_t)total_q * p->num_q_heads > (1 << 28)) return RA_ERR_UNSUPPORTED;
    return RA_OK;
}

enum PlanKind { kRelayDecode, kNaiveDecode, kPrefill };

// Compute units of the current device: asked once (an attribute query, no launch) and cached;
// 256, the MI355X's count, where no device answers (a machine without a GPU still sizes
// workspaces and reports plans).  The decomposition below is a pure function of the parameters
// and this number, so the workspace size a caller asked for and the launch always agree.
constexpr int kReferenceCus = 256;
int device_compute_units() {
    static const int cus = [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
            (void)hipGetLastError();         // leave no sticky error behind for the caller
            return kReferenceCus;
        }
        return n;
    }();
    return cus;
}

// Device address of this device's copy of `scratch`: looked up once per device, with that device
// current (each device has the array at an address of its own), and kept.
constexpr int kMaxDevices = 64;
ra_status static_scratch(void **ptr) {
    static std::mutex lock;
    static void *known[kMaxDevices] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return RA_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return RA_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(lock);
    if (!known[dev]) {
        void *found = nullptr;
        if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) {
            (void)hipGetLastError();
            return RA_ERR_HIP;
        }
        known[dev] = found;
    }
    *ptr = known[dev];
    return RA_OK;
}

// The least work worth giving a wavefront of the tile launch.
constexpr int kMinWaveTiles = 4;
// Row tiles (of 32 stacked query rows per kv head) from which a decode batch takes its system
// part through many-rows items.
constexpr int kRowsSysMinTiles = 8;

// Work decomposition; a pure function of (params, total_q) so that the workspace size the
// caller asked for and the one the launch uses always agree.
Plan make_plan(const ra_params *p, int32_t total_q, PlanKind kind, int32_t max_q_len,
               int64_t sys_base_items = 0, bool allow_rows_sys = true) {
    Plan pl{};
    const bool prefill = kind == kPrefill;
    // Wavefronts the chip holds at once with the tile kernel's two workgroups of four per
    // compute unit.
    const int kWorkgroupSlots = device_compute_units() * 2;
    const int kWaveSlots = kWorkgroupSlots * 4;
    pl.group = p->num_q_heads / p->num_kv_heads;
    pl.rows = total_q * p->num_q_heads;
    pl.n_mtiles = ceil_div(total_q * pl.group, 32);
    pl.block_size_log2 = 0;
    while ((1 << pl.block_size_log2) < p->block_size) ++pl.block_size_log2;
    pl.max_ctx = p->max_context_len > 0 ? p->max_context_len : p->max_blocks_per_seq * p->block_size;

    // Decode: the streaming tile kernel.  Prompt phase: the many-rows kernel, which fetches each
    // K/V tile once per 128 stacked rows.
    // (Wide GQA decode batches use many-rows items too, but inside the tile launch: rows_sys.)
    pl.rows_path = prefill;
    pl.n_sys_rowblocks = ceil_div(total_q * pl.group, 128);
    pl.n_ctx_rowblocks = prefill ? ceil_div(max_q_len * pl.group, 128) : 0;
    const size_t d = (size_t)p->head_dim;
    auto finish = [&]() {
        const size_t n_partials = (size_t)pl.n_sys_chunks + pl.n_ctx_parts;
        size_t at = 0;
        pl.off_o = at;   at = align_up(at + n_partials * pl.rows * d * 4, 256);
        pl.off_lse = at; at = align_up(at + n_partials * pl.rows * 4, 256);
        pl.bytes = at > 0 ? at : 256;
    };
    if (total_q == 0) {
        finish();
        return pl;
    }

    if (kind == kRelayDecode) {
        // One launch holds system workgroups (four wavefronts share a chunk of the prompt) and
        // context wavefronts (each takes an equal span of the stream of context tiles, see the
        // kernel).  The aim is that every wavefront of the launch moves about the same number of
        // 32-key tiles and that all of them are resident at once: t_star tiles each.  The context
        // side is sized from max_context_len (the lengths themselves live on the device); when
        // the real lengths are shorter its wavefronts simply finish earlier.
        const int64_t sys_tiles = ceil_div(p->sys_len, 32);               // per (kv head, row tile)
        const int64_t base_items = sys_base_items > 0 ? sys_base_items
                                                      : (int64_t)p->num_kv_heads * pl.n_mtiles;
        const int64_t t_max = pl.max_ctx > 0 ? ceil_div(pl.max_ctx, 32) : 0;   // tiles of one context
        const int64_t ctx_tiles = (int64_t)total_q * p->num_kv_heads * t_max;
        const int64_t all_tiles = base_items * sys_tiles + ctx_tiles;
        if (ctx_tiles > INT32_MAX) {
            pl.unsupported = true;
            return pl;
        }
        // (in sixteenths of a tile, so that small launches are not rounded to whole tiles)
        int64_t t_star16 = (all_tiles * 16 + kWaveSlots - 1) / kWaveSlots;
        // (small launches: down to a tile and a half per wavefront rather than kMinWaveTiles, more
        // wavefronts in flight matter more than their length there: Llama-7B shape 25.7 -> 24.5 us,
        // batch 16 of the Llama-30B shape at s = 1024 24.0 -> 21.5 us, batch 8 at s = 512
        // 15.4 -> 14.4 us)
        if (t_star16 < 24) t_star16 = 24;
        const int64_t t_star = (t_star16 + 15) / 16;
        int64_t sys_wgs = 0, t_sys = 0;
        // Wide grouped-query batches: with B*G stacked rows per kv head in many row tiles, every
        // 32-row streaming item would pull the system K/V of its chunk into its compute unit
        // (from L2, but what a unit can draw is capped there too: 87 us at the Llama-3-8B shape).
        // Many-rows items share each tile among 128 rows through LDS, a quarter of the draw.
        // (Measured against the streaming items over batch 32..512, 8..32 row tiles, prompts of
        // 512..16384: faster by 4..20 % where the system part is at least about half of the
        // context part, slower by up to 8 % in batches that are mostly context.)
        // From four row tiles (one full block of 128 rows) on it still pays when the system part
        // is both large (64 tiles per compute unit) and at least as large as the context part:
        // batch 128 of the Llama-30B shape at s = 8192 157 -> 128 us, batch 192 at 4096 163 -> 144 us.
        {
            const int64_t sys_all = base_items * sys_tiles;
            const bool wide = pl.n_mtiles >= kRowsSysMinTiles && 2 * sys_all >= ctx_tiles;
            const bool full_block = pl.n_mtiles >= 4 && sys_all >= 64 * (kWorkgroupSlots / 2) &&
                                    sys_all >= ctx_tiles;
            pl.rows_sys = allow_rows_sys && sys_base_items == 0 && p->sys_len > 0 && (wide || full_block);
        }
        if (pl.rows_sys) {
            const int64_t rb_items = (int64_t)p->num_kv_heads * pl.n_sys_rowblocks;
            int chunk = p->sys_chunk_tokens;
            if (chunk == 0) {
                // one workgroup per compute unit if the prompt is long enough (chunks of 256
                // positions or more: batch 64 of a 32/8-head model at s = 1024 34 -> 23 us against
                // chunks of 512), at most sixteen chunks (every chunk is one more partial per row
                // for the fusion to read)
                int64_t n_chunks = (kWorkgroupSlots / 2 + rb_items / 2) / rb_items;
                const int64_t most = ceil_div(p->sys_len, 256) < 16 ? ceil_div(p->sys_len, 256) : 16;
                if (n_chunks > most) n_chunks = most;
                if (n_chunks < 1) n_chunks = 1;
                chunk = (int)((sys_tiles + n_chunks - 1) / n_chunks) * 32;
            }
            pl.sys_chunk = chunk;
            pl.n_sys_chunks = ceil_div(p->sys_len, chunk);
            sys_wgs = rb_items * pl.n_sys_chunks;
            t_sys = chunk / 32;            // each of the four wavefronts walks every tile
        } else
        if (p->sys_len > 0) {
            int chunk = p->sys_chunk_tokens;
            if (chunk == 0) {
                int64_t n_chunks = (sys_tiles * 16 + 2 * t_star16) / (4 * t_star16);   // nearest
                // At most one system workgroup per compute unit: a compute unit cannot draw more
                // than about 1/256 of the memory bandwidth whatever it holds, so two long
                // workgroups on one unit finish last (measured: 208 system workgroups beat 312
                // and 416 at the 8192- and 16384-position prompts, 59 vs 63 us and 92 vs 95 us);
                // the context wavefronts fill the second slot of every unit.
                if (base_items * n_chunks > kWorkgroupSlots / 2) n_chunks = kWorkgroupSlots / 2 / base_items;
                if (n_chunks < 1) n_chunks = 1;
                chunk = (int)((sys_tiles + n_chunks - 1) / n_chunks) * 32;
            }
            pl.sys_chunk = chunk;
            pl.n_sys_chunks = ceil_div(p->sys_len, chunk);
            sys_wgs = base_items * pl.n_sys_chunks;
            t_sys = ceil_div(chunk / 32, 4);
        }
        if (ctx_tiles > 0) {
            // a span's block ids must fit the per-wavefront table in LDS
            int64_t t_cap = ((int64_t)ra::kMaxPartBlocks - 1) * p->block_size / 32;
            if (t_cap < 1) t_cap = 1;
            int64_t wgs;
            // Which workgroups share a compute unit (i and i + 256 of a 512-workgroup grid) was
            // measured on the 256-unit chip only; elsewhere every context wavefront gets an equal
            // span.
            const bool pairing_known = device_compute_units() == kReferenceCus;
            if (p->ctx_part_tokens > 0) {
                const int64_t t_fixed = p->ctx_part_tokens / 32;
                if (t_fixed > t_cap) {
                    pl.unsupported = true;
                    return pl;
                }
                wgs = (ctx_tiles + 4 * t_fixed - 1) / (4 * t_fixed);
                pl.ctx_t_floor = (int)t_fixed;
                pl.n_ctx_parts = (int)((t_max + t_fixed - 1) / t_fixed) + 1;
            } else {
                const int64_t least = (ctx_tiles + 4 * t_cap - 1) / (4 * t_cap);
                const int64_t t_like16 = t_sys * 16 > t_star16 ? t_sys * 16 : t_star16;
                wgs = (ctx_tiles * 16 + 4 * t_like16 - 1) / (4 * t_like16);
                // when the launch is about one machine-full of equally long wavefronts, make it
                // exactly one
                if (all_tiles > (int64_t)kWaveSlots * kMinWaveTiles && sys_wgs <= kWorkgroupSlots * 7 / 8 &&
                    (sys_wgs == 0 || 4 * t_sys >= 3 * t_star) && sys_wgs + wgs <= kWorkgroupSlots * 3 / 2) {
                    wgs = kWorkgroupSlots - sys_wgs;
                    pl.paired = wgs >= least && sys_wgs > 0 && sys_wgs <= kWorkgroupSlots / 2 && pairing_known;
                }
                // a small launch that comes out just above one machine-full is cut back to it (the
                // overflow would run alone afterwards), if that leaves spans of two tiles or more
                else if (sys_wgs + wgs > kWorkgroupSlots && sys_wgs + wgs <= kWorkgroupSlots * 3 / 2 &&
                         sys_wgs < kWorkgroupSlots &&
                         ctx_tiles >= 2 * 4 * (kWorkgroupSlots - sys_wgs)) {
                    wgs = kWorkgroupSlots - sys_wgs;
                    pl.paired = wgs >= least && sys_wgs > 0 && sys_wgs <= kWorkgroupSlots / 2 && pairing_known;
                }
                if (wgs < least) wgs = least;
                if (wgs < 1) wgs = 1;
                // t_est: tiles per wavefront if every context had the maximum length.  Real
                // lengths are shorter and the spans shrink with them, down to the floor below; a
                // floor near t_est would leave most context wavefronts without work (a batch
                // with lengths uniform in [64, 1024] has half the tiles the plan assumed).  So the
                // floor is a quarter of t_est, as far as the partials of a row (system chunks +
                // context slots) do not start another pass of the fusion kernel, which reads
                // them eight at a time.
                const int64_t t_est = (ctx_tiles + 4 * wgs - 1) / (4 * wgs);
                int64_t slots = (t_max + t_est - 1) / t_est + 1;
                int64_t t_low = (t_est + 3) / 4;
                if (t_low < kMinWaveTiles) t_low = kMinWaveTiles < t_est ? kMinWaveTiles : t_est;
                int64_t wide = (t_max + t_low - 1) / t_low + 1;
                const int64_t filled = pl.n_sys_chunks + slots;
                const int64_t room = (filled <= 6 ? 8 : filled <= 14 ? 16 : 24) - pl.n_sys_chunks;
                if (wide > room) wide = room;
                if (wide > slots) slots = wide;
                pl.n_ctx_parts = (int)slots;
                pl.ctx_t_floor = (int)((t_max + slots - 2) / (slots - 1));
            }
            pl.ctx_wgs = (int)wgs;
        }
        finish();
        return pl;
    }

    if (p->sys_len > 0) {
        int chunk = p->sys_chunk_tokens;
        if (chunk == 0) {
            // Many-rows kernel: about 400 workgroups of at least 512 positions (measured).
            const int64_t base_items = (int64_t)p->num_kv_heads * pl.n_sys_rowblocks;
            int64_t n_chunks = (400 + base_items / 2) / base_items;
            const int64_t max_chunks = ceil_div(p->sys_len, 512);
            if (n_chunks > max_chunks) n_chunks = max_chunks;
            if (n_chunks < 1) n_chunks = 1;
            chunk = ceil_div(ceil_div(p->sys_len, (int)n_chunks), 128) * 128;
        }
        pl.sys_chunk = chunk;
        pl.n_sys_chunks = ceil_div(p->sys_len, chunk);
    }
    if (pl.max_ctx > 0) {
        if (p->ctx_part_tokens > 0) {
            pl.ctx_part = p->ctx_part_tokens;
        } else if (prefill) {
            // one part unless the block table of a part would not fit its LDS table
            int64_t cap = (int64_t)ra::kMaxPartBlocks * p->block_size;
            if (cap > 4096) cap = 4096;
            pl.ctx_part = (int)(cap / 128 * 128);
            if (pl.ctx_part < 128) pl.ctx_part = 128;
        } else {
            pl.ctx_part = 256;
        }
        pl.n_ctx_parts = ceil_div(pl.max_ctx, pl.ctx_part);
        // a context part may touch at most kMaxPartBlocks blocks (the per-item block-id table in
        // LDS); parts start at multiples of ctx_part, which are block boundaries only when the
        // block size divides it
        const int touched = pl.ctx_part % p->block_size == 0
                                ? pl.ctx_part >> pl.block_size_log2
                                : ((pl.ctx_part - 1) >> pl.block_size_log2) + 2;
        if (touched > ra::kMaxPartBlocks) pl.unsupported = true;
    }
    finish();
    return pl;
}

// Where the partial-attention launch records the begin and end of its wavefronts (measurement aid).
struct Timeline {
    unsigned long long *entries = nullptr;   // device, 2 per wavefront
    int waves = 0;
};

// The new key/value rows of a decode step that the attention launch writes into the cache itself.
struct NewRows {
    const void *k = nullptr, *v = nullptr;
    int64_t stride_token = 0, stride_head = 0;
};

ra_status run(const ra_params *p, const void *q, const int32_t *cu_seqlens_q, int32_t total_q,
              int32_t max_q_len,
              const void *k_sys, const void *v_sys, const void *k_cache, const void *v_cache,
              const int32_t *block_tables, const int32_t *context_lens, void *out,
              float *lse_out, void *workspace, size_t workspace_bytes, void *hip_stream,
              bool naive, int32_t num_prefixes = 0, const ra_prefix *prefixes = nullptr,
              int phases = 3, const NewRows *append = nullptr,
              const int32_t *req_order = nullptr, const int32_t *req_prefix = nullptr,
              const int32_t *prefix_num_tokens = nullptr, const Timeline *timeline = nullptr) {
    ra_status st = check_params(p, total_q);
    if (st != RA_OK) return st;
    if (naive && p->sys_len != 0) return RA_ERR_INVALID_ARG;
    if (append) {
        if (append->stride_token < 0 || append->stride_head < 0 || append->stride_token % 8 ||
            append->stride_head % 8)
            return RA_ERR_INVALID_ARG;
        if (total_q > 0 && (!append->k || !append->v || !aligned16(append->k) || !aligned16(append->v)))
            return RA_ERR_INVALID_ARG;
        if (append->stride_head < p->head_dim && p->num_kv_heads > 1) return RA_ERR_INVALID_ARG;
    }
    const int kWorkgroupSlots = device_compute_units() * 2;
    // Shared prefixes of the batch: one (the paper's setting) unless the caller lists several.
    ra_prefix one{k_sys, v_sys, p->sys_len, 0, total_q};
    if (!prefixes) {
        prefixes = &one;
        num_prefixes = 1;
    }
    // the run of tokens each prefix owns: its requests in a decode step, their new tokens in the
    // prompt phase (where the caller says how many those are)
    int tok0[ra::kMaxPrefixes], ntok[ra::kMaxPrefixes];
    for (int i = 0, at = 0; i < num_prefixes && i < ra::kMaxPrefixes; ++i) {
        tok0[i] = prefix_num_tokens ? at : prefixes[i].first_request;
        ntok[i] = prefix_num_tokens ? prefix_num_tokens[i] : prefixes[i].num_requests;
        at += ntok[i];
    }
    int64_t sys_base_items = 0;
    bool read_once = true;
    for (int i = 0; i < num_prefixes; ++i) {
        const int mt = ceil_div(prefixes[i].num_requests * (p->num_q_heads / p->num_kv_heads), 32);
        sys_base_items += (int64_t)p->num_kv_heads * mt;
        if (mt > 1) read_once = false;          // several row tiles re-read the same K/V
    }
    const PlanKind kind = cu_seqlens_q ? kPrefill : naive ? kNaiveDecode : kRelayDecode;
    Plan pl = make_plan(p, total_q, kind, max_q_len, num_prefixes > 1 ? sys_base_items : 0);
    // A caller sizes the workspace without knowing the grouping; should the grouping-aware plan
    // need more than that, the grouping-blind one (which is what the size was computed from) is used.
    if (num_prefixes > 1 && !pl.unsupported && pl.bytes > workspace_bytes)
        pl = make_plan(p, total_q, kind, max_q_len, 0, false);
    if (pl.unsupported) return RA_ERR_UNSUPPORTED;
    if (total_q > 0) {
        if (!q || !out || !context_lens) return RA_ERR_INVALID_ARG;
        if (!aligned16(q) || !aligned16(out)) return RA_ERR_INVALID_ARG;
        if (p->sys_len > 0 && (!k_sys || !v_sys || !aligned16(k_sys) || !aligned16(v_sys)))
            return RA_ERR_INVALID_ARG;
        if (pl.max_ctx > 0 &&
            (!k_cache || !v_cache || !block_tables || !aligned16(k_cache) || !aligned16(v_cache)))
            return RA_ERR_INVALID_ARG;
        if (p->q_stride_head < p->head_dim || p->o_stride_head < p->head_dim ||
            (p->sys_len > 1 && p->sys_stride_token < p->head_dim))
            return RA_ERR_INVALID_ARG;
    }
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return RA_ERR_INVALID_ARG;
    if (workspace_bytes < pl.bytes) return RA_ERR_WORKSPACE_TOO_SMALL;
    if (total_q == 0) return RA_OK;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    float *part_o = reinterpret_cast<float *>(ws + pl.off_o);
    float *part_lse = reinterpret_cast<float *>(ws + pl.off_lse);
    const float scale_log2 = p->softmax_scale * 1.4426950408889634f;
    const int mask = phases;

    // A per-request paged pass over a short sequence needs no workspace round trip.
    const bool direct = naive && pl.n_sys_chunks == 0 && pl.n_ctx_parts == 1;

    const bool prefill = cu_seqlens_q != nullptr;
    const int head_fastest = p->sys_stride_head < p->sys_stride_token ? 1 : 0;

    // Prompt phase in ONE launch: when the system prompt is a single chunk anyway (launches with
    // many row blocks) and the requests bring many new tokens each, a work item carries its 128
    // rows through the system prompt and then through the contexts of the requests they belong
    // to, and writes the output itself; no partials, no fusion launch.  With few tokens per
    // request a block would walk through many requests' contexts one after the other, so the
    // split form (context items of their own) stays for those, unless the system prompt is short:
    // then the partials and the fusion launch of the split form weigh more than that walk
    // (measured: 256 requests of 4 .. 12 tokens at s = 512 145 against 162 us, 512 requests of 4
    // tokens at s = 1024 80 against 114 us; 128 requests of 16 tokens at s = 4096 328 against
    // 311 us).  The split form also stays whenever the caller tunes the decomposition by hand or
    // asks for one phase only.
    const bool whole = prefill && !naive && pl.n_sys_chunks <= 1 && mask == 3 &&
                       p->sys_chunk_tokens == 0 && p->ctx_part_tokens == 0 &&
                       ((int64_t)total_q >= kWholeMinTokens * (int64_t)p->batch ||
                        (p->sys_len <= 1024 && (int64_t)total_q >= 4 * (int64_t)p->batch));
    // Many stacked rows per kv head (prompt phase; wide GQA decode batches): the many-rows kernel
    // takes the system part and, in the prompt phase, the causal context part as well.
    if ((mask & 1) && !naive && pl.rows_path) {
        ra::RowsArgs r{};
        r.q = static_cast<const uint16_t *>(q);
        r.k_sys = static_cast<const uint16_t *>(k_sys);
        r.v_sys = static_cast<const uint16_t *>(v_sys);
        r.k_cache = static_cast<const uint16_t *>(k_cache);
        r.v_cache = static_cast<const uint16_t *>(v_cache);
        r.block_tables = block_tables;
        r.context_lens = context_lens;
        r.cu_seqlens_q = cu_seqlens_q;
        r.part_o = part_o;
        r.part_lse = part_lse;
        r.q_stride_token = p->q_stride_token;
        r.q_stride_head = p->q_stride_head;
        r.sys_stride_token = p->sys_stride_token;
        r.sys_stride_head = p->sys_stride_head;
        r.n_tokens = total_q;
        r.Hq = p->num_q_heads;
        r.Hkv = p->num_kv_heads;
        r.G = pl.group;
        r.sys_len = p->sys_len;
        r.sys_chunk = pl.sys_chunk;
        r.n_sys_chunks = pl.n_sys_chunks;
        r.n_sys_rowblocks = pl.n_sys_rowblocks;
        r.n_sys_items = p->num_kv_heads * pl.n_sys_rowblocks * pl.n_sys_chunks;
        r.ctx_part = pl.ctx_part;
        r.n_ctx_parts = pl.n_ctx_parts;
        r.n_ctx_rowblocks = pl.n_ctx_rowblocks;
        r.n_ctx_items = prefill ? p->batch * p->num_kv_heads * pl.n_ctx_rowblocks * pl.n_ctx_parts : 0;
        r.block_size_log2 = pl.block_size_log2;
        r.max_blocks_per_seq = p->max_blocks_per_seq;
        r.rows = pl.rows;
        r.sys_head_fastest = head_fastest;
        r.scale_log2 = scale_log2;
        r.n_prefixes = num_prefixes;
        r.batch = p->batch;
        r.whole = whole ? 1 : 0;
        if (whole) {
            // one item per (kv head, block of 128 stacked rows) that goes through the system prompt
            // and the contexts and writes the output rows itself
            r.out = out;
            r.lse_out = lse_out;
            r.o_stride_token = p->o_stride_token;
            r.o_stride_head = p->o_stride_head;
            r.out_is_fp32 = p->out_is_fp32;
            r.n_sys_chunks = 1;
            r.sys_chunk = p->sys_len > 0 ? pl.sys_chunk : 1;
            r.n_sys_items = p->num_kv_heads * pl.n_sys_rowblocks;
            r.n_ctx_items = 0;
            if (r.n_ctx_parts < 1 || r.ctx_part < 1) r.n_ctx_parts = 0, r.ctx_part = 1;   // no context at all
        }
        if (num_prefixes > 1) {                    // system items prefix by prefix
            int items = 0;
            for (int i = 0; i < num_prefixes; ++i) {
                items += p->num_kv_heads * ceil_div(ntok[i] * pl.group, 128) *
                         (whole ? 1 : pl.sys_chunk > 0 ? ceil_div(prefixes[i].sys_len, pl.sys_chunk) : 0);
                r.pfx_item_end[i] = items;
                r.pfx_tok0[i] = tok0[i];
                r.pfx_ntok[i] = ntok[i];
                r.pfx_len[i] = prefixes[i].sys_len;
                r.pfx_k[i] = static_cast<const uint16_t *>(prefixes[i].k_sys);
                r.pfx_v[i] = static_cast<const uint16_t *>(prefixes[i].v_sys);
            }
            r.n_sys_items = items;
        }
        if (timeline && prefill) r.timeline = timeline->entries, r.timeline_waves = timeline->waves;
        if (ra::launch_relay_rows(r, p->head_dim, stream) != hipSuccess) return RA_ERR_HIP;
    }
    // Decode: system chunks (unless the many-rows kernel took them) and context parts in one
    // launch of the streaming tile kernel.
    if ((mask & 1) && !naive && !prefill) {
        ra::TileArgs t{};
        t.q = static_cast<const uint16_t *>(q);
        t.k_cache = static_cast<const uint16_t *>(k_cache);
        t.v_cache = static_cast<const uint16_t *>(v_cache);
        if (append) {
            t.k_new = static_cast<const uint16_t *>(append->k);
            t.v_new = static_cast<const uint16_t *>(append->v);
            t.new_stride_token = append->stride_token;
            t.new_stride_head = append->stride_head;
        }
        t.req_order = num_prefixes > 1 ? req_order : nullptr;
        t.block_tables = block_tables;
        t.context_lens = context_lens;
        t.part_o = part_o;
        t.part_lse = part_lse;
        t.q_stride_token = p->q_stride_token;
        t.q_stride_head = p->q_stride_head;
        t.sys_stride_token = p->sys_stride_token;
        t.sys_stride_head = p->sys_stride_head;
        t.n_tokens = total_q;
        t.Hq = p->num_q_heads;
        t.Hkv = p->num_kv_heads;
        t.G = pl.group;
        t.sys_chunk = pl.sys_chunk > 0 ? pl.sys_chunk : 128;
        t.n_sys_chunks = pl.n_sys_chunks;
        t.n_prefixes = num_prefixes;
        t.n_sys_rowblocks = pl.rows_sys ? pl.n_sys_rowblocks : 0;
        int items = 0;
        for (int i = 0; i < num_prefixes; ++i) {
            const int mt = pl.rows_sys ? pl.n_sys_rowblocks
                                       : ceil_div(prefixes[i].num_requests * pl.group, 32);
            items += p->num_kv_heads * mt * ceil_div(prefixes[i].sys_len, t.sys_chunk);
            t.pfx_item_end[i] = items;
            t.pfx_first[i] = prefixes[i].first_request;
            t.pfx_tokens[i] = prefixes[i].num_requests;
            t.pfx_len[i] = prefixes[i].sys_len;
            t.pfx_k[i] = static_cast<const uint16_t *>(prefixes[i].k_sys);
            t.pfx_v[i] = static_cast<const uint16_t *>(prefixes[i].v_sys);
        }
        t.n_sys_items = items;
        t.sys_read_once = read_once ? 1 : 0;
        t.ctx_waves = pl.ctx_wgs * 4;
        t.ctx_t_floor = pl.ctx_t_floor;
        {
            const int64_t cap = ((int64_t)ra::kMaxPartBlocks - 1) * p->block_size / 32;
            t.ctx_t_cap = (int)(cap < 1 ? 1 : cap > INT32_MAX / 2 ? INT32_MAX / 2 : cap);
        }
        t.n_ctx_slots = pl.n_ctx_parts;
        t.max_ctx = pl.max_ctx;
        // Workgroups i and i + 256 of a 512-workgroup grid share a compute unit: the context
        // workgroups 256 .. 256 + n_sys - 1 sit next to a system workgroup.
        if (pl.paired && items + pl.ctx_wgs == kWorkgroupSlots && items <= kWorkgroupSlots / 2) {
            t.ctx_light_begin = (kWorkgroupSlots / 2 - items) * 4;
            t.ctx_light_waves = items * 4;
            t.sys_wg_tiles = ceil_div(t.sys_chunk, 32);
            int64_t sum = 0;
            for (int i = 0; i < num_prefixes; ++i)      // (tiles fetched, once per workgroup)
                sum += (int64_t)p->num_kv_heads *
                       (pl.rows_sys ? pl.n_sys_rowblocks : ceil_div(prefixes[i].num_requests * pl.group, 32)) *
                       ceil_div(prefixes[i].sys_len, 32);
            t.sys_tiles_total = (int)(sum > INT32_MAX / 2 ? INT32_MAX / 2 : sum);
        }
        t.block_size_log2 = pl.block_size_log2;
        t.max_blocks_per_seq = p->max_blocks_per_seq;
        t.rows = pl.rows;
        t.sys_head_fastest = head_fastest;
        t.scale_log2 = scale_log2;
        if (timeline) t.timeline = timeline->entries, t.timeline_waves = timeline->waves;
        if (ra::launch_relay_tiles(t, p->head_dim, stream) != hipSuccess) return RA_ERR_HIP;
    }
    // The per-request comparison path.
    if ((mask & 1) && naive) {
        if (pl.n_ctx_parts > 0) {
            ra::CtxArgs c{};
            c.q = static_cast<const uint16_t *>(q);
            c.k_cache = static_cast<const uint16_t *>(k_cache);
            c.v_cache = static_cast<const uint16_t *>(v_cache);
            c.block_tables = block_tables;
            c.context_lens = context_lens;
            c.cu_seqlens_q = nullptr;
            c.part_o = part_o + (size_t)pl.n_sys_chunks * pl.rows * p->head_dim;
            c.part_lse = part_lse + (size_t)pl.n_sys_chunks * pl.rows;
            c.out = out;
            c.lse_out = lse_out;
            c.q_stride_token = p->q_stride_token;
            c.q_stride_head = p->q_stride_head;
            c.o_stride_token = p->o_stride_token;
            c.o_stride_head = p->o_stride_head;
            c.batch = p->batch;
            c.n_tokens = total_q;
            c.Hq = p->num_q_heads;
            c.Hkv = p->num_kv_heads;
            c.block_size_log2 = pl.block_size_log2;
            c.max_blocks_per_seq = p->max_blocks_per_seq;
            c.part_tokens = pl.ctx_part;
            c.n_parts = pl.n_ctx_parts;
            c.rows = pl.rows;
            c.direct = direct ? 1 : 0;
            c.out_is_fp32 = p->out_is_fp32;
            c.scale_log2 = scale_log2;
            if (ra::launch_ctx_decode(c, p->head_dim, pl.group, stream) != hipSuccess)
                return RA_ERR_HIP;
        }
    }
    if ((mask & 2) && !direct && !whole) {
        ra::FuseArgs f{};
        f.part_o = part_o;
        f.part_lse = part_lse;
        f.out = out;
        f.lse_out = lse_out;
        f.o_stride_token = p->o_stride_token;
        f.o_stride_head = p->o_stride_head;
        f.rows = pl.rows;
        f.Hq = p->num_q_heads;
        f.n_partials = pl.n_sys_chunks + pl.n_ctx_parts;
        f.n_sys_chunks = pl.n_sys_chunks;
        f.n_prefixes = num_prefixes;
        f.req_prefix = num_prefixes > 1 ? req_prefix : nullptr;
        for (int i = 0; i < num_prefixes; ++i) {
            f.pfx_token_end[i] = tok0[i] + ntok[i];
            f.pfx_chunks[i] = pl.sys_chunk > 0 ? ceil_div(prefixes[i].sys_len, pl.sys_chunk) : 0;
        }
        f.out_is_fp32 = p->out_is_fp32;
        if (ra::launch_fuse(f, p->head_dim, stream) != hipSuccess) return RA_ERR_HIP;
    }
    return RA_OK;
}

}  // namespace

extern "C" {

size_t relay_attn_workspace_bytes(const ra_params *p, int32_t total_q) {
    if (check_params(p, total_q) != RA_OK) return 0;
    // the caller does not say which entry point will use the workspace: cover both
    size_t most = 0;
    for (PlanKind kind : {kRelayDecode, kNaiveDecode, kPrefill}) {
        const Plan pl = make_plan(p, total_q, kind, kind == kPrefill ? total_q : 1);
        if (!pl.unsupported && pl.bytes > most) most = pl.bytes;
    }
    // (a call with several prefixes may fall back to the decode plan without many-rows items)
    const Plan blind = make_plan(p, total_q, kRelayDecode, 1, 0, false);
    if (!blind.unsupported && blind.bytes > most) most = blind.bytes;
    return most;
}

ra_status relay_attn_decode_plan(const ra_params *p, ra_decode_plan *plan) {
    if (!plan) return RA_ERR_INVALID_ARG;
    const ra_status st = check_params(p, p ? p->batch : 0);
    if (st != RA_OK) return st;
    const Plan pl = make_plan(p, p->batch, kRelayDecode, 1);
    if (pl.unsupported) return RA_ERR_UNSUPPORTED;
    plan->sys_chunk_tokens = pl.sys_chunk;
    plan->num_sys_chunks = pl.n_sys_chunks;
    plan->sys_rows_per_workgroup = pl.rows_sys ? 128 : 32;
    plan->num_sys_workgroups =
        p->num_kv_heads * (pl.rows_sys ? pl.n_sys_rowblocks : pl.n_mtiles) * pl.n_sys_chunks;
    plan->num_ctx_wavefronts = pl.ctx_wgs * 4;
    plan->min_tiles_per_ctx_wavefront = pl.ctx_t_floor;
    plan->num_ctx_slots = pl.n_ctx_parts;
    plan->max_blocks_per_span = ra::kMaxPartBlocks;
    plan->first_light_ctx_wavefront = 0;
    plan->num_light_ctx_wavefronts = 0;
    plan->compute_units = device_compute_units();
    const int kWorkgroupSlots = plan->compute_units * 2;
    plan->sys_workgroup_tiles = pl.sys_chunk > 0 ? ceil_div(pl.sys_chunk, 32) : 0;
    plan->sys_tiles_total = p->num_kv_heads * (pl.rows_sys ? pl.n_sys_rowblocks : pl.n_mtiles) *
                            ceil_div(p->sys_len, 32);
    if (pl.paired && plan->num_sys_workgroups + pl.ctx_wgs == kWorkgroupSlots &&
        plan->num_sys_workgroups <= kWorkgroupSlots / 2) {
        plan->first_light_ctx_wavefront = (kWorkgroupSlots / 2 - plan->num_sys_workgroups) * 4;
        plan->num_light_ctx_wavefronts = plan->num_sys_workgroups * 4;
    }
    return RA_OK;
}

ra_status relay_attn_decode(const ra_params *p, const void *q, const void *k_sys,
                            const void *v_sys, const void *k_cache, const void *v_cache,
                            const int32_t *block_tables, const int32_t *context_lens, void *out,
                            float *lse_out, void *workspace, size_t workspace_bytes,
                            void *hip_stream) {
    if (!p) return RA_ERR_INVALID_ARG;
    return run(p, q, nullptr, p->batch, 1, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, false);
}

ra_status relay_attn_decode_append(const ra_params *p, const void *q, const void *k_new,
                                   const void *v_new, int64_t new_stride_token,
                                   int64_t new_stride_head, const void *k_sys, const void *v_sys,
                                   void *k_cache, void *v_cache, const int32_t *block_tables,
                                   const int32_t *context_lens, void *out, float *lse_out,
                                   void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!p) return RA_ERR_INVALID_ARG;
    NewRows rows;
    rows.k = k_new;
    rows.v = v_new;
    rows.stride_token = new_stride_token;
    rows.stride_head = new_stride_head;
    return run(p, q, nullptr, p->batch, 1, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, false, 0, nullptr,
               3, &rows);
}

size_t relay_attn_static_scratch_bytes(void) { return kStaticScratchBytes; }

ra_status relay_attn_decode_static(const ra_params *p, const void *q, const void *k_sys,
                                   const void *v_sys, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   void *out, float *lse_out, void *hip_stream) {
    if (!p) return RA_ERR_INVALID_ARG;
    ra_status st = check_params(p, p->batch);
    if (st != RA_OK) return st;
    // the same decomposition relay_attn_decode uses, so the same kernels and the same result
    const Plan pl = make_plan(p, p->batch, kRelayDecode, 1);
    if (pl.unsupported) return RA_ERR_UNSUPPORTED;
    if (pl.bytes > kStaticScratchBytes) return RA_ERR_WORKSPACE_TOO_SMALL;
    if (p->batch == 0) return RA_OK;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != RA_OK) return st;
    return run(p, q, nullptr, p->batch, 1, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, ws, kStaticScratchBytes, hip_stream, false);
}

ra_status relay_attn_debug_decode_phases(const ra_params *p, int32_t phases, const void *q,
                                         const void *k_sys, const void *v_sys, const void *k_cache,
                                         const void *v_cache, const int32_t *block_tables,
                                         const int32_t *context_lens, void *out, float *lse_out,
                                         void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!p || phases < 1 || phases > 3) return RA_ERR_INVALID_ARG;
    return run(p, q, nullptr, p->batch, 1, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, false, 0, nullptr,
               phases);
}

ra_status relay_attn_debug_timeline(const ra_params *p, const void *q, const int32_t *cu_seqlens_q,
                                    int32_t total_q, int32_t max_q_len, const void *k_sys,
                                    const void *v_sys, const void *k_cache, const void *v_cache,
                                    const int32_t *block_tables, const int32_t *context_lens,
                                    void *out, float *lse_out, void *workspace,
                                    size_t workspace_bytes, uint64_t *timeline,
                                    int32_t timeline_wavefronts, void *hip_stream) {
    if (!p || !timeline || timeline_wavefronts < 1 || (reinterpret_cast<uintptr_t>(timeline) & 7u))
        return RA_ERR_INVALID_ARG;
    if (!cu_seqlens_q && (total_q != p->batch || max_q_len != 1)) return RA_ERR_INVALID_ARG;
    Timeline tl;
    tl.entries = reinterpret_cast<unsigned long long *>(timeline);
    tl.waves = timeline_wavefronts;
    return run(p, q, cu_seqlens_q, total_q, max_q_len, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, false, 0, nullptr, 3,
               nullptr, nullptr, nullptr, nullptr, &tl);
}

ra_status relay_attn_decode_multi(const ra_params *p, int32_t num_prefixes,
                                  const ra_prefix *prefixes, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *block_tables,
                                  const int32_t *context_lens, void *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!p || !prefixes || num_prefixes < 1) return RA_ERR_INVALID_ARG;
    if (num_prefixes > ra::kMaxPrefixes) return RA_ERR_UNSUPPORTED;
    int next = 0, longest = 0, longest_at = 0;
    for (int i = 0; i < num_prefixes; ++i) {           // groups tile the batch, in order
        const ra_prefix &f = prefixes[i];
        if (f.first_request != next || f.num_requests < 1 || f.sys_len < 0) return RA_ERR_INVALID_ARG;
        if (f.sys_len > 0 && (!f.k_sys || !f.v_sys || !aligned16(f.k_sys) || !aligned16(f.v_sys)))
            return RA_ERR_INVALID_ARG;
        next += f.num_requests;
        if (f.sys_len > longest) longest = f.sys_len, longest_at = i;
    }
    if (next != p->batch || longest != p->sys_len) return RA_ERR_INVALID_ARG;
    return run(p, q, nullptr, p->batch, 1, prefixes[longest_at].k_sys, prefixes[longest_at].v_sys,
               k_cache, v_cache,
               block_tables, context_lens, out, lse_out, workspace, workspace_bytes, hip_stream,
               false, num_prefixes, prefixes);
}

ra_status relay_attn_group_requests(const int32_t *sys_id, int32_t batch, int32_t num_prefixes,
                                    int32_t *request_order, int32_t *num_requests) {
    if (batch < 0 || num_prefixes < 1 || !num_requests || (batch > 0 && (!sys_id || !request_order)))
        return RA_ERR_INVALID_ARG;
    for (int i = 0; i < num_prefixes; ++i) num_requests[i] = 0;
    for (int r = 0; r < batch; ++r) {
        if (sys_id[r] < 0 || sys_id[r] >= num_prefixes) return RA_ERR_INVALID_ARG;
        ++num_requests[sys_id[r]];
    }
    // counting sort: the requests of prefix 0 in batch order, then those of prefix 1, ...
    int32_t at = 0;
    for (int i = 0; i < num_prefixes; ++i) {
        for (int r = 0; r < batch; ++r)
            if (sys_id[r] == i) request_order[at++] = r;
    }
    return RA_OK;
}

ra_status relay_attn_decode_grouped(const ra_params *p, int32_t num_prefixes,
                                    const ra_prefix *prefixes, const int32_t *sys_id,
                                    const int32_t *request_order, const void *q,
                                    const void *k_cache, const void *v_cache,
                                    const int32_t *block_tables, const int32_t *context_lens,
                                    void *out, float *lse_out, void *workspace,
                                    size_t workspace_bytes, void *hip_stream) {
    if (!p || !prefixes || num_prefixes < 1) return RA_ERR_INVALID_ARG;
    if (num_prefixes > ra::kMaxPrefixes) return RA_ERR_UNSUPPORTED;
    if (p->batch > 0 && (!sys_id || !request_order)) return RA_ERR_INVALID_ARG;
    // the same per-prefix table as relay_attn_decode_multi, with runs of request_order in place of
    // runs of the batch
    ra_prefix used[ra::kMaxPrefixes];
    int n_used = 0, next = 0, longest = 0, longest_at = -1;
    for (int i = 0; i < num_prefixes; ++i) {
        const ra_prefix &f = prefixes[i];
        if (f.num_requests < 0 || f.sys_len < 0) return RA_ERR_INVALID_ARG;
        if (f.sys_len > 0 && (!f.k_sys || !f.v_sys || !aligned16(f.k_sys) || !aligned16(f.v_sys)))
            return RA_ERR_INVALID_ARG;
        // (the fusion launch looks chunk counts up by sys_id, so the table keeps every prefix, with
        // zero requests where none uses it)
        used[n_used] = f;
        used[n_used].first_request = next;
        ++n_used;
        next += f.num_requests;
        if (f.num_requests > 0 && f.sys_len >= longest) {
            if (f.sys_len > longest || longest_at < 0) longest_at = i;
            longest = f.sys_len;
        }
    }
    if (next != p->batch || longest != p->sys_len) return RA_ERR_INVALID_ARG;
    if (p->batch == 0) longest_at = 0;
    return run(p, q, nullptr, p->batch, 1, prefixes[longest_at].k_sys, prefixes[longest_at].v_sys,
               k_cache, v_cache, block_tables, context_lens, out, lse_out, workspace,
               workspace_bytes, hip_stream, false, n_used, used, 3, nullptr, request_order, sys_id);
}

ra_status relay_attn_prefill(const ra_params *p, const void *q, const int32_t *cu_seqlens_q,
                             int32_t total_q, int32_t max_q_len, const void *k_sys,
                             const void *v_sys, const void *k_cache, const void *v_cache,
                             const int32_t *block_tables, const int32_t *context_lens, void *out,
                             float *lse_out, void *workspace, size_t workspace_bytes,
                             void *hip_stream) {
    if (!p || max_q_len < 0 || total_q < 0) return RA_ERR_INVALID_ARG;
    if (total_q > 0 && (!cu_seqlens_q || p->batch < 1)) return RA_ERR_INVALID_ARG;
    if ((int64_t)max_q_len * p->batch < total_q) return RA_ERR_INVALID_ARG;
    return run(p, q, cu_seqlens_q, total_q, max_q_len, k_sys, v_sys, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, false);
}

ra_status relay_attn_prefill_multi(const ra_params *p, int32_t num_prefixes,
                                   const ra_prefix *prefixes, const int32_t *prefix_num_tokens,
                                   const void *q, const int32_t *cu_seqlens_q, int32_t total_q,
                                   int32_t max_q_len, const void *k_cache, const void *v_cache,
                                   const int32_t *block_tables, const int32_t *context_lens,
                                   void *out, float *lse_out, void *workspace,
                                   size_t workspace_bytes, void *hip_stream) {
    if (!p || !prefixes || !prefix_num_tokens || num_prefixes < 1 || max_q_len < 0 || total_q < 0)
        return RA_ERR_INVALID_ARG;
    if (num_prefixes > ra::kMaxPrefixes) return RA_ERR_UNSUPPORTED;
    if (total_q > 0 && (!cu_seqlens_q || p->batch < 1)) return RA_ERR_INVALID_ARG;
    if ((int64_t)max_q_len * p->batch < total_q) return RA_ERR_INVALID_ARG;
    int next = 0, longest = 0, longest_at = 0;
    int64_t tokens = 0;
    for (int i = 0; i < num_prefixes; ++i) {           // groups tile the batch, in order
        const ra_prefix &f = prefixes[i];
        if (f.first_request != next || f.num_requests < 1 || f.sys_len < 0) return RA_ERR_INVALID_ARG;
        if (prefix_num_tokens[i] < 0 || (int64_t)prefix_num_tokens[i] > (int64_t)f.num_requests * max_q_len)
            return RA_ERR_INVALID_ARG;
        if (f.sys_len > 0 && (!f.k_sys || !f.v_sys || !aligned16(f.k_sys) || !aligned16(f.v_sys)))
            return RA_ERR_INVALID_ARG;
        next += f.num_requests;
        tokens += prefix_num_tokens[i];
        if (f.sys_len > longest) longest = f.sys_len, longest_at = i;
    }
    if (next != p->batch || tokens != total_q || longest != p->sys_len) return RA_ERR_INVALID_ARG;
    if (total_q == 0 && !cu_seqlens_q) {
        // (run() tells the prompt phase from decode by this pointer; an empty call has nothing to do)
        const ra_status st = check_params(p, 0);
        return st;
    }
    return run(p, q, cu_seqlens_q, total_q, max_q_len, prefixes[longest_at].k_sys,
               prefixes[longest_at].v_sys, k_cache, v_cache, block_tables, context_lens, out, lse_out,
               workspace, workspace_bytes, hip_stream, false, num_prefixes, prefixes, 3, nullptr,
               nullptr, nullptr, prefix_num_tokens);
}

ra_status paged_attn_decode_naive(const ra_params *p, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *block_tables,
                                  const int32_t *context_lens, void *out, float *lse_out,
                                  void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!p) return RA_ERR_INVALID_ARG;
    return run(p, q, nullptr, p->batch, 1, nullptr, nullptr, k_cache, v_cache, block_tables,
               context_lens, out, lse_out, workspace, workspace_bytes, hip_stream, true);
}

ra_status relay_attn_cache_append(const ra_params *p, const void *k_new, const void *v_new,
                                  int64_t new_stride_token, int64_t new_stride_head,
                                  const int32_t *cu_seqlens_q, int32_t total_q, void *k_cache,
                                  void *v_cache, const int32_t *block_tables,
                                  const int32_t *context_lens, void *hip_stream) {
    ra_status st = check_params(p, total_q);
    if (st != RA_OK) return st;
    if (new_stride_token < 0 || new_stride_head < 0 || new_stride_token % 8 || new_stride_head % 8)
        return RA_ERR_INVALID_ARG;
    if (!cu_seqlens_q && total_q != p->batch) return RA_ERR_INVALID_ARG;
    if (total_q == 0) return RA_OK;
    if (p->batch < 1 || !k_new || !v_new || !k_cache || !v_cache || !block_tables || !context_lens)
        return RA_ERR_INVALID_ARG;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache))
        return RA_ERR_INVALID_ARG;
    if (new_stride_head < p->head_dim && p->num_kv_heads > 1) return RA_ERR_INVALID_ARG;
    ra::AppendArgs a{};
    a.k_new = static_cast<const uint16_t *>(k_new);
    a.v_new = static_cast<const uint16_t *>(v_new);
    a.k_cache = static_cast<uint16_t *>(k_cache);
    a.v_cache = static_cast<uint16_t *>(v_cache);
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.cu_seqlens_q = cu_seqlens_q;
    a.new_stride_token = new_stride_token;
    a.new_stride_head = new_stride_head;
    a.batch = p->batch;
    a.total_q = total_q;
    a.Hkv = p->num_kv_heads;
    a.head_dim = p->head_dim;
    a.block_size_log2 = 0;
    while ((1 << a.block_size_log2) < p->block_size) ++a.block_size_log2;
    a.max_blocks_per_seq = p->max_blocks_per_seq;
    if (ra::launch_cache_append(a, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return RA_ERR_HIP;
    return RA_OK;
}

ra_status relay_attn_system_cache_layout(const ra_params *p, int64_t *stride_token_out,
                                         int64_t *stride_head_out, size_t *bytes_out) {
    if (!p || !stride_token_out || !stride_head_out || !bytes_out) return RA_ERR_INVALID_ARG;
    if (p->num_kv_heads < 1 || p->head_dim < 1 || p->head_dim % 8 || p->sys_len < 0)
        return RA_ERR_INVALID_ARG;
    // the smallest row stride >= the dense one that is 384 mod 1024 bytes (192 mod 512 elements)
    const int64_t dense = (int64_t)p->num_kv_heads * p->head_dim;
    int64_t stride = dense / 512 * 512 + 192;
    if (stride < dense) stride += 512;
    *stride_token_out = stride;
    *stride_head_out = p->head_dim;
    // (the last row needs no padding behind it)
    *bytes_out = p->sys_len > 0 ? (size_t)(((int64_t)p->sys_len - 1) * stride + dense) * 2 : 0;
    return RA_OK;
}

ra_status relay_attn_system_fill(const ra_params *p, const void *k_new, const void *v_new,
                                 int64_t new_stride_token, int64_t new_stride_head,
                                 int32_t first_pos, int32_t num_pos, void *k_sys, void *v_sys,
                                 void *hip_stream) {
    ra_status st = check_params(p, 0);
    if (st != RA_OK) return st;
    if (new_stride_token < 0 || new_stride_head < 0 || new_stride_token % 8 || new_stride_head % 8)
        return RA_ERR_INVALID_ARG;
    if (first_pos < 0 || num_pos < 0 || (int64_t)first_pos + num_pos > p->sys_len)
        return RA_ERR_INVALID_ARG;
    if (num_pos == 0) return RA_OK;
    if (!k_new || !v_new || !k_sys || !v_sys) return RA_ERR_INVALID_ARG;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_sys) || !aligned16(v_sys))
        return RA_ERR_INVALID_ARG;
    if (new_stride_head < p->head_dim && p->num_kv_heads > 1) return RA_ERR_INVALID_ARG;
    if (p->sys_stride_head < p->head_dim && p->num_kv_heads > 1) return RA_ERR_INVALID_ARG;
    if (p->sys_stride_token < p->head_dim && p->sys_len > 1) return RA_ERR_INVALID_ARG;
    ra::SysFillArgs a{};
    a.k_new = static_cast<const uint16_t *>(k_new);
    a.v_new = static_cast<const uint16_t *>(v_new);
    a.k_sys = static_cast<uint16_t *>(k_sys);
    a.v_sys = static_cast<uint16_t *>(v_sys);
    a.new_stride_token = new_stride_token;
    a.new_stride_head = new_stride_head;
    a.sys_stride_token = p->sys_stride_token;
    a.sys_stride_head = p->sys_stride_head;
    a.first_pos = first_pos;
    a.num_pos = num_pos;
    a.Hkv = p->num_kv_heads;
    a.head_dim = p->head_dim;
    if (ra::launch_system_fill(a, static_cast<hipStream_t>(hip_stream)) != hipSuccess)
        return RA_ERR_HIP;
    return RA_OK;
}

ra_status relay_attn_debug_validate(const ra_params *p, const int32_t *block_tables,
                                    const int32_t *context_lens, const int32_t *cu_seqlens_q,
                                    int32_t total_q, void *workspace, size_t workspace_bytes,
                                    void *hip_stream, ra_validate_report *report) {
    const ra_status st = check_params(p, total_q);
    if (st != RA_OK) return st;
    if (!cu_seqlens_q && total_q != p->batch) return RA_ERR_INVALID_ARG;
    if (p->batch > 0 && (!context_lens || (!block_tables && p->max_blocks_per_seq > 0)))
        return RA_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return RA_ERR_INVALID_ARG;
    if (workspace_bytes < 256) return RA_ERR_WORKSPACE_TOO_SMALL;
    ra::ValidateArgs a{};
    a.block_tables = block_tables;
    a.context_lens = context_lens;
    a.cu_seqlens_q = cu_seqlens_q;
    a.counters = static_cast<int32_t *>(workspace);
    a.batch = p->batch;
    a.total_q = total_q;
    a.num_blocks = p->num_blocks;
    a.block_size_log2 = 0;
    while ((1 << a.block_size_log2) < p->block_size) ++a.block_size_log2;
    a.max_blocks_per_seq = p->max_blocks_per_seq;
    a.max_len = p->max_context_len > 0 ? p->max_context_len : p->max_blocks_per_seq * p->block_size;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (ra::launch_validate(a, stream) != hipSuccess) return RA_ERR_HIP;
    int32_t host[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(host, a.counters, sizeof(host), hipMemcpyDeviceToHost, stream) != hipSuccess)
        return RA_ERR_HIP;
    if (hipStreamSynchronize(stream) != hipSuccess) return RA_ERR_HIP;
    const bool clean = host[0] == 0 && host[1] == 0 && host[2] == 0;
    if (report) {
        report->bad_context_lens = host[0];
        report->bad_block_ids = host[1];
        report->bad_query_lens = host[2];
        report->first_bad_request = clean ? -1 : host[3];
    }
    return clean ? RA_OK : RA_ERR_INVALID_ARG;
}

ra_status relay_attn_debug_stream_probe(const void *src, size_t bytes, int32_t nontemporal,
                                        void *sink, void *hip_stream) {
    if (!src || !sink || !aligned16(src) || (bytes % 16) != 0) return RA_ERR_INVALID_ARG;
    if (nontemporal != 0 && nontemporal != 1) return RA_ERR_INVALID_ARG;
    if (ra::launch_stream_probe(src, bytes, nontemporal, sink, static_cast<hipStream_t>(hip_stream)) !=
        hipSuccess)
        return RA_ERR_HIP;
    return RA_OK;
}

ra_status relay_attn_debug_launch_probe(void *sink, int32_t count, void *hip_stream) {
    if (!sink || count < 0 || count > (1 << 20)) return RA_ERR_INVALID_ARG;
    if (ra::launch_empty_probe(sink, count, static_cast<hipStream_t>(hip_stream)) != hipSuccess) return RA_ERR_HIP;
    return RA_OK;
}

const char *relay_attn_status_string(ra_status status) {
    switch (status) {
        case RA_OK: return "ok";
        case RA_ERR_INVALID_ARG: return "invalid argument";
        case RA_ERR_UNSUPPORTED: return "unsupported configuration";
        case RA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case RA_ERR_HIP: return "HIP call failed";
    }
    return "unknown status";
}

int32_t relay_attn_abi_version(void) { return kAbiVersion; }

}  // extern "C"
