// Partial attention for MANY query rows per kv head: the prompt phase (Alg. 1 with more than one
// new token per request; Sec. 3.3 notes that the reformulation does not assume a single query
// token) and the system attention of decode batches whose stacked rows B*G exceed a few tiles.
// Here the products are large matrix multiplications (Sec. 3.2, footnote on the prompt phase), so
// the kernel is organised for the matrix unit, not for streaming: a workgroup owns 128 stacked
// query rows (one 32-row tile per wavefront) of one kv head and walks a key range in tiles of 32;
// every K/V tile is fetched ONCE per workgroup into LDS and used by all four wavefronts.
//
//   system item   (kv head, row block, chunk of system positions): no mask (Alg. 1 passes none;
//                 system positions precede every request token);
//   context item  (request, kv head, row block of that request's new tokens, context part):
//                 causal, new token j of m sees context positions 0 .. c-m+j (the new tokens are
//                 the last m positions of the context, which was appended before attending).
//
//   whole item    (kv head, block of 128 stacked rows): the system prompt and then the causal
//                 context of every request that has rows in the block, in one item that writes
//                 the output rows itself: no partials, no fusion launch (used when the system
//                 prompt is one chunk and the requests bring many new tokens each).
//
// Per step of 64 keys: 256 threads load the K and V rows straight into the other half of a
// double-buffered, XOR-swizzled LDS tile (global_load_lds_dwordx4), one barrier; each wavefront
// then computes S^T = K Q^T (v_mfma_f32_32x32x16_bf16, K operands by ds_read_b128, Q in registers),
// the online softmax for its 32 query columns, and O^T += V^T P^T with V^T operands from the LDS
// transpose read ds_read_b64_tr_b16 and P^T taken from the S^T accumulators as a bf16 high + low
// pair.  Each wavefront owns its rows for the whole key range, so the partial (normalised output,
// base-2 log-sum-exp) or the output row is written from registers.
#include "rows_item.h"

namespace ra {

template <int D, bool MULTI, bool WHOLE>
__global__ __launch_bounds__(kThreads, 2) void relay_rows_kernel(const RowsArgs a) {
    const unsigned long long t_begin = a.timeline ? __builtin_amdgcn_s_memrealtime() : 0ull;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * 2 * 64 * D * 2];
    __shared__ int32_t sm_tbl[kMaxPartBlocks];
    rows_item<D, false, MULTI, WHOLE>(a, (int)blockIdx.x, lds, sm_tbl);
    if (a.timeline) {
        const unsigned w = blockIdx.x * (kThreads / kWave) + threadIdx.x / kWave;
        if (threadIdx.x % kWave == 0 && w < (unsigned)a.timeline_waves) {
            a.timeline[2 * w] = t_begin;
            a.timeline[2 * w + 1] = __builtin_amdgcn_s_memrealtime();
        }
    }
}

hipError_t launch_relay_rows(const RowsArgs &a, int head_dim, hipStream_t stream) {
    const int64_t groups = (int64_t)a.n_sys_items + (a.whole ? 0 : a.n_ctx_items);
    if (groups == 0) return hipSuccess;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    const bool multi = a.n_prefixes > 1;
    if (a.whole && (a.n_sys_chunks != 1 || !a.cu_seqlens_q || !a.out)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)groups), block(kThreads);
#define RA_ROWS(D_, MULTI_, WHOLE_) \
    hipLaunchKernelGGL((relay_rows_kernel<D_, MULTI_, WHOLE_>), grid, block, 0, stream, a)
#define RA_ROWS_D(D_)                               \
    do {                                            \
        if (a.whole && multi) RA_ROWS(D_, true, true);   \
        else if (a.whole) RA_ROWS(D_, false, true); \
        else if (multi) RA_ROWS(D_, true, false);   \
        else RA_ROWS(D_, false, false);             \
    } while (0)
    if (head_dim == 128) RA_ROWS_D(128);
    else if (head_dim == 64) RA_ROWS_D(64);
    else return hipErrorInvalidValue;
#undef RA_ROWS_D
#undef RA_ROWS
    return hipGetLastError();
}

}  // namespace ra
