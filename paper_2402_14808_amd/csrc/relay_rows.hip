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
// Per tile: 256 threads load K and V rows with coalesced 16-byte loads into registers (issued two
// tiles ahead, into two alternating sets of landing registers), store them XOR-swizzled into the
// other half of a double-buffered LDS tile, one barrier; each wavefront then computes S^T = K Q^T (v_mfma_f32_32x32x16_bf16, K operands by
// ds_read_b128, Q in registers), the online softmax for its 32 query columns, and
// O^T += V^T P^T with V^T operands from the LDS transpose read ds_read_b64_tr_b16 and P^T taken
// from the S^T accumulators as a bf16 high + low pair.  Each wavefront owns its rows for the whole
// key range, so the partial (normalised output, base-2 log-sum-exp) is written from registers.
#include "rows_item.h"

namespace ra {

template <int D, bool MULTI>
__global__ __launch_bounds__(kThreads, 2) void relay_rows_kernel(const RowsArgs a) {
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * 2 * 64 * D * 2];
    __shared__ int32_t sm_tbl[kMaxPartBlocks];
    rows_item<D, false, MULTI>(a, (int)blockIdx.x, lds, sm_tbl);
}

hipError_t launch_relay_rows(const RowsArgs &a, int head_dim, hipStream_t stream) {
    const int64_t groups = (int64_t)a.n_sys_items + a.n_ctx_items;
    if (groups == 0) return hipSuccess;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    const bool multi = a.n_prefixes > 1;
    const dim3 grid((unsigned)groups), block(kThreads);
    if (head_dim == 128 && multi) hipLaunchKernelGGL((relay_rows_kernel<128, true>), grid, block, 0, stream, a);
    else if (head_dim == 128) hipLaunchKernelGGL((relay_rows_kernel<128, false>), grid, block, 0, stream, a);
    else if (head_dim == 64 && multi) hipLaunchKernelGGL((relay_rows_kernel<64, true>), grid, block, 0, stream, a);
    else if (head_dim == 64) hipLaunchKernelGGL((relay_rows_kernel<64, false>), grid, block, 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ra
