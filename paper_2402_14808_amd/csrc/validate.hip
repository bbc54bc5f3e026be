// Range check of the index arrays the attention kernels take on trust (Alg. 1 indexes the paged
// cache with the block table and the lengths): one workgroup per request counts the entries that
// are out of range.  A debugging aid, never on the serving path.
#include <limits.h>

#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

__global__ void validate_init_kernel(int32_t *counters) {
    if (threadIdx.x < 3) counters[threadIdx.x] = 0;
    if (threadIdx.x == 3) counters[3] = INT_MAX;
}

__global__ __launch_bounds__(kThreads) void validate_kernel(const ValidateArgs a) {
    const int req = blockIdx.x;
    const int len = a.context_lens[req];
    const bool len_ok = len >= 0 && len <= a.max_len;
    bool bad = false;
    if (threadIdx.x == 0) {
        if (!len_ok) {
            atomicAdd(&a.counters[0], 1);
            bad = true;
        }
        if (a.cu_seqlens_q) {
            const int q0 = a.cu_seqlens_q[req], q1 = a.cu_seqlens_q[req + 1];
            const bool ends_ok = (req != 0 || q0 == 0) && (req != a.batch - 1 || q1 == a.total_q);
            if (!ends_ok || q1 < q0 || (len_ok && q1 - q0 > len)) {
                atomicAdd(&a.counters[2], 1);
                bad = true;
            }
        }
    }
    if (len_ok) {
        const int used = (len + (1 << a.block_size_log2) - 1) >> a.block_size_log2;
        const int32_t *row = a.block_tables + (int64_t)req * a.max_blocks_per_seq;
        int n_bad = 0;
        for (int j = threadIdx.x; j < used; j += kThreads) {
            const int32_t b = row[j];
            if (b < 0 || b >= a.num_blocks) ++n_bad;
        }
        if (n_bad > 0) {
            atomicAdd(&a.counters[1], n_bad);
            bad = true;
        }
    }
    if (bad) atomicMin(&a.counters[3], req);
}

hipError_t launch_validate(const ValidateArgs &a, hipStream_t stream) {
    hipLaunchKernelGGL(validate_init_kernel, dim3(1), dim3(64), 0, stream, a.counters);
    if (a.batch > 0)
        hipLaunchKernelGGL(validate_kernel, dim3((unsigned)a.batch), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

}  // namespace ra
