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

// Measurement aids behind the roofline discussion of the decode path: a read-only streaming
// kernel (what the memory system delivers to coalesced 16-byte loads, ordinary or non-temporal,
// with nothing else going on) and an empty kernel (what a launch costs in a stream by itself).
template <bool NT>
__global__ __launch_bounds__(kThreads) void stream_probe_kernel(const u32x4 *src, size_t vec_per_wg,
                                                                size_t n_vec, uint32_t *sink) {
    constexpr int U = 8;                           // loads in flight per lane
    const size_t first = (size_t)blockIdx.x * vec_per_wg;
    const size_t last = first + vec_per_wg < n_vec ? first + vec_per_wg : n_vec;
    uint32_t acc = 0;
    for (size_t i = first + threadIdx.x; i < last; i += (size_t)kThreads * U) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = i + (size_t)u * kThreads;
            v[u] = u32x4{0, 0, 0, 0};
            if (j < last) v[u] = NT ? __builtin_nontemporal_load(src + j) : src[j];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    }
    if (acc == 0x9E3779B9u) sink[0] = acc;         // keeps the loads alive; practically never taken
}

__global__ void empty_probe_kernel(uint32_t *sink) {
    if (sink == nullptr) return;                   // (an argument, so that the launch carries one)
}

hipError_t launch_stream_probe(const void *src, size_t bytes, int nontemporal, void *sink,
                               hipStream_t stream) {
    const size_t n_vec = bytes / 16;
    const size_t vec_per_wg = (256u << 10) / 16;   // 256 KiB per workgroup
    const size_t groups = (n_vec + vec_per_wg - 1) / vec_per_wg;
    if (groups == 0) return hipSuccess;
    if (groups > 0x7fffffffu) return hipErrorInvalidValue;
    if (nontemporal)
        hipLaunchKernelGGL(stream_probe_kernel<true>, dim3((unsigned)groups), dim3(kThreads), 0, stream,
                           static_cast<const u32x4 *>(src), vec_per_wg, n_vec, static_cast<uint32_t *>(sink));
    else
        hipLaunchKernelGGL(stream_probe_kernel<false>, dim3((unsigned)groups), dim3(kThreads), 0, stream,
                           static_cast<const u32x4 *>(src), vec_per_wg, n_vec, static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

hipError_t launch_empty_probe(void *sink, int count, hipStream_t stream) {
    for (int i = 0; i < count; ++i)
        hipLaunchKernelGGL(empty_probe_kernel, dim3(1), dim3(64), 0, stream, static_cast<uint32_t *>(sink));
    return hipGetLastError();
}

}  // namespace ra
