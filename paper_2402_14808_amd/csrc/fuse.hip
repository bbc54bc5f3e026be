// Relay fusion (Alg. 1 "relay fusion"; App. A, Eq. 11-12).  With two partials the output is
//   out = alpha_sys * o_sys + (1 - alpha_sys) * o_ctx,  alpha_sys = 1 / (1 + exp(lse_ctx - lse_sys)).
// The system prompt is processed in several chunks and long contexts in several parts, so the
// same identity is applied to n partials in its max-shifted form: with M = max_p lse_p and
// w_p = exp(lse_p - M), out = sum_p w_p o_p / sum_p w_p and lse = M + log sum_p w_p.  For two
// partials w_sys / (w_sys + w_ctx) is exactly alpha_sys.  Log-sum-exps are kept in base 2
// internally and converted to natural log only for lse_out.
#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

template <int D, bool MULTI>
__global__ __launch_bounds__(kThreads) void fuse_kernel(const FuseArgs a) {
    constexpr int TPR = D / 4;                  // threads per output row (4 elements each)
    constexpr int RPB = kThreads / TPR;         // rows per block
    const int row = blockIdx.x * RPB + threadIdx.x / TPR;
    const int e = (threadIdx.x % TPR) * 4;
    if (row >= a.rows) return;

    // Loads are issued eight partials at a time before any of them is used: the partials were
    // written by other compute units, so each one costs a trip to L2 or memory, and a loop that
    // consumed them one by one would pay those trips back to back.  To keep the eight loads free of
    // branches a slot that does not exist is loaded from slot 0 and discarded by a select.
    constexpr int U = 8;
    // With several shared prefixes (App. D) a request whose prefix is shorter than the longest one
    // has fewer system chunks; the partial slots [skip_lo, skip_hi) of its rows were never written.
    int skip_lo = 0, skip_hi = 0;
    if (MULTI) {
        const int token = row / a.Hq;
        int pfx = 0;
        if (a.req_prefix) pfx = a.req_prefix[token];
        else
            while (pfx + 1 < a.n_prefixes && token >= a.pfx_token_end[pfx]) ++pfx;
        skip_lo = a.pfx_chunks[pfx];
        skip_hi = a.n_sys_chunks;
    }
    auto present = [&](int p) {
        return p < a.n_partials && !(MULTI && p >= skip_lo && p < skip_hi);
    };
    // One trip to memory per eight partials: log-sum-exps and payloads are loaded together and
    // merged with a running maximum (the same online rescaling the attention kernels use), rather
    // than reading all log-sum-exps first to find the maximum and then coming back for the rest.
    float M = -INFINITY, W = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < a.n_partials; p0 += U) {
        float l[U];
        f32x4 o[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const bool ok = present(p0 + j);
            const int64_t slot = (int64_t)(ok ? p0 + j : 0) * a.rows + row;
            l[j] = a.part_lse[slot];
            o[j] = *reinterpret_cast<const f32x4 *>(a.part_o + slot * D + e);
            l[j] = ok ? l[j] : -INFINITY;
        }
        float Mb = M;
#pragma unroll
        for (int j = 0; j < U; ++j) Mb = fmaxf(Mb, l[j]);
        const float m_use = finite_or_zero(Mb);
        const float corr = exp2f(M - m_use);      // M = -inf (nothing yet): 0, and acc, W are 0
        acc *= corr;
        W *= corr;
        M = Mb;
#pragma unroll
        for (int j = 0; j < U; ++j) {
            // An empty or absent slot has w = 0; its payload may never have been written (a context
            // slot an item does not use only gets lse = -inf), so it is dropped by a select.
            const float w = exp2f(l[j] - m_use);
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            acc += (w > 0.f ? o[j] : zero) * w;
            W += w;
        }
    }
    const float inv = W > 0.f ? 1.f / W : 0.f;
    acc *= inv;
    const int token = row / a.Hq, hq = row % a.Hq;
    const int64_t oo = (int64_t)token * a.o_stride_token + (int64_t)hq * a.o_stride_head + e;
    if (a.out_is_fp32) {
        *reinterpret_cast<f32x4 *>(static_cast<float *>(a.out) + oo) = acc;
    } else {
        u32x2 w2 = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3])};
        *reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(a.out) + oo) = w2;
    }
    if (e == 0 && a.lse_out) a.lse_out[row] = W > 0.f ? (finite_or_zero(M) + log2f(W)) * kLn2 : -INFINITY;
}

// Cache append: one thread moves 16 bytes of one (token, kv head) row of K and of V.
__global__ __launch_bounds__(kThreads) void cache_append_kernel(const AppendArgs a) {
    const int cpr = a.head_dim / 8;                       // 16-byte chunks per row
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t total = (int64_t)a.total_q * a.Hkv * cpr;
    if (idx >= total) return;
    const int chunk = (int)(idx % cpr);
    const int g = (int)((idx / cpr) % a.Hkv);
    const int token = (int)(idx / ((int64_t)cpr * a.Hkv));
    int req = token, pos;
    if (a.cu_seqlens_q) {
        int lo = 0, hi = a.batch - 1;
        while (lo < hi) {                                 // last request with cu_seqlens_q[r] <= token
            const int mid = (lo + hi + 1) >> 1;
            if (a.cu_seqlens_q[mid] <= token) lo = mid; else hi = mid - 1;
        }
        req = lo;
        const int q0 = a.cu_seqlens_q[req], q1 = a.cu_seqlens_q[req + 1];
        pos = a.context_lens[req] - (q1 - q0) + (token - q0);
    } else {
        pos = a.context_lens[req] - 1;
    }
    if (pos < 0) return;                                  // malformed lengths: write nothing
    const int64_t blk = a.block_tables[(int64_t)req * a.max_blocks_per_seq + (pos >> a.block_size_log2)];
    const int bmask = (1 << a.block_size_log2) - 1;
    const int64_t dst = (((blk * a.Hkv + g) << a.block_size_log2) + (pos & bmask)) * (int64_t)a.head_dim + chunk * 8;
    const int64_t src = (int64_t)token * a.new_stride_token + (int64_t)g * a.new_stride_head + chunk * 8;
    *reinterpret_cast<u32x4 *>(a.k_cache + dst) = *reinterpret_cast<const u32x4 *>(a.k_new + src);
    *reinterpret_cast<u32x4 *>(a.v_cache + dst) = *reinterpret_cast<const u32x4 *>(a.v_new + src);
}

// System-cache fill: same 16-byte moves, destination addressed by (position, kv head) strides.
__global__ __launch_bounds__(kThreads) void system_fill_kernel(const SysFillArgs a) {
    const int cpr = a.head_dim / 8;
    const int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t total = (int64_t)a.num_pos * a.Hkv * cpr;
    if (idx >= total) return;
    const int chunk = (int)(idx % cpr);
    const int g = (int)((idx / cpr) % a.Hkv);
    const int t = (int)(idx / ((int64_t)cpr * a.Hkv));
    const int64_t src = (int64_t)t * a.new_stride_token + (int64_t)g * a.new_stride_head + chunk * 8;
    const int64_t dst = (int64_t)(a.first_pos + t) * a.sys_stride_token +
                        (int64_t)g * a.sys_stride_head + chunk * 8;
    *reinterpret_cast<u32x4 *>(a.k_sys + dst) = *reinterpret_cast<const u32x4 *>(a.k_new + src);
    *reinterpret_cast<u32x4 *>(a.v_sys + dst) = *reinterpret_cast<const u32x4 *>(a.v_new + src);
}

hipError_t launch_system_fill(const SysFillArgs &a, hipStream_t stream) {
    const int64_t total = (int64_t)a.num_pos * a.Hkv * (a.head_dim / 8);
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(system_fill_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_cache_append(const AppendArgs &a, hipStream_t stream) {
    const int64_t total = (int64_t)a.total_q * a.Hkv * (a.head_dim / 8);
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(cache_append_kernel, dim3((unsigned)((total + kThreads - 1) / kThreads)),
                       dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_fuse(const FuseArgs &a, int head_dim, hipStream_t stream) {
    if (a.rows == 0) return hipSuccess;
    if (head_dim == 128) {
        const int rpb = kThreads / 32;
        const dim3 grid((a.rows + rpb - 1) / rpb);
        if (a.n_prefixes > 1)
            hipLaunchKernelGGL((fuse_kernel<128, true>), grid, dim3(kThreads), 0, stream, a);
        else
            hipLaunchKernelGGL((fuse_kernel<128, false>), grid, dim3(kThreads), 0, stream, a);
    } else if (head_dim == 64) {
        const int rpb = kThreads / 16;
        const dim3 grid((a.rows + rpb - 1) / rpb);
        if (a.n_prefixes > 1)
            hipLaunchKernelGGL((fuse_kernel<64, true>), grid, dim3(kThreads), 0, stream, a);
        else
            hipLaunchKernelGGL((fuse_kernel<64, false>), grid, dim3(kThreads), 0, stream, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace ra
