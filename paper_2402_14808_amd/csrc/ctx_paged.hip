// Context attention of one decode step (Alg. 1 "context attention"; Eq. 7, second term):
// each query attends to its own request's cached keys/values, gathered through the block
// table.  One query row per (request, head) makes this a pair of matrix-vector products per
// request (Sec. 3.2, first observation), so the kernel is built for memory bandwidth:
// every lane issues 16-byte loads, 16 (head_dim 128) or 8 (head_dim 64) adjacent lanes cover
// one token row, a wavefront keeps 2*U such loads in flight, and the G query heads that share
// a KV head reuse each loaded row.  Reductions over a token row use DPP, not LDS.
//
// The order in which positions are accumulated depends only on their logical index in the
// request, never on the physical block number, so any placement of the same logical cache
// gives bit-identical results.  Positions >= context_lens[i] and block-table slots beyond the
// last used block are never loaded.
#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

template <int D, int G, int U>
__global__ __launch_bounds__(kThreads) void ctx_decode_kernel(const CtxArgs a) {
    constexpr int LPT = D / 8;        // lanes per token row (each holds 8 bf16 = 16 bytes)
    constexpr int TPI = kWave / LPT;  // token rows per load instruction of a wavefront
    constexpr int WAVES = kThreads / kWave;

    __shared__ float sm_o[WAVES][G][D];
    __shared__ float sm_m[WAVES][G];
    __shared__ float sm_l[WAVES][G];

    const int item = blockIdx.x;
    const int part = item % a.n_parts;
    const int bg = item / a.n_parts;
    const int g = bg % a.Hkv;
    const int token = bg / a.Hkv;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int sub = lane % LPT;
    const int grp = lane / LPT;

    // decode: token i is request i and sees its whole context.  Prompt phase: the m new tokens
    // of a request are the last m positions of its context; new token j sees c - m + j + 1.
    int b = token;
    int c;
    if (a.cu_seqlens_q) {
        int lo = 0, hi = a.batch - 1;
        while (lo < hi) {                       // last request with cu_seqlens_q[b] <= token
            const int mid = (lo + hi + 1) >> 1;
            if (a.cu_seqlens_q[mid] <= token) lo = mid; else hi = mid - 1;
        }
        b = lo;
        const int q0 = a.cu_seqlens_q[b], q1 = a.cu_seqlens_q[b + 1];
        c = a.context_lens[b] - (q1 - q0) + (token - q0) + 1;
    } else {
        c = a.context_lens[b];
    }
    const int t0 = part * a.part_tokens;
    const int t1 = min(c, t0 + a.part_tokens);

    // the G query rows of this KV head, 8 elements per lane
    u32x4 qv[G];
#pragma unroll
    for (int h = 0; h < G; ++h)
        qv[h] = *reinterpret_cast<const u32x4 *>(
            a.q + (int64_t)token * a.q_stride_token + (int64_t)(g * G + h) * a.q_stride_head + sub * 8);

    float m[G], l[G], o[G][8];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[h][i] = 0.f;
    }

    const int bsl = a.block_size_log2;
    const int bmask = (1 << bsl) - 1;
    const int32_t *bt = a.block_tables + (int64_t)b * a.max_blocks_per_seq;

    for (int base = t0 + wave * (U * TPI); base < t1; base += WAVES * U * TPI) {
        u32x4 kk[U], vv[U];
        bool valid[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int tok = base + u * TPI + grp;
            valid[u] = tok < t1;
            kk[u] = u32x4{0, 0, 0, 0};
            vv[u] = u32x4{0, 0, 0, 0};
            if (valid[u]) {
                const int64_t blk = bt[tok >> bsl];
                const int64_t off =
                    (((blk * a.Hkv + g) << bsl) + (tok & bmask)) * (int64_t)D + sub * 8;
                kk[u] = *reinterpret_cast<const u32x4 *>(a.k_cache + off);
                vv[u] = *reinterpret_cast<const u32x4 *>(a.v_cache + off);
            }
        }
#pragma unroll
        for (int h = 0; h < G; ++h) {
            float s[U];
            float mx = -INFINITY;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float dot = group_sum<LPT>(dot8_bf16(qv[h], kk[u], 0.f));
                s[u] = valid[u] ? dot * a.scale_log2 : -INFINITY;
                mx = fmaxf(mx, s[u]);
            }
            const float m_new = fmaxf(m[h], mx);
            const float m_use = finite_or_zero(m_new);
            const float corr = exp2f(m[h] - m_use);
            m[h] = m_new;
            float lsum = l[h] * corr;
#pragma unroll
            for (int i = 0; i < 8; ++i) o[h][i] *= corr;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const float p = exp2f(s[u] - m_use);
                lsum += p;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    o[h][2 * i] = fmaf(p, bf16_lo(vv[u][i]), o[h][2 * i]);
                    o[h][2 * i + 1] = fmaf(p, bf16_hi(vv[u][i]), o[h][2 * i + 1]);
                }
            }
            l[h] = lsum;
        }
    }

    // fold the TPI token-row groups of this wavefront together (same `sub`, different `grp`)
#pragma unroll
    for (int h = 0; h < G; ++h) {
#pragma unroll
        for (int off = LPT; off < kWave; off <<= 1) {
            const float m2 = __shfl_xor(m[h], off);
            const float l2 = __shfl_xor(l[h], off);
            const float m_new = fmaxf(m[h], m2);
            const float m_use = finite_or_zero(m_new);
            const float f1 = exp2f(m[h] - m_use), f2 = exp2f(m2 - m_use);
            l[h] = l[h] * f1 + l2 * f2;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float o2 = __shfl_xor(o[h][i], off);
                o[h][i] = o[h][i] * f1 + o2 * f2;
            }
            m[h] = m_new;
        }
        if (grp == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sm_o[wave][h][sub * 8 + i] = o[h][i];
            if (sub == 0) {
                sm_m[wave][h] = m[h];
                sm_l[wave][h] = l[h];
            }
        }
    }
    __syncthreads();

    // fold the wavefronts together and write this item's partial
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int h = idx / D, e = idx % D;
        float M = sm_m[0][h];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) M = fmaxf(M, sm_m[w][h]);
        const float m_use = finite_or_zero(M);
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) {
            const float f = exp2f(sm_m[w][h] - m_use);
            L = fmaf(sm_l[w][h], f, L);
            O = fmaf(sm_o[w][h][e], f, O);
        }
        const float val = L > 0.f ? O / L : 0.f;
        const float lse2 = L > 0.f ? M + log2f(L) : -INFINITY;
        const int hq = g * G + h;
        if (a.direct) {
            const int64_t oo = (int64_t)token * a.o_stride_token + (int64_t)hq * a.o_stride_head + e;
            if (a.out_is_fp32)
                static_cast<float *>(a.out)[oo] = val;
            else
                static_cast<uint16_t *>(a.out)[oo] = (uint16_t)f32_to_bf16_bits(val);
            if (e == 0 && a.lse_out) a.lse_out[(int64_t)token * a.Hq + hq] = lse2 * kLn2;
        } else {
            const int64_t row = (int64_t)part * a.rows + (int64_t)token * a.Hq + hq;
            a.part_o[row * D + e] = val;
            if (e == 0) a.part_lse[row] = lse2;
        }
    }
}

template <int D, int G>
static hipError_t launch_ctx_dg(const CtxArgs &a, hipStream_t stream) {
    constexpr int U = (G <= 2) ? 8 : 4;
    const int items = a.n_tokens * a.Hkv * a.n_parts;
    if (items == 0) return hipSuccess;
    hipLaunchKernelGGL((ctx_decode_kernel<D, G, U>), dim3(items), dim3(kThreads), 0, stream, a);
    return hipGetLastError();
}

template <int D>
static hipError_t launch_ctx_d(const CtxArgs &a, int group, hipStream_t stream) {
    switch (group) {
        case 1: return launch_ctx_dg<D, 1>(a, stream);
        case 2: return launch_ctx_dg<D, 2>(a, stream);
        case 3: return launch_ctx_dg<D, 3>(a, stream);
        case 4: return launch_ctx_dg<D, 4>(a, stream);
        case 5: return launch_ctx_dg<D, 5>(a, stream);
        case 6: return launch_ctx_dg<D, 6>(a, stream);
        case 7: return launch_ctx_dg<D, 7>(a, stream);
        case 8: return launch_ctx_dg<D, 8>(a, stream);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_ctx_decode(const CtxArgs &a, int head_dim, int group, hipStream_t stream) {
    if (head_dim == 128) return launch_ctx_d<128>(a, group, stream);
    if (head_dim == 64) return launch_ctx_d<64>(a, group, stream);
    return hipErrorInvalidValue;
}

}  // namespace ra
