// System attention (Alg. 1 "system attention"; Eq. 7, first term): the queries of the whole
// batch that share a KV head are stacked into one row tile, so the shared system keys/values
// are streamed from memory once per batch instead of once per request (Sec. 3.3: the
// matrix-vector products are grouped into matrix-matrix products).
//
// Work item = (kv head, tile of 32 stacked query rows, chunk of system positions).  The four
// wavefronts of a workgroup split the chunk's keys in tiles of 32; each keeps its own running
// softmax state and the four are merged at the end, so there is no barrier inside the key
// loop.  Per 32-key tile a wavefront
//   * loads K and V rows with coalesced 16-byte loads (next tile prefetched into registers),
//   * stages them in its private LDS slice: K row-major (padded), V transposed so that eight
//     consecutive keys of one head_dim column are contiguous,
//   * S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (keys x queries): a lane owns one query
//     column, so the softmax row statistics are in-lane plus one exchange with lane^32,
//   * O^T += V^T P^T with P^T taken straight from the accumulator registers of S^T; the key
//     order inside each 16-key MFMA step is permuted (bits 2 and 3 of the key index swapped)
//     so that the accumulator layout of S^T is already the B-operand layout.
// The partial (normalised output, base-2 log-sum-exp) goes to the workspace; relay fusion
// combines the chunks with the context part.
#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

template <int D>
struct SysTile {
    static constexpr int KROW = D + 8;         // bf16 elements per padded K row in LDS
    static constexpr int VROW = 32 + 8;        // bf16 elements per padded V^T row (32 key slots)
    static constexpr int K_BYTES = 32 * KROW * 2;
    static constexpr int V_BYTES = D * VROW * 2;
    static constexpr int OROW = D + 4;         // fp32 elements per padded output row
    static constexpr int O_BYTES = 32 * OROW * 4;
    static constexpr int WAVE_BYTES =
        (K_BYTES + V_BYTES) > O_BYTES ? (K_BYTES + V_BYTES) : O_BYTES;
};

// slot of key k (0..31) inside a V^T row: bits 2 and 3 swapped
__device__ __forceinline__ int v_slot(int k) {
    return (k & 0x13) | ((k & 4) << 1) | ((k & 8) >> 1);
}

template <int D>
__global__ __launch_bounds__(kThreads) void sys_partial_kernel(const SysArgs a) {
    using T = SysTile<D>;
    constexpr int LPT = D / 8;          // lanes per key row in a global load
    constexpr int KPI = kWave / LPT;    // key rows per load instruction
    constexpr int NI = 32 / KPI;        // load instructions per 32-key tile (K or V)
    constexpr int KSTEPS = D / 16;      // MFMA steps over head_dim for S^T
    constexpr int DBLK = D / 32;        // 32-row blocks of O^T
    constexpr int WAVES = kThreads / kWave;

    __shared__ __attribute__((aligned(16))) unsigned char smem[WAVES * T::WAVE_BYTES];
    __shared__ float sm_m[WAVES][32];
    __shared__ float sm_l[WAVES][32];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col = lane & 31;          // query column owned in MFMA accumulators
    const int hf = lane >> 5;

    const int item = blockIdx.x;
    const int chunk = item % a.n_chunks;
    const int mt = (item / a.n_chunks) % a.n_mtiles;
    const int g = item / (a.n_chunks * a.n_mtiles);

    const int key_begin = chunk * a.chunk_tokens;
    const int key_end = min(a.sys_len, key_begin + a.chunk_tokens);
    const int M = a.n_tokens * a.G;     // stacked query rows of this kv head

    // B operand of S^T = K Q^T: lane (col, hf) holds Q[row col][t*16 + hf*8 .. +7]
    bf16x8 qf[KSTEPS];
    {
        const int n = mt * 32 + col;
        const bool ok = n < M;
        const int token = ok ? n / a.G : 0;
        const int hq = g * a.G + (ok ? n % a.G : 0);
        const uint16_t *qp =
            a.q + (int64_t)token * a.q_stride_token + (int64_t)hq * a.q_stride_head + hf * 8;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 w = u32x4{0, 0, 0, 0};
            if (ok) w = *reinterpret_cast<const u32x4 *>(qp + t * 16);
            qf[t] = __builtin_bit_cast(bf16x8, w);
        }
    }

    unsigned char *my = smem + wave * T::WAVE_BYTES;
    uint16_t *ks = reinterpret_cast<uint16_t *>(my);
    uint16_t *vt = reinterpret_cast<uint16_t *>(my + T::K_BYTES);

    const int lrow = lane / LPT;        // key row inside a load instruction
    const int lcol = (lane % LPT) * 8;  // first head_dim element of this lane's 16 bytes
    const uint16_t *kbase = a.k_sys + (int64_t)g * a.sys_stride_head + lcol;
    const uint16_t *vbase = a.v_sys + (int64_t)g * a.sys_stride_head + lcol;

    u32x4 kr[NI], vr[NI];
    auto load_tile = [&](int tile_key0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int key = tile_key0 + i * KPI + lrow;
            kr[i] = u32x4{0, 0, 0, 0};
            vr[i] = u32x4{0, 0, 0, 0};
            if (key < key_end) {
                kr[i] = *reinterpret_cast<const u32x4 *>(kbase + (int64_t)key * a.sys_stride_token);
                vr[i] = *reinterpret_cast<const u32x4 *>(vbase + (int64_t)key * a.sys_stride_token);
            }
        }
    };

    f32x16 acc_o[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    int tile0 = key_begin + wave * 32;
    if (tile0 < key_end) load_tile(tile0);
    for (; tile0 < key_end; tile0 += WAVES * 32) {
        // registers -> LDS (K row-major, V transposed into MFMA key-slot order)
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            const int k = i * KPI + lrow;
            *reinterpret_cast<u32x4 *>(ks + k * T::KROW + lcol) = kr[i];
            const int slot = v_slot(k);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                vt[(lcol + 2 * j) * T::VROW + slot] = (uint16_t)(vr[i][j] & 0xffffu);
                vt[(lcol + 2 * j + 1) * T::VROW + slot] = (uint16_t)(vr[i][j] >> 16);
            }
        }
        const int next = tile0 + WAVES * 32;
        if (next < key_end) load_tile(next);       // in flight while this tile is computed
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // S^T tile: 32 keys x 32 queries
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(ks + col * T::KROW + t * 16 + hf * 8);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[t], s, 0, 0, 0);
        }
        // accumulator register r of lane (col, hf) is key 8*(r/4) + 4*hf + r%4 of the tile
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = tile0 + 8 * (r / 4) + 4 * hf + (r % 4);
            s[r] = key < key_end ? s[r] * a.scale_log2 : -INFINITY;
            mx = fmaxf(mx, s[r]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);
        const float m_use = finite_or_zero(m_new);
        const float corr = exp2f(m_run - m_use);
        m_run = m_new;
        // P is fed to the MFMA as bf16; a single rounding would leave 2^-9 relative error per
        // weight, so it is split into a high and a low bf16 part (error ~2^-17) and O^T takes two
        // MFMA passes.  The row sum uses the unrounded fp32 weights.
        float psum = 0.f;
        uint32_t pw[8], pw_lo[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = exp2f(s[r] - m_use), p1 = exp2f(s[r + 1] - m_use);
            psum += p0 + p1;
            const uint32_t h0 = f32_to_bf16_bits(p0), h1 = f32_to_bf16_bits(p1);
            pw[r / 2] = h0 | (h1 << 16);
            pw_lo[r / 2] = pack_bf16x2(p0 - __uint_as_float(h0 << 16), p1 - __uint_as_float(h1 << 16));
        }
        l_run = l_run * corr + psum;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc_o[db][r] *= corr;

        // O^T += V^T P^T, two 16-key steps
#pragma unroll
        for (int kstep = 0; kstep < 2; ++kstep) {
            const u32x4 pb = u32x4{pw[4 * kstep], pw[4 * kstep + 1], pw[4 * kstep + 2], pw[4 * kstep + 3]};
            const u32x4 pl = u32x4{pw_lo[4 * kstep], pw_lo[4 * kstep + 1], pw_lo[4 * kstep + 2],
                                   pw_lo[4 * kstep + 3]};
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pb);
            const bf16x8 pf_lo = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                const bf16x8 vf = *reinterpret_cast<const bf16x8 *>(
                    vt + (db * 32 + col) * T::VROW + kstep * 16 + hf * 8);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, acc_o[db], 0, 0, 0);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo, acc_o[db], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }

    // ---- merge the four wavefronts ------------------------------------------------------
    l_run += __shfl_xor(l_run, 32);
    if (hf == 0) {
        sm_m[wave][col] = m_run;
        sm_l[wave][col] = l_run;
    }
    __syncthreads();   // also: every wavefront is done with its K/V slice
    float M_all = sm_m[0][col];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) M_all = fmaxf(M_all, sm_m[w][col]);
    const float f_mine = exp2f(m_run - finite_or_zero(M_all));
    float *osh = reinterpret_cast<float *>(my);
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
            // registers 4*r4 .. 4*r4+3 are head_dim elements db*32 + 8*r4 + 4*hf + 0..3
            f32x4 v = {acc_o[db][4 * r4] * f_mine, acc_o[db][4 * r4 + 1] * f_mine,
                       acc_o[db][4 * r4 + 2] * f_mine, acc_o[db][4 * r4 + 3] * f_mine};
            *reinterpret_cast<f32x4 *>(osh + col * T::OROW + db * 32 + 8 * r4 + 4 * hf) = v;
        }
    __syncthreads();

    constexpr int SEG = D / 8;                 // fp32 elements per thread: 8 threads per row
    const int row = threadIdx.x / 8, seg = threadIdx.x % 8;
    const int n = mt * 32 + row;
    if (n < M) {
        float Mr = sm_m[0][row];
#pragma unroll
        for (int w = 1; w < WAVES; ++w) Mr = fmaxf(Mr, sm_m[w][row]);
        const float m_use = finite_or_zero(Mr);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) L = fmaf(sm_l[w][row], exp2f(sm_m[w][row] - m_use), L);
        const float inv = L > 0.f ? 1.f / L : 0.f;
        const int token = n / a.G, hq = g * a.G + n % a.G;
        const int64_t prow = (int64_t)chunk * a.rows + (int64_t)token * a.Hq + hq;
        float *dst = a.part_o + prow * D + seg * SEG;
#pragma unroll
        for (int e = 0; e < SEG; e += 4) {
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < WAVES; ++w) {
                const float *src = reinterpret_cast<const float *>(smem + w * T::WAVE_BYTES);
                sum += *reinterpret_cast<const f32x4 *>(src + row * T::OROW + seg * SEG + e);
            }
            *reinterpret_cast<f32x4 *>(dst + e) = sum * inv;
        }
        if (seg == 0) a.part_lse[prow] = L > 0.f ? Mr + log2f(L) : -INFINITY;
    }
}

hipError_t launch_sys_partial(const SysArgs &a, int head_dim, hipStream_t stream) {
    const int items = a.Hkv * a.n_mtiles * a.n_chunks;
    if (items == 0) return hipSuccess;
    if (head_dim == 128)
        hipLaunchKernelGGL((sys_partial_kernel<128>), dim3(items), dim3(kThreads), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL((sys_partial_kernel<64>), dim3(items), dim3(kThreads), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ra
