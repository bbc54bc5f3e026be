// One launch for both partial attentions of a decode step (Alg. 1 "system attention" and
// "context attention"; the paper notes they have no dependency on each other).
//
// The grid is a list of work items, system items first:
//   system item  (kv head, tile of 32 stacked query rows, chunk of system positions): the
//                queries of the whole batch that share a kv head form the columns of one
//                matrix product, so the shared system K/V are streamed once per batch
//                (Sec. 3.3; Eq. 7, first term);
//   context item (request, kv head, part of that request's context): the G query heads of the
//                kv head against the request's own paged K/V (Eq. 7, second term).
// Both kinds run the same tile pipeline; a context item simply has G live query columns out of
// 32 and gathers its rows through the block table.  The hardware dispatcher hands the next
// item to whichever compute unit frees a slot, which balances the long system items against
// the short context items without any queue in memory.
//
// Tile pipeline of one wavefront (the four wavefronts of a workgroup take the item's 32-key
// tiles round-robin and merge at the end, so there is no barrier inside the key loop):
//   * K and V rows of the tile go from global memory straight into the wavefront's LDS slice
//     with 16-byte LDS-DMA loads (global_load_lds_dwordx4): no staging registers.  The LDS
//     position of every 16-byte chunk is XOR-swizzled with its row number on the global
//     address side, which makes the MFMA operand reads below bank-conflict free;
//   * S^T = K Q^T (keys x queries) with v_mfma_f32_32x32x16_bf16: a lane owns one query
//     column, so the softmax statistics are in-lane plus one exchange with lane^32;
//   * O^T += V^T P^T: V^T operands come from the row-major V tile through the LDS transpose
//     read ds_read_b64_tr_b16; P^T is taken from the S^T accumulator registers (split into a
//     high and a low bf16 part so that no 2^-9 rounding of the weights reaches the output).
// Reduction order depends only on the logical position of a key, never on the physical block,
// so any block placement of the same cache gives bit-identical results.  Rows past the end of
// an item are never loaded (their lanes re-load the last valid row and the scores are masked).
#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
#define RA_LDS __attribute__((address_space(3)))

constexpr int kWaves = kThreads / kWave;

template <int D>
struct TileCfg {
    static constexpr int ROW_BYTES = D * 2;
    static constexpr int CPR = D / 8;                 // 16-byte chunks per row
    static constexpr int SEGS = D / 32;               // 64-byte segments per row
    static constexpr int RPI = 1024 / ROW_BYTES;      // rows per LDS-DMA instruction
    static constexpr int NI = 32 / RPI;               // instructions per 32-row tile
    static constexpr int K_BYTES = 32 * ROW_BYTES;
    static constexpr int WAVE_BYTES = 2 * K_BYTES;    // K tile + V tile; also 32 x D fp32 / 2...
    static constexpr int O_BYTES = 32 * D * 4;        // merge buffer of one wavefront
    static constexpr int SLICE = WAVE_BYTES > O_BYTES ? WAVE_BYTES : O_BYTES;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Offset (in elements) of one K/V row: a system position, or a context position looked up in
// the request's block table.
template <int D>
__device__ __forceinline__ int64_t kv_row_offset(const TileArgs &a, bool is_sys, int key, int g,
                                                 const int32_t *bt, int bsl, int bmask) {
    if (is_sys) return (int64_t)key * a.sys_stride_token + (int64_t)g * a.sys_stride_head;
    const int64_t blk = bt[key >> bsl];
    return (((blk * a.Hkv + g) << bsl) + (key & bmask)) * (int64_t)D;
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void relay_tile_kernel(const TileArgs a) {
    using T = TileCfg<D>;
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;

    __shared__ __attribute__((aligned(1024))) unsigned char smem[kWaves * T::SLICE];
    __shared__ float sm_m[kWaves][32];
    __shared__ float sm_l[kWaves][32];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int col = lane & 31;
    const int hf = lane >> 5;

    // ---- decode the work item -----------------------------------------------------------
    const int item = blockIdx.x;
    const bool is_sys = item < a.n_sys_items;
    int g, key_begin, key_end, part_index, req = 0, mt = 0;
    if (is_sys) {
        const int chunk = item % a.n_sys_chunks;
        mt = (item / a.n_sys_chunks) % a.n_mtiles;
        g = item / (a.n_sys_chunks * a.n_mtiles);
        key_begin = chunk * a.sys_chunk;
        key_end = min(a.sys_len, key_begin + a.sys_chunk);
        part_index = chunk;
    } else {
        const int j = item - a.n_sys_items;
        const int part = j % a.n_ctx_parts;
        g = (j / a.n_ctx_parts) % a.Hkv;
        req = j / (a.n_ctx_parts * a.Hkv);
        key_begin = part * a.ctx_part;
        key_end = min(a.context_lens[req], key_begin + a.ctx_part);
        part_index = a.n_sys_chunks + part;
    }
    const int M = a.n_tokens * a.G;
    const int ncols = is_sys ? min(32, M - mt * 32) : a.G;     // live query columns

    // query column -> (token, head)
    auto column_row = [&](int c, int &token, int &hq) {
        if (is_sys) {
            const int n = mt * 32 + c;
            token = n / a.G;
            hq = g * a.G + n % a.G;
        } else {
            token = req;
            hq = g * a.G + c;
        }
    };

    unsigned char *my = smem + wave * T::SLICE;
    RA_LDS unsigned char *my_lds = (RA_LDS unsigned char *)my;
    const int bsl = a.block_size_log2;
    const int bmask = (1 << bsl) - 1;
    const int32_t *bt = a.block_tables + (int64_t)req * a.max_blocks_per_seq;

    // LDS-DMA lane geometry: instruction i deposits rows i*RPI .. i*RPI+RPI-1 of the tile;
    // this lane fills chunk position `lpos` of row i*RPI + lrow.
    const int lrow = lane / T::CPR;
    const int lpos = lane % T::CPR;

    // Row offsets (in elements) of this lane's NI rows of a tile; the block-table reads of a
    // context item are issued here, ahead of the DMA, so that they never sit between two DMAs.
    const uint16_t *kbase = is_sys ? a.k_sys : a.k_cache;
    const uint16_t *vbase = is_sys ? a.v_sys : a.v_cache;
    int64_t off[T::NI];

    f32x16 acc_o[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // V^T operand geometry for ds_read_b64_tr_b16: inside each block of 16 lanes, lane r
    // addresses 4 consecutive head_dim elements of row K0 + r/4 starting at D0 + 4*(r%4);
    // lane i of the block receives rows K0..K0+3 of column D0 + i.
    const int blk16 = lane >> 4;                  // 0..3: (blk16 & 1) picks the column half,
    const int r16 = lane & 15;                    //        (blk16 >> 1) == hf picks the key half
    const int tr_row = r16 >> 2;                  // + K0
    const int tr_colbyte = 32 * (blk16 & 1) + 8 * (r16 & 3);

    if (key_begin + wave * 32 < key_end) {
#pragma unroll
        for (int i = 0; i < T::NI; ++i)     // never past the item's end: clamp to its last row
            off[i] = kv_row_offset<D>(a, is_sys, min(key_begin + wave * 32 + i * T::RPI + lrow, key_end - 1),
                                      g, bt, bsl, bmask);
    }

    // B operand of S^T = K Q^T: lane (col, hf) holds Q[column col][t*16 + hf*8 .. +7]
    bf16x8 qf[KSTEPS];
    {
        const bool ok = col < ncols;
        int token = 0, hq = 0;
        if (ok) column_row(col, token, hq);
        const uint16_t *qp =
            a.q + (int64_t)token * a.q_stride_token + (int64_t)hq * a.q_stride_head + hf * 8;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            u32x4 w = u32x4{0, 0, 0, 0};
            if (ok) w = *reinterpret_cast<const u32x4 *>(qp + t * 16);
            qf[t] = __builtin_bit_cast(bf16x8, w);
        }
    }

    for (int tile0 = key_begin + wave * 32; tile0 < key_end; tile0 += kWaves * 32) {
#pragma unroll
        for (int i = 0; i < T::NI; ++i) {
            const int r = i * T::RPI + lrow;                       // row inside the tile
            // K: chunk c of row r sits at position c ^ (r mod CPR)
            const int kc = lpos ^ (r & (T::CPR - 1));
            // V: 64-byte segment s of row r sits at segment s ^ (r mod SEGS)
            const int vc = (((lpos >> 2) ^ (r & (T::SEGS - 1))) << 2) | (lpos & 3);
            // (pointers go through locals: with this compiler an element of a template-sized
            // array used directly in the builtin's argument drops the kernel's host stub)
            const uint16_t *kp = kbase + off[i] + kc * 8;
            const uint16_t *vp = vbase + off[i] + vc * 8;
            __builtin_amdgcn_global_load_lds(kp, (RA_LDS void *)(my_lds + i * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds(vp, (RA_LDS void *)(my_lds + T::K_BYTES + i * 1024), 16, 0, 0);
        }
        if (tile0 + kWaves * 32 < key_end) {      // rows of the next tile (block-table reads)
#pragma unroll
            for (int i = 0; i < T::NI; ++i)
                off[i] = kv_row_offset<D>(a, is_sys, min(tile0 + kWaves * 32 + i * T::RPI + lrow, key_end - 1),
                                          g, bt, bsl, bmask);
        }
        __builtin_amdgcn_s_waitcnt(0);            // vmcnt(0): the tile is in LDS
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // S^T tile: 32 keys x 32 queries
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            const int pos = (2 * t + hf) ^ (col & (T::CPR - 1));
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(my + col * T::ROW_BYTES + pos * 16);
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
        const float m_new = fmaxf(m_run, mx);     // finite: every processed tile has a valid key
        const float corr = fast_exp2(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
        uint32_t pw[8], pw_lo[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(s[r] - m_new), p1 = fast_exp2(s[r + 1] - m_new);
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

        // O^T += V^T P^T.  MFMA step `kstep` contracts keys 16*kstep .. 16*kstep+15; lane half hf
        // supplies slots e = 0..7 standing for keys 16*kstep + 8*(e/4) + 4*hf + e%4, which is the
        // order the S^T accumulator registers 8*kstep .. 8*kstep+7 already hold.
#pragma unroll
        for (int kstep = 0; kstep < 2; ++kstep) {
            const u32x4 pb = u32x4{pw[4 * kstep], pw[4 * kstep + 1], pw[4 * kstep + 2], pw[4 * kstep + 3]};
            const u32x4 pl = u32x4{pw_lo[4 * kstep], pw_lo[4 * kstep + 1], pw_lo[4 * kstep + 2],
                                   pw_lo[4 * kstep + 3]};
            const bf16x8 pf = __builtin_bit_cast(bf16x8, pb);
            const bf16x8 pf_lo = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                s16x4 v4[2];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int row = 16 * kstep + 8 * half + 4 * hf + tr_row;
                    const int seg = db ^ (row & (T::SEGS - 1));
                    v4[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (RA_LDS s16x4 *)(my_lds + T::K_BYTES + row * T::ROW_BYTES + seg * 64 + tr_colbyte));
                }
                const s16x8 v8 = __builtin_shufflevector(v4[0], v4[1], 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, v8);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, acc_o[db], 0, 0, 0);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo, acc_o[db], 0, 0, 0);
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }

    // ---- merge the four wavefronts and write the item's partial -------------------------
    l_run += __shfl_xor(l_run, 32);
    if (hf == 0) {
        sm_m[wave][col] = m_run;
        sm_l[wave][col] = l_run;
    }
    __syncthreads();   // also: every wavefront is done with its K/V slice
    float M_all = sm_m[0][col];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M_all = fmaxf(M_all, sm_m[w][col]);
    const float f_mine = fast_exp2(m_run - finite_or_zero(M_all));
    float *osh = reinterpret_cast<float *>(my);
    constexpr int OCH = D / 4;                    // 16-byte chunks per fp32 output row
    if (col < ncols) {
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                // registers 4*r4 .. 4*r4+3 are head_dim elements db*32 + 8*r4 + 4*hf + 0..3
                f32x4 v = {acc_o[db][4 * r4] * f_mine, acc_o[db][4 * r4 + 1] * f_mine,
                           acc_o[db][4 * r4 + 2] * f_mine, acc_o[db][4 * r4 + 3] * f_mine};
                const int chunk = (db * 8 + 2 * r4 + hf) ^ (col & (OCH - 1));
                *reinterpret_cast<f32x4 *>(osh + col * D + chunk * 4) = v;
            }
    }
    __syncthreads();

    constexpr int SEG = D / 8;                    // fp32 elements per thread: 8 threads per row
    const int row = threadIdx.x / 8, seg = threadIdx.x % 8;
    if (row < ncols) {
        float Mr = sm_m[0][row];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) Mr = fmaxf(Mr, sm_m[w][row]);
        const float m_use = finite_or_zero(Mr);
        float L = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) L = fmaf(sm_l[w][row], fast_exp2(sm_m[w][row] - m_use), L);
        const float inv = L > 0.f ? 1.f / L : 0.f;
        int token, hq;
        column_row(row, token, hq);
        const int64_t prow = (int64_t)part_index * a.rows + (int64_t)token * a.Hq + hq;
        float *dst = a.part_o + prow * D + seg * SEG;
#pragma unroll
        for (int e = 0; e < SEG; e += 4) {
            f32x4 sum = {0.f, 0.f, 0.f, 0.f};
            const int chunk = ((seg * SEG + e) / 4) ^ (row & (OCH - 1));
#pragma unroll
            for (int w = 0; w < kWaves; ++w) {
                const float *src = reinterpret_cast<const float *>(smem + w * T::SLICE);
                sum += *reinterpret_cast<const f32x4 *>(src + row * D + chunk * 4);
            }
            *reinterpret_cast<f32x4 *>(dst + e) = sum * inv;
        }
        if (seg == 0) a.part_lse[prow] = L > 0.f ? Mr + log2f(L) : -INFINITY;
    }
}

hipError_t launch_relay_tiles(const TileArgs &a, int head_dim, hipStream_t stream) {
    const int64_t items = (int64_t)a.n_sys_items + (int64_t)a.n_tokens * a.Hkv * a.n_ctx_parts;
    if (items == 0) return hipSuccess;
    if (items > INT32_MAX) return hipErrorInvalidValue;
    if (head_dim == 128)
        hipLaunchKernelGGL((relay_tile_kernel<128>), dim3((unsigned)items), dim3(kThreads), 0, stream, a);
    else if (head_dim == 64)
        hipLaunchKernelGGL((relay_tile_kernel<64>), dim3((unsigned)items), dim3(kThreads), 0, stream, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace ra
