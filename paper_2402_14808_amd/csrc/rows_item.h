// The work item of the many-rows kernel as a device function, so that the prompt-phase launch
// (relay_rows.hip) and the decode launch for wide grouped-query batches (relay_tiles.hip, where
// system items of this kind share the launch with the context wavefronts) run the same code.
#pragma once
#include "ra_device.h"
#include "ra_kernels.h"

namespace ra {

typedef __attribute__((ext_vector_type(4))) short rows_s16x4;
typedef __attribute__((ext_vector_type(8))) short rows_s16x8;
#define RA_ROWS_LDS __attribute__((address_space(3)))

constexpr int kRowWaves = kThreads / kWave;
constexpr int kRowBlock = 32 * kRowWaves;        // stacked query rows per workgroup

__device__ __forceinline__ float rows_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ uint32_t rows_pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// One work item of the many-rows kernel.  `block` is the item's index in the launch (system
// items first), `lds` points to 4 * 32 * D * 2 bytes of LDS aligned to 1024 (two K and two V
// tiles) and `sm_tbl` to kMaxPartBlocks block-table entries.  SYS_ONLY: the caller guarantees
// block < a.n_sys_items (decode batches), so the context code is left out.
template <int D, bool SYS_ONLY>
__device__ __forceinline__ void rows_item(const RowsArgs &a, const int block, unsigned char *lds,
                                          int32_t *sm_tbl) {
    constexpr int ROW_BYTES = D * 2;
    constexpr int CPR = D / 8;                    // 16-byte chunks per row
    constexpr int SEGS = D / 32;                  // 64-byte segments per row
    constexpr int TILE_BYTES = 32 * ROW_BYTES;
    constexpr int RPL = kThreads / CPR;           // rows covered by one load of the workgroup
    constexpr int NL = 32 / RPL;                  // loads per thread per tile (K or V)
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;

    unsigned char *const sm_k[2] = {lds, lds + TILE_BYTES};
    unsigned char *const sm_v[2] = {lds + 2 * TILE_BYTES, lds + 3 * TILE_BYTES};

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col = lane & 31;
    const int hf = lane >> 5;
    const int bsl = a.block_size_log2;
    const int bmask = (1 << bsl) - 1;

    // ---- decode the work item -----------------------------------------------------------
    const bool is_sys = SYS_ONLY || block < a.n_sys_items;
    int g, rb, key_begin, key_end, part_index, req = 0, first_blk = 0;
    int n_rows;            // stacked rows of this item's row space (system: all tokens; context: m*G)
    int token_base = 0;    // first packed token of the row space
    int ctx_len = 0, q_len = 0;
    if (is_sys) {
        const int item = block;
        int chunk;
        if (a.sys_head_fastest) {
            g = item % a.Hkv;
            rb = (item / a.Hkv) % a.n_sys_rowblocks;
            chunk = item / (a.Hkv * a.n_sys_rowblocks);
        } else {
            chunk = item % a.n_sys_chunks;
            rb = (item / a.n_sys_chunks) % a.n_sys_rowblocks;
            g = item / (a.n_sys_chunks * a.n_sys_rowblocks);
        }
        key_begin = chunk * a.sys_chunk;
        key_end = min(a.sys_len, key_begin + a.sys_chunk);
        part_index = chunk;
        n_rows = a.n_tokens * a.G;
    } else {
        int j = block - a.n_sys_items;
        const int part = j % a.n_ctx_parts;  j /= a.n_ctx_parts;
        rb = j % a.n_ctx_rowblocks;          j /= a.n_ctx_rowblocks;
        g = j % a.Hkv;
        req = j / a.Hkv;
        const int q0 = a.cu_seqlens_q[req];
        q_len = a.cu_seqlens_q[req + 1] - q0;
        token_base = q0;
        n_rows = q_len * a.G;
        if (rb * kRowBlock >= n_rows) return;     // (uniform for the workgroup: before any barrier)
        ctx_len = a.context_lens[req];
        key_begin = part * a.ctx_part;
        // the last row of this block sees the most: positions <= ctx_len - q_len + its token index
        const int last_row = min(n_rows, (rb + 1) * kRowBlock) - 1;
        const int max_limit = ctx_len - q_len + last_row / a.G;
        key_end = min(min(ctx_len, max_limit + 1), key_begin + a.ctx_part);
        part_index = a.n_sys_chunks + part;
        first_blk = key_begin >> bsl;
        const int nblk = ((key_begin + a.ctx_part - 1) >> bsl) - first_blk + 1;
        const int32_t *bt = a.block_tables + (int64_t)req * a.max_blocks_per_seq;
        for (int i = threadIdx.x; i < nblk; i += kThreads)
            sm_tbl[i] = bt[min(first_blk + i, a.max_blocks_per_seq - 1)];
        __syncthreads();
    }

    // this lane's query column: stacked row n -> (token, head)
    const int n = rb * kRowBlock + wave * 32 + col;
    const bool col_ok = n < n_rows;
    const int token = token_base + (col_ok ? n / a.G : 0);
    const int hq = g * a.G + (col_ok ? n % a.G : 0);
    // causal limit of this column (context items): last visible context position
    const int limit = is_sys ? INT32_MAX : ctx_len - q_len + (col_ok ? n / a.G : 0);

    // B operand of S^T = K Q^T: lane (col, hf) holds Q[column col][t*16 + hf*8 .. +7]
    u32x4 qw[KSTEPS];
    {
        const uint16_t *qp =
            a.q + (int64_t)token * a.q_stride_token + (int64_t)hq * a.q_stride_head + hf * 8;
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) {
            qw[t] = u32x4{0, 0, 0, 0};
            if (col_ok) qw[t] = *reinterpret_cast<const u32x4 *>(qp + t * 16);
        }
    }

    const uint16_t *ksrc = is_sys ? a.k_sys + (int64_t)g * a.sys_stride_head : a.k_cache;
    const uint16_t *vsrc = is_sys ? a.v_sys + (int64_t)g * a.sys_stride_head : a.v_cache;
    auto row_offset = [&](int key) -> int64_t {       // `key` already clamped to the item
        if (is_sys) return (int64_t)key * a.sys_stride_token;
        const int64_t blk = sm_tbl[(key >> bsl) - first_blk];
        return (((blk * a.Hkv + g) << bsl) + (key & bmask)) * (int64_t)D;
    };

    // cooperative tile load: load i of this thread covers row i*RPL + lrow, 16-byte chunk lpos
    const int lrow = threadIdx.x / CPR;
    const int lpos = threadIdx.x % CPR;
    // Two sets of landing registers: the loads of tile t+2 are issued while tile t is computed and
    // tile t+1 (already landed, or about to) waits for its turn to go to LDS.  The K/V of a
    // workgroup come from L2 or the last-level cache, two microseconds away under load; with only
    // one tile in flight per workgroup that latency, not the matrix unit, set the pace.
    struct Landing { u32x4 k[NL], v[NL]; };
    Landing la, lb;
    auto load_tile = [&](Landing &r, int tile0) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int key = min(tile0 + i * RPL + lrow, key_end - 1);   // never past the item's end
            const int64_t off = row_offset(key) + lpos * 8;
            r.k[i] = *reinterpret_cast<const u32x4 *>(ksrc + off);
            r.v[i] = *reinterpret_cast<const u32x4 *>(vsrc + off);
        }
    };
    // K: chunk c of row r at position c ^ (r mod CPR); V: 64-byte segment s of row r at s ^ (r mod SEGS)
    auto store_tile = [&](const Landing &r_, int buf) {
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            const int r = i * RPL + lrow;
            const int kpos = lpos ^ (r & (CPR - 1));
            const int vpos = (((lpos >> 2) ^ (r & (SEGS - 1))) << 2) | (lpos & 3);
            *reinterpret_cast<u32x4 *>(sm_k[buf] + r * ROW_BYTES + kpos * 16) = r_.k[i];
            *reinterpret_cast<u32x4 *>(sm_v[buf] + r * ROW_BYTES + vpos * 16) = r_.v[i];
        }
    };

    f32x16 acc_o[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // V^T operand geometry for ds_read_b64_tr_b16 (see relay_tiles.hip)
    const int blk16 = lane >> 4;
    const int r16 = lane & 15;
    const int tr_row = r16 >> 2;
    const int tr_colbyte = 32 * (blk16 & 1) + 8 * (r16 & 3);

    // keys this wavefront needs at all: up to the largest limit among its 32 columns
    int wave_limit = limit;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) wave_limit = max(wave_limit, __shfl_xor(wave_limit, off));
    int wave_min_limit = col_ok ? limit : INT32_MAX;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1)
        wave_min_limit = min(wave_min_limit, __shfl_xor(wave_min_limit, off));

    // (the query registers are made to arrive here, so that no wait for them sits inside the loop)
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) asm volatile("" : "+v"(qw[t]));
    if (key_begin < key_end) {
        load_tile(la, key_begin);
        store_tile(la, 0);
        if (key_begin + 32 < key_end) load_tile(la, key_begin + 32);
    }
    __syncthreads();

    // One step: tile `tile0` is in LDS buffer `buf`, tile0+32 is in (or on its way to) `held`,
    // and the loads of tile0+64 go to `fresh`.
    auto step = [&](int tile0, int buf, Landing &held, Landing &fresh) {
        const bool has_next = tile0 + 32 < key_end;

        if (tile0 <= wave_limit) {                // else: every key of the tile is masked for this wave
            const unsigned char *kt = sm_k[buf];
            RA_ROWS_LDS unsigned char *vt = (RA_ROWS_LDS unsigned char *)sm_v[buf];
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
            // all K operands of the tile are read before the first product, so that the LDS
            // latency is paid once and not once per product
            bf16x8 kf[KSTEPS];
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t) {
                const int pos = (2 * t + hf) ^ (col & (CPR - 1));
                kf[t] = *reinterpret_cast<const bf16x8 *>(kt + col * ROW_BYTES + pos * 16);
            }
#pragma unroll
            for (int t = 0; t < KSTEPS; ++t)
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t], __builtin_bit_cast(bf16x8, qw[t]), s, 0, 0, 0);
            // The loads of the tile after next start here, behind the products: issued any earlier
            // in the iteration they would be waited for at the products above (the compiler's
            // wait bookkeeping is per loop iteration, not per register).
            if (tile0 + 64 < key_end) load_tile(fresh, tile0 + 64);
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] *= a.scale_log2;
            // accumulator register r of lane (col, hf) is key 8*(r/4) + 4*hf + r%4 of the tile
            if (tile0 + 32 > key_end || tile0 + 31 > wave_min_limit) {   // ragged end or causal edge
                const int lim = min(limit, key_end - 1);
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int key = tile0 + 8 * (r / 4) + 4 * hf + (r % 4);
                    s[r] = key <= lim ? s[r] : -INFINITY;
                }
            }
            float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
#pragma unroll
            for (int r = 4; r < 16; r += 4)
                mx = fmaxf(mx, fmaxf(fmaxf(s[r], s[r + 1]), fmaxf(s[r + 2], s[r + 3])));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float m_use = finite_or_zero(m_new);    // a column may have no visible key yet
            if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
                const float corr = rows_exp2(m_run - m_use);
                l_run *= corr;
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc_o[db][r] *= corr;
                m_run = m_new;
            }
            float psum = 0.f;
            uint32_t pw[8], pw_lo[8];
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                const float p0 = rows_exp2(s[r] - m_use), p1 = rows_exp2(s[r + 1] - m_use);
                psum += p0 + p1;
                const uint32_t h = rows_pack_bf16(p0, p1);
                pw[r / 2] = h;
                pw_lo[r / 2] = rows_pack_bf16(p0 - bf16_lo(h), p1 - bf16_hi(h));
            }
            l_run += psum;
#pragma unroll
            for (int kstep = 0; kstep < 2; ++kstep) {
                const u32x4 pb = u32x4{pw[4 * kstep], pw[4 * kstep + 1], pw[4 * kstep + 2], pw[4 * kstep + 3]};
                const u32x4 pl = u32x4{pw_lo[4 * kstep], pw_lo[4 * kstep + 1], pw_lo[4 * kstep + 2],
                                       pw_lo[4 * kstep + 3]};
                const bf16x8 pf = __builtin_bit_cast(bf16x8, pb);
                const bf16x8 pf_lo = __builtin_bit_cast(bf16x8, pl);
#pragma unroll
                for (int db = 0; db < DBLK; ++db) {
                    rows_s16x4 v4[2];
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const int row = 16 * kstep + 8 * half + 4 * hf + tr_row;
                        const int seg = db ^ (row & (SEGS - 1));
                        v4[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                            (RA_ROWS_LDS rows_s16x4 *)(vt + row * ROW_BYTES + seg * 64 + tr_colbyte));
                    }
                    const rows_s16x8 v8 = __builtin_shufflevector(v4[0], v4[1], 0, 1, 2, 3, 4, 5, 6, 7);
                    const bf16x8 vf = __builtin_bit_cast(bf16x8, v8);
                    acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, acc_o[db], 0, 0, 0);
                    acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo, acc_o[db], 0, 0, 0);
                }
            }
        } else if (tile0 + 64 < key_end) {
            load_tile(fresh, tile0 + 64);         // (a wavefront that skips the tile still loads its share)
        }
        if (has_next) store_tile(held, buf ^ 1);
        __syncthreads();   // next tile visible to all; everyone is done reading this one
    };
    for (int tile0 = key_begin; tile0 < key_end; tile0 += 64) {
        step(tile0, 0, la, lb);
        if (tile0 + 32 < key_end) step(tile0 + 32, 1, lb, la);
    }

    // ---- each wavefront writes the partial of its 32 rows from registers ----------------------
    l_run += __shfl_xor(l_run, 32);
    if (col_ok) {
        const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
        const int64_t prow = (int64_t)part_index * a.rows + (int64_t)token * a.Hq + hq;
        float *dst = a.part_o + prow * D;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                // registers 4*r4 .. 4*r4+3 are head_dim elements db*32 + 8*r4 + 4*hf + 0..3
                const f32x4 v = {acc_o[db][4 * r4] * inv, acc_o[db][4 * r4 + 1] * inv,
                                 acc_o[db][4 * r4 + 2] * inv, acc_o[db][4 * r4 + 3] * inv};
                *reinterpret_cast<f32x4 *>(dst + db * 32 + 8 * r4 + 4 * hf) = v;
            }
        if (hf == 0) a.part_lse[prow] = l_run > 0.f ? m_run + log2f(l_run) : -INFINITY;
    }
}

}  // namespace ra
