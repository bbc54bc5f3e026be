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
// items first), `lds` points to 2 * 2 * 64 * D * 2 bytes of LDS aligned to 1024 (two buffers, each
// the K rows and the V rows of one 64-key step) and `sm_tbl` to kMaxPartBlocks block-table
// entries.  SYS_ONLY: the caller guarantees block < a.n_sys_items (decode batches), so the context
// code is left out.
//
// The key range is walked in steps of 64 keys (two 32-key tiles, "A" and "B", whose score
// products are independent chains for the matrix unit), one barrier per step.  Softmax
// bookkeeping per lane (a lane owns a query column):
//   m_run   running maximum of the raw (unscaled) scores the accumulators are expressed against;
//   msc     the same in the scaled base-2 domain (0 while the column has seen no key);
//   l_run   sum of the weights 2^(s*scale - msc);  acc_o the weighted sum of values.
// The reference maximum is only moved when some column's maximum has grown by more than
// kLazyLog2 in the exponent (weights stay below 2^kLazyLog2, far inside fp32 and bf16 range, and
// the result is the same number): most steps then skip the 64-register rescale of acc_o.
constexpr float kLazyLog2 = 8.0f;

// MULTI: several shared prefixes (App. D), each owning a run of the packed tokens.
// WHOLE: the item is a block of 128 stacked rows of the prompt phase with EVERYTHING its rows
// attend to: the whole system prompt first, then, for every request that has rows in the block,
// that request's context with the causal limit of each row (the rows of other requests masked).
// The accumulators never leave the registers, the output row is written by the item itself, and
// neither partials nor a fusion launch are needed (Alg. 1's relay fusion becomes the running
// rescale of one online softmax over [system ; context], which is the same number).  The host
// picks it when the system prompt is one chunk and the requests bring many new tokens each.
template <int D, bool SYS_ONLY, bool MULTI = false, bool WHOLE = false>
__device__ __forceinline__ void rows_item(const RowsArgs &a, const int block, unsigned char *lds,
                                          int32_t *sm_tbl) {
    constexpr int ROW_BYTES = D * 2;
    constexpr int CPR = D / 8;                    // 16-byte chunks per row
    constexpr int SEGS = D / 32;                  // 64-byte segments per row
    constexpr int STEP = 64;                      // keys per step
    constexpr int KV_BYTES = STEP * ROW_BYTES;    // the K rows (or the V rows) of one step
    constexpr int RPL = kThreads / CPR;           // rows covered by one load of the workgroup
    constexpr int NL = STEP / RPL;                // loads per thread per step (K or V)
    constexpr int KSTEPS = D / 16;
    constexpr int DBLK = D / 32;

    // buffer b: K rows at b * 2 * KV_BYTES, V rows KV_BYTES behind them (addressed as LDS, so that
    // the buffer index can be a run-time value without the accesses turning into flat ones)
    RA_ROWS_LDS unsigned char *const lds3 = (RA_ROWS_LDS unsigned char *)lds;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int col = lane & 31;
    const int hf = lane >> 5;
    const int bsl = a.block_size_log2;
    const int bmask = (1 << bsl) - 1;

    // ---- decode the work item -----------------------------------------------------------
    bool is_sys = SYS_ONLY || WHOLE || block < a.n_sys_items;      // (WHOLE: of the phase in progress)
    int g, rb, key_begin, key_end, part_index, req = 0, first_blk = 0;
    int n_rows;            // stacked rows of this item's row space (system: all tokens; context: m*G)
    int token_base = 0;    // first packed token of the row space
    int ctx_len = 0, q_len = 0;
    const uint16_t *k_sys = a.k_sys, *v_sys = a.v_sys;
    if (is_sys) {
        int item = block, chunk;
        int sys_len = a.sys_len, n_rowblocks = a.n_sys_rowblocks, n_chunks = a.n_sys_chunks;
        n_rows = a.n_tokens * a.G;
        if (MULTI) {                               // which prefix the item belongs to
            int pfx = 0;
            while (pfx + 1 < a.n_prefixes && item >= a.pfx_item_end[pfx]) ++pfx;
            if (pfx > 0) item -= a.pfx_item_end[pfx - 1];
            sys_len = a.pfx_len[pfx];
            n_rows = a.pfx_ntok[pfx] * a.G;
            token_base = a.pfx_tok0[pfx];
            n_rowblocks = (n_rows + kRowBlock - 1) / kRowBlock;
            n_chunks = WHOLE ? 1 : (sys_len + a.sys_chunk - 1) / a.sys_chunk;
            k_sys = a.pfx_k[pfx];
            v_sys = a.pfx_v[pfx];
        }
        if (a.sys_head_fastest) {
            g = item % a.Hkv;
            rb = (item / a.Hkv) % n_rowblocks;
            chunk = item / (a.Hkv * n_rowblocks);
        } else {
            chunk = item % n_chunks;
            rb = (item / n_chunks) % n_rowblocks;
            g = item / (n_chunks * n_rowblocks);
        }
        key_begin = chunk * a.sys_chunk;
        key_end = min(sys_len, key_begin + a.sys_chunk);
        part_index = chunk;
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
    int limit = is_sys ? INT32_MAX : ctx_len - q_len + (col_ok ? n / a.G : 0);

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

    const uint16_t *ksrc = is_sys ? k_sys + (int64_t)g * a.sys_stride_head : a.k_cache;
    const uint16_t *vsrc = is_sys ? v_sys + (int64_t)g * a.sys_stride_head : a.v_cache;
    // Cooperative load of one step, straight from global memory into LDS (global_load_lds_dwordx4:
    // no landing registers, no LDS store instructions; moving a step through registers cost a
    // quarter of the loop).  Load i of a wavefront fills 1 KiB of LDS, lane l writing the 16 bytes
    // at l * 16 behind the base in M0, which is where (row i*RPL + lrow, position lpos) of the K
    // (or V) rows lives.  The LDS side of such a load cannot be permuted per lane, so the swizzle
    // sits on the global side: position lpos of a row holds K chunk lpos ^ (row mod CPR), resp. V
    // 64-byte segment (lpos / 4) ^ (row mod SEGS) (both maps are their own inverse), and the lane
    // fetches that chunk; a row is still read as whole cache lines.  RPL is a multiple of CPR, so
    // row mod CPR is the same for every i.
    // The instruction is written in assembly because the compiler, told that a load writes LDS,
    // waits for all of them before any LDS read; here the step being loaded is never the step being
    // read, and the one wait that is needed stands in front of the barrier below.  (The compiler's
    // own wait counts stay correct: they can only wait longer for loads it does not know about.)
    const int lrow = threadIdx.x / CPR;
    const int lpos = threadIdx.x % CPR;
    const int ck = lpos ^ (lrow & (CPR - 1));
    const int cv = (((lpos >> 2) ^ (lrow & (SEGS - 1))) << 2) | (lpos & 3);
    const uint32_t lds_wave =
        (uint32_t)(size_t)lds3 + (uint32_t)__builtin_amdgcn_readfirstlane(wave) * (kWave * 16u);
    auto dma16 = [&](const uint16_t *src, uint32_t lds_addr) {      // lds_addr: wave-uniform
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :: "v"(src), "s"(lds_addr) : "memory");
    };
    // System items walk their rows with a running offset (one 64-bit add per load) instead of
    // recomputing row * stride for every load of every step; steps are loaded in order, so the
    // offset simply advances by 64 rows per call.  The ragged last step of a system item clamps
    // its rows to the item's end; context items find their rows through the block table.
    int64_t run_off = (int64_t)(key_begin + lrow) * a.sys_stride_token;
    const int64_t rpl_stride = (int64_t)RPL * a.sys_stride_token;
    auto load_step = [&](int tile0, int buf) {
        const uint32_t kb = lds_wave + (uint32_t)buf * (2 * KV_BYTES);
        if (is_sys && tile0 + STEP <= key_end) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                dma16(ksrc + run_off + i * rpl_stride + ck * 8, kb + i * (RPL * ROW_BYTES));
                dma16(vsrc + run_off + i * rpl_stride + cv * 8, kb + KV_BYTES + i * (RPL * ROW_BYTES));
            }
        } else if (is_sys) {
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int key = min(tile0 + i * RPL + lrow, key_end - 1);   // never past the item's end
                const int64_t off = (int64_t)key * a.sys_stride_token;
                dma16(ksrc + off + ck * 8, kb + i * (RPL * ROW_BYTES));
                dma16(vsrc + off + cv * 8, kb + KV_BYTES + i * (RPL * ROW_BYTES));
            }
        } else {
            int64_t off[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int key = min(tile0 + i * RPL + lrow, key_end - 1);
                const int64_t blk = sm_tbl[(key >> bsl) - first_blk];
                off[i] = (((blk * a.Hkv + g) << bsl) + (key & bmask)) * (int64_t)D;
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                dma16(ksrc + off[i] + ck * 8, kb + i * (RPL * ROW_BYTES));
                dma16(vsrc + off[i] + cv * 8, kb + KV_BYTES + i * (RPL * ROW_BYTES));
            }
        }
        run_off += NL * rpl_stride;
    };
    auto loads_landed = [] { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };

    f32x16 acc_o[DBLK];
#pragma unroll
    for (int db = 0; db < DBLK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    float m_run = -INFINITY, msc = 0.f, l_run = 0.f;
    // Scores are compared raw and scaled only inside the exponent: 2^(s*scale - msc) is one
    // multiply-add per score.  A negative scale flips the sign of the queries instead (below).
    // (A zero scale is replaced by 1e-30: every finite score still gives the weight 1 exactly and a
    // masked one, -inf, still gives 0, where -inf times zero would not be a number.)
    const bool flip = a.scale_log2 < 0.f;
    const float scale = fmaxf(fabsf(a.scale_log2), 1e-30f);
    const float lazy_raw = kLazyLog2 / scale;

    // V^T operand geometry for ds_read_b64_tr_b16 (see relay_tiles.hip)
    const int blk16 = lane >> 4;
    const int r16 = lane & 15;
    const int tr_row = r16 >> 2;
    const int tr_colbyte = 32 * (blk16 & 1) + 8 * (r16 & 3);

    // keys this wavefront needs at all: up to the largest limit among its 32 columns
    int wave_limit, wave_min_limit;
    auto set_wave_limits = [&]() {
        wave_limit = limit;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) wave_limit = max(wave_limit, __shfl_xor(wave_limit, off));
        wave_min_limit = col_ok ? limit : INT32_MAX;
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1)
            wave_min_limit = min(wave_min_limit, __shfl_xor(wave_min_limit, off));
    };
    set_wave_limits();

    // A negative scale: the sign goes into the queries once (exact in bf16), so that the raw
    // scores below are already the ones whose maximum counts.
    if (flip) {
#pragma unroll
        for (int t = 0; t < KSTEPS; ++t) qw[t] ^= u32x4{0x80008000u, 0x80008000u, 0x80008000u, 0x80008000u};
    }
    // (the query registers are made to arrive here, so that no wait for them sits inside the loop)
#pragma unroll
    for (int t = 0; t < KSTEPS; ++t) asm volatile("" : "+v"(qw[t]));
    // One key range [key_begin, key_end) from the current source, with the current limits.
    auto run_range = [&]() {
    if (key_begin < key_end) {
        load_step(key_begin, 0);
        loads_landed();
    }
    __syncthreads();

    int buf = 0;
    for (int tile0 = key_begin; tile0 < key_end; tile0 += STEP, buf ^= 1) {
        // the next step starts its trip into the other buffer, which every wavefront finished
        // reading before the last barrier; it has this whole step to arrive
        if (tile0 + STEP < key_end) load_step(tile0 + STEP, buf ^ 1);
        if (tile0 <= wave_limit) {                // else: every key of the step is masked for this wave
            RA_ROWS_LDS unsigned char *kt = lds3 + buf * (2 * KV_BYTES);
            RA_ROWS_LDS unsigned char *vt = kt + KV_BYTES;
            const bool edge = tile0 + STEP > key_end || tile0 + STEP - 1 > wave_min_limit;   // ragged end or causal edge
            const int lim = min(limit, key_end - 1);

            // S^T of tile A (keys tile0 .. +31) and tile B (keys tile0+32 .. +63): two independent
            // accumulation chains; K operands are read one batch of products ahead of their use
            auto scores = [&](f32x16 &sa_, f32x16 &sb_) {
#pragma unroll
                for (int r = 0; r < 16; ++r) sa_[r] = 0.f, sb_[r] = 0.f;
                constexpr int KB = 2;
                bf16x8 ka[2][KB], kb[2][KB];
                auto read_k = [&](int slot, int t0) {
#pragma unroll
                    for (int t = 0; t < KB; ++t) {
                        const int pos = (2 * (t0 + t) + hf) ^ (col & (CPR - 1));
                        ka[slot][t] = *(RA_ROWS_LDS const bf16x8 *)(kt + col * ROW_BYTES + pos * 16);
                        kb[slot][t] = *(RA_ROWS_LDS const bf16x8 *)(kt + (32 + col) * ROW_BYTES + pos * 16);
                    }
                };
                read_k(0, 0);
#pragma unroll
                for (int t0 = 0; t0 < KSTEPS; t0 += KB) {
                    const int cur = (t0 / KB) & 1;
                    if (t0 + KB < KSTEPS) read_k(cur ^ 1, t0 + KB);
#pragma unroll
                    for (int t = 0; t < KB; ++t) {
                        const bf16x8 qf = __builtin_bit_cast(bf16x8, qw[t0 + t]);
                        sa_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[cur][t], qf, sa_, 0, 0, 0);
                        sb_ = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[cur][t], qf, sb_, 0, 0, 0);
                    }
                }
            };
            // Bookkeeping of the step: mask (edge steps only), column maximum over both tiles, and the
            // move of the reference maximum when a column outgrew it by the margin or sees its first
            // key.  Accumulator register r of lane (col, hf) is key 8*(r/4) + 4*hf + r%4 of its tile.
            auto settle = [&](f32x16 &sa_, f32x16 &sb_) {
                if (edge) {
                    // (kept a branch: as selects on every step the masking costs as much as the exponentials)
                    asm volatile("" ::: "memory");
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = tile0 + 8 * (r / 4) + 4 * hf + (r % 4);
                        sa_[r] = key <= lim ? sa_[r] : -INFINITY;
                        sb_[r] = key + 32 <= lim ? sb_[r] : -INFINITY;
                    }
                }
                float mx4[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    mx4[c] = fmaxf(sa_[4 * c], sb_[4 * c]);
#pragma unroll
                    for (int r = 4 * c + 1; r < 4 * c + 4; ++r) mx4[c] = fmaxf(fmaxf(mx4[c], sa_[r]), sb_[r]);
                }
                float mx = fmaxf(fmaxf(mx4[0], mx4[1]), fmaxf(mx4[2], mx4[3]));
                mx = max_with_other_half(mx);
                const float m_new = fmaxf(m_run, mx);
                if (__builtin_amdgcn_ballot_w64(m_new > m_run + lazy_raw || (m_run == -INFINITY && m_new > m_run)) != 0) {
                    const float msc_new = m_new == -INFINITY ? 0.f : m_new * scale;
                    const float corr = m_run == -INFINITY ? 0.f : rows_exp2(msc - msc_new);
                    l_run *= corr;
#pragma unroll
                    for (int db = 0; db < DBLK; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc_o[db][r] *= corr;
                    m_run = m_new;
                    msc = msc_new;
                }
            };
            // weights of one tile, their sum, and their bf16 high + low parts (see relay_tiles.hip)
            auto weights = [&](const f32x16 &sc, uint32_t (&pw)[8], uint32_t (&pw_lo)[8]) {
                const float neg_msc = -msc;
                float psum = 0.f;
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    const float p0 = rows_exp2(fmaf(sc[r], scale, neg_msc)), p1 = rows_exp2(fmaf(sc[r + 1], scale, neg_msc));
                    psum += p0 + p1;
                    const uint32_t h = rows_pack_bf16(p0, p1);
                    pw[r / 2] = h;
                    pw_lo[r / 2] = rows_pack_bf16(p0 - bf16_lo(h), p1 - bf16_hi(h));
                }
                l_run += psum;
            };
            // O^T += V^T P^T for one tile: two products of 16 keys per head_dim block, high and low part
            auto accumulate = [&](int row0, const uint32_t (&pw)[8], const uint32_t (&pw_lo)[8]) {
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
                            const int row = row0 + 16 * kstep + 8 * half + 4 * hf + tr_row;
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
            };

            // (Orders that put one tile's exponentials next to the other's products, two bookkeeping
            // passes, and a dot-product form of the low half were all measured slower than this
            // plain sequence, by 5 - 10 % of the step.)
            uint32_t pa[8], pa_lo[8], pb_[8], pb_lo[8];
            f32x16 sa, sb;
            scores(sa, sb);
            settle(sa, sb);
            weights(sa, pa, pa_lo);
            weights(sb, pb_, pb_lo);
            accumulate(0, pa, pa_lo);
            accumulate(32, pb_, pb_lo);
        }
        loads_landed();
        __syncthreads();   // next step visible to all; everyone is done reading this one
    }
    };   // run_range

    if constexpr (!WHOLE) {
        run_range();
    } else {
        // ---- the system prompt, then the context of every request that has rows in this block
        if (key_begin < key_end) run_range();
        const int tok_a = token_base + rb * kRowBlock / a.G;                     // tokens of the block
        const int tok_b = token_base + (min(n_rows, (rb + 1) * kRowBlock) - 1) / a.G;
        is_sys = false;
        ksrc = a.k_cache;
        vsrc = a.v_cache;
        // the first request that ends behind tok_a: requests are scanned 64 at a time, a lane each
        int r = a.batch;
        for (int base = 0; base < a.batch; base += kWave) {
            const int rr = base + lane;
            const int e_lane = rr < a.batch ? a.cu_seqlens_q[rr + 1] : INT32_MAX;
            const uint64_t hit = __builtin_amdgcn_ballot_w64(rr < a.batch && e_lane > tok_a);
            if (hit != 0) {
                r = base + (int)__builtin_ctzll(hit);
                break;
            }
        }
        for (; r < a.batch; ++r) {
            const int q0 = a.cu_seqlens_q[r], q1 = a.cu_seqlens_q[r + 1];
            if (q0 > tok_b) break;
            const int m = q1 - q0;
            if (m <= 0) continue;
            const int c = a.context_lens[r];
            // the last row of the request inside this block sees the most
            // (contexts beyond the host's bound are cut off there, as in the two-launch form)
            const int kend = min(min(c, c - m + (min(tok_b, q1 - 1) - q0) + 1), a.n_ctx_parts * a.ctx_part);
            const int tk = token_base + n / a.G;
            limit = col_ok && tk >= q0 && tk < q1 ? c - m + (tk - q0) : -1;
            set_wave_limits();
            req = r;
            for (int part = 0; part * a.ctx_part < kend; ++part) {
                key_begin = part * a.ctx_part;
                key_end = min(kend, key_begin + a.ctx_part);
                first_blk = key_begin >> bsl;
                const int nblk = ((key_begin + a.ctx_part - 1) >> bsl) - first_blk + 1;
                const int32_t *bt = a.block_tables + (int64_t)r * a.max_blocks_per_seq;
                // (every wavefront left the previous range behind the barrier that ends it)
                for (int i = threadIdx.x; i < nblk; i += kThreads)
                    sm_tbl[i] = bt[min(first_blk + i, a.max_blocks_per_seq - 1)];
                __syncthreads();
                run_range();
            }
        }
        // ---- the block's output rows, from registers (what the fusion launch does otherwise)
        l_run = sum_with_other_half(l_run);
        if (col_ok) {
            const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
            const int64_t oo = (int64_t)token * a.o_stride_token + (int64_t)hq * a.o_stride_head;
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 v = {acc_o[db][4 * r4] * inv, acc_o[db][4 * r4 + 1] * inv,
                                     acc_o[db][4 * r4 + 2] * inv, acc_o[db][4 * r4 + 3] * inv};
                    const int e = db * 32 + 8 * r4 + 4 * hf;
                    if (a.out_is_fp32) {
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(a.out) + oo + e) = v;
                    } else {
                        const u32x2 w2 = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
                        *reinterpret_cast<u32x2 *>(static_cast<uint16_t *>(a.out) + oo + e) = w2;
                    }
                }
            if (hf == 0 && a.lse_out)
                a.lse_out[(int64_t)token * a.Hq + hq] = l_run > 0.f ? (msc + log2f(l_run)) * kLn2 : -INFINITY;
        }
        return;
    }

    // ---- each wavefront writes the partial of its 32 rows from registers ----------------------
    l_run = sum_with_other_half(l_run);
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
        if (hf == 0) a.part_lse[prow] = l_run > 0.f ? msc + log2f(l_run) : -INFINITY;
    }
}

}  // namespace ra
