// One launch for both partial attentions of a decode step (Alg. 1 "system attention" and
// "context attention"; the paper notes they have no dependency on each other).
//
// The grid is a list of workgroups, system work first:
//   system workgroup   one item (kv head, tile of 32 stacked query rows, chunk of system
//                      positions): the queries of the whole batch that share a kv head are the
//                      columns of one matrix product, so the shared system K/V are streamed
//                      once per batch (Sec. 3.3; Eq. 7, first term).  The four wavefronts take
//                      the chunk's 32-key tiles round-robin and merge through LDS at the end.
//   context workgroup  four independent wavefronts.  The 32-key tiles of all (request, kv head)
//                      context items form one stream that is cut into one span per context
//                      wavefront (see run_context_wave); inside its span a wavefront attends
//                      the G query heads of a kv head to that request's own paged K/V, item
//                      by item (Eq. 7, second term).  No barrier, no merge.
// Both kinds run the same tile pipeline; a context item simply has G live query columns out of
// 32 and finds its rows through the block table.  The host sizes the launch so that, when there
// is enough work, all workgroups are resident at once (two per compute unit) and every compute
// unit ends up with about the same number of tiles.  For batches with many stacked rows per kv
// head the system workgroups are items of the many-rows kind instead (rows_item.h; template
// parameter ROWS of the kernel).
//
// Tile pipeline of one wavefront (no barrier inside the key loop), per 32-key tile:
//   * K and V rows are loaded with coalesced 16-byte loads into registers (non-temporal where a
//     row is read once per launch: measured +13 % on a streaming probe) and stored XOR-swizzled
//     into the wavefront's LDS slice only when the previous tile's copy has been consumed, so
//     the registers, not the LDS, are the landing zone;
//   * both loads for tile t+1 are issued as soon as S^T of tile t is done, so about one whole
//     tile per wavefront is in flight for most of the iteration;
//   * S^T = K Q^T (keys x queries) with v_mfma_f32_32x32x16_bf16, K operands by ds_read_b128: a
//     lane owns one query column, so the softmax statistics are in-lane plus one exchange with lane^32;
//   * O^T += V^T P^T: V^T operands come from the row-major V tile through the LDS transpose
//     read ds_read_b64_tr_b16; P^T is taken from the S^T accumulator registers (split into a
//     high and a low bf16 part so that no 2^-9 rounding of the weights reaches the output).
// Reduction order depends only on the logical position of a key, never on the physical block,
// so any block placement of the same cache gives bit-identical results.  Rows past the end of
// an item are never loaded (their lanes re-load the item's last row and the scores are masked);
// block-table slots past the last used block may be read but are never dereferenced.
#include "ra_device.h"
#include "ra_kernels.h"
#include "rows_item.h"

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
    static constexpr int SLICE = 32 * D * 4;          // LDS bytes per wavefront
    static constexpr int KSTEPS = D / 16;
    static constexpr int DBLK = D / 32;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// 16-byte global load.  V rows that are read exactly once per launch, by loads that consume whole
// cache lines, use the non-temporal form: a read-only streaming probe on this chip measured
// 6.98 TB/s with it against 6.19 TB/s with ordinary loads.
template <bool NT>
__device__ __forceinline__ u32x4 load16(const uint16_t *p) {
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    return NT ? __builtin_nontemporal_load(q) : *q;
}

__device__ __forceinline__ uint32_t pack_bf16_hw(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// One work item as the tile pipeline sees it.
struct Item {
    int g;                    // kv head
    int key_begin, key_end;   // positions [key_begin, key_end) of the system prompt / the context
    int part_index;           // partial slot the result goes to
    int req;                  // context item: request (= token of the decode batch)
    int mt, tok0, ncols;      // system item: row tile, first token of its prefix, live columns
    int append_pos;           // context item: position to take from the new rows and write to the
                              // cache (the item's last one; this segment ends with it), or -1
    const uint16_t *k, *v;    // system item: K/V of kv head g (context items use the paged cache)
};

template <int D, bool SYS, bool NT, bool APPEND = false>
__device__ __forceinline__ void attend(const TileArgs &a, const Item &it, const int lane,
                                       unsigned char *smem, float (*sm_m)[32], float (*sm_l)[32],
                                       int32_t (*sm_tbl)[kMaxPartBlocks]) {
    using T = TileCfg<D>;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int col = lane & 31;
    const int hf = lane >> 5;
    const int bsl = a.block_size_log2;
    const int bmask = (1 << bsl) - 1;

    const int g = it.g, key_begin = it.key_begin;
    int key_end = it.key_end;
    const int part_index = it.part_index, req = it.req, mt = it.mt, tok0 = it.tok0;
    const int ncols = SYS ? it.ncols : a.G;
    // a system item's 32-key tiles go round-robin over the four wavefronts; a context span
    // belongs to one wavefront
    const int tile_first = SYS ? key_begin + wave * 32 : key_begin;
    const int tile_stride = SYS ? kWaves * 32 : 32;
    int first_blk = 0;
    int32_t *tbl = sm_tbl[wave];
    if (!SYS) {
        // block ids of the span go to a small LDS table first (one coalesced read)
        first_blk = key_begin >> bsl;
        int nblk = key_end > key_begin ? ((key_end - 1) >> bsl) - first_blk + 1 : 0;
        // (never binding: the host sized the spans for the table and context_lens for the row)
        nblk = min(nblk, min(kMaxPartBlocks, a.max_blocks_per_seq - first_blk));
        key_end = min(key_end, (first_blk + nblk) << bsl);
        const int32_t *bt = a.block_tables + (int64_t)req * a.max_blocks_per_seq + first_blk;
        for (int j = lane; j < nblk; j += kWave) tbl[j] = bt[j];
    }

    // query column -> (token, head)
    auto column_row = [&](int c, int &token, int &hq) {
        if (SYS) {
            const int n = mt * 32 + c;
            token = tok0 + n / a.G;
            if (a.req_order) token = a.req_order[token];      // requests of a prefix in any order
            hq = g * a.G + n % a.G;
        } else {
            token = req;
            hq = g * a.G + c;
        }
    };

    // B operand of S^T = K Q^T: lane (col, hf) holds Q[column col][t*16 + hf*8 .. +7]
    u32x4 qw[T::KSTEPS];
    {
        const bool ok = col < ncols;
        int token = 0, hq = 0;
        if (ok) column_row(col, token, hq);
        const uint16_t *qp =
            a.q + (int64_t)token * a.q_stride_token + (int64_t)hq * a.q_stride_head + hf * 8;
#pragma unroll
        for (int t = 0; t < T::KSTEPS; ++t) {
            qw[t] = u32x4{0, 0, 0, 0};
            if (ok) qw[t] = *reinterpret_cast<const u32x4 *>(qp + t * 16);
        }
    }

    // LDS slice of this wavefront: the V tile (first half) and the K tile (second half) during
    // the key loop, the fp32 merge buffer of a system item afterwards (all 32*D*4 bytes).
    unsigned char *my = smem + wave * T::SLICE;
    unsigned char *my_k = my + 32 * T::ROW_BYTES;
    RA_LDS unsigned char *my_lds = (RA_LDS unsigned char *)my;

    const uint16_t *ksrc = SYS ? it.k : a.k_cache;
    const uint16_t *vsrc = SYS ? it.v : a.v_cache;
    // element offset of row `key` (already clamped to the item) from ksrc / vsrc
    auto row_offset = [&](int key) -> int64_t {
        if (SYS) return (int64_t)key * a.sys_stride_token;
        const int64_t blk = tbl[(key >> bsl) - first_blk];
        return (((blk * a.Hkv + g) << bsl) + (key & bmask)) * (int64_t)D;
    };

    // K and V rows: coalesced 16-byte loads (whole cache lines per load, so rows that are read
    // once can use the non-temporal form); load i covers rows i*RPI .. i*RPI+RPI-1 of the tile and
    // this lane takes 16-byte chunk `lpos` of row i*RPI + lrow.  Rows past the item's end re-load
    // its last row (their scores are masked).  In LDS, K chunk c of row r sits at position
    // c ^ (r mod CPR) and V 64-byte segment s of row r at segment s ^ (r mod SEGS): both make the
    // MFMA operand reads below free of bank conflicts.
    const int lrow = lane / T::CPR;
    const int lpos = lane % T::CPR;
    u32x4 kreg[T::NI], vreg[T::NI];
    // Fused cache write (Alg. 1 writes the new key/value into the cache, then attends): the
    // segment that ends with the item's last position takes that row from the new rows instead
    // of the cache (so what the cache held there is never read), and writes it to the cache when
    // the tile is consumed (append_store).  No other wavefront of the launch reads that row.
    const int append_pos = SYS || !APPEND ? -1 : it.append_pos;
    auto load_kv = [&](int tile0) {
        if (!SYS && APPEND && append_pos >= 0 && tile0 + 32 >= key_end) {      // (uniform) the tile holding it
            const int64_t new_off = (int64_t)req * a.new_stride_token + (int64_t)g * a.new_stride_head;
#pragma unroll
            for (int i = 0; i < T::NI; ++i) {
                const int key = min(tile0 + i * T::RPI + lrow, key_end - 1);
                const bool fresh = key == append_pos;
                const int64_t off = (fresh ? new_off : row_offset(key)) + lpos * 8;
                vreg[i] = load16<NT>((fresh ? a.v_new : vsrc) + off);
                kreg[i] = load16<NT>((fresh ? a.k_new : ksrc) + off);
            }
            return;
        }
#pragma unroll
        for (int i = 0; i < T::NI; ++i) {
            const int key = min(tile0 + i * T::RPI + lrow, key_end - 1);
            const int64_t off = row_offset(key) + lpos * 8;
            vreg[i] = load16<NT>(vsrc + off);
            kreg[i] = load16<NT>(ksrc + off);
        }
    };
    // (called when both landing registers hold tile `tile0`, landed)
    auto append_store = [&](int tile0) {
        if (!SYS && APPEND && append_pos >= 0 && tile0 + 32 >= key_end) {
            const int i = (append_pos - tile0) / T::RPI;              // the load that holds the row
            if ((append_pos - tile0) % T::RPI == lrow) {
                const int64_t off = row_offset(append_pos) + lpos * 8;
#pragma unroll
                for (int k = 0; k < T::NI; ++k)
                    if (k == i) {
                        *reinterpret_cast<u32x4 *>(const_cast<uint16_t *>(ksrc) + off) = kreg[k];
                        *reinterpret_cast<u32x4 *>(const_cast<uint16_t *>(vsrc) + off) = vreg[k];
                    }
            }
        }
    };
    auto store_k = [&]() {
#pragma unroll
        for (int i = 0; i < T::NI; ++i) {
            const int r = i * T::RPI + lrow;
            *reinterpret_cast<u32x4 *>(my_k + r * T::ROW_BYTES + (lpos ^ (r & (T::CPR - 1))) * 16) = kreg[i];
        }
    };
    auto store_v = [&]() {
#pragma unroll
        for (int i = 0; i < T::NI; ++i) {
            const int r = i * T::RPI + lrow;
            const int pos = (((lpos >> 2) ^ (r & (T::SEGS - 1))) << 2) | (lpos & 3);
            *reinterpret_cast<u32x4 *>(my + r * T::ROW_BYTES + pos * 16) = vreg[i];
        }
    };

    if (tile_first < key_end) load_kv(tile_first);

    f32x16 acc_o[T::DBLK];
#pragma unroll
    for (int db = 0; db < T::DBLK; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // V^T operand geometry for ds_read_b64_tr_b16: inside each block of 16 lanes, lane r
    // addresses 4 consecutive head_dim elements of row K0 + r/4 starting at D0 + 4*(r%4);
    // lane i of the block receives rows K0..K0+3 of column D0 + i.
    const int blk16 = lane >> 4;                  // (blk16 & 1) picks the column half,
    const int r16 = lane & 15;                    // (blk16 >> 1) == hf picks the key half
    const int tr_row = r16 >> 2;
    const int tr_colbyte = 32 * (blk16 & 1) + 8 * (r16 & 3);

    if (tile_first < key_end) store_v();          // V of the first tile

    for (int tile0 = tile_first; tile0 < key_end; tile0 += tile_stride) {
        const int next = tile0 + tile_stride;
        const bool has_next = next < key_end;

        // S^T tile: 32 keys x 32 queries.  K of this tile goes from its landing registers into
        // LDS and comes back in the MFMA operand layout (lane = key row).
        store_k();
        append_store(tile0);
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int t = 0; t < T::KSTEPS; ++t) {
            const int pos = (2 * t + hf) ^ (col & (T::CPR - 1));
            const bf16x8 kf = *reinterpret_cast<const bf16x8 *>(my_k + col * T::ROW_BYTES + pos * 16);
            s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, __builtin_bit_cast(bf16x8, qw[t]), s, 0, 0, 0);
        }
        // The landing registers are free again: V and K of the next tile start their trip now and
        // arrive while the rest of this tile is computed.
        if (has_next) load_kv(next);
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] *= a.scale_log2;

        // accumulator register r of lane (col, hf) is key 8*(r/4) + 4*hf + r%4 of the tile
        if (tile0 + 32 > key_end) {               // ragged last tile: mask the missing keys
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = tile0 + 8 * (r / 4) + 4 * hf + (r % 4);
                s[r] = key < key_end ? s[r] : -INFINITY;
            }
        }
        float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
#pragma unroll
        for (int r = 4; r < 16; r += 4)
            mx = fmaxf(mx, fmaxf(fmaxf(s[r], s[r + 1]), fmaxf(s[r + 2], s[r + 3])));
        mx = max_with_other_half(mx);
        const float m_new = fmaxf(m_run, mx);     // finite: every processed tile has a valid key
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {   // some column's maximum moved
            const float corr = fast_exp2(m_run - m_new);
            l_run *= corr;
#pragma unroll
            for (int db = 0; db < T::DBLK; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc_o[db][r] *= corr;
            m_run = m_new;
        }
        // P is fed to the MFMA as bf16; a single rounding would leave 2^-9 relative error per
        // weight, so it is split into a high and a low bf16 part (error ~2^-17) and O^T takes two
        // MFMA passes.  The row sum uses the unrounded fp32 weights.
        float psum = 0.f;
        uint32_t pw[8], pw_lo[8];
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const float p0 = fast_exp2(s[r] - m_run), p1 = fast_exp2(s[r + 1] - m_run);
            psum += p0 + p1;
            const uint32_t h = pack_bf16_hw(p0, p1);
            pw[r / 2] = h;
            pw_lo[r / 2] = pack_bf16_hw(p0 - bf16_lo(h), p1 - bf16_hi(h));
        }
        l_run += psum;

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
            for (int db = 0; db < T::DBLK; ++db) {
                s16x4 v4[2];
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int row = 16 * kstep + 8 * half + 4 * hf + tr_row;
                    const int seg = db ^ (row & (T::SEGS - 1));
                    v4[half] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (RA_LDS s16x4 *)(my_lds + row * T::ROW_BYTES + seg * 64 + tr_colbyte));
                }
                const s16x8 v8 = __builtin_shufflevector(v4[0], v4[1], 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, v8);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, acc_o[db], 0, 0, 0);
                acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf_lo, acc_o[db], 0, 0, 0);
            }
        }
        // every V operand of this tile has been read: the next tile's V takes its place
        if (has_next) store_v();
    }

    l_run = sum_with_other_half(l_run);

    if (!SYS) {
        // ---- context item: the wavefront owns the whole item; write its partial from registers
        if (col < ncols) {
            const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
            int token, hq;
            column_row(col, token, hq);
            const int64_t prow = (int64_t)part_index * a.rows + (int64_t)token * a.Hq + hq;
            float *dst = a.part_o + prow * D;
#pragma unroll
            for (int db = 0; db < T::DBLK; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    // registers 4*r4 .. 4*r4+3 are head_dim elements db*32 + 8*r4 + 4*hf + 0..3
                    const f32x4 v = {acc_o[db][4 * r4] * inv, acc_o[db][4 * r4 + 1] * inv,
                                     acc_o[db][4 * r4 + 2] * inv, acc_o[db][4 * r4 + 3] * inv};
                    *reinterpret_cast<f32x4 *>(dst + db * 32 + 8 * r4 + 4 * hf) = v;
                }
            if (hf == 0) a.part_lse[prow] = l_run > 0.f ? m_run + log2f(l_run) : -INFINITY;
        }
        return;
    }

    // ---- system item: merge the four wavefronts through LDS and write the partial ------------
    if (hf == 0) {
        sm_m[wave][col] = m_run;
        sm_l[wave][col] = l_run;
    }
    __syncthreads();   // also: every wavefront is done with its K/V slice
    float M_all = sm_m[0][col];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) M_all = fmaxf(M_all, sm_m[w][col]);
    const float f_mine = fast_exp2(m_run - finite_or_zero(M_all));
    float *osh = reinterpret_cast<float *>(my) + col * D;      // merge buffer row of this lane
    constexpr int OCH = D / 4;                    // 16-byte chunks per fp32 output row
    if (col < ncols) {
#pragma unroll
        for (int db = 0; db < T::DBLK; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                f32x4 v = {acc_o[db][4 * r4] * f_mine, acc_o[db][4 * r4 + 1] * f_mine,
                           acc_o[db][4 * r4 + 2] * f_mine, acc_o[db][4 * r4 + 3] * f_mine};
                const int chunk = (db * 8 + 2 * r4 + hf) ^ (col & (OCH - 1));
                *reinterpret_cast<f32x4 *>(osh + chunk * 4) = v;
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
                const float *src = reinterpret_cast<const float *>(smem + w * T::SLICE) + row * D;
                sum += *reinterpret_cast<const f32x4 *>(src + chunk * 4);
            }
            *reinterpret_cast<f32x4 *>(dst + e) = sum * inv;
        }
        if (seg == 0) a.part_lse[prow] = L > 0.f ? Mr + log2f(L) : -INFINITY;
    }
}

// System workgroup: decode the grid index into (prefix, kv head, row tile, chunk).
template <int D, bool NT, bool MULTI>
__device__ __forceinline__ void run_system_item(const TileArgs &a, unsigned char *smem,
                                                float (*sm_m)[32], float (*sm_l)[32],
                                                int32_t (*sm_tbl)[kMaxPartBlocks]) {
    // Item order follows the memory layout of the system cache: with token-major storage
    // ([s][Hkv][d]) neighbouring workgroups take the same positions of neighbouring heads, so
    // the workgroups in flight together read whole contiguous rows of DRAM; with head-major
    // storage they take neighbouring chunks of one head.
    // Which shared prefix (App. D: several applications in one batch; one in the paper's main
    // setting) this system item belongs to.  (MULTI is a compile-time switch so that the
    // single-prefix kernel reads its prefix from fixed kernel-argument slots.)
    int item = blockIdx.x, pfx = 0;
    if (MULTI) {
        while (pfx + 1 < a.n_prefixes && item >= a.pfx_item_end[pfx]) ++pfx;
        if (pfx > 0) item -= a.pfx_item_end[pfx - 1];
    }
    const int sys_len = a.pfx_len[pfx];
    const int n_mtiles = (a.pfx_tokens[pfx] * a.G + 31) / 32;
    const int n_chunks = (sys_len + a.sys_chunk - 1) / a.sys_chunk;
    Item it;
    int chunk;
    if (a.sys_head_fastest) {
        it.g = item % a.Hkv;
        it.mt = (item / a.Hkv) % n_mtiles;
        chunk = item / (a.Hkv * n_mtiles);
    } else {
        chunk = item % n_chunks;
        it.mt = (item / n_chunks) % n_mtiles;
        it.g = item / (n_chunks * n_mtiles);
    }
    it.key_begin = chunk * a.sys_chunk;
    it.key_end = min(sys_len, it.key_begin + a.sys_chunk);
    it.part_index = chunk;
    it.req = 0;
    it.append_pos = -1;
    it.tok0 = a.pfx_first[pfx];
    it.ncols = min(32, a.pfx_tokens[pfx] * a.G - it.mt * 32);
    it.k = a.pfx_k[pfx] + (int64_t)it.g * a.sys_stride_head;
    it.v = a.pfx_v[pfx] + (int64_t)it.g * a.sys_stride_head;
    attend<D, true, NT>(a, it, threadIdx.x & (kWave - 1), smem, sm_m, sm_l, sm_tbl);
}

__device__ __forceinline__ int wave_inclusive_scan(int x, int lane) {
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        const int y = __shfl_up(x, d);
        if (lane >= d) x += y;
    }
    return x;
}

// Context wavefront.  The 32-key tiles of all context items, in (request, kv head, position)
// order, form one stream that is cut into one span per context wavefront; the span lengths are
// computed from the context lengths found on the device, so the split is even however the
// lengths are distributed.  A span that crosses from one (request, kv head) item into the next is
// processed as one segment per item; segment number k of an item writes context partial slot k,
// and the wavefront that begins an item marks the slots the item does not use as empty.  The
// host chose ctx_t_floor so that no item has more than n_ctx_slots segments.  An empty context
// counts as one tile without keys, so that its rows still get their (empty) partial.
//
// Span lengths.  A compute unit draws about 1/256 of the memory bandwidth at most, whatever it
// holds, so what has to be even is the number of tiles per compute unit, not per wavefront.  When
// the launch is exactly two workgroups per compute unit, workgroups i and i + 256 of the grid
// share a unit (the dispatcher deals them out in order; measured on every unit in three traces),
// so the context workgroups that sit next to a system workgroup ("light") get spans that bring
// their unit up to the average, and the ones that sit next to each other ("heavy") share the
// rest.  ctx_light_begin .. + ctx_light_waves are the light wavefronts; none: all spans equal.
template <int D, bool APPEND>
__device__ __forceinline__ void run_context_wave(const TileArgs &a, unsigned char *smem,
                                                 float (*sm_m)[32], float (*sm_l)[32],
                                                 int32_t (*sm_tbl)[kMaxPartBlocks]) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int w = ((int)blockIdx.x - a.n_sys_items) * kWaves + wave;
    const int B = a.n_tokens;
    auto len_of = [&](int r) { return r < B ? min(a.context_lens[r], a.max_ctx) : 0; };
    auto tiles_of = [&](int c) { return max(1, (c + 31) >> 5); };

    // lengths of requests chunk_base .. chunk_base+63, one per lane, and their running tile count
    int chunk_base = 0;
    int c_lane = len_of(lane);
    int incl = wave_inclusive_scan(lane < B ? tiles_of(c_lane) : 0, lane);
    int total = __builtin_amdgcn_readlane(incl, kWave - 1);
    for (int base = kWave; base < B; base += kWave) {
        const int r = base + lane;
        const int t = wave_inclusive_scan(r < B ? tiles_of(len_of(r)) : 0, lane);
        total += __builtin_amdgcn_readlane(t, kWave - 1);
    }
    // (the host refuses launches whose tile count could exceed 31 bits)
    const uint32_t n_tiles = (uint32_t)total * a.Hkv;
    const uint32_t floor_t = (uint32_t)a.ctx_t_floor;
    // Two classes of wavefront, "light" (numbers lb .. lb+nl-1) and "heavy" (the others), each
    // described by three numbers: when fix > 0 every wavefront of the class takes `fix` tiles;
    // otherwise workgroup v of the class takes Q_v = per_wg + (v < extra) tiles and its wavefront k
    // takes Q_v / 4 + (k < Q_v % 4) of them, so that workgroups differ by one tile at most and no
    // wavefront is left without work while others carry a rounded-up share.
    uint32_t lb = (uint32_t)a.ctx_light_begin, nl = (uint32_t)a.ctx_light_waves;
    const uint32_t n_heavy = (uint32_t)a.ctx_waves - nl;
    uint32_t l_per_wg = 0, l_fix = 0, l_total = 0;
    if (nl > 0 && n_heavy > 0) {
        // tiles per compute unit, and what a system workgroup leaves of it for its neighbour
        const uint32_t per_unit = ((uint32_t)a.sys_tiles_total + n_tiles) / 256u;
        const uint32_t l4 = per_unit > (uint32_t)a.sys_wg_tiles ? per_unit - (uint32_t)a.sys_wg_tiles : 0;
        if (l4 / kWaves >= floor_t) {
            l_per_wg = l4;
            l_total = l4 * (nl / kWaves);
        } else {                                  // no spans shorter than the floor
            l_fix = 2 * (l4 / kWaves) >= floor_t ? floor_t : 0;
            l_total = l_fix * nl;
        }
        if (l_total > n_tiles) l_per_wg = l_fix = l_total = 0;
    } else {
        lb = (uint32_t)a.ctx_waves;          // no light wavefronts
        nl = 0;
    }
    uint32_t h_per_wg, h_extra, h_fix;
    auto share_heavy = [&](uint32_t n_waves) {
        const uint32_t rest = n_tiles - l_total, nh_wg = n_waves / kWaves;
        h_per_wg = rest / nh_wg;
        h_extra = h_fix = 0;
        if (h_per_wg / kWaves >= floor_t) h_extra = rest - h_per_wg * nh_wg;
        else h_fix = floor_t;
    };
    share_heavy(nl > 0 ? n_heavy : (uint32_t)a.ctx_waves);
    // A span must fit the wavefront's block-id table (ctx_t_cap tiles).  Equal spans do (the
    // host sized the launch for that); should the light / heavy split push a class beyond it,
    // the split is dropped.
    if (nl > 0) {
        const uint32_t most_l = l_fix > 0 ? l_fix : (l_per_wg + 3u) >> 2;
        const uint32_t most_h = h_fix > 0 ? h_fix : (h_per_wg + (h_extra > 0 ? 1u : 0u) + 3u) >> 2;
        if (most_l > (uint32_t)a.ctx_t_cap || most_h > (uint32_t)a.ctx_t_cap) {
            lb = (uint32_t)a.ctx_waves;
            nl = 0;
            l_per_wg = l_fix = l_total = 0;
            share_heavy((uint32_t)a.ctx_waves);
        }
    }
    // Light wavefronts without a span drop out, and the others are numbered as if they were not
    // there (slot numbers count spans, and an item must not skip any).
    uint32_t uw = (uint32_t)w;
    if (nl > 0 && l_total == 0) {
        if (uw >= lb && uw < lb + nl) return;
        if (uw >= lb + nl) uw -= nl;
        lb = n_heavy;
        nl = 0;
    }
    // tiles of wavefront i of a class, and the tiles of the class before it
    auto class_len = [](uint32_t i, uint32_t per_wg, uint32_t extra, uint32_t fix) -> uint32_t {
        if (fix > 0) return fix;
        const uint32_t q = per_wg + ((i >> 2) < extra ? 1u : 0u);
        return (q >> 2) + ((i & 3u) < (q & 3u) ? 1u : 0u);
    };
    auto class_first = [](uint32_t i, uint32_t per_wg, uint32_t extra, uint32_t fix) -> uint32_t {
        if (fix > 0) return i * fix;
        const uint32_t v = i >> 2, k = i & 3u;
        const uint32_t q = per_wg + (v < extra ? 1u : 0u);
        return v * per_wg + min(v, extra) + k * (q >> 2) + min(k, q & 3u);
    };
    auto len_of_wave = [=](uint32_t u) -> uint32_t {
        if (u >= lb && u < lb + nl) return class_len(u - lb, l_per_wg, 0u, l_fix);
        return class_len(u < lb ? u : u - nl, h_per_wg, h_extra, h_fix);
    };
    uint32_t x0;
    if (uw < lb) x0 = class_first(uw, h_per_wg, h_extra, h_fix);
    else if (uw < lb + nl) x0 = class_first(lb, h_per_wg, h_extra, h_fix) + class_first(uw - lb, l_per_wg, 0u, l_fix);
    else x0 = class_first(uw - nl, h_per_wg, h_extra, h_fix) + l_total;
    const uint32_t my_len = len_of_wave(uw);
    if (x0 >= n_tiles || my_len == 0) return;
    const uint32_t x1 = min(x0 + my_len, n_tiles);

    // the request that owns tile x0: first r with Hkv * (tiles of requests 0..r) > x0
    int before = 0;                               // tiles of the requests before chunk_base
    uint64_t hit;
    while ((hit = __builtin_amdgcn_ballot_w64(
                chunk_base + lane < B && (uint32_t)(before + incl) * a.Hkv > x0)) == 0) {
        if (chunk_base + kWave >= B) return;      // (x0 < n_tiles, so this cannot happen)
        before += __builtin_amdgcn_readlane(incl, kWave - 1);
        chunk_base += kWave;
        c_lane = len_of(chunk_base + lane);
        incl = wave_inclusive_scan(chunk_base + lane < B ? tiles_of(c_lane) : 0, lane);
    }
    const int idx = __builtin_ctzll(hit);
    int req = chunk_base + idx;
    int c_req = __builtin_amdgcn_readlane(c_lane, idx);
    uint32_t T = tiles_of(c_req);
    const uint32_t req_first = (uint32_t)(before + __builtin_amdgcn_readlane(incl, idx) - (int)T) * a.Hkv;
    int g = (int)((x0 - req_first) / T);
    uint32_t j = (x0 - req_first) % T;            // tile of the item (req, g) that x0 is

    uint32_t x = x0;
    while (true) {
        const uint32_t seg = min(x1 - x, T - j);
        const uint32_t item_first = x - j;
        // (x is the first tile of an item, or the first tile of this wavefront's span)
        // the segment's slot: how many spans back the item began (only the first segment of a
        // span can continue an item, so the walk starts at this wavefront's own first tile)
        int slot = 0;
        for (uint32_t pos = x0; pos > item_first; ++slot) pos -= len_of_wave(uw - 1 - (uint32_t)slot);
        // The lane id goes through an opaque move so that the per-lane address terms of the slot
        // marking and of the tile pipeline are recomputed for every segment instead of being kept
        // live across this loop, where they would not fit the register file.
        int lane_here = lane;
        asm volatile("" : "+v"(lane_here));
        if (j == 0) {                             // this wavefront begins the item
            // spans the item touches: this one and every later one that begins inside the item
            int n_seg = 1;
            for (uint32_t pos = x0 + my_len; pos < item_first + T; ++n_seg) pos += len_of_wave(uw + (uint32_t)n_seg);
            if (lane_here < a.G)
                for (int sl = n_seg; sl < a.n_ctx_slots; ++sl)
                    a.part_lse[(int64_t)(a.n_sys_chunks + sl) * a.rows + (int64_t)req * a.Hq +
                               g * a.G + lane_here] = -INFINITY;
        }
        Item it;
        it.g = g;
        it.key_begin = 32 * (int)j;
        it.key_end = min(c_req, 32 * (int)(j + seg));
        it.part_index = a.n_sys_chunks + slot;
        it.req = req;
        it.append_pos = APPEND && j + seg == T ? c_req - 1 : -1;   // (-1 for an empty context)
        it.mt = 0; it.tok0 = 0; it.ncols = a.G; it.k = nullptr; it.v = nullptr;
        attend<D, false, true, APPEND>(a, it, lane_here, smem, sm_m, sm_l, sm_tbl);   // rows are read once
        x += seg;
        if (x >= x1) break;
        j = 0;
        if (++g == a.Hkv) {
            g = 0;
            if (++req >= B) break;                // (x < x1 <= n_tiles, so this cannot happen)
            if (req - chunk_base >= kWave) {
                chunk_base += kWave;
                c_lane = len_of(chunk_base + lane);
            }
            c_req = __builtin_amdgcn_readlane(c_lane, req - chunk_base);
            T = tiles_of(c_req);
        }
    }
}

// ROWS: the system items are items of the many-rows kernel (128 stacked query rows share every
// K/V tile through LDS) instead of 32-row streaming items.  For wide grouped-query batches, where
// B*G stacked rows per kv head are many row tiles that would each pull the whole system K/V into
// their compute unit: what a unit can draw, from HBM or from L2, is the bound of this launch.
// APPEND: the context wavefronts also perform the cache write of the decode step (k_new / v_new).
template <int D, bool SYS_NT, bool MULTI, bool ROWS, bool APPEND>
__global__ __launch_bounds__(kThreads, 2) void relay_tile_kernel(const TileArgs a) {
    const unsigned long long t_begin = a.timeline ? __builtin_amdgcn_s_memrealtime() : 0ull;
    __shared__ __attribute__((aligned(1024))) unsigned char smem[kWaves * TileCfg<D>::SLICE];
    __shared__ float sm_m[kWaves][32];
    __shared__ float sm_l[kWaves][32];
    __shared__ int32_t sm_tbl[kWaves][kMaxPartBlocks];
    if ((int)blockIdx.x < a.n_sys_items) {
        if constexpr (ROWS) {
            static_assert(kWaves * TileCfg<D>::SLICE >= 2 * 2 * 64 * D * 2, "LDS for two 64-key steps of K and V");
            RowsArgs r{};
            r.q = a.q;
            r.k_sys = a.pfx_k[0];
            r.v_sys = a.pfx_v[0];
            r.part_o = a.part_o;
            r.part_lse = a.part_lse;
            r.q_stride_token = a.q_stride_token;
            r.q_stride_head = a.q_stride_head;
            r.sys_stride_token = a.sys_stride_token;
            r.sys_stride_head = a.sys_stride_head;
            r.n_tokens = a.n_tokens;
            r.Hq = a.Hq;
            r.Hkv = a.Hkv;
            r.G = a.G;
            r.sys_len = a.pfx_len[0];
            r.sys_chunk = a.sys_chunk;
            r.n_sys_chunks = a.n_sys_chunks;
            r.n_sys_rowblocks = a.n_sys_rowblocks;
            r.n_sys_items = a.n_sys_items;
            r.rows = a.rows;
            r.sys_head_fastest = a.sys_head_fastest;
            r.scale_log2 = a.scale_log2;
            rows_item<D, true>(r, (int)blockIdx.x, smem, &sm_tbl[0][0]);
        } else {
            run_system_item<D, SYS_NT, MULTI>(a, smem, sm_m, sm_l, sm_tbl);
        }
    } else {
        // Context wavefronts issue in short bursts between long waits for memory; at a raised
        // priority a burst is not queued behind the steady instruction stream of a system
        // workgroup on the same SIMD, which shortens the path every tile of the wavefront goes
        // through (grouped-query shape with many-rows system items 75 -> 71 us, Llama-30B shape at
        // a 2048-position prompt 34.2 -> 33.4 us).
        __builtin_amdgcn_s_setprio(3);
        run_context_wave<D, APPEND>(a, smem, sm_m, sm_l, sm_tbl);
    }
    if (a.timeline) {
        const unsigned w = blockIdx.x * kWaves + threadIdx.x / kWave;
        if (threadIdx.x % kWave == 0 && w < (unsigned)a.timeline_waves) {
            a.timeline[2 * w] = t_begin;
            a.timeline[2 * w + 1] = __builtin_amdgcn_s_memrealtime();
        }
    }
}

hipError_t launch_relay_tiles(const TileArgs &a, int head_dim, hipStream_t stream) {
    const int64_t groups = (int64_t)a.n_sys_items + a.ctx_waves / kWaves;
    if (groups == 0) return hipSuccess;
    if (groups > INT32_MAX) return hipErrorInvalidValue;
    // system rows are read once per launch only when all stacked queries fit one row tile
    const bool sys_nt = a.sys_read_once != 0;
    const dim3 grid((unsigned)groups), block(kThreads);
    const bool multi = a.n_prefixes > 1;
    const bool append = a.k_new != nullptr;
    if (append && multi) return hipErrorInvalidValue;          // (no entry point asks for it)
    const bool rows = a.n_sys_rowblocks > 0;                   // system items of the many-rows kind
    if (rows && multi) return hipErrorInvalidValue;
#define RA_LAUNCH(D_, NT_, MULTI_, ROWS_, APPEND_) \
    hipLaunchKernelGGL((relay_tile_kernel<D_, NT_, MULTI_, ROWS_, APPEND_>), grid, block, 0, stream, a)
#define RA_PICK(D_)                                                         \
    do {                                                                    \
        if (rows) {                                                         \
            if (append) RA_LAUNCH(D_, false, false, true, true);            \
            else RA_LAUNCH(D_, false, false, true, false);                  \
        } else if (append) {                                                \
            if (sys_nt) RA_LAUNCH(D_, true, false, false, true);            \
            else RA_LAUNCH(D_, false, false, false, true);                  \
        } else if (multi) {                                                 \
            if (sys_nt) RA_LAUNCH(D_, true, true, false, false);            \
            else RA_LAUNCH(D_, false, true, false, false);                  \
        } else {                                                            \
            if (sys_nt) RA_LAUNCH(D_, true, false, false, false);           \
            else RA_LAUNCH(D_, false, false, false, false);                 \
        }                                                                   \
    } while (0)
    if (head_dim == 128) RA_PICK(128);
    else if (head_dim == 64) RA_PICK(64);
    else return hipErrorInvalidValue;
#undef RA_PICK
#undef RA_LAUNCH
    return hipGetLastError();
}

}  // namespace ra
