// Split-KV block attention for the Orthrus dual-view decode step on gfx950 (Section 3.1, Eq. 4:
// O = Softmax(Q [K_AR || K_blk]^T * scale) [V_AR || V_blk]; diffusion view bidirectional inside
// the block, AR verification view causal inside the block).
//
// Work decomposition
//   grid  = (split, KV head g, sequence b); one workgroup of 4 wavefronts streams cache tokens
//           [split*chunk, min(L_b, (split+1)*chunk)) of KV head g once and serves all
//           R = G*K query rows that share that KV head (G query heads x K block rows).
//   wave  = owns NRB blocks of 32 query rows and every WT-th 32-token tile of the range.  Tiles
//           are wave-private: a wave streams its tile straight from global memory into its own
//           LDS slab (global_load_lds_dwordx4: coalesced 16-byte loads, one 256-byte row per 16
//           lanes, two stages so that the next tile is in flight while this one is computed) and
//           reads it back in MFMA operand order, so the main loop has no workgroup barrier.
//   MFMA  = v_mfma_f32_32x32x16_bf16 for both contractions, transposed problem:
//           S^T[token][row] = K_tile . Q^T   (A = K from LDS, B = Q held in registers)
//           O^T[d][row]    += V^T . P^T      (A = V through the LDS transpose read, B = P)
//           In both results a lane owns one query row (lane%32), so the online-softmax row
//           statistics are per-lane scalars and need a single cross-lane exchange (lane^32).
//   tail  = the block's own K/V rows form one more 32-token tile, masked per view, processed by
//           split 0.  Afterwards the waves of a workgroup merge their (max, sum, O) states through
//           LDS and either write the final bf16 rows (one split) or an fp32 partial that
//           attn_combine_kernel merges in a fixed split order (deterministic).
#include "orthrus_internal.h"

namespace orthrus {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(4))) int32_t const_i32;

union Frag {
    uint4 u;
    bf16x8 v;
    s16x4 h[2];
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

// LDS tile layout.  A wave-wide 16-byte direct load fills 1024 contiguous LDS bytes = one "group" of
// RPI consecutive K/V rows; groups are GS = 1040 bytes apart (the 16 bytes of padding rotate the
// banks from group to group).  Inside a group, row r keeps its 16-byte chunk c at slot c ^ xm(r),
// xm(r) = (r << 2) mod chunks-per-row, i.e. each row of a group starts in a different 64-byte bank
// window.  Both MFMA operand read patterns then spread over the banks: the K read (lanes = 32
// consecutive rows, same chunk) and the V transpose read (16 lanes = 4 rows x 32 bytes).  The
// permutation is applied on the global side (a lane fetches the chunk that belongs in its slot).
constexpr int kGroupStride = 1040;
template <int CH>
__device__ __forceinline__ int xm(int r)
{
    return (r << 2) & (CH - 1);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi)
{
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // v_cvt_pk_bf16_f32, RNE
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <int D, int NRB, int WR>
__global__ void __launch_bounds__(256) attn_split_kernel(const AttnArgs a)
{
    constexpr int WT = 4 / WR;         // wave groups along tokens
    constexpr int CH = D / 8;          // 16-byte chunks per K/V row
    constexpr int ROWB = D * 2;        // bytes per K/V row
    constexpr int RPI = 64 / CH;       // rows per group = tile rows fetched by one wave-wide 16-byte load
    constexpr int NI = 32 / RPI;       // groups (= such loads) per 32-token tile
    constexpr int GS = kGroupStride;   // LDS bytes between groups
    constexpr int TILE_B = NI * GS;    // one 32-token K (or V) tile in LDS
    constexpr int KSTEPS = D / 16;     // MFMA steps along d for S
    constexpr int DBLK = D / 32;       // 32-wide output blocks along d
    constexpr int OROW = D + 4;        // padded fp32 row of the merge buffer
    constexpr int RPW = NRB * 32;      // query rows per wave
    constexpr int RPAD = WR * RPW;     // padded query rows per workgroup

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wr = wave / WT, wt = wave % WT;
    const int col = lane & 31, h = lane >> 5;
    const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
    const int K = a.block_k, G = a.group;
    const int P = 1 << a.page_shift;

    int L = ((const const_i32 *)a.seq_lens)[b];
    if (L < 0 || L > a.max_seq_len) {
        if (tid == 0) atomicExch(a.err_word, -4);
        L = L < 0 ? 0 : a.max_seq_len;
    }
    const int t_begin = split * a.chunk_tokens;
    if (split > 0 && t_begin >= L) return;  // nothing of this sequence falls in the split
    const int t_end = min(L, t_begin + a.chunk_tokens);
    const int n_tiles = t_end > t_begin ? (t_end - t_begin + 31) >> 5 : 0;

    Frag qf[NRB][KSTEPS];  // filled after the first tile's loads are on their way
    int irow[NRB];
    f32x16 o[NRB][DBLK];
    float m_run[NRB], l_run[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        m_run[rb] = kNegBig;
        l_run[rb] = 0.f;
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[rb][db][r] = 0.f;
    }

    // two wave-private LDS stages, each a K tile followed by a V tile
    unsigned char *stage_base = smem + wave * (4 * TILE_B);
    const uint32_t stage_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)stage_base;
    const int ld_tok = lane / CH, ld_ch = lane % CH;  // this lane's (row, slot) inside one wave-wide load
    // The page table and lengths are read-only for the whole launch and every index used here is
    // wave-uniform: reading them through the constant address space makes these scalar loads
    // (s_load_dword), which keeps them off the vector-memory counter that paces the tile loads.
    const const_i32 *pt_row = (const const_i32 *)(a.page_table + (int64_t)b * a.max_pages_per_seq);
    const float c = a.scale_log2e;

    // Direct global->LDS load of 64 x 16 bytes: lane's bytes land at lds_addr + lane*16.  Issued
    // through inline assembly so that the wave can keep a whole tile in flight while it computes on
    // the other stage; completion is awaited explicitly with s_waitcnt vmcnt (loads return in order).
    // M0 carries the LDS destination; nothing else in this kernel reads M0, and the compiler
    // rewrites M0 itself right before any instruction of its own that needs it.
    auto dma16 = [&](const uint16_t *gp, uint32_t lds_addr) __attribute__((always_inline)) {
        asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                     :
                     : "v"(gp), "s"(lds_addr)
                     : "memory");
    };
    // page ids of the two 16-token halves of cache tile j (second = first when the half is past t_end)
    auto tile_pages = [&](int j, int &pg0, int &pg1) __attribute__((always_inline)) {
        const int ts = t_begin + j * 32;
        int p0 = pt_row[ts >> a.page_shift];
        int p1 = p0;
        if (ts + 16 < t_end) p1 = pt_row[(ts + 16) >> a.page_shift];
        if (p0 < 0 || p0 >= a.num_pages || p1 < 0 || p1 >= a.num_pages) {
            if (lane == 0) atomicExch(a.err_word, -4);
            if (p0 < 0 || p0 >= a.num_pages) p0 = 0;
            if (p1 < 0 || p1 >= a.num_pages) p1 = 0;
        }
        pg0 = p0;
        pg1 = p1;
    };
    // start the loads of cache tile j into stage st.  Rows past t_end repeat row t_end-1 (finite data,
    // masked later), so nothing is fetched through an unmapped page and no LDS row is left undefined.
    auto issue_cache = [&](int j, int st, int pg0, int pg1) __attribute__((always_inline)) {
        const int ts = t_begin + j * 32;
        const uint32_t kdst = stage_lds + st * (2 * TILE_B);
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int tok = u * RPI + ld_tok;
            const int tg = min(ts + tok, t_end - 1);
            const int p = (u * RPI < 16) ? pg0 : pg1;
            const int64_t off = (int64_t)p * a.stride_page + (int64_t)g * a.stride_head +
                                (int64_t)(tg & (P - 1)) * a.stride_tok + ((ld_ch ^ xm<CH>(ld_tok)) << 3);
            dma16(a.k_pool + off, kdst + u * GS);
            dma16(a.v_pool + off, kdst + TILE_B + u * GS);
        }
    };
    // the block's own K/V rows (rows >= K repeat row K-1)
    auto issue_block = [&](int st) __attribute__((always_inline)) {
        const uint32_t kdst = stage_lds + st * (2 * TILE_B);
#pragma unroll
        for (int u = 0; u < NI; ++u) {
            const int tok = u * RPI + ld_tok;
            const int64_t off = (((int64_t)b * K + min(tok, K - 1)) * a.num_kv_heads + g) * D +
                                ((ld_ch ^ xm<CH>(ld_tok)) << 3);
            dma16(a.k_blk + off, kdst + u * GS);
            dma16(a.v_blk + off, kdst + TILE_B + u * GS);
        }
    };

    // lane-invariant LDS read offsets (inside one stage)
    int kb[KSTEPS / 2];  // K operand: row `col`, chunks 4q'..4q'+3 where q' = q ^ (xm >> 2)
    {
        const int r = col % RPI;
#pragma unroll
        for (int q = 0; q < KSTEPS / 2; ++q)
            kb[q] = (col / RPI) * GS + r * ROWB + ((q ^ (xm<CH>(r) >> 2)) << 6) + (h << 4);
    }
    int vb[DBLK];  // V operand through the transpose read: lane supplies row 4*h + (lane%16)/4 (+8 per step)
    {
        const int tok0 = 4 * h + ((lane & 15) >> 2);
        const int r = tok0 % RPI;
        const int tr_ch = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);  // chunk inside the 32-wide d block
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
            vb[db] = TILE_B + (tok0 / RPI) * GS + r * ROWB + ((db ^ (xm<CH>(r) >> 2)) << 6) + (tr_ch << 4) +
                     ((lane & 1) << 3);
    }

    // one 32-token tile from LDS stage st.  lim[rb] = number of leading tile tokens this lane's row may see.
    auto compute = [&](int st, bool all_valid, const int (&lim)[NRB]) __attribute__((always_inline)) {
        const unsigned char *tile = stage_base + st * (2 * TILE_B);
        f32x16 s[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[rb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            Frag ka;
            ka.u = *(const uint4 *)(tile + kb[kk >> 1] + ((kk & 1) << 5));
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb)
                s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, qf[rb][kk].v, s[rb], 0, 0, 0);
        }
        Frag p1[NRB], p2[NRB];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (!all_valid) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int tok = 8 * (r >> 2) + 4 * h + (r & 3);  // S^T register r of this lane
                    if (tok >= lim[rb]) s[rb][r] = -INFINITY;
                }
            }
            float mx = s[rb][0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[rb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run[rb], mx * c);
            const float alpha = __builtin_amdgcn_exp2f(m_run[rb] - m_new);
            m_run[rb] = m_new;
            float p[16];
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(s[rb][r] * c - m_new);
                sum += p[r];
            }
            l_run[rb] = l_run[rb] * alpha + sum;
            p1[rb].u = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]),
                                  pack_bf16(p[6], p[7]));
            p2[rb].u = make_uint4(pack_bf16(p[8], p[9]), pack_bf16(p[10], p[11]), pack_bf16(p[12], p[13]),
                                  pack_bf16(p[14], p[15]));
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[rb][db][r] *= alpha;
        }
        // O^T += V^T P^T.  MFMA k-slot (h, j) of the first product is token 8*(j/4) + 4*h + j%4 (what
        // registers 0..7 of S^T hold); the second product is 16 tokens further.
#pragma unroll
        for (int db = 0; db < DBLK; ++db) {
            Frag va[2];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4)
                va[q4 >> 1].h[q4 & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (lds_s16x4 *)(tile + vb[db] + q4 * (8 / RPI) * GS));
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[0].v, p1[rb].v, o[rb][db], 0, 0, 0);
                o[rb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[1].v, p2[rb].v, o[rb][db], 0, 0, 0);
            }
        }
    };

    // ---- main loop: this wave's tiles are wt, wt+WT, ...; tile i+1 streams into the other LDS stage
    //      while tile i is computed.  Page ids are fetched one tile further ahead.
    const int my_tiles = n_tiles > wt ? (n_tiles - wt + WT - 1) / WT : 0;
    const bool do_block = (split == 0 && wt == 0);
    const int total = my_tiles + (do_block ? 1 : 0);  // the in-block tile is this wave's last one
    int pg0 = 0, pg1 = 0;
    if (my_tiles > 0) {
        tile_pages(wt, pg0, pg1);
        issue_cache(wt, 0, pg0, pg1);
        if (my_tiles > 1) tile_pages(wt + WT, pg0, pg1);
    } else if (do_block) {
        issue_block(0);
    }

    // ---- queries: B operand of S^T = K.Q^T, lane holds row `col`, d = 16*kk + 8*h .. +7
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int ridx = (wr * NRB + rb) * 32 + col;
        if (ridx < a.rows) {
            const int i = ridx / G, hl = ridx - i * G;
            irow[rb] = i;
            const uint16_t *qp = a.q + (((int64_t)b * K + i) * a.num_q_heads + (int64_t)g * G + hl) * D;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) qf[rb][kk].u = *(const uint4 *)(qp + kk * 16 + h * 8);
        } else {
            irow[rb] = 31;  // padding rows see every in-block key; their output is never stored
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) qf[rb][kk].u = make_uint4(0, 0, 0, 0);
        }
    }

    // Every vector load the compiler knows about (the queries) is waited for here, before the loop:
    // inside the loop only the hand-issued tile loads are outstanding, so the compiler adds no
    // vmcnt wait of its own there (such a wait would also drain the tile that is being prefetched).
    __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0), other counters untouched

    for (int i = 0; i < total; ++i) {
        const int st = i & 1;
        const int nx = i + 1;
        if (nx < total) {
            if (nx < my_tiles) {
                issue_cache(wt + nx * WT, st ^ 1, pg0, pg1);
                if (nx + 1 < my_tiles) tile_pages(wt + (nx + 1) * WT, pg0, pg1);
            } else {
                issue_block(st ^ 1);
            }
            asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * NI) : "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
        int lim[NRB];
        bool all_valid;
        if (i < my_tiles) {
            const int left = t_end - (t_begin + (wt + i * WT) * 32);
            all_valid = left >= 32;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) lim[rb] = left;
        } else {  // in-block tile: K rows, causal for the AR view
            all_valid = false;
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) lim[rb] = a.view == 0 ? K : min(K, irow[rb] + 1);
        }
        compute(st, all_valid, lim);
    }

    // ---- merge the WT wave states of each row group through LDS
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) l_run[rb] += __shfl_xor(l_run[rb], 32);
    __syncthreads();  // every wave is done with its tile slab; the slabs are reused below
    float *obuf = (float *)smem + (size_t)wave * RPW * OROW;
    float *mlbuf = (float *)smem + (size_t)4 * RPW * OROW;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r4 = 0; r4 < 4; ++r4) {
                float4 v = make_float4(o[rb][db][4 * r4], o[rb][db][4 * r4 + 1], o[rb][db][4 * r4 + 2],
                                       o[rb][db][4 * r4 + 3]);
                *(float4 *)(obuf + (rb * 32 + col) * OROW + 32 * db + 8 * r4 + 4 * h) = v;
            }
        if (h == 0) {
            mlbuf[(wave * RPW + rb * 32 + col) * 2] = m_run[rb];
            mlbuf[(wave * RPW + rb * 32 + col) * 2 + 1] = l_run[rb];
        }
    }
    __syncthreads();

    const int unit = b * a.num_kv_heads + g;
    for (int e = tid; e < RPAD * (D / 4); e += 256) {
        const int row = e / (D / 4), d4 = e % (D / 4);
        const int wrr = row / RPW, rl = row % RPW;
        float mw[WT], M = kNegBig;
#pragma unroll
        for (int w = 0; w < WT; ++w) {
            mw[w] = mlbuf[((wrr * WT + w) * RPW + rl) * 2];
            M = fmaxf(M, mw[w]);
        }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float lsum = 0.f;
#pragma unroll
        for (int w = 0; w < WT; ++w) {
            const float sc = __builtin_amdgcn_exp2f(mw[w] - M);
            const float4 v = *(const float4 *)((float *)smem + ((size_t)(wrr * WT + w) * RPW + rl) * OROW + d4 * 4);
            acc.x += sc * v.x; acc.y += sc * v.y; acc.z += sc * v.z; acc.w += sc * v.w;
            lsum += sc * mlbuf[((wrr * WT + w) * RPW + rl) * 2 + 1];
        }
        if (a.num_splits == 1) {
            if (row < a.rows) {
                const int i = row / G, hl = row - i * G;
                const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
                const int64_t orow = (((int64_t)b * K + i) * a.num_q_heads + (int64_t)g * G + hl);
                uint2 pk;
                pk.x = f32_to_bf16_rne(acc.x * inv) | ((uint32_t)f32_to_bf16_rne(acc.y * inv) << 16);
                pk.y = f32_to_bf16_rne(acc.z * inv) | ((uint32_t)f32_to_bf16_rne(acc.w * inv) << 16);
                *(uint2 *)(a.out + orow * D + d4 * 4) = pk;
                if (a.lse && d4 == 0)
                    a.lse[((int64_t)b * a.num_q_heads + (int64_t)g * G + hl) * K + i] =
                        (M + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
            }
        } else {
            const size_t prow = ((size_t)unit * a.num_splits + split) * RPAD + row;
            *(float4 *)(a.part_o + prow * D + d4 * 4) = acc;
            if (d4 == 0) {
                a.part_ml[prow * 2] = M;
                a.part_ml[prow * 2 + 1] = lsum;
            }
        }
    }
}

// Merge the per-split partials of one (sequence, KV head) in split order and write bf16 rows.
template <int D>
__global__ void __launch_bounds__(256) attn_combine_kernel(const AttnArgs a, int rows_padded)
{
    constexpr int GPR = D / 4;           // float4 groups per row
    constexpr int ROWS_PB = 256 / GPR;   // rows per workgroup
    const int unit = blockIdx.y;
    const int b = unit / a.num_kv_heads, g = unit % a.num_kv_heads;
    const int row = blockIdx.x * ROWS_PB + threadIdx.x / GPR;
    const int d4 = threadIdx.x % GPR;
    if (row >= a.rows) return;
    int L = a.seq_lens[b];
    L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
    int live = (L + a.chunk_tokens - 1) / a.chunk_tokens;
    live = live < 1 ? 1 : (live > a.num_splits ? a.num_splits : live);
    const size_t base = (size_t)unit * a.num_splits * rows_padded + row;
    float M = kNegBig;
    for (int s = 0; s < live; ++s) M = fmaxf(M, a.part_ml[(base + (size_t)s * rows_padded) * 2]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
    for (int s = 0; s < live; ++s) {
        const size_t prow = base + (size_t)s * rows_padded;
        const float sc = __builtin_amdgcn_exp2f(a.part_ml[prow * 2] - M);
        const float4 v = *(const float4 *)(a.part_o + prow * D + d4 * 4);
        acc.x += sc * v.x; acc.y += sc * v.y; acc.z += sc * v.z; acc.w += sc * v.w;
        lsum += sc * a.part_ml[prow * 2 + 1];
    }
    const int G = a.group, K = a.block_k;
    const int i = row / G, hl = row - i * G;
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    const int64_t orow = (((int64_t)b * K + i) * a.num_q_heads + (int64_t)g * G + hl);
    uint2 pk;
    pk.x = f32_to_bf16_rne(acc.x * inv) | ((uint32_t)f32_to_bf16_rne(acc.y * inv) << 16);
    pk.y = f32_to_bf16_rne(acc.z * inv) | ((uint32_t)f32_to_bf16_rne(acc.w * inv) << 16);
    *(uint2 *)(a.out + orow * D + d4 * 4) = pk;
    if (a.lse && d4 == 0)
        a.lse[((int64_t)b * a.num_q_heads + (int64_t)g * G + hl) * K + i] =
            (M + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
}

// ---------------------------------------------------------------------------------------------
// host side

template <int D, int NRB, int WR>
static size_t lds_need()
{
    const size_t tiles = (size_t)4 * 4 * (32 / (64 / (D / 8))) * kGroupStride;  // 4 waves x 2 stages x (K + V tile)
    const size_t merge = (size_t)4 * NRB * 32 * (D + 4) * 4 + (size_t)4 * NRB * 32 * 2 * 4;
    return tiles > merge ? tiles : merge;
}

hipError_t plan_attn(int head_dim, int group, int block_k, int batch, int num_kv_heads, int max_seq_len,
                     int requested_splits, int num_cus, AttnPlan *plan)
{
    const int R = group * block_k;
    plan->rows = R;
    if (R <= 32) { plan->nrb_wave = 1; plan->wr = 1; }
    else if (R <= 64) { plan->nrb_wave = 2; plan->wr = 1; }
    else if (R <= 128) { plan->nrb_wave = 2; plan->wr = 2; }
    else { plan->nrb_wave = 2; plan->wr = 4; }
    plan->rows_padded = plan->wr * plan->nrb_wave * 32;
    const int wt = 4 / plan->wr;
    const int gran = 32 * wt;  // every wave of a token group gets whole tiles
    const int64_t units = (int64_t)batch * num_kv_heads;
    int splits;
    if (requested_splits > 0) {
        splits = requested_splits;
    } else {
        // enough workgroups for ~2 per CU, but never less than 512 tokens per split
        const int64_t want = ((int64_t)2 * num_cus + units - 1) / (units > 0 ? units : 1);
        const int64_t by_len = (max_seq_len + 511) / 512;
        splits = (int)(want < by_len ? want : by_len);
        if (splits < 1) splits = 1;
    }
    int chunk = (max_seq_len + splits - 1) / splits;
    chunk = ((chunk + gran - 1) / gran) * gran;
    if (chunk < gran) chunk = gran;
    splits = max_seq_len > 0 ? (max_seq_len + chunk - 1) / chunk : 1;
    if (splits < 1) splits = 1;
    plan->chunk_tokens = chunk;
    plan->num_splits = splits;
    const int nrb = plan->nrb_wave;
    if (head_dim == 128) plan->lds_bytes = nrb == 1 ? lds_need<128, 1, 1>() : lds_need<128, 2, 1>();
    else plan->lds_bytes = nrb == 1 ? lds_need<64, 1, 1>() : lds_need<64, 2, 1>();
    if (splits > 1) {
        plan->part_o_bytes = (size_t)units * splits * plan->rows_padded * head_dim * sizeof(float);
        plan->part_ml_bytes = (size_t)units * splits * plan->rows_padded * 2 * sizeof(float);
    } else {
        plan->part_o_bytes = plan->part_ml_bytes = 0;
    }
    return hipSuccess;
}

template <int D, int NRB, int WR>
static hipError_t launch_split(const AttnArgs &a, const AttnPlan &plan, hipStream_t stream)
{
    auto kern = attn_split_kernel<D, NRB, WR>;
    static bool attr_set = false;  // the attribute belongs to the function, one process-wide set is enough
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)lds_need<D, NRB, WR>());
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(plan.num_splits, a.num_kv_heads, a.batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), plan.lds_bytes, stream, a);
    return hipGetLastError();
}

hipError_t launch_attn(const AttnArgs &a, const AttnPlan &plan, int head_dim, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    hipError_t e = hipErrorInvalidValue;
    const int key = plan.nrb_wave * 10 + plan.wr;
    if (head_dim == 128) {
        if (key == 11) e = launch_split<128, 1, 1>(a, plan, stream);
        else if (key == 21) e = launch_split<128, 2, 1>(a, plan, stream);
        else if (key == 22) e = launch_split<128, 2, 2>(a, plan, stream);
        else if (key == 24) e = launch_split<128, 2, 4>(a, plan, stream);
    } else if (head_dim == 64) {
        if (key == 11) e = launch_split<64, 1, 1>(a, plan, stream);
        else if (key == 21) e = launch_split<64, 2, 1>(a, plan, stream);
        else if (key == 22) e = launch_split<64, 2, 2>(a, plan, stream);
        else if (key == 24) e = launch_split<64, 2, 4>(a, plan, stream);
    }
    if (e != hipSuccess) return e;
    if (plan.num_splits > 1) {
        const int units = a.batch * a.num_kv_heads;
        if (head_dim == 128) {
            dim3 grid((a.rows + 7) / 8, units);
            hipLaunchKernelGGL(attn_combine_kernel<128>, grid, dim3(256), 0, stream, a, plan.rows_padded);
        } else {
            dim3 grid((a.rows + 15) / 16, units);
            hipLaunchKernelGGL(attn_combine_kernel<64>, grid, dim3(256), 0, stream, a, plan.rows_padded);
        }
        e = hipGetLastError();
    }
    return e;
}

}  // namespace orthrus
