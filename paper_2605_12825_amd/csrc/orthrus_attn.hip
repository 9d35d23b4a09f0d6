// Split-KV block attention for the Orthrus dual-view decode step on gfx950 (Section 3.1, Eq. 4:
// O = Softmax(Q [K_AR || K_blk]^T * scale) [V_AR || V_blk]; diffusion view bidirectional inside
// the block, AR verification view causal inside the block).
//
// Work decomposition
//   grid   = one workgroup per (split, KV head g, sequence b).  A workgroup streams its piece of the
//            cache tokens of KV head g once (the sequence's own tiles, the in-block tile included, dealt
//            out evenly to the splits: split_cut) and serves all R = G*K
//            query rows that share that KV head (G query heads x K block rows).
//            Workgroups are numbered with the sequence index fastest and the KV head slowest
//            (consecutive ids go to different XCDs; see the kernel).
//   waves  = W compute waves per workgroup, one per block of 32 query rows (W = 1 .. 8), plus
//            one loader wave.  Every compute wave reads every K/V tile, so the tile stream is shared:
//            the loader sends 32-token tiles from global memory straight into an NS-stage LDS ring
//            (global_load_lds_dwordx4: coalesced 16-byte loads, one 256-byte row per 16 lanes), NS-1
//            tiles ahead of the one being computed, with one workgroup barrier per tile.  For a
//            launch that can fill the chip the plan lands on one workgroup per CU: that keeps ~32 KB
//            in flight per CU, which already saturates HBM, and shares the bandwidth evenly between
//            the XCDs (with twice as much in flight some XCDs finish 20 % later than others); a
//            smaller launch trades the length of a workgroup's tile chain against the cost of more
//            pieces (plan_attn).
//   MFMA   = v_mfma_f32_32x32x16_bf16 for both contractions, on the transposed problem:
//            S^T[token][row] = K_tile . Q^T   (A = K from LDS, B = Q held in registers)
//            O^T[d][row]    += V^T . P^T      (A = V through the LDS transpose read, B = P)
//            In both results a lane owns one query row (lane%32), so the online-softmax row
//            statistics are per-lane scalars and need a single cross-lane exchange (lane^32).
//   tail   = the block's own K/V rows form one more 32-token tile, masked per view, processed by
//            the unit's last piece.  A wave owns its rows outright, so there is no merge inside the workgroup:
//            it writes final bf16 rows (one split) or an fp32 partial in register order that
//            attn_combine_kernel merges in a fixed split order (deterministic).
//   other forms of the same kernel: the balanced partition of a ragged batch's tiles over the
//            resident workgroups (template flag BALANCED) and the AR view's causal prefill (PREFILL);
//            both are described at the kernel.
//   caches = K/V tiles are read once per call.  When the model streams more K/V between two passes
//            over the same cache than the last-level cache holds, the tile loads carry the
//            non-temporal hint and the fp32 partials leave with non-temporal stores.
#include "orthrus_internal.h"

#include <hip/hip_ext.h>

#include <type_traits>

#pragma clang diagnostic ignored "-Winline-asm"  // the direct-to-LDS loads below name M0 as clobbered

namespace orthrus {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(4))) int32_t const_i32;

union Frag {
    uint4 u;
    bf16x8 v;
    s16x4 h[2];
    u32x4 n;
};

// LDS tile layout.  A wave-wide 16-byte direct load fills 1024 contiguous LDS bytes = one "group" of
// RPI consecutive K/V rows; groups are GS = 1040 bytes apart (the 16 bytes of padding rotate the
// banks from group to group).  Inside a group, row r keeps its 16-byte chunk c at slot c ^ xm(r),
// xm(r) = (r << 2) mod chunks-per-row, i.e. each row of a group starts in a different 64-byte bank
// window.  Both MFMA operand read patterns then spread over the banks: the K read (lanes = 32
// consecutive rows, same chunk) and the V transpose read (16 lanes = 4 rows x 32 bytes).  The
// permutation is applied on the global side (a lane fetches the chunk that belongs in its slot).
constexpr int kGroupStride = 1040;
constexpr float kLazy = 8.0f;  // log2 of the largest exponential the lazy softmax reference allows
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

// Combine a value with the one held by lane ^ 32 (the other half-wave) without going through LDS:
// v_permlane32_swap exchanges the upper half of one register with the lower half of another.
__device__ __forceinline__ float max_with_other_half(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Plain workgroup barrier.  Tile loads are tracked by hand (vmcnt), LDS traffic of the compiler's own
// instructions is complete once their results were consumed; the empty asm statements keep the
// compiler from moving memory operations across the barrier.
__device__ __forceinline__ void wg_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The tiles of one (sequence, KV head) unit, cache tiles of 32 tokens followed by the in-block tile, dealt
// out to `splits` pieces as evenly as whole tiles allow: the first `rem` pieces get one tile more, pieces
// past the tile count get nothing, and the in-block tile (the unit's last) lands in the last piece that
// has any.  A launch ends with its longest piece and the others cannot make up for it (a lone CU streams
// no faster when its neighbours are done), so one tile of imbalance costs a whole tile's time.
struct SplitCut {
    int first;  // first tile of the piece (tile index in the unit)
    int count;  // tiles in it, the in-block tile included if it is the unit's last piece
    int live;   // pieces of this unit that have any tile
};
__host__ __device__ __forceinline__ SplitCut split_cut(int L, int splits, int split)
{
    const int total = ((L + 31) >> 5) + 1;  // cache tiles + the in-block tile
    const int per = total / splits, rem = total - per * splits;
    SplitCut c;
    c.first = split * per + (split < rem ? split : rem);
    c.count = per + (split < rem ? 1 : 0);
    c.live = total < splits ? total : splits;
    return c;
}

template <int D>
struct AttnGeom {
    static constexpr int CH = D / 8;          // 16-byte chunks per K/V row
    static constexpr int ROWB = D * 2;        // bytes per K/V row
    static constexpr int RPI = 64 / CH;       // rows per group = rows fetched by one wave-wide 16-byte load
    static constexpr int NI = 32 / RPI;       // groups (= such loads) per 32-token K (or V) tile
    static constexpr int GS = kGroupStride;   // LDS bytes between groups
    static constexpr int TILE_B = NI * GS;    // one 32-token K (or V) tile in LDS
    static constexpr int STAGE_B = 2 * TILE_B;
    static constexpr int KSTEPS = D / 16;     // MFMA steps along d for S
    static constexpr int DBLK = D / 32;       // 32-wide output blocks along d
};

// D head_dim, W compute waves (= 32-row blocks) per workgroup, NS LDS stages.
//
// A workgroup has W compute waves and one loader wave that issues every tile load and does nothing
// else.  A wave that issues global->LDS loads is held up while the memory pipeline takes them
// (streaming 2 MB per CU costs the issuing wave about as long as the arithmetic on it costs a compute
// wave), so when compute waves issue their own loads the two costs add up; with a dedicated loader
// wave they overlap.  The register budget is 168 (three waves per SIMD), so W + 1 <= 9 waves fit a CU;
// the balanced form spills a dozen values that live across segments, outside the tile loop.
//
// PREFILL = 1 turns the same kernel into the AR view's causal prefill attention (Section 3.1): the new
// tokens' K/V rows are already in the cache, a work item is (sequence, chunk of 32 new tokens, KV head),
// its R = 32*G rows are the chunk's tokens times the G query heads, row (token i) sees cache tokens
// 0 .. L+i (its own position included), and there is no staged block tile and no split.
//
// BALANCED = 1 (decode only) replaces the fixed (sequence, split, head) grid by an even partition of
// the whole launch's tile sequence: the tiles of all (head, sequence) units, cache tiles then the
// in-block tile, are laid end to end (head-major), and workgroup w of the N launched takes tiles
// [w*T/N, (w+1)*T/N).  A workgroup's range is cut into segments at unit boundaries; a segment that
// covers its whole unit writes final rows, any other writes a partial (slot 2w when it starts inside
// the unit, 2w+1 when it starts at the unit's first tile: a range holds at most one of each), which
// attn_combine_kernel finds again from the same arithmetic.  With ragged lengths every workgroup
// still gets the same number of tiles, and with N = resident workgroups nothing queues behind
// the dispatcher.  Each segment runs the pipeline from empty (fill, loop, drain).
//
// PROBE = 1 is the measurement form behind orthrus_kv_stream_probe: the loader wave streams exactly the
// tiles of the call, the compute waves only keep the barriers (no queries, no arithmetic, nothing is
// written), so the launch takes as long as this kernel's K/V stream alone.
template <int D, int W, int NS, int PREFILL = 0, int BALANCED = 0, int PROBE = 0>
__global__ void __launch_bounds__(64 * (W + 1), 3) attn_split_kernel(const AttnArgs a)
{
    static_assert(!(PREFILL && BALANCED), "the balanced partition is a decode mode");
    static_assert(!PROBE || (W == 1 && !PREFILL), "the stream probe is a decode-mode kernel with one idle compute wave");
    using Gm = AttnGeom<D>;
    constexpr int CH = Gm::CH, ROWB = Gm::ROWB, RPI = Gm::RPI, NI = Gm::NI, GS = Gm::GS;
    constexpr int TILE_B = Gm::TILE_B, STAGE_B = Gm::STAGE_B, KSTEPS = Gm::KSTEPS, DBLK = Gm::DBLK;
    constexpr int LPT = 2 * NI;  // load instructions per tile (K groups then V groups), all by the loader wave
    static_assert(NS >= 2 && NS <= 4, "stage count");
    static_assert((NS - 2) * LPT < 64, "outstanding loads must fit the vmcnt field");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave == W;
    const int col = lane & 31, h = lane >> 5;
    const int K = a.block_k, G = a.group;
    const int P = 1 << a.page_shift;

    // The work item (balanced mode: the current segment) as every wave of the workgroup sees it.
    // Lengths and the page table are read-only for the whole launch and every index used here is
    // wave-uniform: reading them through the constant address space makes these scalar loads
    // (s_load_dword), which keeps them off the vector-memory counter that paces the tile loads.
    int b, g;
    int t_begin, t_end, n_cache, n_tiles;  // cache tokens [t_begin, t_end) in n_cache tiles; n_tiles adds the in-block tile
    bool final_out;                        // this item holds every tile of its unit: write finished rows
    size_t part_slot = 0;                  // else: index of the partial it writes
    int row0 = 0, rows_live = K;  // prefill: first new-token index of the chunk, tokens in it; pos0 below
    int pos0 = 0;                 // prefill: cache position of the chunk's first token
    const const_i32 *pt_row;
    int64_t head_off;

    // validated length of sequence x (scalar)
    auto seq_len = [&](int x) __attribute__((always_inline)) {
        int L = ((const const_i32 *)a.seq_lens)[x];
        if (L < 0 || L > a.max_seq_len) {
            if (tid == 0) atomicExch(a.err_word, -4);
            L = L < 0 ? 0 : a.max_seq_len;
        }
        return __builtin_amdgcn_readfirstlane(L);  // wave-uniform by construction; keeps the loop control scalar
    };

    // balanced mode: position in the launch's tile sequence
    int bal_b = 0, bal_g = 0, bal_o = 0, bal_left = 0;
    if constexpr (BALANCED) {
        // tiles of sequence x as a lane sees it (cache tiles + the in-block tile), 0 past the batch
        auto lane_tiles = [&](int x) __attribute__((always_inline)) {
            if (x >= a.batch) return 0;
            int L = a.seq_lens[x];
            L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
            return ((L + 31) >> 5) + 1;
        };
        int per_head = 0;  // tiles of one head's units
        for (int x0 = 0; x0 < a.batch; x0 += 64) {
            int n = lane_tiles(x0 + lane);
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off);
            per_head += n;
        }
        per_head = __builtin_amdgcn_readfirstlane(per_head);
        const int64_t total = (int64_t)per_head * a.num_kv_heads;
        const int64_t nwg = total < (int64_t)gridDim.x ? total : (int64_t)gridDim.x;
        if ((int64_t)blockIdx.x >= nwg) return;
        const int64_t c0 = (int64_t)blockIdx.x * total / nwg, c1 = ((int64_t)blockIdx.x + 1) * total / nwg;
        bal_left = __builtin_amdgcn_readfirstlane((int)(c1 - c0));
        bal_g = __builtin_amdgcn_readfirstlane((int)(c0 / per_head));
        const int r = (int)(c0 - (int64_t)bal_g * per_head);
        // the sequence whose tiles contain offset r of the head: inclusive scan over 64 sequences at a time
        int base = 0;
        for (int x0 = 0; x0 < a.batch; x0 += 64) {
            const int n = lane_tiles(x0 + lane);
            int incl = n;
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            const bool hit = n > 0 && base + incl - n <= r && r < base + incl;
            const uint64_t mask = __ballot(hit);
            if (mask) {
                const int src = __builtin_ctzll(mask);
                bal_b = x0 + src;
                bal_o = r - (base + __shfl(incl - n, src));
                break;
            }
            base += __shfl(incl, 63);
        }
        bal_b = __builtin_amdgcn_readfirstlane(bal_b);
        bal_o = __builtin_amdgcn_readfirstlane(bal_o);
    }

    // Opens the next work item; false when the workgroup has none (left).
    auto open_item = [&]() __attribute__((always_inline)) -> bool {
        if constexpr (BALANCED) {
            if (bal_left <= 0) return false;
            b = bal_b;
            g = bal_g;
            const int L = seq_len(b);
            const int nc = (L + 31) >> 5;                    // cache tiles of the unit; the in-block tile is tile nc
            const int take = min(nc + 1 - bal_o, bal_left);  // tiles of this segment
            const bool has_blk = bal_o + take == nc + 1;
            // (everything here is wave-uniform; readfirstlane keeps it in scalar registers)
            n_tiles = __builtin_amdgcn_readfirstlane(take);
            n_cache = has_blk ? n_tiles - 1 : n_tiles;
            t_begin = __builtin_amdgcn_readfirstlane(bal_o * 32);
            t_end = min(L, t_begin + n_cache * 32);
            final_out = bal_o == 0 && has_blk;
            part_slot = (size_t)(blockIdx.x * 2u + (bal_o == 0 ? 1u : 0u));
            bal_left = __builtin_amdgcn_readfirstlane(bal_left - take);
            bal_o = 0;
            int nb = bal_b + 1, ng = bal_g;
            if (nb == a.batch) {
                nb = 0;
                ++ng;
            }
            bal_b = __builtin_amdgcn_readfirstlane(nb);
            bal_g = __builtin_amdgcn_readfirstlane(ng);
        } else {
            // Workgroup id -> (sequence, split, KV head) with the sequence index fastest and the head
            // slowest.  Consecutive workgroup ids go to different XCDs; a head's rows sit at a fixed
            // offset inside every page, so an order that ties XCD k to head k makes each XCD hammer its
            // own subset of the HBM channels and the XCDs finish far apart.  (Prefill: the middle index
            // is the chunk, longest first.)
            b = (int)(blockIdx.x % (unsigned)a.batch);
            const int split = (int)((blockIdx.x / (unsigned)a.batch) % (unsigned)a.num_splits);
            g = (int)(blockIdx.x / ((unsigned)a.batch * (unsigned)a.num_splits));
            if constexpr (PREFILL) {
                // lengths as the planning kernel left them: validated, 0 new tokens on a capacity error
                const int L0 = __builtin_amdgcn_readfirstlane(((const const_i32 *)a.old_lens)[b]);
                const int n_new = __builtin_amdgcn_readfirstlane(((const const_i32 *)a.new_lens)[b]);
                const int chunk = a.num_splits - 1 - split;  // the chunks with the most cache tokens start first
                row0 = chunk * 32;
                if (row0 >= n_new) return false;
                rows_live = min(32, n_new - row0);
                pos0 = L0 + row0;
                t_begin = 0;
                t_end = pos0 + rows_live;  // everything up to the chunk's last token
                n_cache = (t_end + 31) >> 5;
                n_tiles = n_cache;
                final_out = true;
            } else {
                const int L = seq_len(b);
                // The sequence's own length, not the host's bound on it, is cut into num_splits pieces:
                // they stay equal however loose the bound is (it only sized the grid), e.g. when a
                // decode loop bumps it by K per step without reading back.
                const SplitCut cut = split_cut(L, a.num_splits, split);
                if (cut.count == 0) return false;  // fewer tiles than splits: nothing falls in this one
                n_tiles = __builtin_amdgcn_readfirstlane(cut.count);
                n_cache = split == cut.live - 1 ? n_tiles - 1 : n_tiles;  // the last piece ends with the in-block tile
                t_begin = __builtin_amdgcn_readfirstlane(cut.first * 32);
                t_end = min(L, t_begin + n_cache * 32);
                final_out = a.num_splits == 1;
                part_slot = ((size_t)b * a.num_kv_heads + g) * a.num_splits + split;
            }
        }
        pt_row = (const const_i32 *)(a.page_table + (int64_t)b * a.max_pages_per_seq);
        head_off = (int64_t)g * a.stride_head;
        return true;
    };
    if (!open_item()) return;

    const uint32_t smem_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)smem;
    const int ld_tok = lane / CH, ld_ch = lane % CH;  // this lane's (row, slot) inside one wave-wide load

    // Direct global->LDS load of 64 x 16 bytes: lane's bytes land at lds_addr + lane*16.  Issued
    // through inline assembly so that whole tiles can stay in flight while older ones are computed;
    // completion is awaited explicitly with s_waitcnt vmcnt (loads return in order).  M0 carries the
    // LDS destination and is declared clobbered, so the compiler never carries a value of its own in M0
    // across one of these statements (M0 is a reserved register, which clang remarks on for any clobber
    // list that names it; the remark is switched off for this file).  Two address forms: a 64-bit
    // address per lane, or a wave-uniform 64-bit base plus a 32-bit byte offset per lane.
    //
    // a.kv_nt selects the non-temporal form of the loads: when one call streams more K/V than the
    // last-level cache holds, nothing of it is there for the next call anyway, and loads that do not
    // allocate on their way stream ~7 % faster (measured); a working set that fits keeps the plain
    // form, so that the second view's pass over the same cache still finds it.
    // The choice is made once per wave (two copies of the loader's loop), not per load.
    auto dma16 = [&](auto nt, const uint16_t *gp, uint32_t lds_addr) __attribute__((always_inline)) {
        if constexpr (decltype(nt)::value)
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                         :
                         : "v"(gp), "s"(lds_addr)
                         : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                         :
                         : "v"(gp), "s"(lds_addr)
                         : "memory", "m0");
    };
    auto dma16s = [&](auto nt, const uint16_t *base, uint32_t voff, uint32_t lds_addr) __attribute__((always_inline)) {
        if constexpr (decltype(nt)::value)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt"
                         :
                         : "v"(voff), "s"(base), "s"(lds_addr)
                         : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :
                         : "v"(voff), "s"(base), "s"(lds_addr)
                         : "memory", "m0");
    };

    // Page ids of the two 16-token halves of cache tile t (the second repeats the first when that
    // half lies past the end).  They are fetched one tile ahead of their use, so that the scalar
    // load's latency is never in front of a tile's loads.
    auto fetch_pages = [&](int t, int &p0, int &p1) __attribute__((always_inline)) {
        p0 = 0;
        p1 = 0;
        if (t < n_cache) {
            const int ts = t_begin + t * 32;
            p0 = pt_row[ts >> a.page_shift];
            p1 = p0;
            if (ts + 16 < t_end) p1 = pt_row[(ts + 16) >> a.page_shift];
        }
    };
    // Start the loads of tile t (cache tile, or the in-block tile when
    // t == n_cache) into ring stage t % NS.  A full cache tile takes the cheap address form: page, head
    // and row group go into a wave-uniform base (scalar arithmetic), the lane adds one loop-invariant
    // byte offset.  In the last, ragged cache tile rows past the end repeat the last valid row (finite
    // data, masked later): nothing is fetched through an unmapped page and no LDS row is left
    // undefined; that tile and the in-block tile compute an address per lane.
    const uint32_t lane_off = (uint32_t)(ld_tok * (int)a.stride_tok + ((ld_ch ^ xm<CH>(ld_tok)) << 3)) * 2u;
    auto issue_tile = [&](auto nt, int t, int p0, int p1) __attribute__((always_inline)) {
        const uint32_t dst = smem_lds + (t % NS) * STAGE_B;
        if (t < n_cache) {
            const int ts = t_begin + t * 32;
            if (p0 < 0 || p0 >= a.num_pages || p1 < 0 || p1 >= a.num_pages) {
                if (lane == 0) atomicExch(a.err_word, -4);
                if (p0 < 0 || p0 >= a.num_pages) p0 = 0;
                if (p1 < 0 || p1 >= a.num_pages) p1 = 0;
            }
            if (ts + 32 <= t_end) {
                const int tsp = ts & (P - 1);
#pragma unroll
                for (int e = 0; e < LPT; ++e) {
                    const int id = e;               // 0..LPT-1: K groups, then V groups
                    const int u = id % NI;
                    const int page = (u * RPI < 16) ? p0 : p1;
                    const int tin = (tsp + u * RPI) & (P - 1);
                    const int64_t soff = (int64_t)page * a.stride_page + head_off + (int64_t)tin * a.stride_tok;
                    dma16s(nt, (id < NI ? a.k_pool : a.v_pool) + soff, lane_off, dst + (id < NI ? 0 : TILE_B) + u * GS);
                }
            } else {
#pragma unroll
                for (int e = 0; e < LPT; ++e) {
                    const int id = e;
                    const int u = id % NI;
                    const uint16_t *pool = id < NI ? a.k_pool : a.v_pool;
                    const int tok = u * RPI + ld_tok;
                    const int tg = min(ts + tok, t_end - 1);
                    const int p = (u * RPI < 16) ? p0 : p1;
                    const int64_t off = (int64_t)p * a.stride_page + (int64_t)g * a.stride_head +
                                        (int64_t)(tg & (P - 1)) * a.stride_tok + ((ld_ch ^ xm<CH>(ld_tok)) << 3);
                    dma16(nt, pool + off, dst + (id < NI ? 0 : TILE_B) + u * GS);
                }
            }
        } else if constexpr (!PROBE) {  // (the stream probe has no block inputs: its in-block tile stays empty)
#pragma unroll
            for (int e = 0; e < LPT; ++e) {
                const int id = e;
                const int u = id % NI;
                const uint16_t *blk = id < NI ? a.k_blk : a.v_blk;
                const int tok = u * RPI + ld_tok;
                const int64_t off = ((int64_t)b * K + min(tok, K - 1)) * a.blk_stride_row + (int64_t)g * a.blk_stride_head +
                                    ((ld_ch ^ xm<CH>(ld_tok)) << 3);
                dma16(nt, blk + off, dst + (id < NI ? 0 : TILE_B) + u * GS);
            }
        }
    };

    // One step of the load pipeline, run by the loader wave once per tile i, around the tile's workgroup
    // barrier: before the barrier the loads of tile i are complete; after it every compute wave is done
    // reading stage (i-1) % NS, which is refilled with tile i+NS-1 while tile i is computed.
    int np0 = 0, np1 = 0;  // page ids of the next tile to be issued
    auto pipeline_fill = [&](auto nt) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) {
            fetch_pages(t, np0, np1);
            if (t < n_tiles) issue_tile(nt, t, np0, np1);
        }
        fetch_pages(NS - 1, np0, np1);
    };
    auto pipeline_step = [&](auto nt, int i) __attribute__((always_inline)) {
        const int ahead = min(NS - 2, n_tiles - 1 - i);  // tiles issued after tile i so far
        if (ahead >= 2) wait_vmcnt<2 * LPT>();
        else if (ahead == 1) wait_vmcnt<LPT>();
        else wait_vmcnt<0>();
        wg_barrier();
        if (i + NS - 1 < n_tiles) issue_tile(nt, i + NS - 1, np0, np1);
        fetch_pages(i + NS, np0, np1);
    };

    if (loader) {
        // the loader wave: nothing but the load pipeline; its last wait leaves no load outstanding
        auto run = [&](auto nt) __attribute__((always_inline)) {
            for (;;) {
                pipeline_fill(nt);
                for (int i = 0; i < n_tiles; ++i) pipeline_step(nt, i);
                if (!BALANCED || !open_item()) break;
                wg_barrier();  // every compute wave is done with the previous segment's last tile
            }
        };
        if (a.kv_nt) run(std::true_type{});
        else run(std::false_type{});
        return;
    }

    // ---- compute waves
    if constexpr (PROBE) {
        for (;;) {
            for (int i = 0; i < n_tiles; ++i) wg_barrier();
            if (!BALANCED || !open_item()) break;
            wg_barrier();
        }
        return;
    }
    // lane-invariant LDS read offsets inside one stage
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

    const float c = a.scale_log2e;
    for (;;) {  // one pass per work item (balanced mode: per segment)
        // Queries: B operand of S^T = K.Q^T, lane holds row `col` of this wave's block,
        // d = 16*kk + 8*h .. +7 (fetched while the loader's first tiles are in flight)
        Frag qf[KSTEPS];
        int irow;
        const int ridx = wave * 32 + col;
        // the lane's row exists: inside the R rows and, for prefill, inside the chunk's live tokens
        const bool row_ok = ridx < a.rows && (!PREFILL || ridx / G < rows_live);
        // row of q / out that holds block row (or new token) i of this sequence
        const int64_t row_base = PREFILL ? (int64_t)b * a.max_new + row0 : (int64_t)b * K;
        if (row_ok) {
            const int i = ridx / G, hl = ridx - i * G;
            irow = i;
            const uint16_t *qp = a.q + (row_base + i) * a.q_stride_row + ((int64_t)g * G + hl) * a.q_stride_head;
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) qf[kk].u = *(const uint4 *)(qp + kk * 16 + h * 8);
        } else {
            irow = 31;  // padding rows see every in-block key; their output is never stored
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) qf[kk].u = make_uint4(0, 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): the queries are in registers before the loop starts

        f32x16 o[DBLK];
#pragma unroll
        for (int db = 0; db < DBLK; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
        float m_run = kNegBig, l_run = 0.f;

        // ---- main loop: one barrier per tile
        int stage = 0;  // ring slot of tile i (= i % NS)
        for (int i = 0; i < n_tiles; ++i) {
            wg_barrier();

            // LDS addresses of this tile's operands: one add per base, the rest are instruction offsets
            const uint32_t st_addr = smem_lds + (uint32_t)stage * STAGE_B;
            stage = stage + 1 == NS ? 0 : stage + 1;
            uint32_t ka[KSTEPS / 2], va_[DBLK];
#pragma unroll
            for (int q = 0; q < KSTEPS / 2; ++q) ka[q] = st_addr + kb[q];
#pragma unroll
            for (int db = 0; db < DBLK; ++db) va_[db] = st_addr + vb[db];
            // lim = number of leading tile tokens this lane's row may see
            int lim = 32;
            if (i < n_cache) lim = t_end - (t_begin + i * 32);
            else lim = a.view == 0 ? K : min(K, irow + 1);  // in-block tile: K rows, causal for the AR view
            if constexpr (PREFILL) lim = min(lim, pos0 + irow + 1 - i * 32);  // causal: tokens up to the row's own

            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
            Frag kf[KSTEPS];  // all K operand reads are issued before the first product needs one
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) kf[kk].n = *(const lds_u32x4 *)(uintptr_t)(ka[kk >> 1] + ((kk & 1) << 5));
            __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the products (the scheduler would pair them up)
#pragma unroll
            for (int kk = 0; kk < KSTEPS; ++kk) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kk].v, qf[kk].v, s, 0, 0, 0);
            // first half of the V operand reads goes out now, so that their latency hides behind the softmax
            constexpr int VPRE = DBLK / 2;
            Frag vf[DBLK][2];
#pragma unroll
            for (int db = 0; db < VPRE; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    vf[db][q4 >> 1].h[q4 & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4 *)(uintptr_t)(va_[db] + q4 * (8 / RPI) * GS));
            __builtin_amdgcn_sched_barrier(0);
            if (lim < 32) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int tok = 8 * (r >> 2) + 4 * h + (r & 3);  // S^T register r of this lane
                    if (tok >= lim) s[r] = -INFINITY;
                }
            }
            float mx = s[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
            mx = max_with_other_half(mx);
            // Online softmax with a lazily updated reference maximum (log2 domain): the reference only
            // moves when the running maximum has grown by more than kLazy, so exponentials stay below
            // 2^kLazy and the rescale of the accumulator is skipped for almost every tile.  The result
            // is unchanged: numerator and denominator always share the same reference.
            const float m_cand = fmaxf(m_run, mx * c);
            if (__any(m_cand - m_run > kLazy)) {
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_cand);
                m_run = m_cand;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
            }
            float p[16];
            float sum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = __builtin_amdgcn_exp2f(s[r] * c - m_run);
                sum += p[r];
            }
            l_run += sum;
            Frag p1, p2;
            p1.u = make_uint4(pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]), pack_bf16(p[6], p[7]));
            p2.u = make_uint4(pack_bf16(p[8], p[9]), pack_bf16(p[10], p[11]), pack_bf16(p[12], p[13]),
                              pack_bf16(p[14], p[15]));
            // O^T += V^T P^T.  MFMA k-slot (h, j) of the first product is token 8*(j/4) + 4*h + j%4 (what
            // registers 0..7 of S^T hold); the second product is 16 tokens further.
#pragma unroll
            for (int db = VPRE; db < DBLK; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                    vf[db][q4 >> 1].h[q4 & 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4 *)(uintptr_t)(va_[db] + q4 * (8 / RPI) * GS));
#pragma unroll
            for (int db = 0; db < DBLK; ++db) {
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][0].v, p1.v, o[db], 0, 0, 0);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[db][1].v, p2.v, o[db], 0, 0, 0);
            }
        }

        // ---- write-out: this wave's 32 rows
        l_run = sum_with_other_half(l_run);
        if (final_out) {
            if (row_ok) {
                const int i = irow, hl = ridx - i * G;
                const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
                uint16_t *op = a.out + ((row_base + i) * a.num_q_heads + (int64_t)g * G + hl) * D;
#pragma unroll
                for (int db = 0; db < DBLK; ++db)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        uint2 pk;
                        pk.x = pack_bf16(o[db][4 * r4] * inv, o[db][4 * r4 + 1] * inv);
                        pk.y = pack_bf16(o[db][4 * r4 + 2] * inv, o[db][4 * r4 + 3] * inv);
                        *(uint2 *)(op + 32 * db + 8 * r4 + 4 * h) = pk;
                    }
                if (a.lse && h == 0)
                    a.lse[((int64_t)b * a.num_q_heads + (int64_t)g * G + hl) * K + i] =
                        (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
            }
        } else {
            // partial in register order: [partial][wave][db][r4][lane] float4, then (m, l) per row
            const size_t slot = part_slot * W + wave;
            f32x4 *po = (f32x4 *)a.part_o + slot * (DBLK * 4 * 64) + lane;
#pragma unroll
            for (int db = 0; db < DBLK; ++db)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    const f32x4 v = {o[db][4 * r4], o[db][4 * r4 + 1], o[db][4 * r4 + 2], o[db][4 * r4 + 3]};
                    if (a.kv_nt) __builtin_nontemporal_store(v, &po[(db * 4 + r4) * 64]);
                    else po[(db * 4 + r4) * 64] = v;
                }
            if (h == 0) ((float2 *)a.part_ml)[slot * 32 + col] = make_float2(m_run, l_run);
        }
        if (!BALANCED || !open_item()) break;
        wg_barrier();  // matches the loader's barrier between segments
    }
}

// Merge the per-split partials in split order and write bf16 rows.  One workgroup per (sequence,
// KV head, 32-row block, 32-wide d block), one wave per group of 4 d values: a lane reads exactly the
// float4 it would hold in the split kernel's accumulator, so every load is a contiguous 1 KB per wave
// and all splits of a chunk are in flight together.
//
// BALANCED = 1: the pieces of a unit are found from the split kernel's partition arithmetic (NWG is
// that launch's workgroup count): unit (g, b) covers tiles [U0, U1) of the launch's tile sequence,
// its pieces belong to workgroups w_lo..w_hi, the first in its slot 2w+1 and the others in slot 2w;
// a unit held by one workgroup was finished by the split kernel.
//
// CHUNK = partials merged per round of loads: 8 keeps the registers low for the bandwidth-bound merges
// of many units with few pieces each; 16 or 32 make the latency-bound merge of few units with many
// splits a single memory round trip (a second round costs it ~1 us).
template <int D, int W, int BALANCED = 0, int CHUNK = 8>
__global__ void __launch_bounds__(256) attn_combine_kernel(const AttnArgs a)
{
    constexpr int DBLK = D / 32;
    constexpr int MCHUNK = 32;  // m values fetched per round when there are more than CHUNK partials
    const int lane = threadIdx.x & 63, r4 = threadIdx.x >> 6;
    const int col = lane & 31, h = lane >> 5;
    const int db = blockIdx.x % DBLK;
    const int wave = (blockIdx.x / DBLK) % W;  // row block
    const int unit = blockIdx.x / (DBLK * W);
    const int b = unit / a.num_kv_heads, g = unit % a.num_kv_heads;
    const int ridx = wave * 32 + col;
    int live;           // number of partials of this unit
    size_t first_slot;  // partial index of piece 0; piece s > 0 sits at rest_slot + s * slot_step
    size_t rest_slot, slot_step;
    if constexpr (BALANCED) {
        int before = 0, per_head = 0, mine = 0;  // tiles of the sequences before b, of all, of b
        for (int x0 = 0; x0 < a.batch; x0 += 64) {
            const int x = x0 + lane;
            int n = 0;
            if (x < a.batch) {
                int L = a.seq_lens[x];
                L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
                n = ((L + 31) >> 5) + 1;
            }
            int nb = x < b ? n : 0, nm = x == b ? n : 0;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                n += __shfl_xor(n, off);
                nb += __shfl_xor(nb, off);
                nm += __shfl_xor(nm, off);
            }
            per_head += n;
            before += nb;
            mine += nm;
        }
        const int64_t total = (int64_t)per_head * a.num_kv_heads;
        const int64_t nwg = total < (int64_t)a.bal_wgs ? total : (int64_t)a.bal_wgs;
        const int64_t U0 = (int64_t)g * per_head + before, U1 = U0 + mine;
        // workgroup w starts at tile floor(w * total / nwg): w_lo is the last one that starts at or
        // before U0, w_hi the last one that starts before U1
        const int64_t w_lo = ((U0 + 1) * nwg + total - 1) / total - 1;
        const int64_t w_hi = (U1 * nwg + total - 1) / total - 1;
        if (w_lo == w_hi) return;  // one workgroup held the whole unit and wrote its rows
        live = (int)(w_hi - w_lo + 1);
        first_slot = (size_t)w_lo * 2 + 1;
        rest_slot = (size_t)w_lo * 2;
        slot_step = 2;
    } else {
        int L = ((const const_i32 *)a.seq_lens)[b];
        L = L < 0 ? 0 : (L > a.max_seq_len ? a.max_seq_len : L);
        live = split_cut(L, a.num_splits, 0).live;  // the split kernel's pieces of this sequence
        first_slot = rest_slot = (size_t)unit * a.num_splits;
        slot_step = 1;
    }
    // partial `s` of this unit: (m, l) of the lane's row and the lane's float4 of the accumulator
    auto ml_at = [&](int s) __attribute__((always_inline)) {
        const size_t slot = (s == 0 ? first_slot : rest_slot + (size_t)s * slot_step) * W + wave;
        return (const float2 *)a.part_ml + slot * 32 + col;
    };
    auto po_at = [&](int s) __attribute__((always_inline)) {
        const size_t slot = (s == 0 ? first_slot : rest_slot + (size_t)s * slot_step) * W + wave;
        return (const float4 *)a.part_o + slot * (DBLK * 4 * 64) + (size_t)(db * 4 + r4) * 64 + lane;
    };

    // The loads of the first CHUNK partials go out before anything waits; the reference maximum needs
    // every partial's m, so the remaining m values follow MCHUNK at a time, then the rest of the data.
    // A merge of up to CHUNK partials is one memory round trip, not one per pass.
    float4 v[CHUNK];
    float2 e[CHUNK];
    auto load_chunk = [&](int s0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < CHUNK; ++u) {
            const bool ok = s0 + u < live;
            v[u] = ok ? *po_at(s0 + u) : make_float4(0.f, 0.f, 0.f, 0.f);
            e[u] = ok ? *ml_at(s0 + u) : make_float2(kNegBig, 0.f);
        }
    };
    load_chunk(0);
    float M = kNegBig;
#pragma unroll
    for (int u = 0; u < CHUNK; ++u) M = fmaxf(M, e[u].x);
    for (int s0 = CHUNK; s0 < live; s0 += MCHUNK) {
        float mv[MCHUNK];
#pragma unroll
        for (int u = 0; u < MCHUNK; ++u) mv[u] = (s0 + u < live) ? ml_at(s0 + u)->x : kNegBig;
#pragma unroll
        for (int u = 0; u < MCHUNK; ++u) M = fmaxf(M, mv[u]);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float lsum = 0.f;
    for (int s0 = 0; s0 < live; s0 += CHUNK) {
        if (s0 > 0) load_chunk(s0);
#pragma unroll
        for (int u = 0; u < CHUNK; ++u) {  // fixed split order: the result does not depend on timing
            const float sc = __builtin_amdgcn_exp2f(e[u].x - M);
            lsum += sc * e[u].y;
            acc.x += sc * v[u].x; acc.y += sc * v[u].y; acc.z += sc * v[u].z; acc.w += sc * v[u].w;
        }
    }
    if (ridx >= a.rows) return;
    const int G = a.group, K = a.block_k;
    const int i = ridx / G, hl = ridx - i * G;
    const float inv = lsum > 0.f ? 1.f / lsum : 0.f;
    uint16_t *op = a.out + (((int64_t)b * K + i) * a.num_q_heads + (int64_t)g * G + hl) * D;
    uint2 pk;
    pk.x = pack_bf16(acc.x * inv, acc.y * inv);
    pk.y = pack_bf16(acc.z * inv, acc.w * inv);
    *(uint2 *)(op + 32 * db + 8 * r4 + 4 * h) = pk;
    if (a.lse && db == 0 && r4 == 0 && h == 0)
        a.lse[((int64_t)b * a.num_q_heads + (int64_t)g * G + hl) * K + i] =
            (M + __builtin_amdgcn_logf(lsum)) * 0.6931471805599453f;
}

// ---------------------------------------------------------------------------------------------
// host side

#ifndef ORTHRUS_ATTN_STAGES
#define ORTHRUS_ATTN_STAGES 3
#endif
constexpr int kStages = ORTHRUS_ATTN_STAGES;  // LDS ring depth (2..4)
static size_t lds_need(int head_dim)
{
    return (size_t)kStages * (head_dim == 128 ? AttnGeom<128>::STAGE_B : AttnGeom<64>::STAGE_B);
}

hipError_t plan_attn(int head_dim, int group, int block_k, int batch, int num_kv_heads, int max_seq_len,
                     int requested_splits, int num_cus, int num_layers, AttnPlan *plan)
{
    const int R = group * block_k;
    plan->rows = R;
    const int W = R > 32 ? (R + 31) / 32 : 1;
    plan->waves = W;
    plan->rows_padded = W * 32;
    plan->lds_bytes = lds_need(head_dim);
    const int64_t units = (int64_t)batch * num_kv_heads;
    // workgroups resident per CU: LDS ring size, and 12 waves (3 per SIMD: the kernel stays below 168
    // registers) of W compute waves + the loader wave each
    int per_cu = (int)(160 * 1024 / plan->lds_bytes);
    if (per_cu > 12 / (W + 1)) per_cu = 12 / (W + 1);
    if (per_cu < 1) per_cu = 1;
    plan->bal_wgs = 0;
    // K/V bytes the model streams at most between two passes over the same layer's cache (the other
    // layers' caches come in between), against the 256 MB last-level cache (see the kernel's loads)
    const double stream_bytes = (double)(num_layers > 1 ? num_layers : 1) * batch * max_seq_len * num_kv_heads * 4.0 * head_dim;
    plan->kv_nt = stream_bytes > 1.25 * 256.0 * 1024 * 1024 ? 1 : 0;
    if (requested_splits < 0) {
        // balanced partition: as many workgroups as are resident at once, two partial slots each
        plan->bal_wgs = num_cus * per_cu;
        plan->chunk_tokens = 32;
        plan->num_splits = 1;
        plan->part_o_bytes = (size_t)plan->bal_wgs * 2 * plan->rows_padded * head_dim * sizeof(float);
        plan->part_ml_bytes = (size_t)plan->bal_wgs * 2 * plan->rows_padded * 2 * sizeof(float);
        return hipSuccess;
    }
    int splits;
    if (requested_splits > 0) {
        splits = requested_splits;
    } else {
        // Pick the split count with a small cost model (times in microseconds, constants measured on
        // this chip), using max_seq_len for every sequence.  Workgroups run in rounds of `slots`.  A
        // workgroup needs at least kTile per 32-token tile whatever the stream could deliver (the
        // loader wave's issue rate and the dependent chain of one tile's products and softmax are
        // both about that long: what binds when few CUs are busy, e.g. batch 1), and the tiles of all
        // workgroups of a round together stream no faster than kRate.  Every workgroup costs kWg to
        // dispatch; every piece beyond a unit's first is an fp32 partial (rows x d x 4 bytes) written
        // once and read once, and brings the merge launch with it.
        const double kRate = 7.0e6;      // K/V bytes per microsecond (measured ceiling of the paged stream)
        const double kPartRate = 6.0e6;  // bytes per microsecond for the partials
        const double kTile = W <= 4 ? 0.56 : 1.3;  // more than four 32-row blocks: two per SIMD
        const double kRound = 5.0, kCombine = 4.0, kSplit = 0.12, kWg = 0.008;
        const int64_t slots = (int64_t)num_cus * per_cu;
        const double tile_bytes = 32.0 * 2.0 * head_dim * 2.0;  // K + V bytes of one tile of one KV head
        const double part_bytes = 2.0 * plan->rows_padded * head_dim * 4.0;  // written once, read once
        const int max_s = max_seq_len >= 256 ? (max_seq_len / 128 < 64 ? max_seq_len / 128 : 64) : 1;
        const int tiles = (max_seq_len + 31) / 32;
        double cost[65];
        double best = 1e300;
        for (int s = 1; s <= max_s; ++s) {
            const int64_t wgs = units * s;
            const double tiles_per_wg = (double)((tiles + s - 1) / s);
            double t = s > 1 ? kCombine + kSplit * s : 0.0;  // the merge reads one more partial per output and split
            for (int64_t left = wgs; left > 0; left -= slots) {
                const int64_t now = left < slots ? left : slots;
                const double per_tile = tile_bytes * now / kRate;  // all workgroups of the round share the stream
                t += kRound + tiles_per_wg * (per_tile > kTile ? per_tile : kTile) +
                     now * (kWg + (s > 1 ? part_bytes / kPartRate : 0.0));
            }
            cost[s] = t;
            if (t < best) best = t;
        }
        splits = 1;
        while (cost[splits] > best * 1.01) ++splits;  // the fewest splits within 1 % of the best estimate
    }
    int chunk = (max_seq_len + splits - 1) / splits;
    chunk = ((chunk + 31) / 32) * 32;
    if (chunk < 32) chunk = 32;
    splits = max_seq_len > 0 ? (max_seq_len + chunk - 1) / chunk : 1;
    if (splits < 1) splits = 1;
    plan->chunk_tokens = chunk;
    plan->num_splits = splits;
    if (splits > 1) {
        plan->part_o_bytes = (size_t)units * splits * plan->rows_padded * head_dim * sizeof(float);
        plan->part_ml_bytes = (size_t)units * splits * plan->rows_padded * 2 * sizeof(float);
    } else {
        plan->part_o_bytes = plan->part_ml_bytes = 0;
    }
    return hipSuccess;
}

// One attention call: the split kernel, then the merge when units were cut into pieces.
template <int D, int W, int BALANCED>
static hipError_t launch_variant(const AttnArgs &a, const AttnPlan &plan, hipStream_t stream, AttnLaunchEvents *ev)
{
    auto kern = attn_split_kernel<D, W, kStages, 0, BALANCED>;
    auto comb = attn_combine_kernel<D, W, BALANCED, 8>;
    if constexpr (!BALANCED) {
        if (plan.num_splits > 16) comb = attn_combine_kernel<D, W, 0, 32>;
        else if (plan.num_splits > 8) comb = attn_combine_kernel<D, W, 0, 16>;
    }
    const bool timed = ev && ev->on;
    dim3 grid(BALANCED ? (unsigned)plan.bal_wgs
                       : (unsigned)plan.num_splits * (unsigned)a.num_kv_heads * (unsigned)a.batch);
    dim3 block(64 * (W + 1));
    if (timed) {
        hipExtLaunchKernelGGL(kern, grid, block, plan.lds_bytes, stream, ev->start[0], ev->stop[0], 0, a);
        ev->used[0] = true;
    } else {
        hipLaunchKernelGGL(kern, grid, block, plan.lds_bytes, stream, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (BALANCED || plan.num_splits > 1) {
        dim3 cgrid((unsigned)(a.batch * a.num_kv_heads) * W * (D / 32));
        if (timed) {
            hipExtLaunchKernelGGL(comb, cgrid, dim3(256), 0, stream, ev->start[1], ev->stop[1], 0, a);
            ev->used[1] = true;
        } else {
            hipLaunchKernelGGL(comb, cgrid, dim3(256), 0, stream, a);
        }
        e = hipGetLastError();
    }
    return e;
}

// The stream probe: the same grid, partition and loader as the attention call planned by `plan`, with one
// idle compute wave per workgroup.
template <int D>
static hipError_t launch_probe_d(const AttnArgs &a, const AttnPlan &plan, hipStream_t stream, hipEvent_t start,
                                 hipEvent_t stop)
{
    const bool bal = plan.bal_wgs > 0;
    auto kern = bal ? attn_split_kernel<D, 1, kStages, 0, 1, 1> : attn_split_kernel<D, 1, kStages, 0, 0, 1>;
    dim3 grid(bal ? (unsigned)plan.bal_wgs : (unsigned)plan.num_splits * (unsigned)a.num_kv_heads * (unsigned)a.batch);
    const size_t lds = lds_need(D);
    if (start && stop) hipExtLaunchKernelGGL(kern, grid, dim3(128), lds, stream, start, stop, 0, a);
    else hipLaunchKernelGGL(kern, grid, dim3(128), lds, stream, a);
    return hipGetLastError();
}

hipError_t launch_kv_stream_probe(const AttnArgs &a, const AttnPlan &plan, int head_dim, hipStream_t stream,
                                  hipEvent_t start, hipEvent_t stop)
{
    if (a.batch == 0) return hipSuccess;
    if (head_dim == 128) return launch_probe_d<128>(a, plan, stream, start, stop);
    if (head_dim == 64) return launch_probe_d<64>(a, plan, stream, start, stop);
    return hipErrorInvalidValue;
}

template <int D, int W>
static hipError_t launch_prefill_variant(const AttnArgs &a, size_t lds_bytes, hipStream_t stream)
{
    dim3 grid((unsigned)a.num_splits * (unsigned)a.num_kv_heads * (unsigned)a.batch);
    hipLaunchKernelGGL((attn_split_kernel<D, W, kStages, 1>), grid, dim3(64 * (W + 1)), lds_bytes, stream, a);
    return hipGetLastError();
}

// Prefill attention: a.num_splits carries the number of 32-token chunks per sequence, a.rows = 32 * group.
template <int D>
static hipError_t launch_prefill_d(const AttnArgs &a, size_t lds, hipStream_t stream)
{
    switch (a.group) {  // one compute wave per query head of the group
    case 1: return launch_prefill_variant<D, 1>(a, lds, stream);
    case 2: return launch_prefill_variant<D, 2>(a, lds, stream);
    case 3: return launch_prefill_variant<D, 3>(a, lds, stream);
    case 4: return launch_prefill_variant<D, 4>(a, lds, stream);
    case 5: return launch_prefill_variant<D, 5>(a, lds, stream);
    case 6: return launch_prefill_variant<D, 6>(a, lds, stream);
    case 7: return launch_prefill_variant<D, 7>(a, lds, stream);
    case 8: return launch_prefill_variant<D, 8>(a, lds, stream);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_prefill_attn(const AttnArgs &a, int head_dim, hipStream_t stream)
{
    if (a.batch == 0 || a.num_splits == 0) return hipSuccess;
    const size_t lds = lds_need(head_dim);
    if (head_dim == 128) return launch_prefill_d<128>(a, lds, stream);
    if (head_dim == 64) return launch_prefill_d<64>(a, lds, stream);
    return hipErrorInvalidValue;
}

template <int D, int BALANCED>
static hipError_t launch_attn_d(const AttnArgs &a, const AttnPlan &plan, hipStream_t stream, AttnLaunchEvents *events)
{
    switch (plan.waves) {
    case 1: return launch_variant<D, 1, BALANCED>(a, plan, stream, events);
    case 2: return launch_variant<D, 2, BALANCED>(a, plan, stream, events);
    case 3: return launch_variant<D, 3, BALANCED>(a, plan, stream, events);
    case 4: return launch_variant<D, 4, BALANCED>(a, plan, stream, events);
    case 5: return launch_variant<D, 5, BALANCED>(a, plan, stream, events);
    case 6: return launch_variant<D, 6, BALANCED>(a, plan, stream, events);
    case 7: return launch_variant<D, 7, BALANCED>(a, plan, stream, events);
    case 8: return launch_variant<D, 8, BALANCED>(a, plan, stream, events);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_attn(const AttnArgs &a, const AttnPlan &plan, int head_dim, hipStream_t stream,
                       AttnLaunchEvents *events)
{
    if (a.batch == 0) return hipSuccess;
    const bool bal = plan.bal_wgs > 0;
    if (head_dim == 128)
        return bal ? launch_attn_d<128, 1>(a, plan, stream, events) : launch_attn_d<128, 0>(a, plan, stream, events);
    if (head_dim == 64)
        return bal ? launch_attn_d<64, 1>(a, plan, stream, events) : launch_attn_d<64, 0>(a, plan, stream, events);
    return hipErrorInvalidValue;
}

}  // namespace orthrus
