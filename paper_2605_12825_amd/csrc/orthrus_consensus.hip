// Greedy consensus and in-place commit for the Orthrus decode step on gfx950 (Section 3.3,
// "Architectural Consensus Mechanism", Eq. 8; Fig. 2(b): accepted tokens' KV appended to the
// shared cache).
//
//   argmax_partial_kernel  grid (row * chunks + chunk): each workgroup scans one chunk of one logits
//                          row with 16-byte loads and reduces (value, index) through wavefront
//                          shuffles; one (value, index) pair per chunk goes to the workspace.
//   accept_commit_kernel   grid (sequence): the four waves finish the K row argmaxes (chunk pairs spread
//                          over the lanes, wavefront-shuffle reduction), the first wave finds the
//                          accepted prefix with a wavefront ballot, writes tokens/lengths and checks
//                          that the appended positions are mapped; then the whole workgroup copies
//                          the appended K/V rows into their pages (up to kInlineLayers layers).
//   commit_kernel          grid (sequence, layer): the same copy as its own launch when there are
//                          more layers than one workgroup should copy.
// (A single-launch variant in which the last-arriving workgroup of a sequence finishes the job was
// measured and dropped: the device-scope release/acquire fences it needs per workgroup cost far
// more than the two extra launches.)
//
// Order among candidates: a NaN outranks every number, larger values outrank smaller ones, and
// among equals the smaller index wins; this is a total order, so the result does not depend on
// how the scan is split.
#include "orthrus_internal.h"

#include <mutex>

namespace orthrus {

typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---- device-resident scratch of the allocation-free entry point (orthrus_consensus_commit_noalloc)
// One fixed array per GPU, held until the process ends; it takes the place of the caller's workspace
// (chunk argmax pairs and the per-sequence commit record).  Every entry it uses is written by the
// call's first kernels before anything reads it, so nothing has to start at zero.  Host code never
// passes the array's name to a kernel: the name is only a handle for hipGetSymbolAddress, and each
// device has its own copy at its own address, looked up once with that device current.
constexpr size_t kScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

size_t consensus_scratch_bytes() { return kScratchBytes; }

hipError_t consensus_scratch_init(int device)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device]) return hipSuccess;
    void *ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));  // the current device's copy
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
    return hipSuccess;
}

void *consensus_scratch(int device)
{
    if (device < 0 || device >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    return g_scratch_ptr[device];
}

constexpr int kChunkElems = 8192;  // floats per (row, chunk) workgroup: 32 KiB
int consensus_chunk_elems() { return kChunkElems; }

// true if candidate (v1, i1) outranks (v2, i2)
__device__ __forceinline__ bool outranks(float v1, int i1, float v2, int i2)
{
    const bool n1 = v1 != v1, n2 = v2 != v2;
    if (n1 || n2) return (n1 && n2) ? (i1 < i2) : n1;
    return v1 > v2 || (v1 == v2 && i1 < i2);
}

// update for a candidate known to sit at a larger index than the current best
__device__ __forceinline__ void take_later(float v, int i, float &bv, int &bi)
{
    if (!(bv != bv) && ((v != v) || v > bv)) { bv = v; bi = i; }
}

__device__ __forceinline__ void wave_best(float &bv, int &bi)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (outranks(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
}

constexpr int kInlineLayers = 2;

__global__ void __launch_bounds__(256) argmax_partial_kernel(const ConsensusArgs a)
{
    const int row = blockIdx.x / a.chunks, chunk = blockIdx.x - row * a.chunks;
    const int tid = threadIdx.x;
    const float *base = a.ar_logits + (int64_t)row * a.vocab;
    const int begin = chunk * a.chunk_elems;
    const int end = min(a.vocab, begin + a.chunk_elems);
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    // 16-byte loads need the row start aligned; rows are 4*vocab bytes apart
    const bool vec_ok = ((a.vocab & 3) == 0) && ((((uintptr_t)a.ar_logits) & 15) == 0);
    if (vec_ok) {
        // begin is a multiple of 4 (chunk_elems is); end too since vocab is.  All of a thread's loads of
        // the chunk go out before the first comparison (kChunkElems / 1024 = 8 loads of 16 bytes).
        constexpr int NL = kChunkElems / (256 * 4);
        float4 x[NL];
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = begin + (u * 256 + tid) * 4;
            x[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (i < end) {  // read once, never again: do not let the row displace anything in the caches
                const f32x4 v = __builtin_nontemporal_load((const f32x4 *)(base + i));
                x[u] = make_float4(v[0], v[1], v[2], v[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = begin + (u * 256 + tid) * 4;
            if (i < end) {
                if (bi == 0x7fffffff) { bv = x[u].x; bi = i; } else take_later(x[u].x, i, bv, bi);
                take_later(x[u].y, i + 1, bv, bi);
                take_later(x[u].z, i + 2, bv, bi);
                take_later(x[u].w, i + 3, bv, bi);
            }
        }
    } else {
        for (int i = begin + tid; i < end; i += 256) {
            const float x = base[i];
            if (bi == 0x7fffffff) { bv = x; bi = i; } else take_later(x, i, bv, bi);
        }
    }
    wave_best(bv, bi);
    __shared__ float sv[4];
    __shared__ int si[4];
    if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (outranks(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
        a.part_val[(int64_t)row * a.chunks + chunk] = bv;
        a.part_idx[(int64_t)row * a.chunks + chunk] = bi;
    }
}

__global__ void __launch_bounds__(256) accept_commit_kernel(const ConsensusArgs a)
{
    const int b = blockIdx.x, tid = threadIdx.x;
    const int K = a.block_k;
    __shared__ int s_L, s_m;
    __shared__ int s_am[32], s_pg[32];
    const int wave = tid >> 6, lane = tid & 63;
    // ---- loads that do not depend on the argmaxes go out first (first wave): the drafts, the length
    // and the page ids of the K positions that may be appended
    int draft = -1;
    CommitProbe probe = {0, -1};
    if (wave == 0) {
        if (lane < K) draft = a.draft_tokens[(int64_t)b * K + lane];
        if (a.do_commit) probe = commit_probe(a, b, lane);
    }
    // ---- row argmaxes: wave w finishes rows w, w+4, ...; a lane takes the chunk pairs lane, lane+64, ...
    // All loads of a wave's rows go out before the first reduction, so the phase costs one memory round
    // trip, not one per chunk.  A lane without a chunk holds (-inf, INT_MAX), which every real pair outranks.
    {
        constexpr int kRowsPerWave = 8;  // block_k <= 32 rows over 4 waves
        float bv[kRowsPerWave];
        int bi[kRowsPerWave];
#pragma unroll
        for (int u = 0; u < kRowsPerWave; ++u) {
            const int k = wave + 4 * u;
            bv[u] = -INFINITY;
            bi[u] = 0x7fffffff;
            if (k < K) {
                const int64_t r = ((int64_t)b * K + k) * a.chunks;
                for (int ch = lane; ch < a.chunks; ch += 64) {
                    const float v = a.part_val[r + ch];
                    const int i = a.part_idx[r + ch];
                    if (outranks(v, i, bv[u], bi[u])) { bv[u] = v; bi[u] = i; }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kRowsPerWave; ++u) {
            const int k = wave + 4 * u;
            if (k < K) {  // wave-uniform
                wave_best(bv[u], bi[u]);
                if (lane == 0) s_am[k] = bi[u];
            }
        }
    }
    __syncthreads();
    // ---- accept: the first wave, lane k < K owns block row k of sequence b
    if (wave == 0) {
        int am = -1;
        bool match = false;
        if (lane < K) {
            am = s_am[lane];
            match = draft == am;
        }
        // accepted prefix = run of matching rows starting at row 0
        const unsigned long long mism = ~__ballot(match);           // lanes >= K never match
        const int n_acc = mism ? __ffsll((long long)mism) - 1 : 64;  // first mismatching row (<= K)
        const int m = min(n_acc + 1, K);
        if (lane < K) a.out_tokens[(int64_t)b * K + lane] = lane < m ? am : -1;
        const int anchor = __shfl(am, m - 1);
        int committed = m;
        if (a.do_commit) {
            committed = commit_decide(a, b, lane, m, probe);
            if (lane < K) s_pg[lane] = probe.pg;
        }
        if (lane == 0) {
            a.accept_len[b] = n_acc;
            a.num_committed[b] = committed;
            a.next_anchor[b] = anchor;
            s_L = probe.L;
            s_m = a.do_commit ? committed : 0;
        }
    }
    __syncthreads();
    // ---- commit: the whole workgroup copies the appended rows when there are few layers
    if (a.do_commit && a.num_layers <= kInlineLayers && s_m > 0)
        for (int layer = 0; layer < a.num_layers; ++layer) append_rows(a, b, layer, s_L, s_m, tid, 256, s_pg);
}

// The same copy as its own launch: grid (sequence, layer).
__global__ void __launch_bounds__(256) commit_kernel(const ConsensusArgs a)
{
    const int b = blockIdx.x, layer = blockIdx.y;
    const int L = a.commit_info[b * 2], m = a.commit_info[b * 2 + 1];
    if (m > 0) append_rows(a, b, layer, L, m, threadIdx.x, 256);
}

hipError_t launch_consensus(const ConsensusArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    dim3 g1((unsigned)a.chunks * (unsigned)(a.batch * a.block_k));
    hipLaunchKernelGGL(argmax_partial_kernel, g1, dim3(256), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(accept_commit_kernel, dim3(a.batch), dim3(256), 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.do_commit && a.num_layers > kInlineLayers) {
        hipLaunchKernelGGL(commit_kernel, dim3(a.batch, a.num_layers), dim3(256), 0, stream, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace orthrus
