// Lossless consensus for temperature T > 0 on gfx950 (Section 3.3: exact rejection sampling after the
// speculative-sampling rule the paper cites): with p_k = softmax(ar_logits[k] / T) and
// q_k = softmax(diff_logits[k] / T), draft x of row k is kept iff accept_u[k] * q_k(x) < p_k(x); at the
// first row j that is not kept the emitted token is argmax_v [ log max(0, p_j - q_j)(v) + gumbel(v) ]
// (a draw from the normalised positive part of p_j - q_j; from p_j if that part is empty).  All random
// numbers are inputs, so the step is a deterministic function of its arguments.
//
//   lse_partial_kernel      grid (row * chunks + chunk): (max, sum of exp) of both scaled logit rows
//                           over one 8192-element chunk, 16-byte loads, wavefront shuffles.
//   draw_partial_kernel     grid (chunk, sequence): every workgroup re-derives the K keep decisions of
//                           its sequence from the chunk pairs (same code, same order => same answer
//                           everywhere), and if a row j < K was rejected scans its chunk of row j for the
//                           two candidate maxima.
//   sample_commit_kernel    grid (sequence): decisions again, final maximum over the chunks in chunk
//                           order, outputs, page check and the in-place commit of the kept rows.
#include "orthrus_internal.h"

namespace orthrus {

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kSChunk = 8192;
constexpr int kSInlineLayers = 2;

__device__ __forceinline__ void lse_merge(float &m, float &s, float m2, float s2)
{
    const float mn = fmaxf(m, m2);
    if (mn == -INFINITY) { m = mn; s = 0.f; return; }
    s = s * expf(m - mn) + s2 * expf(m2 - mn);
    m = mn;
}

__global__ void __launch_bounds__(256) lse_partial_kernel(const SamplingArgs a)
{
    const int chunks = a.c.chunks, V = a.c.vocab;
    const int row = blockIdx.x / chunks, chunk = blockIdx.x - row * chunks;
    const int tid = threadIdx.x;
    const float *pr = a.c.ar_logits + (int64_t)row * V;
    const float *qr = a.diff_logits + (int64_t)row * V;
    const int begin = chunk * kSChunk, end = min(V, begin + kSChunk);
    const float it = a.inv_temperature;
    constexpr int PER = kSChunk / 256;  // 32 values per thread and row
    float xp[PER], xq[PER];
    const bool vec_ok = ((V & 3) == 0) && (((((uintptr_t)a.c.ar_logits) | ((uintptr_t)a.diff_logits)) & 15) == 0);
    if (vec_ok) {
#pragma unroll
        for (int u = 0; u < PER / 4; ++u) {
            const int i = begin + (u * 256 + tid) * 4;
            float4 vp = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY), vq = vp;
            if (i < end) {  // one pass over both logit sets: loads that do not displace anything in the caches
                const f32x4 tp = __builtin_nontemporal_load((const f32x4 *)(pr + i));
                const f32x4 tq = __builtin_nontemporal_load((const f32x4 *)(qr + i));
                vp = make_float4(tp[0], tp[1], tp[2], tp[3]);
                vq = make_float4(tq[0], tq[1], tq[2], tq[3]);
            }
            xp[4 * u] = vp.x; xp[4 * u + 1] = vp.y; xp[4 * u + 2] = vp.z; xp[4 * u + 3] = vp.w;
            xq[4 * u] = vq.x; xq[4 * u + 1] = vq.y; xq[4 * u + 2] = vq.z; xq[4 * u + 3] = vq.w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int i = begin + u * 256 + tid;
            xp[u] = i < end ? pr[i] : -INFINITY;
            xq[u] = i < end ? qr[i] : -INFINITY;
        }
    }
    // Per thread: maximum of the raw logits (1/T > 0 keeps the order), then the sum of
    // exp((x - max) / T) as exp2 of one fused multiply-add per element.  Entries past the end are
    // -inf and add exp2(-inf) = 0; a thread that saw nothing but -inf keeps (max, sum) = (-inf, 0).
    float rp = -INFINITY, rq = -INFINITY;
#pragma unroll
    for (int u = 0; u < PER; ++u) { rp = fmaxf(rp, xp[u]); rq = fmaxf(rq, xq[u]); }
    const float c2 = it * 1.4426950408889634f;  // log2(e) / T
    const float bp = rp == -INFINITY ? 0.f : -rp * c2, bq = rq == -INFINITY ? 0.f : -rq * c2;
    float sp = 0.f, sq = 0.f;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        sp += __builtin_amdgcn_exp2f(__builtin_fmaf(xp[u], c2, bp));
        sq += __builtin_amdgcn_exp2f(__builtin_fmaf(xq[u], c2, bq));
    }
    float mp = rp * it, mq = rq * it;  // maxima of the scaled logits (natural-log domain from here on)
    // wavefront, then workgroup merge in a fixed order
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        lse_merge(mp, sp, __shfl_xor(mp, off), __shfl_xor(sp, off));
        lse_merge(mq, sq, __shfl_xor(mq, off), __shfl_xor(sq, off));
    }
    __shared__ float4 sh[4];
    if ((tid & 63) == 0) sh[tid >> 6] = make_float4(mp, sp, mq, sq);
    __syncthreads();
    if (tid == 0) {
        float4 r = sh[0];
#pragma unroll
        for (int w = 1; w < 4; ++w) { lse_merge(r.x, r.y, sh[w].x, sh[w].y); lse_merge(r.z, r.w, sh[w].z, sh[w].w); }
        a.lse_part[(int64_t)row * chunks + chunk] = r;
    }
}

// Keep decisions of sequence b, made by the first wavefront (lane k < K owns row k).  Returns the first
// row that is not kept (K if none) and, for that row, the two log-sum-exps.
__device__ __forceinline__ int first_rejected(const SamplingArgs &a, int b, int lane, float &lsep_j, float &lseq_j)
{
    const int K = a.c.block_k, V = a.c.vocab, chunks = a.c.chunks;
    bool keep = true;  // lanes >= K do not stop the run
    float lsep = 0.f, lseq = 0.f;
    if (lane < K) {
        const int64_t row = (int64_t)b * K + lane;
        float4 r = a.lse_part[row * chunks];
        // the row's chunk pairs, eight loads in flight at a time, merged in chunk order
        for (int c0 = 1; c0 < chunks; c0 += 8) {
            float4 t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = a.lse_part[row * chunks + min(c0 + u, chunks - 1)];
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (c0 + u < chunks) {
                    lse_merge(r.x, r.y, t[u].x, t[u].y);
                    lse_merge(r.z, r.w, t[u].z, t[u].w);
                }
        }
        lsep = r.x + logf(r.y);
        lseq = r.z + logf(r.w);
        const int x = a.c.draft_tokens[row];
        keep = false;
        if (x >= 0 && x < V) {
            const float px = expf(a.c.ar_logits[row * V + x] * a.inv_temperature - lsep);
            const float qx = expf(a.diff_logits[row * V + x] * a.inv_temperature - lseq);
            keep = a.accept_u[row] * qx < px;
        }
    }
    const unsigned long long rej = ~__ballot(keep);
    const int j = rej ? __ffsll((long long)rej) - 1 : 64;
    const int jj = j < K ? j : K;
    lsep_j = __shfl(lsep, jj < K ? jj : 0);
    lseq_j = __shfl(lseq, jj < K ? jj : 0);
    return jj;
}

__device__ __forceinline__ bool better_score(float v1, int i1, float v2, int i2)
{
    return v1 > v2 || (v1 == v2 && i1 < i2);
}

__global__ void __launch_bounds__(256) draw_partial_kernel(const SamplingArgs a)
{
    const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int K = a.c.block_k, V = a.c.vocab, chunks = a.c.chunks;
    __shared__ int s_j;
    __shared__ float s_lsep, s_lseq;
    if (tid < 64) {
        float lp, lq;
        const int j = first_rejected(a, b, tid, lp, lq);
        if (tid == 0) { s_j = j; s_lsep = lp; s_lseq = lq; }
    }
    __syncthreads();
    const int j = s_j;
    if (j >= K) return;  // every draft kept: nothing to draw
    const float lsep = s_lsep, lseq = s_lseq, it = a.inv_temperature;
    const float *pr = a.c.ar_logits + ((int64_t)b * K + j) * V;
    const float *qr = a.diff_logits + ((int64_t)b * K + j) * V;
    const float *gr = a.gumbel + (int64_t)b * V;
    const int begin = chunk * kSChunk, end = min(V, begin + kSChunk);
    float bp = -INFINITY, ba = -INFINITY;   // best among p > q, best of log p + g
    int ip = 0x7fffffff, ia = 0x7fffffff;
    auto visit = [&](int i, float xp, float xq, float g) __attribute__((always_inline)) {
        const float lp = xp * it - lsep, lq = xq * it - lseq;
        const float r = expf(lp) - expf(lq);
        if (r > 0.f) {
            const float sc = logf(r) + g;
            if (better_score(sc, i, bp, ip)) { bp = sc; ip = i; }
        }
        const float sa = lp + g;
        if (better_score(sa, i, ba, ia)) { ba = sa; ia = i; }
    };
    const bool vec_ok = ((V & 3) == 0) &&
                        (((((uintptr_t)a.c.ar_logits) | ((uintptr_t)a.diff_logits) | ((uintptr_t)a.gumbel)) & 15) == 0);
    if (vec_ok) {
        // all of a thread's loads of the chunk go out before the first score is formed
        constexpr int NL = kSChunk / (256 * 4);
        float4 vp[NL], vq[NL], vg[NL];
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = begin + (u * 256 + tid) * 4;
            vp[u] = vq[u] = vg[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < end) {
                vp[u] = *(const float4 *)(pr + i);
                vq[u] = *(const float4 *)(qr + i);
                vg[u] = *(const float4 *)(gr + i);
            }
        }
#pragma unroll
        for (int u = 0; u < NL; ++u) {
            const int i = begin + (u * 256 + tid) * 4;
            if (i < end) {  // indices ascend within a thread, as in the scalar loop
                visit(i, vp[u].x, vq[u].x, vg[u].x);
                visit(i + 1, vp[u].y, vq[u].y, vg[u].y);
                visit(i + 2, vp[u].z, vq[u].z, vg[u].z);
                visit(i + 3, vp[u].w, vq[u].w, vg[u].w);
            }
        }
    } else {
        for (int i = begin + tid; i < end; i += 256) visit(i, pr[i], qr[i], gr[i]);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float op = __shfl_xor(bp, off), oa = __shfl_xor(ba, off);
        const int jp = __shfl_xor(ip, off), ja = __shfl_xor(ia, off);
        if (better_score(op, jp, bp, ip)) { bp = op; ip = jp; }
        if (better_score(oa, ja, ba, ia)) { ba = oa; ia = ja; }
    }
    __shared__ float4 sh[4];
    if ((tid & 63) == 0) sh[tid >> 6] = make_float4(bp, __int_as_float(ip), ba, __int_as_float(ia));
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            if (better_score(sh[w].x, __float_as_int(sh[w].y), bp, ip)) { bp = sh[w].x; ip = __float_as_int(sh[w].y); }
            if (better_score(sh[w].z, __float_as_int(sh[w].w), ba, ia)) { ba = sh[w].z; ia = __float_as_int(sh[w].w); }
        }
        a.draw_part[(int64_t)b * chunks + chunk] = make_float4(bp, __int_as_float(ip), ba, __int_as_float(ia));
    }
}

__global__ void __launch_bounds__(256) sample_commit_kernel(const SamplingArgs a)
{
    const ConsensusArgs &c = a.c;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int K = c.block_k, chunks = c.chunks;
    __shared__ int s_L, s_m;
    __shared__ int s_pg[32];
    if (tid < 64) {
        const int lane = tid;
        // the length and the page ids of the K positions that may be appended do not depend on the
        // decisions: their loads go out first
        CommitProbe probe = {0, -1};
        if (c.do_commit) probe = commit_probe(c, b, lane);
        float lp, lq;
        const int j = first_rejected(a, b, lane, lp, lq);
        int repl = -1;
        if (j < K) {
            float bp = -INFINITY, ba = -INFINITY;
            int ip = 0x7fffffff, ia = 0x7fffffff;
            // every lane walks the chunks in order (same result in all lanes), eight loads in flight at a time
            for (int c0 = 0; c0 < chunks; c0 += 8) {
                float4 t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = a.draw_part[(int64_t)b * chunks + min(c0 + u, chunks - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (c0 + u < chunks) {
                        if (better_score(t[u].x, __float_as_int(t[u].y), bp, ip)) { bp = t[u].x; ip = __float_as_int(t[u].y); }
                        if (better_score(t[u].z, __float_as_int(t[u].w), ba, ia)) { ba = t[u].z; ia = __float_as_int(t[u].w); }
                    }
            }
            repl = ip != 0x7fffffff ? ip : ia;
        }
        const int m = min(j + 1, K);
        if (lane < K) {
            int t = -1;
            if (lane < j) t = c.draft_tokens[(int64_t)b * K + lane];
            else if (lane == j && lane < m) t = repl;
            c.out_tokens[(int64_t)b * K + lane] = lane < m ? t : -1;
        }
        const int last_tok = (j < K) ? repl : c.draft_tokens[(int64_t)b * K + K - 1];
        int committed = m;
        const int L = probe.L;
        if (c.do_commit) {
            committed = commit_decide(c, b, lane, m, probe);
            if (lane < K) s_pg[lane] = probe.pg;
        }
        if (lane == 0) {
            c.accept_len[b] = j;
            c.num_committed[b] = committed;
            c.next_anchor[b] = last_tok;
            s_L = L;
            s_m = c.do_commit ? committed : 0;
        }
    }
    __syncthreads();
    if (c.do_commit && c.num_layers <= kSInlineLayers && s_m > 0)
        for (int layer = 0; layer < c.num_layers; ++layer) append_rows(c, b, layer, s_L, s_m, tid, 256, s_pg);
}

__global__ void __launch_bounds__(256) sample_commit_layers_kernel(const SamplingArgs a)
{
    const int b = blockIdx.x, layer = blockIdx.y;
    const int L = a.c.commit_info[b * 2], m = a.c.commit_info[b * 2 + 1];
    if (m > 0) append_rows(a.c, b, layer, L, m, threadIdx.x, 256);
}

hipError_t launch_sampling_consensus(const SamplingArgs &a, hipStream_t stream)
{
    const ConsensusArgs &c = a.c;
    if (c.batch == 0) return hipSuccess;
    hipLaunchKernelGGL(lse_partial_kernel, dim3((unsigned)c.chunks * (unsigned)(c.batch * c.block_k)), dim3(256), 0,
                       stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(draw_partial_kernel, dim3(c.chunks, c.batch), dim3(256), 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sample_commit_kernel, dim3(c.batch), dim3(256), 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (c.do_commit && c.num_layers > kSInlineLayers) {
        hipLaunchKernelGGL(sample_commit_layers_kernel, dim3(c.batch, c.num_layers), dim3(256), 0, stream, a);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace orthrus
