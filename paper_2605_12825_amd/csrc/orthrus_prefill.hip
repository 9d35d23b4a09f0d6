// Front end of the AR view's prefill (Section 3.1: the frozen AR view processes the context with its
// ordinary causal self-attention and leaves its K/V in the cache that both views share afterwards).
//
//   prefill_plan_kernel    grid (sequence): validates the lengths, checks that every page the new tokens
//                          fall on is mapped, records the length before the call and the accepted number
//                          of new tokens (0 after an error) for the two kernels that follow, and bumps
//                          seq_lens.
//   prefill_append_kernel  grid (token block, sequence): copies the new tokens' K/V rows into their pages
//                          with 16-byte accesses.
// The attention itself is the split kernel of orthrus_attn.hip in its prefill form.
#include "orthrus_internal.h"

namespace orthrus {

__global__ void __launch_bounds__(64) prefill_plan_kernel(const PrefillArgs a)
{
    const int b = blockIdx.x, lane = threadIdx.x;
    const int L = a.seq_lens[b];
    int n = a.new_lens_in[b];
    bool bad = L < 0 || n < 0 || n > a.max_new || (int64_t)L + n > a.max_seq_len;
    if (!bad) {
        // pages of positions L .. L+n-1, one page slot per lane and round
        const int first = L >> a.page_shift, last = n > 0 ? (L + n - 1) >> a.page_shift : first - 1;
        for (int slot = first + lane; slot <= last; slot += 64) {
            if (slot >= a.max_pages_per_seq) bad = true;
            else {
                const int pg = a.page_table[(int64_t)b * a.max_pages_per_seq + slot];
                if (pg < 0 || pg >= a.num_pages) bad = true;
            }
        }
    }
    const bool any_bad = __ballot(bad) != 0ull;
    if (lane == 0) {
        if (any_bad) {
            atomicExch(a.err_word, -4);
            n = 0;
        }
        a.old_lens[b] = L < 0 ? 0 : L;
        a.new_lens[b] = n;
        if (!any_bad) a.seq_lens[b] = L + n;
    }
}

constexpr int kAppendRows = 16;  // new tokens per workgroup

__global__ void __launch_bounds__(256) prefill_append_kernel(const PrefillArgs a)
{
    const int b = blockIdx.y, i0 = blockIdx.x * kAppendRows;
    const int L = a.old_lens[b], n = a.new_lens[b];
    if (i0 >= n) return;
    const int rows = min(kAppendRows, n - i0);
    const int H = a.num_kv_heads, d = a.head_dim;
    const int cpr = d / 8;  // 16-byte chunks per row
    const int per_tok = H * cpr;
    const int P = 1 << a.page_shift;
    for (int e = threadIdx.x; e < rows * per_tok; e += 256) {
        const int k = e / per_tok, rem = e - k * per_tok;
        const int g = rem / cpr, ch = rem - g * cpr;
        const int pos = L + i0 + k;
        const int pg = a.page_table[(int64_t)b * a.max_pages_per_seq + (pos >> a.page_shift)];
        const int64_t src = (((int64_t)b * a.max_new + i0 + k) * H + g) * d + ch * 8;
        const int64_t dst = (int64_t)pg * a.stride_page + (int64_t)g * a.stride_head +
                            (int64_t)(pos & (P - 1)) * a.stride_tok + ch * 8;
        *(uint4 *)(a.k_pool + dst) = *(const uint4 *)(a.k_new + src);
        *(uint4 *)(a.v_pool + dst) = *(const uint4 *)(a.v_new + src);
    }
}

hipError_t launch_prefill_append(const PrefillArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_plan_kernel, dim3(a.batch), dim3(64), 0, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.max_new == 0) return e;
    dim3 grid((unsigned)((a.max_new + kAppendRows - 1) / kAppendRows), (unsigned)a.batch);
    hipLaunchKernelGGL(prefill_append_kernel, grid, dim3(256), 0, stream, a);
    return hipGetLastError();
}

}  // namespace orthrus
