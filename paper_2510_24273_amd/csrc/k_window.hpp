// Mixed-precision recent window (Sec. 5.1): the most recent w tokens, which the selection always keeps
// (Sec. 5.2), live in a second latent cache of higher rank, a ring of w rows with its own projectors.
// Attention over the union of both caches is one softmax (Eq. 5).  It runs as two passes of the sparse-attention
// kernels, the low-rank pass over the sinks and critical tokens and the window pass over the ring: both logits
// kernels leave their tile statistics in one array, so each value kernel weights its tokens with the maximum and
// normaliser of the whole selection, and one output projection adds the two passes' latent value sums through
// their projectors.  The kernel here only splits the selection into the two token lists.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"

namespace sals {

// The selection lists the recent tokens last.  With n = n_sel[b] and n_w = min(w, n):
//   idx_hi[b, :n_w] = idx[b, n - n_w : n] (zero beyond), n_hi[b] = n_w, n_lo[b] = n - n_w.
// grid (B), 256 threads.
__global__ __launch_bounds__(256) void window_split_kernel(const int32_t* __restrict__ idx,
                                                           const int32_t* __restrict__ n_sel, int k_tot, int w,
                                                           int32_t* __restrict__ idx_hi, int32_t* __restrict__ n_lo,
                                                           int32_t* __restrict__ n_hi)
{
    const int b = blockIdx.x;
    const int n = min(max(n_sel[b], 0), k_tot);
    const int nw = min(w, n);
    const int32_t* ib = idx + (size_t)b * k_tot;
    for (int i = threadIdx.x; i < w; i += 256) {
        const int v = ib[min(n - nw + i, k_tot - 1)];
        idx_hi[(size_t)b * w + i] = i < nw ? v : 0;
    }
    if (threadIdx.x == 0) { n_lo[b] = n - nw; n_hi[b] = nw; }
}

}  // namespace sals
