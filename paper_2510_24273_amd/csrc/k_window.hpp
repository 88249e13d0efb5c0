// Mixed-precision recent window (Sec. 5.1): the most recent w tokens, which the selection always keeps
// (Sec. 5.2), live in a second latent cache of higher rank, a ring of w rows with its own projectors.
// Attention over the union of both caches is one softmax; here it is evaluated as two passes of the
// sparse-attention kernels (the low-rank pass over the sinks and critical tokens, the window pass over the
// ring) whose outputs are combined with the weights their softmax statistics give:
//
//   out = (w_lo out_lo + w_hi out_hi) / (w_lo + w_hi),   w_x = Z_x exp(m_x - max(m_lo, m_hi))
//
// which is the same sum as a single softmax over all selected tokens.
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

// out[b,h,:] from the two passes' unrounded outputs [B,H,d] and per-tile statistics [B,H,parts].
// grid (B*H), 128 threads (one per channel); the tiles are merged in a fixed order (in sequence when there are
// at most eight per pass, else as a tree over the 128 threads).
template <typename T>
__global__ __launch_bounds__(128) void window_merge_kernel(const float* __restrict__ out_lo,
                                                           const float2* __restrict__ stats_lo, int parts_lo,
                                                           const float* __restrict__ out_hi,
                                                           const float2* __restrict__ stats_hi, int parts_hi,
                                                           T* __restrict__ out)
{
    __shared__ float2 sm[2][128];
    const size_t bh = blockIdx.x;
    const int c = threadIdx.x;
    const float y_lo = out_lo[bh * kHeadDim + c], y_hi = out_hi[bh * kHeadDim + c];
    float2 a = make_float2(-INFINITY, 0.f), h = a;
    if (parts_lo <= 8 && parts_hi <= 8) {
        // few tiles (the usual case): every thread merges them itself, all loads in flight together
        float2 ea[8], eh[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            ea[u] = stats_lo[bh * parts_lo + min(u, parts_lo - 1)];
            eh[u] = stats_hi[bh * parts_hi + min(u, parts_hi - 1)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (u < parts_lo) a = stat_merge(a, ea[u]);
            if (u < parts_hi) h = stat_merge(h, eh[u]);
        }
    } else {
        for (int t = c; t < parts_lo; t += 128) a = stat_merge(a, stats_lo[bh * parts_lo + t]);
        for (int t = c; t < parts_hi; t += 128) h = stat_merge(h, stats_hi[bh * parts_hi + t]);
        sm[0][c] = a; sm[1][c] = h;
        __syncthreads();
        for (int s = 64; s > 0; s >>= 1) {
            if (c < s) {
                sm[0][c] = stat_merge(sm[0][c], sm[0][c + s]);
                sm[1][c] = stat_merge(sm[1][c], sm[1][c + s]);
            }
            __syncthreads();
        }
        a = sm[0][0]; h = sm[1][0];
    }
    const float m = fmaxf(a.x, h.x);
    const float w_lo = a.y > 0.f ? a.y * __expf(a.x - m) : 0.f;  // Z > 0 implies a finite maximum
    const float w_hi = h.y > 0.f ? h.y * __expf(h.x - m) : 0.f;
    const float den = w_lo + w_hi;
    elem<T>::store(out + bh * kHeadDim + c, den > 0.f ? (w_lo * y_lo + w_hi * y_hi) / den : 0.f);
}

}  // namespace sals
