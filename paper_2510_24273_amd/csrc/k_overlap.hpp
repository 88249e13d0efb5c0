// Overlap score (Sec. 3.2): the share of the dense attention mass that a selected token set C captures,
//   OS[b,h] = sum_{j in C} p_j / sum_{j < S} p_j,   p_j = exp( RoPE(q[b,h]) . K[b,j,g(h)] / sqrt(d) ),
// over the full-rank rotated key cache of the dense baseline.  A diagnostic, not part of the decode path:
// a plain stream over K (16 lanes per token row, as the dense kernel reads it) that keeps, per head, the
// running maximum and sum of all tokens of a chunk and, from a gather of the chunk's share of C, the same
// pair for the selected tokens; a second kernel merges the chunks and takes the ratio.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"

namespace sals {

// part [B, H, n_chunks, 2] float2: (max, sum of exp) over all tokens of the chunk, and over the chunk's
// share of the selected tokens.  grid (n_chunks, H_kv, B), 256 threads.
template <typename T, int GMAX>
__global__ __launch_bounds__(256) void overlap_stats_kernel(const T* __restrict__ q, const int32_t* __restrict__ q_pos,
                                                            const T* __restrict__ K,
                                                            const int32_t* __restrict__ seq_len,
                                                            const int32_t* __restrict__ idx,
                                                            const int32_t* __restrict__ n_sel,
                                                            const float2* __restrict__ rope, InvFreq inv,
                                                            float2* __restrict__ part, int S_max, int H, int H_kv,
                                                            int k_tot, int n_chunks, int tok_per_chunk,
                                                            int sel_per_chunk, int rope_style, float scale)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int NCH = kHeadDim / (16 * VEC);  // 16-byte pieces per lane and row
    __shared__ float sQ[GMAX][kHeadDim];
    __shared__ float2 sCS[kPairs];
    __shared__ float2 sRed[2][GMAX][16];

    const int chunk = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, li = tid & 15, tg = tid >> 4;
    const int G = H / H_kv;
    const int S = min(max(seq_len[b], 0), S_max);
    const int n = min(max(n_sel[b], 0), k_tot);
    const size_t row_stride = (size_t)H_kv * kHeadDim;
    const T* kb = K + ((size_t)b * S_max * H_kv + kvh) * kHeadDim;

    // the rotated, pre-scaled query of this KV head's query heads
    const int qp = q_pos[b];
    if (tid < kPairs) {
        if (qp >= 0 && qp <= S_max) {
            sCS[tid] = rope[(size_t)qp * kPairs + tid];
        } else {
            double sn, c;
            sincos((double)qp * inv.f[tid], &sn, &c);
            sCS[tid] = make_float2((float)c, (float)sn);
        }
    }
    __syncthreads();
    for (int t = tid; t < G * kPairs; t += 256) {
        const int p = t & (kPairs - 1), m = t >> 6;
        const int c1 = pair_first(p, rope_style), c2 = pair_second(p, rope_style);
        const T* qh = q + ((size_t)b * H + kvh * G + m) * kHeadDim;
        const float a = elem<T>::load(qh + c1), bb = elem<T>::load(qh + c2);
        const float2 cs = sCS[p];
        sQ[m][c1] = (a * cs.x - bb * cs.y) * scale;
        sQ[m][c2] = (bb * cs.x + a * cs.y) * scale;
    }
    __syncthreads();
    float qf[GMAX][NCH][VEC];
#pragma unroll
    for (int m = 0; m < GMAX; ++m)
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int v = 0; v < VEC; ++v) qf[m][c][v] = m < G ? sQ[m][(li + 16 * c) * VEC + v] : 0.f;

    float2 st[2][GMAX];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int m = 0; m < GMAX; ++m) st[s][m] = make_float2(-INFINITY, 0.f);

    auto take_row = [&](int row, float2* acc) {  // row < S_max
        float kf[NCH][VEC];
#pragma unroll
        for (int c = 0; c < NCH; ++c) elem<T>::unpack(ld16(kb + (size_t)row * row_stride + (li + 16 * c) * VEC), kf[c]);
#pragma unroll
        for (int m = 0; m < GMAX; ++m) {
            float x = 0.f;
#pragma unroll
            for (int c = 0; c < NCH; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) x = fmaf(qf[m][c][v], kf[c][v], x);
            x = row16_sum(x);
            acc[m] = stat_merge(acc[m], make_float2(x, 1.f));
        }
    };
    // every token of the chunk
    const int j1 = min(S, (chunk + 1) * tok_per_chunk);
    for (int j = chunk * tok_per_chunk + tg; j < j1; j += 16) take_row(j, st[0]);
    // the chunk's share of the selected tokens
    const int c1 = min(n, (chunk + 1) * sel_per_chunk);
    const int32_t* ib = idx + (size_t)b * k_tot;
    for (int jj = chunk * sel_per_chunk + tg; jj < c1; jj += 16) take_row(min(max(ib[jj], 0), S_max - 1), st[1]);

    // the 16 lane groups, merged in group order
    if (li == 0) {
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int m = 0; m < GMAX; ++m) sRed[s][m][tg] = st[s][m];
    }
    __syncthreads();
    if (tid < 2 * G) {
        const int s = tid / G, m = tid % G;
        float2 a = make_float2(-INFINITY, 0.f);
        for (int g = 0; g < 16; ++g) a = stat_merge(a, sRed[s][m][g]);
        part[(((size_t)b * H + kvh * G + m) * n_chunks + chunk) * 2 + s] = a;
    }
}

// os[b,h] = (selected mass) / (total mass); zero for an empty cache.  One thread per (b,h).
__global__ __launch_bounds__(256) void overlap_merge_kernel(const float2* __restrict__ part, float* __restrict__ os,
                                                            int n_bh, int n_chunks)
{
    const int bh = blockIdx.x * 256 + threadIdx.x;
    if (bh >= n_bh) return;
    float2 all = make_float2(-INFINITY, 0.f), sel = all;
    for (int c = 0; c < n_chunks; ++c) {
        all = stat_merge(all, part[((size_t)bh * n_chunks + c) * 2]);
        sel = stat_merge(sel, part[((size_t)bh * n_chunks + c) * 2 + 1]);
    }
    os[bh] = (all.y > 0.f && sel.y > 0.f) ? sel.y * __expf(sel.x - all.x) / all.y : 0.f;
}

}  // namespace sals
