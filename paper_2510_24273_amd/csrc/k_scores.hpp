// Latent scores  s_j = q~_{:r*} . k~_{j,:r*}  (Sec. 4.3; Algorithm 1, score step).
//
// A pure HBM stream over the latent key cache: 16 lanes (one DPP row) own a cache
// row and read it in 16-byte pieces, so each load instruction of a wave covers
// four rows with 256 contiguous bytes each; the 16 partial dot products are
// folded with DPP row rotations.  q~ sits in registers.  fp32 accumulation in a
// fixed order.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kScoreThreads = 256;
constexpr int kScoreRowsPerIter = (kScoreThreads / kWave) * 4;  // 16 rows per workgroup pass

// NCH = 16-byte pieces per lane = ceil(r_score / (vec*16))
template <typename T, int NCH>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(const T* __restrict__ Kc,
                                                               const float* __restrict__ qt,
                                                               const int32_t* __restrict__ seq_len,
                                                               float* __restrict__ scores, int S_max,
                                                               int r, int r_score, int rows_per_wg)
{
    constexpr int VEC = elem<T>::vec;
    const int b = blockIdx.y;
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int li = lane & 15, quad = lane >> 4;
    const int n_pieces = r_score / VEC;
    const int S = min(seq_len[b], S_max);
    const int j_begin = blockIdx.x * rows_per_wg;
    const int j_end = min(S_max, j_begin + rows_per_wg);
    const T* base = Kc + (size_t)b * S_max * r;

    float qf[NCH][VEC];
    bool q_loaded = false;

    for (int j0 = j_begin; j0 < j_end; j0 += kScoreRowsPerIter) {
        const int j = j0 + wave * 4 + quad;
        const bool live = j < S;
        u32x4 piece[NCH];
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            int p = li + 16 * n;
            piece[n] = (live && p < n_pieces) ? ld16(base + (size_t)j * r + p * VEC) : u32x4{0, 0, 0, 0};
        }
        if (!q_loaded) {  // after the first cache loads are in flight
#pragma unroll
            for (int n = 0; n < NCH; ++n) {
                int p = li + 16 * n;
#pragma unroll
                for (int v = 0; v < VEC; v += 4) {
                    f32x4 t = (p < n_pieces)
                                  ? *reinterpret_cast<const f32x4*>(qt + (size_t)b * r + p * VEC + v)
                                  : f32x4{0.f, 0.f, 0.f, 0.f};
                    qf[n][v] = t.x; qf[n][v + 1] = t.y; qf[n][v + 2] = t.z; qf[n][v + 3] = t.w;
                }
            }
            q_loaded = true;
        }
        float acc = 0.f;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            float kf[VEC];
            elem<T>::unpack(piece[n], kf);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc = fmaf(qf[n][v], kf[v], acc);
        }
        acc = row16_sum(acc);
        if (li == 0 && j < j_end) scores[(size_t)b * S_max + j] = live ? acc : -INFINITY;
    }
}

}  // namespace sals
