// Latent scores  s_j = q~_{:r*} . k~_{j,:r*}  (Sec. 4.3; Algorithm 1, score step).
//
// A pure HBM stream over the latent key cache: 16 lanes (one DPP row) own a cache row and
// read it in 16-byte pieces, so each load instruction of a wave covers four rows with 256
// contiguous bytes each; the 16 partial dot products are folded with DPP row rotations.
// The loads of the next four rows are issued before the current ones are consumed (two register sets
// take turns).  q~
// arrives as NP partial sums of the projection kernel (slices of the D axis); they are added
// in slice order into LDS while the first cache loads are in flight, then kept in registers.
// fp32 accumulation in a fixed order.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kScoreThreads = 256;
constexpr int kScoreRowsPerIter = (kScoreThreads / kWave) * 4;  // 16 rows per workgroup pass
constexpr int kScoreMaxR = 1024;  // scoring rank r* at most (q~[:r*] sits in LDS, one 16-byte piece per thread)
constexpr int kScoreMaxParts = 8;   // slices of the D axis the projection may split into

// NCH = 16-byte pieces per lane = ceil(r_score / (vec*16)); STREAM: cache rows are loaded with the read-once hint
template <typename T, int NCH, bool STREAM>
__global__ __launch_bounds__(kScoreThreads) void scores_kernel(const T* __restrict__ Kc,
                                                               const float* __restrict__ qt_part, int np,
                                                               const int32_t* __restrict__ seq_len,
                                                               float* __restrict__ scores, int B, int S_max,
                                                               int r, int r_score, int rows_per_wg,
                                                               uint2* __restrict__ wg_range, int n_sink, int n_recent)
{
    constexpr int VEC = elem<T>::vec;
    __shared__ __attribute__((aligned(16))) float q_s[kScoreMaxR];
    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int li = lane & 15, quad = lane >> 4;
    const int n_pieces = r_score / VEC;
    const int S_v = ld_uniform_i32(seq_len + b);  // (vector memory path: requested ahead of the first cache rows)
    const int j_begin = blockIdx.x * rows_per_wg;
    const int j_end = min(S_max, j_begin + rows_per_wg);
    const T* base = Kc + (size_t)b * S_max * r;

    auto load_row = [&](int j0, u32x4* piece) {
        const int j = j0 + wave * 4 + quad;
        // every row below S_max is readable, so the first pass of loads does not wait for the sequence length;
        // rows past it are overwritten with -inf when the score is stored
        const bool live = j < S_max;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            int p = li + 16 * n;
            const T* src = base + (size_t)j * r + p * VEC;
            piece[n] = (live && p < n_pieces) ? (STREAM ? ld16_stream(src) : ld16(src)) : u32x4{0, 0, 0, 0};
        }
    };

    u32x4 cur[NCH], nxt[NCH];
    load_row(j_begin, cur);

    // q~[b] = sum of the projection's partial sums (at most kScoreMaxParts slices), in slice order; all slices
    // are requested together (a loop with one load per round would cost a memory round trip per slice)
    static_assert(kScoreMaxR <= kScoreThreads * 4, "one 16-byte piece of q~ per thread");
    {
        const int i = tid * 4, ic = min(i, r - 4);  // (loads are unconditional, from clamped addresses: no branches)
        f32x4 t[kScoreMaxParts];
#pragma unroll
        for (int p = 0; p < kScoreMaxParts; ++p)
            t[p] = *reinterpret_cast<const f32x4*>(qt_part + ((size_t)min(p, np - 1) * B + b) * r + ic);
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < kScoreMaxParts; ++p) {
            const bool use = p < np;  // slices past the last one do not count
            s.x += use ? t[p].x : 0.f; s.y += use ? t[p].y : 0.f; s.z += use ? t[p].z : 0.f; s.w += use ? t[p].w : 0.f;
        }
        if (i < r_score) *reinterpret_cast<f32x4*>(&q_s[i]) = s;
    }
    __syncthreads();
    // The stream is paid for the sequence, not for the capacity: after the first pass (requested before the length
    // was known) only rows below the length are loaded; the rest of the workgroup's range is filled with -inf.
    const int S = min(wave_uniform(S_v), S_max);
    const int j_live = min(j_end, max(S, j_begin + kScoreRowsPerIter));
    const int j_tail = min(j_end, j_begin + (j_live - j_begin + kScoreRowsPerIter - 1) / kScoreRowsPerIter * kScoreRowsPerIter);
    for (int j = j_tail + tid; j < j_end; j += kScoreThreads) scores[(size_t)b * S_max + j] = -INFINITY;
    float qf[NCH][VEC];
#pragma unroll
    for (int n = 0; n < NCH; ++n) {
        int p = li + 16 * n;
#pragma unroll
        for (int v = 0; v < VEC; v += 4) {
            f32x4 t = (p < n_pieces) ? *reinterpret_cast<const f32x4*>(&q_s[p * VEC + v]) : f32x4{0.f, 0.f, 0.f, 0.f};
            qf[n][v] = t.x; qf[n][v + 1] = t.y; qf[n][v + 2] = t.z; qf[n][v + 3] = t.w;
        }
    }

    // smallest and largest key of the candidate scores (tokens that are neither sink nor recent) this thread stores;
    // only used when the long-sequence selection asks for them
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    auto finish_rows = [&](int j0, const u32x4* piece) {
        const int j = j0 + wave * 4 + quad;
        float acc = 0.f;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            float kf[VEC];
            elem<T>::unpack(piece[n], kf);
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc = fmaf(qf[n][v], kf[v], acc);
        }
        acc = row16_sum(acc);
        if (li == 0 && j < j_end) scores[(size_t)b * S_max + j] = j < S ? acc : -INFINITY;
        if (li == 0 && j < j_end && j >= n_sink && j < S - n_recent) {
            const uint32_t key = score_key(acc);
            kmin = min(kmin, key);
            kmax = max(kmax, key);
        }
    };
    // two register sets take turns (no copy between them: a copy would wait for the loads it moves)
    for (int j0 = j_begin; j0 < j_live; j0 += 2 * kScoreRowsPerIter) {
        const bool second = j0 + kScoreRowsPerIter < j_live;
        if (second) load_row(j0 + kScoreRowsPerIter, nxt);
        finish_rows(j0, cur);
        if (second) {
            if (j0 + 2 * kScoreRowsPerIter < j_live) load_row(j0 + 2 * kScoreRowsPerIter, cur);
            finish_rows(j0 + kScoreRowsPerIter, nxt);
        }
    }
    // The selection chain for long sequences bins the candidates' scores over their range: every workgroup leaves the
    // key range of the candidates it scored (none: the neutral pair), which saves that chain a pass over the scores.
    if (wg_range != nullptr) {  // uniform
        __shared__ uint32_t s_min[kScoreThreads / kWave], s_max[kScoreThreads / kWave];
        kmin = wave_min_u32(kmin);
        kmax = wave_max_u32(kmax);
        if (lane == 0) { s_min[wave] = kmin; s_max[wave] = kmax; }
        __syncthreads();
        if (tid == 0) {
#pragma unroll
            for (int w = 0; w < kScoreThreads / kWave; ++w) { kmin = min(kmin, s_min[w]); kmax = max(kmax, s_max[w]); }
            wg_range[(size_t)b * gridDim.x + blockIdx.x] = make_uint2(kmin, kmax);
        }
    }
}

}  // namespace sals
