// Dense decode attention over a full-rank KV cache: the baseline the paper's speed-ups are
// quoted against (Sec. 5.3, Table 6), here as an in-library comparison on the same hardware.
//
//   out[b,h] = softmax_j( RoPE(q[b,h], q_pos[b]) . K[b,j,g(h)] / sqrt(d) ) V[b,j,g(h)],  j < seq_len[b]
//
// K [B, S_max, H_kv, d] holds the keys as a dense model caches them (already rotated at their
// positions), V [B, S_max, H_kv, d] the values.  A pure HBM stream of 2*S*D_kv elements per
// sequence: 16 lanes (one DPP row) own a token's head row of K and of V in 16-byte pieces, the
// dot product is folded with DPP rotations, softmax runs online per 16-lane group, and the rows of
// the next token are requested before the current ones are consumed.  A workgroup covers one
// (sequence, KV head, token chunk); its 16 lane groups and then the chunks are merged by
// log-sum-exp in a fixed order.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"

namespace sals {

constexpr int kDnMaxChunks = 64;  // token chunks per sequence at most
constexpr int kDnRec = kHeadDim + 2;  // floats per partial record: running max, normaliser, 128 sums

// part [B, H, n_chunks, kDnRec]
template <typename T, int GMAX>
__global__ __launch_bounds__(256) void dense_attend_kernel(const T* __restrict__ q, const int32_t* __restrict__ q_pos,
                                                           const T* __restrict__ K, const T* __restrict__ V,
                                                           const int32_t* __restrict__ seq_len,
                                                           const float2* __restrict__ rope, InvFreq inv,
                                                           float* __restrict__ part, int S_max, int H, int H_kv,
                                                           int n_chunks, int tok_per_chunk, int rope_style,
                                                           float scale)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int NCH = kHeadDim / (16 * VEC);  // 16-byte pieces per lane and row: 1 (bf16) or 2 (fp32)
    __shared__ float sQ[GMAX][kHeadDim];
    __shared__ float2 sCS[kPairs];
    __shared__ float sRed[16][kDnRec + 2];

    const int chunk = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, li = tid & 15, tg = tid >> 4;
    const int G = H / H_kv;
    const int S = min(seq_len[b], S_max);
    const int j0 = chunk * tok_per_chunk, j1 = min(S, j0 + tok_per_chunk);
    const size_t row_stride = (size_t)H_kv * kHeadDim;
    const T* kb = K + ((size_t)b * S_max * H_kv + kvh) * kHeadDim;
    const T* vb = V + ((size_t)b * S_max * H_kv + kvh) * kHeadDim;

    // every row below S_max is readable, so the first loads do not wait for the sequence length; rows
    // at or past it are requested at most one step ahead and never used
    const int j_readable = min(S_max, j0 + tok_per_chunk);
    auto load_rows = [&](int j, u32x4* kp, u32x4* vp) {
        const bool live = j < j_readable;
        const size_t off = (size_t)(live ? j : 0) * row_stride;
#pragma unroll
        for (int n = 0; n < NCH; ++n) {
            kp[n] = live ? ld16_stream(kb + off + (li + 16 * n) * VEC) : u32x4{0, 0, 0, 0};
            vp[n] = live ? ld16_stream(vb + off + (li + 16 * n) * VEC) : u32x4{0, 0, 0, 0};
        }
    };
    u32x4 kc[NCH], vc[NCH], kn[NCH], vn[NCH];
    load_rows(j0 + tg, kc, vc);

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
        for (int n = 0; n < NCH; ++n)
#pragma unroll
            for (int v = 0; v < VEC; ++v) qf[m][n][v] = m < G ? sQ[m][(li + 16 * n) * VEC + v] : 0.f;

    float mx[GMAX], l[GMAX], acc[GMAX][NCH][VEC];
#pragma unroll
    for (int m = 0; m < GMAX; ++m) {
        mx[m] = -INFINITY; l[m] = 0.f;
#pragma unroll
        for (int n = 0; n < NCH; ++n)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[m][n][v] = 0.f;
    }

    auto consume = [&](const u32x4* kp, const u32x4* vp) {
        float kf[NCH][VEC], vf[NCH][VEC];
#pragma unroll
        for (int n = 0; n < NCH; ++n) { elem<T>::unpack(kp[n], kf[n]); elem<T>::unpack(vp[n], vf[n]); }
#pragma unroll
        for (int m = 0; m < GMAX; ++m) {
            if (m < G) {  // uniform
                float x = 0.f;
#pragma unroll
                for (int n = 0; n < NCH; ++n)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) x = fmaf(qf[m][n][v], kf[n][v], x);
                x = row16_sum(x);
                const float mn = fmaxf(mx[m], x);
                const float r = __expf(mx[m] - mn), p = __expf(x - mn);  // exp(-inf) = 0 on the first token
                mx[m] = mn;
                l[m] = l[m] * r + p;
#pragma unroll
                for (int n = 0; n < NCH; ++n)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) acc[m][n][v] = fmaf(p, vf[n][v], acc[m][n][v] * r);
            }
        }
    };
    // two register sets take turns (a copy between them would wait for the loads it moves)
    for (int j = j0 + tg; j < j1; j += 32) {
        load_rows(j + 16, kn, vn);
        consume(kc, vc);
        if (j + 16 < j1) {
            load_rows(j + 32, kc, vc);
            consume(kn, vn);
        }
    }

    // the 16 lane groups of the workgroup, merged in group order by 128 threads (one per channel)
#pragma unroll
    for (int m = 0; m < GMAX; ++m) {
        if (m < G) {  // uniform
            __syncthreads();
            if (li == 0) { sRed[tg][0] = mx[m]; sRed[tg][1] = l[m]; }
#pragma unroll
            for (int n = 0; n < NCH; ++n)
#pragma unroll
                for (int v = 0; v < VEC; ++v) sRed[tg][2 + (li + 16 * n) * VEC + v] = acc[m][n][v];
            __syncthreads();
            if (tid < kHeadDim) {
                const int c = tid;
                float M = -INFINITY;
#pragma unroll
                for (int g = 0; g < 16; ++g) M = fmaxf(M, sRed[g][0]);
                float L = 0.f, A = 0.f;
                if (M > -INFINITY) {
#pragma unroll
                    for (int g = 0; g < 16; ++g) {
                        const float w = __expf(sRed[g][0] - M);
                        L = fmaf(sRed[g][1], w, L);
                        A = fmaf(sRed[g][2 + c], w, A);
                    }
                }
                float* rec = part + (((size_t)b * H + kvh * G + m) * n_chunks + chunk) * kDnRec;
                if (c == 0) { rec[0] = M; rec[1] = L; }
                rec[2 + c] = A;
            }
        }
    }
}

// out[b,h] = merged chunks / normaliser, rounded once to T.  grid (B*H), 128 threads.  The chunk records are
// read eight at a time (a loop with one load per round would cost a memory round trip per chunk).
template <typename T>
__global__ __launch_bounds__(128) void dense_merge_kernel(const float* __restrict__ part, T* __restrict__ out,
                                                          int n_chunks)
{
    const size_t bh = blockIdx.x;
    const int c = threadIdx.x;
    const float* rec = part + bh * n_chunks * kDnRec;
    float M = -INFINITY;
    for (int k0 = 0; k0 < n_chunks; k0 += 8) {
        float m8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) m8[u] = rec[(size_t)min(k0 + u, n_chunks - 1) * kDnRec];
#pragma unroll
        for (int u = 0; u < 8; ++u) M = fmaxf(M, m8[u]);
    }
    float L = 0.f, A = 0.f;
    if (M > -INFINITY) {
        for (int k0 = 0; k0 < n_chunks; k0 += 8) {
            float m8[8], l8[8], a8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float* r = rec + (size_t)min(k0 + u, n_chunks - 1) * kDnRec;
                m8[u] = r[0]; l8[u] = r[1]; a8[u] = r[2 + c];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float w = k0 + u < n_chunks ? __expf(m8[u] - M) : 0.f;
                L = fmaf(l8[u], w, L);
                A = fmaf(a8[u], w, A);
            }
        }
    }
    elem<T>::store(out + bh * kHeadDim + c, L > 0.f ? A / L : 0.f);
}

}  // namespace sals
