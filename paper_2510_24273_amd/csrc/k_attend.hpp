// Selective reconstruction, RoPE and sparse attention (Sec. 4.4, Eq. 5;
// Algorithm 1, reconstruction to output steps).
//
//   attend_prep    cos/sin of (position x frequency) for every selected token, and the
//                  rotated, 1/sqrt(d)-scaled query, both in fp64-accurate angles
//   attend_logits  K_C = K~_C U_k^T on the matrix cores, RoPE and q.K in the epilogue;
//                  the reconstructed keys never leave registers
//   attend_stats   per (sequence, head) softmax maximum and normaliser
//   attend_pv      T[h,:] = sum_j exp(l_hj - m_h) V~_C[j,:]      (latent-space value sum)
//   attend_out     y[h] = (T[h,:] U_v[g(h) block]^T) / Z_h       (one pass over U_v)
//
// The value product uses  p (V~_C U_v^T) = (p V~_C) U_v^T : the same sum in another
// order, which avoids reconstructing V_C.
//
// Head dims are handled in "pair order": slot p < 64 is the first element of RoPE pair
// p, slot 64+p its partner, for either pairing style; the packed U_k panel (see
// pack_weights_kernel) already has its rows in that order, so both elements of a pair land
// in the same lane of the MFMA result.
#pragma once
#include "common.hpp"

namespace sals {

__device__ __forceinline__ int pair_first(int p, int style) { return style ? 2 * p : p; }
__device__ __forceinline__ int pair_second(int p, int style) { return style ? 2 * p + 1 : p + kPairs; }
__device__ __forceinline__ int slot_to_dim(int slot, int style)
{
    return slot < kPairs ? pair_first(slot, style) : pair_second(slot - kPairs, style);
}

struct InvFreq { double f[kPairs]; };  // theta^(-2p/d), computed on the host in fp64

// ---------------------------------------------------------------------------------
// prep
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attend_prep_kernel(const T* __restrict__ q,
                                                          const int32_t* __restrict__ q_pos,
                                                          const int32_t* __restrict__ idx,
                                                          const int32_t* __restrict__ n_sel,
                                                          float2* __restrict__ cs, float* __restrict__ qR,
                                                          InvFreq inv, int B, int H, int k_tot,
                                                          int n_tab_blocks, int style, float scale)
{
    const int p = threadIdx.x & 63, sub = threadIdx.x >> 6;
    if ((int)blockIdx.x < n_tab_blocks) {
        int slot = blockIdx.x * 4 + sub;  // flat (b, j)
        if (slot >= B * k_tot) return;
        int b = slot / k_tot, j = slot - b * k_tot;
        int pos = j < n_sel[b] ? idx[slot] : 0;
        double sn, c;
        sincos((double)pos * inv.f[p], &sn, &c);
        cs[(size_t)slot * kPairs + p] = make_float2((float)c, (float)sn);
    } else {
        int bh = (blockIdx.x - n_tab_blocks) * 4 + sub;  // flat (b, h)
        if (bh >= B * H) return;
        int b = bh / H;
        double sn, c;
        sincos((double)q_pos[b] * inv.f[p], &sn, &c);
        float x1 = elem<T>::load(q + (size_t)bh * kHeadDim + pair_first(p, style));
        float x2 = elem<T>::load(q + (size_t)bh * kHeadDim + pair_second(p, style));
        float cf = (float)c, sf = (float)sn;
        qR[(size_t)bh * kHeadDim + p] = (x1 * cf - x2 * sf) * scale;
        qR[(size_t)bh * kHeadDim + kPairs + p] = (x2 * cf + x1 * sf) * scale;
    }
}

// ---------------------------------------------------------------------------------
// logits: gathered-row GEMM on MFMA with RoPE + q.K epilogue
// ---------------------------------------------------------------------------------
constexpr int kMaxGroup = 8;                 // query heads per KV head

template <typename T> struct mma_op;
template <> struct mma_op<bf16_t> {  // one v_mfma_f32_32x32x16_bf16 per 16-byte fragment pair
    static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                    __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
};
template <> struct mma_op<float> {   // four v_mfma_f32_32x32x2_f32 per 16-byte fragment pair
    static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x16& c)
    {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------------
// softmax over the selected tokens (Eq. 5): one workgroup per (sequence, head) row turns
// the logits into normalised weights stored for the matrix cores: a bf16 head plane and
// a bf16 remainder plane (fp32 storage: one fp32 plane), zero past the selected tokens.
// ---------------------------------------------------------------------------------
constexpr int kSmThreads = 256;
constexpr int kSmBatch = 8;  // values per thread per round; the first round stays in registers

__device__ __forceinline__ float block_reduce_256(float v, float* sh, bool is_max)
{
    v = is_max ? wave_max(v) : wave_sum(v);
    __syncthreads();
    if (lane_id() == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float a = sh[0], b = sh[1], c = sh[2], d = sh[3];
    return is_max ? fmaxf(fmaxf(a, b), fmaxf(c, d)) : (a + b) + (c + d);
}

template <typename T>
__global__ __launch_bounds__(kSmThreads) void attend_softmax_kernel(const float* __restrict__ logits,
                                                                    const int32_t* __restrict__ n_sel,
                                                                    T* __restrict__ P, int B, int H, int lk)
{
    __shared__ float sh[4];
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int n = n_sel[bh / H];
    const float* lrow = logits + (size_t)bh * lk;
    T* p_hi = P + (size_t)bh * lk;
    T* p_lo = P + (size_t)B * H * lk + (size_t)bh * lk;  // second plane (bf16 storage only)
    constexpr int SPAN = kSmThreads * kSmBatch;

    float first[kSmBatch];
#pragma unroll
    for (int u = 0; u < kSmBatch; ++u) { int j = u * kSmThreads + tid; first[u] = j < n ? lrow[j] : -INFINITY; }
    float mx = -INFINITY;
#pragma unroll
    for (int u = 0; u < kSmBatch; ++u) mx = fmaxf(mx, first[u]);
    for (int j0 = SPAN; j0 < n; j0 += SPAN) {
        float v[kSmBatch];
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) { int j = j0 + u * kSmThreads + tid; v[u] = j < n ? lrow[j] : -INFINITY; }
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) mx = fmaxf(mx, v[u]);
    }
    mx = block_reduce_256(mx, sh, true);
    float z = 0.f;
#pragma unroll
    for (int u = 0; u < kSmBatch; ++u) z += first[u] > -INFINITY ? __expf(first[u] - mx) : 0.f;
    for (int j0 = SPAN; j0 < n; j0 += SPAN) {
        float v[kSmBatch];
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) { int j = j0 + u * kSmThreads + tid; v[u] = j < n ? lrow[j] : -INFINITY; }
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) z += v[u] > -INFINITY ? __expf(v[u] - mx) : 0.f;
    }
    z = block_reduce_256(z, sh, false);
    const float zi = z > 0.f ? 1.f / z : 0.f;
    for (int j0 = 0; j0 < lk; j0 += SPAN) {
        float v[kSmBatch];
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) {
            int j = j0 + u * kSmThreads + tid;
            v[u] = j0 == 0 ? first[u] : (j < n ? lrow[j] : -INFINITY);
        }
#pragma unroll
        for (int u = 0; u < kSmBatch; ++u) {
            int j = j0 + u * kSmThreads + tid;
            if (j < lk) {
                float pj = v[u] > -INFINITY ? __expf(v[u] - mx) * zi : 0.f;
                if constexpr (sizeof(T) == 2) {
                    bf16_t ph = f32_to_bf16(pj);
                    p_hi[j] = ph;
                    p_lo[j] = f32_to_bf16(pj - bf16_to_f32(ph));
                } else {
                    p_hi[j] = pj;
                }
            }
        }
    }
}

}  // namespace sals
