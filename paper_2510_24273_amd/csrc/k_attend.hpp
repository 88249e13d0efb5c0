// Selective reconstruction, RoPE and sparse attention (Sec. 4.4, Eq. 5;
// Algorithm 1, reconstruction to output steps).
//
//   attend_logits  K_C = K~_C U_k^T on the matrix cores; RoPE and q.K in the epilogue, so the
//                  reconstructed keys never leave registers.  Also rotates the query in its
//                  prologue and leaves, per (head, token tile), the softmax maximum and
//                  normaliser of the tile.
//   attend_pv      combines the tile statistics into the softmax of Eq. 5 and forms
//                  T[h,:] = sum_j p_hj V~_C[j,:]                 (latent-space value sum)
//   attend_out     y[h] = T[h,:] U_v[g(h) block]^T               (one pass over U_v)
//
// The value product uses  p (V~_C U_v^T) = (p V~_C) U_v^T : the same sum in another
// order, which avoids reconstructing V_C.
//
// Head dims are handled in "pair order": slot p < 64 is the first element of RoPE pair
// p, slot 64+p its partner, for either pairing style; the packed U_k panel (see
// pack_weights_kernel) already has its rows in that order, so both elements of a pair land
// in the same lane of the MFMA result.
//
// RoPE angles.  The angle of token position t and pair p is t * theta^(-2p/d), evaluated in
// fp64.  The query's cos/sin are computed in the logits kernel; those of the cached tokens
// come from a table over the positions 0 .. S_max that is filled once per context.
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

// cos/sin of every (position, pair): tab[t][p] = (cos, sin)(t * f_p)
__global__ __launch_bounds__(256) void rope_table_kernel(float2* __restrict__ tab, InvFreq inv, int rows)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (size_t)rows * kPairs) return;
    double sn, c;
    sincos((double)(e / kPairs) * inv.f[e % kPairs], &sn, &c);
    tab[e] = make_float2((float)c, (float)sn);
}

constexpr int kMaxGroup = 8;                 // query heads per KV head

// softmax statistics of a set of logits: maximum m and sum of exp(x - m)
__device__ __forceinline__ float2 stat_merge(float2 a, float2 b)
{
    const float m = fmaxf(a.x, b.x);
    if (m == -INFINITY) return make_float2(-INFINITY, 0.f);
    return make_float2(m, a.y * __expf(a.x - m) + b.y * __expf(b.x - m));
}

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

}  // namespace sals
