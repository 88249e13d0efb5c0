// The value path of the sparse attention (Eq. 5; Algorithm 1, output step), evaluated as
// y_h = ((p_h V~_C) U_v[g(h) block]^T) : the same sum as p_h (V~_C U_v^T) in another order,
// so the selected values are never reconstructed.
//
//   attend_pv   per (sequence, token range, 32 latent columns):
//               T[h,:] = sum_j p_hj V~[C_j,:]  on the matrix cores, tokens being the
//               contraction axis (split over the four waves).  The softmax weights are formed
//               on the fly, p = exp(logit - m_h) / Z_h, with m_h and Z_h merged in the prologue
//               from the per-tile statistics the logits kernel left.  With one range T is
//               written in matrix-core form; with several, each range writes an fp32 partial sum.
//   attend_out  y[(b,h), c] = sum_i T[(b,h), i] U_v[g*128 + c, i]  on the matrix cores; adds the
//               range partials in order first when there are several.
//
// bf16 storage: the fp32 weights p and the fp32 T are split into a bf16 head and a bf16
// remainder (two MFMAs each), which keeps about 16 mantissa bits.  fp32 storage: fp32 MFMAs.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"
#include "k_project.hpp"

namespace sals {

constexpr int kPvTJ = 64;          // tokens per wave step
constexpr int kPvCols = 32;        // latent columns per workgroup
constexpr int kPvMaxHeads = 64;    // H_q limit of these kernels
constexpr int kMaxRanges = 32;     // token ranges per sequence

// split an fp32 value for storage type T: bf16 -> (head, remainder); fp32 -> itself
template <typename T>
__device__ __forceinline__ void store_split(T* hi_arr, T* lo_arr, size_t at, float v)
{
    if constexpr (sizeof(T) == 2) {
        bf16_t h = f32_to_bf16(v);
        hi_arr[at] = h;
        lo_arr[at] = f32_to_bf16(v - bf16_to_f32(h));
    } else {
        hi_arr[at] = v;
    }
}

template <typename T>
__global__ __launch_bounds__(256, 2) void attend_pv_kernel(const T* __restrict__ Vc,
                                                        const int32_t* __restrict__ idx,
                                                        const int32_t* __restrict__ n_sel,
                                                        const float* __restrict__ logits,
                                                        const float2* __restrict__ stats, int n_parts,
                                                        float* __restrict__ Tpart, T* __restrict__ Tfin,
                                                        int B, int S_max, int r, int H, int k_tot, int lk,
                                                        int tok_per_wg, int n_tr)
{
    constexpr int VEC = elem<T>::vec;        // tokens per lane per MFMA group
    constexpr int KG = 2 * VEC;              // tokens per MFMA group (both half-waves)
    constexpr int NKG = kPvTJ / KG;
    constexpr bool kSplit = sizeof(T) == 2;

    __shared__ __attribute__((aligned(16))) float red[3][64][33];
    __shared__ float2 sMZ[kPvMaxHeads];  // per head: softmax maximum, 1 / normaliser

    const int b = blockIdx.z, tr = blockIdx.y, cb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hi = lane >> 5;
    const int n = n_sel[b];
    const int j_begin = min(n, tr * tok_per_wg), j_end = min(n, j_begin + tok_per_wg);
    const int col = cb * kPvCols + l32;
    const int n_mb = (H + 31) >> 5;
    const float* lg = logits + (size_t)b * H * lk;

    // softmax maximum and normaliser of every head: four lanes share a head's tiles and merge
    // them in a fixed order
    {
        const int h = tid >> 2, sub = tid & 3;
        float2 st = make_float2(-INFINITY, 0.f);
        if (h < H) {
            const float2* sp = stats + ((size_t)b * H + h) * n_parts;
            for (int t = sub; t < n_parts; t += 4) st = stat_merge(st, sp[t]);
        }
        st = stat_merge(st, make_float2(__shfl_xor(st.x, 1, kWave), __shfl_xor(st.y, 1, kWave)));
        st = stat_merge(st, make_float2(__shfl_xor(st.x, 2, kWave), __shfl_xor(st.y, 2, kWave)));
        if (sub == 0) sMZ[h] = make_float2(st.x > -INFINITY ? st.x : 0.f, st.y > 0.f ? 1.f / st.y : 0.f);
    }
    __syncthreads();
    float2 mz[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) mz[mb] = sMZ[mb * 32 + l32];
    const T* vbase = Vc + (size_t)b * S_max * r + col;
    const int32_t* ib = idx + (size_t)b * k_tot;
    T* Thi_arr = Tfin;
    T* Tlo_arr = Tfin + (size_t)B * H * r;

    f32x16 acc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mb][v] = 0.f;

    // every wave takes every fourth 64-token step of the range; weights past the selected
    // tokens are zero, so a ragged last step only has to read valid rows
    const int n_steps = (j_end - j_begin + kPvTJ - 1) / kPvTJ;
    for (int step = wave; step < n_steps; step += 4) {
        const int j0 = j_begin + step * kPvTJ;  // multiple of 64
        int rows[NKG][VEC];
#pragma unroll
        for (int ks = 0; ks < NKG; ++ks)
#pragma unroll
            for (int t = 0; t < VEC; ++t) {
                int j = min(j0 + ks * KG + hi * VEC + t, n - 1);
                rows[ks][t] = min(max(ib[j], 0), S_max - 1);
            }
        u32x4 ah[NKG][2], al[NKG][2];
#pragma unroll
        for (int ks = 0; ks < NKG; ++ks)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                const int h = mb * 32 + l32;
                const size_t off = (size_t)h * lk + j0 + ks * KG + hi * VEC;
                const bool ok = mb < n_mb && h < H;
                float pj[VEC];
#pragma unroll
                for (int v = 0; v < VEC; v += 4) {
                    const f32x4 x = ok ? *reinterpret_cast<const f32x4*>(lg + off + v)
                                       : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
                    // slots past the selected tokens carry no weight (their logits may be unwritten)
                    const int jt = j0 + ks * KG + hi * VEC + v;
                    pj[v] = jt < n ? __expf(x.x - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 1] = jt + 1 < n ? __expf(x.y - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 2] = jt + 2 < n ? __expf(x.z - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 3] = jt + 3 < n ? __expf(x.w - mz[mb].x) * mz[mb].y : 0.f;
                }
                if constexpr (kSplit) {
                    uint32_t ph[VEC], pl[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const bf16_t hb = f32_to_bf16(pj[v]);
                        ph[v] = hb;
                        pl[v] = f32_to_bf16(pj[v] - bf16_to_f32(hb));
                    }
                    ah[ks][mb] = u32x4{ph[0] | (ph[1] << 16), ph[2] | (ph[3] << 16), ph[4] | (ph[5] << 16),
                                       ph[6] | (ph[7] << 16)};
                    al[ks][mb] = u32x4{pl[0] | (pl[1] << 16), pl[2] | (pl[3] << 16), pl[4] | (pl[5] << 16),
                                       pl[6] | (pl[7] << 16)};
                } else {
                    ah[ks][mb] = u32x4{__float_as_uint(pj[0]), __float_as_uint(pj[1]), __float_as_uint(pj[2]),
                                       __float_as_uint(pj[3])};
                }
            }
        u32x4 vfrag[NKG];
#pragma unroll
        for (int ks = 0; ks < NKG; ++ks) {
            if constexpr (kSplit) {
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) e[t] = vbase[(size_t)rows[ks][t] * r];
                vfrag[ks] = u32x4{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                                  e[6] | (e[7] << 16)};
            } else {
                float e[4];
#pragma unroll
                for (int t = 0; t < 4; ++t) e[t] = vbase[(size_t)rows[ks][t] * r];
                vfrag[ks] = u32x4{__float_as_uint(e[0]), __float_as_uint(e[1]), __float_as_uint(e[2]),
                                  __float_as_uint(e[3])};
            }
        }
#pragma unroll
        for (int ks = 0; ks < NKG; ++ks)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                if (mb < n_mb) {
                    mma_op<T>::run(ah[ks][mb], vfrag[ks], acc[mb]);
                    if constexpr (kSplit) mma_op<T>::run(al[ks][mb], vfrag[ks], acc[mb]);
                }
            }
    }

    // add the four waves' sums in wave order; acc[mb][4a+c] is head mb*32+8a+4hi+c, column l32
    if (wave > 0) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave - 1][lane][mb * 16 + v] = acc[mb][v];
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                int h = mb * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
                if (h < H) {
                    float t = acc[mb][v] + red[0][lane][mb * 16 + v] + red[1][lane][mb * 16 + v] +
                              red[2][lane][mb * 16 + v];
                    if (n_tr == 1) store_split<T>(Thi_arr, Tlo_arr, ((size_t)b * H + h) * r + col, t);
                    else Tpart[(((size_t)tr * B + b) * H + h) * r + col] = t;
                }
            }
    }
}

// ---------------------------------------------------------------------------------
// output projection: y[(b,h), c] = sum_i T[(b,h), i] U_v[g*128 + c, i]
//
// One workgroup per (KV head, 16 output channels): 8 x H_kv workgroups, so that the single
// pass over U_v is spread over the whole chip.  16x16 MFMA tiles: rows are the (sequence,
// head of the group) pairs, columns the channels; the latent axis is split over the four
// waves, every wave issuing all of its loads as one batch.
// ---------------------------------------------------------------------------------
constexpr int kOutBatch = 8;  // latent steps of loads kept in flight per round

template <typename T>
__global__ __launch_bounds__(256) void attend_out_kernel(const T* __restrict__ Uv, const T* __restrict__ Tfin,
                                                         const float* __restrict__ Tpart, T* __restrict__ out,
                                                         int B, int r, int H, int H_kv, int n_tr)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int KS = 4 * VEC;  // latent coordinates per MFMA step
    constexpr bool kSplit = sizeof(T) == 2;
    __shared__ __attribute__((aligned(16))) float red[3][64][5];

    const int g = blockIdx.y, cb = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int G = H / H_kv;
    const int n_rows = B * G;  // (sequence, head of this group) pairs
    const int nks = r / KS;
    const T* urow = Uv + ((size_t)g * kHeadDim + cb * 16 + l16) * r + kg * VEC;
    const T* Thi_arr = Tfin;
    const T* Tlo_arr = Tfin + (size_t)B * H * r;
    const size_t tstride = (size_t)B * H * r;

    for (int row0 = 0; row0 < n_rows; row0 += 16) {
        const int row = row0 + l16;
        const bool row_ok = row < n_rows;
        const int bb = row_ok ? row / G : 0, h = row_ok ? g * G + row % G : 0;
        const size_t trow = ((size_t)bb * H + h) * r + kg * VEC;
        f32x4v acc = {0.f, 0.f, 0.f, 0.f};
        for (int ks0 = wave; ks0 < nks; ks0 += 4 * kOutBatch) {  // this wave: ks0, ks0+4, ...
            u32x4 bf[kOutBatch], ah[kOutBatch], al[kOutBatch];
#pragma unroll
            for (int u = 0; u < kOutBatch; ++u) {
                const int ks = ks0 + 4 * u;
                const bool ok = ks < nks;
                const int i0 = ks * KS;
                bf[u] = ok ? ld16(urow + i0) : u32x4{0, 0, 0, 0};
                ah[u] = u32x4{0, 0, 0, 0};
                al[u] = u32x4{0, 0, 0, 0};
                if (ok && row_ok) {
                    if (n_tr == 1) {
                        ah[u] = ld16(Thi_arr + trow + i0);
                        if constexpr (kSplit) al[u] = ld16(Tlo_arr + trow + i0);
                    } else {
                        // several token ranges: add their fp32 partial sums in range order, then split
                        float tm[VEC];
#pragma unroll
                        for (int v = 0; v < VEC; ++v) tm[v] = 0.f;
                        for (int t0 = 0; t0 < n_tr; t0 += 4) {
                            f32x4 x[4][VEC / 4];
#pragma unroll
                            for (int w = 0; w < 4; ++w)
#pragma unroll
                                for (int v = 0; v < VEC / 4; ++v)
                                    x[w][v] = t0 + w < n_tr
                                                  ? *reinterpret_cast<const f32x4*>(Tpart + (size_t)(t0 + w) * tstride +
                                                                                    trow + i0 + 4 * v)
                                                  : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int w = 0; w < 4; ++w)
#pragma unroll
                                for (int v = 0; v < VEC / 4; ++v) {
                                    tm[4 * v] += x[w][v].x; tm[4 * v + 1] += x[w][v].y;
                                    tm[4 * v + 2] += x[w][v].z; tm[4 * v + 3] += x[w][v].w;
                                }
                        }
                        if constexpr (kSplit) {
                            uint32_t hw[8], lw[8];
#pragma unroll
                            for (int v = 0; v < 8; ++v) {
                                bf16_t ph = f32_to_bf16(tm[v]);
                                hw[v] = ph;
                                lw[v] = f32_to_bf16(tm[v] - bf16_to_f32(ph));
                            }
                            ah[u] = u32x4{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16), hw[4] | (hw[5] << 16),
                                          hw[6] | (hw[7] << 16)};
                            al[u] = u32x4{lw[0] | (lw[1] << 16), lw[2] | (lw[3] << 16), lw[4] | (lw[5] << 16),
                                          lw[6] | (lw[7] << 16)};
                        } else {
                            ah[u] = u32x4{__float_as_uint(tm[0]), __float_as_uint(tm[1]), __float_as_uint(tm[2]),
                                          __float_as_uint(tm[3])};
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kOutBatch; ++u) {
                mma16_op<T>::run(ah[u], bf[u], acc);
                if constexpr (kSplit) mma16_op<T>::run(al[u], bf[u], acc);
            }
        }
        // fold the four latent slices (waves) in order; acc[v] is tile row 4*kg+v, channel l16
        __syncthreads();
        if (wave > 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave - 1][lane][v] = acc[v];
        }
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float y = acc[v] + red[0][lane][v] + red[1][lane][v] + red[2][lane][v];
                int orow = row0 + kg * 4 + v;
                if (orow < n_rows) {
                    int ob = orow / G, oh = g * G + orow % G;
                    elem<T>::store(out + ((size_t)ob * H + oh) * kHeadDim + cb * 16 + l16, y);
                }
            }
        }
    }
}

}  // namespace sals
