// Latent projection  x~ = U^T x  (Sec. 4.3; Algorithm 1, projection step).
//
// U is [D x r] row-major, so the reduction runs down the columns: the kernel
// streams U once for the whole batch (it is the only large operand), each
// workgroup owning a [rows_per_wg x CW] panel.  Partial sums of the row panels
// go to a workspace and the last workgroup to finish a column panel adds them
// up in a fixed order, so the result is bit-reproducible from run to run.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kProjThreads = 256;
constexpr int kProjRowLanes = 32;   // threads along the reduction axis
constexpr int kProjBT = 4;          // batch entries accumulated per pass
constexpr int kProjMaxRows = 256;   // max rows per workgroup panel

struct ProjArgs {
    const void* X[2];     // QUERY: q [B,H,d]; else [B,D]
    const void* U[2];     // [D,r]
    void* cache[2];       // append: [B,S_max,r]
    float* out_f32;       // QUERY: [B,r]
    float* partial;       // [nproj][nchunk][B][r]
    uint32_t* counters;   // [nproj*ncol] panel counters, then 1 "all done" counter
    int32_t* seq_len;     // append: [B], incremented at the very end
    int B, D, r, H, H_kv, d, S_max, rows_per_wg, nchunk, ncol, nproj;
};

template <typename T, bool QUERY>
__global__ __launch_bounds__(kProjThreads) void project_kernel(ProjArgs a)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int CW = 8 * VEC;  // columns per workgroup
    const int tid = threadIdx.x;
    const int tx = tid & 7, ty = tid >> 3;
    const int proj = blockIdx.z;
    const int col0 = blockIdx.x * CW;
    const int c_begin = blockIdx.y * a.rows_per_wg;
    const int c_end = min(a.D, c_begin + a.rows_per_wg);
    const T* X = static_cast<const T*>(a.X[proj]);
    const T* U = static_cast<const T*>(a.U[proj]);
    float* partial = a.partial + ((size_t)proj * a.nchunk + blockIdx.y) * a.B * a.r;

    __shared__ float xs[kProjBT][kProjMaxRows];
    __shared__ float red[kProjRowLanes][CW + 1];
    __shared__ int is_last;

    const int G = a.H / a.H_kv;
    for (int b0 = 0; b0 < a.B; b0 += kProjBT) {
        // stage the slice of x for this row panel (group-summed heads for a query)
        for (int t = tid; t < kProjBT * a.rows_per_wg; t += kProjThreads) {
            int bb = t / a.rows_per_wg, cc = t - bb * a.rows_per_wg;
            int b = b0 + bb, c = c_begin + cc;
            float v = 0.f;
            if (b < a.B && c < c_end) {
                if (QUERY) {
                    int g = c / a.d, e = c - g * a.d;
                    for (int m = 0; m < G; ++m)
                        v += elem<T>::load(X + ((size_t)b * a.H + g * G + m) * a.d + e);
                } else {
                    v = elem<T>::load(X + (size_t)b * a.D + c);
                }
            }
            xs[bb][cc] = v;
        }
        __syncthreads();
        float acc[kProjBT][VEC];
#pragma unroll
        for (int bb = 0; bb < kProjBT; ++bb)
#pragma unroll
            for (int v = 0; v < VEC; ++v) acc[bb][v] = 0.f;
        for (int c = c_begin + ty; c < c_end; c += kProjRowLanes) {
            float uf[VEC];
            elem<T>::unpack(ld16(U + (size_t)c * a.r + col0 + tx * VEC), uf);
#pragma unroll
            for (int bb = 0; bb < kProjBT; ++bb) {
                float xv = xs[bb][c - c_begin];
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[bb][v] = fmaf(xv, uf[v], acc[bb][v]);
            }
        }
        // reduce over the 32 row lanes, one batch entry at a time
#pragma unroll
        for (int bb = 0; bb < kProjBT; ++bb) {
            __syncthreads();
#pragma unroll
            for (int v = 0; v < VEC; ++v) red[ty][tx * VEC + v] = acc[bb][v];
            __syncthreads();
            if (tid < CW && b0 + bb < a.B) {
                float s = 0.f;
                for (int y = 0; y < kProjRowLanes; ++y) s += red[y][tid];
                partial[(size_t)(b0 + bb) * a.r + col0 + tid] = s;
            }
        }
        __syncthreads();
    }

    // last workgroup of this column panel adds the row-panel partials
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t old = atomicAdd(&a.counters[proj * a.ncol + blockIdx.x], 1u);
        is_last = (old == (uint32_t)a.nchunk - 1u);
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();
    const float* pbase = a.partial + (size_t)proj * a.nchunk * a.B * a.r;
    for (int t = tid; t < a.B * CW; t += kProjThreads) {
        int b = t / CW, col = col0 + (t - b * CW);
        float s = 0.f;
        for (int ch = 0; ch < a.nchunk; ++ch)
            s += __hip_atomic_load(pbase + ((size_t)ch * a.B + b) * a.r + col, __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
        if (QUERY) {
            a.out_f32[(size_t)b * a.r + col] = s;
        } else {
            int row = a.seq_len[b];
            if (row < a.S_max)
                elem<T>::store(static_cast<T*>(a.cache[proj]) + ((size_t)b * a.S_max + row) * a.r + col, s);
        }
    }
    if (tid == 0) a.counters[proj * a.ncol + blockIdx.x] = 0u;
    if (QUERY) return;
    // append: the very last panel (over both projections) advances the lengths
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        uint32_t* done = a.counters + a.nproj * a.ncol;
        uint32_t old = atomicAdd(done, 1u);
        is_last = (old == (uint32_t)(a.nproj * a.ncol) - 1u);
        if (is_last) *done = 0u;
    }
    __syncthreads();
    if (!is_last) return;
    for (int b = tid; b < a.B; b += kProjThreads)
        if (a.seq_len[b] < a.S_max) a.seq_len[b] += 1;
}

}  // namespace sals
