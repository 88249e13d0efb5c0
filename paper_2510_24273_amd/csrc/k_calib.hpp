// Offline calibration (Sec. 4.2): covariance of the calibration keys, C = K^T K, and its leading eigenvectors.
//
//   covariance   The contraction runs over the tokens, the axis along which the keys are NOT contiguous.  The keys of
//                a chunk are therefore transposed once (calib_transpose_kernel, a plain LDS tile transpose) and the
//                product is then the row-by-row form the matrix-core GEMM of the prompt compression computes,
//                C += K^T (K^T)^T, with fp32 tile sums added to the fp64 matrix per chunk.
//   eigenvectors One-sided Jacobi on the rows of G = C: a plane rotation of rows p, q makes them orthogonal.  With R the
//                product of all rotations, G = R C; once all rows are orthogonal, G G^T = R C^2 R^T is diagonal, so
//                the normalised rows of G are eigenvectors of C^2, hence of the positive semi-definite C, and the row
//                norms are the eigenvalues.  A step rotates D/2 disjoint pairs at once (round-robin pairing, D - 1
//                steps visit every pair: one sweep), one workgroup per pair, all accesses along contiguous rows, fp64
//                throughout; nothing but G itself is kept.  Rows whose norm is below 1e-13 of the largest stand for
//                eigenvalues that are zero to working precision and are left alone.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kCalTile = 64;        // transpose tile (elements)
constexpr int kCalThreads = 256;    // Jacobi workgroup
constexpr int kCalMaxEpt = 32;      // row elements per thread: D <= 8192
constexpr int kCalMaxD = kCalThreads * kCalMaxEpt;

// XT[d, t] = X[t, d] for t < n, zero for n <= t < n_pad; X [n, D], XT [D, n_pad]
template <typename T>
__global__ __launch_bounds__(256) void calib_transpose_kernel(const T* __restrict__ X, T* __restrict__ XT, long long n, int D,
                                                              long long n_pad)
{
    __shared__ T tile[kCalTile][kCalTile + 2];
    const long long t0 = (long long)blockIdx.x * kCalTile;
    const int d0 = blockIdx.y * kCalTile;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 x 4
#pragma unroll
    for (int i = 0; i < kCalTile; i += 4) {
        const long long t = t0 + ty + i;
        const int d = d0 + tx;
        T v;
        if (t < n && d < D) v = X[(size_t)t * D + d];
        else {
            if constexpr (sizeof(T) == 2) v = 0; else v = 0.f;
        }
        tile[ty + i][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kCalTile; i += 4) {
        const int d = d0 + ty + i;
        const long long t = t0 + tx;
        if (d < D && t < n_pad) XT[(size_t)d * n_pad + t] = tile[tx][ty + i];
    }
}

// C[i, j] += sum over the slices of P[slice][i, j], for the elements the covariance kernel computed: those of the
// tiles (tile_rows x tile_cols) that reach the upper triangle.  Slices are added in slice order, in fp64.
__global__ __launch_bounds__(256) void calib_reduce_kernel(double* __restrict__ C, const float* __restrict__ P, int D,
                                                           int slices, int tile_rows, int tile_cols)
{
    const size_t e = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;  // four consecutive columns
    if (e >= (size_t)D * D) return;
    const int i = (int)(e / D), j = (int)(e % D);
    if (j / tile_cols < (i / tile_rows) * (tile_rows / tile_cols)) return;  // tile not computed (mirrored later)
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    for (int z = 0; z < slices; ++z) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(P + (size_t)z * D * D + e);
        s0 += (double)v.x; s1 += (double)v.y; s2 += (double)v.z; s3 += (double)v.w;
    }
    C[e] += s0; C[e + 1] += s1; C[e + 2] += s2; C[e + 3] += s3;
}

// C[i, j] = C[j, i] for i > j: the covariance kernel fills the tiles that reach the upper triangle only
__global__ __launch_bounds__(256) void calib_mirror_kernel(double* __restrict__ C, int D)
{
    __shared__ double tile[32][33];
    const int bi = blockIdx.y, bj = blockIdx.x;   // tile of rows bi*32.., columns bj*32..
    if (bj > bi) return;                           // (strictly upper tiles are sources only)
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
#pragma unroll
    for (int k = 0; k < 32; k += 8) tile[ty + k][tx] = C[(size_t)(bj * 32 + ty + k) * D + bi * 32 + tx];  // the upper twin, [col][row]
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 32; k += 8) {
        const int i = bi * 32 + ty + k, j = bj * 32 + tx;
        if (i > j) C[(size_t)i * D + j] = tile[tx][ty + k];
    }
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// pair k of step s in the round-robin schedule over n (even) rows: n - 1 steps, every pair once
__device__ __forceinline__ void calib_pair(int n, int s, int k, int* p, int* q)
{
    if (k == 0) { *p = n - 1; *q = s; return; }
    const int m = n - 1;
    *p = (s + k) % m;
    *q = (s - k + m) % m;
}

// One step: workgroup k rotates rows (p, q) of G so that they become orthogonal.
// conv[k] keeps the largest |tan| of a rotation angle this workgroup slot has applied, since the host cleared it, to a
// pair with at least one row of norm >= lead (the rows that can still change a leading eigenvector); floor: rows
// with a smaller norm are left alone.
__global__ __launch_bounds__(kCalThreads) void calib_jacobi_step_kernel(double* __restrict__ G, int D, int step,
                                                                        double floor, double lead, double* __restrict__ conv)
{
    __shared__ double red[3][kCalThreads / kWave];
    int p, q;
    calib_pair(D, step, blockIdx.x, &p, &q);
    if (p > q) { const int t = p; p = q; q = t; }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ept = D / kCalThreads;  // D is a multiple of kCalThreads
    double* gp = G + (size_t)p * D; double* gq = G + (size_t)q * D;
    double a[kCalMaxEpt], b[kCalMaxEpt];
    double aa = 0.0, bb = 0.0, ab = 0.0;
#pragma unroll
    for (int e = 0; e < kCalMaxEpt; ++e) {
        if (e < ept) {  // uniform
            a[e] = gp[e * kCalThreads + tid];
            b[e] = gq[e * kCalThreads + tid];
        } else {
            a[e] = 0.0; b[e] = 0.0;
        }
    }
#pragma unroll
    for (int e = 0; e < kCalMaxEpt; ++e) { aa += a[e] * a[e]; bb += b[e] * b[e]; ab += a[e] * b[e]; }
    aa = wave_sum_f64(aa); bb = wave_sum_f64(bb); ab = wave_sum_f64(ab);
    if (lane == 0) { red[0][wave] = aa; red[1][wave] = bb; red[2][wave] = ab; }
    __syncthreads();
    aa = 0.0; bb = 0.0; ab = 0.0;
#pragma unroll
    for (int w = 0; w < kCalThreads / kWave; ++w) { aa += red[0][w]; bb += red[1][w]; ab += red[2][w]; }  // same order in every thread
    const double na = sqrt(aa), nb = sqrt(bb);
    if (!(fmin(na, nb) > floor)) return;                 // a row that stands for a zero eigenvalue
    if (!(fabs(ab) > 1e-15 * na * nb)) return;           // orthogonal to working precision
    // rotation that zeroes g_p . g_q:  t = tan(phi), the smaller root of  t^2 + 2 zeta t - 1 = 0
    const double zeta = (bb - aa) / (2.0 * ab);
    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
    const double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
    if (tid == 0 && fmax(na, nb) >= lead) conv[blockIdx.x] = fmax(conv[blockIdx.x], fabs(t));
#pragma unroll
    for (int e = 0; e < kCalMaxEpt; ++e) {
        if (e < ept) {
            gp[e * kCalThreads + tid] = c * a[e] - s * b[e];
            gq[e * kCalThreads + tid] = s * a[e] + c * b[e];
        }
    }
}

// norm of every row (the eigenvalue estimate lambda_i) and the sign that makes the row's largest component positive
__global__ __launch_bounds__(kCalThreads) void calib_rownorm_kernel(const double* __restrict__ G, int D, double* __restrict__ lam,
                                                                    double* __restrict__ sgn)
{
    __shared__ double red[kCalThreads / kWave], bestv[kCalThreads / kWave], bests[kCalThreads / kWave];
    __shared__ int besti[kCalThreads / kWave];
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    double acc = 0.0, bv = -1.0, bs = 1.0;
    int bi = 0;
    for (int d = tid; d < D; d += kCalThreads) {
        const double g = G[(size_t)i * D + d];
        acc += g * g;
        if (fabs(g) > bv) { bv = fabs(g); bi = d; bs = g < 0.0 ? -1.0 : 1.0; }
    }
    acc = wave_sum_f64(acc);
    // largest |component|, the first index among equals
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double ov = __shfl_xor(bv, o, kWave), os = __shfl_xor(bs, o, kWave);
        const int oi = __shfl_xor(bi, o, kWave);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; bs = os; }
    }
    if (lane == 0) { red[wave] = acc; bestv[wave] = bv; besti[wave] = bi; bests[wave] = bs; }
    __syncthreads();
    if (tid == 0) {
        double sum = 0.0;
        for (int w = 0; w < kCalThreads / kWave; ++w) sum += red[w];
        int best = 0;
        for (int w = 1; w < kCalThreads / kWave; ++w)
            if (bestv[w] > bestv[best] || (bestv[w] == bestv[best] && besti[w] < besti[best])) best = w;
        lam[i] = sqrt(sum);
        sgn[i] = bests[best];
    }
}

// Row i takes rank = number of rows with a larger norm (equal ones by row index); eigval[rank] = lambda_i and, for
// rank < r, column rank of U [D, r] = sgn_i * row i of G / lambda_i, rounded to the storage type (a zero row gives a
// zero column).
template <typename T>
__global__ __launch_bounds__(kCalThreads) void calib_select_kernel(const double* __restrict__ G, const double* __restrict__ lam,
                                                                   const double* __restrict__ sgn, int D, int r,
                                                                   double* __restrict__ eigval, T* __restrict__ U)
{
    __shared__ int cnt[kCalThreads / kWave];
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double li = lam[i];
    int c = 0;
    for (int j = tid; j < D; j += kCalThreads) {
        const double lj = lam[j];
        c += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, kWave);
    if (lane == 0) cnt[wave] = c;
    __syncthreads();
    int rank = 0;
#pragma unroll
    for (int w = 0; w < kCalThreads / kWave; ++w) rank += cnt[w];
    if (tid == 0) eigval[rank] = li;
    if (rank < r) {
        const double s = li > 0.0 ? sgn[i] / li : 0.0;
        for (int d = tid; d < D; d += kCalThreads) elem<T>::store(U + (size_t)d * r + rank, (float)(s * G[(size_t)i * D + d]));
    }
}

}  // namespace sals
