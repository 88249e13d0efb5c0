// Latent projection  x~ = U^T x  (Sec. 4.3; Algorithm 1, projection step) and the one-time
// repacking of the projectors.
//
// The projection reads the TRANSPOSED projector U^T [r x D] (made once by pack_weights),
// so each output coordinate is a dot product along a contiguous row: a workgroup owns 16
// latent coordinates and one slice of the D axis (the slices' partial sums are added by
// the score kernel, in slice order), its 4 waves split the slice, and every wave keeps all
// of its 16-byte row pieces in flight at once.  The products run on 16x16 MFMA tiles whose
// columns are the (sequence, query head of the KV group) pairs, so a whole batch costs
// one pass over U^T; the heads of a group are added in fp32 afterwards, which equals
// projecting their sum.  Single pass, fixed summation order, bit-reproducible.
#pragma once
#include "common.hpp"

namespace sals {

typedef float f32x4v __attribute__((ext_vector_type(4)));

template <typename T> struct mma16_op;
template <> struct mma16_op<bf16_t> {  // v_mfma_f32_16x16x32_bf16
    static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x4v& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                    c, 0, 0, 0);
    }
};
template <> struct mma16_op<float> {   // four v_mfma_f32_16x16x4_f32
    static __device__ __forceinline__ void run(const u32x4& a, const u32x4& b, f32x4v& c)
    {
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    }
};

constexpr int kProjWaves = 4;
constexpr int kProjThreads = 64 * kProjWaves;
constexpr int kProjMaxCols = 128;  // B * (H_q / H_kv) handled per call
constexpr int kProjBatch = 8;      // row pieces a wave keeps in flight per round

struct ProjArgs {  // (what the first loads need comes first: those 14 words arrive preloaded in scalar registers)
    const void* UT[2];   // transposed projectors [r, D]
    const void* X[2];    // QUERY: q [B,H,d] (X[0]); else new key / value [B,D]
    int D, np, B, H, H_kv, r;
    int d, S_max, nproj;
    int ring;            // append: > 0 = the cache is a ring of this many rows, token t in row t mod ring
    void* cache[2];      // append: [B,S_max,r], or [B,ring,r] when ring > 0
    float* out_f32;      // QUERY: partial q~ [np,B,r], one slice of the D axis each
    const int32_t* seq_len;  // append: [B] row to write
};

template <typename T, bool QUERY>
__global__ __launch_bounds__(kProjThreads) void project_kernel(ProjArgs a)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int KS = 4 * VEC;  // elements of the D axis per MFMA step
    const int proj = blockIdx.z, slice = blockIdx.y;
    const int i0 = blockIdx.x * 16;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int G = QUERY ? a.H / a.H_kv : 1;
    const int ncols = a.B * G, n_nblk = (ncols + 15) >> 4;
    const int nks_all = a.D / KS, nks = nks_all / a.np;   // steps of this workgroup's slice
    const int ks_first = slice * nks;
    const T* UT = static_cast<const T*>(a.UT[proj]);
    const T* X = static_cast<const T*>(a.X[proj]);
    const T* arow = UT + (size_t)(i0 + l16) * a.D + kg * VEC;

    __shared__ __attribute__((aligned(16))) float red[kProjWaves][64][4];
    __shared__ float colsum[kProjMaxCols][16];

    f32x4v acc[kProjMaxCols / 16];
#pragma unroll
    for (int nb = 0; nb < kProjMaxCols / 16; ++nb) acc[nb] = f32x4v{0.f, 0.f, 0.f, 0.f};

    // this wave's steps: wave, wave+4, ... ; kProjBatch steps of loads per round
    for (int ks0 = wave; ks0 < nks; ks0 += kProjWaves * kProjBatch) {
        u32x4 af[kProjBatch];
#pragma unroll
        for (int u = 0; u < kProjBatch; ++u) {
            int ks = ks0 + u * kProjWaves;
            af[u] = ks < nks ? ld16(arow + (size_t)(ks_first + ks) * KS) : u32x4{0, 0, 0, 0};
        }
        // the x operands of two column blocks are requested together, ahead of their products: a round costs
        // one memory round trip per pair of column blocks
#pragma unroll
        for (int nb0 = 0; nb0 < kProjMaxCols / 16; nb0 += 2) {
            if (nb0 < n_nblk) {  // uniform
                u32x4 bf[2][kProjBatch];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int n = (nb0 + h) * 16 + l16;
#pragma unroll
                    for (int u = 0; u < kProjBatch; ++u) {
                        int ks = ks0 + u * kProjWaves;
                        bf[h][u] = u32x4{0, 0, 0, 0};
                        if (ks < nks && n < ncols) {
                            int c = (ks_first + ks) * KS + kg * VEC;
                            const T* xp;
                            if (QUERY) {
                                int b = n / G, m = n - b * G, g = c / a.d;
                                xp = X + ((size_t)b * a.H + g * G + m) * a.d + (c - g * a.d);
                            } else {
                                xp = X + (size_t)n * a.D + c;
                            }
                            bf[h][u] = ld16(xp);
                        }
                    }
                }
                asm volatile("" ::: "memory");  // (keeps the loads above from sinking towards their products)
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int u = 0; u < kProjBatch; ++u) mma16_op<T>::run(af[u], bf[h][u], acc[nb0 + h]);
            }
        }
    }

    // fold the four waves' sums in wave order; acc[nb][v] is (coordinate 4*kg+v, column nb*16+l16)
#pragma unroll
    for (int nb = 0; nb < kProjMaxCols / 16; ++nb) {
        if (nb < n_nblk) {  // uniform
            __syncthreads();
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][lane][v] = acc[nb][v];
            __syncthreads();
            {
                int col = tid & 15, rr = tid >> 4;
                int src_lane = (rr >> 2) * 16 + col, v = rr & 3;
                float s = 0.f;
#pragma unroll
                for (int w = 0; w < kProjWaves; ++w) s += red[w][src_lane][v];
                colsum[nb * 16 + col][rr] = s;
            }
        }
    }
    __syncthreads();
    // add the heads of each group and write
    for (int t = tid; t < a.B * 16; t += kProjThreads) {
        int b = t >> 4, rr = t & 15;
        float s = 0.f;
        for (int m = 0; m < G; ++m) s += colsum[b * G + m][rr];
        if (QUERY) {
            a.out_f32[((size_t)slice * a.B + b) * a.r + i0 + rr] = s;
        } else {
            const int t_new = a.seq_len[b];
            const int rows = a.ring > 0 ? a.ring : a.S_max;
            const int row = a.ring > 0 ? t_new % a.ring : t_new;
            if (t_new >= 0 && t_new < a.S_max)
                elem<T>::store(static_cast<T*>(a.cache[proj]) + ((size_t)b * rows + row) * a.r + i0 + rr, s);
        }
    }
}

// after an append: advance the sequence lengths (separate launch, so that every cache row
// has been written before any length changes)
__global__ void bump_seq_len_kernel(int32_t* __restrict__ seq_len, int B, int S_max)
{
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B && seq_len[b] < S_max) seq_len[b] += 1;
}

// ---------------------------------------------------------------------------------
// one-time weight repacking (model-load time; not on the decode path)
// ---------------------------------------------------------------------------------
// section 0: UkT [r, D]      section 1: UvT [r, D]
// section 2: Uk in reconstruction order: [H_kv][r/KE][128 slots][KE] (KE = 64 bytes of the latent
//            axis) with the head dims in RoPE pair order (slot p < 64: first element of pair p; 64+p: its partner)
// section 3: Uv [D, r] unchanged
template <typename T>
__global__ __launch_bounds__(256) void pack_weights_kernel(const T* __restrict__ Uk, const T* __restrict__ Uv,
                                                           T* __restrict__ packed, size_t section_elems,
                                                           int D, int r, int style)
{
    constexpr int KE = 64 / (int)sizeof(T);
    const int sec = blockIdx.y;
    T* dst = packed + (size_t)sec * section_elems;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < section_elems; e += (size_t)gridDim.x * 256) {
        T v;
        if (sec == 0 || sec == 1) {
            size_t i = e / D, c = e - i * D;
            v = (sec == 0 ? Uk : Uv)[c * r + i];
        } else if (sec == 2) {
            size_t per_head = (size_t)kHeadDim * r;
            size_t g = e / per_head, rem = e - g * per_head;
            size_t kc = rem / ((size_t)kHeadDim * KE), rem2 = rem - kc * kHeadDim * KE;
            int slot = (int)(rem2 / KE), ke = (int)(rem2 - (size_t)slot * KE);
            int dim = slot < kPairs ? (style ? 2 * slot : slot) : (style ? 2 * (slot - kPairs) + 1 : slot);
            v = Uk[(g * kHeadDim + dim) * r + kc * KE + ke];
        } else {
            v = Uv[e];
        }
        dst[e] = v;
    }
}

}  // namespace sals
