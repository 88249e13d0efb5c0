// Quantised full-rank value cache (Sec. 5.1; the V-hat of Algorithm 1).
//
// The paper keeps values at full rank and stores them with channel-wise group quantisation
// (4 bit at its 25 % setting, 2 bit at 12.5 %), following KIVI's asymmetric uniform scheme.
// Layout used here: a token's D_kv channels form groups of 32 consecutive channels; per group
// the cache holds (scale, zero) as two elements of the storage type T, and per channel an
// unsigned code of BITS bits, channel c in byte c*BITS/8 at bit (c*BITS) % 8:
//     scale = T((max - min) / (2^BITS - 1)),  zero = min,
//     code  = clamp(rint((v - zero) / scale), 0, 2^BITS - 1)   (fp32, IEEE division, ties to even),
//     v^    = zero + scale * code.
//
//   Vq    [B, S_max, D_kv*BITS/8] bytes      Vmeta [B, S_max, D_kv/32, 2] T
//
// qv_quantize_kernel writes the new token's row.  attend_qv_kernel evaluates the last step of
// Algorithm 1, y[h] = sum_j p[h,j] v^[C_j, g(h)], from the logits and tile statistics the logits
// kernel left behind: a gather of k rows of D_kv*BITS/8 bytes, no matrix product.  A thread owns
// 16 channels of one KV head for the whole token range, so the sum over tokens never leaves its
// registers; with  p*v^ = (p*zero) + (p*scale)*code  a token costs one multiply per head and one
// fused multiply-add per (head, channel).
#pragma once
#include <type_traits>

#include "common.hpp"
#include "k_attend.hpp"

namespace sals {

constexpr int kQvGroup = 32;        // channels per quantisation group
constexpr int kQvCh = 16;           // channels per thread of the attention kernel
constexpr int kQvMaxRanges = 32;    // token ranges a sequence's selection is split into at most
constexpr int kQvMaxTok = 4096;     // tokens per range at most

template <typename T> struct qv_meta;
template <> struct qv_meta<float> {
    static __device__ __forceinline__ float2 load(const float* p) { return *reinterpret_cast<const float2*>(p); }
    static __device__ __forceinline__ float round(float s) { return s; }
    static __device__ __forceinline__ void store(float* p, float s, float z) { *reinterpret_cast<float2*>(p) = make_float2(s, z); }
};
template <> struct qv_meta<bf16_t> {
    static __device__ __forceinline__ float2 load(const bf16_t* p)
    {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(p);
        return make_float2(bf16lo(w), bf16hi(w));
    }
    static __device__ __forceinline__ float round(float s) { return bf16_to_f32(f32_to_bf16(s)); }
    static __device__ __forceinline__ void store(bf16_t* p, float s, float z)
    {
        *reinterpret_cast<uint32_t*>(p) = (uint32_t)f32_to_bf16(s) | ((uint32_t)f32_to_bf16(z) << 16);
    }
};

// One group per 32 lanes: row seq_len[b] of the quantised cache from the new token's value.
// A sequence whose cache is full is left untouched.  grid (D/32/8, B), 256 threads.
// ring > 0: the cache is a ring of that many rows per sequence (recent window), token t in row t mod ring.
template <typename T, int BITS>
__global__ __launch_bounds__(256) void qv_quantize_kernel(const T* __restrict__ v_new, unsigned char* __restrict__ Vq,
                                                          T* __restrict__ Vmeta, const int32_t* __restrict__ seq_len,
                                                          int D, int S_max, int ring)
{
    constexpr float kLevels = (float)((1 << BITS) - 1);
    constexpr int PER = 32 / BITS;  // codes per 32-bit word
    const int b = blockIdx.y;
    const int gi = blockIdx.x * 8 + (threadIdx.x >> 5), l = threadIdx.x & 31;
    const int n_groups = D / kQvGroup;
    const int row = seq_len[b];
    if (gi >= n_groups || row < 0 || row >= S_max) return;
    const float v = elem<T>::load(v_new + (size_t)b * D + gi * kQvGroup + l);
    float mn = v, mx = v;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o, 32));
        mx = fmaxf(mx, __shfl_xor(mx, o, 32));
    }
    const float scale = qv_meta<T>::round((mx - mn) / kLevels);
    float t = scale > 0.f ? rintf((v - mn) / scale) : 0.f;
    t = fminf(fmaxf(t, 0.f), kLevels);
    uint32_t w = (uint32_t)t << ((l % PER) * BITS);
#pragma unroll
    for (int o = 1; o < PER; o <<= 1) w |= (uint32_t)__shfl_xor((int)w, o, 32);
    const size_t tok = ring > 0 ? (size_t)b * ring + row % ring : (size_t)b * S_max + row;
    if (l % PER == 0)
        *reinterpret_cast<uint32_t*>(Vq + tok * ((size_t)D * BITS / 8) + (size_t)(gi * kQvGroup + l) * BITS / 8) = w;
    if (l == 0) qv_meta<T>::store(Vmeta + (tok * n_groups + gi) * 2, scale, mn);
}

struct QvArgs {
    const unsigned char* Vq;
    const void* Vmeta;
    const int32_t* idx;
    const int32_t* n_sel;
    const float* logits;
    const float2* stats;
    float* part;   // [n_tr, B, H, 128] fp32 partial outputs; unused when n_tr == 1
    void* out;     // [B, H, 128] T
    int n_parts, B, S_max, H, H_kv, k_tot, lk, tok_per_wg, n_tr;
    // recent window (kernels with WIN): the last n_sel - n_lo[b] selected tokens are read from a ring of `ring` rows
    // per sequence with 8-bit codes (token t in row t mod ring); their logits are those of the window's logits pass
    const unsigned char* Vq_w;
    const void* Vmeta_w;
    const float* logits_w;   // [B, H, lk_w], slot j - n_lo[b]
    const int32_t* n_lo;     // [B] tokens of the low-precision pass
    int lk_w, ring;
    int part0, n_tr_all;     // partial outputs: this launch writes ranges part0 .. of n_tr_all (n_tr_all == 1: straight to out)
};

constexpr int kQvTpt = kHeadDim / kQvCh;  // threads per token: 8
constexpr int kQvSlots = 256 / kQvTpt;    // tokens in progress side by side: 32

// One workgroup per (sequence, token range, KV head): 8 threads cover the head's 128 channels of a
// token, 32 tokens ("slots") are in progress side by side and are added up through LDS at the end,
// in slot order.  1-D grid of B * n_tr * H_kv workgroups; ids are dealt round-robin to the XCDs and
// mapped so that each XCD gets a contiguous run of the work list (KV head fastest): the heads of a
// token range read neighbouring pieces of the same cache rows and meet in one L2.
template <typename T, int BITS, int GMAX, bool WIN = false>
__global__ __launch_bounds__(256) void attend_qv_kernel(QvArgs a)
{
    constexpr int UN = GMAX > 4 ? 4 : 8;  // tokens whose loads are in flight together, per thread
    __shared__ int sRow[kQvMaxTok];
    __shared__ float2 sMZ[kMaxGroup];
    __shared__ __attribute__((aligned(16))) float red[256][kQvCh + 1];

    int tr, kvh, b;
    {
        const int total = a.B * a.n_tr * a.H_kv;  // = gridDim.x
        const int xcd = blockIdx.x % kXcds, sl = blockIdx.x / kXcds, qn = total / kXcds, rem = total % kXcds;
        const int item = (xcd < rem ? xcd * (qn + 1) : rem * (qn + 1) + (xcd - rem) * qn) + sl;
        kvh = item % a.H_kv; tr = (item / a.H_kv) % a.n_tr; b = item / (a.H_kv * a.n_tr);
    }
    const int tid = threadIdx.x;
    const int H = a.H, G = H / a.H_kv;
    const int slot = tid / kQvTpt, u = tid % kQvTpt, c0 = u * kQvCh;
    const int32_t* ib = a.idx + (size_t)b * a.k_tot;

    // Everything the prologue needs from memory is requested before anything is waited for: the
    // first tile statistics of this KV head's query heads (32 lanes per head), the selection count
    // and up to four token indices per thread.  (Whole 8-byte loads: a float2 load would be split and
    // its second half sunk behind the merge's early exit.)
    const int sm = tid >> 5, sub = tid & 31;
    const float2* sp = a.stats + ((size_t)b * H + kvh * G + min(sm, G - 1)) * a.n_parts;
    constexpr unsigned long long kNeutral = 0x00000000ff800000ull;  // (-inf, 0)
    const unsigned long long st0 = (sm < G && sub < a.n_parts) ? *reinterpret_cast<const unsigned long long*>(sp + sub) : kNeutral;
    const int n_v = ld_uniform_i32(a.n_sel + b);  // (vector memory path: in flight with the loads around)
    const int nlo_v = WIN ? ld_uniform_i32(a.n_lo + b) : 0;
    int iv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = tid + 256 * i, j = tr * a.tok_per_wg + t;
        iv[i] = (t < a.tok_per_wg && j < a.k_tot) ? ib[j] : 0;
    }
    asm volatile("" ::: "memory");
    const int n = wave_uniform(n_v);
    const int j_begin = min(n, tr * a.tok_per_wg), j_end = min(n, j_begin + a.tok_per_wg);
    const int ntok = j_end - j_begin;
    // tokens [0, nlow) of the range come from the main cache, [nlow, ntok) from the window's ring
    const int nlow = WIN ? min(max(wave_uniform(nlo_v) - j_begin, 0), ntok) : ntok;
    auto row_of = [&](int t, int token) {
        if (WIN && t >= nlow) return max(token, 0) % a.ring;
        return min(max(token, 0), a.S_max - 1);
    };
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int t = tid + 256 * i;
        if (t < ntok) sRow[t] = row_of(t, iv[i]);
    }
    for (int t = tid + 1024; t < ntok; t += 256)  // long ranges: the rest, one load per round
        sRow[t] = row_of(t, ib[tr * a.tok_per_wg + t]);
    {   // softmax maximum and normaliser per query head: the head's tile statistics merged in a fixed order
        float2 st = make_float2(__uint_as_float((uint32_t)st0), __uint_as_float((uint32_t)(st0 >> 32)));
        if (sm < G)
            for (int t0 = sub + 32; t0 < a.n_parts; t0 += 32) st = stat_merge(st, sp[t0]);
#pragma unroll
        for (int o = 1; o < 32; o <<= 1)
            st = stat_merge(st, make_float2(__shfl_xor(st.x, o, kWave), __shfl_xor(st.y, o, kWave)));
        if (sub == 0 && sm < G) sMZ[sm] = make_float2(st.x > -INFINITY ? st.x : 0.f, st.y > 0.f ? 1.f / st.y : 0.f);
    }
    __syncthreads();
    float2 mz[GMAX];
#pragma unroll
    for (int m = 0; m < GMAX; ++m) mz[m] = m < G ? sMZ[m] : make_float2(0.f, 0.f);

    float acc[GMAX][kQvCh], bias[GMAX];
#pragma unroll
    for (int m = 0; m < GMAX; ++m) {
        bias[m] = 0.f;
#pragma unroll
        for (int c = 0; c < kQvCh; ++c) acc[m][c] = 0.f;
    }

    const int n_groups = a.H_kv * (kHeadDim / kQvGroup);
    // One pass over tokens [t_lo, t_hi) of the range, whose rows lie in a cache of `rows` rows per sequence with
    // NBITS-bit codes; lgp points at the logit of token t_lo for the group's first query head.
    auto pass = [&](auto nbits_tag, const unsigned char* codes, const void* meta, int rows, const float* lgp, int lk,
                    int t_lo, int t_hi) {
        constexpr int NBITS = decltype(nbits_tag)::value;
        constexpr int CB = kQvCh * NBITS / 8;  // code bytes per thread and token: 16, 8 or 4
        constexpr int NW = CB / 4;
        const size_t row_bytes = (size_t)a.H_kv * kHeadDim * NBITS / 8;
        const unsigned char* vq = codes + (size_t)b * rows * row_bytes + (size_t)(kvh * kHeadDim + c0) * NBITS / 8;
        const T* vm = static_cast<const T*>(meta) + ((size_t)b * rows * n_groups + kvh * (kHeadDim / kQvGroup) + c0 / kQvGroup) * 2;
        for (int t0 = t_lo + slot; t0 < t_hi; t0 += kQvSlots * UN) {
            uint32_t cw[UN][NW];
            float2 sz[UN];
            float x[UN][GMAX];
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                const int t = t0 + i * kQvSlots;
                const int tc = min(t, t_hi - 1);  // a token past the range re-reads the last row with weight zero
                const size_t row = (size_t)sRow[tc];
                if (NW == 4) {
                    const u32x4 w4 = *reinterpret_cast<const u32x4*>(vq + row * row_bytes);
                    cw[i][0] = w4.x; cw[i][1 % NW] = w4.y; cw[i][2 % NW] = w4.z; cw[i][3 % NW] = w4.w;
                } else if (NW == 2) {
                    const uint2 w2 = *reinterpret_cast<const uint2*>(vq + row * row_bytes);
                    cw[i][0] = w2.x; cw[i][NW - 1] = w2.y;
                } else {
                    cw[i][0] = *reinterpret_cast<const uint32_t*>(vq + row * row_bytes);
                }
                sz[i] = qv_meta<T>::load(vm + row * n_groups * 2);
#pragma unroll
                for (int m = 0; m < GMAX; ++m) x[i][m] = (m < G && t < t_hi) ? lgp[(size_t)m * lk + (tc - t_lo)] : -INFINITY;
            }
#pragma unroll
            for (int i = 0; i < UN; ++i) {
                float cf[kQvCh];
#pragma unroll
                for (int c = 0; c < kQvCh; ++c)
                    cf[c] = (float)((cw[i][(c * NBITS) / 32] >> ((c * NBITS) % 32)) & ((1u << NBITS) - 1u));
#pragma unroll
                for (int m = 0; m < GMAX; ++m) {
                    if (m < G) {  // uniform
                        const float p = __expf(x[i][m] - mz[m].x) * mz[m].y;  // exp(-inf) = 0 masks the padding
                        const float ps = p * sz[i].x;
                        bias[m] = fmaf(p, sz[i].y, bias[m]);
#pragma unroll
                        for (int c = 0; c < kQvCh; ++c) acc[m][c] = fmaf(ps, cf[c], acc[m][c]);
                    }
                }
            }
        }
    };
    pass(std::integral_constant<int, BITS>{}, a.Vq, a.Vmeta, a.S_max, a.logits + ((size_t)b * H + (size_t)kvh * G) * a.lk + j_begin,
         a.lk, 0, nlow);
    if constexpr (WIN) {
        if (nlow < ntok) {  // uniform: the window's tokens, slot j - n_lo of the window's logits
            const int nlo = wave_uniform(nlo_v);
            pass(std::integral_constant<int, 8>{}, a.Vq_w, a.Vmeta_w, a.ring,
                 a.logits_w + ((size_t)b * H + (size_t)kvh * G) * a.lk_w + (j_begin + nlow - nlo), a.lk_w, nlow, ntok);
        }
    }
#pragma unroll
    for (int m = 0; m < GMAX; ++m)
#pragma unroll
        for (int c = 0; c < kQvCh; ++c) acc[m][c] += bias[m];

    // the 32 token slots' sums: thread e < 128 adds channel e of the head over the slots, in slot order
#pragma unroll
    for (int m = 0; m < GMAX; ++m) {
        if (m < G) {  // uniform
            __syncthreads();
#pragma unroll
            for (int c = 0; c < kQvCh; ++c) red[tid][c] = acc[m][c];
            __syncthreads();
            if (tid < kHeadDim) {
                const int uu = tid / kQvCh, cc = tid % kQvCh;
                float s = 0.f;
#pragma unroll 8
                for (int sl = 0; sl < kQvSlots; ++sl) s += red[sl * kQvTpt + uu][cc];
                const int h = kvh * G + m;
                if (a.n_tr_all > 1) a.part[(((size_t)(a.part0 + tr) * a.B + b) * H + h) * kHeadDim + tid] = s;
                else elem<T>::store(static_cast<T*>(a.out) + ((size_t)b * H + h) * kHeadDim + tid, s);
            }
        }
    }
}

// out = sum over the token ranges' partial outputs, in range order, rounded once to T.
// One thread per 4 output elements.
template <typename T>
__global__ __launch_bounds__(256) void qv_merge_kernel(const float* __restrict__ part, T* __restrict__ out, int n_tr,
                                                       size_t n4)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n4) return;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    for (int t0 = 0; t0 < n_tr; t0 += 8) {
        f32x4 x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            x[i] = t0 + i < n_tr ? *reinterpret_cast<const f32x4*>(part + ((size_t)(t0 + i) * n4 + e) * 4) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < 8; ++i) { s.x += x[i].x; s.y += x[i].y; s.z += x[i].z; s.w += x[i].w; }
    }
    T* dst = out + e * 4;
    elem<T>::store(dst, s.x); elem<T>::store(dst + 1, s.y); elem<T>::store(dst + 2, s.z); elem<T>::store(dst + 3, s.w);
}

}  // namespace sals
