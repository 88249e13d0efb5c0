// Critical-token selection  C = TopK(s, k)  (Algorithm 1, TopK step), with the
// sink / recent composition of Sec. 5.2.
//
// One workgroup per sequence runs an exact radix select on order-preserving
// 32-bit keys of the fp32 scores: three passes (12 + 10 + 10 bits) with an LDS
// histogram find the key of the k-th largest candidate, then one counting pass and
// a single block-wide prefix sum place every selected index.  Keys live in
// registers when the sequence fits (up to 32 per thread); longer sequences
// re-read the scores, which sit in L2.  Equal scores are resolved towards the
// smaller index, so the output is a deterministic function of the scores.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkBins = 4096;

struct TopkShared {
    uint32_t hist[kTopkBins];
    uint32_t wave_tot[kTopkWaves + 1];
    uint32_t sel_prefix, sel_kk;
};

// exclusive prefix sum of v over the 1024 threads; *total gets the block sum
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* wave_tot, uint32_t* total)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t incl = wave_incl_scan(v);
    __syncthreads();  // protect wave_tot from the previous use
    if (lane == kWave - 1) wave_tot[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        uint32_t t = lane < kTopkWaves ? wave_tot[lane] : 0u;
        uint32_t ti = wave_incl_scan(t);
        if (lane < kTopkWaves) wave_tot[lane] = ti - t;
        if (lane == kTopkWaves - 1) wave_tot[kTopkWaves] = ti;
    }
    __syncthreads();
    *total = wave_tot[kTopkWaves];
    return wave_tot[wave] + incl - v;
}

// F4 > 0: keys of F4 float4 groups per thread stay in registers.  F4 == 0: stream.
template <int F4>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ scores,
                                                            const int32_t* __restrict__ seq_len,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ n_sel, int S_max,
                                                            int top_k, int n_sink, int n_recent)
{
    __shared__ TopkShared sh;
    const int tid = threadIdx.x;
    const int b = blockIdx.x;
    const int k_tot = top_k + n_sink + n_recent;
    const int S = min(seq_len[b], S_max);
    const float* s = scores + (size_t)b * S_max;
    int32_t* out = idx + (size_t)b * k_tot;

    if (S <= k_tot) {  // short cache: every token is selected
        for (int t = tid; t < k_tot; t += kTopkThreads) out[t] = t < S ? t : 0;
        if (tid == 0) n_sel[b] = S > 0 ? S : 0;
        return;
    }
    const int lo = n_sink, hi = S - n_recent;
    for (int t = tid; t < n_sink; t += kTopkThreads) out[t] = t;
    for (int t = tid; t < n_recent; t += kTopkThreads) out[n_sink + top_k + t] = hi + t;
    if (tid == 0) n_sel[b] = k_tot;

    // group c of this thread covers tokens 4*(c*1024 + tid) .. +3  (coalesced float4 loads)
    const int n_groups = (S + 3) >> 2;
    const bool vec_ok = (((size_t)b * S_max) & 3) == 0;  // this row starts 16-byte aligned
    const int n_iter = F4 > 0 ? F4 : (n_groups + kTopkThreads - 1) / kTopkThreads;
    constexpr int NREG = F4 > 0 ? F4 * 4 : 4;
    uint32_t keys[NREG];

    auto load_group = [&](int c, uint32_t* k4) {
        int grp = c * kTopkThreads + tid;
        int j = grp << 2;
        float f[4] = {0.f, 0.f, 0.f, 0.f};
        if (grp < n_groups) {
            if (vec_ok && j + 3 < S_max) {
                f32x4 v = *reinterpret_cast<const f32x4*>(s + j);
                f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j + e < S_max) f[e] = s[j + e];
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int jj = j + e;
            k4[e] = (jj >= lo && jj < hi) ? score_key(f[e]) : 0u;  // key 0 sorts below -inf
        }
    };
    if (F4 > 0) {
#pragma unroll
        for (int c = 0; c < (F4 > 0 ? F4 : 1); ++c) load_group(c, keys + 4 * c);
    }

    // ---- radix select of the top_k-th largest key --------------------------------
    uint32_t prefix = 0u, mask = 0u, kk = (uint32_t)top_k;
#pragma unroll 1
    for (int pass = 0; pass < 3; ++pass) {
        const int bits = pass == 0 ? 12 : 10;
        const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
        const uint32_t nb = 1u << bits;
        for (uint32_t t = tid; t < nb; t += kTopkThreads) sh.hist[t] = 0u;
        __syncthreads();
        // histogram indexed from the top: slot 0 is the largest digit
        if (F4 > 0) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                uint32_t k = keys[i];
                if (k != 0u && (k & mask) == prefix) atomicAdd(&sh.hist[nb - 1u - ((k >> shift) & (nb - 1u))], 1u);
            }
        } else {
            for (int c = 0; c < n_iter; ++c) {
                uint32_t k4[4];
                load_group(c, k4);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (k4[e] != 0u && (k4[e] & mask) == prefix)
                        atomicAdd(&sh.hist[nb - 1u - ((k4[e] >> shift) & (nb - 1u))], 1u);
            }
        }
        __syncthreads();
        // each thread owns nb/1024 consecutive slots; find the slot where the running
        // count from the top first reaches kk
        const int per = (int)(nb / kTopkThreads);  // 4 or 1
        uint32_t cnt[4] = {0u, 0u, 0u, 0u}, mine = 0u;
        for (int i = 0; i < per; ++i) { cnt[i] = sh.hist[tid * per + i]; mine += cnt[i]; }
        uint32_t total;
        uint32_t above = block_excl_scan(mine, sh.wave_tot, &total);
        for (int i = 0; i < per; ++i) {
            if (above < kk && kk <= above + cnt[i]) {
                uint32_t digit = nb - 1u - (uint32_t)(tid * per + i);
                sh.sel_prefix = prefix | (digit << shift);
                sh.sel_kk = kk - above;
            }
            above += cnt[i];
        }
        __syncthreads();
        prefix = sh.sel_prefix;
        kk = sh.sel_kk;
        mask |= (nb - 1u) << shift;
    }
    const uint32_t tau = prefix;       // key of the top_k-th largest candidate
    const uint32_t need_eq = kk;       // how many keys equal to tau are selected
    const uint32_t n_gt = (uint32_t)top_k - need_eq;

    // ---- count, then place ----------------------------------------------------------
    uint32_t my_gt = 0u, my_eq = 0u;
    if (F4 > 0) {
#pragma unroll
        for (int i = 0; i < NREG; ++i) { my_gt += keys[i] > tau; my_eq += keys[i] == tau; }
    } else {
        for (int c = 0; c < n_iter; ++c) {
            uint32_t k4[4];
            load_group(c, k4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { my_gt += k4[e] > tau; my_eq += k4[e] == tau; }
        }
    }
    uint32_t tot_gt, tot_eq;
    uint32_t pos_gt = block_excl_scan(my_gt, sh.wave_tot, &tot_gt);
    uint32_t pos_eq = block_excl_scan(my_eq, sh.wave_tot, &tot_eq);

    // ties that straddle the cut: keep the need_eq smallest token indices among them
    int j_cut = hi;  // select ties with index < j_cut
    if (tot_eq > need_eq) {
        int lo_j = lo, hi_j = hi;  // smallest J with #(eq && j < J) >= need_eq
        while (lo_j < hi_j) {
            int mid = (lo_j + hi_j) >> 1;
            uint32_t c_mine = 0u;
            if (F4 > 0) {
#pragma unroll
                for (int i = 0; i < NREG; ++i) {
                    int jj = (((i >> 2) * kTopkThreads + tid) << 2) + (i & 3);
                    c_mine += (keys[i] == tau && jj < mid);
                }
            } else {
                for (int c = 0; c < n_iter; ++c) {
                    uint32_t k4[4];
                    load_group(c, k4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        int jj = ((c * kTopkThreads + tid) << 2) + e;
                        c_mine += (k4[e] == tau && jj < mid);
                    }
                }
            }
            uint32_t c_tot;
            block_excl_scan(c_mine, sh.wave_tot, &c_tot);
            if (c_tot >= need_eq) hi_j = mid; else lo_j = mid + 1;
        }
        j_cut = lo_j;
        // recount this thread's selected ties and their offsets
        my_eq = 0u;
        if (F4 > 0) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) {
                int jj = (((i >> 2) * kTopkThreads + tid) << 2) + (i & 3);
                my_eq += (keys[i] == tau && jj < j_cut);
            }
        } else {
            for (int c = 0; c < n_iter; ++c) {
                uint32_t k4[4];
                load_group(c, k4);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    int jj = ((c * kTopkThreads + tid) << 2) + e;
                    my_eq += (k4[e] == tau && jj < j_cut);
                }
            }
        }
        pos_eq = block_excl_scan(my_eq, sh.wave_tot, &tot_eq);
    }

    // (the end pointers only guard against out-of-range writes on malformed scores, e.g. NaN)
    int32_t* out_gt = out + n_sink + pos_gt;
    int32_t* out_eq = out + n_sink + n_gt + pos_eq;
    int32_t* const end_gt = out + n_sink + n_gt;
    int32_t* const end_eq = out + n_sink + top_k;
    if (F4 > 0) {
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            int jj = (((i >> 2) * kTopkThreads + tid) << 2) + (i & 3);
            if (keys[i] > tau) { if (out_gt < end_gt) *out_gt++ = jj; }
            else if (keys[i] == tau && jj < j_cut) { if (out_eq < end_eq) *out_eq++ = jj; }
        }
    } else {
        for (int c = 0; c < n_iter; ++c) {
            uint32_t k4[4];
            load_group(c, k4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                int jj = ((c * kTopkThreads + tid) << 2) + e;
                if (k4[e] > tau) { if (out_gt < end_gt) *out_gt++ = jj; }
                else if (k4[e] == tau && jj < j_cut) { if (out_eq < end_eq) *out_eq++ = jj; }
            }
        }
    }
}

}  // namespace sals
