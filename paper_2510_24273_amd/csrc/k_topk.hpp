// Critical-token selection  C = TopK(s, k)  (Algorithm 1, TopK step), with the
// sink / recent composition of Sec. 5.2.
//
// One workgroup per sequence finds the key of the k-th largest candidate exactly and then
// places every selected index with one block-wide prefix sum.  Scores are handled as
// order-preserving 32-bit keys, kept in registers when the sequence fits (up to 32 per
// thread); longer sequences re-read the scores, which sit in L2.
//
// Finding the k-th key:
//   fast path  a 4096-bin histogram over the LINEAR range [min, max] of the candidates (a
//              monotone map, so bins are ordered like the scores).  Unlike a histogram over
//              float bit fields it spreads clustered scores over many bins, which matters:
//              LDS atomics that hit one address from many lanes serialise.  The bin holding
//              the k-th score usually has a few dozen members; they are copied to LDS and
//              ranked against each other.
//   fallback   (degenerate range, or too many members in that bin) an exact radix select
//              over the key bits, 12 + 10 + 10.
// Equal scores are resolved towards the smaller index, so the output is a deterministic
// function of the scores.
#pragma once
#include "common.hpp"

namespace sals {

constexpr int kTopkThreads = 1024;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkBins = 4096;
constexpr int kTopkCand = 512;  // members of the threshold bin handled by the fast path

struct TopkShared {
    __attribute__((aligned(16))) uint32_t hist[kTopkBins];
    __attribute__((aligned(16))) uint32_t cand[kTopkCand];
    uint32_t scan_a[2][kTopkWaves], scan_b[2][kTopkWaves];  // wave totals, double buffered
    uint32_t wave_a[kTopkWaves], wave_b[kTopkWaves];
    uint32_t sel_prefix, sel_kk, n_cand;
};

__device__ __forceinline__ float key_to_score(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

// Exclusive prefix sums of a and b over the workgroup's NW waves (at most 16; one barrier); *ta, *tb get the
// block sums.  `phase` alternates the LDS buffer, so back-to-back calls need no second barrier.
template <int NW = kTopkWaves>
__device__ __forceinline__ void block_excl_scan2(uint32_t& a, uint32_t& b, TopkShared& sh, int& phase,
                                                 uint32_t* ta, uint32_t* tb)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t ia = wave_incl_scan(a), ib = wave_incl_scan(b);
    if (lane == kWave - 1) { sh.scan_a[phase][wave] = ia; sh.scan_b[phase][wave] = ib; }
    __syncthreads();
    static_assert(kTopkWaves == 16 && NW <= 16, "one DPP row holds the wave totals");
    const bool has = (lane & 15) < NW;  // (slots of waves that do not exist are never written)
    const uint32_t wa = has ? sh.scan_a[phase][lane & 15] : 0u, wb = has ? sh.scan_b[phase][lane & 15] : 0u;
    const bool before = (lane & 15) < wave;
    *ta = row16_sum_u32(wa);
    *tb = row16_sum_u32(wb);
    a = row16_sum_u32(before ? wa : 0u) + ia - a;
    b = row16_sum_u32(before ? wb : 0u) + ib - b;
    phase ^= 1;
}
template <int NW = kTopkWaves>
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, TopkShared& sh, int& phase, uint32_t* total)
{
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t iv = wave_incl_scan(v);
    if (lane == kWave - 1) sh.scan_a[phase][wave] = iv;
    __syncthreads();
    const uint32_t wv = (lane & 15) < NW ? sh.scan_a[phase][lane & 15] : 0u;
    *total = row16_sum_u32(wv);
    const uint32_t r = row16_sum_u32((lane & 15) < wave ? wv : 0u) + iv - v;
    phase ^= 1;
    return r;
}

// Selection for sequence b by the calling workgroup (NTH threads, all of them must call).
// F4 > 0: keys of F4 float4 groups per thread stay in registers.  F4 == 0: stream.
// CONSEC: a thread's keys are 4*F4 consecutive tokens (otherwise group c of thread t covers tokens
// 4*(c*NTH + t) .. +3): with it, selected indices come out in token order inside each score class whatever NTH is,
// i.e. in the order the 1024-thread kernel with one group per thread produces.
// `idx` / `n_sel` may point to LDS (the caller reads them after a barrier of its own).
template <int F4, int NTH = kTopkThreads, bool CONSEC = false>
__device__ __forceinline__ void topk_select_sequence(TopkShared& sh, const float* __restrict__ scores,
                                                     const int32_t* __restrict__ seq_len,
                                                     int32_t* __restrict__ idx, int32_t* __restrict__ n_sel,
                                                     int b, int S_max, int top_k, int n_sink, int n_recent)
{
    const int tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const int k_tot = top_k + n_sink + n_recent;
    const float* s = scores + (size_t)b * S_max;
    int32_t* out = idx + (size_t)b * k_tot;
    const bool vec_ok = (((size_t)b * S_max) & 3) == 0;  // this row starts 16-byte aligned
    constexpr int NREG = F4 > 0 ? F4 * 4 : 4;
    constexpr int NW = NTH / kWave;              // waves
    constexpr int BPT = kTopkBins / NTH;         // histogram bins per thread
    static_assert(NTH % kWave == 0 && NTH >= kTopkCand && NTH <= kTopkThreads && kTopkBins % NTH == 0 && (!CONSEC || F4 > 0),
                  "workgroup shape");
    // token of this thread's key i (i = 4*group + element)
    auto token_of = [&](int i) { return CONSEC ? tid * NREG + i : ((((i >> 2) * NTH) + tid) << 2) + (i & 3); };

    // group c of this thread covers tokens 4*(c*1024 + tid) .. +3  (coalesced float4 loads);
    // the loads depend on S_max only, so they are in flight together with the length
    auto load_group = [&](int c, float* f) {
        const int j = token_of(4 * c);
        f[0] = f[1] = f[2] = f[3] = 0.f;
        if (vec_ok && j + 3 < S_max) {
            f32x4 v = *reinterpret_cast<const f32x4*>(s + j);
            f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < S_max) f[e] = s[j + e];
        }
    };
    const int S_in_v = ld_uniform_i32(seq_len + b);  // (through the vector memory path: in flight with the scores)
    float raw[NREG];
    if (F4 > 0) {
        if (vec_ok && (S_max & 3) == 0 && S_max >= 4) {  // uniform: every group lies wholly inside or outside the row
            // all groups requested at once from clamped addresses (a load inside a branch would be waited for at the
            // end of that branch: one memory round trip per group)
            f32x4 v[F4 > 0 ? F4 : 1];
#pragma unroll
            for (int c = 0; c < (F4 > 0 ? F4 : 1); ++c)
                v[c] = *reinterpret_cast<const f32x4*>(s + min(token_of(4 * c), S_max - 4));
#pragma unroll
            for (int c = 0; c < (F4 > 0 ? F4 : 1); ++c) {
                const bool in = token_of(4 * c) < S_max;
                raw[4 * c] = in ? v[c].x : 0.f; raw[4 * c + 1] = in ? v[c].y : 0.f;
                raw[4 * c + 2] = in ? v[c].z : 0.f; raw[4 * c + 3] = in ? v[c].w : 0.f;
            }
        } else {
#pragma unroll
            for (int c = 0; c < (F4 > 0 ? F4 : 1); ++c) load_group(c, raw + 4 * c);
        }
    }
    const int S = min(wave_uniform(S_in_v), S_max);

    if (S <= k_tot) {  // short cache: every token is selected
        for (int t = tid; t < k_tot; t += NTH) out[t] = t < S ? t : 0;
        if (tid == 0) n_sel[b] = S > 0 ? S : 0;
        return;
    }
    const int lo = n_sink, hi = S - n_recent;
    for (int t = tid; t < n_sink; t += NTH) out[t] = t;
    for (int t = tid; t < n_recent; t += NTH) out[n_sink + top_k + t] = hi + t;
    if (tid == 0) n_sel[b] = k_tot;
    if (top_k <= 0) return;

    // candidates are the tokens lo <= j < hi; every other slot carries key 0 (below -inf)
    uint32_t keys[NREG];
    if (F4 > 0) {
#pragma unroll
        for (int i = 0; i < NREG; ++i) {
            const int jj = token_of(i);
            keys[i] = (jj >= lo && jj < hi) ? score_key(raw[i]) : 0u;
        }
    }
    const int n_iter = F4 > 0 ? F4 : (((S + 3) >> 2) + NTH - 1) / NTH;
    // visit every (key, token index) of this thread
    auto for_each_key = [&](auto&& fn) {
        if (F4 > 0) {
#pragma unroll
            for (int i = 0; i < NREG; ++i) fn(keys[i], token_of(i));
        } else {
            for (int c = 0; c < n_iter; ++c) {
                float f[4];
                load_group(c, f);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int jj = token_of(4 * c) + e;
                    fn((jj >= lo && jj < hi) ? score_key(f[e]) : 0u, jj);
                }
            }
        }
    };

    int phase = 0;
    uint32_t tau = 0u, need_eq = 0u;  // key of the top_k-th largest candidate; ties taken at it
    bool found = false;

    // ---- fast path: linear-range histogram ---------------------------------------------
    {
        // key 0 (no candidate) never wins the maximum, and k - 1 turns it into the largest value for the minimum
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        for_each_key([&](uint32_t k, int) { kmin = min(kmin, k - 1u); kmax = max(kmax, k); });
        kmin = kmin == 0xffffffffu ? kmin : kmin + 1u;
        kmin = wave_min_u32(kmin);
        kmax = wave_max_u32(kmax);
        if (lane == 0) { sh.wave_a[wave] = kmin; sh.wave_b[wave] = kmax; }
        for (uint32_t t = tid; t < kTopkBins; t += NTH) sh.hist[t] = 0u;
        if (tid < kTopkCand) sh.cand[tid] = 0u;  // key 0 ranks below every candidate
        if (tid == 0) sh.n_cand = 0u;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < NW; ++w) { kmin = min(kmin, sh.wave_a[w]); kmax = max(kmax, sh.wave_b[w]); }
        const float flo = key_to_score(kmin), fhi = key_to_score(kmax);
        const float span = fhi - flo;
        const float scale = (span > 0.f && span < 3.0e38f) ? (float)kTopkBins / span : 0.f;
        const float off = fhi * scale;
        if (scale > 0.f && scale < 3.0e38f && fabsf(off) < 3.0e38f) {  // uniform
            // a monotone map of the score onto slots, (max - score) * bins / span; slot 0 is the top of the range
            auto slot_of_score = [&](float sc) { return min(max((int)fmaf(sc, -scale, off), 0), kTopkBins - 1); };
            auto slot_of = [&](uint32_t k) { return slot_of_score(key_to_score(k)); };
            // keys in registers: every key's slot is kept too (two per register; 0xffff for a non-candidate), so the
            // pass that collects the threshold slot's members compares instead of mapping every score again
            uint32_t slot2[F4 > 0 ? NREG / 2 : 1];
            if constexpr (F4 > 0) {
#pragma unroll
                for (int i = 0; i < NREG; i += 2) {
                    // up to 16 keys per thread the raw scores are still in registers and save the way back from the
                    // key (same slot: the two only differ for -0, which maps like +0); with 32 they would spill
                    constexpr bool kRaw = F4 <= 4;
                    const uint32_t s0 = keys[i] == 0u ? 0xffffu
                                        : (uint32_t)(kRaw ? slot_of_score(raw[i]) : slot_of(keys[i]));
                    const uint32_t s1 = keys[i + 1] == 0u ? 0xffffu
                                        : (uint32_t)(kRaw ? slot_of_score(raw[i + 1]) : slot_of(keys[i + 1]));
                    if (keys[i] != 0u) atomicAdd(&sh.hist[s0], 1u);
                    if (keys[i + 1] != 0u) atomicAdd(&sh.hist[s1], 1u);
                    slot2[i >> 1] = s0 | (s1 << 16);
                }
            } else {
                for_each_key([&](uint32_t k, int) { if (k != 0u) atomicAdd(&sh.hist[slot_of(k)], 1u); });
            }
            __syncthreads();
            uint32_t cnt[BPT], mine = 0u;  // this thread's BPT consecutive slots
#pragma unroll
            for (int i4 = 0; i4 < BPT; i4 += 4) {
                const u32x4 c4 = *reinterpret_cast<const u32x4*>(&sh.hist[tid * BPT + i4]);
                cnt[i4] = c4.x; cnt[i4 + 1] = c4.y; cnt[i4 + 2] = c4.z; cnt[i4 + 3] = c4.w;
                mine += c4.x + c4.y + c4.z + c4.w;
            }
            uint32_t total;
            uint32_t above = block_excl_scan<NW>(mine, sh, phase, &total);
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                if (above < (uint32_t)top_k && (uint32_t)top_k <= above + cnt[i]) {
                    sh.sel_prefix = (uint32_t)(tid * BPT + i);  // slot holding the k-th score
                    sh.sel_kk = (uint32_t)top_k - above;      // how many of its members are selected
                }
                above += cnt[i];
            }
            __syncthreads();
            const int t_slot = (int)sh.sel_prefix;
            const uint32_t kk = sh.sel_kk;
            const uint32_t members = sh.hist[t_slot];
            if (members <= (uint32_t)kTopkCand) {  // uniform
                if constexpr (F4 > 0) {
#pragma unroll
                    for (int i = 0; i < NREG; ++i) {
                        const uint32_t si = (i & 1) ? slot2[i >> 1] >> 16 : slot2[i >> 1] & 0xffffu;
                        if (si == (uint32_t)t_slot) sh.cand[atomicAdd(&sh.n_cand, 1u)] = keys[i];
                    }
                } else {
                    for_each_key([&](uint32_t k, int) {
                        if (k != 0u && slot_of(k) == t_slot) sh.cand[atomicAdd(&sh.n_cand, 1u)] = k;
                    });
                }
                __syncthreads();
                // the member with  #(greater) < kk <= #(greater or equal)  carries the k-th key
                if (tid < (int)members) {
                    const uint32_t mykey = sh.cand[tid];
                    uint32_t gt = 0u, ge = 0u;
                    for (uint32_t c = 0; c < members; c += 4) {
                        u32x4 o = *reinterpret_cast<const u32x4*>(&sh.cand[c]);
                        gt += (o.x > mykey) + (o.y > mykey) + (o.z > mykey) + (o.w > mykey);
                        ge += (o.x >= mykey) + (o.y >= mykey) + (o.z >= mykey) + (o.w >= mykey);
                    }
                    if (gt < kk && kk <= ge) { sh.sel_prefix = mykey; sh.sel_kk = kk - gt; }
                }
                __syncthreads();
                tau = sh.sel_prefix;
                need_eq = sh.sel_kk;
                found = true;
            }
        }
    }

    // ---- fallback: radix select over the key bits -----------------------------------------
    if (!found) {  // uniform
        uint32_t prefix = 0u, mask = 0u, kk = (uint32_t)top_k;
#pragma unroll 1
        for (int pass = 0; pass < 3; ++pass) {
            const int bits = pass == 0 ? 12 : 10;
            const int shift = pass == 0 ? 20 : (pass == 1 ? 10 : 0);
            const uint32_t nb = 1u << bits;
            __syncthreads();
            for (uint32_t t = tid; t < nb; t += NTH) sh.hist[t] = 0u;
            __syncthreads();
            // histogram indexed from the top: slot 0 is the largest digit
            for_each_key([&](uint32_t k, int) {
                if (k != 0u && (k & mask) == prefix) atomicAdd(&sh.hist[nb - 1u - ((k >> shift) & (nb - 1u))], 1u);
            });
            __syncthreads();
            const int per = (int)(nb / NTH);  // BPT for the 12-bit pass, a quarter of it for the 10-bit ones
            uint32_t cnt[BPT], mine = 0u;
#pragma unroll
            for (int i = 0; i < BPT; ++i) { cnt[i] = i < per ? sh.hist[tid * per + i] : 0u; mine += cnt[i]; }
            uint32_t total;
            uint32_t above = block_excl_scan<NW>(mine, sh, phase, &total);
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                if (i < per && above < kk && kk <= above + cnt[i]) {
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
        tau = prefix;
        need_eq = kk;
    }
    const uint32_t n_gt = (uint32_t)top_k - need_eq;

    // ---- count, then place ----------------------------------------------------------------
    uint32_t pos_gt = 0u, pos_eq = 0u;
    for_each_key([&](uint32_t k, int) { pos_gt += k > tau; pos_eq += k == tau; });
    uint32_t tot_gt, tot_eq;
    block_excl_scan2<NW>(pos_gt, pos_eq, sh, phase, &tot_gt, &tot_eq);

    // ties that straddle the cut: keep the need_eq smallest token indices among them
    int j_cut = hi;  // select ties with index < j_cut
    if (tot_eq > need_eq) {  // uniform
        int lo_j = lo, hi_j = hi;  // smallest J with #(eq && j < J) >= need_eq
        while (lo_j < hi_j) {
            int mid = (lo_j + hi_j) >> 1;
            uint32_t c_mine = 0u;
            for_each_key([&](uint32_t k, int jj) { c_mine += (k == tau && jj < mid); });
            uint32_t c_tot;
            block_excl_scan<NW>(c_mine, sh, phase, &c_tot);
            if (c_tot >= need_eq) hi_j = mid; else lo_j = mid + 1;
        }
        j_cut = lo_j;
        uint32_t my_eq = 0u;
        for_each_key([&](uint32_t k, int jj) { my_eq += (k == tau && jj < j_cut); });
        pos_eq = block_excl_scan<NW>(my_eq, sh, phase, &tot_eq);
    }

    // greater-than keys fill [0, n_gt), ties [n_gt, top_k), each in token order.  (The limits
    // only guard against out-of-range writes on malformed scores, e.g. NaN.)
    int32_t* const sel = out + n_sink;
    uint32_t og = pos_gt, oe = n_gt + pos_eq;
    for_each_key([&](uint32_t k, int jj) {
        const bool g = k > tau, e = (k == tau) && (jj < j_cut);
        const uint32_t p = g ? og : oe, lim = g ? n_gt : (uint32_t)top_k;
        if ((g || e) && p < lim) sel[p] = jj;
        og += g;
        oe += e;
    });
}

// Recent-window attention splits a selection into the tokens before the window and the window's own list (the
// last min(w, n_sel) entries, which are the most recent tokens in token order).  Both follow from the sequence length
// alone, so the selection kernel can leave them beside its output: idx_hi [B, w] (zero beyond the count),
// n_lo[b] = n_sel - n_w, n_hi[b] = n_w.  idx_hi == nullptr: nothing to do.
struct WindowLists { int32_t* idx_hi; int32_t* n_lo; int32_t* n_hi; int w; };
__device__ __forceinline__ void write_window_lists(const WindowLists& wl, const int32_t* __restrict__ seq_len, int b,
                                                   int S_max, int k_tot, int n_threads)
{
    if (wl.idx_hi == nullptr) return;
    const int S = min(max(seq_len[b], 0), S_max), n = min(S, k_tot), nw = min(wl.w, n);
    for (int t = threadIdx.x; t < wl.w; t += n_threads) wl.idx_hi[(size_t)b * wl.w + t] = t < nw ? S - nw + t : 0;
    if (threadIdx.x == 0) { wl.n_lo[b] = n - nw; wl.n_hi[b] = nw; }
}

template <int F4>
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ scores,
                                                            const int32_t* __restrict__ seq_len,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ n_sel, int S_max,
                                                            int top_k, int n_sink, int n_recent)
{
    __shared__ TopkShared sh;
    const int b = blockIdx.x;
    topk_select_sequence<F4>(sh, scores, seq_len, idx, n_sel, b, S_max, top_k, n_sink, n_recent);
}

// The same with the recent-window lists (a kernel of its own: the plain one keeps its shorter argument list).
template <int F4>
__global__ __launch_bounds__(kTopkThreads) void topk_window_kernel(const float* __restrict__ scores,
                                                                   const int32_t* __restrict__ seq_len,
                                                                   int32_t* __restrict__ idx,
                                                                   int32_t* __restrict__ n_sel, int S_max,
                                                                   int top_k, int n_sink, int n_recent, WindowLists wl)
{
    __shared__ TopkShared sh;
    const int b = blockIdx.x;
    write_window_lists(wl, seq_len, b, S_max, top_k + n_sink + n_recent, kTopkThreads);
    topk_select_sequence<F4>(sh, scores, seq_len, idx, n_sel, b, S_max, top_k, n_sink, n_recent);
}

}  // namespace sals
