// Critical-token selection for long sequences (Algorithm 1, TopK step; Sec. 5.2 composition),
// spread over many workgroups.
//
// One workgroup walks a compute unit's worth of instructions per key and pass, so beyond a few
// ten thousand scores a single workgroup per sequence is the bottleneck.  Here a sequence is cut
// into chunks of 8192 scores, one workgroup each, and the selection runs as a chain of small
// kernels that exchange a few kilobytes:
//   range    per chunk: minimum and maximum candidate key
//   hist     per chunk: histogram over 2048 linear bins of the sequence's [min, max], stored as running
//            counts from the top bin down (entry s = the chunk's scores in bins above s)
//   place    per chunk: the bin holding the top_k-th score, how many of its members are selected and
//            where the chunk's output starts (every workgroup of the sequence derives the same
//            numbers, in two passes over the chunks' running counts: at every 32nd bin, then at the
//            32 bins of the step that holds the threshold); then the indices of the scores in
//            higher bins go to their final positions (chunk order, then token order) and the
//            members of the threshold bin to a candidate list
//   finish   per sequence: ranks the candidates (ties towards the smaller index), writes the
//            selected ones in token order, the sink / recent entries and n_sel
// The result is the same set as topk_kernel's, a deterministic function of the scores; only
// the order inside the top_k block differs (bins above the threshold first).  Cases this chain
// does not cover (a cache no longer than the selection, a degenerate or non-finite score range,
// more than 512 members in the threshold bin) raise a flag, and the finish kernel's workgroup
// then selects that sequence from scratch the way topk_kernel does.
#pragma once
#include "common.hpp"
#include "k_topk.hpp"

namespace sals {

constexpr int kTmChunk = 8192;            // scores per workgroup
constexpr int kTmF4 = kTmChunk / (4 * kTopkThreads);  // float4 groups per thread: 2
constexpr int kTmBins = 2048;
constexpr int kTmMaxChunks = 128;         // S_max <= 2^20
constexpr int kTmCand = 512;              // candidates the finish kernel ranks
constexpr int kTmCoarse = 32;             // bins per coarse step of the threshold search
constexpr int kTmNC = kTmBins / kTmCoarse;   // coarse steps
constexpr int kTmCum = kTmBins + 4;       // running counts per chunk: entries 0 .. kTmBins (rows stay 16-byte aligned)

struct TopkMeta {        // per sequence, written by the place kernel
    uint32_t fallback;   // 1: topk_kernel must redo the sequence
    uint32_t t_slot;     // threshold bin (slot 0 = top of the range)
    uint32_t kk;         // members of the threshold bin that are selected
    uint32_t n_above;    // scores in higher bins
    uint32_t members;    // scores in the threshold bin
    float flo, scale;    // slot = kTmBins-1 - clamp(int((x - flo) * scale))
    uint32_t pad;
};

// workspace of the chain, per sequence
struct TopkMultiWs {
    const uint2* range;  // [B][n_range] (min key, max key) pairs that cover the sequence's candidates: `part`, or the
    int n_range;         //   pairs the score kernel left per workgroup (then over all scores below the length)
    uint2* part;         // [B][n_chunk] (min key, max key) of the chunk's candidates
    uint32_t* hist;      // [B][n_chunk][kTmCum]: entry s = the chunk's candidates in slots above s (slot 0 = top bin)
    TopkMeta* meta;      // [B]
    uint2* cand;         // [B][kTmCand] (key, token index)
};

// keys of this thread's 8 scores of chunk `chunk`: tokens chunk*8192 + 4*(c*1024 + tid) + e;
// non-candidates (sink / recent tokens, positions past the sequence) carry key 0
__device__ __forceinline__ void tm_load_keys(const float* __restrict__ s, int S_max, int chunk, int lo, int hi,
                                            uint32_t* keys)
{
    const int tid = threadIdx.x;
    float f[4 * kTmF4];
    if ((S_max & 3) == 0 && S_max >= 4 && (reinterpret_cast<uintptr_t>(s) & 15) == 0) {  // uniform
        // both groups requested at once from clamped addresses (no load inside a branch)
        f32x4 v[kTmF4];
#pragma unroll
        for (int c = 0; c < kTmF4; ++c)
            v[c] = *reinterpret_cast<const f32x4*>(s + min(chunk * kTmChunk + ((c * kTopkThreads + tid) << 2), S_max - 4));
#pragma unroll
        for (int c = 0; c < kTmF4; ++c) { f[4 * c] = v[c].x; f[4 * c + 1] = v[c].y; f[4 * c + 2] = v[c].z; f[4 * c + 3] = v[c].w; }
    } else {
#pragma unroll
        for (int c = 0; c < kTmF4; ++c) {
            const int j = chunk * kTmChunk + ((c * kTopkThreads + tid) << 2);
#pragma unroll
            for (int e = 0; e < 4; ++e) f[4 * c + e] = 0.f;
            if (j + 3 < S_max && ((reinterpret_cast<uintptr_t>(s + j) & 15) == 0)) {
                const f32x4 v = *reinterpret_cast<const f32x4*>(s + j);
                f[4 * c] = v.x; f[4 * c + 1] = v.y; f[4 * c + 2] = v.z; f[4 * c + 3] = v.w;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (j + e < S_max) f[4 * c + e] = s[j + e];
            }
        }
    }
    // (a group past the row read the row's last group: its tokens are at or past S_max >= hi, so their keys are 0)
#pragma unroll
    for (int c = 0; c < kTmF4; ++c) {
        const int j = chunk * kTmChunk + ((c * kTopkThreads + tid) << 2);
#pragma unroll
        for (int e = 0; e < 4; ++e) keys[4 * c + e] = (j + e >= lo && j + e < hi) ? score_key(f[4 * c + e]) : 0u;
    }
}
__device__ __forceinline__ int tm_token(int chunk, int i)
{
    return chunk * kTmChunk + ((((i >> 2) * kTopkThreads) + threadIdx.x) << 2) + (i & 3);
}

// the sequence's linear map from the (min key, max key) pairs of its parts (the chunks of the range kernel, or the
// workgroups of the score kernel): every workgroup derives the same numbers.  All threads of the workgroup must call
// (one barrier); `red` is LDS scratch of 2 * kTopkWaves words.
__device__ __forceinline__ bool tm_range(const uint2* __restrict__ part, int n_part, uint32_t* red, float* flo, float* scale)
{
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    for (int c0 = 0; c0 < n_part; c0 += 2 * kTopkThreads) {  // two loads per thread and trip, from clamped part numbers
        const uint2 a = part[min(c0 + tid, n_part - 1)], b = part[min(c0 + kTopkThreads + tid, n_part - 1)];
        kmin = min(kmin, min(a.x, b.x));
        kmax = max(kmax, max(a.y, b.y));
    }
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if (lane == 0) { red[wave] = kmin; red[kTopkWaves + wave] = kmax; }
    __syncthreads();
    static_assert(kTopkWaves == 16, "one DPP row of wave results");
    kmin = wave_min_u32(red[lane & 15]);
    kmax = wave_max_u32(red[kTopkWaves + (lane & 15)]);
    if (kmax == 0u) return false;  // no candidate at all
    const float a = key_to_score(kmin), span = key_to_score(kmax) - a;
    const float sc = (span > 0.f && span < 3.0e38f) ? (float)kTmBins / span : 0.f;
    *flo = a;
    *scale = sc;
    return sc > 0.f && sc < 3.0e38f && fabsf(a * sc) < 3.0e38f;
}
__device__ __forceinline__ int tm_slot(uint32_t key, float flo, float scale)
{
    const int bin = (int)((key_to_score(key) - flo) * scale);
    return kTmBins - 1 - min(max(bin, 0), kTmBins - 1);
}

__global__ __launch_bounds__(kTopkThreads) void topk_range_kernel(const float* __restrict__ scores,
                                                                  const int32_t* __restrict__ seq_len,
                                                                  TopkMultiWs ws, int S_max, int n_chunk,
                                                                  int n_sink, int n_recent)
{
    __shared__ uint32_t s_min[kTopkWaves], s_max[kTopkWaves];
    const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int S = min(ld_uniform_i32(seq_len + b), S_max);  // (vector memory path: in flight with the scores)
    uint32_t keys[4 * kTmF4];
    tm_load_keys(scores + (size_t)b * S_max, S_max, chunk, n_sink, S - n_recent, keys);
    uint32_t kmin = 0xffffffffu, kmax = 0u;
#pragma unroll
    for (int i = 0; i < 4 * kTmF4; ++i)
        if (keys[i] != 0u) { kmin = min(kmin, keys[i]); kmax = max(kmax, keys[i]); }
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
    if ((tid & 63) == 0) { s_min[tid >> 6] = kmin; s_max[tid >> 6] = kmax; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 0; w < kTopkWaves; ++w) { kmin = min(kmin, s_min[w]); kmax = max(kmax, s_max[w]); }
        ws.part[(size_t)b * n_chunk + chunk] = make_uint2(kmin, kmax);
    }
}

__global__ __launch_bounds__(kTopkThreads) void topk_hist_kernel(const float* __restrict__ scores,
                                                                 const int32_t* __restrict__ seq_len,
                                                                 TopkMultiWs ws, int S_max, int n_chunk,
                                                                 int n_sink, int n_recent)
{
    __shared__ TopkShared sh;  // (its histogram array and scan buffers)
    static_assert(kTmBins == 2 * kTopkThreads && kTmBins <= kTopkBins, "two bins per thread");
    uint32_t* hist = sh.hist;
    const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int S = min(ld_uniform_i32(seq_len + b), S_max);  // (vector memory path: in flight with the scores)
    uint32_t keys[4 * kTmF4];
    tm_load_keys(scores + (size_t)b * S_max, S_max, chunk, n_sink, S - n_recent, keys);
    for (int t = tid; t < kTmBins; t += kTopkThreads) hist[t] = 0u;
    float flo, scale;
    const bool ok = tm_range(ws.range + (size_t)b * ws.n_range, ws.n_range, sh.cand, &flo, &scale);  // (barrier inside)
    if (ok) {
#pragma unroll
        for (int i = 0; i < 4 * kTmF4; ++i)
            if (keys[i] != 0u) atomicAdd(&hist[tm_slot(keys[i], flo, scale)], 1u);
    }
    __syncthreads();
    // running counts from the top: entry s = members of slots 0 .. s-1, entry kTmBins = all of the chunk's candidates
    const uint2 c = *reinterpret_cast<const uint2*>(&hist[2 * tid]);
    int phase = 0;
    uint32_t total;
    const uint32_t above = block_excl_scan(c.x + c.y, sh, phase, &total);
    uint32_t* out = ws.hist + ((size_t)b * n_chunk + chunk) * kTmCum;
    *reinterpret_cast<uint2*>(out + 2 * tid) = make_uint2(above, above + c.x);
    if (tid == 0) out[kTmBins] = total;
}

// The sequence-level decisions, taken identically by every workgroup of the sequence from the chunks' running
// counts: threshold bin, selected members, and the first output position / candidate slot of chunk `chunk`.
// Returns the meta record (fallback set if the chain does not apply).
struct TmResolveLds {
    uint32_t coarse[kTmNC];                       // all chunks' candidates above slot 32 (p + 1)
    uint32_t fine[kTmCoarse + 1];                 // ... above slot 32 P + i
    uint32_t fv[kTmMaxChunks][kTmCoarse + 1];     // the chunks' own counts at those slots
    uint32_t red[2 * kTopkWaves];
    int P, I;
};
__device__ __forceinline__ TopkMeta tm_resolve(TmResolveLds& L, const TopkMultiWs& ws, int b, int chunk, int S,
                                               int n_chunk, int top_k, int n_sink, int n_recent,
                                               uint32_t* base_above, uint32_t* base_cand)
{
    const int tid = threadIdx.x;
    TopkMeta m{};
    const uint32_t* cum = ws.hist + (size_t)b * n_chunk * kTmCum;
    // first pass: the counts at every 32nd slot, summed over the chunks (four loads per thread and trip in flight, from
    // clamped element numbers: no load in a branch)
    const int n1 = kTmNC * n_chunk;
    for (int t = tid; t < kTmNC + kTmCoarse + 1; t += kTopkThreads) (t < kTmNC ? L.coarse[t] : L.fine[t - kTmNC]) = 0u;
    if (tid == 0) { L.P = -1; L.I = -1; }
    uint32_t v1[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int e = min(tid + u * kTopkThreads, n1 - 1);
        v1[u] = cum[(size_t)(e / kTmNC) * kTmCum + (e % kTmNC + 1) * kTmCoarse];
    }
    const bool ok = tm_range(ws.range + (size_t)b * ws.n_range, ws.n_range, L.red, &m.flo, &m.scale) &&  // (barrier inside)
                    S > top_k + n_sink + n_recent && top_k > 0;
    if (!ok) {  // uniform
        m.fallback = 1u;
        return m;
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int e = tid + u * kTopkThreads;
        if (e < n1) atomicAdd(&L.coarse[e % kTmNC], v1[u]);
    }
    for (int e0 = 4 * kTopkThreads; e0 < n1; e0 += 4 * kTopkThreads) {  // (more than 64 chunks)
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = min(e0 + tid + u * kTopkThreads, n1 - 1);
            v[u] = cum[(size_t)(e / kTmNC) * kTmCum + (e % kTmNC + 1) * kTmCoarse];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + tid + u * kTopkThreads;
            if (e < n1) atomicAdd(&L.coarse[e % kTmNC], v[u]);
        }
    }
    __syncthreads();
    if (tid < kTmNC) {
        const uint32_t lo = tid ? L.coarse[tid - 1] : 0u, hi = L.coarse[tid];
        if (lo < (uint32_t)top_k && (uint32_t)top_k <= hi) L.P = tid;
    }
    __syncthreads();
    const int P = L.P;
    if (P < 0) {  // uniform: fewer candidates than top_k in the histograms (cannot happen for a valid range)
        m.fallback = 1u;
        return m;
    }
    // second pass: the counts at the 33 slot boundaries of coarse step P, per chunk and summed
    const int n2 = (kTmCoarse + 1) * n_chunk;
    for (int e0 = 0; e0 < n2; e0 += 4 * kTopkThreads) {
        uint32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = min(e0 + tid + u * kTopkThreads, n2 - 1);
            v[u] = cum[(size_t)(e / (kTmCoarse + 1)) * kTmCum + P * kTmCoarse + e % (kTmCoarse + 1)];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int e = e0 + tid + u * kTopkThreads;
            if (e < n2) {
                L.fv[e / (kTmCoarse + 1)][e % (kTmCoarse + 1)] = v[u];
                atomicAdd(&L.fine[e % (kTmCoarse + 1)], v[u]);
            }
        }
    }
    __syncthreads();
    if (tid < kTmCoarse) {
        const uint32_t lo = L.fine[tid], hi = L.fine[tid + 1];
        if (lo < (uint32_t)top_k && (uint32_t)top_k <= hi) L.I = tid;
    }
    __syncthreads();
    const int I = L.I;
    if (I < 0) {  // uniform (as above)
        m.fallback = 1u;
        return m;
    }
    m.t_slot = (uint32_t)(P * kTmCoarse + I);
    m.n_above = L.fine[I];
    m.members = L.fine[I + 1] - L.fine[I];
    m.kk = (uint32_t)top_k - m.n_above;
    uint32_t a = 0u, mm = 0u;
    for (int c = 0; c < chunk; ++c) {
        a += L.fv[c][I];
        mm += L.fv[c][I + 1] - L.fv[c][I];
    }
    *base_above = a;
    *base_cand = mm;
    m.fallback = m.members > (uint32_t)kTmCand ? 1u : 0u;
    return m;
}

__global__ __launch_bounds__(kTopkThreads) void topk_place_kernel(const float* __restrict__ scores,
                                                                  const int32_t* __restrict__ seq_len,
                                                                  TopkMultiWs ws, int32_t* __restrict__ idx,
                                                                  int S_max, int n_chunk, int top_k, int n_sink,
                                                                  int n_recent)
{
    __shared__ TopkShared sh;
    __shared__ TmResolveLds rl;
    const int chunk = blockIdx.x, b = blockIdx.y;
    const int S = min(ld_uniform_i32(seq_len + b), S_max);  // (vector memory path: in flight with the scores)
    uint32_t keys[4 * kTmF4];
    tm_load_keys(scores + (size_t)b * S_max, S_max, chunk, n_sink, S - n_recent, keys);
    uint32_t base_above = 0u, base_cand = 0u;
    const TopkMeta m = tm_resolve(rl, ws, b, chunk, wave_uniform(S), n_chunk, top_k, n_sink, n_recent, &base_above,
                                  &base_cand);
    if (chunk == 0 && threadIdx.x == 0) ws.meta[b] = m;  // for the finish kernel
    if (m.fallback) return;
    int slot[4 * kTmF4];
    uint32_t n_ab = 0u, n_eq = 0u;
#pragma unroll
    for (int i = 0; i < 4 * kTmF4; ++i) {
        slot[i] = keys[i] != 0u ? tm_slot(keys[i], m.flo, m.scale) : kTmBins;  // non-candidates: below every bin
        n_ab += slot[i] < (int)m.t_slot;
        n_eq += slot[i] == (int)m.t_slot;
    }
    int phase = 0;
    uint32_t tot_ab, tot_eq;
    __syncthreads();
    block_excl_scan2(n_ab, n_eq, sh, phase, &tot_ab, &tot_eq);
    int32_t* out = idx + (size_t)b * (top_k + n_sink + n_recent) + n_sink;
    uint2* cand = ws.cand + (size_t)b * kTmCand;
    uint32_t pa = base_above + n_ab, pc = base_cand + n_eq;
#pragma unroll
    for (int i = 0; i < 4 * kTmF4; ++i) {
        const int j = tm_token(chunk, i);
        if (slot[i] < (int)m.t_slot) { if (pa < (uint32_t)top_k) out[pa] = j; ++pa; }
        else if (slot[i] == (int)m.t_slot) { if (pc < (uint32_t)kTmCand) cand[pc] = make_uint2(keys[i], (uint32_t)j); ++pc; }
    }
}

// finish: ranks the candidates; a flagged sequence is selected from scratch by this workgroup
__global__ __launch_bounds__(kTopkThreads) void topk_finish_kernel(const float* __restrict__ scores,
                                                                   const int32_t* __restrict__ seq_len,
                                                                   TopkMultiWs ws, int32_t* __restrict__ idx,
                                                                   int32_t* __restrict__ n_sel, int S_max, int top_k,
                                                                   int n_sink, int n_recent, WindowLists wl)
{
    __shared__ TopkShared sh;
    __shared__ uint2 s_c[kTmCand];
    __shared__ uint32_t s_sel[kTmCand];
    const int b = blockIdx.x, tid = threadIdx.x;
    write_window_lists(wl, seq_len, b, S_max, top_k + n_sink + n_recent, kTopkThreads);
    // (the candidate pair, the length and the meta record are requested together; slots past the member count hold
    // stale pairs and are masked)
    const uint2 me_raw = ws.cand[(size_t)b * kTmCand + min(tid, kTmCand - 1)];
    const int S_v = ld_uniform_i32(seq_len + b);
    const TopkMeta m = ws.meta[b];
    if (m.fallback) {  // uniform
        topk_select_sequence<0>(sh, scores, seq_len, idx, n_sel, b, S_max, top_k, n_sink, n_recent);
        return;
    }
    const int S = min(wave_uniform(S_v), S_max);
    const int k_tot = top_k + n_sink + n_recent;
    int32_t* out = idx + (size_t)b * k_tot;
    for (int t = tid; t < n_sink; t += kTopkThreads) out[t] = t;
    for (int t = tid; t < n_recent; t += kTopkThreads) out[n_sink + top_k + t] = S - n_recent + t;
    if (tid == 0) n_sel[b] = k_tot;
    const uint32_t nm = m.members;
    const uint2 me = (uint32_t)tid < nm ? me_raw : make_uint2(0u, 0u);
    if (tid < kTmCand) s_c[tid] = me;
    __syncthreads();
    // rank among the members: larger key first, equal keys by smaller token index
    uint32_t before = 0u;
    if ((uint32_t)tid < nm)
        for (uint32_t c = 0; c < nm; ++c) {
            const uint2 o = s_c[c];
            before += (o.x > me.x) || (o.x == me.x && o.y < me.y);
        }
    const uint32_t sel = ((uint32_t)tid < nm && before < m.kk) ? 1u : 0u;
    if (tid < kTmCand) s_sel[tid] = sel;
    __syncthreads();
    if (sel) {  // position in token order among the selected members
        uint32_t pos = 0u;
        for (uint32_t c = 0; c < nm; ++c) pos += s_sel[c] && s_c[c].y < me.y;
        out[n_sink + m.n_above + pos] = (int32_t)me.y;
    }
}

}  // namespace sals
