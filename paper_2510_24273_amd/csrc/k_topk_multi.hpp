// Critical-token selection for long sequences (Algorithm 1, TopK step; Sec. 5.2 composition),
// spread over many workgroups.
//
// One workgroup walks a compute unit's worth of instructions per key and pass, so beyond a few
// ten thousand scores a single workgroup per sequence is the bottleneck.  Here a sequence is cut
// into chunks of 8192 scores, one workgroup each, and the selection runs as a chain of small
// kernels that exchange a few kilobytes:
//   range    per chunk: minimum and maximum candidate key
//   hist     per chunk: histogram over 2048 linear bins of the sequence's [min, max]
//   place    per chunk: from all chunk histograms, the bin holding the top_k-th score, how many of
//            its members are selected and where the chunk's output starts (every workgroup of the
//            sequence derives the same numbers); then the indices of the scores in higher bins go
//            to their final positions (chunk order, then token order) and the members of the
//            threshold bin to a candidate list
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
    uint2* part;         // [B][n_chunk] (min key, max key) of the chunk's candidates
    uint32_t* hist;      // [B][n_chunk][kTmBins]
    TopkMeta* meta;      // [B]
    uint2* cand;         // [B][kTmCand] (key, token index)
};

// keys of this thread's 8 scores of chunk `chunk`: tokens chunk*8192 + 4*(c*1024 + tid) + e;
// non-candidates (sink / recent tokens, positions past the sequence) carry key 0
__device__ __forceinline__ void tm_load_keys(const float* __restrict__ s, int S_max, int chunk, int lo, int hi,
                                            uint32_t* keys)
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int c = 0; c < kTmF4; ++c) {
        const int j = chunk * kTmChunk + ((c * kTopkThreads + tid) << 2);
        float f[4] = {0.f, 0.f, 0.f, 0.f};
        if (j + 3 < S_max && ((reinterpret_cast<uintptr_t>(s + j) & 15) == 0)) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(s + j);
            f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (j + e < S_max) f[e] = s[j + e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) keys[4 * c + e] = (j + e >= lo && j + e < hi) ? score_key(f[e]) : 0u;
    }
}
__device__ __forceinline__ int tm_token(int chunk, int i)
{
    return chunk * kTmChunk + ((((i >> 2) * kTopkThreads) + threadIdx.x) << 2) + (i & 3);
}

// the sequence's linear map from its chunks' (min, max): every workgroup derives the same numbers
__device__ __forceinline__ bool tm_range(const uint2* __restrict__ part, int n_chunk, float* flo, float* scale)
{
    // every wave reads all chunks' pairs itself, two per lane and round, and folds them with lane shuffles: no
    // barrier, and one memory round trip instead of one per chunk
    uint32_t kmin = 0xffffffffu, kmax = 0u;
    const int lane = threadIdx.x & (kWave - 1);
    for (int c0 = 0; c0 < n_chunk; c0 += 2 * kWave) {
        const int ca = c0 + lane, cb = c0 + kWave + lane;
        const uint2 a = part[min(ca, n_chunk - 1)], b = part[min(cb, n_chunk - 1)];  // (clamped: duplicates are harmless)
        kmin = min(kmin, min(a.x, b.x));
        kmax = max(kmax, max(a.y, b.y));
    }
    kmin = wave_min_u32(kmin);
    kmax = wave_max_u32(kmax);
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
    __shared__ uint32_t hist[kTmBins];
    const int chunk = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int S = min(ld_uniform_i32(seq_len + b), S_max);  // (vector memory path: in flight with the scores)
    uint32_t keys[4 * kTmF4];
    tm_load_keys(scores + (size_t)b * S_max, S_max, chunk, n_sink, S - n_recent, keys);
    for (int t = tid; t < kTmBins; t += kTopkThreads) hist[t] = 0u;
    float flo, scale;
    const bool ok = tm_range(ws.part + (size_t)b * n_chunk, n_chunk, &flo, &scale);
    __syncthreads();
    if (ok) {
#pragma unroll
        for (int i = 0; i < 4 * kTmF4; ++i)
            if (keys[i] != 0u) atomicAdd(&hist[tm_slot(keys[i], flo, scale)], 1u);
    }
    __syncthreads();
    uint32_t* out = ws.hist + ((size_t)b * n_chunk + chunk) * kTmBins;
    for (int t = tid; t < kTmBins; t += kTopkThreads) out[t] = hist[t];
}

// The sequence-level decisions, taken identically by every workgroup of the sequence from the
// chunk histograms: threshold bin, selected members, and the first output position / candidate
// slot of chunk `chunk`.  Returns the meta record (fallback set if the chain does not apply).
__device__ __forceinline__ TopkMeta tm_resolve(TopkShared& sh, uint32_t* s_above, uint32_t* s_memb,
                                               const TopkMultiWs& ws, int b, int chunk, int S, int n_chunk,
                                               int top_k, int n_sink, int n_recent, uint32_t* base_above,
                                               uint32_t* base_cand)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    TopkMeta m{};
    // this thread's two bins, summed over the chunks; the first eight chunks' loads are requested together with
    // the chunks' score ranges (from clamped chunk numbers: no load in a branch)
    const uint32_t* hb = ws.hist + (size_t)b * n_chunk * kTmBins + 2 * tid;
    uint2 v0[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v0[u] = *reinterpret_cast<const uint2*>(hb + (size_t)min(u, n_chunk - 1) * kTmBins);
    const bool ok = tm_range(ws.part + (size_t)b * n_chunk, n_chunk, &m.flo, &m.scale) &&
                    S > top_k + n_sink + n_recent && top_k > 0;
    if (!ok) {  // uniform
        m.fallback = 1u;
        return m;
    }
    uint32_t c0 = 0u, c1 = 0u;
#pragma unroll
    for (int u = 0; u < 8; ++u) { c0 += u < n_chunk ? v0[u].x : 0u; c1 += u < n_chunk ? v0[u].y : 0u; }
    for (int c = 8; c < n_chunk; c += 8) {
        uint2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = c + u < n_chunk ? *reinterpret_cast<const uint2*>(hb + (size_t)(c + u) * kTmBins) : make_uint2(0u, 0u);
#pragma unroll
        for (int u = 0; u < 8; ++u) { c0 += v[u].x; c1 += v[u].y; }
    }
    int phase = 0;
    uint32_t total;
    uint32_t above = block_excl_scan(c0 + c1, sh, phase, &total);
    if (above < (uint32_t)top_k && (uint32_t)top_k <= above + c0) {
        sh.sel_prefix = 2 * tid; sh.sel_kk = (uint32_t)top_k - above; sh.n_cand = c0;
    } else if (above + c0 < (uint32_t)top_k && (uint32_t)top_k <= above + c0 + c1) {
        sh.sel_prefix = 2 * tid + 1; sh.sel_kk = (uint32_t)top_k - above - c0; sh.n_cand = c1;
    }
    __syncthreads();
    m.t_slot = sh.sel_prefix; m.kk = sh.sel_kk; m.members = sh.n_cand;
    // per chunk: scores in bins above the threshold, members of the threshold bin (a wave per chunk)
    for (int c = wave; c < n_chunk; c += kTopkWaves) {
        const uint32_t* hc = ws.hist + ((size_t)b * n_chunk + c) * kTmBins;
        u32x4 v[kTmBins / (4 * kWave)];  // the whole histogram of the chunk, all loads in flight at once
#pragma unroll
        for (int i = 0; i < kTmBins / (4 * kWave); ++i) v[i] = *reinterpret_cast<const u32x4*>(hc + 4 * (lane + kWave * i));
        uint32_t sum = 0u;
#pragma unroll
        for (int i = 0; i < kTmBins / (4 * kWave); ++i) {
            const uint32_t s0 = 4u * (lane + kWave * i);
            sum += (s0 < m.t_slot ? v[i].x : 0u) + (s0 + 1 < m.t_slot ? v[i].y : 0u) + (s0 + 2 < m.t_slot ? v[i].z : 0u) +
                   (s0 + 3 < m.t_slot ? v[i].w : 0u);
        }
        sum = wave_sum_u32(sum);
        if (lane == 0) { s_above[c] = sum; s_memb[c] = hc[m.t_slot]; }
    }
    __syncthreads();
    uint32_t a = 0u, mm = 0u, a_here = 0u, m_here = 0u;
    for (int c = 0; c < n_chunk; ++c) {
        if (c == chunk) { a_here = a; m_here = mm; }
        a += s_above[c]; mm += s_memb[c];
    }
    *base_above = a_here;
    *base_cand = m_here;
    m.n_above = a;
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
    __shared__ uint32_t s_above[kTmMaxChunks], s_memb[kTmMaxChunks];
    const int chunk = blockIdx.x, b = blockIdx.y;
    const int S = min(ld_uniform_i32(seq_len + b), S_max);  // (vector memory path: in flight with the scores)
    uint32_t keys[4 * kTmF4];
    tm_load_keys(scores + (size_t)b * S_max, S_max, chunk, n_sink, S - n_recent, keys);
    uint32_t base_above = 0u, base_cand = 0u;
    const TopkMeta m = tm_resolve(sh, s_above, s_memb, ws, b, chunk, wave_uniform(S), n_chunk, top_k, n_sink, n_recent,
                                  &base_above, &base_cand);
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
    // (requested together with the meta record; slots past the member count hold stale pairs and are masked)
    const uint2 me_raw = tid < kTmCand ? ws.cand[(size_t)b * kTmCand + tid] : make_uint2(0u, 0u);
    const TopkMeta m = ws.meta[b];
    if (m.fallback) {  // uniform
        topk_select_sequence<0>(sh, scores, seq_len, idx, n_sel, b, S_max, top_k, n_sink, n_recent);
        return;
    }
    const int S = min(seq_len[b], S_max);
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
