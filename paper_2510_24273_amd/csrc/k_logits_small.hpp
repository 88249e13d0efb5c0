// Selective key reconstruction with fused RoPE and query dot product, latency-oriented
// variant for problems with few (sequence, head, token tile) combinations
// (Algorithm 1, reconstruction / RoPE / logit steps; Sec. 4.4).
//
// Same arithmetic as attend_logits_kernel, on a 1 KV head x 64 token tile per workgroup.
// With few workgroups the time is set by how many bytes a compute unit keeps in flight, so
// every thread issues its loads for NST <= 10 128-byte steps of the latent axis (the whole
// axis for r = 640 in bf16) before anything is consumed: up to 120 registers of staging per lane.
// The steps then move through a double-buffered LDS stage two at a time; the eight waves are
// (k-step parity) x (half of the RoPE pairs) x (32-token block), so both steps of an
// iteration are multiplied concurrently.  Afterwards the two parities exchange halves of
// their accumulators, every wave rotates and dots a quarter of the pairs, and the first wave
// adds the four partial dot products per token and reduces the tile's softmax statistics.
//
// With very few tiles (a recent window at batch 1, a GQA model at batch 1) the latent axis is also split over
// `ksplit` workgroups per tile: the logit is a sum over latent coordinates (reconstruction, rotation and the dot
// product are all linear in K~), so every slice writes its partial logits and logits_finish_kernel adds the slices
// in slice order and takes the statistics.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"
#include "k_logits.hpp"
#include "k_topk.hpp"

namespace sals {

constexpr int kLsThreads = 512;
constexpr int kLsTok = 64;                                   // tokens per workgroup
constexpr int kLsMaxChunk = 10;                              // latent steps loaded ahead, at most
constexpr int kLsStepBytes = (kHeadDim + kLsTok) * kLgChunk;  // U_k panel + gathered rows: 24 KB
constexpr int kLsIterBytes = 2 * kLsStepBytes;               // two steps per iteration
constexpr size_t kLsLds = 2 * (size_t)kLsIterBytes;          // double buffered: 96 KB

// FUSED: the kernel also selects.  With one short sequence the selection kernel is a launch of its own that costs more
// than its work (a dependent launch is worth about 2.3 us, the kernel 4.4 us at 4096 tokens), so here every workgroup
// of a sequence repeats the selection itself from the scores (S_max <= 4096: eight keys per thread, in LDS that the
// stage buffers only need later) while its first U_k steps are in flight, and takes its tile from the list; the
// workgroups of KV head 0 write the list and the count to `idx` / `n_sel` for the stages that follow.  The list is the
// one topk_kernel would have written, entry for entry.
struct FusedSelect {
    const float* scores;      // [B, S_max]
    const int32_t* seq_len;   // [B]
    int top_k, n_sink, n_recent;
};
constexpr int kLsFusedMaxS = 4096, kLsFusedMaxK = 1024;

template <typename T, int NST, bool FUSED = false>
__global__ __launch_bounds__(kLsThreads) void attend_logits_small_kernel(
    // (what the workgroup's first loads need comes first: those 14 words arrive preloaded in scalar registers)
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_sel, const T* __restrict__ UkP,
    int B, int H_kv, int n_parts, int heads_fastest, int ksplit, int k_tot, int r, int H,
    const T* __restrict__ Kc, const T* __restrict__ q, const int32_t* __restrict__ q_pos,
    const float2* __restrict__ rope, InvFreq inv,
    float* __restrict__ logits, float2* __restrict__ stats, int S_max,
    int lk, int style, float scale, int ring,
    float* __restrict__ plogits, int stats_stride, FusedSelect fs)
{
    constexpr int ES = (int)sizeof(T);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int ksel = wave & 1, dh = (wave >> 1) & 1, tb = wave >> 2;
    const int G = H / H_kv;

    // workgroup id -> (sequence, token tile, KV head), one contiguous range of the list per XCD
    int b, g, part, kz;  // kz: this workgroup's slice of the latent axis (the slices of a tile are neighbours)
    {
        const int N = n_parts * H_kv * B * ksplit;
        const int id = blockIdx.x, xcd = id % kXcds, slot = id / kXcds;
        const int qn = N / kXcds, rem = N % kXcds;
        const int wk = (xcd < rem ? xcd * (qn + 1) : rem * (qn + 1) + (xcd - rem) * qn) + slot;
        const int w = wk / ksplit;
        kz = wk - w * ksplit;
        if (heads_fastest) {
            const int bt = w / H_kv;
            g = w - bt * H_kv; b = bt / n_parts; part = bt - b * n_parts;
        } else {
            g = w / (n_parts * B);
            const int bt = w - g * (n_parts * B);
            b = bt / n_parts; part = bt - b * n_parts;
        }
    }
    const int tok0 = part * kLsTok;

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // [2][2 steps][A | B]
    __shared__ __attribute__((aligned(16))) float sQ[kMaxGroup][kHeadDim];

    // ---- everything the tile loads depend on is requested first, in one round trip ----------
    // per step, piece t of the U_k panel is (slot t/8, column t%8) and piece 512+t is slot
    // 64 + t/8; piece t of the gathered rows is (token t/8, column t%8)
    const int prow = tid >> 3, pcol = tid & 7;
    const int my_slot = tok0 + prow;
    const int e_slot = tok0 + tb * 32 + l32;  // token this lane finishes in the epilogue
    const int32_t* ib = idx + (size_t)b * k_tot;
    int idx_my = 0, idx_e = 0, idx_0 = 0, n_v = 0;
    if constexpr (!FUSED) {
        idx_my = ib[min(my_slot, k_tot - 1)]; idx_e = ib[min(e_slot, k_tot - 1)]; idx_0 = ib[0];
        n_v = ld_uniform_i32(n_sel + b);
    }
    const int qpos_v = ld_uniform_i32(q_pos + b);  // in flight with the loads around
    // raw query pair (m = tid / 64, p = tid % 64) and the cos/sin of the query position for pair p
    const int qp = tid & (kPairs - 1), qm = min(tid >> 6, G - 1);
    const T* qrow = q + ((size_t)b * H + (size_t)g * G + qm) * kHeadDim;
    const float qa = elem<T>::load(qrow + pair_first(qp, style));
    const float qb = elem<T>::load(qrow + pair_second(qp, style));

    // the packed U_k panel is [64-byte block of the latent axis][128 slots][64 B]: a 128-byte step is two
    // blocks 8 KB apart, and piece (slot, column c) lies in block c/4 at slot*64 + (c%4)*16
    const unsigned char* a_src = reinterpret_cast<const unsigned char*>(UkP + (size_t)g * kHeadDim * r) +
                                 (pcol >> 2) * (kHeadDim * 64) + prow * 64 + (pcol & 3) * 16;
    const int a_dst0 = swz(prow, pcol), a_dst1 = swz(64 + prow, pcol);
    const int b_dst = kHeadDim * kLgChunk + swz(prow, pcol);
    const int nkc = r * ES / kLgChunk / ksplit;  // 128-byte steps of this slice (the host makes it a whole number)
    a_src += (size_t)kz * nkc * (kHeadDim * kLgChunk);

    f32x16 acc0, acc1;  // slots dh*32 + (8a + 4hi + c) and their pair partners (+64)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc0[v] = acc1[v] = 0.f;

    auto compute = [&](const unsigned char* stage) {
        const unsigned char* pa = stage;
        const unsigned char* pb = stage + kHeadDim * kLgChunk;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const u32x4 bf = *reinterpret_cast<const u32x4*>(pb + swz(tb * 32 + l32, ks * 2 + hi));
            const u32x4 a0 = *reinterpret_cast<const u32x4*>(pa + swz(dh * 32 + l32, ks * 2 + hi));
            const u32x4 a1 = *reinterpret_cast<const u32x4*>(pa + swz((dh + 2) * 32 + l32, ks * 2 + hi));
            mma_op<T>::run(a0, bf, acc0);
            mma_op<T>::run(a1, bf, acc1);
        }
    };

    // ---- main loop: chunks of NST steps (NST divides the step count), all loads of a chunk issued
    // at once in the order the iterations consume them.  Trip counts are compile-time constants
    // and nothing below is conditional, so every wait names exactly the loads it needs. ------------
    u32x4 P[NST][3];
    auto load_a = [&](int c0, int s) {
        const size_t ao = (size_t)(c0 + s) * (kHeadDim * kLgChunk);
        P[s][0] = ld16(a_src + ao);
        P[s][1] = ld16(a_src + ao + 64 * 64);  // slot 64 + t/8
    };
    // U_k steps requested before the row indices arrive (all of them when the selection runs here first: it takes
    // longer than a load of the list)
    constexpr int EARLY = FUSED ? NST : (NST < 4 ? NST : 4);
#pragma unroll
    for (int s = 0; s < EARLY; ++s) load_a(0, s);
    if constexpr (FUSED) {
        // the selection, in LDS that the stage buffers take over afterwards
        TopkShared& sh = *reinterpret_cast<TopkShared*>(lds);
        int32_t* s_idx = reinterpret_cast<int32_t*>(lds + ((sizeof(TopkShared) + 255) & ~(size_t)255));  // [k_tot], then the count
        topk_select_sequence<kLsFusedMaxS / (4 * kLsThreads), kLsThreads, true>(
            sh, fs.scores + (size_t)b * S_max, fs.seq_len + b, s_idx, s_idx + kLsFusedMaxK, 0, S_max, fs.top_k, fs.n_sink,
            fs.n_recent);
        __syncthreads();
        n_v = s_idx[kLsFusedMaxK];
        idx_my = s_idx[min(my_slot, k_tot - 1)]; idx_e = s_idx[min(e_slot, k_tot - 1)]; idx_0 = s_idx[0];
        if (g == 0 && kz == 0) {  // this tile's share of the list for the value stages (idx is an output here)
            int32_t* ob = const_cast<int32_t*>(idx) + (size_t)b * k_tot;
            if (tid < kLsTok && tok0 + tid < k_tot) ob[tok0 + tid] = s_idx[tok0 + tid];
            if (part == 0 && tid == 0) const_cast<int32_t*>(n_sel)[b] = n_v;
        }
        __syncthreads();  // (the list has been read: the stage buffers may be written)
    }
    const int n = wave_uniform(n_v);
    if (tok0 >= n) {  // no selected token in this tile: neutral statistics (split tiles: the finishing kernel's job)
        if (tid < G && ksplit == 1)
            stats[((size_t)b * H + (size_t)g * G + tid) * stats_stride + part] = make_float2(-INFINITY, 0.f);
        return;
    }
    // slots past the selected tokens read the first selected row; they get no weight
    const int my_pos = min(max(my_slot < n ? idx_my : idx_0, 0), S_max - 1);
    const int my_row = ring > 0 ? my_pos % ring : my_pos;  // ring cache: token t lies in row t mod ring
    const unsigned char* b_src =
        reinterpret_cast<const unsigned char*>(Kc + ((size_t)b * (ring > 0 ? ring : S_max) + my_row) * r) + pcol * 16 +
        (size_t)kz * nkc * kLgChunk;
#pragma unroll
    for (int s = 0; s < NST; ++s) P[s][2] = ld16(b_src + (size_t)s * kLgChunk);
#pragma unroll
    for (int s = EARLY; s < NST; ++s) load_a(0, s);
    const int qpos = wave_uniform(qpos_v);
    const bool q_in_table = qpos >= 0 && qpos <= S_max;  // the table holds exactly the needed values
    float2 qcs = rope[(size_t)(q_in_table ? qpos : 0) * kPairs + qp];
    f32x4 cs0[2], cs1[2];  // cos/sin of this lane's pairs
    {
        const int e_pos = min(max(e_slot < n ? idx_e : idx_0, 0), S_max - 1);
        const float2* csrow = rope + (size_t)e_pos * kPairs;
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) {
            const int p0 = dh * 32 + (2 * ksel + aa) * 8 + hi * 4;
            cs0[aa] = *reinterpret_cast<const f32x4*>(csrow + p0);      // (c,s) of pairs p0, p0+1
            cs1[aa] = *reinterpret_cast<const f32x4*>(csrow + p0 + 2);  // pairs p0+2, p0+3
        }
    }
    // compiler-level fence: keeps every load above from being sunk towards its first use
    asm volatile("" ::: "memory");
    int it = 0;
    for (int c0 = 0;;) {
#pragma unroll
        for (int i = 0; i < (NST + 1) / 2; ++i) {
            unsigned char* buf = lds + (size_t)(it & 1) * kLsIterBytes;
            ++it;
#pragma unroll
            for (int h2 = 0; h2 < 2; ++h2) {
                if (2 * i + h2 < NST) {
                    unsigned char* st = buf + h2 * kLsStepBytes;
                    *reinterpret_cast<u32x4*>(st + a_dst0) = P[2 * i + h2][0];
                    *reinterpret_cast<u32x4*>(st + a_dst1) = P[2 * i + h2][1];
                    *reinterpret_cast<u32x4*>(st + b_dst) = P[2 * i + h2][2];
                }
            }
            __syncthreads();
            if (2 * i + 1 < NST || ksel == 0) compute(buf + ksel * kLsStepBytes);
        }
        c0 += NST;
        if (c0 >= nkc) break;
#pragma unroll
        for (int s = 0; s < NST; ++s) {
            load_a(c0, s);
            P[s][2] = ld16(b_src + (size_t)(c0 + s) * kLgChunk);
        }
        asm volatile("" ::: "memory");
    }
    // rotated, scaled query
    if (!q_in_table) {  // uniform
        double sn, c;
        sincos((double)qpos * inv.f[qp], &sn, &c);
        qcs = make_float2((float)c, (float)sn);
    }
    if (tid < G * kPairs) {
        sQ[tid >> 6][qp] = (qa * qcs.x - qb * qcs.y) * scale;
        sQ[tid >> 6][kPairs + qp] = (qb * qcs.x + qa * qcs.y) * scale;
    }
    __syncthreads();  // every product is done: the stage buffers are free

    // ---- the two k-step parities exchange halves: parity 0 keeps a in {0,1}, parity 1 a in {2,3}
    {
        float* xch = reinterpret_cast<float*>(lds);  // [pair of waves 4][parity 2][16][64]
        float* mine = xch + ((size_t)((wave >> 1) * 2 + ksel) * 16) * 64 + lane;
        const float* theirs = xch + ((size_t)((wave >> 1) * 2 + (ksel ^ 1)) * 16) * 64 + lane;
        // (static register indices on both sides of a uniform branch: a select between two
        // accumulator elements would turn into a long chain of per-element selects)
        float x1[8], x2[8];  // this wave's kept first / second pair elements, index aa*4 + c
        if (ksel) {
#pragma unroll
            for (int v = 0; v < 8; ++v) { mine[v * 64] = acc0[v]; mine[(8 + v) * 64] = acc1[v]; x1[v] = acc0[8 + v]; x2[v] = acc1[8 + v]; }
        } else {
#pragma unroll
            for (int v = 0; v < 8; ++v) { mine[v * 64] = acc0[8 + v]; mine[(8 + v) * 64] = acc1[8 + v]; x1[v] = acc0[v]; x2[v] = acc1[v]; }
        }
        __syncthreads();
        float k1[2][4], k2[2][4];
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) {
            const f32x4 t0 = cs0[aa], t1 = cs1[aa];
            const float cc[4] = {t0.x, t0.z, t1.x, t1.z}, ss[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                const int v = aa * 4 + c;
                const float y1 = x1[v] + theirs[v * 64];
                const float y2 = x2[v] + theirs[(8 + v) * 64];
                k1[aa][c] = y1 * cc[c] - y2 * ss[c];
                k2[aa][c] = y2 * cc[c] + y1 * ss[c];
            }
        }
        // partial dot products over this wave's 16 pairs, per query head of the group
        float* sDot = xch + 8 * 16 * 64;  // [token block 2][wave part 4][kMaxGroup][32]
#pragma unroll
        for (int m = 0; m < kMaxGroup; ++m) {
            if (m < G) {  // uniform
                float d = 0.f;
#pragma unroll
                for (int aa = 0; aa < 2; ++aa) {
                    const int p0 = dh * 32 + (2 * ksel + aa) * 8 + hi * 4;
                    const f32x4 q1 = *reinterpret_cast<const f32x4*>(&sQ[m][p0]);
                    const f32x4 q2 = *reinterpret_cast<const f32x4*>(&sQ[m][kPairs + p0]);
                    d += q1.x * k1[aa][0] + q1.y * k1[aa][1] + q1.z * k1[aa][2] + q1.w * k1[aa][3] +
                         q2.x * k2[aa][0] + q2.y * k2[aa][1] + q2.z * k2[aa][2] + q2.w * k2[aa][3];
                }
                d += __shfl_xor(d, 32, kWave);
                if (hi == 0) sDot[((tb * 4 + dh * 2 + ksel) * kMaxGroup + m) * 32 + l32] = d;
            }
        }
        __syncthreads();
        // ---- first wave: logits of the 64 tokens and the tile's softmax statistics ---------------
        if (wave == 0) {
            const int slot = tok0 + lane;
            const bool valid = slot < n;
            for (int m = 0; m < G; ++m) {
                const float* dp = sDot + ((size_t)(lane >> 5) * 4 * kMaxGroup + m) * 32 + (lane & 31);
                const float d = (dp[0] + dp[kMaxGroup * 32]) + (dp[2 * kMaxGroup * 32] + dp[3 * kMaxGroup * 32]);
                const size_t hrow = (size_t)b * H + (size_t)g * G + m;
                if (ksplit > 1) {  // uniform: this slice's share of the logit
                    if (slot < lk) plogits[((size_t)kz * B * H + hrow) * lk + slot] = d;
                    continue;
                }
                if (slot < lk) logits[hrow * lk + slot] = valid ? d : -INFINITY;
                const float mx = wave_max(valid ? d : -INFINITY);
                const float se = wave_sum(valid ? __expf(d - mx) : 0.f);
                if (lane == 0) stats[hrow * stats_stride + part] = make_float2(mx, se);
            }
        }
    }
}

// Split tiles: logits = sum of the latent slices' partial logits, in slice order, and the tile's softmax
// statistics.  grid (n_parts, B*H), 64 threads (one per token of the tile).
constexpr int kLsMaxSplit = 8;
__global__ __launch_bounds__(64) void logits_finish_kernel(const float* __restrict__ plogits, int ksplit,
                                                           const int32_t* __restrict__ n_sel,
                                                           float* __restrict__ logits, float2* __restrict__ stats,
                                                           int B, int H, int lk, int stats_stride)
{
    const int part = blockIdx.x, lane = threadIdx.x;
    const size_t hrow = blockIdx.y;
    const int slot = part * kLsTok + lane;
    float v[kLsMaxSplit];
#pragma unroll
    for (int u = 0; u < kLsMaxSplit; ++u)  // all slices requested together, from clamped addresses
        v[u] = plogits[((size_t)min(u, ksplit - 1) * B * H + hrow) * lk + min(slot, lk - 1)];
    const int n = n_sel[hrow / H];
    float d = 0.f;
#pragma unroll
    for (int u = 0; u < kLsMaxSplit; ++u) d += u < ksplit ? v[u] : 0.f;
    const bool valid = slot < n;
    if (slot < lk) logits[hrow * lk + slot] = valid ? d : -INFINITY;
    const float mx = wave_max(valid ? d : -INFINITY);
    const float se = wave_sum(valid ? __expf(d - mx) : 0.f);
    if (lane == 0) stats[hrow * stats_stride + part] = make_float2(mx, se);
}

}  // namespace sals
