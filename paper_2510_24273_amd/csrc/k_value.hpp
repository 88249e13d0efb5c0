// The value path of the sparse attention (Eq. 5; Algorithm 1, output step), evaluated as
// y_h = ((p_h V~_C) U_v[g(h) block]^T) : the same sum as p_h (V~_C U_v^T) in another order,
// so the selected values are never reconstructed.
//
//   attend_pv   per (sequence, token range, 64 latent columns):
//               T[h,:] = sum_j p_hj V~[C_j,:]  on the matrix cores, tokens being the
//               contraction axis (each step split over the workgroup's four or eight waves); the gathered
//               rows are transposed through LDS on the way.  The softmax weights are formed
//               on the fly, p = exp(logit - m_h) / Z_h, with m_h and Z_h merged in the prologue
//               from the per-tile statistics the logits kernel left.  Each token range writes an
//               fp32 partial sum.
//   attend_out  y[(b,h), c] = sum_i T[(b,h), i] U_v[g*128 + c, i]  on the matrix cores, after
//               adding the range partials in range order.
//
// bf16 storage: the fp32 weights p and the fp32 T are split into a bf16 head and a bf16
// remainder (two MFMAs each), which keeps about 16 mantissa bits.  fp32 storage: fp32 MFMAs.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"
#include "k_project.hpp"

namespace sals {

constexpr int kPvTJ = 64;          // token ranges are whole multiples of this (of twice this for the eight-wave kernel)
constexpr int kPvCols = 64;        // latent columns per workgroup
constexpr int kPvMaxHeads = 64;    // H_q limit of these kernels
constexpr int kMaxRanges = 8;      // token ranges per sequence (the output projection adds them up)
constexpr int kPvMaxTok = 4096;    // tokens per workgroup, at most (their cache rows sit in LDS)

// NW waves (4 or 8), each with one MFMA token group of every step: the eight-wave form halves the number of
// steps (a step is a chain of dependent latencies), the four-wave form starts and finishes faster.
template <typename T, int NW>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void attend_pv_kernel(
    // (what the workgroup's first loads need comes first: those 14 words arrive preloaded in scalar registers)
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_sel, const float2* __restrict__ stats,
    int B, int r, int n_tr, int n_parts, int tok_per_wg, int k_tot, int H, int lk,
    const T* __restrict__ Vc, const float* __restrict__ logits, float* __restrict__ Tpart, int S_max, int ring)
{
    static_assert(NW == 4 || NW == 8, "four or eight waves");
    constexpr int kPvThreads = NW * 64, kPvWaves = NW;
    constexpr int ES = (int)sizeof(T);
    constexpr int VEC = elem<T>::vec;        // tokens per lane per MFMA group = elements per 16 bytes
    constexpr int KG = 2 * VEC;              // tokens per MFMA group (both half-waves)
    constexpr int TJ = kPvWaves * KG;        // tokens per step: one MFMA group per wave
    constexpr int NKG = TJ / KG;             // MFMA groups per step, dealt to the waves
    constexpr bool kSplit = ES == 2;
    constexpr int PPR = kPvCols * ES / 16;   // 16-byte pieces per gathered row
    constexpr int NPC = TJ * PPR / kPvThreads;  // pieces per thread per step
    constexpr int PITCH = TJ * ES + 8;       // bytes per column of the transposed tile (8-byte reads stay aligned)

    // V~ rows arrive as they lie in memory (16 bytes = VEC columns of one token per lane) and are
    // written to LDS transposed, [column][token], so that an MFMA operand (one column, VEC consecutive
    // tokens per lane) is two 8-byte reads.
    constexpr int VT_BYTES = 2 * kPvCols * PITCH, RED_BYTES = 4 * 64 * 33 * 4;
    __shared__ __attribute__((aligned(16))) unsigned char sBuf[VT_BYTES > RED_BYTES ? VT_BYTES : RED_BYTES];
    unsigned char (*sVt)[kPvCols * PITCH] = reinterpret_cast<unsigned char (*)[kPvCols * PITCH]>(sBuf);
    float (*red)[64][33] = reinterpret_cast<float (*)[64][33]>(sBuf);  // cross-wave sums, after the loop
    __shared__ int sRow[kPvMaxTok];          // cache row of every token of the range
    __shared__ float2 sMZ[kPvMaxHeads];      // per head: softmax maximum, 1 / normaliser

    // Work items are ordered (sequence, token range, column block) with the column block fastest.
    // Workgroup ids are dealt round-robin to the XCDs; the map below gives each XCD a contiguous run of
    // the list, so the column blocks of one token range (same indices, logits and statistics, adjacent
    // 128-byte pieces of the same cache rows) meet in one L2.
    const int n_cb = r / kPvCols;
    const int total = n_cb * n_tr * B;  // = gridDim.x
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds, qn = total / kXcds, rem = total % kXcds;
    const int item = (xcd < rem ? xcd * (qn + 1) : rem * (qn + 1) + (xcd - rem) * qn) + slot;
    const int cb = item % n_cb, tr = (item / n_cb) % n_tr, b = item / (n_cb * n_tr);
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    // the count and this thread's first index are requested together (both through the vector memory path)
    const int n_v = ld_uniform_i32(n_sel + b);
    const int v_first = idx[(size_t)b * k_tot + min(tr * tok_per_wg + tid, k_tot - 1)];
    const int n = wave_uniform(n_v);
    const int j_begin = min(n, tr * tok_per_wg), j_end = min(n, j_begin + tok_per_wg);
    const int ntok = j_end - j_begin;
    const int col0 = cb * kPvCols;
    const int n_mb = (H + 31) >> 5;
    const float* lg = logits + (size_t)b * H * lk;
    const int32_t* ib = idx + (size_t)b * k_tot;

    // (the index loads only depend on the nominal range, so they are in flight together with n)
    for (int t = tid; t < tok_per_wg; t += kPvThreads) {
        const int j = tr * tok_per_wg + t;
        const int v = t == tid ? v_first : (j < k_tot ? ib[j] : 0);
        const int pos = min(max(v, 0), S_max - 1);
        if (t < ntok) sRow[t] = ring > 0 ? pos % ring : pos;  // ring cache: token t lies in row t mod ring
    }
    // softmax maximum and normaliser of every head: four lanes share a head's tiles and merge
    // them in a fixed order
    {
        const int h = tid >> 2, sub = tid & 3;
        float2 st = make_float2(-INFINITY, 0.f);
        if (h < H) {
            const float2* sp = stats + ((size_t)b * H + h) * n_parts;
            for (int t0 = sub; t0 < n_parts; t0 += 32) {  // eight loads in flight per round
                float2 e[8];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    e[u] = t0 + 4 * u < n_parts ? sp[t0 + 4 * u] : make_float2(-INFINITY, 0.f);
#pragma unroll
                for (int u = 0; u < 8; ++u) st = stat_merge(st, e[u]);
            }
        }
        st = stat_merge(st, make_float2(__shfl_xor(st.x, 1, kWave), __shfl_xor(st.y, 1, kWave)));
        st = stat_merge(st, make_float2(__shfl_xor(st.x, 2, kWave), __shfl_xor(st.y, 2, kWave)));
        if (sub == 0 && h < kPvMaxHeads) sMZ[h] = make_float2(st.x > -INFINITY ? st.x : 0.f, st.y > 0.f ? 1.f / st.y : 0.f);
    }
    __syncthreads();
    float2 mz[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) mz[mb] = sMZ[mb * 32 + l32];

    f32x16 acc[2][2];  // [head block][column block]
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    const unsigned char* vbytes = reinterpret_cast<const unsigned char*>(Vc + (size_t)b * (ring > 0 ? ring : S_max) * r + col0);
    const size_t row_bytes = (size_t)r * ES;
    constexpr int NKQ = (NKG + kPvWaves - 1) / kPvWaves;  // MFMA groups per wave per step (1)
    // what a step needs from global memory: the gathered row pieces and this lane's logits; two
    // such sets alternate, so the loads run two steps ahead
    struct Stage { u32x4 R[NPC]; f32x4 X[NKQ][2][VEC / 4]; };
    auto g_load = [&](Stage& S, int step) {
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int q = tid + kPvThreads * i, jj = q / PPR, pc = q % PPR;
            // tokens past the range re-read its last row; their weights are zero
            const int row = sRow[min(step * TJ + jj, ntok - 1)];
            S.R[i] = ld16(vbytes + (size_t)row * row_bytes + pc * 16);
        }
#pragma unroll
        for (int kq = 0; kq < NKQ; ++kq) {
            const int ks = kq * kPvWaves + wave;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                const int h = mb * 32 + l32;
                const bool ok = ks < NKG && mb < n_mb && h < H;
                const size_t off = (size_t)h * lk + j_begin + step * TJ + ks * KG + hi * VEC;
#pragma unroll
                for (int v = 0; v < VEC / 4; ++v)
                    S.X[kq][mb][v] = ok ? *reinterpret_cast<const f32x4*>(lg + off + 4 * v)
                                      : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            }
        }
    };
    auto l_store = [&](const Stage& S, int buf) {
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int q = tid + kPvThreads * i, jj = q / PPR, pc = q % PPR;
            unsigned char* dst = sVt[buf] + (size_t)(pc * VEC) * PITCH + jj * ES;
            const uint32_t w[4] = {S.R[i].x, S.R[i].y, S.R[i].z, S.R[i].w};
            if constexpr (kSplit) {
                // lanes l and l^8 hold the same columns of tokens jj and jj^1: they swap halves, so that each
                // writes four whole 32-bit words {token even, token odd} instead of eight 16-bit ones
                const bool odd = (jj & 1) != 0;
                unsigned char* dst2 = dst - (odd ? ES : 0);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w[k], 0x128, 0xf, 0xf, false);  // row_ror:8
                    const uint32_t word = odd ? ((other >> 16) | (w[k] & 0xffff0000u)) : ((w[k] & 0xffffu) | (other << 16));
                    *reinterpret_cast<uint32_t*>(dst2 + (size_t)(2 * k + (odd ? 1 : 0)) * PITCH) = word;
                }
            } else {
#pragma unroll
                for (int e = 0; e < VEC; ++e) *reinterpret_cast<uint32_t*>(dst + (size_t)e * PITCH) = w[e];
            }
        }
    };

    const int n_steps = (ntok + TJ - 1) / TJ;
    auto do_step = [&](Stage& S, int step) {
        const int buf = step & 1;
        l_store(S, buf);
        // softmax weights of this step from the logits fetched a step ahead
        const int j0 = j_begin + step * TJ;
        u32x4 ah[NKQ][2], al[NKQ][2];
#pragma unroll
        for (int kq = 0; kq < NKQ; ++kq) {
            const int tok = (kq * kPvWaves + wave) * KG + hi * VEC;  // first of this lane's VEC tokens within the step
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                if (mb >= n_mb) {  // uniform: no heads in this block
                    ah[kq][mb] = al[kq][mb] = u32x4{0, 0, 0, 0};
                    continue;
                }
                float pj[VEC];
#pragma unroll
                for (int v = 0; v < VEC; v += 4) {
                    const f32x4 x = S.X[kq][mb][v / 4];
                    // slots past the range carry no weight (their logits may be unwritten)
                    const int jt = j0 + tok + v;
                    pj[v] = jt < j_end ? __expf(x.x - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 1] = jt + 1 < j_end ? __expf(x.y - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 2] = jt + 2 < j_end ? __expf(x.z - mz[mb].x) * mz[mb].y : 0.f;
                    pj[v + 3] = jt + 3 < j_end ? __expf(x.w - mz[mb].x) * mz[mb].y : 0.f;
                }
                if constexpr (kSplit) {
                    uint32_t ph[VEC], pl[VEC];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        const bf16_t hb = f32_to_bf16(pj[v]);
                        ph[v] = hb;
                        pl[v] = f32_to_bf16(pj[v] - bf16_to_f32(hb));
                    }
                    ah[kq][mb] = u32x4{ph[0] | (ph[1] << 16), ph[2] | (ph[3] << 16), ph[4] | (ph[5] << 16),
                                       ph[6] | (ph[7] << 16)};
                    al[kq][mb] = u32x4{pl[0] | (pl[1] << 16), pl[2] | (pl[3] << 16), pl[4] | (pl[5] << 16),
                                       pl[6] | (pl[7] << 16)};
                } else {
                    ah[kq][mb] = u32x4{__float_as_uint(pj[0]), __float_as_uint(pj[1]), __float_as_uint(pj[2]),
                                       __float_as_uint(pj[3])};
                }
            }
        }
        if (step + 2 < n_steps) g_load(S, step + 2);
        __syncthreads();  // tile `buf` complete; the other tile was last read a barrier ago
#pragma unroll
        for (int kq = 0; kq < NKQ; ++kq) {
            const int ks = kq * kPvWaves + wave;
            if (ks < NKG) {  // uniform
                const int tok = ks * KG + hi * VEC;
#pragma unroll
                for (int nb = 0; nb < 2; ++nb) {
                    const unsigned char* src = sVt[buf] + (size_t)(nb * 32 + l32) * PITCH + tok * ES;
                    const uint2 lo8 = *reinterpret_cast<const uint2*>(src);
                    const uint2 hi8 = *reinterpret_cast<const uint2*>(src + 8);
                    const u32x4 vf = u32x4{lo8.x, lo8.y, hi8.x, hi8.y};
#pragma unroll
                    for (int mb = 0; mb < 2; ++mb) {
                        if (mb < n_mb) {
                            mma_op<T>::run(ah[kq][mb], vf, acc[mb][nb]);
                            if constexpr (kSplit) mma_op<T>::run(al[kq][mb], vf, acc[mb][nb]);
                        }
                    }
                }
            }
        }
    };
    Stage S0, S1;
    if (n_steps > 0) g_load(S0, 0);
    if (n_steps > 1) g_load(S1, 1);
    for (int step = 0; step < n_steps; step += 2) {
        do_step(S0, step);
        if (step + 1 < n_steps) do_step(S1, step + 1);
    }

    // The waves' sums, one column block at a time: of eight waves, 4..7 first hand theirs to waves 0..3, which
    // add them (wave w + wave w+4); the four then share out the final sum in wave order, wave w finishing heads
    // 8w..8w+7 of each head block.  acc[mb][nb][4a+c] is head mb*32+8a+4hi+c, column nb*32+l32
    float* out_t = Tpart + (((size_t)tr * B + b) * H) * r;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        __syncthreads();
        if constexpr (NW == 8) {
            if (wave >= 4) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) red[wave - 4][lane][mb * 16 + v] = acc[mb][nb][v];
            }
            __syncthreads();
            if (wave < 4) {
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mb][nb][v] += red[wave][lane][mb * 16 + v];
            }
            __syncthreads();
        }
        if (wave < 4) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int v = 0; v < 16; ++v) red[wave][lane][mb * 16 + v] = acc[mb][nb][v];
        }
        __syncthreads();
        if (wave < 4) {
            const int col = col0 + nb * 32 + l32;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int v = wave * 4 + c;  // a = wave
                    const int h = mb * 32 + wave * 8 + hi * 4 + c;
                    if (h < H)
                        out_t[(size_t)h * r + col] = ((red[0][lane][mb * 16 + v] + red[1][lane][mb * 16 + v]) +
                                                      red[2][lane][mb * 16 + v]) + red[3][lane][mb * 16 + v];
                }
        }
    }
}

// ---------------------------------------------------------------------------------
// output projection: y[(b,h), c] = sum_i T[(b,h), i] U_v[g*128 + c, i]
//
// One workgroup per (KV head, 16 output channels, tile of 16 rows): 8 x H_kv x ceil(B*G/16)
// workgroups, so that the pass over U_v is spread over the whole chip.  16x16 MFMA tiles: rows are the (sequence,
// head of the group) pairs, columns the channels; the latent axis is split over the four
// waves, every wave issuing all of its loads as one batch.
// ---------------------------------------------------------------------------------
// BATCH latent steps of loads and RPR token ranges are in flight per round and wave: (8,2) covers any rank, (5,3)
// and (4,4) merge more ranges per memory round trip when a wave has at most 5 / 4 steps.
template <typename T, int BATCH, int RPR>
__global__ __launch_bounds__(256) void attend_out_kernel(const T* __restrict__ Uv, const float* __restrict__ Tpart,
                                                         T* __restrict__ out,
                                                         int B, int r, int H, int H_kv, int n_tr,
                                                         const T* __restrict__ Uv2, const float* __restrict__ Tpart2,
                                                         int r2, int n_tr2)
{
    constexpr int VEC = elem<T>::vec;
    constexpr int KS = 4 * VEC;  // latent coordinates per MFMA step
    constexpr bool kSplit = sizeof(T) == 2;
    __shared__ __attribute__((aligned(16))) float red[3][64][5];

    // KV head fastest: workgroup ids are dealt round-robin to the XCDs, so the eight channel blocks of
    // a head (which read the same value sums) share one XCD's L2 whenever H_kv is a multiple of 8
    const int g = blockIdx.x, cb = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, kg = lane >> 4;
    const int G = H / H_kv;
    const int n_rows = B * G;  // (sequence, head of this group) pairs

    {
        const int row0 = blockIdx.z * 16;  // this workgroup's tile of 16 rows
        const int row = row0 + l16;
        const bool row_ok = row < n_rows;
        const int bb = row_ok ? row / G : 0, h = row_ok ? g * G + row % G : 0;
        f32x4v acc = {0.f, 0.f, 0.f, 0.f};
        // A second pair (value sums of another latent cache, its projector) is added into the same output when
        // r2 > 0: the recent window's higher-rank cache beside the low-rank one.
        for (int pass = 0; pass < (r2 > 0 ? 2 : 1); ++pass) {
        const T* const Uv_p = pass ? Uv2 : Uv;
        const float* const Tpart_p = pass ? Tpart2 : Tpart;
        const int r_p = pass ? r2 : r, n_tr_p = pass ? n_tr2 : n_tr;
        const int nks = r_p / KS;
        const T* urow = Uv_p + ((size_t)g * kHeadDim + cb * 16 + l16) * r_p + kg * VEC;
        const size_t tstride = (size_t)B * H * r_p;
        const size_t trow = ((size_t)bb * H + h) * r_p + kg * VEC;
        for (int ks0 = wave; ks0 < nks; ks0 += 4 * BATCH) {  // this wave: ks0, ks0+4, ...
            u32x4 bf[BATCH], ah[BATCH], al[BATCH];
            float tm[BATCH][VEC];  // T of this lane's row: the token ranges' partial sums, added in range order
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                const int ks = ks0 + 4 * u;
                bf[u] = ks < nks ? ld16(urow + ks * KS) : u32x4{0, 0, 0, 0};
#pragma unroll
                for (int v = 0; v < VEC; ++v) tm[u][v] = 0.f;
            }
            // RPR ranges per round, the loads of all BATCH steps in flight together
            for (int t0 = 0; t0 < n_tr_p; t0 += RPR) {
                f32x4 x[BATCH][RPR][VEC / 4];
#pragma unroll
                for (int u = 0; u < BATCH; ++u) {
                    const int ks = ks0 + 4 * u;
#pragma unroll
                    for (int w = 0; w < RPR; ++w)
#pragma unroll
                        for (int v = 0; v < VEC / 4; ++v)
                            x[u][w][v] = (ks < nks && row_ok && t0 + w < n_tr_p)
                                             ? *reinterpret_cast<const f32x4*>(Tpart_p + (size_t)(t0 + w) * tstride + trow +
                                                                               ks * KS + 4 * v)
                                             : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int u = 0; u < BATCH; ++u)
#pragma unroll
                    for (int w = 0; w < RPR; ++w)
#pragma unroll
                        for (int v = 0; v < VEC / 4; ++v) {
                            tm[u][4 * v] += x[u][w][v].x; tm[u][4 * v + 1] += x[u][w][v].y;
                            tm[u][4 * v + 2] += x[u][w][v].z; tm[u][4 * v + 3] += x[u][w][v].w;
                        }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                if constexpr (kSplit) {
                    uint32_t hw[8], lw[8];
#pragma unroll
                    for (int v = 0; v < 8; ++v) {
                        bf16_t ph = f32_to_bf16(tm[u][v]);
                        hw[v] = ph;
                        lw[v] = f32_to_bf16(tm[u][v] - bf16_to_f32(ph));
                    }
                    ah[u] = u32x4{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16), hw[4] | (hw[5] << 16),
                                  hw[6] | (hw[7] << 16)};
                    al[u] = u32x4{lw[0] | (lw[1] << 16), lw[2] | (lw[3] << 16), lw[4] | (lw[5] << 16),
                                  lw[6] | (lw[7] << 16)};
                } else {
                    ah[u] = u32x4{__float_as_uint(tm[u][0]), __float_as_uint(tm[u][1]), __float_as_uint(tm[u][2]),
                                  __float_as_uint(tm[u][3])};
                }
            }
#pragma unroll
            for (int u = 0; u < BATCH; ++u) {
                mma16_op<T>::run(ah[u], bf[u], acc);
                if constexpr (kSplit) mma16_op<T>::run(al[u], bf[u], acc);
            }
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
