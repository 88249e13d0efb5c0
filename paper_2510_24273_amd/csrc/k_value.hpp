// The value path of the sparse attention (Eq. 5; Algorithm 1, output step), evaluated as
// y_h = ((p_h V~_C) U_v[g(h) block]^T) : the same sum as p_h (V~_C U_v^T) in another order,
// so the selected values are never reconstructed.
//
//   attend_pv   per (sequence, token range, 64 latent columns):
//               T[h,:] = sum_j p_hj V~[C_j,:]  on the matrix cores, tokens being the
//               contraction axis (dealt in groups to the workgroup's four or eight waves); the gathered
//               rows are transposed in registers on the way.  The softmax weights are formed
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

constexpr int kPvTJ = 64;          // token ranges are whole multiples of this
constexpr int kPvCols = 64;        // latent columns per workgroup
constexpr int kPvMaxHeads = 64;    // H_q limit of these kernels
constexpr int kMaxRanges = 8;      // token ranges per sequence (the output projection adds them up)
constexpr int kPvMaxTok = 4096;    // tokens per workgroup, at most (their cache rows sit in LDS)
constexpr int kPvDepth = 4;        // token groups whose loads a wave keeps in flight

// NW waves (4 or 8), MB blocks of 32 heads.  The range's tokens are dealt to the waves in groups of one MFMA
// contraction step (16 tokens for bf16, 8 for fp32: half of them per half-wave); a wave works through its groups on
// its own, no barrier inside the loop, and keeps the loads of kPvDepth groups in flight.
//
// The MFMA's second operand wants, per lane, consecutive TOKENS of one column, while memory holds consecutive
// columns of one token.  bf16: lane l32 fetches the 32-bit word (columns 2 l32, 2 l32 + 1) of each of its eight
// tokens, a half-wave thus a whole 128-byte piece per token, and two byte permutes per token pair turn the eight words
// into the operand of the even column and the operand of the odd column: the transposition never leaves the
// registers.  fp32 (two tokens per MFMA, one per half-wave): the loaded words are the operands as they are.
template <typename T, int NW, int MB>
__global__ __launch_bounds__(NW * 64) void attend_pv_kernel(
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_sel, const float2* __restrict__ stats,
    int B, int r, int n_tr, int n_parts, int tok_per_wg, int k_tot, int H, int lk,
    const T* __restrict__ Vc, const float* __restrict__ logits, float* __restrict__ Tpart, int S_max, int ring)
{
    static_assert((NW == 4 || NW == 8) && (MB == 1 || MB == 2), "four or eight waves, one or two head blocks");
    constexpr int kPvThreads = NW * 64;
    constexpr int ES = (int)sizeof(T);
    constexpr int VEC = elem<T>::vec;        // tokens per lane per group = elements per 16 bytes
    constexpr int KG = 2 * VEC;              // tokens per group (both half-waves)
    constexpr bool kSplit = ES == 2;
    constexpr int ND = 8;                    // gathered words per lane and group: 8 tokens (bf16) | 4 tokens x 2 column blocks (fp32)

    __shared__ __attribute__((aligned(16))) int sRow[kPvMaxTok];  // cache row of every token of the nominal range
    __shared__ float2 sMZ[kPvMaxHeads];      // per head: softmax maximum, 1 / normaliser
    __shared__ float red[NW][64][17];        // cross-wave sums, after the loop

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
    const int col0 = cb * kPvCols;
    const float* lg = logits + (size_t)b * H * lk;
    const int32_t* ib = idx + (size_t)b * k_tot;

    // everything that depends on nothing is requested at once: the count, the range's indices, the tile statistics
    const int n_v = ld_uniform_i32(n_sel + b);
    for (int t = tid; t < tok_per_wg; t += kPvThreads) {
        const int j = tr * tok_per_wg + t;
        const int v = ib[min(j, k_tot - 1)];
        const int pos = min(max(v, 0), S_max - 1);
        sRow[t] = ring > 0 ? pos % ring : pos;  // ring cache: token t lies in row t mod ring
    }
    const int sh = tid >> 2, sub = tid & 3;     // four lanes share a head's tiles
    float2 st8[8];
    {
        const float2* sp = stats + ((size_t)b * H + min(sh, H - 1)) * n_parts;
#pragma unroll
        for (int u = 0; u < 8; ++u) st8[u] = sub + 4 * u < n_parts ? sp[sub + 4 * u] : make_float2(-INFINITY, 0.f);
    }
    __syncthreads();  // rows of the range in LDS

    const unsigned char* vbytes =
        reinterpret_cast<const unsigned char*>(Vc + (size_t)b * (ring > 0 ? ring : S_max) * r + col0) + l32 * 4;
    const size_t row_bytes = (size_t)r * ES;
    const int g_last = tok_per_wg / KG - 1;  // (the range is a whole number of groups)
    // what a group needs from global memory: the gathered words and this lane's logits
    struct Stage { uint32_t R[ND]; f32x4 X[MB][VEC / 4]; };
    auto g_load = [&](Stage& S, int g) {
        const int t0 = min(g, g_last) * KG + hi * VEC;  // first of this lane's VEC tokens within the range
        int rows[VEC];
#pragma unroll
        for (int v = 0; v < VEC; v += 4) {
            const int4 r4 = *reinterpret_cast<const int4*>(&sRow[t0 + v]);
            rows[v] = r4.x; rows[v + 1] = r4.y; rows[v + 2] = r4.z; rows[v + 3] = r4.w;
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const unsigned char* src = vbytes + (size_t)rows[v] * row_bytes;
            S.R[v] = *reinterpret_cast<const uint32_t*>(src);
            if constexpr (!kSplit) S.R[VEC + v] = *reinterpret_cast<const uint32_t*>(src + 32 * 4);
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            const int h = min(mb * 32 + l32, H - 1);  // (rows past the last head: any head's logits, never stored)
            const size_t off = (size_t)h * lk + tr * tok_per_wg + t0;
#pragma unroll
            for (int v = 0; v < VEC / 4; ++v) S.X[mb][v] = *reinterpret_cast<const f32x4*>(lg + off + 4 * v);
        }
    };
    Stage S[kPvDepth];
#pragma unroll
    for (int u = 0; u < kPvDepth; ++u)
        if (wave + NW * u <= g_last) g_load(S[u], wave + NW * u);  // (the count is not known yet: nominal groups)

    // softmax maximum and normaliser of every head, merged in a fixed order (under the loads above)
    {
        float2 st = make_float2(-INFINITY, 0.f);
        if (sh < H) {
#pragma unroll
            for (int u = 0; u < 8; ++u) st = stat_merge(st, st8[u]);
            const float2* sp = stats + ((size_t)b * H + sh) * n_parts;
            for (int t0 = sub + 32; t0 < n_parts; t0 += 32) {  // (more than 32 tiles: further rounds of eight loads)
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
        if (sub == 0 && sh < kPvMaxHeads) sMZ[sh] = make_float2(st.x > -INFINITY ? st.x : 0.f, st.y > 0.f ? 1.f / st.y : 0.f);
    }
    __syncthreads();
    float2 mz[MB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) mz[mb] = sMZ[mb * 32 + l32];

    const int n = wave_uniform(n_v);
    const int j_begin = min(n, tr * tok_per_wg), j_end = min(n, j_begin + tok_per_wg);
    const int ntok = j_end - j_begin;        // (0 for a range past the selection: it still writes its zero sums)
    const int n_groups = (ntok + KG - 1) / KG;

    f32x16 acc[MB][2];  // [head block][column block]
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    auto do_group = [&](const Stage& S, int g) {
        const int t0 = g * KG + hi * VEC;
        // words of slots past the range count as zero (their rows may never have been written)
        uint32_t w[ND];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const bool ok = t0 + v < ntok;
            w[v] = ok ? S.R[v] : 0u;
            if constexpr (!kSplit) w[VEC + v] = ok ? S.R[VEC + v] : 0u;
        }
        u32x4 vf[2];
        if constexpr (kSplit) {
            vf[0] = u32x4{__builtin_amdgcn_perm(w[1], w[0], 0x05040100u), __builtin_amdgcn_perm(w[3], w[2], 0x05040100u),
                          __builtin_amdgcn_perm(w[5], w[4], 0x05040100u), __builtin_amdgcn_perm(w[7], w[6], 0x05040100u)};
            vf[1] = u32x4{__builtin_amdgcn_perm(w[1], w[0], 0x07060302u), __builtin_amdgcn_perm(w[3], w[2], 0x07060302u),
                          __builtin_amdgcn_perm(w[5], w[4], 0x07060302u), __builtin_amdgcn_perm(w[7], w[6], 0x07060302u)};
        } else {
            vf[0] = u32x4{w[0], w[1], w[2], w[3]};
            vf[1] = u32x4{w[4], w[5], w[6], w[7]};
        }
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
            float pj[VEC];
#pragma unroll
            for (int v = 0; v < VEC; v += 4) {
                const f32x4 x = S.X[mb][v / 4];
                // slots past the range carry no weight (their logits may be unwritten)
                const int jt = t0 + v;
                pj[v] = jt < ntok ? __expf(x.x - mz[mb].x) * mz[mb].y : 0.f;
                pj[v + 1] = jt + 1 < ntok ? __expf(x.y - mz[mb].x) * mz[mb].y : 0.f;
                pj[v + 2] = jt + 2 < ntok ? __expf(x.z - mz[mb].x) * mz[mb].y : 0.f;
                pj[v + 3] = jt + 3 < ntok ? __expf(x.w - mz[mb].x) * mz[mb].y : 0.f;
            }
            u32x4 ah, al;
            if constexpr (kSplit) {
                uint32_t ph[VEC], pl[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const bf16_t hb = f32_to_bf16(pj[v]);
                    ph[v] = hb;
                    pl[v] = f32_to_bf16(pj[v] - bf16_to_f32(hb));
                }
                ah = u32x4{ph[0] | (ph[1] << 16), ph[2] | (ph[3] << 16), ph[4] | (ph[5] << 16), ph[6] | (ph[7] << 16)};
                al = u32x4{pl[0] | (pl[1] << 16), pl[2] | (pl[3] << 16), pl[4] | (pl[5] << 16), pl[6] | (pl[7] << 16)};
            } else {
                ah = u32x4{__float_as_uint(pj[0]), __float_as_uint(pj[1]), __float_as_uint(pj[2]), __float_as_uint(pj[3])};
            }
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                mma_op<T>::run(ah, vf[nb], acc[mb][nb]);
                if constexpr (kSplit) mma_op<T>::run(al, vf[nb], acc[mb][nb]);
            }
        }
    };
    for (int i0 = 0; wave + NW * i0 < n_groups; i0 += kPvDepth) {
#pragma unroll
        for (int u = 0; u < kPvDepth; ++u) {
            const int g = wave + NW * (i0 + u);  // wave-uniform
            if (g < n_groups) do_group(S[u], g);
            if (g + NW * kPvDepth < n_groups) g_load(S[u], g + NW * kPvDepth);
        }
    }

    // The waves' sums, one (head block, column block) at a time, added in wave order; wave w finishes 16 / NW of a
    // lane's 16 values.  acc[mb][nb][4a+c] is head mb*32 + 8a + 4hi + c; its column is 2 l32 + nb (bf16: even / odd
    // operand) or nb*32 + l32 (fp32).
    float* out_t = Tpart + (((size_t)tr * B + b) * H) * r;
    constexpr int PER = 16 / NW;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            if (mb + nb > 0) __syncthreads();
#pragma unroll
            for (int v = 0; v < 16; ++v) red[wave][lane][v] = acc[mb][nb][v];
            __syncthreads();
            const int col = col0 + (kSplit ? 2 * l32 + nb : nb * 32 + l32);
#pragma unroll
            for (int c = 0; c < PER; ++c) {
                const int v = wave * PER + c;
                const int h = mb * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
                float sum = red[0][lane][v];
#pragma unroll
                for (int w = 1; w < NW; ++w) sum += red[w][lane][v];
                if (h < H) out_t[(size_t)h * r + col] = sum;
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
