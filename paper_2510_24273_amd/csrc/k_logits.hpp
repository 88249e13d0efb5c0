// Selective key reconstruction with fused RoPE and query dot product
// (Algorithm 1, reconstruction / RoPE / logit steps; Sec. 4.4):
//   logits[b, h, j] = RoPE(q[b,h], q_pos[b]) . RoPE(U_k[g(h) block] K~[b, C_j], C_j) / sqrt(d)
//
// A gathered-row GEMM on the matrix cores: for one sequence, HEADS KV heads and a tile of
// selected tokens, D[dim, token] = sum_i U_k[dim, i] K~[C_token, i].  Both operands are
// staged through LDS in 64-byte steps of the latent axis: the packed U_k panel (shared by
// the waves of a head) and the gathered latent rows (shared by the heads), each loaded
// with 16 contiguous bytes per lane and written to a swizzled layout that the MFMA
// fragment reads hit without bank conflicts.  Three LDS stages and two fragment register sets
// form a software pipeline in which every wave overlaps its own LDS traffic with its MFMAs.
//
// The reconstructed keys stay in the accumulators.  The epilogue streams the tokens' cos/sin
// rows through the same LDS buffers, 16 RoPE pairs per pass, rotates the accumulators and
// dots them with the rotated query, so only logits are written, plus each (head, token
// tile)'s softmax maximum and normaliser for the value kernel.  The query itself is rotated
// (fp64-accurate angles) and scaled by 1/sqrt(d) in the prologue, while the first tile loads
// are in flight.
//
// Wave tile: 128 head dims (4 MFMA row blocks, in RoPE pair order) x 32*NB tokens.
// Workgroup: HEADS x NTG waves, i.e. HEADS heads x (NTG*32*NB) tokens.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"

namespace sals {

constexpr int kLgChunk = 128;  // bytes per row of a [rows][128 B] swizzled LDS tile
constexpr int kLgStep = 64;    // bytes of the latent axis per pipeline step (= one packed U_k block)

// LDS tiles are read and written 16 bytes per lane; such an access is conflict-free when each
// group of 16 consecutive lanes covers all 16 bank groups (address / 16 mod 16).  A fragment read
// takes one piece index from 16 consecutive rows, a staging write takes consecutive pieces, so
// the piece index is XOR-ed with row bits.
// byte offset of 16-byte piece `pc` of row `row` inside a [rows][128 B] tile
__device__ __forceinline__ int swz(int row, int pc) { return row * kLgChunk + ((pc ^ ((row >> 1) & 7)) << 4); }
// the same for a [rows][64 B] tile
__device__ __forceinline__ int swz64(int row, int pc) { return row * kLgStep + ((pc ^ ((row >> 2) & 3)) << 4); }

template <int HEADS, int NTG, int NB> struct logits_cfg {
    static constexpr int NT = 64 * HEADS * NTG;            // threads
    static constexpr int TOK = NTG * NB * 32;              // tokens per workgroup
    static constexpr int A_BYTES = HEADS * 128 * kLgStep;  // U_k panel per step
    static constexpr int B_BYTES = TOK * kLgStep;          // gathered rows per step
    static constexpr int STAGE = A_BYTES + B_BYTES;
    static constexpr int NA = A_BYTES / 16 / NT;           // 16-byte pieces per thread per step
    static constexpr int NBP = B_BYTES / 16 / NT;
    static constexpr int CS_BYTES = TOK * kLgChunk;        // cos/sin of 16 pairs for every token
    static constexpr int NCS = CS_BYTES / 16 / NT;
    static constexpr size_t LDS = 3 * (size_t)STAGE > 2 * (size_t)CS_BYTES ? 3 * (size_t)STAGE : 2 * (size_t)CS_BYTES;
};

// GB: query heads of a KV head handled as one block of straight-line code (1, or 4 when the group size is a multiple
// of 4): the LDS reads and the reductions of a block's heads are in flight together instead of one head after the other.
// GFIX: the group size when it is known at compile time (1 and 4, the common ones; 0: read from the arguments), which
// takes the per-block branches out of the epilogue.
// MULTI: a tile of NTG x 64 tokens is made of the (at most 64 token) selections of NTG consecutive SEQUENCES, one per
// token group, instead of 256 tokens of one sequence: short selections such as a recent window then share one pass
// over the head's projector among NTG sequences.  Each token group has its own query, count, index list and cache;
// the latent axis may be cut into `ksplit` slices (the logit is additive over latent coordinates), whose partial
// logits go to `plogits` for logits_finish_kernel.
template <typename T, int HEADS, int NTG, int NB, int GB, int GFIX, bool MULTI = false>
__global__ __launch_bounds__(64 * HEADS * NTG, HEADS * NTG >= 8 ? 2 : 1) void attend_logits_kernel(
    const T* __restrict__ Kc, const T* __restrict__ UkP, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ n_sel, const T* __restrict__ q, const int32_t* __restrict__ q_pos,
    const float2* __restrict__ rope, InvFreq inv,
    float* __restrict__ logits, float2* __restrict__ stats, int B, int S_max, int r, int H, int H_kv,
    int k_tot, int lk, int n_parts, int heads_fastest, int style, float scale, int ring, int stats_stride,
    float* __restrict__ plogits, int ksplit)
{
    typedef logits_cfg<HEADS, NTG, NB> C;
    static_assert(!MULTI || (HEADS == 1 && NB * 32 == 64), "a token group is one sequence's 64 slots");
    constexpr int SQ = MULTI ? NTG : 1;   // sequences per tile
    constexpr int NT = C::NT, NA = C::NA, NBP = C::NBP, NCS = C::NCS;
    constexpr int ES = (int)sizeof(T);
    static_assert(C::A_BYTES % (16 * NT) == 0 && C::B_BYTES % (16 * NT) == 0 && C::CS_BYTES % (16 * NT) == 0,
                  "tile / thread mismatch");
    static_assert(kMaxGroup % GB == 0 && (GFIX == 0 || (GFIX % GB == 0 && GFIX <= kMaxGroup)), "head blocks tile the group");
    constexpr int kGroupEnd = GFIX > 0 ? GFIX : kMaxGroup;

    // Workgroup id -> (sequence, token tile, head block).  Consecutive ids are dispatched to
    // different XCDs, each with its own L2, so every XCD gets one contiguous range of the work
    // list; the list is ordered so that a range shares the larger operand: heads fastest keeps
    // the gathered rows of a few token tiles in that L2 (U_k is re-read per XCD), tiles fastest
    // keeps the U_k panels of a few heads there (the rows are re-read per XCD).
    int b, g0, part, kz = 0;   // MULTI: b is the first sequence of the tile
    if constexpr (MULTI) {
        // list order (head, sequence group, latent slice): an XCD's range keeps a few heads' projector slices
        const int nb4 = (B + NTG - 1) / NTG, N = nb4 * H_kv * ksplit;
        const int id = blockIdx.x, xcd = id % kXcds, slot = id / kXcds;
        const int qn = N / kXcds, rem = N % kXcds;
        const int w = (xcd < rem ? xcd * (qn + 1) : rem * (qn + 1) + (xcd - rem) * qn) + slot;
        g0 = w / (nb4 * ksplit);
        const int rest = w - g0 * (nb4 * ksplit);
        b = (rest / ksplit) * NTG; kz = rest % ksplit; part = 0;
    } else {
        const int n_y = H_kv / HEADS, N = n_parts * n_y * B;
        const int id = blockIdx.x, xcd = id % kXcds, slot = id / kXcds;
        const int qn = N / kXcds, rem = N % kXcds;
        const int w = (xcd < rem ? xcd * (qn + 1) : rem * (qn + 1) + (xcd - rem) * qn) + slot;
        if (heads_fastest) {
            const int bt = w / n_y;
            g0 = (w - bt * n_y) * HEADS; b = bt / n_parts; part = bt - b * n_parts;
        } else {
            const int hb = w / (n_parts * B), bt = w - hb * (n_parts * B);
            g0 = hb * HEADS; b = bt / n_parts; part = bt - b * n_parts;
        }
    }
    const int tok0 = part * C::TOK;
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int hh = wave / NTG, tg = wave % NTG;   // head of the tile, token group
    // sequence of tile token t (MULTI: token group t / 64 is sequence b + t / 64; groups past the batch repeat the last
    // sequence and get no weight)
    auto seq_of = [&](int t) { return MULTI ? min(b + (t >> 6), B - 1) : b; };
    // count and query position: of this wave's sequence (MULTI: wave = token group; the position is needed per thread
    // for the thread's share of the cos/sin rows, see rotate_query)
    const int n_v = ld_uniform_i32(n_sel + (MULTI ? seq_of(tg * 64) : b));
    const int qpos_v = MULTI ? q_pos[seq_of(tid & ~63)] : ld_uniform_i32(q_pos + b);  // in flight with the loads below
    const int G = GFIX > 0 ? GFIX : H / H_kv;
    const int g = g0 + hh;

    // Everything the prologue needs from memory is requested before anything is waited for, from clamped
    // addresses so that no load sits in a branch: the tile's token rows (slots at or past the selection count
    // read whatever the index array holds there, clamped to a valid row; they get no weight), the raw query
    // pairs of the tile's heads and the query position.
    const int rows_per_seq = ring > 0 ? ring : S_max;
    // cache row (= RoPE position) of tile token t: slot t of the one sequence, or slot t % 64 of sequence b + t / 64
    auto row_of = [&](int t) {
        const int32_t* ib = idx + (size_t)seq_of(t) * k_tot;
        return min(max(ib[min(MULTI ? (t & 63) : tok0 + t, k_tot - 1)], 0), S_max - 1);
    };
    int b_row[NBP];  // gathered rows: piece q = tid + i*NT -> token q/4 of the tile, column q%4
#pragma unroll
    for (int i = 0; i < NBP; ++i) {
        const int t = (tid + i * NT) >> 2;
        b_row[i] = row_of(t);
        if (ring > 0) b_row[i] %= ring;  // ring cache: token t lies in row t mod ring
        if (MULTI) b_row[i] += (seq_of(t) - b) * rows_per_seq;  // (rows counted from the tile's first sequence)
    }
    constexpr int NSP = (C::TOK + NT - 1) / NT;
    int pos_reg[NSP];
#pragma unroll
    for (int u = 0; u < NSP; ++u) pos_reg[u] = row_of(min(tid + u * NT, C::TOK - 1));
    constexpr int QP = (SQ * HEADS * (GFIX > 0 ? GFIX : kMaxGroup) * kPairs + NT - 1) / NT;
    float qa[QP], qb[QP];
#pragma unroll
    for (int u = 0; u < QP; ++u) {
        // query pair t: (sequence of the tile, head of the tile's heads, pair)
        const int t = min(tid + u * NT, SQ * HEADS * G * kPairs - 1), p = t & (kPairs - 1);
        const int hq = t >> 6, sq = MULTI ? hq / G : 0, hm = MULTI ? hq - sq * G : hq;
        const T* qrow = q + ((size_t)seq_of(sq * 64) * H + (size_t)g0 * G + hm) * kHeadDim;
        qa[u] = elem<T>::load(qrow + pair_first(p, style));
        qb[u] = elem<T>::load(qrow + pair_second(p, style));
    }
    asm volatile("" ::: "memory");  // (keeps the loads above ahead of the wait for the count)
    // MULTI: a token group past the batch has no tokens
    const int n = (MULTI && b + tg >= B) ? 0 : wave_uniform(n_v);
    const int qpos = MULTI ? qpos_v : wave_uniform(qpos_v);
    if (!MULTI && tok0 >= n) {  // no selected token in this tile: neutral statistics
        if (tid < HEADS * G)
            stats[((size_t)b * H + (size_t)g0 * G + tid) * stats_stride + part] = make_float2(-INFINITY, 0.f);
        return;
    }

    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // [3][A | B], later [2][cos/sin]
    __shared__ __attribute__((aligned(16))) float sQ[SQ * HEADS][kMaxGroup][kHeadDim];
    __shared__ float2 sCS[SQ][kPairs];
    __shared__ float2 sStat[HEADS][NTG][kMaxGroup];
    __shared__ int sPos[C::TOK];  // cache row (= RoPE position) of every token of the tile

#pragma unroll
    for (int u = 0; u < NSP; ++u)
        if (tid + u * NT < C::TOK) sPos[tid + u * NT] = pos_reg[u];
    // cos/sin of the query position: thread -> (sequence tid / 64, pair tid % 64); qpos is that sequence's.  Requested
    // here, ahead of the first operand loads, so that the wait for it does not include theirs.
    const bool q_in_table = qpos >= 0 && qpos <= S_max;  // the table holds exactly these positions
    float2 qcs = make_float2(1.f, 0.f);
    if (tid < SQ * kPairs) qcs = rope[(size_t)(q_in_table ? qpos : 0) * kPairs + (tid & (kPairs - 1))];
    auto rotate_query = [&]() {
        if (tid < SQ * kPairs) {
            const int pr = tid & (kPairs - 1);
            if (!q_in_table) {
                double sn, c;
                sincos((double)qpos * inv.f[pr], &sn, &c);
                qcs = make_float2((float)c, (float)sn);
            }
            sCS[tid >> 6][pr] = qcs;
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < QP; ++u) {
            const int t = tid + u * NT;
            if (t < SQ * HEADS * G * kPairs) {
                // (MULTI: t / 64 = sequence * G + head of the group; otherwise head of the tile * G + head of the group)
                const int p = t & (kPairs - 1), hm = t >> 6;
                const float2 c = sCS[MULTI ? hm / G : 0][p];
                float* dst = &sQ[0][0][0] + (size_t)((hm / G) * kMaxGroup + hm % G) * kHeadDim;
                dst[p] = (qa[u] * c.x - qb[u] * c.y) * scale;
                dst[kPairs + p] = (qb[u] * c.x + qa[u] * c.y) * scale;
            }
        }
    };

    // ---- global sources of this thread's pieces ---------------------------------------
    // U_k panel: piece q = tid + i*NT -> head q/512, slot (q%512)/4, 16-byte column q%4.  The
    // packed layout is [head][step][128 slots][64 B]: inside a head the pieces of a step are
    // contiguous, and a step adds 8 KB.
    const unsigned char* a_base = reinterpret_cast<const unsigned char*>(UkP + (size_t)g0 * kHeadDim * r);
    const size_t head_bytes = (size_t)kHeadDim * r * ES;
    auto a_src = [&](int i, int kc) {
        const int qd = tid + i * NT;
        return a_base + (size_t)(qd >> 9) * head_bytes + (size_t)kc * (128 * kLgStep) + (qd & 511) * 16;
    };
    auto a_dst = [&](int i) {
        const int qd = tid + i * NT;
        return (qd >> 9) * 128 * kLgStep + swz64((qd >> 2) & 127, qd & 3);
    };
    const unsigned char* b_base = reinterpret_cast<const unsigned char*>(Kc + (size_t)b * rows_per_seq * r) + (tid & 3) * 16;
    const size_t row_bytes = (size_t)r * ES;
    auto b_dst = [&](int i) { return C::A_BYTES + swz64((tid + i * NT) >> 2, tid & 3); };

    f32x16 acc[4][NB];
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    // steps of the latent axis: all of them, or this workgroup's slice
    const int nkc = MULTI ? r * ES / kLgStep / ksplit : r * ES / kLgStep;
    const int kc_base = MULTI ? kz * nkc : 0;
    struct Regs { u32x4 a[NA]; u32x4 b[NBP]; };
    auto g_load = [&](Regs& R, int kc) {
#pragma unroll
        for (int i = 0; i < NA; ++i) R.a[i] = ld16(a_src(i, kc_base + kc));
#pragma unroll
        for (int i = 0; i < NBP; ++i) R.b[i] = ld16(b_base + (size_t)b_row[i] * row_bytes + (size_t)(kc_base + kc) * kLgStep);
    };
    auto l_store = [&](const Regs& R, int buf) {
        unsigned char* base = lds + (size_t)buf * C::STAGE;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(base + a_dst(i)) = R.a[i];
#pragma unroll
        for (int i = 0; i < NBP; ++i) *reinterpret_cast<u32x4*>(base + b_dst(i)) = R.b[i];
    };
    // cos/sin rows of the tile's tokens for the epilogue, 128 bytes (16 pairs) per token and pass
    const unsigned char* rope_b = reinterpret_cast<const unsigned char*>(rope) + (tid & 7) * 16;
    size_t cs_off[NCS];  // byte offset of this thread's token rows in the table
    u32x4 CR[NCS];
    auto cs_load = [&](int ps) {
#pragma unroll
        for (int i = 0; i < NCS; ++i) CR[i] = ld16(rope_b + cs_off[i] + ps * kLgChunk);
    };
    auto cs_store = [&](int buf) {
#pragma unroll
        for (int i = 0; i < NCS; ++i)
            *reinterpret_cast<u32x4*>(lds + (size_t)buf * C::CS_BYTES + swz((tid + i * NT) >> 3, tid & 7)) = CR[i];
    };

    // MFMA fragments of one half step (32 latent bytes): NB token blocks, 4 head-dim blocks
    struct Frags { u32x4 b[NB]; u32x4 a[4]; };
    auto read_frags = [&](Frags& F, int buf, int ks) {
        const unsigned char* pa = lds + (size_t)buf * C::STAGE + hh * 128 * kLgStep;
        const unsigned char* pb = lds + (size_t)buf * C::STAGE + C::A_BYTES + tg * NB * 32 * kLgStep;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) F.b[nb] = *reinterpret_cast<const u32x4*>(pb + swz64(nb * 32 + l32, ks * 2 + hi));
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) F.a[mb] = *reinterpret_cast<const u32x4*>(pa + swz64(mb * 32 + l32, ks * 2 + hi));
    };
    auto mma_frags = [&](const Frags& F) {
#pragma unroll
        for (int mb = 0; mb < 4; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) mma_op<T>::run(F.a[mb], F.b[nb], acc[mb][nb]);
    };

    // Software pipeline over three LDS stages.  After the barrier every wave of the workgroup is
    // in the same phase, so LDS traffic and MFMAs only overlap if each wave overlaps them itself:
    // while the MFMAs of one half step run, the fragments of the next half step are being read
    // (from this stage, then from the next one, which the previous barrier already published),
    // and the step after that moves from registers to the third stage.  The scheduling fences
    // keep the compiler from sinking the reads behind the MFMAs that are meant to cover them.
    {
        Regs R;
        Frags F0, F1;
        {
            Regs R1;  // second set for the fill only: the first two steps are requested together
            g_load(R, 0);
            g_load(R1, min(1, nkc - 1));
            rotate_query();  // (its barrier also publishes sPos)
#pragma unroll
            for (int i = 0; i < NCS; ++i) cs_off[i] = (size_t)sPos[(tid + i * NT) >> 3] * (kPairs * sizeof(float2));
            cs_load(0);      // cos/sin of the first epilogue pass: in flight during the whole main loop
            l_store(R, 0);
            l_store(R1, 1);
        }
        g_load(R, min(2, nkc - 1));
        __syncthreads();
        read_frags(F0, 0, 0);
        int cur = 0, nxt = 1, third = 2;  // stage of step kc, kc+1, kc+2
        for (int kc = 0; kc < nkc; ++kc) {
            read_frags(F1, cur, 1);
            mma_frags(F0);
            l_store(R, third);                       // step kc+2 (a copy of the last step past the end)
            g_load(R, min(kc + 3, nkc - 1));
            read_frags(F0, nxt, 0);
            mma_frags(F1);
            // issue order: LDS and global memory instructions between the MFMAs that cover them
            {
                constexpr int NM = 4 * NB;            // MFMAs per half step
                constexpr int NR = 4 + NB;            // fragment reads per half step
                constexpr int NW = NA + NBP;          // staging writes = global loads per step
                static_assert(NR <= NM && NW < NM, "not enough MFMAs to cover the memory instructions");
#pragma unroll
                for (int i = 0; i < NR; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA (first half step)
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);  // LDS read (second half step)
                }
                if constexpr (NM > NR) __builtin_amdgcn_sched_group_barrier(0x008, NM - NR, 0);
#pragma unroll
                for (int i = 0; i < NW; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA (second half step)
                    __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // LDS write (step + 2)
                    __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // global load (step + 3)
                }
                constexpr int REM = NM - NW, RPM = (NR + REM - 1) / REM;
#pragma unroll
                for (int i = 0; i < REM; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);  // LDS reads (next step, first half)
                }
            }
            __syncthreads();
            const int t = cur; cur = nxt; nxt = third; third = t;
        }
    }

    // ---- epilogue.  A lane holds, for token l32 of each block, slots mb*32 + 8a + 4hi + c; slot < 64
    // is the first element of pair (slot), slot+64 its partner (mb+2).  Pass ps = 2*ml + ah covers
    // the pairs ml*32 + ah*16 .. +16: the tokens' 128-byte cos/sin pieces are staged in LDS, double
    // buffered, with the loads of the next pass in flight. ------------------------------------------
    float dot[kMaxGroup][NB];
#pragma unroll
    for (int m = 0; m < kMaxGroup; ++m)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) dot[m][nb] = 0.f;
    {
        cs_store(0);
        cs_load(1);
        __syncthreads();
#pragma unroll
        for (int ps = 0; ps < 4; ++ps) {
            const int ml = ps >> 1, ah = ps & 1;
            const unsigned char* cb = lds + (size_t)(ps & 1) * C::CS_BYTES;
#pragma unroll
            for (int al = 0; al < 2; ++al) {
                const int a = 2 * ah + al;
                const int p0 = ml * 32 + a * 8 + hi * 4;
                // the rotated key elements of this lane's NB tokens first, then every query head's pieces are read
                // from LDS once and used for all NB tokens
                float k1[NB][4], k2[NB][4];
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int row = (tg * NB + nb) * 32 + l32;
                    const f32x4 t0 = *reinterpret_cast<const f32x4*>(cb + swz(row, al * 4 + hi * 2));      // pairs p0, p0+1
                    const f32x4 t1 = *reinterpret_cast<const f32x4*>(cb + swz(row, al * 4 + hi * 2 + 1));  // p0+2, p0+3
                    const float cc[4] = {t0.x, t0.z, t1.x, t1.z}, ss[4] = {t0.y, t0.w, t1.y, t1.w};
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float x1 = acc[ml][nb][a * 4 + c], x2 = acc[ml + 2][nb][a * 4 + c];
                        k1[nb][c] = x1 * cc[c] - x2 * ss[c];
                        k2[nb][c] = x2 * cc[c] + x1 * ss[c];
                    }
                }
#pragma unroll
                for (int m0 = 0; m0 < kGroupEnd; m0 += GB) {
                    if (GFIX > 0 || m0 < G) {  // uniform; G is a multiple of GB
                        f32x4 q1[GB], q2[GB];
#pragma unroll
                        for (int mi = 0; mi < GB; ++mi) {
                            q1[mi] = *reinterpret_cast<const f32x4*>(&sQ[MULTI ? tg : hh][m0 + mi][p0]);
                            q2[mi] = *reinterpret_cast<const f32x4*>(&sQ[MULTI ? tg : hh][m0 + mi][kPairs + p0]);
                        }
#pragma unroll
                        for (int mi = 0; mi < GB; ++mi)
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
                                dot[m0 + mi][nb] += q1[mi].x * k1[nb][0] + q1[mi].y * k1[nb][1] + q1[mi].z * k1[nb][2] +
                                                    q1[mi].w * k1[nb][3] + q2[mi].x * k2[nb][0] + q2[mi].y * k2[nb][1] +
                                                    q2[mi].z * k2[nb][2] + q2[mi].w * k2[nb][3];
                    }
                }
            }
            if (ps + 1 < 4) cs_store((ps + 1) & 1);
            if (ps + 2 < 4) cs_load(ps + 2);
            __syncthreads();
        }
    }

    bool ok[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) ok[nb] = (MULTI ? nb * 32 + l32 : tok0 + (tg * NB + nb) * 32 + l32) < n;
    const int bs = MULTI ? seq_of(tg * 64) : b;          // sequence of this wave's tokens
    const bool seq_real = !MULTI || b + tg < B;          // (a token group past the batch writes nothing)
#pragma unroll
    for (int m0 = 0; m0 < kGroupEnd; m0 += GB) {
        if (GFIX > 0 || m0 < G) {  // uniform
#pragma unroll
            for (int mi = 0; mi < GB; ++mi)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) dot[m0 + mi][nb] += __shfl_xor(dot[m0 + mi][nb], 32, kWave);
#pragma unroll
            for (int mi = 0; mi < GB; ++mi)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    const int slot = MULTI ? nb * 32 + l32 : tok0 + (tg * NB + nb) * 32 + l32;
                    const size_t at = ((size_t)bs * H + g * G + m0 + mi) * lk + slot;
                    if (MULTI && ksplit > 1) {  // uniform: this slice's share of the logit
                        if (hi == 0 && slot < lk && seq_real) plogits[(size_t)kz * B * H * lk + at] = dot[m0 + mi][nb];
                    } else if (hi == 0 && slot < lk && seq_real) {
                        logits[at] = ok[nb] ? dot[m0 + mi][nb] : -INFINITY;
                    }
                }
            if (MULTI && ksplit > 1) continue;  // (statistics are taken when the slices are added up)
            // softmax statistics of this tile, per head: the waves' (max, sum exp) merged in wave order below
            float mx[GB], se[GB];
#pragma unroll
            for (int mi = 0; mi < GB; ++mi) {
                mx[mi] = -INFINITY;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) mx[mi] = ok[nb] ? fmaxf(mx[mi], dot[m0 + mi][nb]) : mx[mi];
            }
#pragma unroll
            for (int mi = 0; mi < GB; ++mi) mx[mi] = wave_max(mx[mi]);
#pragma unroll
            for (int mi = 0; mi < GB; ++mi) {
                se[mi] = 0.f;
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) se[mi] += (ok[nb] && hi == 0) ? __expf(dot[m0 + mi][nb] - mx[mi]) : 0.f;
            }
#pragma unroll
            for (int mi = 0; mi < GB; ++mi) se[mi] = wave_sum(se[mi]);
            if (lane == 0) {
#pragma unroll
                for (int mi = 0; mi < GB; ++mi) {
                    if constexpr (MULTI) {  // a token group is the whole (single) tile of its sequence
                        if (seq_real) stats[((size_t)bs * H + (size_t)g * G + m0 + mi) * stats_stride + part] = make_float2(mx[mi], se[mi]);
                    } else {
                        sStat[hh][tg][m0 + mi] = make_float2(mx[mi], se[mi]);
                    }
                }
            }
        }
    }
    if constexpr (MULTI) return;
    __syncthreads();
    if (tid < HEADS * G) {
        const int h2 = tid / G, m = tid - h2 * G;
        float2 st = sStat[h2][0][m];
#pragma unroll
        for (int t = 1; t < NTG; ++t) st = stat_merge(st, sStat[h2][t][m]);
        stats[((size_t)b * H + (size_t)(g0 + h2) * G + m) * stats_stride + part] = st;
    }
}

}  // namespace sals
