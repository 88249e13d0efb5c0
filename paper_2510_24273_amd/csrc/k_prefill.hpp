// Prefill-time bulk compression (Eq. 1; Algorithm 1, projection and append steps, applied to a whole
// prompt at once):  K~ = K U_k,  V~ = V U_v  for n_tok new tokens per sequence, written to the
// cache rows seq_len[b] .. seq_len[b] + n_new[b] - 1.
//
// A plain GEMM on the matrix cores, [tokens x D_kv] . [D_kv x r], both operands read along their
// contiguous axis: the token rows as they lie in memory and the TRANSPOSED projector U^T [r x D_kv]
// (section 0 / 1 of the packed weights, the same rows the one-token projection reads).  One workgroup
// owns TOK tokens x NL latent coordinates of one sequence and one projection; its eight waves are
// 4 token groups x 2 latent groups (NL = 128) or 8 token groups (NL = 64), a wave tile being TOK/4 (TOK/8) tokens
// x 64 latent coordinates.  TOK = 256, or 128 when the larger tile would leave most of the chip without a workgroup.  Both operand tiles walk the D axis in 64-byte steps
// through three swizzled LDS stages with the software pipeline of the logits kernel (fragments of the
// next half step are read under the MFMAs of the current one; the step after next moves from registers
// to the third stage).  fp32 accumulation, one rounding to the storage type at the store, so a row
// equals the one-token projection of the same token up to the order of the fp32 sum.
#pragma once
#include "common.hpp"
#include "k_attend.hpp"
#include "k_logits.hpp"

namespace sals {

constexpr int kPfThreads = 512;
constexpr size_t prefill_lds_bytes(int tok, int nl) { return 3 * (size_t)(tok + nl) * kLgStep; }

struct PrefillArgs {
    const void* X[2];        // new keys / values [B, n_tok, D]
    const void* UT[2];       // transposed projectors [r, D]
    void* cache[2];          // [B, S_max, r]
    const int32_t* seq_len;  // [B] first row to write
    const int32_t* n_new;    // [B] tokens of each sequence (<= n_tok), or nullptr: n_tok everywhere
    int n_tok, D, r, S_max, B, nproj;
    float* pacc;             // SYRK form only: [slices][n_tok, r] fp32 tile sums of each slice of the contraction axis
    int kslice_steps;        // SYRK form only: 64-byte steps of the contraction axis per slice (blockIdx.y = slice)
};

// SYRK: the same tiles and pipeline as a plain product of two row-major operands, out[t, l] = sum_c X[t, c] UT[l, c],
// whose fp32 tile sums are stored as they are instead of becoming cache rows (the covariance of the offline
// calibration, Sec. 4.2, with X = UT = the transposed keys and c running over the calibration tokens).  The
// contraction axis is cut into slices (blockIdx.y), each with its own output matrix, so that narrow matrices still
// fill the chip; a second kernel adds the slices to the fp64 covariance.
template <typename T, int TOK, int NL, bool SYRK = false>
__global__ __launch_bounds__(kPfThreads, 2) void prefill_compress_kernel(PrefillArgs a)
{
    static_assert((NL == 128 || NL == 64) && (TOK == 256 || (TOK == 128 && NL == 128)), "tile");
    constexpr int kPfTok = TOK;
    constexpr int ES = (int)sizeof(T);
    constexpr int WN = NL / 64;                 // latent groups of 64 among the waves
    constexpr int WM = 8 / WN;                  // token groups
    constexpr int MB = kPfTok / WM / 32;        // 32-token MFMA blocks per wave: 2 | 1
    constexpr int A_BYTES = kPfTok * kLgStep, B_BYTES = NL * kLgStep, STAGE = A_BYTES + B_BYTES;
    constexpr int NA = A_BYTES / 16 / kPfThreads;                       // 2
    constexpr int NBP = (B_BYTES / 16 + kPfThreads - 1) / kPfThreads;   // 1
    constexpr bool kBAll = B_BYTES / 16 >= kPfThreads;                   // every thread has a piece of the B tile
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // [3][A | B]

    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hi = lane >> 5;
    const int wm = wave / WN, wn = wave % WN;
    const int b = blockIdx.z / a.nproj, proj = blockIdx.z - b * a.nproj;
    int tile_x = blockIdx.x, tile_y = blockIdx.y;
    if constexpr (SYRK) {
        // The result is symmetric: only the tiles that reach the upper triangle (column tile >= row tile, in units of
        // NL columns) are computed, the rest is mirrored afterwards.  blockIdx.x numbers those tiles row by row.
        constexpr int RPT = kPfTok / NL;                // column tiles a row tile spans: 2 | 1
        const int ncol = a.r / NL;
        int id = blockIdx.x, row = 0;
        while (id >= ncol - row * RPT) { id -= ncol - row * RPT; ++row; }   // (at most n_tok / TOK rounds, uniform)
        tile_x = row; tile_y = row * RPT + id;
    }
    const int tok0 = tile_x * kPfTok, lat0 = tile_y * NL;
    const int n_b = (!SYRK && a.n_new) ? min(max(ld_uniform_i32(a.n_new + b), 0), a.n_tok) : a.n_tok;
    const int row0_v = SYRK ? 0 : ld_uniform_i32(a.seq_len + b);
    const T* X = static_cast<const T*>(a.X[proj]) + (size_t)b * a.n_tok * a.D;
    const T* UT = static_cast<const T*>(a.UT[proj]);

    // global sources of this thread's 16-byte pieces: piece q -> row q/4, column q%4 of the tile
    const unsigned char* a_src[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int q = tid + i * kPfThreads;
        const int t = min(tok0 + (q >> 2), a.n_tok - 1);  // rows past the prompt re-read its last token; never stored
        a_src[i] = reinterpret_cast<const unsigned char*>(X + (size_t)t * a.D) + (q & 3) * 16;
    }
    const unsigned char* b_src;
    {
        const int q = kBAll ? tid : (tid & (B_BYTES / 16 - 1));
        b_src = reinterpret_cast<const unsigned char*>(UT + (size_t)(lat0 + (q >> 2)) * a.D) + (q & 3) * 16;
    }
    auto a_dst = [&](int i) { const int q = tid + i * kPfThreads; return swz64(q >> 2, q & 3); };
    const int b_dst = A_BYTES + swz64((tid & (B_BYTES / 16 - 1)) >> 2, tid & 3);
    const bool b_mine = kBAll || tid < B_BYTES / 16;

    f32x16 acc[MB][2];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mb][nb][v] = 0.f;

    const int nkc_all = a.D * ES / kLgStep;
    const int kc_base = SYRK ? (int)blockIdx.y * a.kslice_steps : 0;
    const int nkc = SYRK ? min(a.kslice_steps, nkc_all - kc_base) : nkc_all;  // (the host gives every slice >= 1 step)
    struct Regs { u32x4 a[NA]; u32x4 b[NBP]; };
    auto g_load = [&](Regs& R, int kc) {
#pragma unroll
        for (int i = 0; i < NA; ++i) R.a[i] = ld16(a_src[i] + (size_t)(kc_base + kc) * kLgStep);
        R.b[0] = ld16(b_src + (size_t)(kc_base + kc) * kLgStep);
    };
    auto l_store = [&](const Regs& R, int buf) {
        unsigned char* base = lds + (size_t)buf * STAGE;
#pragma unroll
        for (int i = 0; i < NA; ++i) *reinterpret_cast<u32x4*>(base + a_dst(i)) = R.a[i];
        if (b_mine) *reinterpret_cast<u32x4*>(base + b_dst) = R.b[0];
    };
    struct Frags { u32x4 a[MB]; u32x4 b[2]; };
    auto read_frags = [&](Frags& F, int buf, int ks) {
        const unsigned char* pa = lds + (size_t)buf * STAGE + wm * MB * 32 * kLgStep;
        const unsigned char* pb = lds + (size_t)buf * STAGE + A_BYTES + wn * 64 * kLgStep;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) F.a[mb] = *reinterpret_cast<const u32x4*>(pa + swz64(mb * 32 + l32, ks * 2 + hi));
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) F.b[nb] = *reinterpret_cast<const u32x4*>(pb + swz64(nb * 32 + l32, ks * 2 + hi));
    };
    auto mma_frags = [&](const Frags& F) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) mma_op<T>::run(F.a[mb], F.b[nb], acc[mb][nb]);
    };

    {
        Regs R, R1;
        Frags F0, F1;
        g_load(R, 0);
        g_load(R1, min(1, nkc - 1));
        l_store(R, 0);
        l_store(R1, 1);
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
            __syncthreads();
            const int t = cur; cur = nxt; nxt = third; third = t;
        }
    }

    // acc[mb][nb][4a+c] is token wm*MB*32 + mb*32 + 8a + 4hi + c of the tile, latent coordinate wn*64 + nb*32 + l32:
    // for fixed (a, c) the 32 lanes of a half wave write 32 consecutive elements of one cache row
    if constexpr (SYRK) {
        float* pout = a.pacc + (size_t)blockIdx.y * a.n_tok * a.r;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = tok0 + (wm * MB + mb) * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
                if (t < n_b) {
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb) pout[(size_t)t * a.r + lat0 + wn * 64 + nb * 32 + l32] = acc[mb][nb][v];
                }
            }
        return;
    }
    const int row0 = wave_uniform(row0_v);
    T* cache = static_cast<T*>(a.cache[proj]) + (size_t)b * a.S_max * a.r;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int t = tok0 + (wm * MB + mb) * 32 + (v >> 2) * 8 + hi * 4 + (v & 3);
            const long long row = (long long)row0 + t;
            if (t < n_b && row0 >= 0 && row < a.S_max) {
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
                    elem<T>::store(cache + (size_t)row * a.r + lat0 + wn * 64 + nb * 32 + l32, acc[mb][nb][v]);
            }
        }
}

// after a bulk append: advance every sequence by its token count (separate launch, so that every cache row
// has been written before any length changes)
__global__ void advance_seq_len_kernel(int32_t* __restrict__ seq_len, const int32_t* __restrict__ n_new, int n_tok, int B,
                                       int S_max)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const int n = n_new ? min(max(n_new[b], 0), n_tok) : n_tok;
    const int s = seq_len[b];
    if (s >= 0) seq_len[b] = (int)min((long long)s + n, (long long)S_max);
}

}  // namespace sals
