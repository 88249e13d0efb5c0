// C ABI of the SALS decode-step attention library: descriptor validation, workspace
// carving and kernel launches.  Every entry point only enqueues work on the caller's
// stream; nothing here allocates device memory or synchronises.
#include "../../include/sals.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <functional>
#include <mutex>
#include <new>
#include <vector>

#include "common.hpp"
#include "k_attend.hpp"
#include "k_calib.hpp"
#include "k_dense.hpp"
#include "k_logits.hpp"
#include "k_logits_small.hpp"
#include "k_overlap.hpp"
#include "k_prefill.hpp"
#include "k_project.hpp"
#include "k_scores.hpp"
#include "k_topk.hpp"
#include "k_topk_multi.hpp"
#include "k_qvalue.hpp"
#include "k_value.hpp"
#include "k_window.hpp"

using namespace sals;

// Scratch of sals_latent_scores_noalloc: part of the device image, one copy per GPU.  In host code the
// name is only a handle for hipGetSymbolAddress; kernels are given the address looked up there.
static __device__ __align__(256) unsigned char scratch[SALS_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

struct Layout {  // byte offsets into the workspace
    size_t qt, scores, idx, n_sel, n_lo, logits, plogits, stats, rope, tpart, qv_part, dn_part, tm_part, tm_hist, tm_meta, tm_cand, tm_srange, total;
    int lk;                      // logits row stride (floats)
    int max_parts;               // token tiles per head of the logits kernel, at most
    int pv_tok_per_wg, pv_ntr, pv_waves;  // value-sum token ranges, waves per workgroup (4 | 8)
    int qv_tok_per_wg, qv_ntr;   // quantised-value attention: token ranges
    int dn_chunks, dn_tok;       // dense baseline: token chunks per sequence, tokens per chunk
    int proj_np;                 // D-axis slices of the query projection
    int tm_chunks;               // chunks of the multi-workgroup selection (0: one workgroup per sequence)
    size_t w_section;            // elements per section of the packed weights
};


}  // namespace

struct ProfRecord { int kernel; hipEvent_t start, stop; };

// which logits kernel a context's shape gets: 1 = 2 heads x 256 tokens, 2 = 1 head x 256 tokens, 3 = 1 head x 64
// tokens (then: slices of the latent axis per tile, 128-byte steps loaded ahead); n_parts = token tiles per head
struct LogitsPlan { int pick, n_parts, ksplit, nst; };

struct sals_ctx {
    sals_desc d;
    Layout L;
    unsigned char* ws;
    size_t ws_bytes;
    InvFreq inv;
    // launch shapes, fixed when the context is made (sals_create): nothing on the launch path reads the
    // environment, plans or sets kernel attributes
    LogitsPlan plan{3, 0, 1, 1};
    int score_rows = 16;         // cache rows per workgroup of the score kernel
    int score_stream = -1;       // read-once hint on the score kernel's cache loads: -1 by size, 0 / 1 forced (tuning aid)
    bool fuse_select = true;     // decode steps may select inside the logits kernel (tuning aid SALS_TUNE_FUSE_SELECT=0)
    // cos/sin table over the positions 0 .. S_max (in the workspace): 0 = not filled, 1 = fill enqueued on
    // rope_stream and marked by rope_ev, 2 = known to be complete
    int rope_state = 0;
    hipStream_t rope_stream = nullptr;
    hipEvent_t rope_ev = nullptr;
    bool lds_allowed = false;    // the logits kernels' dynamic-LDS attribute has been raised
    bool profiling = false;
    std::vector<ProfRecord> prof;
};

namespace {

const char* const kKernelNames[SALS_N_KERNELS] = {
    "project", "scores", "topk", "attend_logits", "attend_pv", "attend_out", "attend_qv", "dense_attend", "prefill"};

// Brackets one kernel launch with a pair of events while profiling is on.
struct ProfScope {
    sals_ctx* c;
    hipStream_t st;
    ProfRecord rec{};
    bool on;
    ProfScope(const sals_ctx* ctx, int kernel, hipStream_t s) : c(const_cast<sals_ctx*>(ctx)), st(s), on(ctx->profiling)
    {
        if (!on) return;
        rec.kernel = kernel;
        if (hipEventCreate(&rec.start) != hipSuccess || hipEventCreate(&rec.stop) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(rec.start, st);
    }
    ~ProfScope()
    {
        if (!on) return;
        (void)hipEventRecord(rec.stop, st);
        c->prof.push_back(rec);
    }
};

sals_status validate(const sals_desc* d)
{
    if (!d) return SALS_ERR_INVALID_ARG;
    if (d->dtype != SALS_F32 && d->dtype != SALS_BF16) return SALS_ERR_INVALID_ARG;
    if (d->rope_style != SALS_ROPE_HALF && d->rope_style != SALS_ROPE_INTERLEAVED) return SALS_ERR_INVALID_ARG;
    if (d->B < 1 || d->S_max < 1 || d->H_q < 1 || d->H_kv < 1 || d->d < 2 || (d->d & 1)) return SALS_ERR_INVALID_ARG;
    if (d->H_q % d->H_kv != 0) return SALS_ERR_INVALID_ARG;
    if (d->r < 1 || d->r_score < 1 || d->r_score > d->r) return SALS_ERR_INVALID_ARG;
    if (d->top_k < 1 || d->n_recent < 0 || d->n_sink < 0) return SALS_ERR_INVALID_ARG;
    if (!(d->rope_theta > 0.f) || !std::isfinite(d->rope_theta)) return SALS_ERR_INVALID_ARG;
    // what the kernels cover
    if (d->d != kHeadDim) return SALS_ERR_UNSUPPORTED;
    if (d->r % 64 != 0 || d->r > 2048) return SALS_ERR_UNSUPPORTED;
    if (d->r_score % 8 != 0 || d->r_score > kScoreMaxR) return SALS_ERR_UNSUPPORTED;
    if (d->H_q / d->H_kv > kMaxGroup || d->H_q > kPvMaxHeads) return SALS_ERR_UNSUPPORTED;
    if (d->S_max > (1 << 20)) return SALS_ERR_UNSUPPORTED;  // the RoPE table takes 512 B per position
    if ((long long)d->B * (d->H_q / d->H_kv) > kProjMaxCols) return SALS_ERR_UNSUPPORTED;
    if ((long long)d->top_k + d->n_recent + d->n_sink > 65536) return SALS_ERR_UNSUPPORTED;
    return SALS_OK;
}

Layout make_layout(const sals_desc& d)
{
    Layout L{};
    const int D = d.H_kv * d.d;
    const int k_tot = d.top_k + d.n_sink + d.n_recent;
    L.lk = ceil_div(k_tot, 128) * 128;  // whole steps of the value kernel (its last step may read up to the row end)
    L.w_section = (size_t)D * d.r;
    {   // query projection: slice the D axis until at least 160 workgroups stream U_k^T (measured: at r = 640 four
        // slices = 160 workgroups project as fast as eight, and the score kernel then adds four partial sums, not eight)
        int nks = D / (d.dtype == SALS_BF16 ? 32 : 16);
        int np = 1;
        while (np < kScoreMaxParts && (d.r / 16) * np < 160 && nks % (np * 2) == 0 && nks / (np * 2) >= 4) np *= 2;
        if (const char* e = std::getenv("SALS_TUNE_PROJ_NP")) { const int v = std::atoi(e); if (v >= 1 && v <= kScoreMaxParts && nks % v == 0) np = v; }  // tuning aid
        L.proj_np = np;
    }
    // value sum: split the selected tokens into ranges of whole 64-token steps (at least two steps, at
    // most kPvMaxTok tokens) as long as every workgroup still gets a CU of its own (measured: a few CUs
    // with two workgroups set the kernel's duration)
    {
        int blocks = d.r / kPvCols;
        int want = std::max(1, 256 / (blocks * d.B));
        int n_tr = std::max(1, std::min(std::min(want, kMaxRanges), ceil_div(k_tot, 2 * kPvTJ)));
        if (const char* e = std::getenv("SALS_TUNE_PV_RANGES")) n_tr = std::max(1, std::min(64, std::atoi(e)));  // tuning aid
        n_tr = std::max(n_tr, ceil_div(k_tot, kPvMaxTok));
        int tok = ceil_div(ceil_div(k_tot, n_tr), kPvTJ) * kPvTJ;
        // eight waves once each of them has two groups of 16 tokens (measured: 128 tokens are 0.5 us faster with four)
        L.pv_waves = tok >= 4 * kPvTJ ? 8 : 4;
        if (const char* e = std::getenv("SALS_TUNE_PV_WAVES")) L.pv_waves = std::atoi(e) == 4 ? 4 : 8;  // tuning aid
        L.pv_tok_per_wg = tok;
        L.pv_ntr = ceil_div(k_tot, tok);
    }
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    L.qt = take((size_t)L.proj_np * d.B * d.r * 4);
    L.scores = take((size_t)d.B * d.S_max * 4);
    L.idx = take((size_t)d.B * k_tot * 4);
    L.n_sel = take((size_t)d.B * 4);
    L.n_lo = take((size_t)d.B * 4);                          // recent-window attention: tokens of the low-rank pass
    L.logits = take((size_t)d.B * d.H_q * L.lk * 4);
    // partial logits of the latent slices, for shapes with so few 64-token tiles that the latent axis is split too
    // (also for batches of short selections, whose multi-sequence tiles may split the latent axis)
    L.plogits = take((ceil_div(k_tot, kLsTok) * d.H_kv * d.B <= 128 || k_tot <= 64)
                         ? (size_t)kLsMaxSplit * d.B * d.H_q * L.lk * 4 : 0);
    L.max_parts = ceil_div(k_tot, 32) + 2;  // (room for the tiles of a recent-window pass beside the context's own)
    L.stats = take((size_t)d.B * d.H_q * L.max_parts * 8);
    L.rope = take((size_t)(d.S_max + 1) * kPairs * 8);  // positions 0 .. S_max (the query after a full cache)
    L.tpart = take((size_t)L.pv_ntr * d.B * d.H_q * d.r * 4);
    {   // quantised-value attention: one workgroup per (sequence, token range, KV head), 32 tokens side
        // by side; a second range (and with it the merge launch) only pays above ~32 tokens per slot
        int n_tr = k_tot <= 32 * kQvSlots ? 1 : std::min(kQvMaxRanges, ceil_div(k_tot, 16 * kQvSlots));
        if (const char* e = std::getenv("SALS_TUNE_QV_RANGES")) n_tr = std::max(1, std::min(kQvMaxRanges, std::atoi(e)));  // tuning aid
        n_tr = std::max(n_tr, ceil_div(k_tot, kQvMaxTok));
        L.qv_tok_per_wg = ceil_div(k_tot, n_tr);
        L.qv_ntr = ceil_div(k_tot, L.qv_tok_per_wg);
        L.qv_part = take((size_t)L.qv_ntr * d.B * d.H_q * kHeadDim * 4);
    }
    {   // dense baseline: token chunks until about 2048 workgroups stream the cache, 256 tokens at least
        int n = std::min(kDnMaxChunks, std::max(1, ceil_div(2048, d.B * d.H_kv)));
        n = std::max(1, std::min(n, d.S_max / 256));
        L.dn_tok = ceil_div(ceil_div(d.S_max, n), 16) * 16;
        L.dn_chunks = ceil_div(d.S_max, L.dn_tok);
        L.dn_part = take((size_t)d.B * d.H_q * L.dn_chunks * kDnRec * 4);
    }
    // long sequences: selection spread over 8192-score chunks
    L.tm_chunks = d.S_max > 32768 ? ceil_div(d.S_max, kTmChunk) : 0;
    if (L.tm_chunks > 0) {
        L.tm_part = take((size_t)d.B * L.tm_chunks * sizeof(uint2));
        L.tm_hist = take((size_t)d.B * L.tm_chunks * kTmCum * 4);
        L.tm_meta = take((size_t)d.B * sizeof(TopkMeta));
        L.tm_cand = take((size_t)d.B * kTmCand * sizeof(uint2));
        // key ranges the score kernel leaves per workgroup inside a decode step (at least 16 rows per workgroup)
        L.tm_srange = take((size_t)d.B * ceil_div(d.S_max, kScoreRowsPerIter) * sizeof(uint2));
    }
    L.total = o;
    return L;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool bad(const void* p) { return p == nullptr || !aligned16(p); }

inline sals_status launch_status()
{
    return hipGetLastError() == hipSuccess ? SALS_OK : SALS_ERR_HIP;
}

template <typename T> inline const T* w_section(const sals_ctx* c, const void* W, int sec)
{
    return static_cast<const T*>(W) + (size_t)sec * c->L.w_section;
}

// QUERY: x0 = q.  Otherwise x0 / x1 = new key / value rows (x1 may be null: keys only); `bump` advances
// the sequence lengths afterwards; ring > 0: the caches are rings of that many rows.
template <typename T, bool QUERY>
sals_status launch_project(const sals_ctx* c, const void* W, const void* x0, const void* x1, void* cache0,
                           void* cache1, int32_t* seq_len, hipStream_t st, bool bump = true, int ring = 0)
{
    const sals_desc& d = c->d;
    ProjArgs a{};
    a.UT[0] = w_section<T>(c, W, 0);
    a.UT[1] = w_section<T>(c, W, 1);
    a.X[0] = x0; a.X[1] = x1;
    a.cache[0] = cache0; a.cache[1] = cache1;
    a.out_f32 = reinterpret_cast<float*>(c->ws + c->L.qt);
    a.seq_len = seq_len;
    a.B = d.B; a.D = d.H_kv * d.d; a.r = d.r; a.H = d.H_q; a.H_kv = d.H_kv; a.d = d.d;
    a.S_max = d.S_max; a.nproj = (QUERY || x1 == nullptr) ? 1 : 2; a.np = QUERY ? c->L.proj_np : 1;
    a.ring = ring;
    {
        ProfScope ps(c, SALS_K_PROJECT, st);
        hipLaunchKernelGGL((project_kernel<T, QUERY>), dim3(d.r / 16, a.np, a.nproj), dim3(kProjThreads), 0, st, a);
    }
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    if (!QUERY && bump)
        hipLaunchKernelGGL(bump_seq_len_kernel, dim3(ceil_div(d.B, 128)), dim3(128), 0, st, seq_len, d.B, d.S_max);
    return launch_status();
}

template <typename T>
// wg_range: where every workgroup leaves the key range of its scores (for the long-sequence selection of the same
// step), or nullptr
sals_status launch_scores(const sals_ctx* c, const void* Kc, const int32_t* seq_len, float* scores,
                          hipStream_t st, uint2* wg_range = nullptr)
{
    const sals_desc& d = c->d;
    constexpr int VEC = elem<T>::vec;
    const int nch = ceil_div(d.r_score / VEC, 16);
    const int rows = c->score_rows;
    dim3 grid(ceil_div(d.S_max, rows), d.B);
    const float* qt = reinterpret_cast<const float*>(c->ws + c->L.qt);
    const T* K = static_cast<const T*>(Kc);
    // a cache prefix of 32 MB and more is read as a stream the caches need not keep; a smaller one with plain loads (it
    // may still be cached from the previous step)
    bool stream = (size_t)d.B * d.S_max * d.r_score * sizeof(T) >= ((size_t)32 << 20);
    if (c->score_stream >= 0) stream = c->score_stream != 0;
    ProfScope ps(c, SALS_K_SCORES, st);
#define SALS_SCORES_CASE(N)                                                                         \
    case N:                                                                                         \
        if (stream)                                                                                  \
            hipLaunchKernelGGL((scores_kernel<T, N, true>), grid, dim3(kScoreThreads), 0, st, K, qt,    \
                               c->L.proj_np, seq_len, scores, d.B, d.S_max, d.r, d.r_score, rows,       \
                               wg_range, d.n_sink, d.n_recent);                                                         \
        else                                                                                         \
            hipLaunchKernelGGL((scores_kernel<T, N, false>), grid, dim3(kScoreThreads), 0, st, K, qt,   \
                               c->L.proj_np, seq_len, scores, d.B, d.S_max, d.r, d.r_score, rows,       \
                               wg_range, d.n_sink, d.n_recent);                                                         \
        break;
    switch (nch) {
        SALS_SCORES_CASE(1) SALS_SCORES_CASE(2) SALS_SCORES_CASE(3) SALS_SCORES_CASE(4)
        SALS_SCORES_CASE(5) SALS_SCORES_CASE(6) SALS_SCORES_CASE(7) SALS_SCORES_CASE(8)
        SALS_SCORES_CASE(9) SALS_SCORES_CASE(10) SALS_SCORES_CASE(11) SALS_SCORES_CASE(12)
        SALS_SCORES_CASE(13) SALS_SCORES_CASE(14) SALS_SCORES_CASE(15) SALS_SCORES_CASE(16)
        default: return SALS_ERR_UNSUPPORTED;
    }
#undef SALS_SCORES_CASE
    return launch_status();
}

// wl: also leave the recent-window lists (see WindowLists); by default none
// score_ranges: the scores were written by this context's score kernel in the same step, which left its workgroups'
// key ranges in the workspace (the chain then needs no range pass of its own)
sals_status launch_topk(const sals_ctx* c, const float* scores, const int32_t* seq_len, int32_t* idx,
                        int32_t* n_sel, hipStream_t st, WindowLists wl = WindowLists{nullptr, nullptr, nullptr, 0},
                        bool score_ranges = false)
{
    const sals_desc& d = c->d;
    dim3 grid(d.B), block(kTopkThreads);
    ProfScope ps(c, SALS_K_TOPK, st);
#define SALS_TOPK(F4)                                                                                \
    hipLaunchKernelGGL((topk_kernel<F4>), grid, block, 0, st, scores, seq_len, idx, n_sel, d.S_max, \
                       d.top_k, d.n_sink, d.n_recent)
    if (c->L.tm_chunks > 0) {
        const Layout& L = c->L;
        const int nc = L.tm_chunks;
        TopkMultiWs ws{};
        ws.part = reinterpret_cast<uint2*>(c->ws + L.tm_part); ws.hist = reinterpret_cast<uint32_t*>(c->ws + L.tm_hist);
        ws.meta = reinterpret_cast<TopkMeta*>(c->ws + L.tm_meta); ws.cand = reinterpret_cast<uint2*>(c->ws + L.tm_cand);
        ws.range = ws.part; ws.n_range = nc;
        dim3 cgrid(nc, d.B);
        if (score_ranges) {
            ws.range = reinterpret_cast<const uint2*>(c->ws + L.tm_srange);
            ws.n_range = ceil_div(d.S_max, c->score_rows);
        } else {
            hipLaunchKernelGGL(topk_range_kernel, cgrid, block, 0, st, scores, seq_len, ws, d.S_max, nc, d.n_sink,
                               d.n_recent);
        }
        hipLaunchKernelGGL(topk_hist_kernel, cgrid, block, 0, st, scores, seq_len, ws, d.S_max, nc, d.n_sink, d.n_recent);
        hipLaunchKernelGGL(topk_place_kernel, cgrid, block, 0, st, scores, seq_len, ws, idx, d.S_max, nc, d.top_k,
                           d.n_sink, d.n_recent);
        hipLaunchKernelGGL(topk_finish_kernel, grid, block, 0, st, scores, seq_len, ws, idx, n_sel, d.S_max, d.top_k,
                           d.n_sink, d.n_recent, wl);
        return launch_status();
    }
#define SALS_TOPK_W(F4)                                                                                    \
    hipLaunchKernelGGL((topk_window_kernel<F4>), grid, block, 0, st, scores, seq_len, idx, n_sel, d.S_max, \
                       d.top_k, d.n_sink, d.n_recent, wl)
    if (wl.idx_hi != nullptr) {
        if (d.S_max <= 4096) SALS_TOPK_W(1);
        else if (d.S_max <= 8192) SALS_TOPK_W(2);
        else if (d.S_max <= 16384) SALS_TOPK_W(4);
        else SALS_TOPK_W(8);
        return launch_status();
    }
#undef SALS_TOPK_W
    if (d.S_max <= 4096) SALS_TOPK(1);
    else if (d.S_max <= 8192) SALS_TOPK(2);
    else if (d.S_max <= 16384) SALS_TOPK(4);
    else SALS_TOPK(8);
#undef SALS_TOPK
    return launch_status();
}

// rows per workgroup of the score kernel: a multiple of 16 giving roughly 1024 workgroups, 16..64 rows
// (measured optimum; the first 16 rows of a workgroup are requested before the sequence length is known, so
// shorter ranges would pay more for the empty part of a cache)
int plan_score_rows(const sals_desc& d)
{
    long long total_rows = (long long)d.B * d.S_max;
    int rows = (int)std::min<long long>(64, std::max<long long>(16, total_rows / 1024));
    if (const char* e = std::getenv("SALS_TUNE_SCORE_ROWS")) rows = std::max(16, std::min(1 << 16, std::atoi(e)));  // tuning aid
    return ceil_div(rows, kScoreRowsPerIter) * kScoreRowsPerIter;
}

// Enqueues the fill of the context's cos/sin table on `st` and marks it with an event.
sals_status enqueue_rope_table(sals_ctx* c, hipStream_t st)
{
    const size_t n = (size_t)(c->d.S_max + 1) * kPairs;
    hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       reinterpret_cast<float2*>(c->ws + c->L.rope), c->inv, c->d.S_max + 1);
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    if (!c->rope_ev && hipEventCreateWithFlags(&c->rope_ev, hipEventDisableTiming) != hipSuccess) return SALS_ERR_HIP;
    if (hipEventRecord(c->rope_ev, st) != hipSuccess) return SALS_ERR_HIP;
    c->rope_stream = st;
    c->rope_state = 1;
    return SALS_OK;
}

// Before a kernel that reads the cos/sin table is enqueued on `st`.  A prepared context (sals_prepare) costs one
// comparison.  Otherwise the fill is enqueued on first use and later calls are ordered behind it: same stream by
// stream order, another stream by waiting for the event.  A stream under graph capture needs a prepared context
// (a captured fill would not run before eager work, and events of other streams cannot be consulted there).
sals_status ensure_rope_table(const sals_ctx* cc, hipStream_t st)
{
    sals_ctx* c = const_cast<sals_ctx*>(cc);
    if (c->rope_state == 2) return SALS_OK;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) return SALS_ERR_HIP;
    if (cap != hipStreamCaptureStatusNone) return SALS_ERR_INVALID_ARG;
    if (c->rope_state == 0) return enqueue_rope_table(c, st);
    if (hipEventQuery(c->rope_ev) == hipSuccess) { c->rope_state = 2; return SALS_OK; }
    (void)hipGetLastError();  // (hipErrorNotReady is not an error here)
    if (st == c->rope_stream) return SALS_OK;
    return hipStreamWaitEvent(st, c->rope_ev, 0) == hipSuccess ? SALS_OK : SALS_ERR_HIP;
}

// the logits kernels use more than the default 48 KB of dynamic LDS: raised once per context, on first use
template <typename T> sals_status allow_logits_lds(const LogitsPlan& P, int group);
template <typename T> sals_status ensure_lds_attr(const sals_ctx* cc)
{
    sals_ctx* c = const_cast<sals_ctx*>(cc);
    if (c->lds_allowed) return SALS_OK;
    if (allow_logits_lds<T>(c->plan, c->d.H_q / c->d.H_kv) != SALS_OK) return SALS_ERR_HIP;
    c->lds_allowed = true;
    return SALS_OK;
}

template <typename T>
sals_status launch_dense(const sals_ctx* c, const void* q, const int32_t* q_pos, const void* K, const void* V,
                         const int32_t* seq_len, void* out, hipStream_t st)
{
    const sals_desc& d = c->d;
    const Layout& L = c->L;
    if (ensure_rope_table(c, st) != SALS_OK) return SALS_ERR_HIP;
    float* part = reinterpret_cast<float*>(c->ws + L.dn_part);
    const float2* rope = reinterpret_cast<const float2*>(c->ws + L.rope);
    const int G = d.H_q / d.H_kv;
    const dim3 grid(L.dn_chunks, d.H_kv, d.B);
    ProfScope ps(c, SALS_K_DENSE, st);
#define SALS_DENSE(GMAX)                                                                                   \
    hipLaunchKernelGGL((dense_attend_kernel<T, GMAX>), grid, dim3(256), 0, st, static_cast<const T*>(q), q_pos, \
                       static_cast<const T*>(K), static_cast<const T*>(V), seq_len, rope, c->inv, part, d.S_max, \
                       d.H_q, d.H_kv, L.dn_chunks, L.dn_tok, d.rope_style, 1.0f / std::sqrt((float)d.d))
    if (G <= 1) SALS_DENSE(1); else if (G <= 2) SALS_DENSE(2); else if (G <= 4) SALS_DENSE(4); else SALS_DENSE(8);
#undef SALS_DENSE
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    hipLaunchKernelGGL((dense_merge_kernel<T>), dim3(d.B * d.H_q), dim3(128), 0, st, part, static_cast<T*>(out),
                       L.dn_chunks);
    return launch_status();
}

// quantised full-rank value cache; codes_w != nullptr: plus the recent window's ring of 8-bit rows (the last
// n_sel - n_lo[b] selected tokens), whose logits a second logits pass left in logits_w [B, H, lk_w]
struct QvCache {
    const void* codes; const void* meta; int bits;
    const void* codes_w = nullptr; const void* meta_w = nullptr; const float* logits_w = nullptr;
    const int32_t* n_lo = nullptr; int lk_w = 0, ring = 0;
};

// qv == nullptr: latent value cache Vc, value sum in latent space and output projection through U_v.
// Otherwise: values are the de-quantised rows of the quantised cache (Vc unused).
// ring > 0: Kc, Vc are rings of that many rows per sequence (token t in row t mod ring).
// phases: which of the three launches to enqueue (all of them by default).  link: where the logits kernel leaves
// its tile statistics and where the value kernel finds the statistics of the whole softmax, when two passes over
// different caches share one softmax (recent window); by default the context's own array.
enum { kPhaseLogits = 1, kPhaseValue = 2, kPhaseOut = 4, kPhaseAll = 7 };
struct StatsLink { float2* stats; int stride; int part0; };  // [B*H][stride] records, this pass's tiles from part0 on

template <typename T> LogitsPlan plan_logits(const sals_desc& d)
{
    const int k_tot = d.top_k + d.n_sink + d.n_recent;
    auto n_wg = [&](int heads, int tok) { return (long long)ceil_div(k_tot, tok) * (d.H_kv / heads) * d.B; };
    LogitsPlan P{3, 0, 1, 1};
    // the 64-token kernel's split of the latent axis: with fewer workgroups than half the chip, as far as every slice
    // keeps at least two steps and the workgroups still fit the chip in one round
    const int nkc128 = d.r * (int)sizeof(T) / kLgChunk;
    const long long n_wg1 = n_wg(1, kLsTok);
    const bool allow_split = [] { const char* e = std::getenv("SALS_TUNE_LOGITS_KSPLIT"); return !e || std::atoi(e) != 0; }();  // tuning aid
    if (allow_split && n_wg1 <= 128)
        for (int ks = kLsMaxSplit; ks >= 2; ks /= 2)
            if (n_wg1 * ks <= 256 && nkc128 % ks == 0 && nkc128 / ks >= 2) { P.ksplit = ks; break; }
    // Estimated duration of each kernel for this shape, from measured per-step and per-workgroup figures (microseconds):
    // a 256-token tile walks the latent axis in 64-byte steps of 0.88 us (two heads) or 0.65 us (one head) whatever
    // part of the tile is filled, workgroups beyond one per compute unit queue up, and the epilogue grows with the
    // query heads per KV head; a 64-token tile is bound by pulling its operands (the head's projector slice and 64
    // rows) into the compute unit at about 51 GB/s.
    {
        const double steps = (double)d.r * sizeof(T) / kLgStep, G = (double)(d.H_q / d.H_kv);
        auto rounds = [](long long n) { return (double)((n + 255) / 256); };
        const double over = 4.0 + 2.2 * G;
        const double t1 = d.H_kv % 2 == 0 ? rounds(n_wg(2, 256)) * steps * 0.88 + over : 1e30;
        const double t2 = rounds(n_wg(1, 256)) * steps * 0.65 + over;
        const double bytes3 = (double)(kHeadDim + kLsTok) * d.r * sizeof(T) / P.ksplit;
        const double t3 = rounds(n_wg1 * P.ksplit) * (bytes3 / 51e3 + 3.0 + 0.3 * G) + (P.ksplit > 1 ? 3.0 : 0.0);
        P.pick = t1 <= t2 && t1 <= t3 ? 1 : (t2 <= t3 ? 2 : 3);
    }
    if (const char* e = std::getenv("SALS_TUNE_LOGITS")) {  // tuning aid: 1 | 2 | 3
        const int v = std::atoi(e);
        if (v == 1 && d.H_kv % 2 == 0) P.pick = 1;
        if (v == 2 || v == 3) P.pick = v;
    }
    // A selection of at most 64 tokens per sequence (a recent window) in a batch: tiles of four sequences' selections,
    // 256 tokens against one pass over the head's projector, the latent axis cut until the launch fills the chip.
    // Estimated like the one-head 256-token tile (0.57 us per step measured at such shapes, 8 us around the loop, 4 us
    // for the finishing launch of a split).
    const char* const force = std::getenv("SALS_TUNE_LOGITS");  // tuning aid: "4" asks for these tiles at any batch
    const bool forced4 = force && std::atoi(force) == 4;
    if (k_tot <= 64 && ((P.pick == 3 && d.B >= 8) || forced4)) {
        const int steps = d.r * (int)sizeof(T) / kLgStep;
        const long long tiles = (long long)ceil_div(d.B, 4) * d.H_kv;
        int ks = 1;
        while (ks < kLsMaxSplit && tiles * ks < 256 && steps % (2 * ks) == 0 && steps / (2 * ks) >= 8) ks *= 2;
        if (const char* e = std::getenv("SALS_TUNE_MULTI_KSPLIT")) {  // tuning aid: any divisor of the step count up to 8
            const int v = std::atoi(e);
            if (v >= 1 && v <= kLsMaxSplit && steps % v == 0) ks = v;
        }
        const double t4 = (double)((tiles * ks + 255) / 256) * ((double)steps / ks * 0.57 + 8.0) + (ks > 1 ? 4.0 : 0.0);
        const double bytes3 = (double)(kHeadDim + kLsTok) * d.r * sizeof(T);
        const double t3 = (double)((n_wg1 + 255) / 256) * (bytes3 / 51e3 + 3.0 + 0.3 * (d.H_q / d.H_kv));
        if (t4 < t3 || forced4) {
            P.pick = 4; P.n_parts = 1; P.ksplit = ks;
            return P;
        }
    }
    if (P.pick != 3) {
        P.n_parts = ceil_div(k_tot, 256);
        P.ksplit = 1;
        return P;
    }
    P.n_parts = ceil_div(k_tot, kLsTok);
    const int nkc = nkc128 / P.ksplit;
    P.nst = kLsMaxChunk;  // steps loaded ahead: the largest divisor of the step count
    while (nkc % P.nst != 0) --P.nst;
    return P;
}

// the 64-token logits kernel for a number of steps loaded ahead, with or without the selection inside
template <typename T> struct SmallLogits {
    typedef void (*Fn)(const int32_t*, const int32_t*, const T*, int, int, int, int, int, int, int, int, const T*, const T*,
                       const int32_t*, const float2*, InvFreq, float*, float2*, int, int, int, float, int, float*, int,
                       FusedSelect);
    static Fn get(int nst, bool fused)
    {
#define SALS_LS(N) case N: return fused ? (Fn)attend_logits_small_kernel<T, N, true> : (Fn)attend_logits_small_kernel<T, N, false>;
        switch (nst) {
            SALS_LS(1) SALS_LS(2) SALS_LS(3) SALS_LS(4) SALS_LS(5) SALS_LS(6) SALS_LS(7) SALS_LS(8) SALS_LS(9)
            default: return fused ? (Fn)attend_logits_small_kernel<T, 10, true> : (Fn)attend_logits_small_kernel<T, 10, false>;
        }
#undef SALS_LS
    }
};

// Whether a whole decode step on this context lets the logits kernel select by itself (no selection launch): the
// 64-token kernel without a split of the latent axis, a cache of at most 4096 rows whose score rows start 16-byte
// aligned, a selection that fits the kernel's list.
bool fused_selection(const sals_ctx* c)
{
    const sals_desc& d = c->d;
    return c->plan.pick == 3 && c->plan.ksplit == 1 && d.S_max <= kLsFusedMaxS && d.S_max % 4 == 0 &&
           d.top_k + d.n_sink + d.n_recent <= kLsFusedMaxK && c->fuse_select;
}

// the instantiation of the 256-token logits kernel for a group size (query heads per KV head)
template <typename T, int HEADS, int NTG, int NB, bool MULTI = false> auto logits_kernel_for(int group)
{
    if (group == 1) return attend_logits_kernel<T, HEADS, NTG, NB, 1, 1, MULTI>;
    if (group == 4) return attend_logits_kernel<T, HEADS, NTG, NB, 4, 4, MULTI>;
    if (group % 4 == 0) return attend_logits_kernel<T, HEADS, NTG, NB, 4, 0, MULTI>;
    return attend_logits_kernel<T, HEADS, NTG, NB, 1, 0, MULTI>;
}

template <typename T> sals_status allow_logits_lds(const LogitsPlan& P, int group)
{
    auto allow = [](const void* kern, size_t bytes) {
        return bytes <= 48 * 1024 ||
               hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess;
    };
    bool ok = true;
    if (P.pick == 1) ok = allow(reinterpret_cast<const void*>(logits_kernel_for<T, 2, 4, 2>(group)), logits_cfg<2, 4, 2>::LDS);
    else if (P.pick == 2) ok = allow(reinterpret_cast<const void*>(logits_kernel_for<T, 1, 4, 2>(group)), logits_cfg<1, 4, 2>::LDS);
    else if (P.pick == 4) ok = allow(reinterpret_cast<const void*>(logits_kernel_for<T, 1, 4, 2, true>(group)), logits_cfg<1, 4, 2>::LDS);
    else {
        ok = allow(reinterpret_cast<const void*>(SmallLogits<T>::get(P.nst, false)), kLsLds) &&
             allow(reinterpret_cast<const void*>(SmallLogits<T>::get(P.nst, true)), kLsLds);
    }
    return ok ? SALS_OK : SALS_ERR_HIP;
}

template <typename T>
sals_status launch_attend(const sals_ctx* c, const void* q, const int32_t* q_pos, const void* Kc,
                          const void* Vc, const void* W, const int32_t* idx, const int32_t* n_sel, void* out,
                          hipStream_t st, const QvCache* qv = nullptr, int ring = 0, int phases = kPhaseAll,
                          const StatsLink* link = nullptr, const FusedSelect* fs = nullptr)
{
    const sals_desc& d = c->d;
    const Layout& L = c->L;
    const int k_tot = d.top_k + d.n_sink + d.n_recent;
    float* logits = reinterpret_cast<float*>(c->ws + L.logits);
    const LogitsPlan P = c->plan;
    // tile statistics: written by this pass's logits kernel from record `part0` on, read as a whole by the value kernel
    float2* const stats_all = link ? link->stats : reinterpret_cast<float2*>(c->ws + L.stats);
    float2* const stats = stats_all + (link ? link->part0 : 0);
    const int stats_stride = link ? link->stride : P.n_parts;
    const float2* rope = reinterpret_cast<const float2*>(c->ws + L.rope);
    float* tpart = reinterpret_cast<float*>(c->ws + L.tpart);
    const int n_parts = P.n_parts;
    if (phases & kPhaseLogits) {
        sals_status rs = ensure_rope_table(c, st);
        if (rs == SALS_OK) rs = ensure_lds_attr<T>(c);
        if (rs != SALS_OK) return rs;
        // replicate the smaller operand across the XCDs' L2s: all of U_k, or the gathered rows
        const size_t a_bytes = (size_t)d.H_kv * kHeadDim * d.r, b_bytes = (size_t)d.B * k_tot * d.r;
        const int heads_fastest = a_bytes <= b_bytes ? 1 : 0;
        ProfScope ps(c, SALS_K_ATTEND_LOGITS, st);
#define SALS_LOGITS(HEADS, NTG, NB)                                                                              \
    do {                                                                                                     \
        typedef logits_cfg<HEADS, NTG, NB> LC;                                                               \
        auto kern = logits_kernel_for<T, HEADS, NTG, NB>(d.H_q / d.H_kv);                                    \
        hipLaunchKernelGGL(kern, dim3(n_parts * (d.H_kv / HEADS) * d.B), dim3(LC::NT), LC::LDS, st,          \
                           static_cast<const T*>(Kc), w_section<T>(c, W, 2), idx, n_sel,                     \
                           static_cast<const T*>(q), q_pos, rope, c->inv, logits, stats, d.B,                \
                           d.S_max, d.r, d.H_q, d.H_kv, k_tot, L.lk, n_parts, heads_fastest, d.rope_style,   \
                           1.0f / std::sqrt((float)d.d), ring, stats_stride, static_cast<float*>(nullptr), 1);       \
    } while (0)
        const int pick = P.pick;
        if (pick == 1) SALS_LOGITS(2, 4, 2);        // 2 heads x 256 tokens, 8 waves
        else if (pick == 2) SALS_LOGITS(1, 4, 2);   // 1 head  x 256 tokens
        else if (pick == 4) {  // four sequences' short selections per 256-token tile, latent axis in P.ksplit slices
            typedef logits_cfg<1, 4, 2> LC;
            auto kern = logits_kernel_for<T, 1, 4, 2, true>(d.H_q / d.H_kv);
            float* plogits = reinterpret_cast<float*>(c->ws + L.plogits);
            hipLaunchKernelGGL(kern, dim3(ceil_div(d.B, 4) * d.H_kv * P.ksplit), dim3(LC::NT), LC::LDS, st,
                               static_cast<const T*>(Kc), w_section<T>(c, W, 2), idx, n_sel, static_cast<const T*>(q), q_pos,
                               rope, c->inv, logits, stats, d.B, d.S_max, d.r, d.H_q, d.H_kv, k_tot, L.lk, 1, heads_fastest,
                               d.rope_style, 1.0f / std::sqrt((float)d.d), ring, stats_stride, plogits, P.ksplit);
            if (P.ksplit > 1) {
                if (launch_status() != SALS_OK) return SALS_ERR_HIP;
                hipLaunchKernelGGL(logits_finish_kernel, dim3(1, d.B * d.H_q), dim3(64), 0, st, plogits, P.ksplit, n_sel,
                                   logits, stats, d.B, d.H_q, L.lk, stats_stride);
            }
        }
        else {  // few tiles: 1 head x 64 tokens with the whole latent axis loaded ahead
            const int ksplit = P.ksplit, nst = P.nst;
            // fs: idx / n_sel are outputs of this launch (the kernel selects from fs->scores itself)
            const typename SmallLogits<T>::Fn kern = SmallLogits<T>::get(nst, fs != nullptr);
            const FusedSelect fsel = fs ? *fs : FusedSelect{nullptr, nullptr, 0, 0, 0};
            float* plogits = reinterpret_cast<float*>(c->ws + L.plogits);
            hipLaunchKernelGGL(kern, dim3(n_parts * d.H_kv * d.B * ksplit), dim3(kLsThreads), kLsLds, st,
                               idx, n_sel, w_section<T>(c, W, 2), d.B, d.H_kv, n_parts, heads_fastest, ksplit, k_tot,
                               d.r, d.H_q, static_cast<const T*>(Kc), static_cast<const T*>(q), q_pos, rope, c->inv,
                               logits, stats, d.S_max, L.lk, d.rope_style, 1.0f / std::sqrt((float)d.d), ring,
                               plogits, stats_stride, fsel);
            if (ksplit > 1) {
                if (launch_status() != SALS_OK) return SALS_ERR_HIP;
                hipLaunchKernelGGL(logits_finish_kernel, dim3(n_parts, d.B * d.H_q), dim3(64), 0, st, plogits, ksplit,
                                   n_sel, logits, stats, d.B, d.H_q, L.lk, stats_stride);
            }
        }
#undef SALS_LOGITS
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    }
    if (qv != nullptr) {
        ProfScope ps(c, SALS_K_ATTEND_QV, st);
        QvArgs a{};
        a.Vq = static_cast<const unsigned char*>(qv->codes); a.Vmeta = qv->meta; a.idx = idx; a.n_sel = n_sel;
        a.logits = logits; a.stats = stats_all; a.part = reinterpret_cast<float*>(c->ws + L.qv_part); a.out = out;
        a.n_parts = stats_stride; a.B = d.B; a.S_max = d.S_max; a.H = d.H_q; a.H_kv = d.H_kv; a.k_tot = k_tot; a.lk = L.lk;
        a.tok_per_wg = L.qv_tok_per_wg; a.n_tr = L.qv_ntr; a.part0 = 0; a.n_tr_all = L.qv_ntr;
        a.Vq_w = static_cast<const unsigned char*>(qv->codes_w); a.Vmeta_w = qv->meta_w; a.logits_w = qv->logits_w;
        a.n_lo = qv->n_lo; a.lk_w = qv->lk_w; a.ring = qv->ring;
        const bool win = qv->codes_w != nullptr;
        const dim3 grid(L.qv_ntr * d.H_kv * d.B);
        const int G = d.H_q / d.H_kv;
#define SALS_QV(BITS, GMAX)                                                                             \
    do {                                                                                                \
        if (win) hipLaunchKernelGGL((attend_qv_kernel<T, BITS, GMAX, true>), grid, dim3(256), 0, st, a); \
        else hipLaunchKernelGGL((attend_qv_kernel<T, BITS, GMAX, false>), grid, dim3(256), 0, st, a);   \
    } while (0)
#define SALS_QV_G(BITS)                                                                                 \
    do {                                                                                                \
        if (G <= 1) SALS_QV(BITS, 1); else if (G <= 2) SALS_QV(BITS, 2);                                \
        else if (G <= 4) SALS_QV(BITS, 4); else SALS_QV(BITS, 8);                                       \
    } while (0)
        if (qv->bits == 4) SALS_QV_G(4); else SALS_QV_G(2);
#undef SALS_QV_G
#undef SALS_QV
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
        if (L.qv_ntr > 1) {
            const size_t n4 = (size_t)d.B * d.H_q * kHeadDim / 4;
            hipLaunchKernelGGL((qv_merge_kernel<T>), dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st, a.part,
                               static_cast<T*>(out), L.qv_ntr, n4);
        }
        return launch_status();
    }
    if (phases & kPhaseValue) {
        ProfScope ps(c, SALS_K_ATTEND_PV, st);
        const int n_items = (d.r / kPvCols) * L.pv_ntr * d.B;
#define SALS_PV(NW, MB)                                                                                            \
    hipLaunchKernelGGL((attend_pv_kernel<T, NW, MB>), dim3(n_items), dim3(NW * 64), 0, st, idx, n_sel, stats_all, d.B, \
                       d.r, L.pv_ntr, stats_stride, L.pv_tok_per_wg, k_tot, d.H_q, L.lk, static_cast<const T*>(Vc),    \
                       logits, tpart, d.S_max, ring)
        if (d.H_q <= 32) { if (L.pv_waves == 8) SALS_PV(8, 1); else SALS_PV(4, 1); }
        else { if (L.pv_waves == 8) SALS_PV(8, 2); else SALS_PV(4, 2); }
#undef SALS_PV
    }
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    if (phases & kPhaseOut) {
        ProfScope ps(c, SALS_K_ATTEND_OUT, st);
        // steps of the latent axis per wave decide how many token ranges fit in one round of loads
        const int spw = ceil_div(d.r / (4 * elem<T>::vec), 4);
        const dim3 grid(d.H_kv, kHeadDim / 16, ceil_div(d.B * (d.H_q / d.H_kv), 16));
#define SALS_OUT(BATCH, RPR)                                                                                     \
    hipLaunchKernelGGL((attend_out_kernel<T, BATCH, RPR>), grid, dim3(256), 0, st, w_section<T>(c, W, 3), tpart, \
                       static_cast<T*>(out), d.B, d.r, d.H_q, d.H_kv, L.pv_ntr, static_cast<const T*>(nullptr),     \
                       static_cast<const float*>(nullptr), 0, 0)
        if (sizeof(T) == 2 && spw <= 4 && L.pv_ntr > 2) SALS_OUT(4, 4);
        else if (sizeof(T) == 2 && spw <= 5 && L.pv_ntr > 2) SALS_OUT(5, 3);
        else SALS_OUT(8, 2);
#undef SALS_OUT

    }
    return launch_status();
}

}  // namespace

extern "C" {

const char* sals_status_string(sals_status s)
{
    switch (s) {
        case SALS_OK: return "SALS_OK";
        case SALS_ERR_INVALID_ARG: return "SALS_ERR_INVALID_ARG";
        case SALS_ERR_UNSUPPORTED: return "SALS_ERR_UNSUPPORTED";
        case SALS_ERR_WORKSPACE: return "SALS_ERR_WORKSPACE";
        case SALS_ERR_HIP: return "SALS_ERR_HIP";
    }
    return "SALS_ERR_UNKNOWN";
}

sals_status sals_workspace_bytes(const sals_desc* desc, size_t* bytes)
{
    if (!bytes) return SALS_ERR_INVALID_ARG;
    sals_status s = validate(desc);
    if (s != SALS_OK) return s;
    *bytes = make_layout(*desc).total;
    return SALS_OK;
}

sals_status sals_packed_weight_bytes(const sals_desc* desc, size_t* bytes)
{
    if (!bytes) return SALS_ERR_INVALID_ARG;
    sals_status s = validate(desc);
    if (s != SALS_OK) return s;
    *bytes = align_up(4 * make_layout(*desc).w_section * (desc->dtype == SALS_BF16 ? 2 : 4));
    return SALS_OK;
}

sals_status sals_create(const sals_desc* desc, void* d_workspace, size_t workspace_bytes, sals_ctx** out)
{
    if (!out) return SALS_ERR_INVALID_ARG;
    *out = nullptr;
    sals_status s = validate(desc);
    if (s != SALS_OK) return s;
    Layout L = make_layout(*desc);
    if (!d_workspace || (reinterpret_cast<uintptr_t>(d_workspace) % kAlign) != 0 || workspace_bytes < L.total)
        return SALS_ERR_WORKSPACE;
    sals_ctx* c = new (std::nothrow) sals_ctx;
    if (!c) return SALS_ERR_INVALID_ARG;
    c->d = *desc;
    c->L = L;
    c->ws = static_cast<unsigned char*>(d_workspace);
    c->ws_bytes = workspace_bytes;
    for (int p = 0; p < kPairs; ++p)
        c->inv.f[p] = std::pow((double)desc->rope_theta, -2.0 * (double)p / (double)desc->d);
    const bool bf = desc->dtype == SALS_BF16;
    c->plan = bf ? plan_logits<bf16_t>(c->d) : plan_logits<float>(c->d);
    c->score_rows = plan_score_rows(c->d);
    if (const char* e = std::getenv("SALS_TUNE_SCORE_STREAM")) c->score_stream = std::atoi(e) != 0;  // tuning aid
    if (const char* e = std::getenv("SALS_TUNE_FUSE_SELECT")) c->fuse_select = std::atoi(e) != 0;  // tuning aid
    *out = c;
    return SALS_OK;
}

sals_status sals_prepare(sals_ctx* ctx, void* hip_stream)
{
    if (!ctx) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (ctx->rope_state != 2) {
        if (ctx->rope_state == 0) {
            sals_status s = enqueue_rope_table(ctx, st);
            if (s != SALS_OK) return s;
        }
        if (hipEventSynchronize(ctx->rope_ev) != hipSuccess) return SALS_ERR_HIP;
        ctx->rope_state = 2;
    }
    return ctx->d.dtype == SALS_BF16 ? ensure_lds_attr<bf16_t>(ctx) : ensure_lds_attr<float>(ctx);
}

void sals_destroy(sals_ctx* ctx)
{
    if (!ctx) return;
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    if (ctx->rope_ev) (void)hipEventDestroy(ctx->rope_ev);
    delete ctx;
}

sals_status sals_pack_weights(sals_ctx* ctx, const void* Uk, const void* Uv, void* W, void* hip_stream)
{
    if (!ctx || bad(Uk) || bad(Uv) || !W || (reinterpret_cast<uintptr_t>(W) % kAlign) != 0)
        return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const sals_desc& d = ctx->d;
    const size_t n = ctx->L.w_section;
    dim3 grid((unsigned)std::min<size_t>(2048, (n + 255) / 256), 4);
    if (d.dtype == SALS_BF16)
        hipLaunchKernelGGL((pack_weights_kernel<bf16_t>), grid, dim3(256), 0, st, static_cast<const bf16_t*>(Uk),
                           static_cast<const bf16_t*>(Uv), static_cast<bf16_t*>(W), n, d.H_kv * d.d, d.r,
                           d.rope_style);
    else
        hipLaunchKernelGGL((pack_weights_kernel<float>), grid, dim3(256), 0, st, static_cast<const float*>(Uk),
                           static_cast<const float*>(Uv), static_cast<float*>(W), n, d.H_kv * d.d, d.r,
                           d.rope_style);
    return launch_status();
}

const char* sals_kernel_name(int kernel)
{
    return (kernel >= 0 && kernel < SALS_N_KERNELS) ? kKernelNames[kernel] : "unknown";
}

sals_status sals_profile_enable(sals_ctx* ctx, int on)
{
    if (!ctx) return SALS_ERR_INVALID_ARG;
    ctx->profiling = on != 0;
    return SALS_OK;
}

sals_status sals_profile_collect(sals_ctx* ctx, double* total_ms, int32_t* launches)
{
    if (!ctx || !total_ms || !launches) return SALS_ERR_INVALID_ARG;
    for (int k = 0; k < SALS_N_KERNELS; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
    sals_status st = SALS_OK;
    for (auto& r : ctx->prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
            st = SALS_ERR_HIP;
        total_ms[r.kernel] += ms;
        launches[r.kernel] += 1;
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    ctx->prof.clear();
    return st;
}

sals_status sals_compress_append(sals_ctx* ctx, const void* k_new, const void* v_new, const void* W, void* Kc,
                                 void* Vc, int32_t* seq_len, void* hip_stream)
{
    if (!ctx || bad(k_new) || bad(v_new) || bad(W) || bad(Kc) || bad(Vc) || !seq_len) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return ctx->d.dtype == SALS_BF16
               ? launch_project<bf16_t, false>(ctx, W, k_new, v_new, Kc, Vc, seq_len, st)
               : launch_project<float, false>(ctx, W, k_new, v_new, Kc, Vc, seq_len, st);
}

sals_status sals_compress_prefill(sals_ctx* ctx, const void* k_new, const void* v_new, const void* W, void* Kc,
                                  void* Vc, int32_t* seq_len, const int32_t* n_new, int32_t n_tok, void* hip_stream)
{
    if (!ctx || bad(k_new) || bad(v_new) || bad(W) || bad(Kc) || bad(Vc) || !seq_len) return SALS_ERR_INVALID_ARG;
    if (n_tok < 1 || n_tok > ctx->d.S_max) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const sals_desc& d = ctx->d;
    const bool bf = d.dtype == SALS_BF16;
    PrefillArgs a{};
    a.X[0] = k_new; a.X[1] = v_new;
    a.cache[0] = Kc; a.cache[1] = Vc;
    a.seq_len = seq_len; a.n_new = n_new;
    a.n_tok = n_tok; a.D = d.H_kv * d.d; a.r = d.r; a.S_max = d.S_max; a.B = d.B; a.nproj = 2;
    for (int p = 0; p < 2; ++p)
        a.UT[p] = bf ? static_cast<const void*>(w_section<bf16_t>(ctx, W, p)) : static_cast<const void*>(w_section<float>(ctx, W, p));
    const int nl = d.r % 128 == 0 ? 128 : 64;
    // 256-token tiles unless they would fill less than three quarters of the chip's 512 workgroup slots
    const int tok = (nl == 128 && (long long)ceil_div(n_tok, 256) * (d.r / nl) * d.B * 2 < 384) ? 128 : 256;
    const dim3 grid(ceil_div(n_tok, tok), d.r / nl, d.B * 2);
    const size_t lds = prefill_lds_bytes(tok, nl);
#define SALS_PREFILL(T, TOKT, NLT)                                                                                \
    do {                                                                                                          \
        auto kern = prefill_compress_kernel<T, TOKT, NLT>;                                                        \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,  \
                                (int)lds) != hipSuccess)                                                          \
            return SALS_ERR_HIP;                                                                                  \
        hipLaunchKernelGGL(kern, grid, dim3(kPfThreads), lds, st, a);                                             \
    } while (0)
#define SALS_PREFILL_T(T)                                                                                         \
    do {                                                                                                          \
        if (nl == 64) SALS_PREFILL(T, 256, 64); else if (tok == 128) SALS_PREFILL(T, 128, 128);                   \
        else SALS_PREFILL(T, 256, 128);                                                                           \
    } while (0)
    {
        ProfScope ps(ctx, SALS_K_PREFILL, st);
        if (bf) SALS_PREFILL_T(bf16_t); else SALS_PREFILL_T(float);
    }
#undef SALS_PREFILL_T
#undef SALS_PREFILL
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    hipLaunchKernelGGL(advance_seq_len_kernel, dim3(ceil_div(d.B, 128)), dim3(128), 0, st, seq_len, n_new, n_tok, d.B, d.S_max);
    return launch_status();
}

sals_status sals_latent_scores(sals_ctx* ctx, const void* q, const void* W, const void* Kc,
                               const int32_t* seq_len, float* scores, void* hip_stream)
{
    if (!ctx || bad(q) || bad(W) || bad(Kc) || !seq_len || bad(scores)) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    sals_status s = ctx->d.dtype == SALS_BF16
                        ? launch_project<bf16_t, true>(ctx, W, q, nullptr, nullptr, nullptr, nullptr, st)
                        : launch_project<float, true>(ctx, W, q, nullptr, nullptr, nullptr, nullptr, st);
    if (s != SALS_OK) return s;
    return ctx->d.dtype == SALS_BF16 ? launch_scores<bf16_t>(ctx, Kc, seq_len, scores, st)
                                     : launch_scores<float>(ctx, Kc, seq_len, scores, st);
}

namespace {
// The score stage inside a decode step: as sals_latent_scores, and for sequences long enough for the selection
// chain the score kernel also leaves its workgroups' key ranges for it.
sals_status step_scores(sals_ctx* ctx, const void* q, const void* W, const void* Kc, const int32_t* seq_len,
                        float* scores, hipStream_t st)
{
    if (!ctx || bad(q) || bad(W) || bad(Kc) || !seq_len || bad(scores)) return SALS_ERR_INVALID_ARG;
    sals_status s = ctx->d.dtype == SALS_BF16
                        ? launch_project<bf16_t, true>(ctx, W, q, nullptr, nullptr, nullptr, nullptr, st)
                        : launch_project<float, true>(ctx, W, q, nullptr, nullptr, nullptr, nullptr, st);
    if (s != SALS_OK) return s;
    uint2* wg_range = ctx->L.tm_chunks > 0 ? reinterpret_cast<uint2*>(ctx->ws + ctx->L.tm_srange) : nullptr;
    return ctx->d.dtype == SALS_BF16 ? launch_scores<bf16_t>(ctx, Kc, seq_len, scores, st, wg_range)
                                     : launch_scores<float>(ctx, Kc, seq_len, scores, st, wg_range);
}
}  // namespace

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];  // per device: address of `scratch` there (nullptr: not looked up yet)

// address of the current device's copy of `scratch`; looked up once per device, with that device current
sals_status scratch_on_current_device(unsigned char** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SALS_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SALS_ERR_HIP;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return SALS_OK;
}
}  // namespace

sals_status sals_latent_scores_noalloc(const sals_desc* desc, const void* q, const void* W, const void* Kc,
                                       const int32_t* seq_len, float* scores, void* hip_stream)
{
    sals_status s = validate(desc);
    if (s != SALS_OK) return s;
    if (bad(q) || bad(W) || bad(Kc) || !seq_len || bad(scores)) return SALS_ERR_INVALID_ARG;
    // a context on the stack whose "workspace" is the static array: these two launches only use the slot of
    // the partial sums of q~, placed at offset 0
    sals_ctx tmp;
    tmp.d = *desc;
    tmp.L = make_layout(*desc);
    tmp.L.qt = 0;
    tmp.score_rows = plan_score_rows(*desc);
    const size_t need = (size_t)tmp.L.proj_np * desc->B * desc->r * 4;
    if (need > (size_t)SALS_NOALLOC_SCRATCH_BYTES) return SALS_ERR_WORKSPACE;
    s = scratch_on_current_device(&tmp.ws);
    if (s != SALS_OK) return s;
    tmp.ws_bytes = SALS_NOALLOC_SCRATCH_BYTES;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    s = desc->dtype == SALS_BF16 ? launch_project<bf16_t, true>(&tmp, W, q, nullptr, nullptr, nullptr, nullptr, st)
                                 : launch_project<float, true>(&tmp, W, q, nullptr, nullptr, nullptr, nullptr, st);
    if (s != SALS_OK) return s;
    return desc->dtype == SALS_BF16 ? launch_scores<bf16_t>(&tmp, Kc, seq_len, scores, st)
                                    : launch_scores<float>(&tmp, Kc, seq_len, scores, st);
}

sals_status sals_topk_select(sals_ctx* ctx, const float* scores, const int32_t* seq_len, int32_t* idx,
                             int32_t* n_sel, void* hip_stream)
{
    if (!ctx || bad(scores) || !seq_len || !idx || !n_sel) return SALS_ERR_INVALID_ARG;
    return launch_topk(ctx, scores, seq_len, idx, n_sel, static_cast<hipStream_t>(hip_stream));
}

sals_status sals_sparse_attend(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* Kc,
                               const void* Vc, const void* W, const int32_t* idx, const int32_t* n_sel,
                               void* out, void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(Kc) || bad(Vc) || bad(W) || !idx || !n_sel || bad(out))
        return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return ctx->d.dtype == SALS_BF16 ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, Vc, W, idx, n_sel, out, st)
                                     : launch_attend<float>(ctx, q, q_pos, Kc, Vc, W, idx, n_sel, out, st);
}

sals_status sals_decode_step(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* Kc,
                             const void* Vc, const void* W, const int32_t* seq_len, void* out, float* scores,
                             int32_t* idx, int32_t* n_sel, void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(Kc) || bad(Vc) || bad(W) || !seq_len || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (scores && !aligned16(scores)) return SALS_ERR_INVALID_ARG;
    if (!scores) scores = reinterpret_cast<float*>(ctx->ws + ctx->L.scores);
    if (!idx) idx = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.idx);
    if (!n_sel) n_sel = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.n_sel);
    sals_status s = step_scores(ctx, q, W, Kc, seq_len, scores, static_cast<hipStream_t>(hip_stream));
    if (s != SALS_OK) return s;
    if (fused_selection(ctx)) {  // one launch fewer: the logits kernel selects and leaves idx / n_sel behind
        if (bad(Vc)) return SALS_ERR_INVALID_ARG;
        const FusedSelect fs{scores, seq_len, ctx->d.top_k, ctx->d.n_sink, ctx->d.n_recent};
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        return ctx->d.dtype == SALS_BF16
                   ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, Vc, W, idx, n_sel, out, st, nullptr, 0, kPhaseAll, nullptr, &fs)
                   : launch_attend<float>(ctx, q, q_pos, Kc, Vc, W, idx, n_sel, out, st, nullptr, 0, kPhaseAll, nullptr, &fs);
    }
    s = launch_topk(ctx, scores, seq_len, idx, n_sel, static_cast<hipStream_t>(hip_stream),
                    WindowLists{nullptr, nullptr, nullptr, 0}, ctx->L.tm_chunks > 0);
    if (s != SALS_OK) return s;
    return sals_sparse_attend(ctx, q, q_pos, Kc, Vc, W, idx, n_sel, out, hip_stream);
}

sals_status sals_qv_row_bytes(const sals_desc* desc, int bits, size_t* code_bytes, size_t* meta_bytes)
{
    if (!code_bytes || !meta_bytes) return SALS_ERR_INVALID_ARG;
    sals_status s = validate(desc);
    if (s != SALS_OK) return s;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    const size_t D = (size_t)desc->H_kv * desc->d;
    *code_bytes = D * bits / 8;
    *meta_bytes = D / kQvGroup * 2 * (desc->dtype == SALS_BF16 ? 2 : 4);
    return SALS_OK;
}

sals_status sals_compress_append_qv(sals_ctx* ctx, const void* k_new, const void* v_new, const void* W, void* Kc,
                                    void* Vq, void* Vmeta, int bits, int32_t* seq_len, void* hip_stream)
{
    if (!ctx || bad(k_new) || bad(v_new) || bad(W) || bad(Kc) || bad(Vq) || bad(Vmeta) || !seq_len)
        return SALS_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const sals_desc& d = ctx->d;
    const bool bf = d.dtype == SALS_BF16;
    sals_status s = bf ? launch_project<bf16_t, false>(ctx, W, k_new, nullptr, Kc, nullptr, seq_len, st, false)
                       : launch_project<float, false>(ctx, W, k_new, nullptr, Kc, nullptr, seq_len, st, false);
    if (s != SALS_OK) return s;
    const int D = d.H_kv * d.d;
    const dim3 grid(ceil_div(D / kQvGroup, 8), d.B);
    unsigned char* codes = static_cast<unsigned char*>(Vq);
#define SALS_QUANT(T, BITS)                                                                                   \
    hipLaunchKernelGGL((qv_quantize_kernel<T, BITS>), grid, dim3(256), 0, st, static_cast<const T*>(v_new), codes, \
                       static_cast<T*>(Vmeta), seq_len, D, d.S_max, 0)
    if (bf) { if (bits == 4) SALS_QUANT(bf16_t, 4); else SALS_QUANT(bf16_t, 2); }
    else    { if (bits == 4) SALS_QUANT(float, 4); else SALS_QUANT(float, 2); }
#undef SALS_QUANT
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    hipLaunchKernelGGL(bump_seq_len_kernel, dim3(ceil_div(d.B, 128)), dim3(128), 0, st, seq_len, d.B, d.S_max);
    return launch_status();
}

sals_status sals_sparse_attend_qv(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* Kc,
                                  const void* Vq, const void* Vmeta, int bits, const void* W, const int32_t* idx,
                                  const int32_t* n_sel, void* out, void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(Kc) || bad(Vq) || bad(Vmeta) || bad(W) || !idx || !n_sel || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const QvCache qv{Vq, Vmeta, bits};
    return ctx->d.dtype == SALS_BF16 ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv)
                                     : launch_attend<float>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv);
}

sals_status sals_decode_step_qv(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* Kc,
                                const void* Vq, const void* Vmeta, int bits, const void* W, const int32_t* seq_len,
                                void* out, float* scores, int32_t* idx, int32_t* n_sel, void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(Kc) || bad(Vq) || bad(Vmeta) || bad(W) || !seq_len || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    if (scores && !aligned16(scores)) return SALS_ERR_INVALID_ARG;
    if (!scores) scores = reinterpret_cast<float*>(ctx->ws + ctx->L.scores);
    if (!idx) idx = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.idx);
    if (!n_sel) n_sel = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.n_sel);
    sals_status s = step_scores(ctx, q, W, Kc, seq_len, scores, static_cast<hipStream_t>(hip_stream));
    if (s != SALS_OK) return s;
    if (fused_selection(ctx)) {  // one launch fewer: the logits kernel selects and leaves idx / n_sel behind
        const FusedSelect fs{scores, seq_len, ctx->d.top_k, ctx->d.n_sink, ctx->d.n_recent};
        const QvCache qv{Vq, Vmeta, bits};
        hipStream_t st = static_cast<hipStream_t>(hip_stream);
        return ctx->d.dtype == SALS_BF16
                   ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv, 0, kPhaseAll, nullptr, &fs)
                   : launch_attend<float>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv, 0, kPhaseAll, nullptr, &fs);
    }
    s = launch_topk(ctx, scores, seq_len, idx, n_sel, static_cast<hipStream_t>(hip_stream),
                    WindowLists{nullptr, nullptr, nullptr, 0}, ctx->L.tm_chunks > 0);
    if (s != SALS_OK) return s;
    return sals_sparse_attend_qv(ctx, q, q_pos, Kc, Vq, Vmeta, bits, W, idx, n_sel, out, hip_stream);
}

sals_status sals_dense_attend(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* K, const void* V,
                              const int32_t* seq_len, void* out, void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(K) || bad(V) || !seq_len || bad(out)) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    return ctx->d.dtype == SALS_BF16 ? launch_dense<bf16_t>(ctx, q, q_pos, K, V, seq_len, out, st)
                                     : launch_dense<float>(ctx, q, q_pos, K, V, seq_len, out, st);
}

// ---- recent window (second, higher-rank ring cache) ------------------------------------------------

namespace {
// `win` must describe the same model and batch as `ctx`, at another rank, and select exactly the recent tokens
sals_status window_pair_ok(const sals_ctx* ctx, const sals_ctx* win)
{
    if (!ctx || !win || ctx == win) return SALS_ERR_INVALID_ARG;
    const sals_desc &a = ctx->d, &b = win->d;
    if (a.B != b.B || a.S_max != b.S_max || a.H_q != b.H_q || a.H_kv != b.H_kv || a.d != b.d ||
        a.rope_theta != b.rope_theta || a.rope_style != b.rope_style || a.dtype != b.dtype)
        return SALS_ERR_INVALID_ARG;
    if (b.n_sink != 0 || b.n_recent != 0 || a.n_recent < 1 || b.top_k != a.n_recent) return SALS_ERR_INVALID_ARG;
    return SALS_OK;
}
}  // namespace

sals_status sals_window_append(sals_ctx* win, const void* k_new, const void* v_new, const void* W_hi, void* Kw,
                               void* Vw, const int32_t* seq_len, void* hip_stream)
{
    if (!win || bad(k_new) || bad(v_new) || bad(W_hi) || bad(Kw) || bad(Vw) || !seq_len) return SALS_ERR_INVALID_ARG;
    if (win->d.n_sink != 0 || win->d.n_recent != 0) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int32_t* sl = const_cast<int32_t*>(seq_len);  // read only: no length is advanced here
    const int ring = win->d.top_k;
    return win->d.dtype == SALS_BF16
               ? launch_project<bf16_t, false>(win, W_hi, k_new, v_new, Kw, Vw, sl, st, false, ring)
               : launch_project<float, false>(win, W_hi, k_new, v_new, Kw, Vw, sl, st, false, ring);
}

namespace {
// where the two passes' token lists live: the window's list and count in the window context's workspace, the
// low-rank pass's count in the main context's
WindowLists window_lists(sals_ctx* ctx, sals_ctx* win)
{
    return WindowLists{reinterpret_cast<int32_t*>(win->ws + win->L.idx), reinterpret_cast<int32_t*>(ctx->ws + ctx->L.n_lo),
                       reinterpret_cast<int32_t*>(win->ws + win->L.n_sel), win->d.top_k};
}

// lists_ready: the selection kernel has already written the two passes' lists (decode step); otherwise they are
// split off the caller's selection here
sals_status window_attend(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos, const void* Kc,
                          const void* Vc, const void* W, const void* Kw, const void* Vw, const void* W_hi,
                          const int32_t* idx, const int32_t* n_sel, void* out, hipStream_t st, bool lists_ready)
{
    sals_status s = SALS_OK;
    const sals_desc& d = ctx->d;
    const int k_tot = d.top_k + d.n_sink + d.n_recent, w = win->d.top_k;
    const WindowLists wl = window_lists(ctx, win);
    int32_t* idx_hi = wl.idx_hi;
    int32_t* n_hi = wl.n_hi;
    int32_t* n_lo = wl.n_lo;
    if (!lists_ready) {
        hipLaunchKernelGGL(window_split_kernel, dim3(d.B), dim3(256), 0, st, idx, n_sel, k_tot, w, idx_hi, n_lo, n_hi);
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    }
    // One softmax over both caches: the two logits passes leave their tile statistics side by side in the main
    // context's array, each value pass normalises with the statistics of all tiles, and one output projection adds
    // both passes' value sums through their projectors.
    const bool bf = d.dtype == SALS_BF16;
    const LogitsPlan p_lo = ctx->plan, p_hi = win->plan;
    if (p_lo.n_parts + p_hi.n_parts > ctx->L.max_parts) return SALS_ERR_UNSUPPORTED;
    float2* shared = reinterpret_cast<float2*>(ctx->ws + ctx->L.stats);
    const StatsLink l_lo{shared, p_lo.n_parts + p_hi.n_parts, 0}, l_hi{shared, p_lo.n_parts + p_hi.n_parts, p_lo.n_parts};
    for (int phase : {(int)kPhaseLogits, (int)kPhaseValue}) {
        s = bf ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, Vc, W, idx, n_lo, nullptr, st, nullptr, 0, phase, &l_lo)
               : launch_attend<float>(ctx, q, q_pos, Kc, Vc, W, idx, n_lo, nullptr, st, nullptr, 0, phase, &l_lo);
        if (s != SALS_OK) return s;
        s = bf ? launch_attend<bf16_t>(win, q, q_pos, Kw, Vw, W_hi, idx_hi, n_hi, nullptr, st, nullptr, w, phase, &l_hi)
               : launch_attend<float>(win, q, q_pos, Kw, Vw, W_hi, idx_hi, n_hi, nullptr, st, nullptr, w, phase, &l_hi);
        if (s != SALS_OK) return s;
    }
    {
        ProfScope ps(ctx, SALS_K_ATTEND_OUT, st);
        const dim3 grid(d.H_kv, kHeadDim / 16, ceil_div(d.B * (d.H_q / d.H_kv), 16));
        const float* t_lo = reinterpret_cast<const float*>(ctx->ws + ctx->L.tpart);
        const float* t_hi = reinterpret_cast<const float*>(win->ws + win->L.tpart);
        if (bf)
            hipLaunchKernelGGL((attend_out_kernel<bf16_t, 8, 2>), grid, dim3(256), 0, st, w_section<bf16_t>(ctx, W, 3), t_lo,
                               static_cast<bf16_t*>(out), d.B, d.r, d.H_q, d.H_kv, ctx->L.pv_ntr,
                               w_section<bf16_t>(win, W_hi, 3), t_hi, win->d.r, win->L.pv_ntr);
        else
            hipLaunchKernelGGL((attend_out_kernel<float, 8, 2>), grid, dim3(256), 0, st, w_section<float>(ctx, W, 3), t_lo,
                               static_cast<float*>(out), d.B, d.r, d.H_q, d.H_kv, ctx->L.pv_ntr,
                               w_section<float>(win, W_hi, 3), t_hi, win->d.r, win->L.pv_ntr);
    }
    return launch_status();
}
}  // namespace

sals_status sals_sparse_attend_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                      const void* Kc, const void* Vc, const void* W, const void* Kw,
                                      const void* Vw, const void* W_hi, const int32_t* idx, const int32_t* n_sel,
                                      void* out, void* hip_stream)
{
    sals_status s = window_pair_ok(ctx, win);
    if (s != SALS_OK) return s;
    if (bad(q) || !q_pos || bad(Kc) || bad(Vc) || bad(W) || bad(Kw) || bad(Vw) || bad(W_hi) || !idx || !n_sel ||
        bad(out))
        return SALS_ERR_INVALID_ARG;
    return window_attend(ctx, win, q, q_pos, Kc, Vc, W, Kw, Vw, W_hi, idx, n_sel, out, static_cast<hipStream_t>(hip_stream),
                         false);
}

sals_status sals_decode_step_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                    const void* Kc, const void* Vc, const void* W, const void* Kw, const void* Vw,
                                    const void* W_hi, const int32_t* seq_len, void* out, float* scores,
                                    int32_t* idx, int32_t* n_sel, void* hip_stream)
{
    sals_status s = window_pair_ok(ctx, win);
    if (s != SALS_OK) return s;
    if (bad(q) || !q_pos || bad(Kc) || bad(Vc) || bad(W) || bad(Kw) || bad(Vw) || bad(W_hi) || !seq_len || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (scores && !aligned16(scores)) return SALS_ERR_INVALID_ARG;
    if (!scores) scores = reinterpret_cast<float*>(ctx->ws + ctx->L.scores);
    if (!idx) idx = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.idx);
    if (!n_sel) n_sel = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.n_sel);
    s = step_scores(ctx, q, W, Kc, seq_len, scores, static_cast<hipStream_t>(hip_stream));
    if (s != SALS_OK) return s;
    // the selection kernel also writes the two passes' token lists (they follow from the sequence lengths)
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    s = launch_topk(ctx, scores, seq_len, idx, n_sel, st, window_lists(ctx, win), ctx->L.tm_chunks > 0);
    if (s != SALS_OK) return s;
    return window_attend(ctx, win, q, q_pos, Kc, Vc, W, Kw, Vw, W_hi, idx, n_sel, out, st, true);
}

// ---- recent window of the quantised value path: keys in the rank-r_hi ring, values as 8-bit codes ----

sals_status sals_window_append_qv(sals_ctx* win, const void* k_new, const void* v_new, const void* W_hi, void* Kw,
                                  void* Vqw, void* Vmeta_w, const int32_t* seq_len, void* hip_stream)
{
    if (!win || bad(k_new) || bad(v_new) || bad(W_hi) || bad(Kw) || bad(Vqw) || bad(Vmeta_w) || !seq_len)
        return SALS_ERR_INVALID_ARG;
    if (win->d.n_sink != 0 || win->d.n_recent != 0) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int32_t* sl = const_cast<int32_t*>(seq_len);  // read only: no length is advanced here
    const sals_desc& d = win->d;
    const int ring = d.top_k;
    const bool bf = d.dtype == SALS_BF16;
    sals_status s = bf ? launch_project<bf16_t, false>(win, W_hi, k_new, nullptr, Kw, nullptr, sl, st, false, ring)
                       : launch_project<float, false>(win, W_hi, k_new, nullptr, Kw, nullptr, sl, st, false, ring);
    if (s != SALS_OK) return s;
    const int D = d.H_kv * d.d;
    const dim3 grid(ceil_div(D / kQvGroup, 8), d.B);
    if (bf)
        hipLaunchKernelGGL((qv_quantize_kernel<bf16_t, 8>), grid, dim3(256), 0, st, static_cast<const bf16_t*>(v_new),
                           static_cast<unsigned char*>(Vqw), static_cast<bf16_t*>(Vmeta_w), seq_len, D, d.S_max, ring);
    else
        hipLaunchKernelGGL((qv_quantize_kernel<float, 8>), grid, dim3(256), 0, st, static_cast<const float*>(v_new),
                           static_cast<unsigned char*>(Vqw), static_cast<float*>(Vmeta_w), seq_len, D, d.S_max, ring);
    return launch_status();
}

namespace {
sals_status window_attend_qv(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos, const void* Kc,
                             const void* Vq, const void* Vmeta, int bits, const void* W, const void* Kw, const void* Vqw,
                             const void* Vmeta_w, const void* W_hi, const int32_t* idx, const int32_t* n_sel, void* out,
                             hipStream_t st, bool lists_ready)
{
    const sals_desc& d = ctx->d;
    const int k_tot = d.top_k + d.n_sink + d.n_recent, w = win->d.top_k;
    const WindowLists wl = window_lists(ctx, win);
    if (!lists_ready) {
        hipLaunchKernelGGL(window_split_kernel, dim3(d.B), dim3(256), 0, st, idx, n_sel, k_tot, w, wl.idx_hi, wl.n_lo, wl.n_hi);
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    }
    // two logits passes (low-rank cache, ring) with their tile statistics side by side, then one pass over the values
    // of the whole selection: the tokens before the window from the low-bit cache, the window's from its 8-bit ring
    const bool bf = d.dtype == SALS_BF16;
    const LogitsPlan p_lo = ctx->plan, p_hi = win->plan;
    if (p_lo.n_parts + p_hi.n_parts > ctx->L.max_parts) return SALS_ERR_UNSUPPORTED;
    float2* shared = reinterpret_cast<float2*>(ctx->ws + ctx->L.stats);
    const int n_all = p_lo.n_parts + p_hi.n_parts;
    const StatsLink l_lo{shared, n_all, 0}, l_hi{shared, n_all, p_lo.n_parts};
    sals_status s = bf ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, nullptr, W, idx, wl.n_lo, nullptr, st, nullptr, 0, kPhaseLogits, &l_lo)
                       : launch_attend<float>(ctx, q, q_pos, Kc, nullptr, W, idx, wl.n_lo, nullptr, st, nullptr, 0, kPhaseLogits, &l_lo);
    if (s != SALS_OK) return s;
    s = bf ? launch_attend<bf16_t>(win, q, q_pos, Kw, nullptr, W_hi, wl.idx_hi, wl.n_hi, nullptr, st, nullptr, w, kPhaseLogits, &l_hi)
           : launch_attend<float>(win, q, q_pos, Kw, nullptr, W_hi, wl.idx_hi, wl.n_hi, nullptr, st, nullptr, w, kPhaseLogits, &l_hi);
    if (s != SALS_OK) return s;
    QvCache qv{Vq, Vmeta, bits};
    qv.codes_w = Vqw; qv.meta_w = Vmeta_w;
    qv.logits_w = reinterpret_cast<const float*>(win->ws + win->L.logits);
    qv.n_lo = wl.n_lo; qv.lk_w = win->L.lk; qv.ring = w;
    return bf ? launch_attend<bf16_t>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv, 0, 0, &l_lo)
              : launch_attend<float>(ctx, q, q_pos, Kc, nullptr, W, idx, n_sel, out, st, &qv, 0, 0, &l_lo);
}
}  // namespace

sals_status sals_sparse_attend_qv_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                         const void* Kc, const void* Vq, const void* Vmeta, int bits, const void* W,
                                         const void* Kw, const void* Vqw, const void* Vmeta_w, const void* W_hi,
                                         const int32_t* idx, const int32_t* n_sel, void* out, void* hip_stream)
{
    sals_status s = window_pair_ok(ctx, win);
    if (s != SALS_OK) return s;
    if (bad(q) || !q_pos || bad(Kc) || bad(Vq) || bad(Vmeta) || bad(W) || bad(Kw) || bad(Vqw) || bad(Vmeta_w) || bad(W_hi) ||
        !idx || !n_sel || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    return window_attend_qv(ctx, win, q, q_pos, Kc, Vq, Vmeta, bits, W, Kw, Vqw, Vmeta_w, W_hi, idx, n_sel, out,
                            static_cast<hipStream_t>(hip_stream), false);
}

sals_status sals_decode_step_qv_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                       const void* Kc, const void* Vq, const void* Vmeta, int bits, const void* W,
                                       const void* Kw, const void* Vqw, const void* Vmeta_w, const void* W_hi,
                                       const int32_t* seq_len, void* out, float* scores, int32_t* idx, int32_t* n_sel,
                                       void* hip_stream)
{
    sals_status s = window_pair_ok(ctx, win);
    if (s != SALS_OK) return s;
    if (bad(q) || !q_pos || bad(Kc) || bad(Vq) || bad(Vmeta) || bad(W) || bad(Kw) || bad(Vqw) || bad(Vmeta_w) || bad(W_hi) ||
        !seq_len || bad(out))
        return SALS_ERR_INVALID_ARG;
    if (bits != 2 && bits != 4) return SALS_ERR_UNSUPPORTED;
    if (scores && !aligned16(scores)) return SALS_ERR_INVALID_ARG;
    if (!scores) scores = reinterpret_cast<float*>(ctx->ws + ctx->L.scores);
    if (!idx) idx = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.idx);
    if (!n_sel) n_sel = reinterpret_cast<int32_t*>(ctx->ws + ctx->L.n_sel);
    s = step_scores(ctx, q, W, Kc, seq_len, scores, static_cast<hipStream_t>(hip_stream));
    if (s != SALS_OK) return s;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    s = launch_topk(ctx, scores, seq_len, idx, n_sel, st, window_lists(ctx, win), ctx->L.tm_chunks > 0);
    if (s != SALS_OK) return s;
    return window_attend_qv(ctx, win, q, q_pos, Kc, Vq, Vmeta, bits, W, Kw, Vqw, Vmeta_w, W_hi, idx, n_sel, out, st, true);
}

// ---- overlap score ----------------------------------------------------------------------------------

sals_status sals_overlap_score(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* K,
                               const int32_t* seq_len, const int32_t* idx, const int32_t* n_sel, float* os,
                               void* hip_stream)
{
    if (!ctx || bad(q) || !q_pos || bad(K) || !seq_len || !idx || !n_sel || !os) return SALS_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const sals_desc& d = ctx->d;
    const Layout& L = ctx->L;
    if (ensure_rope_table(ctx, st) != SALS_OK) return SALS_ERR_HIP;
    const int k_tot = d.top_k + d.n_sink + d.n_recent;
    float2* part = reinterpret_cast<float2*>(ctx->ws + L.dn_part);  // the dense baseline's partials: larger
    const float2* rope = reinterpret_cast<const float2*>(ctx->ws + L.rope);
    const int G = d.H_q / d.H_kv;
    const dim3 grid(L.dn_chunks, d.H_kv, d.B);
    const float scale = 1.0f / std::sqrt((float)d.d);
#define SALS_OS(T, GMAX)                                                                                          \
    hipLaunchKernelGGL((overlap_stats_kernel<T, GMAX>), grid, dim3(256), 0, st, static_cast<const T*>(q), q_pos,     \
                       static_cast<const T*>(K), seq_len, idx, n_sel, rope, ctx->inv, part, d.S_max, d.H_q, d.H_kv, \
                       k_tot, L.dn_chunks, L.dn_tok, ceil_div(k_tot, L.dn_chunks), d.rope_style, scale)
#define SALS_OS_G(T)                                                                                              \
    do {                                                                                                          \
        if (G <= 1) SALS_OS(T, 1); else if (G <= 2) SALS_OS(T, 2); else if (G <= 4) SALS_OS(T, 4); else SALS_OS(T, 8); \
    } while (0)
    if (d.dtype == SALS_BF16) SALS_OS_G(bf16_t); else SALS_OS_G(float);
#undef SALS_OS_G
#undef SALS_OS
    if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    hipLaunchKernelGGL(overlap_merge_kernel, dim3(ceil_div(d.B * d.H_q, 256)), dim3(256), 0, st, part, os,
                       d.B * d.H_q, L.dn_chunks);
    return launch_status();
}


}  // extern "C"

// ---- offline calibration (Sec. 4.2) ----------------------------------------------------
namespace {
constexpr int64_t kCalChunk = 4096;  // tokens whose products are summed in fp32 before they are added to the fp64 matrix
size_t cal_es(int32_t dtype) { return dtype == SALS_BF16 ? 2 : 4; }

// slices of a chunk's token axis (each a separate fp32 output of the GEMM): as many as bring the launch to about two
// workgroups per compute unit, at most 8, every slice at least 256 tokens long
int cal_slices(int D)
{
    const bool big = D % 256 == 0 && D >= 2048;
    const int n = big ? D / 256 : D / 128;
    const int tiles = big ? n * n + n : n * (n + 1) / 2;
    int z = 1;
    while (z < 8 && tiles * z < 512 && kCalChunk / (2 * z) >= 256) z *= 2;
    return z;
}

template <typename T>
sals_status calib_accumulate_t(const void* K, int64_t n_tok, int D, double* C, void* ws, hipStream_t st)
{
    const T* X = static_cast<const T*>(K);
    T* XT = static_cast<T*>(ws);
    float* P = reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + align_up((size_t)D * kCalChunk * sizeof(T)));
    const bool big = D % 256 == 0 && D >= 2048;  // (below that the larger tile leaves most of the chip without a workgroup)
    const int step_tok = kLgStep / (int)sizeof(T);  // tokens per 64-byte step of the contraction axis
    for (int64_t t0 = 0; t0 < n_tok; t0 += kCalChunk) {
        const int64_t n = std::min(kCalChunk, n_tok - t0);
        const int64_t n_pad = (n + 63) / 64 * 64;  // whole 64-byte steps of the contraction axis, zero filled
        hipLaunchKernelGGL((calib_transpose_kernel<T>), dim3((unsigned)(n_pad / kCalTile), (unsigned)ceil_div(D, kCalTile)),
                           dim3(256), 0, st, X + (size_t)t0 * D, XT, (long long)n, D, (long long)n_pad);
        const int steps = (int)(n_pad / step_tok);
        const int per = ceil_div(steps, std::min(cal_slices(D), std::max(1, steps / 2)));  // >= 2 steps per slice
        const int slices = ceil_div(steps, per);
        PrefillArgs a{};
        a.X[0] = XT; a.UT[0] = XT; a.cache[0] = nullptr; a.seq_len = nullptr; a.n_new = nullptr;
        a.n_tok = D; a.D = (int)n_pad; a.r = D; a.S_max = D; a.B = 1; a.nproj = 1; a.pacc = P; a.kslice_steps = per;
        // tiles that reach the upper triangle only (the kernel numbers them row by row)
        if (big) {
            const int nt = D / 256;
            hipLaunchKernelGGL((prefill_compress_kernel<T, 256, 128, true>), dim3(nt * nt + nt, slices, 1), dim3(kPfThreads),
                               prefill_lds_bytes(256, 128), st, a);
        } else {
            const int nt = D / 128;
            hipLaunchKernelGGL((prefill_compress_kernel<T, 128, 128, true>), dim3(nt * (nt + 1) / 2, slices, 1),
                               dim3(kPfThreads), prefill_lds_bytes(128, 128), st, a);
        }
        hipLaunchKernelGGL(calib_reduce_kernel, dim3((unsigned)(((size_t)D * D / 4 + 255) / 256)), dim3(256), 0, st, C, P, D,
                           slices, big ? 256 : 128, 128);
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
    }
    // the lower triangle from the upper one (which also makes the matrix exactly symmetric)
    hipLaunchKernelGGL(calib_mirror_kernel, dim3(D / 32, D / 32), dim3(256), 0, st, C, D);
    return launch_status();
}

template <typename T> sals_status calib_lds_attr()
{
    static std::mutex m;
    static bool done[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SALS_ERR_HIP;
    std::lock_guard<std::mutex> lock(m);
    if (done[dev]) return SALS_OK;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_compress_kernel<T, 256, 128, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_lds_bytes(256, 128)) != hipSuccess ||
        hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_compress_kernel<T, 128, 128, true>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_lds_bytes(128, 128)) != hipSuccess)
        return SALS_ERR_HIP;
    done[dev] = true;
    return SALS_OK;
}
}  // namespace

extern "C" {

size_t sals_calib_accumulate_workspace_bytes(int32_t dtype, int32_t D)
{
    if ((dtype != SALS_BF16 && dtype != SALS_F32) || D < 128 || D % 128 != 0 || D > kCalMaxD) return 0;
    // the transposed keys of a chunk, then the fp32 tile sums of its slices
    return align_up((size_t)D * kCalChunk * cal_es(dtype)) + align_up((size_t)cal_slices(D) * D * D * 4);
}

sals_status sals_calib_accumulate(int32_t dtype, const void* K, int64_t n_tok, int32_t D, double* C, void* workspace,
                                  size_t workspace_bytes, void* hip_stream)
{
    if ((dtype != SALS_BF16 && dtype != SALS_F32) || bad(K) || bad(C) || n_tok < 1 || D < 128 || D % 128 != 0 || D > kCalMaxD)
        return SALS_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 ||
        workspace_bytes < sals_calib_accumulate_workspace_bytes(dtype, D))
        return SALS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (dtype == SALS_BF16) {
        if (calib_lds_attr<bf16_t>() != SALS_OK) return SALS_ERR_HIP;
        return calib_accumulate_t<bf16_t>(K, n_tok, D, C, workspace, st);
    }
    if (calib_lds_attr<float>() != SALS_OK) return SALS_ERR_HIP;
    return calib_accumulate_t<float>(K, n_tok, D, C, workspace, st);
}

size_t sals_calib_eigenvectors_workspace_bytes(int32_t D)
{
    if (D < kCalThreads || D % kCalThreads != 0 || D > kCalMaxD) return 0;
    // convergence slots [D / 2], row norms and signs [D] each
    return align_up((size_t)(D / 2) * 8) + 2 * align_up((size_t)D * 8);
}

sals_status sals_calib_eigenvectors(double* C, int32_t D, int32_t r, int32_t dtype, double* eigval, void* U, void* workspace,
                                    size_t workspace_bytes, int32_t max_sweeps, int32_t* sweeps, void* hip_stream)
{
    if ((dtype != SALS_BF16 && dtype != SALS_F32) || bad(C) || !eigval || bad(U) || D < kCalThreads || D % kCalThreads != 0 ||
        D > kCalMaxD || r < 1 || r > D || max_sweeps < 1)
        return SALS_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 ||
        workspace_bytes < sals_calib_eigenvectors_workspace_bytes(D))
        return SALS_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    double* conv = reinterpret_cast<double*>(ws);
    double* lam = reinterpret_cast<double*>(ws + align_up((size_t)(D / 2) * 8));
    double* sgn = reinterpret_cast<double*>(reinterpret_cast<unsigned char*>(lam) + align_up((size_t)D * 8));
    std::vector<double> h_conv((size_t)D / 2), h_lam((size_t)D);
    auto row_norms = [&]() -> bool {  // row norms to the host (blocking)
        hipLaunchKernelGGL(calib_rownorm_kernel, dim3(D), dim3(kCalThreads), 0, st, C, D, lam, sgn);
        return hipMemcpyAsync(h_lam.data(), lam, (size_t)D * 8, hipMemcpyDeviceToHost, st) == hipSuccess &&
               hipStreamSynchronize(st) == hipSuccess;
    };
    if (!row_norms()) return SALS_ERR_HIP;
    const double n0 = *std::max_element(h_lam.begin(), h_lam.end());
    const double floor = 1e-13 * n0;
    double lead = 0.0;  // first sweep: every rotation counts
    int done = 0;
    bool converged = !(n0 > 0.0);  // the zero matrix needs no rotation
    while (done < max_sweeps && !converged) {
        if (hipMemsetAsync(conv, 0, (size_t)(D / 2) * 8, st) != hipSuccess) return SALS_ERR_HIP;
        for (int step = 0; step < D - 1; ++step)
            hipLaunchKernelGGL(calib_jacobi_step_kernel, dim3(D / 2), dim3(kCalThreads), 0, st, C, D, step, floor, lead, conv);
        if (launch_status() != SALS_OK) return SALS_ERR_HIP;
        if (hipMemcpyAsync(h_conv.data(), conv, (size_t)(D / 2) * 8, hipMemcpyDeviceToHost, st) != hipSuccess) return SALS_ERR_HIP;
        if (!row_norms()) return SALS_ERR_HIP;
        double worst = 0.0;
        for (double v : h_conv) worst = std::max(worst, v);
        ++done;
        // a rotation by less than 1e-11 no longer moves an eigenvector; only pairs with a row among the r largest
        // (a little below the r-th largest norm, so that the r-th itself is in) are asked to have converged
        converged = worst <= 1e-11;
        std::vector<double> sorted(h_lam);
        std::nth_element(sorted.begin(), sorted.begin() + (r - 1), sorted.end(), std::greater<double>());
        lead = 0.999 * sorted[(size_t)r - 1];
    }
    if (dtype == SALS_BF16)
        hipLaunchKernelGGL((calib_select_kernel<bf16_t>), dim3(D), dim3(kCalThreads), 0, st, C, lam, sgn, D, r, eigval,
                           static_cast<bf16_t*>(U));
    else
        hipLaunchKernelGGL((calib_select_kernel<float>), dim3(D), dim3(kCalThreads), 0, st, C, lam, sgn, D, r, eigval,
                           static_cast<float*>(U));
    if (sweeps) *sweeps = converged ? done : -done;
    return launch_status();
}

}  // extern "C"
