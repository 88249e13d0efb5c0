/*
 * sals.h - C ABI of the SALS decode-step attention library for MI355X (gfx950).
 *
 * The operator is Algorithm 1 of "SALS: Sparse Attention in Latent Space for KV
 * cache Compression" (arXiv 2510.24273): per sequence, project the pre-RoPE
 * query into the shared single-head latent space (Sec. 4.3), score every cached
 * token against the latent key cache without RoPE, keep the top-k tokens,
 * reconstruct only those tokens' keys (and values) through the projector, apply
 * RoPE at their positions and run softmax attention over the selected set
 * (Sec. 4.4, Eq. 5).
 *
 * General conventions
 * -------------------
 * Pointers.  Every `const void*` / `void*` / `float*` / `int32_t*` data argument
 *   is a DEVICE pointer on the GPU that is current when the call is made; only
 *   the descriptor, the context handle and out-parameters of the sizing / create
 *   calls are host pointers.  Data pointers must be 16-byte aligned.
 * Ownership.  The caller allocates and frees every device buffer, including the
 *   workspace and the packed weights.  The library never allocates or frees
 *   device memory and keeps no device pointer beyond a call, except the workspace
 *   handed to sals_create, which must stay valid until sals_destroy.
 * Layout.  All arrays are dense and row-major.  Element type `T` is the
 *   descriptor's storage type: 32-bit float, or bfloat16 (upper 16 bits of a
 *   float, round-to-nearest-even).  Token t of a sequence has RoPE position t.
 * Projectors.  `Uk`, `Uv` are the joint projectors U_r of Sec. 4.2 in the paper's
 *   own orientation, [D_kv x r] with D_kv = H_kv*d: row c holds the r latent
 *   coefficients of stacked key (value) channel c.  Down-projection is U^T x,
 *   up-projection (reconstruction) is U x~.  Nothing assumes orthonormality.
 *   The projectors are fixed after calibration, so the decode calls read them from
 *   a packed copy `W` that sals_pack_weights makes once per layer (transposed
 *   copies for the projections, a matrix-core tile order for the reconstruction).
 * Asynchrony.  Each call only enqueues kernels on `hip_stream` (a hipStream_t
 *   passed as void*, NULL = the default stream) and returns; nothing synchronises
 *   and no device data is read on the host.  Calls that share one context must be
 *   ordered on one stream (they share the workspace).
 * Errors.  Every call returns a sals_status; nothing throws or aborts.  Argument
 *   and descriptor errors are detected on the host before anything is enqueued.
 *   A failed launch returns SALS_ERR_HIP.
 */
#ifndef SALS_H
#define SALS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SALS_OK = 0,
    SALS_ERR_INVALID_ARG = 1,  /* NULL pointer, misaligned pointer, bad descriptor field */
    SALS_ERR_UNSUPPORTED = 2,  /* valid request outside what the kernels cover */
    SALS_ERR_WORKSPACE = 3,    /* workspace NULL, misaligned or too small */
    SALS_ERR_HIP = 4           /* a HIP runtime call or kernel launch failed */
} sals_status;

enum { SALS_F32 = 0, SALS_BF16 = 1 };                 /* sals_desc.dtype      */
enum { SALS_ROPE_HALF = 0,        /* pair (i, i+d/2) */
       SALS_ROPE_INTERLEAVED = 1  /* pair (2i, 2i+1) */ };  /* sals_desc.rope_style */

/* Problem descriptor (plain data, host memory).
 * Supported by the kernels: d == 128; r a multiple of 64, 64 <= r <= 2048;
 * r_score a multiple of 8, 8 <= r_score <= min(r, 1024); H_q a multiple of H_kv with
 * H_q/H_kv <= 8 and H_q <= 64; B >= 1 with B*(H_q/H_kv) <= 128; 1 <= S_max <= 2^20;
 * top_k >= 1; n_sink, n_recent >= 0; top_k + n_sink + n_recent <= 65536. */
typedef struct {
    int32_t B;          /* sequences per call                                         */
    int32_t S_max;      /* row capacity of each sequence's latent caches              */
    int32_t H_q;        /* query heads  (the paper's n)                               */
    int32_t H_kv;       /* key/value heads; query head h reads KV head h/(H_q/H_kv)   */
    int32_t d;          /* head width                                                 */
    int32_t r;          /* latent rank                                                */
    int32_t r_score;    /* leading latent coordinates used for scoring (paper: r*)    */
    int32_t top_k;      /* critical tokens chosen by score                            */
    int32_t n_recent;   /* most recent tokens always kept (Sec. 5.2), not candidates  */
    int32_t n_sink;     /* first tokens always kept (Sec. 5.2), not candidates        */
    float   rope_theta; /* RoPE base; pair i turns by pos * theta^(-2i/d)             */
    int32_t rope_style; /* SALS_ROPE_HALF | SALS_ROPE_INTERLEAVED                     */
    int32_t dtype;      /* SALS_F32 | SALS_BF16: type of q, caches, projectors, out   */
} sals_desc;

typedef struct sals_ctx sals_ctx;   /* opaque host object: descriptor + workspace pointer */

/* Human-readable name of a status code (static string, never NULL). */
const char* sals_status_string(sals_status s);

/* Bytes of device workspace a context for `desc` needs.  Host-only. */
sals_status sals_workspace_bytes(const sals_desc* desc, size_t* bytes);

/* Validate `desc`, bind the caller's device workspace (256-byte aligned, at least
 * sals_workspace_bytes) and return a context in *out.  No initial contents are
 * required; after this call the workspace belongs to the library and the caller
 * must not write to it.  Part of it holds a constant table (RoPE cos/sin of every
 * position 0 .. S_max, 512 bytes per position), see sals_prepare.  The launch shapes
 * of every stage are fixed here.  Host-only, allocates only host memory. */
sals_status sals_create(const sals_desc* desc, void* d_workspace, size_t workspace_bytes,
                        sals_ctx** out);
void sals_destroy(sals_ctx* ctx);

/* One-time device set-up of a context: fills the cos/sin table of the workspace with one
 * kernel on `hip_stream`, WAITS for it (the only call of this library that blocks the host),
 * and raises the LDS limit of the kernels the context will launch.  Afterwards calls on the
 * context may come from any stream and may be captured into HIP graphs.
 * A context that was never prepared still works: the first call that needs the table
 * enqueues the fill on its own stream, calls on the same stream follow by stream order and
 * calls on other streams wait for an event; but such a context must not be used under
 * graph capture (SALS_ERR_INVALID_ARG) until a call outside capture has seen the fill
 * complete.  Idempotent. */
sals_status sals_prepare(sals_ctx* ctx, void* hip_stream);

/* Bytes of one layer's packed projectors (4 * D_kv * r elements of T).  Host-only. */
sals_status sals_packed_weight_bytes(const sals_desc* desc, size_t* bytes);

/* One-time repacking of a layer's projectors (Sec. 4.2: they are computed offline and
 * never change), outside the decode path.  Writes into `W` (caller-allocated,
 * 256-byte aligned, sals_packed_weight_bytes): Uk^T and Uv^T [r, D_kv] for the
 * projections, Uk in the tile order of the reconstruction kernel with each head's
 * channels in RoPE pair order (the descriptor's rope_style), and Uv unchanged.
 *   Uk, Uv [D_kv, r] T   (may be freed once the call has completed on the stream) */
sals_status sals_pack_weights(sals_ctx* ctx, const void* Uk, const void* Uv, void* W,
                              void* hip_stream);

/* Stage 1, latent compression of the new token (Eq. 1; Algorithm 1, projection and
 * append steps):  k~ = Uk^T k_new, v~ = Uv^T v_new, rounded to T and written to
 * row seq_len[b] of Kc[b] / Vc[b]; then seq_len[b] += 1.  A sequence whose cache is
 * full (seq_len[b] >= S_max) is left untouched.
 *   k_new, v_new [B, D_kv] T   pre-RoPE key / value of the new token
 *   W                          packed projectors of this layer
 *   Kc, Vc       [B, S_max, r] T   in/out
 *   seq_len      [B] int32         in/out (device) */
sals_status sals_compress_append(sals_ctx* ctx, const void* k_new, const void* v_new,
                                 const void* W, void* Kc, void* Vc, int32_t* seq_len,
                                 void* hip_stream);

/* Bulk compression of a whole prompt (Eq. 1, K~ = K U_r; Algorithm 1, projection and append steps
 * for n_tok tokens at once; the prefill-time counterpart of sals_compress_append):
 *   Kc[b, seq_len[b] + t, :] = Uk^T k_new[b, t],   Vc[b, seq_len[b] + t, :] = Uv^T v_new[b, t]
 * for t < n_new[b], as one GEMM per projection on the matrix cores (fp32 accumulation, one rounding
 * to T, so a row equals what sals_compress_append writes for the same token up to the order of the
 * fp32 sum); then seq_len[b] += n_new[b].  Rows that would fall past S_max are dropped and the length
 * stops at S_max.
 *   k_new, v_new [B, n_tok, D_kv] T   pre-RoPE keys / values of the prompt tokens
 *   W                                 packed projectors of this layer
 *   Kc, Vc       [B, S_max, r] T      in/out
 *   seq_len      [B] int32            in/out (device)
 *   n_new        [B] int32 (device) tokens of each sequence, clamped to [0, n_tok]; NULL: n_tok everywhere
 *   n_tok        1 .. S_max (host)    token capacity of k_new / v_new per sequence */
sals_status sals_compress_prefill(sals_ctx* ctx, const void* k_new, const void* v_new,
                                  const void* W, void* Kc, void* Vc, int32_t* seq_len,
                                  const int32_t* n_new, int32_t n_tok, void* hip_stream);

/* Stage 2a, query projection and latent scores (Sec. 4.3; Algorithm 1, score step):
 *   q~ = Uk^T (sum of the query heads of each KV group, stacked)     [r], fp32
 *   scores[b, j] = sum_{i < r_score} q~[i] * Kc[b, j, i]   for j <  seq_len[b]
 *   scores[b, j] = -inf                                    for j >= seq_len[b]
 * Raw dot products (no 1/sqrt(d), no softmax, no RoPE), fp32 accumulation.
 *   q       [B, H_q, d] T      pre-RoPE query
 *   Kc      [B, S_max, r] T
 *   seq_len [B] int32
 *   scores  [B, S_max] fp32    out */
sals_status sals_latent_scores(sals_ctx* ctx, const void* q, const void* W, const void* Kc,
                               const int32_t* seq_len, float* scores, void* hip_stream);

/* sals_latent_scores for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same kernels and the same results
 * as sals_latent_scores, bit for bit; no context is needed.  The partial sums of q~ (one per slice of
 * the D axis, the only scratch this stage uses) live in an array of SALS_NOALLOC_SCRATCH_BYTES that is
 * part of the library's device image: every GPU the library runs on holds its own copy until the process
 * ends, and its address on the current device is looked up once, on the first call there.
 *   - allocates nothing: no hipMalloc / hipFree, no allocating library routine;
 *   - descriptors whose partial sums need more than SALS_NOALLOC_SCRATCH_BYTES are rejected with
 *     SALS_ERR_WORKSPACE before anything is enqueued (the need is slices * B * r * 4 bytes, at most
 *     8 slices: e.g. 320 KB at B = 16, r = 640);
 *   - every call on a GPU shares that GPU's array, which keeps the last call's contents (each call
 *     overwrites all the entries it later reads, so nothing has to be cleared): calls that overlap on one
 *     GPU, on different streams or from different threads, race.  Calls on one stream are ordered.
 * Arguments as sals_latent_scores; `desc` is read on the host. */
#define SALS_NOALLOC_SCRATCH_BYTES (1u << 20)
sals_status sals_latent_scores_noalloc(const sals_desc* desc, const void* q, const void* W,
                                       const void* Kc, const int32_t* seq_len, float* scores,
                                       void* hip_stream);

/* Stage 2b, critical-token selection (Algorithm 1, TopK step; composition with sink
 * and recent tokens as in Sec. 5.2).  With S = seq_len[b] and
 * k_tot = top_k + n_sink + n_recent:
 *   S <= k_tot : every token is selected, n_sel[b] = S, idx[b, :S] = 0..S-1.
 *   otherwise  : n_sel[b] = k_tot; idx[b] holds the n_sink first tokens, then the
 *                top_k candidates j in [n_sink, S-n_recent) with the largest scores
 *                (equal scores: smaller j wins; -0 equals +0), then the n_recent last
 *                tokens.  The order inside the critical block is unspecified (callers
 *                treat it as a set) but is a deterministic function of the scores.
 * Entries idx[b, n_sel[b]:] are set to 0.
 *   scores [B, S_max] fp32 (NaN-free)
 *   idx    [B, k_tot] int32   out
 *   n_sel  [B] int32          out */
sals_status sals_topk_select(sals_ctx* ctx, const float* scores, const int32_t* seq_len,
                             int32_t* idx, int32_t* n_sel, void* hip_stream);

/* Stage 3, selective reconstruction, RoPE and sparse attention (Sec. 4.4, Eq. 5;
 * Algorithm 1, reconstruction to output steps).  For each sequence and the tokens
 * t = idx[b, j], j < n_sel[b] (indices in [0, S_max), unique):
 *   K_C[j] = Uk Kc[b, t]  reshaped [H_kv, d], rotated by RoPE at position t
 *   V_C[j] = Uv Vc[b, t]  reshaped [H_kv, d]
 *   out[b, h] = sum_j softmax_j( RoPE(q[b,h], q_pos[b]) . K_C[j, g(h)] / sqrt(d) ) V_C[j, g(h)]
 * Keys are reconstructed on the matrix cores (bf16 x bf16 -> fp32, or fp32), RoPE,
 * logits and softmax are fp32; the value product is evaluated in the exact
 * re-associated order  ((p . V~_C) . Uv^T)  and rounded once to T.  If
 * n_sel[b] == 0, out[b] is zero.
 *   q [B,H_q,d] T;  q_pos [B] int32;  Kc, Vc [B,S_max,r] T;  W packed projectors
 *   idx [B,k_tot] int32;  n_sel [B] int32;  out [B,H_q,d] T */
sals_status sals_sparse_attend(sals_ctx* ctx, const void* q, const int32_t* q_pos,
                               const void* Kc, const void* Vc, const void* W,
                               const int32_t* idx, const int32_t* n_sel, void* out,
                               void* hip_stream);

/* The whole decode step of Algorithm 1 on one stream: sals_latent_scores,
 * sals_topk_select, sals_sparse_attend.  `scores`, `idx`, `n_sel` may each be NULL,
 * in which case that intermediate lives in the workspace. */
sals_status sals_decode_step(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* Kc,
                             const void* Vc, const void* W, const int32_t* seq_len, void* out,
                             float* scores, int32_t* idx, int32_t* n_sel, void* hip_stream);

/* ---- quantised full-rank value cache -----------------------------------------------
 * The paper's own value path (Sec. 5.1; the quantised cache V-hat that Algorithm 1 appends
 * to and reads in its last step): values are not projected; each token's D_kv value channels
 * are stored with channel-wise group quantisation, `bits` = 4 (the 25 % setting) or 2
 * (12.5 %), asymmetric and uniform as in KIVI.  Where the paper gives no detail the layout is:
 * groups of SALS_QV_GROUP = 32 consecutive channels; per group  zero = min,
 * scale = T((max - min) / (2^bits - 1));  per channel
 * code = clamp(rint((v - zero) / scale), 0, 2^bits - 1)  evaluated in fp32 (IEEE division,
 * ties to even; code 0 when scale == 0);  de-quantised value  v^ = zero + scale * code.
 *   Vq    [B, S_max, D_kv*bits/8] bytes: channel c of a token in byte c*bits/8 at bit (c*bits) % 8
 *   Vmeta [B, S_max, D_kv/32, 2] T     : (scale, zero) of each group
 * The three calls mirror sals_compress_append / sals_sparse_attend / sals_decode_step with this
 * cache in place of the latent value cache; keys, scores and selection are unchanged, and the
 * U_v sections of `W` are not read (any [D_kv, r] array may be packed in their place). */
enum { SALS_QV_GROUP = 32 };

/* Bytes per token of the code array and of the (scale, zero) array.  Host-only. */
sals_status sals_qv_row_bytes(const sals_desc* desc, int bits, size_t* code_bytes,
                              size_t* meta_bytes);

/* Algorithm 1, projection and append steps:  k~ = Uk^T k_new to row seq_len[b] of Kc[b]; the
 * quantised v_new to row seq_len[b] of Vq[b] / Vmeta[b]; then seq_len[b] += 1.  A sequence
 * whose cache is full is left untouched.
 *   k_new, v_new [B, D_kv] T;  Kc [B,S_max,r] T in/out;  Vq, Vmeta in/out;  seq_len [B] in/out */
sals_status sals_compress_append_qv(sals_ctx* ctx, const void* k_new, const void* v_new,
                                    const void* W, void* Kc, void* Vq, void* Vmeta, int bits,
                                    int32_t* seq_len, void* hip_stream);

/* Algorithm 1, reconstruction to output steps, with
 *   out[b, h] = sum_j softmax_j( RoPE(q[b,h]) . K_C[j, g(h)] / sqrt(d) ) v^[b, idx[b,j], g(h)]
 * (fp32 accumulation, one rounding to T).  Everything else as sals_sparse_attend. */
sals_status sals_sparse_attend_qv(sals_ctx* ctx, const void* q, const int32_t* q_pos,
                                  const void* Kc, const void* Vq, const void* Vmeta, int bits,
                                  const void* W, const int32_t* idx, const int32_t* n_sel,
                                  void* out, void* hip_stream);

/* sals_latent_scores, sals_topk_select, sals_sparse_attend_qv on one stream; `scores`, `idx`,
 * `n_sel` may each be NULL (then they live in the workspace). */
sals_status sals_decode_step_qv(sals_ctx* ctx, const void* q, const int32_t* q_pos,
                                const void* Kc, const void* Vq, const void* Vmeta, int bits,
                                const void* W, const int32_t* seq_len, void* out, float* scores,
                                int32_t* idx, int32_t* n_sel, void* hip_stream);

/* ---- dense baseline -----------------------------------------------------------------
 * Dense decode attention over a full-rank KV cache, the baseline the paper quotes its
 * speed-ups against (Sec. 5.3, Table 6), for comparisons on the same hardware:
 *   out[b,h] = softmax_j( RoPE(q[b,h], q_pos[b]) . K[b,j,g(h)] / sqrt(d) ) V[b,j,g(h)],  j < seq_len[b]
 * with every cached token attended (Eq. 5 with the selected set = everything).  K holds the
 * keys as a dense model caches them, already rotated at their positions; fp32 online softmax,
 * one rounding to T.  out[b] is zero when seq_len[b] == 0.
 *   q [B,H_q,d] T pre-RoPE;  q_pos [B] int32;  K, V [B,S_max,H_kv,d] T;  seq_len [B] int32;
 *   out [B,H_q,d] T */
sals_status sals_dense_attend(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* K,
                              const void* V, const int32_t* seq_len, void* out, void* hip_stream);

/* ---- high-precision recent window ----------------------------------------------------
 * The mixed-precision scheme of Sec. 5.1: the most recent w tokens are compressed less than the
 * rest, and this window is the set of recent tokens the selection always keeps (Sec. 5.2).
 * Where the paper gives no detail the format is: a second pair of latent caches Kw, Vw of rank
 * r_hi > r with projectors of their own (the leading r_hi principal directions of the same
 * calibration; r_hi = D_kv/2 is the paper's 50 % setting), held as
 * a ring of w rows per sequence: token t lies in row t mod w while it is among the last w tokens.
 * Every token is written to both caches when it is appended, so nothing is re-compressed when it
 * leaves the window: its ring row is simply overwritten w tokens later.
 *
 * The window has a context of its own, `win`, created from a descriptor that equals the main
 * one in B, S_max, H_q, H_kv, d, rope_theta, rope_style and dtype and has r = r_hi, top_k = w
 * (= the main descriptor's n_recent >= 1), n_sink = n_recent = 0 (r_score: any valid value <= 1024, unused), with its
 * own workspace and its own packed projectors W_hi (sals_pack_weights on `win`).
 *   Kw, Vw [B, w, r_hi] T */

/* Eq. 1 for the window: k~ = Uk_hi^T k_new, v~ = Uv_hi^T v_new into row seq_len[b] mod w of
 * Kw[b] / Vw[b].  seq_len is only read: call this BEFORE the sals_compress_append that writes the
 * same token to the main caches and advances seq_len.  A sequence with seq_len[b] >= S_max is left
 * untouched, as there. */
sals_status sals_window_append(sals_ctx* win, const void* k_new, const void* v_new, const void* W_hi,
                               void* Kw, void* Vw, const int32_t* seq_len, void* hip_stream);

/* sals_sparse_attend with the window: idx / n_sel are a selection in the order sals_topk_select
 * writes it on `ctx` (recent tokens last).  The last n_w = min(w, n_sel[b]) entries of idx[b] are
 * reconstructed from ring rows idx mod w of Kw / Vw through W_hi, all entries before them from Kc / Vc
 * through W; one softmax (Eq. 5) runs over the union: both passes weight their tokens with the
 * maximum and normaliser of the whole selection, and one output projection adds their latent value
 * sums through Uv and Uv_hi (fp32, rounded once to T).  The call uses the workspaces of both
 * contexts. */
sals_status sals_sparse_attend_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                      const void* Kc, const void* Vc, const void* W, const void* Kw,
                                      const void* Vw, const void* W_hi, const int32_t* idx,
                                      const int32_t* n_sel, void* out, void* hip_stream);

/* sals_latent_scores and sals_topk_select on `ctx` (scores over the low-rank key cache, which holds
 * every token), then sals_sparse_attend_window.  `scores`, `idx`, `n_sel` may each be NULL. */
sals_status sals_decode_step_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                    const void* Kc, const void* Vc, const void* W, const void* Kw,
                                    const void* Vw, const void* W_hi, const int32_t* seq_len, void* out,
                                    float* scores, int32_t* idx, int32_t* n_sel, void* hip_stream);

/* ---- the recent window over the paper's own cache formats (Sec. 5.1, Sec. 5.2) --------------------
 * The paper's setting keeps latent keys and group-quantised full-rank values, and lets the most recent
 * window of tokens keep half of its original size.  Where the paper gives no detail the format is: the
 * window's keys are the rank-r_hi ring Kw of the calls above (r_hi = D_kv/2), the window's values the same
 * group quantiser at 8 bits (half of a 16-bit channel) in a ring of w rows,
 *   Vqw     [B, w, D_kv] bytes        code of channel c of token t in row t mod w, byte c
 *   Vmeta_w [B, w, D_kv/32, 2] T      (scale, zero) of each group, scale = T((max - min) / 255)
 * with codes decided in fp32 exactly as for 2 / 4 bits.  `win` is the window's context as above. */

/* The new token into ring row seq_len[b] mod w: k~ = Uk_hi^T k_new into Kw, the 8-bit quantised v_new into
 * Vqw / Vmeta_w.  Reads seq_len, does not advance it: call before the sals_compress_append_qv of the same
 * token.   k_new, v_new [B, D_kv] T */
sals_status sals_window_append_qv(sals_ctx* win, const void* k_new, const void* v_new, const void* W_hi,
                                  void* Kw, void* Vqw, void* Vmeta_w, const int32_t* seq_len,
                                  void* hip_stream);

/* sals_sparse_attend_qv with the window: the last n_w = min(w, n_sel[b]) entries of idx[b] (the recent tokens,
 * in the order sals_topk_select writes them) take their keys from ring rows idx mod w of Kw through W_hi and
 * their values from the 8-bit ring, all entries before them from Kc through W and from the `bits`-bit cache
 * Vq / Vmeta; one softmax (Eq. 5) over the union, fp32 accumulation, one rounding to T. */
sals_status sals_sparse_attend_qv_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                         const void* Kc, const void* Vq, const void* Vmeta, int bits,
                                         const void* W, const void* Kw, const void* Vqw, const void* Vmeta_w,
                                         const void* W_hi, const int32_t* idx, const int32_t* n_sel, void* out,
                                         void* hip_stream);

/* The paper's whole decode step in its own setting: sals_latent_scores and sals_topk_select on `ctx`
 * (16 sink + critical + w recent tokens, Sec. 5.2), then sals_sparse_attend_qv_window.  `scores`, `idx`,
 * `n_sel` may each be NULL. */
sals_status sals_decode_step_qv_window(sals_ctx* ctx, sals_ctx* win, const void* q, const int32_t* q_pos,
                                       const void* Kc, const void* Vq, const void* Vmeta, int bits,
                                       const void* W, const void* Kw, const void* Vqw, const void* Vmeta_w,
                                       const void* W_hi, const int32_t* seq_len, void* out, float* scores,
                                       int32_t* idx, int32_t* n_sel, void* hip_stream);

/* ---- overlap score -------------------------------------------------------------------
 * The diagnostic of Sec. 3.2: the share of the dense attention mass that a selected set captures,
 *   os[b,h] = sum_{j < n_sel[b]} p[idx[b,j]] / sum_{j < seq_len[b]} p[j],
 *   p[j] = exp( RoPE(q[b,h], q_pos[b]) . K[b,j,g(h)] / sqrt(d) ),
 * over the dense baseline's rotated full-rank key cache.  idx entries must be unique tokens below
 * seq_len[b]; os[b,:] is zero for an empty cache or selection.
 *   q [B,H_q,d] T pre-RoPE;  K [B,S_max,H_kv,d] T;  idx [B,k_tot] int32;  os [B,H_q] fp32 out */
sals_status sals_overlap_score(sals_ctx* ctx, const void* q, const int32_t* q_pos, const void* K,
                               const int32_t* seq_len, const int32_t* idx, const int32_t* n_sel,
                               float* os, void* hip_stream);

/* ---- offline calibration (Sec. 4.2) -------------------------------------------------
 * The projection into the latent space is found offline from the pre-RoPE keys of a calibration set: with all
 * heads of a token merged into one row of width D = n*d, the covariance C = K^T K of the stacked keys is
 * eigen-decomposed and the r leading eigenvectors form U_r.  These two calls need no context.
 *
 * sals_calib_accumulate adds the tokens of one call to the covariance:  C += K^T K  (fp64 C; products of the
 * stored values, summed in fp32 over at most 4096 tokens at a time on the matrix cores, then added in fp64; the
 * upper triangle is computed and mirrored, so C leaves the call exactly symmetric).
 *   dtype      SALS_BF16 | SALS_F32 (host)
 *   K          [n_tok, D] T (device)   calibration keys, one token per row
 *   n_tok      >= 1 (host)
 *   D          multiple of 128, at most 8192 (host)
 *   C          [D, D] fp64 (device)    in/out; the caller zeroes it before the first call
 *   workspace  device, 256-byte aligned, at least sals_calib_accumulate_workspace_bytes(dtype, D) bytes, no contents
 *              kept between calls (it holds the transposed keys of a chunk and the fp32 tile sums of its slices)
 * Asynchronous on hip_stream.  Errors: SALS_ERR_INVALID_ARG (NULL or misaligned pointer, bad size),
 * SALS_ERR_WORKSPACE, SALS_ERR_HIP.
 *
 * sals_calib_eigenvectors computes the eigen-decomposition of C (symmetric, positive semi-definite) by one-sided
 * Jacobi rotations of its rows in fp64 and returns all eigenvalues in descending order and the r leading eigenvectors:
 *   C          [D, D] fp64 (device)    in; OVERWRITTEN (its rows become eigenvalue times eigenvector)
 *   D          multiple of 256, at most 8192;  r  1 .. D
 *   dtype      storage type T of U
 *   eigval     [D] fp64 (device)       out, descending: the first r are converged eigenvalues; the others are the
 *                                      norms their rows had when the leading ones had converged (approximations)
 *   U          [D, r] T (device)       out: column i is the eigenvector of eigval[i], unit length, signed so that
 *                                      its largest component is positive, rounded once to T; the layout
 *                                      sals_pack_weights takes.  Eigenvalues below 1e-13 of the largest are zero to
 *                                      working precision: their vectors are not resolved (whatever direction the
 *                                      row was left with).
 *   workspace  device, 256-byte aligned, at least sals_calib_eigenvectors_workspace_bytes(D) bytes
 *   max_sweeps at least 1 (host): a sweep rotates every pair of rows once; the call stops after the first sweep in
 *              which no rotation that involved one of the r largest rows turned by more than 1e-11, or after
 *              max_sweeps
 *   sweeps     host int32, out (may be NULL): sweeps run; the negative of that number if the limit was reached
 *              before convergence (the results are then the current approximation)
 * BLOCKING: it waits for hip_stream once per sweep to read the convergence measure, so it cannot be captured.
 * Errors as above. */
size_t sals_calib_accumulate_workspace_bytes(int32_t dtype, int32_t D);
sals_status sals_calib_accumulate(int32_t dtype, const void* K, int64_t n_tok, int32_t D, double* C,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);
size_t sals_calib_eigenvectors_workspace_bytes(int32_t D);
sals_status sals_calib_eigenvectors(double* C, int32_t D, int32_t r, int32_t dtype, double* eigval, void* U,
                                    void* workspace, size_t workspace_bytes, int32_t max_sweeps, int32_t* sweeps,
                                    void* hip_stream);

/* ---- measurement aid --------------------------------------------------------------
 * Per-stage timing for roofline figures.  While enabled, every stage below (one kernel;
 * for the selection of sequences above 32768 tokens a chain of four, for the logits of very
 * short selections two) is bracketed by a
 * pair of HIP events on the call's stream (host-side event objects; no device memory).  sals_profile_collect waits for the recorded events, adds
 * the elapsed milliseconds and launch counts per kernel into total_ms / launches (host
 * arrays of SALS_N_KERNELS entries, overwritten) and forgets the records.  Timing with
 * events serialises neighbouring launches slightly; leave it off in timed runs. */
enum {
    SALS_K_PROJECT = 0,        /* latent projection (query, or new key/value)  */
    SALS_K_SCORES = 1,         /* latent score stream over the key cache       */
    SALS_K_TOPK = 2,           /* exact top-k selection                        */
    SALS_K_ATTEND_LOGITS = 3,  /* MFMA key reconstruction + RoPE + q.K         */
    SALS_K_ATTEND_PV = 4,      /* softmax + latent-space value sum             */
    SALS_K_ATTEND_OUT = 5,     /* output projection through U_v                */
    SALS_K_ATTEND_QV = 6,      /* softmax + sum over the quantised value cache */
    SALS_K_DENSE = 7,          /* dense baseline attention (+ its chunk merge)  */
    SALS_K_PREFILL = 8,        /* bulk compression of a prompt (MFMA GEMM)     */
    SALS_N_KERNELS = 9
};
const char* sals_kernel_name(int kernel);
sals_status sals_profile_enable(sals_ctx* ctx, int on);
sals_status sals_profile_collect(sals_ctx* ctx, double* total_ms, int32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* SALS_H */
