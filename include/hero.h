/*
 * hero.h -- C ABI of the MI355X (gfx950) implementation of HERO's cached DiT
 * denoising step (patch-wise refresh in shallow layers, linear extrapolation
 * in deep layers; paper Sec. 3.3, 3.4, Alg. 1).
 *
 * Conventions (all entry points)
 *   - Every function returns an int status (HERO_OK = 0 or a HERO_ERR_* code).
 *     hero_last_error() returns a thread-local human-readable message for the
 *     last non-zero status on the calling thread.  Nothing throws across the ABI.
 *   - "dev" pointers are device (HBM) pointers of the current HIP device, "host"
 *     pointers are ordinary host memory.  The library never allocates or frees
 *     device memory: the caller passes a cache buffer and a workspace buffer,
 *     sized by hero_cache_bytes(), and keeps them alive while the handle lives.
 *   - All device work is enqueued on the caller's stream (a hipStream_t passed
 *     as void*, NULL = the default stream) and is asynchronous; the library
 *     never synchronises.  Calls on one handle must be issued in program order
 *     on one stream (or on streams the caller orders).
 *   - Token rows: the joint sequence has N = n_text + frames*height*width rows;
 *     text rows come first, video token (t, y, x) sits at row
 *     n_text + (t*height + y)*width + x.  Activations x are [N, hidden]
 *     row-major, fp32 or bf16 according to resid_dtype, updated in place.
 *   - Parameters (weights, biases, LayerNorm gain/bias) are bf16.  Linear
 *     weights are [out_features, in_features] row-major.
 *   - Caches are bf16.  Per layer the library keeps S = G_attn + G_ffn, the sum
 *     of the two residual-branch features the paper caches (Eq. 2), for all N
 *     rows; shallow layers (l < n_shallow) also keep K [N, hidden] and V
 *     transposed [hidden, N_pad]; deep layers keep S of the previous full step
 *     as well (the paper's Delta G = G_t - G_{t+M}, Sec. 3.4).
 */
#ifndef HERO_H_
#define HERO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  HERO_OK = 0,
  HERO_ERR_INVALID_ARG = 1,      /* null pointer, out-of-range layer/step/k, bad enum      */
  HERO_ERR_SHAPE = 2,            /* configuration the kernels do not support               */
  HERO_ERR_STATE = 3,            /* e.g. refresh before the layer's cache was filled       */
  HERO_ERR_BUFFER_TOO_SMALL = 4, /* caller's cache / workspace buffer is too small         */
  HERO_ERR_HIP = 5               /* a HIP runtime call or kernel launch failed             */
};

enum { HERO_DTYPE_BF16 = 0, HERO_DTYPE_FP32 = 1 };
/* Sample(P, R) of Eq. 4 under the frequency-aware tracking of Sec. 3.3, two readings:
 * AGE_PRIORITY: the n_p tokens of a patch with the largest (age, hash) key, listed by decreasing key;
 * AGE_WEIGHTED: n_p draws without replacement, probability proportional to min(age, 65535) + 1 among
 * the tokens still left (row-major order inside the patch), listed in draw order. */
enum { HERO_SELECT_AGE_PRIORITY = 0, HERO_SELECT_AGE_WEIGHTED = 1 };
/* Block internals that Sec. 3.2 leaves out "for clarity", as CogVideoX-style DiT blocks have them
 * (rows < n_text are the text stream, all others the video stream):
 * ADALN:  u = LN(x) * (1 + scale_s) + shift_s before each branch and G = gate_s * F(u) after it,
 *         with per-stream vectors from the layer's modulation table (hero_layer_weights.mod);
 *         the cached features are the gated ones (what is added to the stream).
 * QKNORM: LayerNorm (eps 1e-6, gain/bias of head_dim elements shared by the heads) over each
 *         head's channels of q and of k.
 * ROPE:   3-D rotary positions on q and k of video rows: of a head's head_dim/2 channel pairs
 *         (2i, 2i+1) the first head_dim/8 turn with t, the next 3*head_dim/16 with y, the rest
 *         with x; pair i of an axis with n pairs turns by pos * 10000^(-i/n).  Text rows and V are
 *         not rotated.  Order: projection, QKNORM, ROPE, softmax scale. */
enum { HERO_BLOCK_ADALN = 1, HERO_BLOCK_QKNORM = 2, HERO_BLOCK_ROPE = 4 };
/* Extra caches, so that the per-layer calls can be used across the K boundary of Alg. 1 (the step
 * schedule of hero_step is not affected):
 * KV_ALL_LAYERS:   every layer keeps K / V^T, so hero_refresh_layer works on any layer (with
 *                  n_sel = 0 on every layer this is plain feature reuse, as FoRA does);
 * PREV_ALL_LAYERS: every layer keeps the previous full step's S, so hero_extrapolate_layer works
 *                  on any layer (first-order forecasting on every layer without setting K = 0). */
enum { HERO_CACHE_KV_ALL_LAYERS = 1, HERO_CACHE_PREV_ALL_LAYERS = 2 };
/* CHECK_IDX: hero_refresh_layer first verifies on the device that dev_idx holds n_sel distinct rows
 * in [0, N) and returns HERO_ERR_INVALID_ARG, launching nothing else, if it does not.  The check
 * reads its verdict back, i.e. it synchronises the stream: a debugging aid, not for timed runs. */
enum { HERO_DEBUG_CHECK_IDX = 1 };

/* Plain-data configuration, copied at hero_cache_create(). */
typedef struct hero_config {
  int32_t n_layers;    /* L                                                              */
  int32_t n_shallow;   /* K: layers 0..K-1 refresh, K..L-1 extrapolate (Alg. 1)          */
  int32_t interval;    /* M: a full step when step % M == 0                              */
  int32_t hidden;      /* d, multiple of 64                                              */
  int32_t n_heads;     /* hidden == n_heads * head_dim                                   */
  int32_t head_dim;    /* 32 or 64                                                       */
  int32_t ffn_dim;     /* multiple of 64                                                 */
  int32_t frames, height, width;  /* video token grid f x h' x w'                         */
  int32_t n_text;      /* text rows, placed first                                        */
  int32_t patch_h, patch_w;       /* spatial patch of Eq. 4 (edge patches are clipped)    */
  float   ratio;       /* R of Eq. 4; tokens per patch = clamp(floor(R*|P|+1/2),1,|P|)   */
  int32_t resid_dtype; /* dtype of x: HERO_DTYPE_FP32 or HERO_DTYPE_BF16                 */
  float   ln_eps;
  uint64_t seed;       /* selection seed                                                 */
  int32_t select_mode; /* HERO_SELECT_AGE_PRIORITY or HERO_SELECT_AGE_WEIGHTED (Sec. 3.3 tracking) */
  int32_t block_flags; /* 0: the plain block of Eq. 2; or a sum of HERO_BLOCK_* (see above)        */
  int32_t cache_flags; /* 0, or a sum of HERO_CACHE_*: caches beyond those Alg. 1 needs              */
  int32_t debug_flags; /* 0, or HERO_DEBUG_CHECK_IDX                                                 */
} hero_config;

/* Borrowed device pointers to one block's parameters (bf16). */
typedef struct hero_layer_weights {
  const void *ln1_g, *ln1_b;   /* [hidden]                */
  const void *w_qkv, *b_qkv;   /* [3*hidden, hidden], [3*hidden]; rows: Q, then K, then V outputs */
  const void *w_o, *b_o;       /* [hidden, hidden], [hidden]   */
  const void *ln2_g, *ln2_b;   /* [hidden]                */
  const void *w_ff1, *b_ff1;   /* [ffn_dim, hidden], [ffn_dim] */
  const void *w_ff2, *b_ff2;   /* [hidden, ffn_dim], [hidden]  */
  /* used only with the matching HERO_BLOCK_* flag (may be NULL otherwise) */
  const void *q_norm_g, *q_norm_b, *k_norm_g, *k_norm_b;   /* [head_dim] each (QKNORM) */
  const void *mod;             /* [12, hidden] bf16 (ADALN), rows: shift, scale, gate of the attention branch for
                                  the video stream, the same three for the text stream, then the six of the FFN
                                  branch in the same order.  Borrowed: the caller may rewrite its contents between
                                  calls (a new timestep), in stream order. */
} hero_layer_weights;

typedef struct hero_cache* hero_cache_t;   /* opaque host-side handle owned by the library */

const char* hero_last_error(void);

/* Number of rows a cached step refreshes (|S(z)| of Eq. 4) for this configuration. */
int hero_num_selected(const hero_config* cfg, int32_t* n_sel_host);

/* Bytes of device memory the handle needs: cache (persistent features, K/V,
 * token ages) and workspace (per-call temporaries).  HERO_ERR_SHAPE for a configuration
 * the kernels do not support; among the limits, (tokens + 512) * max(hidden, ffn_dim) * 2
 * must stay below 2^32 (32-bit operand offsets in the GEMM and attention kernels), e.g.
 * about 174 000 tokens at ffn_dim 12288. */
int hero_cache_bytes(const hero_config* cfg, size_t* cache_bytes, size_t* workspace_bytes);

/* Carves the caller's two device buffers (256-byte aligned) into slabs and
 * enqueues their zero-fill on `stream`.  Ownership of the buffers stays with
 * the caller.  Errors: INVALID_ARG, SHAPE, BUFFER_TOO_SMALL, HIP. */
int hero_cache_create(const hero_config* cfg, void* dev_cache, size_t cache_bytes,
                      void* dev_workspace, size_t workspace_bytes, void* stream,
                      hero_cache_t* out);

/* Frees the host-side handle only. */
int hero_cache_destroy(hero_cache_t c);

/* Start a new video: token ages = 0, no cached generations (Alg. 1 restarts). */
int hero_cache_reset(hero_cache_t c, void* stream);

/* Registers (borrows) the parameters of one layer. */
int hero_set_layer_weights(hero_cache_t c, int32_t layer, const hero_layer_weights* w);

/* Alg. 1 "Initial Caching" for one layer (Eq. 2 on all N rows): x <- block(x),
 * cache S = G_attn + G_ffn for all rows, K/V for shallow layers; deep layers keep the
 * S they held as the previous generation (the new one is written beside it and the two
 * change places once every launch has been accepted).  If a launch fails part-way the
 * layer is left with at most one valid generation: a shallow layer counts as never filled,
 * a deep layer keeps its current S and loses its previous one. */
int hero_full_layer(hero_cache_t c, int32_t layer, void* dev_x, void* stream);

/* S(z) of Eq. 4 with frequency-aware tracking (Sec. 3.3): writes n_sel row
 * indices (int32, joint-sequence rows, patch-major, inside a patch in the order
 * of the configured select_mode) to dev_idx and updates the token ages.  n_sel_host (optional)
 * receives the count, which depends on the configuration only. */
int hero_select(hero_cache_t c, int32_t step, int32_t* dev_idx, int32_t* n_sel_host, void* stream);

/* Sets every token age to zero (done by hero_step after a full step). */
int hero_reset_ages(hero_cache_t c, void* stream);

/* Eq. 3 / Alg. 1 (l < K): recompute QKV, attention against the full cached K/V,
 * and FFN for the n_sel rows in dev_idx (unique, in [0, N)), scatter the
 * results into the caches, then x += S on all N rows.  n_sel = 0 is pure reuse.
 * dev_idx must hold distinct rows in [0, N): a row listed twice is a write race, a row out of range
 * an out-of-bounds write; with HERO_DEBUG_CHECK_IDX the call verifies this first.
 * Errors: STATE if the layer has not been filled; INVALID_ARG if the layer keeps no K/V
 * (layer >= K without HERO_CACHE_KV_ALL_LAYERS), or if the index check fails. */
int hero_refresh_layer(hero_cache_t c, int32_t layer, void* dev_x, const int32_t* dev_idx,
                       int32_t n_sel, void* stream);

/* Eq. 5 / Alg. 1 (l >= K): x += S_t + (S_t - S_{t+M}) * k / M on all rows; the
 * difference is taken as zero while only one full-step generation exists.
 * 0 <= k <= M.  Errors: STATE if not filled; INVALID_ARG if the layer keeps no previous
 * generation (layer < K without HERO_CACHE_PREV_ALL_LAYERS). */
int hero_extrapolate_layer(hero_cache_t c, int32_t layer, void* dev_x, int32_t k, void* stream);

/* Alg. 1 for one denoising step: full step if step % M == 0 (every layer via
 * hero_full_layer, then ages = 0), otherwise select once and run
 * refresh (l < K) / extrapolate (l >= K) with k = step - last full step.
 * On a cached step the deep layers only add their extrapolated features to x
 * (Eq. 5, Alg. 1), so with two or more deep layers hero_step applies them in one
 * pass: it keeps T = sum over deep layers of S (fp32, one array per full-step
 * generation, summed once after each full step) and adds
 * (1 + k/M) T_t - (k/M) T_{t+M}.  The result equals calling
 * hero_extrapolate_layer for every deep layer up to fp32 summation order.
 * Likewise, between the shallow layers of a cached step only the refreshed rows
 * of x are read, so at large shapes hero_step updates those rows layer by layer
 * and adds the shallow layers' cached features to all other rows once, in the
 * same final pass; x equals the result of the per-layer calls up to fp32
 * summation order and the caches are identical.
 * The call enqueues kernels only (no memsets, copies or synchronisation), so once every kernel has
 * run eagerly it may be recorded under stream capture; the step number and k are launch scalars and
 * the schedule state advances at record time, so a graph holds one position of the schedule. */
int hero_step(hero_cache_t c, void* dev_x, int32_t step, void* stream);

/* Read-only views into the handle, for tests and tools.  `what`:
 *   0 S_cur [N,hidden]   1 S_prev [N,hidden] (deep)   2 K [N,hidden] (shallow)
 *   3 V^T [hidden,N_pad] (shallow)   4 ages int32 [n_video]   5 last idx int32 [n_sel]
 *   6 uint32 [1]: attention workgroups (256 queries of one head) that, since create / reset, found
 *     a row sum outside the range of the maximum-free softmax and recomputed their block with the
 *     running-maximum form (see hero_attention_counted); 0 for activations of ordinary scale
 * Returns the device pointer and the leading dimension in elements. */
int hero_cache_view(hero_cache_t c, int32_t layer, int32_t what, void** dev_ptr, int64_t* ld);

/* Schedule state: number of full steps taken and the index of the last one (-1 if none). */
int hero_cache_state(hero_cache_t c, int32_t* n_full, int32_t* last_full_step);

/* ---- per-kernel timing (measurement hook; not part of the method) ------------------
 * Between hero_profile_begin() and hero_profile_end() every kernel launch made through the
 * handle is bracketed by HIP events on the launch stream.  hero_profile_end() synchronises
 * the stream and sums, per slot, the elapsed milliseconds, the number of launches and the
 * algorithmic work (FLOPs for GEMMs and attention, bytes for the row kernels).
 * Slot = kind for launches made by hero_full_layer, kind + HERO_PROF_KINDS otherwise.
 * HERO_PROF_EXTRAP covers both the per-layer update and hero_step's one-pass update of the
 * whole deep stack; HERO_PROF_DEEPSUM is the once-per-generation summation behind the latter.
 * A full layer of a large problem adds its features to x inside the FFN2 kernel: it then has
 * no HERO_PROF_RESID launch and the time is part of HERO_PROF_GEMM_FF2.  A cached hero_step of a
 * large problem does the same for the refreshed rows and adds the features of all other rows,
 * of all shallow layers, in its one pass at the end of the step (HERO_PROF_EXTRAP).
 * The three output arrays have 2 * HERO_PROF_KINDS entries (any may be NULL). */
enum {
  HERO_PROF_SELECT = 0, HERO_PROF_LN = 1, HERO_PROF_GEMM_QKV = 2, HERO_PROF_ATTN = 3,
  HERO_PROF_GEMM_O = 4, HERO_PROF_GEMM_FF1 = 5, HERO_PROF_GEMM_FF2 = 6, HERO_PROF_RESID = 7,
  HERO_PROF_EXTRAP = 8, HERO_PROF_DEEPSUM = 9, HERO_PROF_QKPOST = 10, HERO_PROF_KINDS = 11
};
int hero_profile_begin(hero_cache_t c);
/* The same, bracketing only the kinds whose bit (1u << kind) is set in kind_mask: each bracket
 * costs two stream markers, which a timed run may want to spend on a few kinds only. */
int hero_profile_begin_kinds(hero_cache_t c, uint32_t kind_mask);
int hero_profile_end(hero_cache_t c, void* stream, double* ms, int64_t* launches, double* work);

/* ---- building blocks, exposed so each kernel can be checked on its own -------------
 * An empty problem (n_rows, M, r or n_elems of 0) is a no-op whose row buffers (x / out, A / C,
 * Q / O, x / s_cur) are not touched and may be NULL. */

/* out[i,:] = LayerNorm(x[rows[i],:] (+ add[rows[i],:])) * gain + bias, bf16 out [n_rows, hidden].
 * rows == NULL means rows[i] = i.  add may be NULL.  (Eq. 2's LN on gathered rows.) */
int hero_gather_ln(const void* dev_x, int32_t x_dtype, const void* dev_add_bf16, const int32_t* dev_rows,
                   int32_t n_rows, int32_t hidden, const void* gain, const void* bias, float eps,
                   void* dev_out_bf16, void* stream);

/* C[M,N] = act(A[M,K] W[N,K]^T + bias[N]) in bf16 with fp32 accumulation.
 * act: 0 none, 1 tanh-GELU.  K % 64 == 0, N % 64 == 0.  All device pointers of the building blocks
 * must be 16-byte aligned (index lists 4-byte), else HERO_ERR_INVALID_ARG.  Operands are addressed with 32-bit byte
 * offsets: (M + 512) * K * 2 and (N + 512) * K * 2 must stay below 2^32, else HERO_ERR_SHAPE. */
int hero_linear(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c,
                int32_t m, int32_t n, int32_t k, int32_t act, void* stream);

/* The same product, computed the way the layer entry points compute theirs: with device scratch
 * (caller-owned, 16-byte aligned, any size; 64 MiB lets every problem use it) the tiles of the
 * last, partly filled round of workgroups are cut along K, their fp32 partial sums pass through
 * the scratch and a second kernel adds them up and applies bias and activation.  The result
 * differs from hero_linear's only by the order of the fp32 additions.  Calls that share a
 * scratch buffer must not overlap. */
int hero_linear_scratch(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c,
                        int32_t m, int32_t n, int32_t k, int32_t act, void* dev_scratch,
                        size_t scratch_bytes, void* stream);

/* The same, and *dev_fallbacks (device uint32, optional) += the number of workgroups (256 queries of
 * one head) that took the slower way out.  head_dim 64 evaluates softmax as 2^(q.k log2(e)/sqrt(head_dim))
 * without a running maximum, which is exact while every row sum stays within [2^-80, 2^80]; a workgroup
 * in which some row sum leaves that range recomputes its 256 queries with the running-maximum form
 * (the result is the plain definition's either way; the cost of such a block roughly triples).
 * With scores of a few units, as LayerNorm-ed activations give, that never happens; it takes
 * |q.k| / sqrt(head_dim) beyond about 50. */
int hero_attention_counted(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt,
                           void* dev_o, int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim,
                           void* dev_scratch, size_t scratch_bytes, uint32_t* dev_fallbacks, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): hero_linear_scratch with the partial sums
 * kept in a 32 MiB array that lives inside the library's code object, one copy per device, held
 * until the process ends.  The call allocates and frees nothing (the first call on a device looks
 * the array's device address up once).  Same product, same cut and therefore bit-identical results
 * to hero_linear_scratch with a 32 MiB scratch.  A problem whose k-split wants more than the array
 * holds (tile slots of the last round x k-chunks x 256 KiB > 32 MiB) is refused with
 * HERO_ERR_BUFFER_TOO_SMALL and launches nothing.  Nothing in the array has to start at zero (every
 * block is written before it is read), but all calls on one device share it: calls that overlap in
 * time on one device (two streams, two host threads) race and must be ordered by the caller. */
int hero_linear_static(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c,
                       int32_t m, int32_t n, int32_t k, int32_t act, void* stream);

/* O[r,hidden] = softmax(Q K^T / sqrt(head_dim)) V per head; Q [r,hidden], K [n_keys,hidden],
 * V given transposed as vt [hidden, ld_vt] with ld_vt >= n_keys, ld_vt % 64 == 0 and
 * columns n_keys..ld_vt-1 finite (zero).  (FullAttn of Eq. 2 for refreshed queries, Eq. 3.)
 * K and V^T are addressed with 32-bit byte offsets: (n_keys + 256) * hidden * 2 and
 * hidden * ld_vt * 2 must stay below 2^32, else HERO_ERR_SHAPE. */
int hero_attention(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt,
                   void* dev_o, int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim,
                   void* stream);

/* The same attention, computed the way the layer entry points compute theirs: with device scratch
 * (caller-owned, 16-byte aligned; 128 MiB lets every problem use it) the query blocks of the last,
 * partly filled round of workgroups are cut along the keys (head_dim 64 only); their unnormalised
 * partial outputs and row sums pass through the scratch and a second kernel adds them up,
 * normalises and stores.  The result differs from hero_attention's only by the order of the fp32
 * additions.  Calls that share a scratch buffer must not overlap. */
int hero_attention_scratch(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt,
                           void* dev_o, int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim,
                           void* dev_scratch, size_t scratch_bytes, void* stream);

/* x[N,hidden] += (1+alpha) * s_cur - alpha * s_prev (Eq. 5 followed by the residual add);
 * s_prev may be NULL (alpha is then ignored: plain x += s_cur, Eq. 3's merge-and-add). */
int hero_axpy_features(void* dev_x, int32_t x_dtype, const void* s_cur, const void* s_prev,
                       float alpha, int64_t n_elems, void* stream);

/* ---- stability analysis (Sec. 3.2: which layers are steady enough to extrapolate) ---- */

/* Second-order temporal difference of one layer's feature, D = f_next - 2 f_cur + f_prev, over
 * n_elems bf16 elements (device arrays, n_elems % 8 == 0): dev_stats[0] (+)= sum D, dev_stats[1]
 * (+)= sum D^2, in fp64, with a fixed summation order (reproducible).  accumulate != 0 adds to
 * what dev_stats holds (for more than three steps), else overwrites.  dev_scratch: caller-owned
 * device memory of at least 16 KiB, 8-byte aligned; calls sharing it must not overlap.
 * The variance of Sec. 3.2 is stats[1]/n - (stats[0]/n)^2 with n the number of elements summed. */
int hero_second_diff_stats(const void* f_prev, const void* f_cur, const void* f_next, int64_t n_elems,
                           void* dev_scratch, size_t scratch_bytes, double* dev_stats, int32_t accumulate,
                           void* stream);

/* Host only: per-layer variances -> stability scores in [0, 1], higher = steadier
 * (1 - (v - min) / (max - min); all equal -> 1). */
int hero_stability_scores(const double* variances, int32_t n_layers, double* scores);

#ifdef __cplusplus
}
#endif
#endif /* HERO_H_ */
