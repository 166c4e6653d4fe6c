// Host-callable launchers of the HERO kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;

// Patch grid of Eq. 4 and the closed-form output offsets of the selection list.
// n_take[class]: tokens taken per patch; class = 2*(clipped bottom row) + (clipped right column).
struct SelectGeom {
  int32_t frames, height, width, n_text;
  int32_t patch_h, patch_w;
  int32_t grid_h, grid_w;        // patches per frame along y / x (ceil)
  int32_t n_patches;             // frames * grid_h * grid_w
  int32_t n_take[4];
  int32_t take_per_full_row;     // picks of one patch-row that is not the last one
  int32_t take_per_frame;
  int32_t n_sel;                 // total picks
};

hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t st);
// clears `seen` (ceil(n_tokens/32) bitmap words and one verdict word) and marks the listed rows;
// verdict bit 0: a row outside [0, n_tokens), bit 1: a row listed twice
hipError_t launch_check_idx(const int32_t* idx, int n_sel, int n_tokens, uint32_t* seen, hipStream_t st);
// mode 0: age priority (largest (age, hash) keys); mode 1: age-weighted sampling without replacement
hipError_t launch_select(const SelectGeom& g, int mode, uint32_t step_salt, int32_t* ages, int32_t* idx,
                         hipStream_t st);
// adaLN modulation of a LayerNorm's output, u * (1 + scale) + shift, with the vectors of the row's
// stream (rows < n_text: text).  scale_v == nullptr: none.
struct LnMod {
  const bf16_t *scale_v = nullptr, *shift_v = nullptr, *scale_t = nullptr, *shift_t = nullptr;
  int32_t n_text = 0;
};
hipError_t launch_gather_ln(const void* x, bool x_fp32, const bf16_t* add, const int32_t* rows, int n_rows,
                            int hidden, const bf16_t* gain, const bf16_t* bias, float eps, bf16_t* out,
                            hipStream_t st, const LnMod& mod = LnMod());

// q / k post-processing (per-head LayerNorm, rotary positions on video rows, softmax scale on q), in place
struct QkPostArgs {
  bf16_t* q;                 // [n_rows, d]
  bf16_t* k;                 // [*, d], row rows[i] (or i)
  const int32_t* rows;
  int32_t n_rows, d, head_dim, n_text;
  const bf16_t *qn_g, *qn_b, *kn_g, *kn_b;   // [head_dim]; qn_g == nullptr: no normalisation
  const float2* rope;        // [n_video, head_dim/2] (cos, sin); nullptr: no rotation
  float q_scale;
};
hipError_t launch_qk_post(const QkPostArgs& a, hipStream_t st);
hipError_t launch_rope_table(float2* table, int frames, int height, int width, int head_dim, hipStream_t st);
hipError_t launch_axpy_features(void* x, bool x_fp32, const bf16_t* s_cur, const bf16_t* s_prev, float alpha,
                                int64_t n_elems, hipStream_t st);

// Deep-stack collapse: t = (accumulate ? t : 0) + sum of up to 48 bf16 feature arrays (fp32 result),
// and x += t_cur + (t_cur - t_prev) * alpha (t_prev may be null: x += t_cur).
struct FeatureList {
  const bf16_t* p[48];
  int32_t n;
};
hipError_t launch_sum_features(const FeatureList& fl, float* t, bool accumulate, int64_t n_elems, hipStream_t st);
hipError_t launch_apply_sums(void* x, bool x_fp32, const float* t_cur, const float* t_prev, float alpha,
                             int64_t n_elems, hipStream_t st);
// rows whose age is not 0 (and text rows): x += sum of the listed features; all rows: x += the deep-stack term
// from t_cur / t_prev (both optional)
hipError_t launch_end_of_cached_step(void* x, bool x_fp32, const FeatureList& shallow, const int32_t* ages, int n_text,
                                     int hidden, const float* t_cur, const float* t_prev, float alpha,
                                     int64_t n_elems, hipStream_t st);

// GEMM epilogues: what happens to act(A W^T + bias)
enum GemmEpilogue {
  EPI_PLAIN = 0,        // C[m, n]                       (ldc = n)
  EPI_GELU = 1,         // C[m, n] = gelu_tanh(.)
  EPI_QKV = 2,          // n < d: Q[m, n];  d <= n < 2d: K[row(m), n-d];  else V^T[n-2d, row(m)]
  EPI_SCATTER = 3,      // S[row(m), n] = .
  EPI_SCATTER_ADD = 4   // S[row(m), n] += .
};

// sums of D and D^2, D = f_next - 2 f_cur + f_prev (fp64), into stats[0..1]; scratch: second_diff_scratch_bytes()
size_t second_diff_scratch_bytes();
hipError_t launch_second_diff_stats(const bf16_t* f_prev, const bf16_t* f_cur, const bf16_t* f_next, int64_t n_elems,
                                    double* scratch, double* stats, bool accumulate, hipStream_t st);

struct GemmArgs {
  const bf16_t* a;      // [M, K] row-major
  const bf16_t* w;      // [N, K] row-major
  const bf16_t* bias;   // [N]
  int32_t m, n, k;
  int32_t epilogue;
  const int32_t* rows;  // row(m) = rows ? rows[m] : m   (scatter epilogues)
  bf16_t* c;            // PLAIN/GELU: C; QKV: Q [M, d]; SCATTER*: S [*, n]
  bf16_t* k_out;        // QKV: K cache [*, d]
  bf16_t* vt_out;       // QKV: V^T cache [d, ld_vt]
  int64_t ld_vt;
  int32_t d;            // QKV: hidden
  float q_scale;        // QKV: the Q third is stored multiplied by this (softmax scale folded into Q)
  float* splitk_ws;     // optional device scratch for k-split partial sums (nullptr: never split)
  size_t splitk_ws_bytes;
  void* x;              // SCATTER_ADD, optional: x[row(m), :] += the stored (rounded) S[row(m), :]  (Alg. 1 residual add)
  int32_t x_fp32;       // x holds fp32 (else bf16)
  const bf16_t* gate_v; // SCATTER*, optional: (acc + bias) is multiplied by gate[n] of the row's stream (adaLN gate)
  const bf16_t* gate_t; //   rows (after row(m)) below n_text use gate_t, the others gate_v
  int32_t n_text;
};

hipError_t launch_gemm(const GemmArgs& g, hipStream_t st);
// bytes of scratch launch_gemm would use for this problem if it had all it wanted (0: the problem is not cut along k)
size_t gemm_wanted_scratch_bytes(const GemmArgs& g);
// whether launch_gemm would honour g.x for this problem (only the large-tile kernel does)
bool gemm_can_update_x(const GemmArgs& g);

struct AttnArgs {
  const bf16_t* q;      // [r, n_heads*head_dim]
  const bf16_t* k;      // [n_keys, n_heads*head_dim]
  const bf16_t* vt;     // [n_heads*head_dim, ld_vt]
  int64_t ld_vt;
  bf16_t* o;            // [r, n_heads*head_dim]
  int32_t r, n_keys, n_heads, head_dim;
  float q_scale;        // scores are exp2(q_scale * q.k): log2(e)/sqrt(head_dim), or 1 if folded into Q
  float* split_ws;      // optional device scratch for the partial results of key-split query blocks (nullptr: never split)
  size_t split_ws_bytes;
  uint32_t* fallback_count;   // optional device counter: += 1 per workgroup (NW * 64 queries of one head) whose row sums
                              // left the range of the reference-free form and that recomputed with the running maximum
};

hipError_t launch_attention(const AttnArgs& a, hipStream_t st);
