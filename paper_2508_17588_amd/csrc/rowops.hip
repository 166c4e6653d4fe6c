// Bandwidth-bound row kernels of the cached DiT step: token selection (Eq. 4 with
// age tracking), row gather + LayerNorm (Eq. 2's LN on the refreshed rows), and the
// fused residual / extrapolation update over all rows (Eq. 3 merge-and-add, Eq. 5).
#include "hero_device.h"
#include "hero_kernels.h"

// ---------------------------------------------------------------------------------
// fill
// ---------------------------------------------------------------------------------
__global__ void fill_i32_kernel(int32_t* p, int32_t v, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int32_t* p, int32_t v, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int blocks = (int)((n + 255) / 256);
  hipLaunchKernelGGL(fill_i32_kernel, dim3(blocks), dim3(256), 0, st, p, v, n);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Index-list check (debugging aid of the refresh entry point): marks every listed row in a bitmap
// of one bit per token; verdict bit 0: some row is outside [0, n_tokens), bit 1: some row is
// listed twice.  `seen` (the bitmap followed by the verdict word) must be zero on entry.
// ---------------------------------------------------------------------------------
__global__ void check_idx_kernel(const int32_t* __restrict__ idx, int n_sel, int n_tokens, uint32_t* seen,
                                 uint32_t* verdict) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_sel) return;
  const int32_t v = idx[i];
  if (v < 0 || v >= n_tokens) { atomicOr(verdict, 1u); return; }
  const uint32_t bit = 1u << (v & 31);
  if (atomicOr(seen + (v >> 5), bit) & bit) atomicOr(verdict, 2u);
}

hipError_t launch_check_idx(const int32_t* idx, int n_sel, int n_tokens, uint32_t* seen, hipStream_t st) {
  const int words = (n_tokens + 31) / 32;
  hipError_t e = launch_fill_i32(reinterpret_cast<int32_t*>(seen), 0, words + 1, st);
  if (e != hipSuccess || n_sel <= 0) return e;
  hipLaunchKernelGGL(check_idx_kernel, dim3((n_sel + 255) / 256), dim3(256), 0, st, idx, n_sel, n_tokens, seen,
                     seen + words);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// selection: one thread per spatial patch
// ---------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fmix32(uint32_t h) {
  h ^= h >> 16; h *= 0x85EBCA6Bu;
  h ^= h >> 13; h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}

__global__ void select_kernel(SelectGeom g, uint32_t step_salt, int32_t* __restrict__ ages,
                              int32_t* __restrict__ idx) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= g.n_patches) return;
  int per_frame = g.grid_h * g.grid_w;
  int t = p / per_frame;
  int rem = p - t * per_frame;
  int py = rem / g.grid_w;
  int px = rem - py * g.grid_w;
  int y0 = py * g.patch_h, x0 = px * g.patch_w;
  int hh = min(g.patch_h, g.height - y0);
  int ww = min(g.patch_w, g.width - x0);
  bool last_row = (py == g.grid_h - 1), last_col = (px == g.grid_w - 1);
  int cls_row = last_row ? 1 : 0;
  // tokens taken from this patch and where its picks go in the output list
  int n_p = g.n_take[cls_row * 2 + (last_col ? 1 : 0)];
  int out = t * g.take_per_frame + py * g.take_per_full_row + px * g.n_take[cls_row * 2];

  int size = hh * ww;
  uint64_t prev = ~0ull;      // keys are < 2^63, so this is above every key
  uint64_t kmin = ~0ull;
  for (int rank = 0; rank < n_p; ++rank) {
    uint64_t best = 0; int best_tok = -1;
    for (int e = 0; e < size; ++e) {
      int dy = e / ww, dx = e - dy * ww;
      int tok = (t * g.height + y0 + dy) * g.width + x0 + dx;
      uint64_t key = ((uint64_t)(uint32_t)ages[tok] << 32) | fmix32(step_salt ^ ((uint32_t)tok * 0x85EBCA6Bu));
      if (key < prev && (best_tok < 0 || key > best)) { best = key; best_tok = tok; }
    }
    idx[out + rank] = g.n_text + best_tok;
    prev = best;
    kmin = best;
  }
  for (int e = 0; e < size; ++e) {
    int dy = e / ww, dx = e - dy * ww;
    int tok = (t * g.height + y0 + dy) * g.width + x0 + dx;
    int32_t a = ages[tok];
    uint64_t key = ((uint64_t)(uint32_t)a << 32) | fmix32(step_salt ^ ((uint32_t)tok * 0x85EBCA6Bu));
    ages[tok] = (n_p > 0 && key >= kmin) ? 0 : a + 1;
  }
}

// Age-weighted reading of the frequency-aware tracking (Sec. 3.3): n_p draws without replacement,
// each taking a token with probability proportional to min(age, 65535) + 1 among those left.
// Draw j of a patch uses the word u = fmix32(hash(first token of the patch) + 0x9E3779B9 * (j+1)),
// maps it to r = floor(u * W / 2^32) with W the weight still left, and takes the first remaining
// token, in row-major order, whose running weight sum exceeds r.  Taken tokens are marked by a
// negative age until the final pass writes the new ages (a patch belongs to one thread).
__global__ void select_weighted_kernel(SelectGeom g, uint32_t step_salt, int32_t* ages, int32_t* __restrict__ idx) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= g.n_patches) return;
  int per_frame = g.grid_h * g.grid_w;
  int t = p / per_frame;
  int rem = p - t * per_frame;
  int py = rem / g.grid_w;
  int px = rem - py * g.grid_w;
  int y0 = py * g.patch_h, x0 = px * g.patch_w;
  int hh = min(g.patch_h, g.height - y0);
  int ww = min(g.patch_w, g.width - x0);
  bool last_row = (py == g.grid_h - 1), last_col = (px == g.grid_w - 1);
  int cls_row = last_row ? 1 : 0;
  int n_p = g.n_take[cls_row * 2 + (last_col ? 1 : 0)];
  int out = t * g.take_per_frame + py * g.take_per_full_row + px * g.n_take[cls_row * 2];
  int size = hh * ww;
  int first_tok = (t * g.height + y0) * g.width + x0;
  uint32_t base = fmix32(step_salt ^ ((uint32_t)first_tok * 0x85EBCA6Bu));
  uint32_t total = 0;
  for (int e = 0; e < size; ++e) {
    int dy = e / ww, dx = e - dy * ww;
    total += (uint32_t)min(ages[first_tok + dy * g.width + dx], 0xFFFF) + 1u;
  }
  for (int j = 0; j < n_p; ++j) {
    uint32_t u = fmix32(base + 0x9E3779B9u * (uint32_t)(j + 1));
    uint32_t r = (uint32_t)(((uint64_t)u * total) >> 32);
    uint32_t run = 0;
    for (int e = 0; e < size; ++e) {
      int dy = e / ww, dx = e - dy * ww;
      int tok = first_tok + dy * g.width + dx;
      int32_t a = ages[tok];
      if (a < 0) continue;
      uint32_t w = (uint32_t)min(a, 0xFFFF) + 1u;
      run += w;
      if (run > r) {
        idx[out + j] = g.n_text + tok;
        ages[tok] = -1;
        total -= w;
        break;
      }
    }
  }
  for (int e = 0; e < size; ++e) {
    int dy = e / ww, dx = e - dy * ww;
    int tok = first_tok + dy * g.width + dx;
    int32_t a = ages[tok];
    ages[tok] = a < 0 ? 0 : a + 1;
  }
}

hipError_t launch_select(const SelectGeom& g, int mode, uint32_t step_salt, int32_t* ages, int32_t* idx,
                         hipStream_t st) {
  if (g.n_patches <= 0) return hipSuccess;
  int blocks = (g.n_patches + 127) / 128;
  if (mode == 1) hipLaunchKernelGGL(select_weighted_kernel, dim3(blocks), dim3(128), 0, st, g, step_salt, ages, idx);
  else hipLaunchKernelGGL(select_kernel, dim3(blocks), dim3(128), 0, st, g, step_salt, ages, idx);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// gather + (optional add) + LayerNorm -> bf16 rows.
// Rows of up to 1024 elements: one wave per row, four rows per workgroup (gather_ln_kernel).
// Longer rows: one workgroup per row, each of its WPR waves holding 1024 elements or fewer (two
// 8-element pieces per lane), the row statistics combined through LDS (gather_ln_split_kernel).
// The kernel is bound by how the memory system takes its access stream, and many waves with
// little state each are the better stream: at 3072 elements three waves per row move 5.7 TB/s
// where one wave per row (48 elements per lane) moved 4.9.
// ---------------------------------------------------------------------------------
template <typename XT, int ITERS>
__global__ __launch_bounds__(256) void gather_ln_kernel(
    const XT* __restrict__ x, const bf16_t* __restrict__ add, const int32_t* __restrict__ rows,
    int n_rows, int hidden, const bf16_t* __restrict__ gain, const bf16_t* __restrict__ bias,
    float eps, bf16_t* __restrict__ out, LnMod mod) {
  int lane = threadIdx.x & 63;
  int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= n_rows) return;
  int64_t src = rows ? (int64_t)rows[r] : (int64_t)r;
  // adaLN: the row's stream (text rows come first) picks the scale and shift vectors
  const bf16_t* mscale = mod.scale_v ? (src < mod.n_text ? mod.scale_t : mod.scale_v) : nullptr;
  const bf16_t* mshift = mod.scale_v ? (src < mod.n_text ? mod.shift_t : mod.shift_v) : nullptr;
  const XT* xr = x + src * hidden;
  const bf16_t* ar = add ? add + src * hidden : nullptr;
  int n_chunks = hidden >> 3;
  float v[ITERS][8];
  float sum = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    int c = lane + it * 64;
    if (c < n_chunks) {
      ResidIO<XT>::load8(xr + c * 8, v[it]);
      if (ar) {
        float a8[8];
        ResidIO<bf16_t>::load8(ar + c * 8, a8);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[it][j] += a8[j];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[it][j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[it][j] = 0.f;
    }
  }
  float mean = wave_sum(sum) / (float)hidden;
  float sq = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    int c = lane + it * 64;
    if (c < n_chunks) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { float dlt = v[it][j] - mean; sq += dlt * dlt; }
    }
  }
  float rstd = rsqrtf(wave_sum(sq) / (float)hidden + eps);
  bf16_t* orow = out + (int64_t)r * hidden;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    int c = lane + it * 64;
    if (c < n_chunks) {
      float g8[8], b8[8], o8[8];
      ResidIO<bf16_t>::load8(gain + c * 8, g8);
      ResidIO<bf16_t>::load8(bias + c * 8, b8);
#pragma unroll
      for (int j = 0; j < 8; ++j) o8[j] = (v[it][j] - mean) * rstd * g8[j] + b8[j];
      if (mscale) {
        float sc8[8], sh8[8];
        ResidIO<bf16_t>::load8(mscale + c * 8, sc8);
        ResidIO<bf16_t>::load8(mshift + c * 8, sh8);
#pragma unroll
        for (int j = 0; j < 8; ++j) o8[j] = o8[j] * (1.0f + sc8[j]) + sh8[j];
      }
      ResidIO<bf16_t>::store8(orow + c * 8, o8);
    }
  }
}

template <typename XT, int WPR, int ITERS = 2>
__global__ __launch_bounds__(64 * WPR) void gather_ln_split_kernel(
    const XT* __restrict__ x, const bf16_t* __restrict__ add, const int32_t* __restrict__ rows,
    int hidden, const bf16_t* __restrict__ gain, const bf16_t* __restrict__ bias,
    float eps, bf16_t* __restrict__ out, LnMod mod) {
  __shared__ float red[2][WPR];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = blockIdx.x;
  const int64_t src = rows ? (int64_t)rows[r] : (int64_t)r;
  // adaLN: the row's stream (text rows come first) picks the scale and shift vectors
  const bf16_t* mscale = mod.scale_v ? (src < mod.n_text ? mod.scale_t : mod.scale_v) : nullptr;
  const bf16_t* mshift = mod.scale_v ? (src < mod.n_text ? mod.shift_t : mod.shift_v) : nullptr;
  const XT* xr = x + src * hidden;
  const bf16_t* ar = add ? add + src * hidden : nullptr;
  const int n_chunks = hidden >> 3;
  const int c0 = wave * (ITERS * 64) + lane;      // this lane's pieces: c0, c0 + 64, ...
  float v[ITERS][8];
  u32x4_t gp[ITERS], bp[ITERS];                   // gain and bias of the lane's pieces, as loaded (bf16 pairs)
  float sum = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = c0 + it * 64;
    if (c < n_chunks) {
      ResidIO<XT>::load8(xr + c * 8, v[it]);
      if (ar) {
        float a8[8];
        ResidIO<bf16_t>::load8(ar + c * 8, a8);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[it][j] += a8[j];
      }
      // the parameters are fetched now, so that their latency passes behind the two reductions
      gp[it] = *reinterpret_cast<const u32x4_t*>(gain + c * 8);
      bp[it] = *reinterpret_cast<const u32x4_t*>(bias + c * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) sum += v[it][j];
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[it][j] = 0.f;
      gp[it] = u32x4_t{0u, 0u, 0u, 0u};
      bp[it] = u32x4_t{0u, 0u, 0u, 0u};
    }
  }
  sum = wave_sum(sum);
  if (lane == 0) red[0][wave] = sum;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < WPR; ++i) tot += red[0][i];
  const float mean = tot / (float)hidden;
  float sq = 0.f;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    if (c0 + it * 64 < n_chunks) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { float dlt = v[it][j] - mean; sq += dlt * dlt; }
    }
  }
  sq = wave_sum(sq);
  if (lane == 0) red[1][wave] = sq;
  __syncthreads();
  float tsq = 0.f;
#pragma unroll
  for (int i = 0; i < WPR; ++i) tsq += red[1][i];
  const float rstd = rsqrtf(tsq / (float)hidden + eps);
  bf16_t* orow = out + (int64_t)r * hidden;
#pragma unroll
  for (int it = 0; it < ITERS; ++it) {
    const int c = c0 + it * 64;
    if (c < n_chunks) {
      float o8[8];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        o8[2 * j] = (v[it][2 * j] - mean) * rstd * unpack_lo(gp[it][j]) + unpack_lo(bp[it][j]);
        o8[2 * j + 1] = (v[it][2 * j + 1] - mean) * rstd * unpack_hi(gp[it][j]) + unpack_hi(bp[it][j]);
      }
      if (mscale) {
        float sc8[8], sh8[8];
        ResidIO<bf16_t>::load8(mscale + c * 8, sc8);
        ResidIO<bf16_t>::load8(mshift + c * 8, sh8);
#pragma unroll
        for (int j = 0; j < 8; ++j) o8[j] = o8[j] * (1.0f + sc8[j]) + sh8[j];
      }
      ResidIO<bf16_t>::store8(orow + c * 8, o8);
    }
  }
}

template <typename XT>
static hipError_t gather_ln_dispatch(const void* x, const bf16_t* add, const int32_t* rows, int n_rows,
                                     int hidden, const bf16_t* gain, const bf16_t* bias, float eps,
                                     bf16_t* out, const LnMod& mod, hipStream_t st) {
  const int iters = (hidden / 8 + 63) / 64;      // 8-element pieces per lane if one wave held the row
  const XT* xp = static_cast<const XT*>(x);
  if (iters <= 2) {
    dim3 grid((n_rows + 3) / 4), block(256);
    if (iters <= 1)
      hipLaunchKernelGGL((gather_ln_kernel<XT, 1>), grid, block, 0, st, xp, add, rows, n_rows, hidden, gain, bias, eps,
                         out, mod);
    else
      hipLaunchKernelGGL((gather_ln_kernel<XT, 2>), grid, block, 0, st, xp, add, rows, n_rows, hidden, gain, bias, eps,
                         out, mod);
    return hipGetLastError();
  }
  const int wpr = (iters + 1) / 2;               // waves per row, two pieces per lane each (hidden <= 8192: <= 8)
#define LAUNCH(W)                                                                                        \
  hipLaunchKernelGGL((gather_ln_split_kernel<XT, W>), dim3(n_rows), dim3(64 * W), 0, st, xp, add, rows, hidden, \
                     gain, bias, eps, out, mod)
  if (wpr <= 2) LAUNCH(2);
  else if (wpr <= 3) LAUNCH(3);
  else if (wpr <= 4) LAUNCH(4);
  else if (wpr <= 6) LAUNCH(6);
  else if (wpr <= 8) LAUNCH(8);
  else return hipErrorInvalidValue;
#undef LAUNCH
  return hipGetLastError();
}

hipError_t launch_gather_ln(const void* x, bool x_fp32, const bf16_t* add, const int32_t* rows, int n_rows,
                            int hidden, const bf16_t* gain, const bf16_t* bias, float eps, bf16_t* out,
                            hipStream_t st, const LnMod& mod) {
  if (n_rows <= 0) return hipSuccess;
  return x_fp32 ? gather_ln_dispatch<float>(x, add, rows, n_rows, hidden, gain, bias, eps, out, mod, st)
                : gather_ln_dispatch<bf16_t>(x, add, rows, n_rows, hidden, gain, bias, eps, out, mod, st);
}

// ---------------------------------------------------------------------------------
// x += s_cur + (s_cur - s_prev) * alpha   (s_prev == nullptr: x += s_cur)
// ---------------------------------------------------------------------------------
// The cached features are read once per call and must not push x out of the memory-side
// cache: consecutive layers of a step update the same x, which then stays resident there while
// only the feature streams come from HBM.  Hence the non-temporal loads of s_cur / s_prev.
__device__ __forceinline__ void load8_stream(const bf16_t* p, float* v) {
  u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
#pragma unroll
  for (int i = 0; i < 4; ++i) { v[2 * i] = unpack_lo(a[i]); v[2 * i + 1] = unpack_hi(a[i]); }
}

template <typename XT, bool HAS_PREV>
__global__ __launch_bounds__(256) void axpy_features_kernel(
    XT* __restrict__ x, const bf16_t* __restrict__ s_cur, const bf16_t* __restrict__ s_prev,
    float alpha, int64_t n_chunks) {
  int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < n_chunks; c += stride) {
    float xv[8], cv[8];
    ResidIO<XT>::load8(x + c * 8, xv);
    load8_stream(s_cur + c * 8, cv);
    if (HAS_PREV) {
      float pv[8];
      load8_stream(s_prev + c * 8, pv);
#pragma unroll
      for (int j = 0; j < 8; ++j) xv[j] += cv[j] + (cv[j] - pv[j]) * alpha;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) xv[j] += cv[j];
    }
    ResidIO<XT>::store8(x + c * 8, xv);
  }
}

hipError_t launch_axpy_features(void* x, bool x_fp32, const bf16_t* s_cur, const bf16_t* s_prev, float alpha,
                                int64_t n_elems, hipStream_t st) {
  int64_t n_chunks = n_elems / 8;
  if (n_chunks <= 0) return hipSuccess;
  int64_t want = (n_chunks + 255) / 256;
  int blocks = (int)(want < (1 << 20) ? want : (1 << 20));     // one 8-element chunk per thread up to 2^31 elements
  dim3 grid(blocks), block(256);
#define LAUNCH(XT, HP)                                                                       \
  hipLaunchKernelGGL((axpy_features_kernel<XT, HP>), grid, block, 0, st, static_cast<XT*>(x), \
                     s_cur, s_prev, alpha, n_chunks)
  if (x_fp32) { if (s_prev) LAUNCH(float, true); else LAUNCH(float, false); }
  else        { if (s_prev) LAUNCH(bf16_t, true); else LAUNCH(bf16_t, false); }
#undef LAUNCH
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Deep-stack collapse.  On a cached step the deep layers only add to x (Eq. 5 followed by the
// residual add, Alg. 1), so their sum over layers can be taken once per full-step generation:
//   T = sum_l S^l  (fp32),   x += (1 + alpha) * T_cur - alpha * T_prev.
// ---------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void sum_features_kernel(FeatureList fl, float* __restrict__ t, int accumulate,
                                                           int64_t n_chunks) {
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_chunks) return;
  float acc[8];
  if (accumulate) ResidIO<float>::load8(t + c * 8, acc);
  else {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  }
  for (int l = 0; l < fl.n; ++l) {
    float v[8];
    load8_stream(fl.p[l] + c * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] += v[j];
  }
  ResidIO<float>::store8(t + c * 8, acc);
}

hipError_t launch_sum_features(const FeatureList& fl, float* t, bool accumulate, int64_t n_elems, hipStream_t st) {
  int64_t n_chunks = n_elems / 8;
  if (n_chunks <= 0 || fl.n <= 0) return hipSuccess;
  int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > (1 << 30)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(sum_features_kernel, dim3((unsigned)blocks), dim3(256), 0, st, fl, t, accumulate ? 1 : 0, n_chunks);
  return hipGetLastError();
}

template <typename XT, bool HAS_PREV>
__global__ __launch_bounds__(256) void apply_sums_kernel(XT* __restrict__ x, const float* __restrict__ t_cur,
                                                         const float* __restrict__ t_prev, float alpha,
                                                         int64_t n_chunks) {
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_chunks) return;
  float xv[8], cv[8];
  ResidIO<XT>::load8(x + c * 8, xv);
  ResidIO<float>::load8(t_cur + c * 8, cv);
  if (HAS_PREV) {
    float pv[8];
    ResidIO<float>::load8(t_prev + c * 8, pv);
#pragma unroll
    for (int j = 0; j < 8; ++j) xv[j] += cv[j] + (cv[j] - pv[j]) * alpha;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) xv[j] += cv[j];
  }
  ResidIO<XT>::store8(x + c * 8, xv);
}

hipError_t launch_apply_sums(void* x, bool x_fp32, const float* t_cur, const float* t_prev, float alpha,
                             int64_t n_elems, hipStream_t st) {
  int64_t n_chunks = n_elems / 8;
  if (n_chunks <= 0) return hipSuccess;
  int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > (1 << 30)) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(256);
#define LAUNCH(XT, HP)                                                                    \
  hipLaunchKernelGGL((apply_sums_kernel<XT, HP>), grid, block, 0, st, static_cast<XT*>(x), \
                     t_cur, t_prev, alpha, n_chunks)
  if (x_fp32) { if (t_prev) LAUNCH(float, true); else LAUNCH(float, false); }
  else        { if (t_prev) LAUNCH(bf16_t, true); else LAUNCH(bf16_t, false); }
#undef LAUNCH
  return hipGetLastError();
}

// End of a cached step in one pass (Alg. 1's residual adds of the whole step, deferred):
//   rows not refreshed in this step:  x += sum over the shallow layers of their cached S
//   every row:                        x += (1 + alpha) T_cur - alpha T_prev   (the deep stack, if any)
// Refreshed rows got their shallow features added layer by layer by the FFN2 epilogue (the next
// layer's refresh reads them); a row is refreshed iff it is a video row whose age the selection
// of this step has just set to 0.
template <typename XT>
__global__ __launch_bounds__(256) void end_of_cached_step_kernel(
    XT* __restrict__ x, FeatureList shallow, const int32_t* __restrict__ ages, int n_text, int hidden,
    const float* __restrict__ t_cur, const float* __restrict__ t_prev, float alpha, int64_t n_chunks) {
  int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= n_chunks) return;
  const int row = (int)((c * 8) / hidden);
  // the row's age decides whether the shallow features are read at all: ask for it first, and let the
  // loads that do not depend on it (x and the deep-stack sums) go out while it is on its way
  const int32_t age = row >= n_text ? ages[row - n_text] : 1;
  float xv[8], acc[8];
  ResidIO<XT>::load8(x + c * 8, xv);
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  if (t_cur != nullptr) {
    float cv[8];
    ResidIO<float>::load8(t_cur + c * 8, cv);
    if (t_prev != nullptr) {
      float pv[8];
      ResidIO<float>::load8(t_prev + c * 8, pv);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += cv[j] + (cv[j] - pv[j]) * alpha;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += cv[j];
    }
  }
  if (age != 0) {                       // not refreshed in this step
    for (int l = 0; l < shallow.n; ++l) {
      float v[8];
      load8_stream(shallow.p[l] + c * 8, v);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += v[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) xv[j] += acc[j];
  ResidIO<XT>::store8(x + c * 8, xv);
}

hipError_t launch_end_of_cached_step(void* x, bool x_fp32, const FeatureList& shallow, const int32_t* ages, int n_text,
                                     int hidden, const float* t_cur, const float* t_prev, float alpha,
                                     int64_t n_elems, hipStream_t st) {
  int64_t n_chunks = n_elems / 8;
  if (n_chunks <= 0) return hipSuccess;
  if (hidden % 8 != 0) return hipErrorInvalidValue;
  int64_t blocks = (n_chunks + 255) / 256;
  if (blocks > (1 << 30)) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks), block(256);
  if (x_fp32)
    hipLaunchKernelGGL(end_of_cached_step_kernel<float>, grid, block, 0, st, static_cast<float*>(x), shallow, ages, n_text,
                       hidden, t_cur, t_prev, alpha, n_chunks);
  else
    hipLaunchKernelGGL(end_of_cached_step_kernel<bf16_t>, grid, block, 0, st, static_cast<bf16_t*>(x), shallow, ages,
                       n_text, hidden, t_cur, t_prev, alpha, n_chunks);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// Stability analysis (Sec. 3.2): sums of D and D^2 over all elements, where
// D = F_{t+1} - 2 F_t + F_{t-1} is the second-order temporal difference of a layer's feature.
// Fixed launch shape and fixed summation order, so the result is reproducible: 1024 workgroups
// leave one (sum, sum of squares) pair each, a single wave adds the pairs up.  All in fp64.
// ---------------------------------------------------------------------------------
constexpr int STAB_BLOCKS = 1024;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

__global__ __launch_bounds__(256) void second_diff_partial_kernel(
    const bf16_t* __restrict__ f_prev, const bf16_t* __restrict__ f_cur, const bf16_t* __restrict__ f_next,
    int64_t n_chunks, double* __restrict__ partial) {
  __shared__ double red[2][4];
  double s1 = 0.0, s2 = 0.0;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < n_chunks; c += stride) {
    float a[8], b[8], e[8];
    load8_stream(f_prev + c * 8, a);
    load8_stream(f_cur + c * 8, b);
    load8_stream(f_next + c * 8, e);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const double d = (double)e[j] - 2.0 * (double)b[j] + (double)a[j];
      s1 += d;
      s2 += d * d;
    }
  }
  s1 = wave_sum_f64(s1);
  s2 = wave_sum_f64(s2);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = s1; red[1][wave] = s2; }
  __syncthreads();
  if (threadIdx.x == 0) {
    partial[2 * blockIdx.x] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
    partial[2 * blockIdx.x + 1] = (red[1][0] + red[1][1]) + (red[1][2] + red[1][3]);
  }
}

__global__ __launch_bounds__(64) void second_diff_final_kernel(const double* __restrict__ partial, int n_blocks,
                                                               double* __restrict__ stats, int accumulate) {
  double s1 = 0.0, s2 = 0.0;
  for (int b = threadIdx.x; b < n_blocks; b += 64) { s1 += partial[2 * b]; s2 += partial[2 * b + 1]; }
  s1 = wave_sum_f64(s1);
  s2 = wave_sum_f64(s2);
  if (threadIdx.x == 0) {
    stats[0] = (accumulate ? stats[0] : 0.0) + s1;
    stats[1] = (accumulate ? stats[1] : 0.0) + s2;
  }
}

size_t second_diff_scratch_bytes() { return (size_t)STAB_BLOCKS * 2 * sizeof(double); }

hipError_t launch_second_diff_stats(const bf16_t* f_prev, const bf16_t* f_cur, const bf16_t* f_next, int64_t n_elems,
                                    double* scratch, double* stats, bool accumulate, hipStream_t st) {
  const int64_t n_chunks = n_elems / 8;
  hipLaunchKernelGGL(second_diff_partial_kernel, dim3(STAB_BLOCKS), dim3(256), 0, st, f_prev, f_cur, f_next, n_chunks,
                     scratch);
  hipLaunchKernelGGL(second_diff_final_kernel, dim3(1), dim3(64), 0, st, scratch, STAB_BLOCKS, stats,
                     accumulate ? 1 : 0);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------
// q / k post-processing of the modulated block: LayerNorm over each head's channels (eps 1e-6,
// one gain / bias vector of head_dim elements shared by the heads), then 3-D rotary positions on
// video rows, then (q only) the softmax scale.  In place, one wave per row: a lane holds 8
// consecutive channels = 4 rotation pairs, a head spans head_dim / 8 neighbouring lanes.
// ---------------------------------------------------------------------------------
template <int HD>
__global__ __launch_bounds__(256) void qk_post_kernel(QkPostArgs a) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= a.n_rows) return;
  const int64_t src = a.rows ? (int64_t)a.rows[r] : (int64_t)r;
  const bool rotate = a.rope != nullptr && src >= a.n_text;
  const float2* table = rotate ? a.rope + (src - a.n_text) * (HD / 2) : nullptr;
  const int n_chunks = a.d >> 3;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    bf16_t* row = which == 0 ? a.q + (int64_t)r * a.d : a.k + src * a.d;
    const bf16_t* gain = which == 0 ? a.qn_g : a.kn_g;
    const bf16_t* bias = which == 0 ? a.qn_b : a.kn_b;
    const float scale = which == 0 ? a.q_scale : 1.0f;
    for (int c = lane; c < n_chunks; c += 64) {      // whole heads stay inside one pass: 512 % HD == 0
      float v[8];
      ResidIO<bf16_t>::load8(row + c * 8, v);
      const int ch = (c * 8) % HD;                    // first channel of this lane inside its head
      if (gain != nullptr) {
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) s += v[j];
#pragma unroll
        for (int o = 1; o < HD / 8; o <<= 1) s += __shfl_xor(s, o, 64);
        const float mean = s * (1.0f / HD);
        float sq = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) { const float dl = v[j] - mean; sq += dl * dl; }
#pragma unroll
        for (int o = 1; o < HD / 8; o <<= 1) sq += __shfl_xor(sq, o, 64);
        const float rstd = rsqrtf(sq * (1.0f / HD) + 1e-6f);
        float g8[8], b8[8];
        ResidIO<bf16_t>::load8(gain + ch, g8);
        ResidIO<bf16_t>::load8(bias + ch, b8);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (v[j] - mean) * rstd * g8[j] + b8[j];
      }
      if (rotate) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const float2 cs = table[ch / 2 + p];
          const float x0 = v[2 * p], x1 = v[2 * p + 1];
          v[2 * p] = x0 * cs.x - x1 * cs.y;
          v[2 * p + 1] = x0 * cs.y + x1 * cs.x;
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] *= scale;
      ResidIO<bf16_t>::store8(row + c * 8, v);
    }
  }
}

hipError_t launch_qk_post(const QkPostArgs& a, hipStream_t st) {
  if (a.n_rows <= 0) return hipSuccess;
  if (a.d % a.head_dim != 0 || (a.head_dim != 32 && a.head_dim != 64)) return hipErrorInvalidValue;
  dim3 grid((a.n_rows + 3) / 4), block(256);
  if (a.head_dim == 64) hipLaunchKernelGGL(qk_post_kernel<64>, grid, block, 0, st, a);
  else hipLaunchKernelGGL(qk_post_kernel<32>, grid, block, 0, st, a);
  return hipGetLastError();
}

// (cos, sin) of the rotation angle of every (video token, channel pair); evaluated in fp64
__global__ void rope_table_kernel(float2* __restrict__ table, int frames, int height, int width, int half_dim) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t n = (int64_t)frames * height * width * half_dim;
  if (i >= n) return;
  const int p = (int)(i % half_dim);
  const int64_t tok = i / half_dim;
  const int x = (int)(tok % width), y = (int)((tok / width) % height), t = (int)(tok / ((int64_t)width * height));
  const int n_t = half_dim / 4, n_y = (half_dim / 8) * 3;      // head_dim/8 pairs, 3*head_dim/16 pairs
  int pos, idx, cnt;
  if (p < n_t) { pos = t; idx = p; cnt = n_t; }
  else if (p < n_t + n_y) { pos = y; idx = p - n_t; cnt = n_y; }
  else { pos = x; idx = p - n_t - n_y; cnt = half_dim - n_t - n_y; }
  const double angle = (double)pos * pow(10000.0, -(double)idx / (double)cnt);
  table[i] = make_float2((float)cos(angle), (float)sin(angle));
}

hipError_t launch_rope_table(float2* table, int frames, int height, int width, int head_dim, hipStream_t st) {
  const int64_t n = (int64_t)frames * height * width * (head_dim / 2);
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, table, frames, height, width,
                     head_dim / 2);
  return hipGetLastError();
}
