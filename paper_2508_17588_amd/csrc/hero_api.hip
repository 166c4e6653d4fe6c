// Host side of the HERO library: cache handle, layer operations (fixed sequences of
// kernel launches on the caller's stream) and the step schedule of Alg. 1.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <initializer_list>
#include <cstring>
#include <mutex>
#include <new>
#include <algorithm>
#include <utility>
#include <vector>

#include "../../include/hero.h"
#include "hero_kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                      \
  do {                                                                                     \
    hipError_t e_ = (expr);                                                                \
    if (e_ != hipSuccess) return fail(HERO_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// true when every pointer is null or 16-byte aligned (the kernels use 8- and 16-byte vector accesses)
bool aligned16(std::initializer_list<const void*> ptrs) {
  for (const void* p : ptrs)
    if ((uintptr_t)p & 15) return false;
  return true;
}

// ---- scratch owned by the library, for the entry point that must not allocate -----------------
// Every device the library runs on holds its own copy of this array, at its own address, until
// the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device and that pointer is what kernels are given.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)32 << 20;
constexpr int STATIC_SCRATCH_MAX_DEVICES = 64;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

int static_scratch(void** out) {
  static std::mutex mu;
  static void* ptrs[STATIC_SCRATCH_MAX_DEVICES] = {};
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= STATIC_SCRATCH_MAX_DEVICES)
    return fail(HERO_ERR_INVALID_ARG, "device ordinal %d outside [0, %d)", dev, STATIC_SCRATCH_MAX_DEVICES);
  std::lock_guard<std::mutex> lock(mu);
  if (ptrs[dev] == nullptr) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // the current device's copy
    if (p == nullptr) return fail(HERO_ERR_HIP, "hipGetSymbolAddress returned a null address");
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return HERO_OK;
}

uint32_t fmix32_host(uint32_t h) {
  h ^= h >> 16; h *= 0x85EBCA6Bu;
  h ^= h >> 13; h *= 0xC2B2AE35u;
  h ^= h >> 16;
  return h;
}

// tokens per patch: clamp(floor(R*|P| + 1/2), 1, |P|), 0 if R <= 0 (R at float precision; the
// product and the sum are exact in double)
int tokens_per_patch(float ratio, int size) {
  if (!(ratio > 0.f)) return 0;
  double v = std::floor((double)ratio * (double)size + 0.5);
  if (v < 1.0) v = 1.0;
  if (v > (double)size) v = (double)size;
  return (int)v;
}

// The GEMM and attention kernels address their operands with 32-bit byte offsets; a tile may form
// offsets for up to 512 rows (GEMM) or 256 keys (attention) past the end of an operand, which the
// hardware bounds check then discards.  These mirror the launchers' own guards.
bool gemm_offsets_fit(int64_t m, int64_t n, int64_t k) {
  const int64_t lim = (int64_t)1 << 32;
  return (m + 512) * k * 2 < lim && (n + 512) * k * 2 < lim;
}
bool attention_offsets_fit(int64_t n_keys, int64_t hidden, int64_t ld_vt) {
  const int64_t lim = (int64_t)1 << 32;
  return (n_keys + 256) * hidden * 2 < lim && hidden * ld_vt * 2 < lim;
}

int check_config(const hero_config* c) {
  if (!c) return fail(HERO_ERR_INVALID_ARG, "config is null");
  if (c->n_layers < 1 || c->n_shallow < 0 || c->n_shallow > c->n_layers || c->interval < 1)
    return fail(HERO_ERR_INVALID_ARG, "need n_layers >= 1, 0 <= n_shallow <= n_layers, interval >= 1");
  if (c->frames < 1 || c->height < 1 || c->width < 1 || c->n_text < 0 || c->patch_h < 1 || c->patch_w < 1)
    return fail(HERO_ERR_INVALID_ARG, "token grid / patch sizes must be positive");
  if (c->resid_dtype != HERO_DTYPE_FP32 && c->resid_dtype != HERO_DTYPE_BF16)
    return fail(HERO_ERR_INVALID_ARG, "resid_dtype must be HERO_DTYPE_FP32 or HERO_DTYPE_BF16");
  if (!(c->ratio >= 0.f) || !(c->ln_eps >= 0.f)) return fail(HERO_ERR_INVALID_ARG, "ratio and ln_eps must be >= 0");
  if (c->select_mode != HERO_SELECT_AGE_PRIORITY && c->select_mode != HERO_SELECT_AGE_WEIGHTED)
    return fail(HERO_ERR_INVALID_ARG, "select_mode must be HERO_SELECT_AGE_PRIORITY or HERO_SELECT_AGE_WEIGHTED");
  if (c->select_mode == HERO_SELECT_AGE_WEIGHTED && (int64_t)c->patch_h * c->patch_w > 65535)
    return fail(HERO_ERR_SHAPE, "age-weighted selection needs patches of at most 65535 tokens");
  if (c->block_flags < 0 || c->block_flags > (HERO_BLOCK_ADALN | HERO_BLOCK_QKNORM | HERO_BLOCK_ROPE))
    return fail(HERO_ERR_INVALID_ARG, "block_flags must be a sum of HERO_BLOCK_* values");
  if (c->cache_flags < 0 || c->cache_flags > (HERO_CACHE_KV_ALL_LAYERS | HERO_CACHE_PREV_ALL_LAYERS))
    return fail(HERO_ERR_INVALID_ARG, "cache_flags must be a sum of HERO_CACHE_* values");
  if (c->debug_flags < 0 || c->debug_flags > HERO_DEBUG_CHECK_IDX)
    return fail(HERO_ERR_INVALID_ARG, "debug_flags must be 0 or HERO_DEBUG_CHECK_IDX");
  if ((c->block_flags & HERO_BLOCK_ROPE) && c->head_dim % 16 != 0)
    return fail(HERO_ERR_SHAPE, "rotary positions need head_dim to be a multiple of 16");
  if (c->head_dim != 32 && c->head_dim != 64) return fail(HERO_ERR_SHAPE, "head_dim must be 32 or 64");
  if (c->hidden != c->n_heads * c->head_dim || c->n_heads < 1)
    return fail(HERO_ERR_SHAPE, "hidden must equal n_heads * head_dim");
  if (c->hidden % 64 != 0 || c->ffn_dim % 64 != 0 || c->ffn_dim < 64)
    return fail(HERO_ERR_SHAPE, "hidden and ffn_dim must be multiples of 64");
  if (c->hidden > 8192) return fail(HERO_ERR_SHAPE, "hidden must be <= 8192");
  int64_t n = (int64_t)c->n_text + (int64_t)c->frames * c->height * c->width;
  if (n > (1 << 24)) return fail(HERO_ERR_SHAPE, "more than 2^24 tokens");
  // every GEMM of the block on all n rows, and attention over n keys
  const int64_t d = c->hidden, f = c->ffn_dim, n_pad = (n + 63) / 64 * 64;
  if (!gemm_offsets_fit(n, 3 * d, d) || !gemm_offsets_fit(n, f, d) || !gemm_offsets_fit(n, d, f) ||
      !attention_offsets_fit(n, d, n_pad))
    return fail(HERO_ERR_SHAPE,
                "%lld tokens x max(hidden, ffn_dim) = %lld exceeds the kernels' 32-bit operand offsets: "
                "(tokens + 512) * max(hidden, ffn_dim) * 2 must stay below 2^32",
                (long long)n, (long long)(d > f ? d : f));
  return HERO_OK;
}

SelectGeom make_geom(const hero_config& c) {
  SelectGeom g;
  g.frames = c.frames; g.height = c.height; g.width = c.width; g.n_text = c.n_text;
  g.patch_h = c.patch_h; g.patch_w = c.patch_w;
  g.grid_h = (c.height + c.patch_h - 1) / c.patch_h;
  g.grid_w = (c.width + c.patch_w - 1) / c.patch_w;
  g.n_patches = c.frames * g.grid_h * g.grid_w;
  int hh_last = c.height - (g.grid_h - 1) * c.patch_h;
  int ww_last = c.width - (g.grid_w - 1) * c.patch_w;
  g.n_take[0] = tokens_per_patch(c.ratio, c.patch_h * c.patch_w);
  g.n_take[1] = tokens_per_patch(c.ratio, c.patch_h * ww_last);
  g.n_take[2] = tokens_per_patch(c.ratio, hh_last * c.patch_w);
  g.n_take[3] = tokens_per_patch(c.ratio, hh_last * ww_last);
  g.take_per_full_row = (g.grid_w - 1) * g.n_take[0] + g.n_take[1];
  int last_row = (g.grid_w - 1) * g.n_take[2] + g.n_take[3];
  g.take_per_frame = (g.grid_h - 1) * g.take_per_full_row + last_row;
  g.n_sel = c.frames * g.take_per_frame;
  return g;
}

struct Layout {
  int64_t n_tokens, n_video, n_pad;
  size_t ages_off;
  bool kv_all, prev_all;         // HERO_CACHE_*: K/V^T on deep layers too, S_prev on shallow layers too
  size_t s_bytes, k_bytes, vt_bytes;
  size_t t_off[2], t_bytes;      // fp32 sums of the deep layers' features (two generations); 0 bytes if < 2 deep layers
  size_t rope_off, rope_bytes;   // (cos, sin) of every video token's rotation angles; 0 bytes without HERO_BLOCK_ROPE
  size_t cache_bytes;
  // workspace
  size_t idx_off, a_off, q_off, o_off, f_off, ktmp_off, vtmp_off, splitk_off, splitk_bytes, ws_bytes;
  size_t seen_off, seen_bytes;   // index check: one bit per token, then one verdict word
  size_t stat_off;               // counters (word 0: attention workgroups that took the running-maximum path)
  // bytes of one layer's slabs: S_cur, then K and V^T if it keeps them, then S_prev if it keeps one
  bool keeps_kv(const hero_config& c, int l) const { return l < c.n_shallow || kv_all; }
  bool keeps_prev(const hero_config& c, int l) const { return l >= c.n_shallow || prev_all; }
  size_t layer_bytes(const hero_config& c, int l) const {
    return s_bytes + (keeps_kv(c, l) ? k_bytes + vt_bytes : 0) + (keeps_prev(c, l) ? s_bytes : 0);
  }
};

Layout make_layout(const hero_config& c) {
  Layout L;
  L.n_video = (int64_t)c.frames * c.height * c.width;
  L.n_tokens = L.n_video + c.n_text;
  L.n_pad = (int64_t)align_up((size_t)L.n_tokens, 64);
  L.s_bytes = align_up((size_t)L.n_tokens * c.hidden * 2, 256);
  L.k_bytes = L.s_bytes;
  L.vt_bytes = align_up((size_t)c.hidden * L.n_pad * 2, 256);
  L.ages_off = 0;
  size_t off = align_up((size_t)L.n_video * 4, 256);
  L.kv_all = (c.cache_flags & HERO_CACHE_KV_ALL_LAYERS) != 0;
  L.prev_all = (c.cache_flags & HERO_CACHE_PREV_ALL_LAYERS) != 0;
  for (int l = 0; l < c.n_layers; ++l) off += L.layer_bytes(c, l);
  L.t_bytes = (c.n_layers - c.n_shallow >= 2) ? align_up((size_t)L.n_tokens * c.hidden * 4, 256) : 0;
  L.t_off[0] = off; off += L.t_bytes;
  L.t_off[1] = off; off += L.t_bytes;
  L.rope_bytes = (c.block_flags & HERO_BLOCK_ROPE) ? align_up((size_t)L.n_video * (c.head_dim / 2) * sizeof(float2), 256) : 0;
  L.rope_off = off; off += L.rope_bytes;
  L.cache_bytes = off;
  size_t w = 0;
  L.idx_off = w; w += align_up((size_t)L.n_tokens * 4, 256);
  L.a_off = w; w += L.s_bytes;
  L.q_off = w; w += L.s_bytes;
  L.o_off = w; w += L.s_bytes;
  L.f_off = w; w += align_up((size_t)L.n_tokens * c.ffn_dim * 2, 256);
  L.ktmp_off = w; L.vtmp_off = w;
  if (c.n_shallow < c.n_layers && !L.kv_all) {       // transient K / V^T of a deep layer's full step
    w += L.k_bytes;
    L.vtmp_off = w;
    w += L.vt_bytes;
  }
  // partial sums of GEMM tiles cut along k: up to 512 blocks of 256 x 256 fp32 (large problems only)
  L.splitk_off = w;
  L.splitk_bytes = L.n_tokens >= 2048 ? (size_t)512 * 262144 : 0;
  w += L.splitk_bytes;
  L.seen_off = w;
  L.seen_bytes = align_up(((size_t)L.n_tokens + 31) / 32 * 4 + 4, 256);
  w += L.seen_bytes;
  L.stat_off = w;
  w += 256;
  L.ws_bytes = w;
  return L;
}

struct Profiler {
  struct Rec { int slot; size_t e0, e1; double work; };
  bool on = false;
  uint32_t mask = 0xffffffffu;       // kinds that are bracketed while on
  std::vector<hipEvent_t> pool;
  size_t used = 0;
  std::vector<Rec> recs;
  hipError_t next(hipEvent_t* ev, size_t* id) {
    if (used == pool.size()) {
      hipEvent_t e;
      hipError_t rc = hipEventCreate(&e);
      if (rc != hipSuccess) return rc;
      pool.push_back(e);
    }
    *id = used;
    *ev = pool[used++];
    return hipSuccess;
  }
  ~Profiler() { for (hipEvent_t e : pool) (void)hipEventDestroy(e); }
};

struct LayerState {
  bf16_t* s_cur = nullptr;
  bf16_t* s_prev = nullptr;   // deep layers (every layer with HERO_CACHE_PREV_ALL_LAYERS)
  bf16_t* k = nullptr;        // shallow layers (every layer with HERO_CACHE_KV_ALL_LAYERS)
  bf16_t* vt = nullptr;
  int fills = 0;
  bool has_weights = false;
  hero_layer_weights w;
};

}  // namespace

struct hero_cache {
  hero_config cfg;
  Layout lay;
  SelectGeom geom;
  char* cache = nullptr;
  char* ws = nullptr;
  int32_t* ages = nullptr;
  int32_t* idx = nullptr;
  bf16_t *a = nullptr, *q = nullptr, *o = nullptr, *f = nullptr, *ktmp = nullptr, *vtmp = nullptr;
  float* splitk = nullptr;        // GEMM k-split partial sums (nullptr when the problem is too small to need them)
  uint32_t* seen = nullptr;       // index check: token bitmap followed by the verdict word
  uint32_t* stats = nullptr;      // word 0: attention fallback workgroups since create / reset
  float2* rope = nullptr;         // rotation table (nullptr without HERO_BLOCK_ROPE)
  std::vector<LayerState> layers;
  // deep-stack sums: slot i holds sum_l S_cur^l taken when the deep layers' fill counts were
  // t_key[i] (t_is_prev[i] false), or the matching previous-generation sum (t_is_prev[i] true)
  float* t[2] = {nullptr, nullptr};
  std::vector<int> t_key[2];
  bool t_is_prev[2] = {false, false};
  int n_full = 0;
  int last_full = -1;
  int last_n_sel = 0;
  Profiler prof;
  bool in_full = false;   // launches come from hero_full_layer (profiling slot selection)
};

namespace {

int check_handle(hero_cache_t c) {
  if (!c) return fail(HERO_ERR_INVALID_ARG, "cache handle is null");
  return HERO_OK;
}

int check_layer(hero_cache_t c, int layer) {
  if (layer < 0 || layer >= c->cfg.n_layers)
    return fail(HERO_ERR_INVALID_ARG, "layer %d out of range [0, %d)", layer, c->cfg.n_layers);
  return HERO_OK;
}

// Launch `expr` on stream `st`; when profiling is on, bracket it with events.
#define PROF_LAUNCH(c, kind, work_, st, expr)                                        \
  do {                                                                               \
    if ((c)->prof.on && (((c)->prof.mask >> (kind)) & 1u)) {                         \
      hipEvent_t e0_, e1_; size_t i0_, i1_;                                          \
      HIP_TRY((c)->prof.next(&e0_, &i0_));                                           \
      HIP_TRY((c)->prof.next(&e1_, &i1_));                                           \
      HIP_TRY(hipEventRecord(e0_, st));                                              \
      HIP_TRY(expr);                                                                 \
      HIP_TRY(hipEventRecord(e1_, st));                                              \
      (c)->prof.recs.push_back({(kind) + ((c)->in_full ? 0 : HERO_PROF_KINDS), i0_, i1_, (double)(work_)}); \
    } else {                                                                         \
      HIP_TRY(expr);                                                                 \
    }                                                                                \
  } while (0)

// The block of Eq. 2 on the rows listed in `rows` (nullptr = all N rows), writing K/V to
// (k_dst, vt_dst) and the branch features to s_dst.  It ends before the residual add, unless
// fuse_resid is given and the FFN2 kernel can add the stored features of its rows to x itself
// (then *fuse_resid is set; only valid when the listed rows are all the rows x += S applies to).
int run_block_rows(hero_cache_t c, LayerState& ls, void* x, const int32_t* rows, int n_rows, bf16_t* k_dst,
                   bf16_t* vt_dst, bf16_t* s_dst, hipStream_t st, bool* fuse_resid = nullptr) {
  const hero_config& cfg = c->cfg;
  const bool x_fp32 = cfg.resid_dtype == HERO_DTYPE_FP32;
  const int d = cfg.hidden;
  const hero_layer_weights& w = ls.w;
  const double xsz = x_fp32 ? 4.0 : 2.0;
  const double rd = (double)n_rows * d;
  const double n_all = (double)c->lay.n_tokens;
  // modulated block: rows of the modulation table (d elements each): shift, scale, gate of the
  // attention branch for the video stream, then for the text stream, then the same six for the FFN
  const bool adaln = (cfg.block_flags & HERO_BLOCK_ADALN) != 0;
  const bool qk_post = (cfg.block_flags & (HERO_BLOCK_QKNORM | HERO_BLOCK_ROPE)) != 0;
  const bf16_t* mod = (const bf16_t*)w.mod;
  LnMod m1, m2;
  if (adaln) {
    m1.shift_v = mod + 0 * d; m1.scale_v = mod + 1 * d; m1.shift_t = mod + 3 * d; m1.scale_t = mod + 4 * d;
    m2.shift_v = mod + 6 * d; m2.scale_v = mod + 7 * d; m2.shift_t = mod + 9 * d; m2.scale_t = mod + 10 * d;
    m1.n_text = m2.n_text = cfg.n_text;
  }
  PROF_LAUNCH(c, HERO_PROF_LN, rd * (xsz + 2.0), st,
              launch_gather_ln(x, x_fp32, nullptr, rows, n_rows, d, (const bf16_t*)w.ln1_g,
                               (const bf16_t*)w.ln1_b, cfg.ln_eps, c->a, st, m1));
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.a = c->a; g.w = (const bf16_t*)w.w_qkv; g.bias = (const bf16_t*)w.b_qkv;
  g.m = n_rows; g.n = 3 * d; g.k = d; g.epilogue = EPI_QKV; g.rows = rows;
  g.c = c->q; g.k_out = k_dst; g.vt_out = vt_dst; g.ld_vt = c->lay.n_pad; g.d = d;
  // softmax scale and the change to base 2 are folded into Q before its single bf16 rounding
  // (with q/k post-processing the scale is applied there, after the normalisation and rotation)
  const float softmax_scale = 1.4426950408889634f / sqrtf((float)cfg.head_dim);
  g.q_scale = qk_post ? 1.0f : softmax_scale;
  g.splitk_ws = c->splitk; g.splitk_ws_bytes = c->lay.splitk_bytes;
  PROF_LAUNCH(c, HERO_PROF_GEMM_QKV, 6.0 * rd * d, st, launch_gemm(g, st));
  if (qk_post) {
    QkPostArgs qa;
    memset(&qa, 0, sizeof(qa));
    qa.q = c->q; qa.k = k_dst; qa.rows = rows; qa.n_rows = n_rows; qa.d = d; qa.head_dim = cfg.head_dim;
    qa.n_text = cfg.n_text; qa.q_scale = softmax_scale;
    if (cfg.block_flags & HERO_BLOCK_QKNORM) {
      qa.qn_g = (const bf16_t*)w.q_norm_g; qa.qn_b = (const bf16_t*)w.q_norm_b;
      qa.kn_g = (const bf16_t*)w.k_norm_g; qa.kn_b = (const bf16_t*)w.k_norm_b;
    }
    if (cfg.block_flags & HERO_BLOCK_ROPE) qa.rope = c->rope;
    PROF_LAUNCH(c, HERO_PROF_QKPOST, rd * 8.0, st, launch_qk_post(qa, st));      // q and k rows, in and out
  }

  AttnArgs at;
  at.q = c->q; at.k = k_dst; at.vt = vt_dst; at.ld_vt = c->lay.n_pad; at.o = c->o;
  at.r = n_rows; at.n_keys = (int)c->lay.n_tokens; at.n_heads = cfg.n_heads; at.head_dim = cfg.head_dim;
  at.q_scale = 1.0f;
  at.split_ws = c->splitk; at.split_ws_bytes = c->lay.splitk_bytes;    // shared with the GEMMs: same stream, never concurrent
  at.fallback_count = c->stats;
  PROF_LAUNCH(c, HERO_PROF_ATTN, 4.0 * rd * n_all, st, launch_attention(at, st));

  memset(&g, 0, sizeof(g));
  g.a = c->o; g.w = (const bf16_t*)w.w_o; g.bias = (const bf16_t*)w.b_o;
  g.m = n_rows; g.n = d; g.k = d; g.epilogue = EPI_SCATTER; g.rows = rows; g.c = s_dst;
  if (adaln) { g.gate_v = mod + 2 * d; g.gate_t = mod + 5 * d; g.n_text = cfg.n_text; }
  g.splitk_ws = c->splitk; g.splitk_ws_bytes = c->lay.splitk_bytes;
  PROF_LAUNCH(c, HERO_PROF_GEMM_O, 2.0 * rd * d, st, launch_gemm(g, st));

  PROF_LAUNCH(c, HERO_PROF_LN, rd * (xsz + 4.0), st,
              launch_gather_ln(x, x_fp32, s_dst, rows, n_rows, d, (const bf16_t*)w.ln2_g,
                               (const bf16_t*)w.ln2_b, cfg.ln_eps, c->a, st, m2));
  memset(&g, 0, sizeof(g));
  g.a = c->a; g.w = (const bf16_t*)w.w_ff1; g.bias = (const bf16_t*)w.b_ff1;
  g.m = n_rows; g.n = cfg.ffn_dim; g.k = d; g.epilogue = EPI_GELU; g.c = c->f;
  g.splitk_ws = c->splitk; g.splitk_ws_bytes = c->lay.splitk_bytes;
  PROF_LAUNCH(c, HERO_PROF_GEMM_FF1, 2.0 * rd * cfg.ffn_dim, st, launch_gemm(g, st));

  memset(&g, 0, sizeof(g));
  g.a = c->f; g.w = (const bf16_t*)w.w_ff2; g.bias = (const bf16_t*)w.b_ff2;
  g.m = n_rows; g.n = d; g.k = cfg.ffn_dim; g.epilogue = EPI_SCATTER_ADD; g.rows = rows; g.c = s_dst;
  if (adaln) { g.gate_v = mod + 8 * d; g.gate_t = mod + 11 * d; g.n_text = cfg.n_text; }
  if (fuse_resid != nullptr) {
    *fuse_resid = gemm_can_update_x(g);
    if (*fuse_resid) { g.x = x; g.x_fp32 = x_fp32 ? 1 : 0; }
  }
  g.splitk_ws = c->splitk; g.splitk_ws_bytes = c->lay.splitk_bytes;
  PROF_LAUNCH(c, HERO_PROF_GEMM_FF2, 2.0 * rd * cfg.ffn_dim, st, launch_gemm(g, st));
  return HERO_OK;
}

// Sums the listed feature arrays into t (fp32), 48 arrays per launch.
int sum_feature_arrays(hero_cache_t c, const std::vector<const bf16_t*>& src, float* t, hipStream_t st) {
  const int64_t n_elems = c->lay.n_tokens * c->cfg.hidden;
  for (size_t i = 0; i < src.size(); i += 48) {
    FeatureList fl;
    fl.n = (int)std::min<size_t>(48, src.size() - i);
    for (int j = 0; j < fl.n; ++j) fl.p[j] = src[i + j];
    const double bytes = (double)n_elems * (2.0 * fl.n + (i ? 8.0 : 4.0));
    PROF_LAUNCH(c, HERO_PROF_DEEPSUM, bytes, st, launch_sum_features(fl, t, i != 0, n_elems, st));
  }
  return HERO_OK;
}

// The deep layers of a cached step in one pass (Eq. 5 summed over l >= K):
//   x += (1 + k/M) T_cur - (k/M) T_prev,  T_cur = sum_l S_t^l,  T_prev = sum_l (S_{t+M}^l, or S_t^l
// for a layer that has only one generation, which then contributes no difference).
// The sums are cached per state of the deep layers' fill counts and recomputed when it changes;
// the current sum of one generation serves as the previous sum of the next.
// Makes the fp32 sums over the deep layers current (recomputing what a re-fill made stale);
// *cur / *prev: which of the two arrays holds the sum of S_cur / of S_prev (-1: no previous generation).
int ensure_deep_sums(hero_cache_t c, hipStream_t st, int* cur_out, int* prev_out) {
  const hero_config& cfg = c->cfg;
  std::vector<int> fills;
  bool any_prev = false;
  for (int l = cfg.n_shallow; l < cfg.n_layers; ++l) {
    if (c->layers[l].fills == 0) return fail(HERO_ERR_STATE, "layer %d extrapolated before a full step filled its cache", l);
    fills.push_back(c->layers[l].fills);
    any_prev = any_prev || c->layers[l].fills >= 2;
  }
  std::vector<int> fills_before(fills);
  for (int& f : fills_before) f -= 1;
  auto is_cur = [&](int i) { return !c->t_is_prev[i] && c->t_key[i] == fills; };
  auto is_prev = [&](int i) {
    return (c->t_is_prev[i] && c->t_key[i] == fills) || (!c->t_is_prev[i] && c->t_key[i] == fills_before);
  };
  int cur = is_cur(0) ? 0 : is_cur(1) ? 1 : -1;
  int prev = !any_prev ? -1 : is_prev(0) ? 0 : is_prev(1) ? 1 : -1;
  int rc;
  if (cur < 0) {
    cur = prev == 0 ? 1 : 0;
    std::vector<const bf16_t*> src;
    for (int l = cfg.n_shallow; l < cfg.n_layers; ++l) src.push_back(c->layers[l].s_cur);
    c->t_key[cur].clear();
    if ((rc = sum_feature_arrays(c, src, c->t[cur], st)) != HERO_OK) return rc;
    c->t_key[cur] = fills; c->t_is_prev[cur] = false;
  }
  if (any_prev && prev < 0) {
    prev = cur ^ 1;
    std::vector<const bf16_t*> src;
    for (int l = cfg.n_shallow; l < cfg.n_layers; ++l)
      src.push_back(c->layers[l].fills >= 2 ? c->layers[l].s_prev : c->layers[l].s_cur);
    c->t_key[prev].clear();
    if ((rc = sum_feature_arrays(c, src, c->t[prev], st)) != HERO_OK) return rc;
    c->t_key[prev] = fills; c->t_is_prev[prev] = true;
  }
  *cur_out = cur;
  *prev_out = any_prev ? prev : -1;
  return HERO_OK;
}

int apply_deep_stack(hero_cache_t c, void* x, int k, hipStream_t st) {
  const hero_config& cfg = c->cfg;
  int cur, prev;
  int rc = ensure_deep_sums(c, st, &cur, &prev);
  if (rc) return rc;
  const bool x_fp32 = cfg.resid_dtype == HERO_DTYPE_FP32;
  const int64_t n_elems = c->lay.n_tokens * cfg.hidden;
  const float alpha = (float)k / (float)cfg.interval;
  const double bytes = (double)n_elems * ((x_fp32 ? 8.0 : 4.0) + (prev >= 0 ? 8.0 : 4.0));
  PROF_LAUNCH(c, HERO_PROF_EXTRAP, bytes, st,
              launch_apply_sums(x, x_fp32, c->t[cur], prev >= 0 ? c->t[prev] : nullptr, alpha, n_elems, st));
  return HERO_OK;
}

// Refresh of one shallow layer inside a cached step whose residual adds are deferred to the end
// of the step: only the refreshed rows of x are updated here (by the FFN2 epilogue).
int refresh_layer_deferred(hero_cache_t c, int layer, void* x, const int32_t* idx, int n_sel, hipStream_t st) {
  LayerState& ls = c->layers[layer];
  if (!ls.has_weights) return fail(HERO_ERR_STATE, "layer %d has no weights", layer);
  if (ls.fills == 0) return fail(HERO_ERR_STATE, "layer %d refreshed before a full step filled its cache", layer);
  if (n_sel <= 0) return HERO_OK;
  bool fused = false;
  int rc = run_block_rows(c, ls, x, idx, n_sel, ls.k, ls.vt, ls.s_cur, st, &fused);
  if (rc) return rc;
  if (!fused) return fail(HERO_ERR_STATE, "internal: the FFN2 kernel did not take the residual update");
  return HERO_OK;
}

// Whether a cached step with n_sel refreshed rows can defer its residual adds: the FFN2 kernel
// must be the one that updates x for its rows.
bool can_defer_residual(hero_cache_t c, int n_sel) {
  const hero_config& cfg = c->cfg;
  if (cfg.n_shallow < 1 || cfg.n_shallow > 48) return false;
  if (n_sel == 0) return true;
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.m = n_sel; g.n = cfg.hidden; g.k = cfg.ffn_dim; g.epilogue = EPI_SCATTER_ADD;
  return gemm_can_update_x(g);
}

// The deferred adds of a cached step (see end_of_cached_step_kernel), incl. the deep stack when it
// has fp32 sums (two or more deep layers).
int end_of_cached_step(hero_cache_t c, void* x, int k, int n_sel, hipStream_t st) {
  const hero_config& cfg = c->cfg;
  const int n_deep = cfg.n_layers - cfg.n_shallow;
  int cur = -1, prev = -1;
  if (n_deep >= 2) {
    int rc = ensure_deep_sums(c, st, &cur, &prev);
    if (rc) return rc;
  }
  FeatureList fl;
  fl.n = cfg.n_shallow;
  for (int l = 0; l < cfg.n_shallow; ++l) fl.p[l] = c->layers[l].s_cur;
  const bool x_fp32 = cfg.resid_dtype == HERO_DTYPE_FP32;
  const int64_t n_elems = c->lay.n_tokens * cfg.hidden;
  const float alpha = (float)k / (float)cfg.interval;
  const double bytes = (double)n_elems * (x_fp32 ? 8.0 : 4.0) +
                       (double)(c->lay.n_tokens - n_sel) * cfg.hidden * 2.0 * cfg.n_shallow +
                       (cur >= 0 ? (double)n_elems * (prev >= 0 ? 8.0 : 4.0) : 0.0);
  PROF_LAUNCH(c, HERO_PROF_EXTRAP, bytes, st,
              launch_end_of_cached_step(x, x_fp32, fl, c->ages, cfg.n_text, cfg.hidden, cur >= 0 ? c->t[cur] : nullptr,
                                        prev >= 0 ? c->t[prev] : nullptr, alpha, n_elems, st));
  return HERO_OK;
}

}  // namespace

extern "C" {

const char* hero_last_error(void) { return g_err; }

int hero_num_selected(const hero_config* cfg, int32_t* n_sel_host) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!n_sel_host) return fail(HERO_ERR_INVALID_ARG, "n_sel_host is null");
  *n_sel_host = make_geom(*cfg).n_sel;
  return HERO_OK;
}

int hero_cache_bytes(const hero_config* cfg, size_t* cache_bytes, size_t* workspace_bytes) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!cache_bytes || !workspace_bytes) return fail(HERO_ERR_INVALID_ARG, "output pointer is null");
  Layout L = make_layout(*cfg);
  *cache_bytes = L.cache_bytes;
  *workspace_bytes = L.ws_bytes;
  return HERO_OK;
}

int hero_cache_create(const hero_config* cfg, void* dev_cache, size_t cache_bytes, void* dev_workspace,
                      size_t workspace_bytes, void* stream, hero_cache_t* out) {
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!dev_cache || !dev_workspace || !out) return fail(HERO_ERR_INVALID_ARG, "null buffer or output pointer");
  if (((uintptr_t)dev_cache | (uintptr_t)dev_workspace) & 255)
    return fail(HERO_ERR_INVALID_ARG, "cache and workspace buffers must be 256-byte aligned");
  Layout L = make_layout(*cfg);
  if (cache_bytes < L.cache_bytes)
    return fail(HERO_ERR_BUFFER_TOO_SMALL, "cache buffer has %zu bytes, %zu needed", cache_bytes, L.cache_bytes);
  if (workspace_bytes < L.ws_bytes)
    return fail(HERO_ERR_BUFFER_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, L.ws_bytes);
  hero_cache* c = new (std::nothrow) hero_cache();
  if (!c) return fail(HERO_ERR_INVALID_ARG, "out of host memory");
  c->cfg = *cfg;
  c->lay = L;
  c->geom = make_geom(*cfg);
  c->cache = (char*)dev_cache;
  c->ws = (char*)dev_workspace;
  c->ages = (int32_t*)(c->cache + L.ages_off);
  c->idx = (int32_t*)(c->ws + L.idx_off);
  c->a = (bf16_t*)(c->ws + L.a_off);
  c->q = (bf16_t*)(c->ws + L.q_off);
  c->o = (bf16_t*)(c->ws + L.o_off);
  c->f = (bf16_t*)(c->ws + L.f_off);
  c->ktmp = (bf16_t*)(c->ws + L.ktmp_off);
  c->vtmp = (bf16_t*)(c->ws + L.vtmp_off);
  c->splitk = L.splitk_bytes ? (float*)(c->ws + L.splitk_off) : nullptr;
  c->seen = (uint32_t*)(c->ws + L.seen_off);
  c->stats = (uint32_t*)(c->ws + L.stat_off);
  c->layers.resize(cfg->n_layers);
  if (L.t_bytes) { c->t[0] = (float*)(c->cache + L.t_off[0]); c->t[1] = (float*)(c->cache + L.t_off[1]); }
  if (L.rope_bytes) c->rope = (float2*)(c->cache + L.rope_off);
  size_t off = align_up((size_t)L.n_video * 4, 256);
  for (int l = 0; l < cfg->n_layers; ++l) {
    LayerState& ls = c->layers[l];
    size_t o = off;
    ls.s_cur = (bf16_t*)(c->cache + o); o += L.s_bytes;
    if (L.keeps_kv(*cfg, l)) {
      ls.k = (bf16_t*)(c->cache + o); o += L.k_bytes;
      ls.vt = (bf16_t*)(c->cache + o); o += L.vt_bytes;
    }
    if (L.keeps_prev(*cfg, l)) { ls.s_prev = (bf16_t*)(c->cache + o); o += L.s_bytes; }
    off += L.layer_bytes(*cfg, l);
  }
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = hipMemsetAsync(dev_cache, 0, L.cache_bytes, st);
  if (e == hipSuccess) e = hipMemsetAsync(dev_workspace, 0, L.ws_bytes, st);
  if (e == hipSuccess && c->rope)
    e = launch_rope_table(c->rope, cfg->frames, cfg->height, cfg->width, cfg->head_dim, st);
  if (e != hipSuccess) {
    delete c;
    return fail(HERO_ERR_HIP, "cache set-up: %s", hipGetErrorString(e));
  }
  *out = c;
  return HERO_OK;
}

int hero_cache_destroy(hero_cache_t c) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  delete c;
  return HERO_OK;
}

int hero_reset_ages(hero_cache_t c, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  HIP_TRY(launch_fill_i32(c->ages, 0, c->lay.n_video, (hipStream_t)stream));
  return HERO_OK;
}

int hero_cache_reset(hero_cache_t c, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  for (auto& ls : c->layers) ls.fills = 0;
  c->t_key[0].clear(); c->t_key[1].clear();
  c->n_full = 0;
  c->last_full = -1;
  c->last_n_sel = 0;
  HIP_TRY(launch_fill_i32(reinterpret_cast<int32_t*>(c->stats), 0, 1, (hipStream_t)stream));
  return hero_reset_ages(c, stream);
}

int hero_set_layer_weights(hero_cache_t c, int32_t layer, const hero_layer_weights* w) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!w) return fail(HERO_ERR_INVALID_ARG, "weights pointer is null");
  const void* const* p = reinterpret_cast<const void* const*>(w);
  const int flags = c->cfg.block_flags;
  for (size_t i = 0; i < sizeof(*w) / sizeof(void*); ++i) {
    const bool needed = i < 12 || (i < 16 ? (flags & HERO_BLOCK_QKNORM) != 0 : (flags & HERO_BLOCK_ADALN) != 0);
    if (!needed) continue;
    if (!p[i]) return fail(HERO_ERR_INVALID_ARG, "weight pointer %zu of layer %d is null", i, layer);
    if ((uintptr_t)p[i] & 15) return fail(HERO_ERR_INVALID_ARG, "weight pointer %zu of layer %d is not 16-byte aligned", i, layer);
  }
  c->layers[layer].w = *w;
  c->layers[layer].has_weights = true;
  return HERO_OK;
}

int hero_full_layer(hero_cache_t c, int32_t layer, void* dev_x, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!dev_x) return fail(HERO_ERR_INVALID_ARG, "x is null");
  LayerState& ls = c->layers[layer];
  if (!ls.has_weights) return fail(HERO_ERR_STATE, "layer %d has no weights", layer);
  hipStream_t st = (hipStream_t)stream;
  // A layer that keeps two generations writes the new one over the older (G_{t+M} <- G_t, Sec. 3.4)
  // and the two change places only once every launch has been accepted.
  const bool rotate = ls.s_prev != nullptr && ls.fills > 0;
  bf16_t* s_dst = rotate ? ls.s_prev : ls.s_cur;
  bf16_t* k_dst = ls.k ? ls.k : c->ktmp;
  bf16_t* vt_dst = ls.vt ? ls.vt : c->vtmp;
  c->in_full = true;
  bool resid_done = false;
  rc = run_block_rows(c, ls, dev_x, nullptr, (int)c->lay.n_tokens, k_dst, vt_dst, s_dst, st, &resid_done);
  const bool x_fp32 = c->cfg.resid_dtype == HERO_DTYPE_FP32;
  const double nd = (double)c->lay.n_tokens * c->cfg.hidden;
  if (rc == HERO_OK)
    rc = [&]() -> int {
      if (resid_done) return HERO_OK;
      PROF_LAUNCH(c, HERO_PROF_RESID, nd * (x_fp32 ? 10.0 : 6.0), st,
                  launch_axpy_features(dev_x, x_fp32, s_dst, nullptr, 0.f, c->lay.n_tokens * c->cfg.hidden, st));
      return HERO_OK;
    }();
  c->in_full = false;
  if (rc) {
    // the slab written to may hold part of a new generation: what it held before is gone
    ls.fills = rotate ? 1 : 0;
    c->t_key[0].clear(); c->t_key[1].clear();      // and no sum over the deep layers is current any more
    return rc;
  }
  if (rotate) std::swap(ls.s_cur, ls.s_prev);
  ls.fills += 1;
  return HERO_OK;
}

int hero_select(hero_cache_t c, int32_t step, int32_t* dev_idx, int32_t* n_sel_host, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  if (step < 0) return fail(HERO_ERR_INVALID_ARG, "step must be >= 0");
  if (!dev_idx && c->geom.n_sel > 0) return fail(HERO_ERR_INVALID_ARG, "dev_idx is null");
  uint64_t seed = c->cfg.seed;
  uint32_t s0 = (uint32_t)seed ^ (uint32_t)(seed >> 32);
  uint32_t salt = fmix32_host(s0 + 0x9E3779B9u * ((uint32_t)step + 1u));
  PROF_LAUNCH(c, HERO_PROF_SELECT, 8.0 * c->lay.n_video + 4.0 * c->geom.n_sel, (hipStream_t)stream,
              launch_select(c->geom, c->cfg.select_mode, salt, c->ages, dev_idx, (hipStream_t)stream));
  if (n_sel_host) *n_sel_host = c->geom.n_sel;
  return HERO_OK;
}

int hero_refresh_layer(hero_cache_t c, int32_t layer, void* dev_x, const int32_t* dev_idx, int32_t n_sel,
                       void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!dev_x) return fail(HERO_ERR_INVALID_ARG, "x is null");
  LayerState& ls = c->layers[layer];
  if (ls.k == nullptr)
    return fail(HERO_ERR_INVALID_ARG, "layer %d is a deep layer (n_shallow = %d) and keeps no K/V cache "
                "(configure HERO_CACHE_KV_ALL_LAYERS to refresh it)", layer, c->cfg.n_shallow);
  if (n_sel < 0 || n_sel > c->lay.n_tokens) return fail(HERO_ERR_INVALID_ARG, "n_sel %d out of range", n_sel);
  if (n_sel > 0 && !dev_idx) return fail(HERO_ERR_INVALID_ARG, "dev_idx is null");
  if (!ls.has_weights) return fail(HERO_ERR_STATE, "layer %d has no weights", layer);
  if (ls.fills == 0) return fail(HERO_ERR_STATE, "layer %d refreshed before a full step filled its cache", layer);
  hipStream_t st = (hipStream_t)stream;
  if ((c->cfg.debug_flags & HERO_DEBUG_CHECK_IDX) && n_sel > 0) {
    // before anything is scattered: are the listed rows distinct and inside [0, N)?
    const int n_tok = (int)c->lay.n_tokens;
    HIP_TRY(launch_check_idx(dev_idx, n_sel, n_tok, c->seen, st));
    uint32_t verdict = 0;
    HIP_TRY(hipMemcpyAsync(&verdict, c->seen + (n_tok + 31) / 32, sizeof(verdict), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (verdict != 0)
      return fail(HERO_ERR_INVALID_ARG, "dev_idx holds %s%s%s", (verdict & 1) ? "a row outside [0, N)" : "",
                  verdict == 3 ? " and " : "", (verdict & 2) ? "a row listed twice" : "");
  }
  if (n_sel > 0) {
    rc = run_block_rows(c, ls, dev_x, dev_idx, n_sel, ls.k, ls.vt, ls.s_cur, st);
    if (rc) return rc;
  }
  const bool x_fp32 = c->cfg.resid_dtype == HERO_DTYPE_FP32;
  PROF_LAUNCH(c, HERO_PROF_RESID, (double)c->lay.n_tokens * c->cfg.hidden * (x_fp32 ? 10.0 : 6.0), st,
              launch_axpy_features(dev_x, x_fp32, ls.s_cur, nullptr, 0.f, c->lay.n_tokens * c->cfg.hidden, st));
  return HERO_OK;
}

int hero_extrapolate_layer(hero_cache_t c, int32_t layer, void* dev_x, int32_t k, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  int rc = check_layer(c, layer);
  if (rc) return rc;
  if (!dev_x) return fail(HERO_ERR_INVALID_ARG, "x is null");
  LayerState& ls = c->layers[layer];
  if (ls.s_prev == nullptr)
    return fail(HERO_ERR_INVALID_ARG, "layer %d is a shallow layer (n_shallow = %d) and keeps one generation "
                "(configure HERO_CACHE_PREV_ALL_LAYERS to extrapolate it)", layer, c->cfg.n_shallow);
  if (k < 0 || k > c->cfg.interval) return fail(HERO_ERR_INVALID_ARG, "k = %d outside [0, %d]", k, c->cfg.interval);
  if (ls.fills == 0) return fail(HERO_ERR_STATE, "layer %d extrapolated before a full step filled its cache", layer);
  const bf16_t* prev = ls.fills >= 2 ? ls.s_prev : nullptr;
  float alpha = (float)k / (float)c->cfg.interval;
  const bool x_fp32 = c->cfg.resid_dtype == HERO_DTYPE_FP32;
  // algorithmic bytes: x in, x out, S_t and (when it exists) S_{t+M}
  const double bytes = (double)c->lay.n_tokens * c->cfg.hidden * ((x_fp32 ? 8.0 : 4.0) + (prev ? 4.0 : 2.0));
  PROF_LAUNCH(c, HERO_PROF_EXTRAP, bytes, (hipStream_t)stream,
              launch_axpy_features(dev_x, x_fp32, ls.s_cur, prev, alpha, c->lay.n_tokens * c->cfg.hidden,
                                   (hipStream_t)stream));
  return HERO_OK;
}

int hero_step(hero_cache_t c, void* dev_x, int32_t step, void* stream) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  if (!dev_x) return fail(HERO_ERR_INVALID_ARG, "x is null");
  if (step < 0) return fail(HERO_ERR_INVALID_ARG, "step must be >= 0");
  const hero_config& cfg = c->cfg;
  int rc;
  if (step % cfg.interval == 0) {
    for (int l = 0; l < cfg.n_layers; ++l)
      if ((rc = hero_full_layer(c, l, dev_x, stream)) != HERO_OK) {
        // layers before l hold the new generation, the others the old one: no cached step until a
        // full step has gone through
        c->n_full = 0;
        c->last_full = -1;
        return rc;
      }
    if ((rc = hero_reset_ages(c, stream)) != HERO_OK) return rc;
    c->n_full += 1;
    c->last_full = step;
    c->last_n_sel = 0;
    return HERO_OK;
  }
  if (c->n_full == 0) return fail(HERO_ERR_STATE, "cached step %d before any full step", step);
  int k = step - c->last_full;
  if (k < 1 || k > cfg.interval) return fail(HERO_ERR_STATE, "step %d is %d steps after the last full step %d", step, k, c->last_full);
  int32_t n_sel = 0;
  if ((rc = hero_select(c, step, c->idx, &n_sel, stream)) != HERO_OK) return rc;
  c->last_n_sel = n_sel;
  const int n_deep = cfg.n_layers - cfg.n_shallow;
  if (can_defer_residual(c, n_sel)) {
    // Only the refreshed rows of x are needed between the shallow layers of a cached step, so the
    // residual adds of all other rows wait for one pass at the end of the step (together with the
    // deep stack): one launch instead of one per shallow layer.
    for (int l = 0; l < cfg.n_shallow; ++l)
      if ((rc = refresh_layer_deferred(c, l, dev_x, c->idx, n_sel, (hipStream_t)stream)) != HERO_OK) return rc;
    if ((rc = end_of_cached_step(c, dev_x, k, n_sel, (hipStream_t)stream)) != HERO_OK) return rc;
    if (n_deep == 1) return hero_extrapolate_layer(c, cfg.n_shallow, dev_x, k, stream);
    return HERO_OK;
  }
  for (int l = 0; l < cfg.n_shallow; ++l)
    if ((rc = hero_refresh_layer(c, l, dev_x, c->idx, n_sel, stream)) != HERO_OK) return rc;
  if (n_deep >= 2) return apply_deep_stack(c, dev_x, k, (hipStream_t)stream);
  for (int l = cfg.n_shallow; l < cfg.n_layers; ++l)
    if ((rc = hero_extrapolate_layer(c, l, dev_x, k, stream)) != HERO_OK) return rc;
  return HERO_OK;
}

int hero_cache_view(hero_cache_t c, int32_t layer, int32_t what, void** dev_ptr, int64_t* ld) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  if (!dev_ptr || !ld) return fail(HERO_ERR_INVALID_ARG, "output pointer is null");
  if (what == 4) { *dev_ptr = c->ages; *ld = c->lay.n_video; return HERO_OK; }
  if (what == 5) { *dev_ptr = c->idx; *ld = c->last_n_sel; return HERO_OK; }
  if (what == 6) { *dev_ptr = c->stats; *ld = 1; return HERO_OK; }
  int rc = check_layer(c, layer);
  if (rc) return rc;
  LayerState& ls = c->layers[layer];
  switch (what) {
    case 0: *dev_ptr = ls.s_cur; *ld = c->cfg.hidden; break;
    case 1: *dev_ptr = ls.s_prev; *ld = c->cfg.hidden; break;
    case 2: *dev_ptr = ls.k; *ld = c->cfg.hidden; break;
    case 3: *dev_ptr = ls.vt; *ld = c->lay.n_pad; break;
    default: return fail(HERO_ERR_INVALID_ARG, "unknown view %d", what);
  }
  if (!*dev_ptr) return fail(HERO_ERR_STATE, "layer %d keeps no such cache (view %d)", layer, what);
  return HERO_OK;
}

int hero_cache_state(hero_cache_t c, int32_t* n_full, int32_t* last_full_step) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  if (n_full) *n_full = c->n_full;
  if (last_full_step) *last_full_step = c->last_full;
  return HERO_OK;
}

int hero_profile_begin(hero_cache_t c) { return hero_profile_begin_kinds(c, 0xffffffffu); }

int hero_profile_begin_kinds(hero_cache_t c, uint32_t kind_mask) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  c->prof.on = true;
  c->prof.mask = kind_mask;
  c->prof.used = 0;
  c->prof.recs.clear();
  return HERO_OK;
}

int hero_profile_end(hero_cache_t c, void* stream, double* ms, int64_t* launches, double* work) {
  if (check_handle(c)) return HERO_ERR_INVALID_ARG;
  if (!c->prof.on) return fail(HERO_ERR_STATE, "hero_profile_end without hero_profile_begin");
  c->prof.on = false;
  HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
  for (int i = 0; i < 2 * HERO_PROF_KINDS; ++i) {
    if (ms) ms[i] = 0.0;
    if (launches) launches[i] = 0;
    if (work) work[i] = 0.0;
  }
  for (const Profiler::Rec& r : c->prof.recs) {
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, c->prof.pool[r.e0], c->prof.pool[r.e1]));
    if (ms) ms[r.slot] += (double)t;
    if (launches) launches[r.slot] += 1;
    if (work) work[r.slot] += r.work;
  }
  c->prof.recs.clear();
  c->prof.used = 0;
  return HERO_OK;
}

// ---- building blocks ---------------------------------------------------------------

int hero_gather_ln(const void* dev_x, int32_t x_dtype, const void* dev_add_bf16, const int32_t* dev_rows,
                   int32_t n_rows, int32_t hidden, const void* gain, const void* bias, float eps,
                   void* dev_out_bf16, void* stream) {
  // (the row buffers of an empty problem are never touched and may be null)
  if (!gain || !bias || (n_rows > 0 && (!dev_x || !dev_out_bf16))) return fail(HERO_ERR_INVALID_ARG, "null pointer");
  if (x_dtype != HERO_DTYPE_FP32 && x_dtype != HERO_DTYPE_BF16) return fail(HERO_ERR_INVALID_ARG, "bad x_dtype");
  if (n_rows < 0) return fail(HERO_ERR_INVALID_ARG, "n_rows < 0");
  if (hidden < 8 || hidden % 8 != 0 || hidden > 8192) return fail(HERO_ERR_SHAPE, "hidden must be a multiple of 8, <= 8192");
  if (!aligned16({dev_x, dev_add_bf16, gain, bias, dev_out_bf16}) || ((uintptr_t)dev_rows & 3))
    return fail(HERO_ERR_INVALID_ARG, "x, add, gain, bias and out must be 16-byte aligned, rows 4-byte aligned");
  HIP_TRY(launch_gather_ln(dev_x, x_dtype == HERO_DTYPE_FP32, (const bf16_t*)dev_add_bf16, dev_rows, n_rows, hidden,
                           (const bf16_t*)gain, (const bf16_t*)bias, eps, (bf16_t*)dev_out_bf16, (hipStream_t)stream));
  return HERO_OK;
}

static int check_linear_args(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c, int32_t m,
                             int32_t n, int32_t k, int32_t act) {
  if (!dev_w || !dev_bias || (m > 0 && (!dev_a || !dev_c))) return fail(HERO_ERR_INVALID_ARG, "null pointer");
  if (m < 0 || n <= 0 || k <= 0) return fail(HERO_ERR_INVALID_ARG, "bad sizes");
  if (k % 64 != 0 || n % 64 != 0) return fail(HERO_ERR_SHAPE, "k and n must be multiples of 64");
  if (act != 0 && act != 1) return fail(HERO_ERR_INVALID_ARG, "act must be 0 or 1");
  if (!gemm_offsets_fit(m, n, k))
    return fail(HERO_ERR_SHAPE, "(m + 512) * k * 2 and (n + 512) * k * 2 must stay below 2^32 (32-bit operand offsets)");
  if (!aligned16({dev_a, dev_w, dev_bias, dev_c})) return fail(HERO_ERR_INVALID_ARG, "a, w, bias and c must be 16-byte aligned");
  return HERO_OK;
}

int hero_linear_scratch(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c, int32_t m,
                        int32_t n, int32_t k, int32_t act, void* dev_scratch, size_t scratch_bytes, void* stream) {
  int rc = check_linear_args(dev_a, dev_w, dev_bias, dev_c, m, n, k, act);
  if (rc) return rc;
  if (!aligned16({dev_scratch})) return fail(HERO_ERR_INVALID_ARG, "scratch must be 16-byte aligned");
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.a = (const bf16_t*)dev_a; g.w = (const bf16_t*)dev_w; g.bias = (const bf16_t*)dev_bias;
  g.m = m; g.n = n; g.k = k; g.epilogue = act ? EPI_GELU : EPI_PLAIN; g.c = (bf16_t*)dev_c;
  g.splitk_ws = (float*)dev_scratch; g.splitk_ws_bytes = dev_scratch ? scratch_bytes : 0;
  HIP_TRY(launch_gemm(g, (hipStream_t)stream));
  return HERO_OK;
}

int hero_linear(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c, int32_t m, int32_t n,
                int32_t k, int32_t act, void* stream) {
  return hero_linear_scratch(dev_a, dev_w, dev_bias, dev_c, m, n, k, act, nullptr, 0, stream);
}

int hero_linear_static(const void* dev_a, const void* dev_w, const void* dev_bias, void* dev_c, int32_t m, int32_t n,
                       int32_t k, int32_t act, void* stream) {
  int rc = check_linear_args(dev_a, dev_w, dev_bias, dev_c, m, n, k, act);
  if (rc) return rc;
  if (m == 0) return HERO_OK;
  // what hero_linear_scratch would want for this problem; anything beyond the library's array is refused
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  g.m = m; g.n = n; g.k = k; g.epilogue = act ? EPI_GELU : EPI_PLAIN;
  const size_t want = gemm_wanted_scratch_bytes(g);
  if (want > STATIC_SCRATCH_BYTES)
    return fail(HERO_ERR_BUFFER_TOO_SMALL,
                "hero_linear_static: the k-split of this %d x %d x %d problem needs %zu bytes of partial sums, the "
                "library's own scratch holds %zu; use hero_linear_scratch with a buffer of yours",
                m, n, k, want, STATIC_SCRATCH_BYTES);
  void* ws = nullptr;
  if ((rc = static_scratch(&ws)) != HERO_OK) return rc;
  return hero_linear_scratch(dev_a, dev_w, dev_bias, dev_c, m, n, k, act, ws, STATIC_SCRATCH_BYTES, stream);
}

int hero_attention_counted(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt, void* dev_o,
                           int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim, void* dev_scratch,
                           size_t scratch_bytes, uint32_t* dev_fallbacks, void* stream) {
  if (!dev_k || !dev_vt || (r > 0 && (!dev_q || !dev_o))) return fail(HERO_ERR_INVALID_ARG, "null pointer");
  if (r < 0 || n_keys < 1 || n_heads < 1) return fail(HERO_ERR_INVALID_ARG, "bad sizes");
  if (head_dim != 32 && head_dim != 64) return fail(HERO_ERR_SHAPE, "head_dim must be 32 or 64");
  if (ld_vt % 64 != 0 || ld_vt < n_keys) return fail(HERO_ERR_SHAPE, "ld_vt must be a multiple of 64 and >= n_keys");
  if (!attention_offsets_fit(n_keys, (int64_t)n_heads * head_dim, ld_vt))
    return fail(HERO_ERR_SHAPE, "(n_keys + 256) * hidden * 2 and hidden * ld_vt * 2 must stay below 2^32 (32-bit operand offsets)");
  AttnArgs a;
  a.q = (const bf16_t*)dev_q; a.k = (const bf16_t*)dev_k; a.vt = (const bf16_t*)dev_vt; a.ld_vt = ld_vt;
  a.o = (bf16_t*)dev_o; a.r = r; a.n_keys = n_keys; a.n_heads = n_heads; a.head_dim = head_dim;
  a.q_scale = 1.4426950408889634f / sqrtf((float)head_dim);
  if (!aligned16({dev_q, dev_k, dev_vt, dev_o, dev_scratch}))
    return fail(HERO_ERR_INVALID_ARG, "q, k, vt, o and scratch must be 16-byte aligned");
  if ((uintptr_t)dev_fallbacks & 3) return fail(HERO_ERR_INVALID_ARG, "the fallback counter must be 4-byte aligned");
  a.split_ws = (float*)dev_scratch; a.split_ws_bytes = dev_scratch ? scratch_bytes : 0;
  a.fallback_count = dev_fallbacks;
  HIP_TRY(launch_attention(a, (hipStream_t)stream));
  return HERO_OK;
}

int hero_attention_scratch(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt, void* dev_o,
                           int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim, void* dev_scratch,
                           size_t scratch_bytes, void* stream) {
  return hero_attention_counted(dev_q, dev_k, dev_vt, ld_vt, dev_o, r, n_keys, n_heads, head_dim, dev_scratch,
                                scratch_bytes, nullptr, stream);
}

int hero_attention(const void* dev_q, const void* dev_k, const void* dev_vt, int64_t ld_vt, void* dev_o,
                   int32_t r, int32_t n_keys, int32_t n_heads, int32_t head_dim, void* stream) {
  return hero_attention_scratch(dev_q, dev_k, dev_vt, ld_vt, dev_o, r, n_keys, n_heads, head_dim, nullptr, 0, stream);
}

int hero_axpy_features(void* dev_x, int32_t x_dtype, const void* s_cur, const void* s_prev, float alpha,
                       int64_t n_elems, void* stream) {
  if (n_elems > 0 && (!dev_x || !s_cur)) return fail(HERO_ERR_INVALID_ARG, "null pointer");
  if (x_dtype != HERO_DTYPE_FP32 && x_dtype != HERO_DTYPE_BF16) return fail(HERO_ERR_INVALID_ARG, "bad x_dtype");
  if (n_elems < 0 || n_elems % 8 != 0) return fail(HERO_ERR_SHAPE, "n_elems must be a non-negative multiple of 8");
  if (!aligned16({dev_x, s_cur, s_prev})) return fail(HERO_ERR_INVALID_ARG, "x, s_cur and s_prev must be 16-byte aligned");
  HIP_TRY(launch_axpy_features(dev_x, x_dtype == HERO_DTYPE_FP32, (const bf16_t*)s_cur, (const bf16_t*)s_prev, alpha,
                               n_elems, (hipStream_t)stream));
  return HERO_OK;
}

int hero_second_diff_stats(const void* f_prev, const void* f_cur, const void* f_next, int64_t n_elems,
                           void* dev_scratch, size_t scratch_bytes, double* dev_stats, int32_t accumulate,
                           void* stream) {
  if (!f_prev || !f_cur || !f_next || !dev_scratch || !dev_stats) return fail(HERO_ERR_INVALID_ARG, "null pointer");
  if (n_elems < 0 || n_elems % 8 != 0) return fail(HERO_ERR_SHAPE, "n_elems must be a non-negative multiple of 8");
  if (scratch_bytes < second_diff_scratch_bytes())
    return fail(HERO_ERR_BUFFER_TOO_SMALL, "scratch has %zu bytes, %zu needed", scratch_bytes, second_diff_scratch_bytes());
  if ((uintptr_t)dev_scratch % 8 != 0 || (uintptr_t)dev_stats % 8 != 0)
    return fail(HERO_ERR_INVALID_ARG, "scratch and stats must be 8-byte aligned");
  if (!aligned16({f_prev, f_cur, f_next})) return fail(HERO_ERR_INVALID_ARG, "the feature arrays must be 16-byte aligned");
  HIP_TRY(launch_second_diff_stats((const bf16_t*)f_prev, (const bf16_t*)f_cur, (const bf16_t*)f_next, n_elems,
                                   (double*)dev_scratch, dev_stats, accumulate != 0, (hipStream_t)stream));
  return HERO_OK;
}

int hero_stability_scores(const double* variances, int32_t n_layers, double* scores) {
  if (!variances || !scores || n_layers < 1) return fail(HERO_ERR_INVALID_ARG, "bad arguments");
  double lo = variances[0], hi = variances[0];
  for (int i = 0; i < n_layers; ++i) {
    if (!(variances[i] >= 0.0)) return fail(HERO_ERR_INVALID_ARG, "variance %d is negative or not a number", i);
    lo = variances[i] < lo ? variances[i] : lo;
    hi = variances[i] > hi ? variances[i] : hi;
  }
  for (int i = 0; i < n_layers; ++i) scores[i] = hi == lo ? 1.0 : 1.0 - (variances[i] - lo) / (hi - lo);
  return HERO_OK;
}

}  // extern "C"
