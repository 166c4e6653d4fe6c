// bf16 MFMA GEMM for the refreshed rows: C = act(A W^T + bias), A [M,K], W [N,K] both
// K-contiguous (QKV projection, out-projection and FFN of Eq. 2 / Eq. 3), fp32 accumulate.
//
// Tiling (gfx950, wave64): a workgroup owns a BM x BN tile of C and walks K in steps of 64.
// Each wave owns a WM x WN sub-tile made of 32x32 blocks computed by
// v_mfma_f32_32x32x16_bf16 (A fragment: lane holds row lane%32, eight consecutive k
// starting at 8*(lane/32); B fragment likewise for column lane%32; accumulator register i
// of a lane is row 8*(i/4) + 4*(lane/32) + i%4, column lane%32).
// A and W tiles are staged through LDS in rows of 128 B (64 bf16) whose eight 16-byte
// chunks are XOR-swizzled with (row/2)%8, which makes the ds_read_b128 fragment reads of
// 16 consecutive rows hit 16 distinct bank groups.
// Latency hiding: global (buffer) loads run two K steps ahead of the MFMAs through two
// register sets; fragments are read from LDS one 16-wide k slice ahead.  Buffer loads are
// bounds-checked by the hardware (rows past M or N read as zero), so ragged M needs no
// padding.  Workgroup ids are remapped so that each XCD works on a contiguous range of
// tiles, walked in groups of 8 row-tiles, which keeps the A / W panels an XCD streams
// concurrently small enough for its L2.
// The epilogue adds the bias, applies GELU where asked, and either stores C or scatters
// rows into the feature / K / V^T caches (Eq. 3's merge).  Waves whose columns belong to
// the V third of the QKV projection run their MFMAs with the operands swapped, so their
// accumulators hold the transposed block and V^T rows are written with row-contiguous
// lanes.
#include <type_traits>

#include "hero_device.h"
#include "hero_kernels.h"

namespace {

constexpr int BK = 64;           // bf16 elements per K step (128 B per row)
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per tile row
constexpr int GROUP_M = 8;       // row-tiles walked together (L2 locality)

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float gelu_tanh(float x) {
  // x/2 (1 + tanh u) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
  float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
  return x * __builtin_amdgcn_rcpf(1.0f + e);
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_kernel(GemmArgs g, int tiles_m, int tiles_n,
                                                                           int per_xcd) {
  constexpr int WAVES_M = BM / WM;
  constexpr int T = (BM / WM) * (BN / WN) * 64;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int NA = BM * CHUNKS / T, NBL = BN * CHUNKS / T;
  constexpr int ROWS_PER_PASS = T / CHUNKS;      // tile rows covered by one chunk per thread
  static_assert(BM * CHUNKS % T == 0 && BN * CHUNKS % T == 0, "tile/threads mismatch");

  // ---- workgroup id -> tile ----
  const int n_tiles = tiles_m * tiles_n;
  int p = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (p >= n_tiles) return;
  const int group = p / (GROUP_M * tiles_n);
  const int first_m = group * GROUP_M;
  const int gsize = min(tiles_m - first_m, GROUP_M);
  const int in_group = p - group * GROUP_M * tiles_n;
  const int tm = first_m + in_group % gsize, tn = in_group / gsize;
  const int m0 = tm * BM, n0 = tn * BN;

  extern __shared__ u32x4_t smem[];
  u32x4_t* sA = smem;                         // [2][BM*CHUNKS]
  u32x4_t* sB = smem + 2 * BM * CHUNKS;       // [2][BN*CHUNKS]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
  const int lr = lane & 31, lh = lane >> 5;

  // ---- global loads: thread t loads chunk (t % 8) of rows t/8 + i*ROWS_PER_PASS ----
  const int ld_row = tid / CHUNKS, ld_c = tid % CHUNKS;
  const uint32_t row_bytes = (uint32_t)g.k * 2u;
  const __amdgpu_buffer_rsrc_t rsA = make_rsrc(g.a, (uint32_t)g.m * row_bytes);
  const __amdgpu_buffer_rsrc_t rsB = make_rsrc(g.w, (uint32_t)g.n * row_bytes);
  // the whole address lives in the bounds-checked vector offset
  uint32_t voffA[NA], voffB[NBL];
#pragma unroll
  for (int i = 0; i < NA; ++i) voffA[i] = (uint32_t)(m0 + ld_row + i * ROWS_PER_PASS) * row_bytes + ld_c * 16;
#pragma unroll
  for (int i = 0; i < NBL; ++i) voffB[i] = (uint32_t)(n0 + ld_row + i * ROWS_PER_PASS) * row_bytes + ld_c * 16;
  // ROWS_PER_PASS is a multiple of 16, so the swizzle term is the same for every pass
  const int st_off = ld_row * CHUNKS + swz(ld_row, ld_c);

  u32x4_t ra[2][NA], rb[2][NBL];
  constexpr int LPS_A = NA / 4, LPS_B = NBL / 4;   // global loads / LDS writes per 16-wide k slice
  static_assert(NA % 4 == 0 && NBL % 4 == 0, "loads must split evenly over the four k slices");
  auto gload = [&](auto PAR, int kt) {
    constexpr int P = decltype(PAR)::value;
    const uint32_t koff = (uint32_t)kt * (BK * 2);
#pragma unroll
    for (int i = 0; i < NA; ++i) ra[P][i] = __builtin_amdgcn_raw_buffer_load_b128(rsA, voffA[i] + koff, 0, 0);
#pragma unroll
    for (int i = 0; i < NBL; ++i) rb[P][i] = __builtin_amdgcn_raw_buffer_load_b128(rsB, voffB[i] + koff, 0, 0);
  };
  auto lstore = [&](auto PAR, int buf) {
    constexpr int P = decltype(PAR)::value;
    u32x4_t* dA = sA + buf * BM * CHUNKS + st_off;
    u32x4_t* dB = sB + buf * BN * CHUNKS + st_off;
#pragma unroll
    for (int i = 0; i < NA; ++i) dA[i * ROWS_PER_PASS * CHUNKS] = ra[P][i];
#pragma unroll
    for (int i = 0; i < NBL; ++i) dB[i * ROWS_PER_PASS * CHUNKS] = rb[P][i];
  };

  floatx16_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // V third of the QKV projection: accumulate the transposed block (operands swapped)
  const bool transposed = (EPI == EPI_QKV) && (n0 + wn0 >= 2 * g.d);

  int fa_row[MB], fb_row[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) fa_row[i] = wm0 + i * 32 + lr;
#pragma unroll
  for (int j = 0; j < NB; ++j) fb_row[j] = wn0 + j * 32 + lr;

  // One K step: multiply the tile in LDS buffer `buf`; meanwhile issue the global loads of
  // tile kt_load into register set P and write register set P^1 (loaded one step ago) to
  // the other LDS buffer.  Loads, LDS writes, fragment reads and MFMAs of each 16-wide k
  // slice are interleaved so that no unit sees a burst.
  auto kstep = [&](auto PAR, int buf, int kt_load, bool pipeline) {
    constexpr int P = decltype(PAR)::value;
    const u32x4_t* cA = sA + buf * BM * CHUNKS;
    const u32x4_t* cB = sB + buf * BN * CHUNKS;
    u32x4_t* dA = sA + (buf ^ 1) * BM * CHUNKS + st_off;
    u32x4_t* dB = sB + (buf ^ 1) * BN * CHUNKS + st_off;
    const uint32_t koff = (uint32_t)kt_load * (BK * 2);
    bf16x8_t fa[2][MB], fb[2][NB];
    auto fload = [&](int slot, int ks) {
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        u32x4_t t = cA[fa_row[i] * CHUNKS + swz(fa_row[i], 2 * ks + lh)];
        fa[slot][i] = *reinterpret_cast<bf16x8_t*>(&t);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        u32x4_t t = cB[fb_row[j] * CHUNKS + swz(fb_row[j], 2 * ks + lh)];
        fb[slot][j] = *reinterpret_cast<bf16x8_t*>(&t);
      }
    };
    fload(0, 0);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int cur = ks & 1;
      __builtin_amdgcn_sched_barrier(0);       // one k slice per scheduling region
      if (pipeline) {
#pragma unroll
        for (int i = ks * LPS_A; i < (ks + 1) * LPS_A; ++i) {
          dA[i * ROWS_PER_PASS * CHUNKS] = ra[P ^ 1][i];
        }
#pragma unroll
        for (int i = ks * LPS_B; i < (ks + 1) * LPS_B; ++i) {
          dB[i * ROWS_PER_PASS * CHUNKS] = rb[P ^ 1][i];
        }
#pragma unroll
        for (int i = ks * LPS_A; i < (ks + 1) * LPS_A; ++i)
          ra[P][i] = __builtin_amdgcn_raw_buffer_load_b128(rsA, voffA[i] + koff, 0, 0);
#pragma unroll
        for (int i = ks * LPS_B; i < (ks + 1) * LPS_B; ++i)
          rb[P][i] = __builtin_amdgcn_raw_buffer_load_b128(rsB, voffB[i] + koff, 0, 0);
      }
      if (ks + 1 < BK / 16) fload(cur ^ 1, ks + 1);
      if (EPI == EPI_QKV && transposed) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][i], fb[cur][j], acc[i][j], 0, 0, 0);
      }
      // spread the memory instructions of this slice between its MFMAs
      constexpr int MFMAS = MB * NB, GROUPS = 4;
#pragma unroll
      for (int gq = 0; gq < GROUPS; ++gq) {
        if (pipeline) {
          __builtin_amdgcn_sched_group_barrier(0x200, (LPS_A + LPS_B + GROUPS - 1) / GROUPS, 0);  // LDS writes
          __builtin_amdgcn_sched_group_barrier(0x020, (LPS_A + LPS_B + GROUPS - 1) / GROUPS, 0);  // global loads
        }
        __builtin_amdgcn_sched_group_barrier(0x100, (MB + NB + GROUPS - 1) / GROUPS, 0);          // LDS reads
        __builtin_amdgcn_sched_group_barrier(0x008, MFMAS / GROUPS, 0);                           // MFMA
      }
    }
  };

  using P0 = std::integral_constant<int, 0>;
  using P1 = std::integral_constant<int, 1>;
  const int kt_n = g.k / BK;
  // Loads and LDS writes past the last K step are issued unconditionally: out-of-range
  // buffer loads return zero and the tile they would fill is never multiplied.
  gload(P0{}, 0);
  gload(P1{}, 1);
  lstore(P0{}, 0);
  __syncthreads();

  int kt = 0;
  for (; kt + 1 < kt_n; kt += 2) {
    kstep(P0{}, 0, kt + 2, true);     // multiplies tile kt, writes tile kt+1, loads tile kt+2
    __syncthreads();
    kstep(P1{}, 1, kt + 3, true);
    __syncthreads();
  }
  if (kt < kt_n) kstep(P0{}, 0, 0, false);

  // ---- epilogue ----
  if (EPI == EPI_QKV && transposed) {
    // acc[i][j][4q+e] = C[m = mblk + lr][n = nblk + 8q + 4lh + e]: lanes run along m
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int m = m0 + wm0 + i * 32 + lr;
      const bool m_ok = m < g.m;
      const int64_t col = m_ok ? (g.rows ? (int64_t)g.rows[m] : (int64_t)m) : 0;
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int nblk = n0 + wn0 + j * 32;
        if (nblk < g.n) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int n = nblk + 8 * q + 4 * lh + e;
              const float v = acc[i][j][4 * q + e] + bf16_to_f32(g.bias[n]);
              if (m_ok) g.vt_out[(int64_t)(n - 2 * g.d) * g.ld_vt + col] = f32_to_bf16_hw(v);
            }
        }
      }
    }
    return;
  }

  // destination of element (m, n): base[row(m) * ld + n - n_shift]
  bf16_t* base = g.c;
  int ld = g.n, n_shift = 0;
  bool use_rows = (EPI == EPI_SCATTER || EPI == EPI_SCATTER_ADD) && g.rows != nullptr;
  if (EPI == EPI_QKV) {
    ld = g.d;
    if (n0 + wn0 >= g.d) { base = g.k_out; n_shift = g.d; use_rows = g.rows != nullptr; }
  }
  float bias[NB];
  bool n_ok[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int n = n0 + wn0 + j * 32 + lr;
    n_ok[j] = n < g.n;
    bias[j] = n_ok[j] ? bf16_to_f32(g.bias[n]) : 0.f;
  }
  const float out_scale = (EPI == EPI_QKV && n0 + wn0 < g.d) ? g.q_scale : 1.0f;
  const int ncol = n0 + wn0 + lr - n_shift;
#pragma unroll
  for (int i = 0; i < MB; ++i) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + wm0 + i * 32 + 8 * q + 4 * lh + e;
        if (m < g.m) {
          const int64_t row = use_rows ? (int64_t)g.rows[m] : (int64_t)m;
          bf16_t* prow = base + row * ld + ncol;
#pragma unroll
          for (int j = 0; j < NB; ++j) {
            if (n_ok[j]) {
              float v = acc[i][j][4 * q + e] + bias[j];
              if (EPI == EPI_QKV) v *= out_scale;
              if (EPI == EPI_GELU) v = gelu_tanh(v);
              if (EPI == EPI_SCATTER_ADD) v += bf16_to_f32(prow[j * 32]);
              prow[j * 32] = f32_to_bf16_hw(v);
            }
          }
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t st) {
  constexpr int T = (BM / WM) * (BN / WN) * 64;
  constexpr size_t smem = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
  int tiles_m = (g.m + BM - 1) / BM, tiles_n = (g.n + BN - 1) / BN;
  int n_tiles = tiles_m * tiles_n;
  int per_xcd = (n_tiles + 7) / 8;
  dim3 grid(per_xcd * 8), block(T);
#define HERO_GEMM_LAUNCH(E)                                                                              \
  do {                                                                                                   \
    auto kern = gemm_kernel<BM, BN, WM, WN, E>;                                                          \
    static bool attr_set = false;                                                                        \
    if (!attr_set) {                                                                                     \
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),                            \
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);         \
      if (e != hipSuccess) return e;                                                                     \
      attr_set = true;                                                                                   \
    }                                                                                                    \
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, tiles_m, tiles_n, per_xcd);                       \
  } while (0)
  switch (g.epilogue) {
    case EPI_PLAIN: HERO_GEMM_LAUNCH(EPI_PLAIN); break;
    case EPI_GELU: HERO_GEMM_LAUNCH(EPI_GELU); break;
    case EPI_QKV: HERO_GEMM_LAUNCH(EPI_QKV); break;
    case EPI_SCATTER: HERO_GEMM_LAUNCH(EPI_SCATTER); break;
    case EPI_SCATTER_ADD: HERO_GEMM_LAUNCH(EPI_SCATTER_ADD); break;
    default: return hipErrorInvalidValue;
  }
#undef HERO_GEMM_LAUNCH
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.m <= 0 || g.n <= 0) return hipSuccess;
  if (g.k <= 0 || g.k % BK != 0 || g.n % 64 != 0) return hipErrorInvalidValue;
  if (g.epilogue == EPI_QKV && (g.d % 64 != 0 || g.n != 3 * g.d)) return hipErrorInvalidValue;
  // operands are addressed with 32-bit byte offsets
  if (((int64_t)g.m + 512) * g.k * 2 >= (int64_t)1 << 32 || ((int64_t)g.n + 512) * g.k * 2 >= (int64_t)1 << 32)
    return hipErrorInvalidValue;
  // large problems: 256x256 tiles, 8 waves of 128x64; small ones: 128x128 tiles, 4 waves of 64x64
  int64_t big_tiles = (int64_t)((g.m + 255) / 256) * ((g.n + 255) / 256);
  // (a wave's columns must lie inside one of the Q / K / V thirds, so the 128-wide wave tiles need d % 128 == 0)
  const bool qkv_split_ok = g.epilogue != EPI_QKV || g.d % 128 == 0;
  if (big_tiles >= 128 && qkv_split_ok) return launch_cfg<256, 256, 128, 128>(g, st);
  return launch_cfg<128, 128, 64, 64>(g, st);
}
