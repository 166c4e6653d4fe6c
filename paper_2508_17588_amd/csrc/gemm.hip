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
// 16 consecutive rows hit 16 distinct bank groups.  Global loads of tile k+1 are issued
// into registers before the MFMAs of tile k and written to the other LDS buffer after
// them (one barrier per K step).
// The epilogue adds the bias, applies GELU where asked, and either stores C or scatters
// rows into the feature / K / V^T caches (Eq. 3's merge).
#include "hero_device.h"
#include "hero_kernels.h"

namespace {

constexpr int BK = 64;           // bf16 elements per K step (128 B per row)
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per tile row

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float gelu_tanh(float x) {
  // x/2 (1 + tanh u) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
  float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
  float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * u);
  return x / (1.0f + e);
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__((BM / WM) * (BN / WN) * 64) void gemm_kernel(GemmArgs g, int tiles_m, int n_tiles,
                                                                           int per_xcd) {
  constexpr int WAVES_M = BM / WM;
  constexpr int T = (BM / WM) * (BN / WN) * 64;
  constexpr int MB = WM / 32, NB = WN / 32;
  constexpr int NA = BM * CHUNKS / T, NBL = BN * CHUNKS / T;
  static_assert(BM * CHUNKS % T == 0 && BN * CHUNKS % T == 0, "tile/threads mismatch");

  // consecutive workgroup ids land on different XCDs; give each XCD a contiguous tile range
  int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= n_tiles) return;
  const int tm = logical % tiles_m, tn = logical / tiles_m;
  const int m0 = tm * BM, n0 = tn * BN;

  extern __shared__ u32x4_t smem[];
  u32x4_t* sA = smem;                         // [2][BM*CHUNKS]
  u32x4_t* sB = smem + 2 * BM * CHUNKS;       // [2][BN*CHUNKS]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
  const int lr = lane & 31, lh = lane >> 5;

  // global source pointers of this thread's chunks (rows clamped: out-of-range rows are never stored)
  const u32x4_t* ga[NA];
  const u32x4_t* gb[NBL];
  int sa_off[NA], sb_off[NBL];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int q = tid + i * T, row = q / CHUNKS, c = q % CHUNKS;
    int gr = min(m0 + row, g.m - 1);
    ga[i] = reinterpret_cast<const u32x4_t*>(g.a + (int64_t)gr * g.k + c * 8);
    sa_off[i] = row * CHUNKS + swz(row, c);
  }
#pragma unroll
  for (int i = 0; i < NBL; ++i) {
    int q = tid + i * T, row = q / CHUNKS, c = q % CHUNKS;
    int gr = min(n0 + row, g.n - 1);
    gb[i] = reinterpret_cast<const u32x4_t*>(g.w + (int64_t)gr * g.k + c * 8);
    sb_off[i] = row * CHUNKS + swz(row, c);
  }

  floatx16_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4_t ra[NA], rb[NBL];
  const int kt_n = g.k / BK;
#pragma unroll
  for (int i = 0; i < NA; ++i) ra[i] = ga[i][0];
#pragma unroll
  for (int i = 0; i < NBL; ++i) rb[i] = gb[i][0];
#pragma unroll
  for (int i = 0; i < NA; ++i) sA[sa_off[i]] = ra[i];
#pragma unroll
  for (int i = 0; i < NBL; ++i) sB[sb_off[i]] = rb[i];
  __syncthreads();

  for (int kt = 0; kt < kt_n; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < kt_n;
    if (more) {
#pragma unroll
      for (int i = 0; i < NA; ++i) ra[i] = ga[i][(kt + 1) * (BK / 8)];
#pragma unroll
      for (int i = 0; i < NBL; ++i) rb[i] = gb[i][(kt + 1) * (BK / 8)];
    }
    const u32x4_t* cA = sA + cur * BM * CHUNKS;
    const u32x4_t* cB = sB + cur * BN * CHUNKS;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[MB], fb[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        int row = wm0 + i * 32 + lr;
        u32x4_t t = cA[row * CHUNKS + swz(row, 2 * ks + lh)];
        fa[i] = *reinterpret_cast<bf16x8_t*>(&t);
      }
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        int row = wn0 + j * 32 + lr;
        u32x4_t t = cB[row * CHUNKS + swz(row, 2 * ks + lh)];
        fb[j] = *reinterpret_cast<bf16x8_t*>(&t);
      }
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      u32x4_t* nA = sA + (cur ^ 1) * BM * CHUNKS;
      u32x4_t* nB = sB + (cur ^ 1) * BN * CHUNKS;
#pragma unroll
      for (int i = 0; i < NA; ++i) nA[sa_off[i]] = ra[i];
#pragma unroll
      for (int i = 0; i < NBL; ++i) nB[sb_off[i]] = rb[i];
    }
    __syncthreads();
  }

  // ---- epilogue ----
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int nblk = n0 + wn0 + j * 32;
    if (nblk >= g.n) continue;             // N is a multiple of 32: whole blocks are in or out
    const int n = nblk + lr;
    const float bias = bf16_to_f32(g.bias[n]);
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      const int mblk = m0 + wm0 + i * 32 + 4 * lh;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int mq = mblk + 8 * q;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = acc[i][j][4 * q + e] + bias;
          if (EPI == EPI_GELU) v[e] = gelu_tanh(v[e]);
        }
        if (EPI == EPI_PLAIN || EPI == EPI_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (mq + e < g.m) g.c[(int64_t)(mq + e) * g.n + n] = f32_to_bf16(v[e]);
        } else if (EPI == EPI_QKV) {
          const int which = nblk / g.d;    // uniform over the 32-column block (d % 32 == 0)
          if (which == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (mq + e < g.m) g.c[(int64_t)(mq + e) * g.d + n] = f32_to_bf16(v[e]);
          } else if (which == 1) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (mq + e < g.m) {
                int64_t row = g.rows ? g.rows[mq + e] : (mq + e);
                g.k_out[row * g.d + (n - g.d)] = f32_to_bf16(v[e]);
              }
          } else {
            bf16_t* vrow = g.vt_out + (int64_t)(n - 2 * g.d) * g.ld_vt;
            if (!g.rows && mq + 3 < g.m) {
              u32x2_t pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
              *reinterpret_cast<u32x2_t*>(vrow + mq) = pk;     // mq % 4 == 0, ld_vt % 4 == 0
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (mq + e < g.m) {
                  int64_t row = g.rows ? g.rows[mq + e] : (mq + e);
                  vrow[row] = f32_to_bf16(v[e]);
                }
            }
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (mq + e < g.m) {
              int64_t row = g.rows ? g.rows[mq + e] : (mq + e);
              bf16_t* p = g.c + row * g.n + n;
              float val = v[e];
              if (EPI == EPI_SCATTER_ADD) val += bf16_to_f32(*p);
              *p = f32_to_bf16(val);
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
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, tiles_m, n_tiles, per_xcd);                       \
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
  if (g.k <= 0 || g.k % BK != 0 || g.n % 32 != 0) return hipErrorInvalidValue;
  // large problems: 256x256 tiles, 8 waves of 128x64; small ones: 128x128 tiles, 4 waves of 64x64
  int64_t big_tiles = (int64_t)((g.m + 255) / 256) * ((g.n + 255) / 256);
  if (big_tiles >= 128) return launch_cfg<256, 256, 128, 64>(g, st);
  return launch_cfg<128, 128, 64, 64>(g, st);
}
