// bf16 MFMA GEMM for the refreshed rows: C = act(A W^T + bias), A [M,K], W [N,K] both
// K-contiguous (QKV projection, out-projection and FFN of Eq. 2 / Eq. 3), fp32 accumulate.
//
// Two kernels: problems with fewer than 128 tiles of 256 x 256 use the 128 x 128-tile kernel
// described here (register-staged loads); larger ones use gemm256_kernel further down (direct
// global -> LDS loads into rings of three A slots and two W slots, k-split of a thin last round;
// described there).
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
#include <algorithm>
#include <atomic>
#include <type_traits>

#include "hero_device.h"
#include "hero_kernels.h"

namespace {

constexpr int BK = 64;           // bf16 elements per K step (128 B per row)
constexpr int CHUNKS = BK / 8;   // 16-byte chunks per tile row
constexpr int GROUP_M = 8;       // row-tiles walked together (L2 locality)

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

__device__ __forceinline__ float gelu_tanh(float x) {
  // x/2 (1 + tanh u) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3);
  // -2u log2(e) = x (C1 + C2 x^2) with the constants folded: five plain operations and two
  // transcendentals per element (the epilogue runs while the matrix pipe idles)
  constexpr float C1 = -2.302208198144325f;     // -2 log2(e) sqrt(2/pi)
  constexpr float C2 = -0.1029432395800235f;    // C1 * 0.044715
  float e = __builtin_amdgcn_exp2f(x * __builtin_fmaf(x * x, C2, C1));
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
  // adaLN gate of the lane's columns, for the video and the text stream
  const bool gated = (EPI == EPI_SCATTER || EPI == EPI_SCATTER_ADD) && g.gate_v != nullptr;
  float gate_v[NB], gate_t[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int n = n0 + wn0 + j * 32 + lr;
    gate_v[j] = (gated && n_ok[j]) ? bf16_to_f32(g.gate_v[n]) : 1.f;
    gate_t[j] = (gated && n_ok[j]) ? bf16_to_f32(g.gate_t[n]) : 1.f;
  }
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
              if (gated) v *= row < g.n_text ? gate_t[j] : gate_v[j];
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

// ------------------------------------------------------------------------------------------
// Large problems: 256 x 256 tile, eight waves (two per SIMD) of 128 x 64, K walked in stages of
// 64 through LDS rings (three slots for A, two for W: all 160 KB of a CU) that are filled by
// direct global -> LDS loads (16 bytes per lane).
//
//  * What bounds this kernel is the rate at which a CU's vector cache can keep cache-line
//    requests in flight, so every request must be a whole 128-byte line: a wave-wide load
//    fetches eight rows of 128 bytes (eight consecutive lanes per row).
//  * Two waves per SIMD: a wave whose load waits for the address unit cannot issue MFMAs
//    meanwhile; with a second wave on the SIMD the matrix pipe keeps running.  Each wave issues
//    eight loads in the first quarter of a stage, one per MFMA: its W blocks of the next stage
//    and its A blocks of the stage after that.  The weight panels are shared by every row tile
//    and mostly hit in the caches, so one stage is enough for them; the activation panels
//    stream from HBM (few workgroups read each), and the extra stage of distance takes their
//    misses off the barrier's wait.
//  * LDS layout of a stage: rows of 128 B whose eight 16-byte chunks are XOR-swizzled with
//    (row/2)%8 (conflict-free ds_read_b128 fragment reads).  A direct load writes lane l to
//    byte 16*l of its 1 KB block, i.e. row l/8, chunk slot l%8, so the lane fetches the chunk
//    that belongs in that slot.
//  * One barrier per stage.  Loads complete in issue order, so "all but my four newest" before
//    the barrier of stage t means A and W of stage t are in LDS.  After that barrier every wave
//    holds the fragments of the last k-slice of stage t-1 in registers and has no LDS read
//    outstanding, so the new loads can overwrite the slots of stage t-1 at once (W of t+1 into
//    the other W slot, A of t+2 into the third A slot); they have one and two whole stages
//    (~2000 cycles each) to land.  The fragments of the first slice of stage t are read while the
//    MFMAs of that last slice run, which hides the LDS latency behind the barrier.
//  * The waves accumulate C^T blocks (operands swapped), so a lane owns one row m and four
//    consecutive columns n per accumulator quad.  The epilogue adds the bias, applies the
//    activation, rounds to bf16 and stages the wave's 128 x 64 sub-tile in LDS (8-byte writes,
//    row stride 136 B), then streams it out in 16-byte pieces, one 128-byte line per row.
//    Waves in the V third of the QKV projection keep the operands unswapped and stage the
//    transposed sub-tile, so V^T rows leave the same way.  The accumulating epilogue (FFN2)
//    stages fp32 in two halves and rounds once after adding the cached row.
// ------------------------------------------------------------------------------------------
constexpr int SBK = 64;                       // k elements per stage: one 128-byte line per row
constexpr int RING_B = 2;                     // W slots: its fills run one stage ahead
constexpr int STAGE_BYTES = 256 * SBK * 2;    // one operand, one stage: 32 KB
constexpr int RING_A = 3;                     // A slots: its fills run two stages ahead
constexpr int RING_B_OFF = RING_A * STAGE_BYTES;   // the W ring starts after the A ring
constexpr int CST = 136;                      // bf16 staging: bytes per 64-column row (+8 pad)
constexpr int CSTT = 264;                     // bf16 staging of a transposed sub-tile: 128 columns (+8 pad)
constexpr int CST32 = 264;                    // fp32 staging: bytes per 64-column row (+8 pad)
constexpr int STAGE_REGION = 128 * CST;       // per-wave staging region (17408 B)
constexpr int RING_BYTES = (RING_A + RING_B) * STAGE_BYTES;   // 160 KB
constexpr int GEMM256_LDS = 8 * STAGE_REGION > RING_BYTES ? 8 * STAGE_REGION : RING_BYTES;
static_assert(64 * CST32 <= STAGE_REGION && 64 * CSTT <= STAGE_REGION, "half-tile / transposed tile must fit the staging region");

// buffer resource words: base address, no stride, byte count, raw 32-bit data format
__device__ __forceinline__ u32x4_t rsrc_words(const void* p, uint32_t bytes) {
  const uint64_t addr = (uint64_t)p;
  u32x4_t r = {(uint32_t)addr, (uint32_t)(addr >> 32) & 0xffffu, bytes, 0x00020000u};
  r[0] = __builtin_amdgcn_readfirstlane(r[0]); r[1] = __builtin_amdgcn_readfirstlane(r[1]);
  r[2] = __builtin_amdgcn_readfirstlane(r[2]); r[3] = __builtin_amdgcn_readfirstlane(r[3]);
  return r;
}

// 16 bytes per lane from a buffer straight into LDS at lds_addr + 16*lane.  The bounds check
// covers voffset only (rows past the end arrive as zero); soffset carries the k advance.  Issued
// by hand so that the compiler does not make later LDS reads wait for it: completion is awaited
// explicitly with vmcnt before the stage's barrier.  Nothing else in the kernel uses m0.
__device__ __forceinline__ void lds_fill(u32x4_t rsrc, uint32_t lds_addr, uint32_t voffset, uint32_t soffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc), "s"(soffset) : "memory");
}

// keeps a wave-uniform value in a scalar register and stops the compiler from hoisting the
// comparisons made with it out of the loop (hoisted, they come back as lane masks that need
// VALU instructions at every use)
__device__ __forceinline__ int opaque(int v) {
  asm volatile("" : "+s"(v));
  return v;
}

// Split of the last, partly filled wave of tiles along k.  Tile slots 0 .. full_items-1 are
// whole work items; every later slot is cut into `split` k-chunks whose fp32 partial sums go to a
// workspace (one 256 KB block per chunk, in accumulator order: [i][j][quad][thread] float4) and
// are added up, and sent through the epilogue, by the fix-up kernel.
struct SplitK {
  int32_t full_items;   // tile slots computed whole
  int32_t split;        // k-chunks per remaining tile slot (1: none)
  float* ws;
};

// tile slot -> tile origin (each XCD owns a contiguous range of tiles, walked in groups of
// group_m row tiles); false for the empty slots that pad the range to a multiple of 8
__device__ __forceinline__ bool tile_origin(int slot, int tiles_m, int tiles_n, int per_xcd, int group_m,
                                            int& m0, int& n0) {
  const int p = (slot % 8) * per_xcd + slot / 8;
  if (p >= tiles_m * tiles_n) return false;
  const int group = p / (group_m * tiles_n);
  const int first_m = group * group_m;
  const int gsize = min(tiles_m - first_m, group_m);
  const int in_group = p - group * group_m * tiles_n;
  m0 = (first_m + in_group % gsize) * 256;
  n0 = (in_group / gsize) * 256;
  return true;
}

template <int EPI>
__device__ __forceinline__ void epilogue256(const GemmArgs& g, floatx16_t (&acc)[4][2], int m0, int n0, int wave,
                                            int lane, char* region);

template <int EPI>
__global__ __launch_bounds__(512) void gemm256_kernel(GemmArgs g, int tiles_m, int tiles_n, int per_xcd,
                                                      int group_m, SplitK sk) {
  // ---- workgroup id -> tile slot and k-chunk ----
  int slot = blockIdx.x, chunk = 0, n_chunks = 1;
  if (slot >= sk.full_items) {
    const int r = slot - sk.full_items;
    slot = sk.full_items + r / sk.split;
    chunk = r - (r / sk.split) * sk.split;
    n_chunks = sk.split;
  }
  int m0, n0;
  if (!tile_origin(slot, tiles_m, tiles_n, per_xcd, group_m, m0, n0)) return;

  extern __shared__ u32x4_t smem[];
  const uint32_t lds0 = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // waves w and w+4 share a SIMD
  const int wm0 = (wave & 1) * 128, wn0 = (wave >> 1) * 64;
  const int lr = lane & 31, lh = lane >> 5;

  // ---- direct loads: per stage this wave fills A blocks wave+8i and W blocks wave+8i, i = 0..3
  //      (8 rows each); lane l fetches, for row l/8 of the block, the chunk that belongs in
  //      LDS chunk slot l%8 ----
  const uint32_t row_bytes = (uint32_t)g.k * 2u;
  const u32x4_t rsA = rsrc_words(g.a, (uint32_t)g.m * row_bytes);
  const u32x4_t rsB = rsrc_words(g.w, (uint32_t)g.n * row_bytes);
  uint32_t voffA[4], voffB[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (wave + 8 * i) * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    voffA[i] = (uint32_t)(m0 + row) * row_bytes + chunk * 16;
    voffB[i] = (uint32_t)(n0 + row) * row_bytes + chunk * 16;
  }
  const uint32_t fillA = lds0 + wave * 1024, fillB = lds0 + RING_B_OFF + wave * 1024;
  const int n_stages = g.k / SBK;
  const int stage_begin = chunk * n_stages / n_chunks, stage_end = (chunk + 1) * n_stages / n_chunks;
  auto fill_a = [&](int slot, int stage, int q) {
    lds_fill(rsA, fillA + (uint32_t)slot * STAGE_BYTES + q * 8192, voffA[q], (uint32_t)stage * (SBK * 2));
  };
  auto fill_b = [&](int slot, int stage, int q) {
    lds_fill(rsB, fillB + (uint32_t)slot * STAGE_BYTES + q * 8192, voffB[q], (uint32_t)stage * (SBK * 2));
  };

  // ---- fragment reads: row R, k-chunk c of a stage sits at R*128 + (c ^ ((R/2)%8))*16 ----
  const char* lbase = reinterpret_cast<const char*>(smem);
  const char* fa_ks[4];
  const char* fb_ks[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int off = lr * 128 + (((2 * ks + lh) ^ ((lr >> 1) & 7)) * 16);     // wm0, wn0, 32i are multiples of 16 rows
    fa_ks[ks] = lbase + wm0 * 128 + off;
    fb_ks[ks] = lbase + RING_B_OFF + wn0 * 128 + off;
  }
  auto frag = [&](const char* ks_base, int slot, int i) {
    u32x4_t t = *reinterpret_cast<const u32x4_t*>(ks_base + slot * STAGE_BYTES + i * 4096);
    return *reinterpret_cast<bf16x8_t*>(&t);
  };

  floatx16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // V third of the QKV projection: keep the natural orientation (lanes along n) so that the
  // staged sub-tile is V^T
  const bool natural = (EPI == EPI_QKV) && (n0 + wn0 >= 2 * g.d);

  // Main loop.  Fragment set [1] holds the k-slice consumed first in a stage (the last slice of
  // the previous stage); the four slices of a stage alternate between the sets.
  auto main_loop = [&](auto NAT) {
    constexpr bool NATURAL = decltype(NAT)::value;
    bf16x8_t fa[2][4], fb[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      u32x4_t z = {0u, 0u, 0u, 0u};
      fa[1][i] = *reinterpret_cast<bf16x8_t*>(&z);
      if (i < 2) fb[1][i] = *reinterpret_cast<bf16x8_t*>(&z);
    }
    // order in which the 6 fragments of a slice are read (the MFMAs use them in the same order)
    auto read_frag = [&](int set, int slot_a, int slot_b, int ks, int q) {
      switch (q) {
        case 0: fa[set][0] = frag(fa_ks[ks], slot_a, 0); break;
        case 1: fb[set][0] = frag(fb_ks[ks], slot_b, 0); break;
        case 2: fb[set][1] = frag(fb_ks[ks], slot_b, 1); break;
        case 3: fa[set][1] = frag(fa_ks[ks], slot_a, 1); break;
        case 4: fa[set][2] = frag(fa_ks[ks], slot_a, 2); break;
        default: fa[set][3] = frag(fa_ks[ks], slot_a, 3); break;
      }
    };
    auto mma_one = [&](int set, int x) {
      const int i = x >> 1, j = x & 1;
      if (NATURAL) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
      else acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[set][j], fa[set][i], acc[i][j], 0, 0, 0);
    };
    // one stage: A slot SA and W slot SB hold stage t
    auto stage = [&](auto SLOT_A, auto SLOT_B, int t) {
      constexpr int SA = decltype(SLOT_A)::value, SB = decltype(SLOT_B)::value;
      // All but the four newest fills (A of stage t+1) have landed: A and W of stage t are in LDS.
      // Own fragment reads of stage t-1 are complete; after the barrier the same holds for every
      // wave: stage t is readable, and the slots of stage t-1 are free.
      asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int sl = 0; sl < 4; ++sl) {
        // MFMAs of slice sl-1 (set (sl+1)&1) while the fragments of slice sl arrive in set sl&1
#pragma unroll
        for (int x = 0; x < 8; ++x) {
          // (after the last stage the same stage is fetched once more into the idle slot: cheaper than
          //  eight branches per stage, and in bounds)
          if (sl == 0) {
            if (x < 4) fill_b(SB ^ 1, min(t + 1, stage_end - 1), x);
            else fill_a((SA + 2) % 3, min(t + 2, stage_end - 1), x - 4);
          }
          if (x < 6) read_frag(sl & 1, SA, SB, sl, x);
          mma_one((sl + 1) & 1, x);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    };
#pragma unroll
    for (int q = 0; q < 4; ++q) fill_a(0, stage_begin, q);
#pragma unroll
    for (int q = 0; q < 4; ++q) fill_b(0, stage_begin, q);
#pragma unroll
    for (int q = 0; q < 4; ++q) fill_a(1, min(stage_begin + 1, stage_end - 1), q);
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    for (int t = stage_begin; t < stage_end; t += 6) {
      stage(I0{}, I0{}, t);
      if (t + 1 < stage_end) stage(I1{}, I1{}, t + 1);
      if (t + 2 < stage_end) stage(I2{}, I0{}, t + 2);
      if (t + 3 < stage_end) stage(I0{}, I1{}, t + 3);
      if (t + 4 < stage_end) stage(I1{}, I0{}, t + 4);
      if (t + 5 < stage_end) stage(I2{}, I1{}, t + 5);
    }
    // last slice of the last stage
#pragma unroll
    for (int x = 0; x < 8; ++x) mma_one(1, x);
  };
  if (EPI == EPI_QKV && natural) main_loop(std::true_type{});
  else main_loop(std::false_type{});

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (n_chunks > 1) {
    // partial sums of a k-chunk: 8 KB per store instruction, contiguous over the workgroup
    float* part = sk.ws + ((size_t)(slot - sk.full_items) * sk.split + chunk) * 65536 + tid * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          floatx4_t v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<floatx4_t*>(part + ((i * 2 + j) * 4 + q) * 2048) = v;
        }
    return;
  }
  __syncthreads();                       // every wave is done with the ring
  epilogue256<EPI>(g, acc, m0, n0, wave, lane, reinterpret_cast<char*>(smem) + wave * STAGE_REGION);
}

// Adds up the k-chunks of the split tiles and sends the sums through the epilogue.  One
// single-wave workgroup per 128 x 64 wave sub-tile (8 per tile), so that even a few dozen split
// tiles spread over the whole chip; the 32 loads of a chunk are independent and in flight together.
template <int EPI>
__global__ __launch_bounds__(64) void gemm256_fixup_kernel(GemmArgs g, int tiles_m, int tiles_n, int per_xcd,
                                                           int group_m, SplitK sk) {
  const int tile = blockIdx.x >> 3, wave = blockIdx.x & 7;
  int m0, n0;
  if (!tile_origin(sk.full_items + tile, tiles_m, tiles_n, per_xcd, group_m, m0, n0)) return;
  extern __shared__ u32x4_t smem[];
  const int lane = threadIdx.x;
  floatx16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  const float* part = sk.ws + (size_t)tile * sk.split * 65536 + (wave * 64 + lane) * 4;
  for (int c = 0; c < sk.split; ++c, part += 65536) {
    floatx4_t v[32];
#pragma unroll
    for (int x = 0; x < 32; ++x) v[x] = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t*>(part + x * 2048));
#pragma unroll
    for (int x = 0; x < 32; ++x)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[x >> 3][(x >> 2) & 1][4 * (x & 3) + e] += v[x][e];
  }
  epilogue256<EPI>(g, acc, m0, n0, wave, lane, reinterpret_cast<char*>(smem));
}

template <int EPI>
__device__ __forceinline__ void epilogue256(const GemmArgs& g, floatx16_t (&acc)[4][2], int m0, int n0, int wave,
                                            int lane, char* region) {
  const int wm0 = (wave & 1) * 128, wn0 = (wave >> 1) * 64;
  const int lr = lane & 31, lh = lane >> 5;
  const bool natural = (EPI == EPI_QKV) && (n0 + wn0 >= 2 * g.d);
  const int mw = m0 + wm0, nw = n0 + wn0;            // origin of this wave's sub-tile; region: its LDS staging space

  if (EPI == EPI_QKV && natural) {
    // acc[i][j][4q+e] = C[m = mw + 32i + 8q + 4lh + e][n = nw + 32j + lr]; stage [n][m]
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int n = nw + 32 * j + lr;
      const float bias = n < g.n ? bf16_to_f32(g.bias[n]) : 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          u32x2_t pk = {pack_bf16x2_hw(acc[i][j][4 * q] + bias, acc[i][j][4 * q + 1] + bias),
                        pack_bf16x2_hw(acc[i][j][4 * q + 2] + bias, acc[i][j][4 * q + 3] + bias)};
          *reinterpret_cast<u32x2_t*>(region + (32 * j + lr) * CSTT + (32 * i + 8 * q + 4 * lh) * 2) = pk;
        }
    }
    if (g.rows != nullptr) {
      // scattered columns (refresh): lanes run along m, so the 64 two-byte stores of one instruction
      // fall into the few cache lines of one V^T row that hold the neighbouring selected tokens
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        const int m = mw + 64 * half + lane;
        const bool m_ok = m < g.m;
        const int64_t col = m_ok ? (int64_t)g.rows[m] : 0;
#pragma unroll 8
        for (int nl = 0; nl < 64; ++nl) {
          const bf16_t v = *reinterpret_cast<const bf16_t*>(region + nl * CSTT + (64 * half + lane) * 2);
          const int n = nw + nl;
          if (m_ok && n < g.n) g.vt_out[(int64_t)(n - 2 * g.d) * g.ld_vt + col] = v;
        }
      }
      return;
    }
    // contiguous columns (full layer): rows of the region are n (64 of them), 16-byte pieces hold 8 consecutive m
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
      const int nl = it * 4 + (lane >> 4), piece = lane & 15;
      const u32x2_t lo = *reinterpret_cast<const u32x2_t*>(region + nl * CSTT + piece * 16);
      const u32x2_t hi = *reinterpret_cast<const u32x2_t*>(region + nl * CSTT + piece * 16 + 8);
      const int n = nw + nl, m = mw + piece * 8;
      if (n < g.n && m < g.m) {
        bf16_t* dst = g.vt_out + (int64_t)(n - 2 * g.d) * g.ld_vt;
        if (m + 8 <= g.m) {
          u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
          *reinterpret_cast<u32x4_t*>(dst + m) = v;
        } else {
          const uint32_t w4[4] = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (m + e < g.m) dst[m + e] = (bf16_t)(w4[e >> 1] >> ((e & 1) * 16));
        }
      }
    }
    return;
  }

  // acc[i][j][4q+e] = C[m = mw + 32i + lr][n = nw + 32j + 8q + 4lh + e]
  const float out_scale = (EPI == EPI_QKV && nw < g.d) ? g.q_scale : 1.0f;
  // destination of element (m, n): base[row(m) * ld + n - n_shift]
  bf16_t* base = g.c;
  int ld = g.n, n_shift = 0;
  bool use_rows = (EPI == EPI_SCATTER || EPI == EPI_SCATTER_ADD) && g.rows != nullptr;
  if (EPI == EPI_QKV) {
    ld = g.d;
    if (nw >= g.d) { base = g.k_out; n_shift = g.d; use_rows = g.rows != nullptr; }
  }
  // bias of the lane's columns: [j][q] holds n = nw + 32j + 8q + 4lh .. +3
  u32x2_t bias4[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int n = min(nw + 32 * j + 8 * q + 4 * lh, g.n - 4);     // columns past N are never stored
      bias4[j][q] = *reinterpret_cast<const u32x2_t*>(g.bias + n);
    }
  // adaLN gate of the lane's columns, for both streams; the lane's row i picks one.  (Loaded
  // unconditionally, from the bias vector when there is no gate, so that the arrays stay in registers.)
  constexpr bool CAN_GATE = EPI == EPI_SCATTER || EPI == EPI_SCATTER_ADD;
  const bool gated = CAN_GATE && g.gate_v != nullptr;
  u32x2_t gate4_v[2][4], gate4_t[2][4];
  bool text_row[4];
  if (CAN_GATE) {
    const bf16_t* gv = gated ? g.gate_v : g.bias;
    const bf16_t* gt = gated ? g.gate_t : g.bias;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = min(nw + 32 * j + 8 * q + 4 * lh, g.n - 4);
        gate4_v[j][q] = *reinterpret_cast<const u32x2_t*>(gv + n);
        gate4_t[j][q] = *reinterpret_cast<const u32x2_t*>(gt + n);
      }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m = min(mw + 32 * i + lr, g.m - 1);
      text_row[i] = (use_rows ? g.rows[m] : m) < g.n_text;
    }
  }
  auto biased = [&](int i, int j, int q, float* v) {
    v[0] = acc[i][j][4 * q] + unpack_lo(bias4[j][q][0]);
    v[1] = acc[i][j][4 * q + 1] + unpack_hi(bias4[j][q][0]);
    v[2] = acc[i][j][4 * q + 2] + unpack_lo(bias4[j][q][1]);
    v[3] = acc[i][j][4 * q + 3] + unpack_hi(bias4[j][q][1]);
    if (CAN_GATE && gated) {
      const u32x2_t gg = text_row[i] ? gate4_t[j][q] : gate4_v[j][q];
      v[0] *= unpack_lo(gg[0]); v[1] *= unpack_hi(gg[0]);
      v[2] *= unpack_lo(gg[1]); v[3] *= unpack_hi(gg[1]);
    }
  };

  if (EPI == EPI_SCATTER_ADD) {
    // two halves of 64 rows staged in fp32; S[row] += . with one rounding
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float v[4];
            biased(2 * h + ii, j, q, v);
            char* dst = region + (32 * ii + lr) * CST32 + (32 * j + 8 * q + 4 * lh) * 4;
            u32x2_t a0 = {__float_as_uint(v[0]), __float_as_uint(v[1])}, a1 = {__float_as_uint(v[2]), __float_as_uint(v[3])};
            *reinterpret_cast<u32x2_t*>(dst) = a0;
            *reinterpret_cast<u32x2_t*>(dst + 8) = a1;
          }
      // 64 rows x 8 pieces of 8 columns
#pragma unroll 4
      for (int it = 0; it < 8; ++it) {
        const int rl = it * 8 + (lane >> 3), piece = lane & 7;
        const char* src = region + rl * CST32 + piece * 32;
        float v[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          u32x2_t t = *reinterpret_cast<const u32x2_t*>(src + 8 * e);
          v[2 * e] = __uint_as_float(t[0]); v[2 * e + 1] = __uint_as_float(t[1]);
        }
        const int m = mw + 64 * h + rl, n = nw + piece * 8;
        if (m < g.m && n < g.n) {
          const int64_t row = use_rows ? (int64_t)g.rows[m] : (int64_t)m;
          u32x4_t* d = reinterpret_cast<u32x4_t*>(base + row * ld + n);
          u32x4_t old = *d, out;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            out[e] = pack_bf16x2_hw(v[2 * e] + unpack_lo(old[e]), v[2 * e + 1] + unpack_hi(old[e]));
          *d = out;
          if (g.x != nullptr) {
            // residual add with the feature as stored (rounded), so x matches x += S done afterwards
            if (g.x_fp32) {
              floatx4_t* xp = reinterpret_cast<floatx4_t*>(static_cast<float*>(g.x) + row * ld + n);
              floatx4_t x0 = xp[0], x1 = xp[1];
              x0[0] += unpack_lo(out[0]); x0[1] += unpack_hi(out[0]); x0[2] += unpack_lo(out[1]); x0[3] += unpack_hi(out[1]);
              x1[0] += unpack_lo(out[2]); x1[1] += unpack_hi(out[2]); x1[2] += unpack_lo(out[3]); x1[3] += unpack_hi(out[3]);
              xp[0] = x0; xp[1] = x1;
            } else {
              u32x4_t* xp = reinterpret_cast<u32x4_t*>(static_cast<bf16_t*>(g.x) + row * ld + n);
              u32x4_t xv = *xp, xo;
#pragma unroll
              for (int e = 0; e < 4; ++e)
                xo[e] = pack_bf16x2(unpack_lo(xv[e]) + unpack_lo(out[e]), unpack_hi(xv[e]) + unpack_hi(out[e]));
              *xp = xo;
            }
          }
        }
      }
    }
    return;
  }

#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v[4];
        biased(i, j, q, v);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (EPI == EPI_QKV) v[e] *= out_scale;
          if (EPI == EPI_GELU) v[e] = gelu_tanh(v[e]);
        }
        u32x2_t pk = {pack_bf16x2_hw(v[0], v[1]), pack_bf16x2_hw(v[2], v[3])};
        *reinterpret_cast<u32x2_t*>(region + (32 * i + lr) * CST + (32 * j + 8 * q + 4 * lh) * 2) = pk;
      }
  // 128 rows x 8 pieces of 8 columns: one 128-byte line per row
#pragma unroll 4
  for (int it = 0; it < 16; ++it) {
    const int rl = it * 8 + (lane >> 3), piece = lane & 7;
    const u32x2_t lo = *reinterpret_cast<const u32x2_t*>(region + rl * CST + piece * 16);
    const u32x2_t hi = *reinterpret_cast<const u32x2_t*>(region + rl * CST + piece * 16 + 8);
    const int m = mw + rl, n = nw + piece * 8;
    if (m < g.m && n < g.n) {
      const int64_t row = use_rows ? (int64_t)g.rows[m] : (int64_t)m;
      u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
      *reinterpret_cast<u32x4_t*>(base + row * ld + (n - n_shift)) = v;
    }
  }
}

// A kernel that uses more than 64 KB of dynamic LDS must be told so once on every device it runs
// on.  `done` holds one bit per device ordinal (devices past 63 are told on every launch); the
// runtime call is idempotent, so two host threads that meet here at most repeat it.
hipError_t allow_dynamic_lds(const void* kern, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev < 64 ? 1ull << dev : 0;
  if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// The chip runs 256 workgroups at a time, so the last round of tiles may leave most of it
// idle.  Cutting those n_rem tiles into s k-chunks makes the round take ceil(n_rem*s/256)/s of
// a tile's time, and costs a fix-up pass that moves n_rem*s blocks of 256 KB twice (about
// 0.1*n_rem/stages of a tile's time per chunk, measured).  Take the s that minimises the sum,
// with chunks of at least 16 stages, among those whose partial sums fit ws_bytes.  At the
// 17776-token shapes this cuts FFN2 (k = 12288; 3 rounds + 72 tiles) in 3 and makes it 9 %
// faster; the out-projection (k = 3072, the same tiles) is cut in 2 for 3 %, FFN1 (13 rounds +
// 32 tiles) in 3 for 0.4 %.  Returns the number of k-chunks (1: no cut); *n_rem_out: the tile
// slots of the last round.
int choose_k_split(const GemmArgs& g, size_t ws_bytes, int* n_rem_out) {
  const int tiles_m = (g.m + 255) / 256, tiles_n = (g.n + 255) / 256;
  const int slots = (tiles_m * tiles_n + 7) / 8 * 8;
  const int n_rem = slots - slots / 256 * 256;
  *n_rem_out = n_rem;
  // (the QKV projection is never cut: its k is the hidden size, too short to pay at the supported sizes)
  if (g.epilogue == EPI_QKV || n_rem == 0) return 1;
  const int stages = g.k / SBK;
  const int s_max = (int)std::min<size_t>((size_t)std::min(stages / 16, 8), ws_bytes / ((size_t)n_rem * 262144));
  const double per_chunk = 0.1 * n_rem / stages;
  double best = 1.0;
  int split = 1;
  for (int sp = 2; sp <= s_max; ++sp) {
    const double t = (double)((n_rem * sp + 255) / 256) / sp + per_chunk * sp;
    if (t < best - 0.02) { best = t; split = sp; }
  }
  return split;
}

hipError_t launch_gemm256(const GemmArgs& g, hipStream_t st) {
  int tiles_m = (g.m + 255) / 256, tiles_n = (g.n + 255) / 256;
  int n_tiles = tiles_m * tiles_n;
  int per_xcd = (n_tiles + 7) / 8;
  const int slots = per_xcd * 8;
  // Row tiles walked together by an XCD.  Operand panels of a long-k problem are several MB each,
  // and a problem with few row tiles gives each XCD only a few groups: both do better with short
  // groups (in-session A/B at the 5B shapes: QKV of 4485 rows 4 % faster with 4, the 17776-row
  // problems with k = 3072 0.5 % faster with 8, 16 is 1-7 % slower everywhere).
  const int group_m = (g.k >= 8192 || tiles_m <= 24) ? 4 : 8;
  SplitK sk;
  sk.full_items = slots / 256 * 256;
  sk.ws = g.splitk_ws;
  int n_rem = 0;
  sk.split = choose_k_split(g, g.splitk_ws != nullptr ? g.splitk_ws_bytes : 0, &n_rem);
  if (sk.split == 1) sk.full_items = slots;
  const int n_split_tiles = slots - sk.full_items;
  dim3 grid(sk.full_items + n_split_tiles * sk.split), block(512);
#define HERO_GEMM256_LAUNCH(E)                                                                           \
  do {                                                                                                   \
    auto kern = gemm256_kernel<E>;                                                                       \
    auto fix = gemm256_fixup_kernel<E>;                                                                  \
    static std::atomic<uint64_t> lds_allowed{0};                                                         \
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), GEMM256_LDS, lds_allowed);     \
    if (e != hipSuccess) return e;                                                                       \
    hipLaunchKernelGGL(kern, grid, block, GEMM256_LDS, st, g, tiles_m, tiles_n, per_xcd, group_m, sk);   \
    if (n_split_tiles > 0)                                                                               \
      hipLaunchKernelGGL(fix, dim3(n_split_tiles * 8), dim3(64), STAGE_REGION, st, g, tiles_m, tiles_n,  \
                         per_xcd, group_m, sk);                                                          \
  } while (0)
  switch (g.epilogue) {
    case EPI_PLAIN: HERO_GEMM256_LAUNCH(EPI_PLAIN); break;
    case EPI_GELU: HERO_GEMM256_LAUNCH(EPI_GELU); break;
    case EPI_QKV: HERO_GEMM256_LAUNCH(EPI_QKV); break;
    case EPI_SCATTER: HERO_GEMM256_LAUNCH(EPI_SCATTER); break;
    case EPI_SCATTER_ADD: HERO_GEMM256_LAUNCH(EPI_SCATTER_ADD); break;
    default: return hipErrorInvalidValue;
  }
#undef HERO_GEMM256_LAUNCH
  return hipGetLastError();
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
    static std::atomic<uint64_t> lds_allowed{0};                                                         \
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void*>(kern), (int)smem, lds_allowed);       \
    if (e != hipSuccess) return e;                                                                       \
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

namespace {
bool uses_large_tiles(const GemmArgs& g) {
  // large problems: 256x256 tiles, 8 waves of 128x64; small ones: 128x128 tiles, 4 waves of 64x64
  const int64_t big_tiles = (int64_t)((g.m + 255) / 256) * ((g.n + 255) / 256);
  // (a wave's columns must lie inside one of the Q / K / V thirds)
  const bool qkv_split_ok = g.epilogue != EPI_QKV || g.d % 128 == 0;
  return big_tiles >= 128 && qkv_split_ok;
}
}  // namespace

size_t gemm_wanted_scratch_bytes(const GemmArgs& g) {
  if (g.m <= 0 || g.n <= 0 || g.k <= 0 || !uses_large_tiles(g)) return 0;
  int n_rem = 0;
  const int split = choose_k_split(g, (size_t)-1, &n_rem);
  return split > 1 ? (size_t)n_rem * split * 262144 : 0;
}

bool gemm_can_update_x(const GemmArgs& g) { return g.epilogue == EPI_SCATTER_ADD && uses_large_tiles(g); }

hipError_t launch_gemm(const GemmArgs& g, hipStream_t st) {
  if (g.m <= 0 || g.n <= 0) return hipSuccess;
  if (g.k <= 0 || g.k % BK != 0 || g.n % 64 != 0) return hipErrorInvalidValue;
  if (g.epilogue == EPI_QKV && (g.d % 64 != 0 || g.n != 3 * g.d)) return hipErrorInvalidValue;
  // operands are addressed with 32-bit byte offsets
  if (((int64_t)g.m + 512) * g.k * 2 >= (int64_t)1 << 32 || ((int64_t)g.n + 512) * g.k * 2 >= (int64_t)1 << 32)
    return hipErrorInvalidValue;
  if (uses_large_tiles(g)) return launch_gemm256(g, st);
  if (g.x != nullptr) return hipErrorInvalidValue;       // only the large-tile epilogue updates x
  return launch_cfg<128, 128, 64, 64>(g, st);
}
