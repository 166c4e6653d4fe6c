// Flash-style attention of refreshed queries against the full cached K/V
// (FullAttn of Eq. 2 evaluated on the selected rows of Eq. 3): O = softmax(Q K^T / sqrt(hd)) V
// per head, never materialising the score matrix.
//
// Layout: Q [r, H*hd] and K [N, H*hd] row-major, V transposed [H*hd, ld_vt] (key index
// contiguous), O [r, H*hd].  The scores are taken in the base-2 domain: exp2(q_scale * q.k),
// where the caller either pre-multiplied Q by log2(e)/sqrt(hd) (q_scale = 1) or passes that
// factor in q_scale.
//
// One workgroup = NW waves x 64 queries of one head; keys are walked in tiles of 64 staged
// through LDS (K tile [64 keys][hd], V^T tile [hd][64 keys], 16-byte chunks XOR-swizzled so
// that ds_read_b128 fragment reads are bank-conflict free).  A wave computes S^T = K Q^T with
// v_mfma_f32_32x32x16_bf16 (A = K rows, B = Q rows held in registers for the whole kernel),
// so every lane owns one query column: its accumulator values are different keys of the same
// query and the softmax reductions are in-lane plus one exchange with lane^32.  P^T goes
// straight from the accumulators (rounded to bf16) into the B operand of O^T += V^T P^T: the
// K rows are read in a permuted order (bits 2 and 3 of the row index swapped) so that the
// eight k-slots a lane feeds to one PV MFMA are eight consecutive keys, which makes the V^T
// fragment a single 16-byte LDS read.
//
// Two code paths share that layout:
//
//  * head_dim 64, the production path: a software pipeline over 32-key blocks in which the
//    QK^T MFMAs of block b+1, the exponentials of block b and the PV MFMAs of block b-1 are
//    issued together, so the matrix pipe and the VALU/transcendental pipe overlap inside one
//    wave.  The exponentials are reference-free, p = exp2(s): fp32 and bf16 share an 8-bit
//    exponent, so no running maximum is needed as long as the scores of a query stay well
//    inside +-100 (in log2 units), and the softmax is invariant to the reference point.  The
//    row sum is accumulated in fp32 alongside.  After the last key the row sums are checked:
//    if any query of the workgroup has a row sum outside [2^-80, 2^80] (or NaN), i.e. its
//    scores were too large or too small for the reference-free form, the whole workgroup
//    recomputes its output with the general path below.  K/V tiles go global -> LDS directly
//    (buffer_load ... lds, 16 bytes per lane) into three rotating buffers, one barrier per
//    64-key tile; K/V fragments are refilled from LDS half a step before they are used.
//    The chip holds 512 workgroups at a time; the query blocks of the last, partly filled round
//    are cut into key ranges, each a work item of its own whose unnormalised output and row sums
//    go to a caller-provided workspace (they simply add, there being no reference point), and a
//    fix-up kernel adds them, makes the row-sum check on the totals and finishes the block.
//
//  * the general path (head_dim 32, and the fallback of the production path): classic online
//    softmax with a running maximum that is only raised when some query exceeds it by more
//    than 2^8, one 64-key tile at a time, register-staged double-buffered LDS.
#include <algorithm>
#include <type_traits>

#include "hero_device.h"
#include "hero_kernels.h"

namespace {

constexpr int BKV = 64;   // keys per tile

// ------------------------------------------------------------------------------------------
// general path: online softmax with running maximum; one workgroup = NW waves x 64 queries
// ------------------------------------------------------------------------------------------
template <int HD, int NW>
__device__ __forceinline__ void attention_general(const AttnArgs& a, int head, int q0, float scale_log2e,
                                                  u32x4_t* sK, u32x4_t* sV) {
  constexpr int T = NW * 64;
  constexpr int KCH = HD / 8;             // 16-byte chunks per K-tile row
  constexpr int VCH = BKV / 8;            // 16-byte chunks per V^T-tile row
  constexpr int KS = HD / 16;             // k-steps of the QK^T MFMA
  constexpr int CB = HD / 32;             // 32-row blocks of O^T
  constexpr int NKL = BKV * KCH / T;      // K chunks per thread per tile
  constexpr int NVL = HD * VCH / T;       // V^T chunks per thread per tile
  static_assert(BKV * KCH % T == 0 && HD * VCH % T == 0, "tile/threads mismatch");
  constexpr int K_TILE = BKV * KCH, V_TILE = HD * VCH;   // in 16-byte chunks; sK, sV hold two tiles each

  const int d = a.n_heads * HD;
  const int tid = threadIdx.x, lane = tid & 63;
  const int lr = lane & 31, lh = lane >> 5;

  // Q fragments (B operand): lane holds query q0 + ig*32 + lr, channels 16s + 8*lh .. +7
  bf16x8_t qf[2][KS];
#pragma unroll
  for (int ig = 0; ig < 2; ++ig) {
    int qrow = min(q0 + ig * 32 + lr, a.r - 1);
    const u32x4_t* qp = reinterpret_cast<const u32x4_t*>(a.q + (int64_t)qrow * d + head * HD);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      u32x4_t t = qp[2 * s + lh];
      qf[ig][s] = *reinterpret_cast<bf16x8_t*>(&t);
    }
  }

  // global -> LDS staging of this thread's chunks
  const bf16_t* kbase = a.k + head * HD;
  const bf16_t* vbase = a.vt + (int64_t)head * HD * a.ld_vt;
  int k_row[NKL], k_c[NKL], k_off[NKL];
#pragma unroll
  for (int i = 0; i < NKL; ++i) {
    int q = tid + i * T;
    k_row[i] = q / KCH; k_c[i] = q % KCH;
    k_off[i] = k_row[i] * KCH + (k_c[i] ^ ((k_row[i] >> 1) & (KCH - 1)));
  }
  const u32x4_t* v_src[NVL];
  int v_off[NVL];
#pragma unroll
  for (int i = 0; i < NVL; ++i) {
    int q = tid + i * T, row = q / VCH, c = q % VCH;
    v_src[i] = reinterpret_cast<const u32x4_t*>(vbase + (int64_t)row * a.ld_vt + c * 8);
    v_off[i] = row * VCH + (c ^ ((row >> 1) & (VCH - 1)));
  }

  floatx16_t o[CB][2];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int ig = 0; ig < 2; ++ig)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[cb][ig][e] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};
  float l_run[2] = {0.f, 0.f};

  const int n_tiles = (a.n_keys + BKV - 1) / BKV;
  u32x4_t rk[NKL], rv[NVL];

  auto load_tile = [&](int tile) {
    int kv0 = tile * BKV;
#pragma unroll
    for (int i = 0; i < NKL; ++i) {
      int row = min(kv0 + k_row[i], a.n_keys - 1);
      rk[i] = *reinterpret_cast<const u32x4_t*>(kbase + (int64_t)row * d + k_c[i] * 8);
    }
#pragma unroll
    for (int i = 0; i < NVL; ++i) rv[i] = v_src[i][kv0 / 8];
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NKL; ++i) sK[buf * K_TILE + k_off[i]] = rk[i];
#pragma unroll
    for (int i = 0; i < NVL; ++i) sV[buf * V_TILE + v_off[i]] = rv[i];
  };

  load_tile(0);
  store_tile(0);
  __syncthreads();

  // K row read by lane lr as MFMA row: swap bits 2 and 3
  const int krow_perm = (lr & ~12) | ((lr & 4) << 1) | ((lr & 8) >> 1);

  for (int tile = 0; tile < n_tiles; ++tile) {
    const int cur = tile & 1;
    const bool more = tile + 1 < n_tiles;
    if (more) load_tile(tile + 1);

    // ---- S^T = K Q^T ----
    floatx16_t s[2][2];   // [jb][ig]
#pragma unroll
    for (int jb = 0; jb < 2; ++jb)
#pragma unroll
      for (int ig = 0; ig < 2; ++ig)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[jb][ig][e] = 0.f;
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      const int row = jb * 32 + krow_perm;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        u32x4_t t = sK[cur * K_TILE + row * KCH + ((2 * ks + lh) ^ ((row >> 1) & (KCH - 1)))];
        bf16x8_t kf = *reinterpret_cast<bf16x8_t*>(&t);
#pragma unroll
        for (int ig = 0; ig < 2; ++ig)
          s[jb][ig] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ig][ks], s[jb][ig], 0, 0, 0);
      }
    }

    // ---- mask the ragged last tile ----
    if (!more && (a.n_keys % BKV) != 0) {
      const int kv0 = tile * BKV;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            int j = kv0 + jb * 32 + 16 * (g >> 1) + 8 * lh + 4 * (g & 1) + e;
            if (j >= a.n_keys) { s[jb][0][4 * g + e] = -INFINITY; s[jb][1][4 * g + e] = -INFINITY; }
          }
    }

    // ---- online softmax (per query column), P^T packed to bf16 ----
    // The running maximum is only raised when some query of the wave exceeds it by more
    // than 2^8 (the reference point of exp2 is arbitrary as long as O and the row sum use
    // the same one), so the rescale of O is skipped on most tiles.
    bf16x8_t pf[2][2][2];   // [ig][jb][t]
#pragma unroll
    for (int ig = 0; ig < 2; ++ig) {
      float mx = fmaxf(s[0][ig][0], s[1][ig][0]);
#pragma unroll
      for (int e = 1; e < 16; e += 1) mx = fmaxf(fmaxf(mx, s[0][ig][e]), s[1][ig][e]);
      {
        auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(mx), __float_as_uint(mx), false, false);
        mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));   // both halves of the query's keys
      }
      const float cand = mx * scale_log2e;
      if (__builtin_amdgcn_ballot_w64(cand > m_run[ig] + 8.0f) != 0) {
        const float m_new = fmaxf(m_run[ig], cand);
        const float alpha = __builtin_amdgcn_exp2f(m_run[ig] - m_new);
        m_run[ig] = m_new;
        l_run[ig] *= alpha;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[cb][ig][e] *= alpha;
      }
      const float m_ref = m_run[ig];
      float psum = l_run[ig];
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        uint32_t pk[8];
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) {
          float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[jb][ig][2 * e2], scale_log2e, -m_ref));
          float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[jb][ig][2 * e2 + 1], scale_log2e, -m_ref));
          pk[e2] = pack_bf16x2_hw(p0, p1);
          psum += p0 + p1;
        }
        u32x4_t t0 = {pk[0], pk[1], pk[2], pk[3]};
        u32x4_t t1 = {pk[4], pk[5], pk[6], pk[7]};
        pf[ig][jb][0] = *reinterpret_cast<bf16x8_t*>(&t0);
        pf[ig][jb][1] = *reinterpret_cast<bf16x8_t*>(&t1);
      }
      l_run[ig] = psum;
    }

    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
      const int row = cb * 32 + lr;
#pragma unroll
      for (int jb = 0; jb < 2; ++jb)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          u32x4_t tv = sV[cur * V_TILE + row * VCH + ((4 * jb + 2 * t + lh) ^ ((row >> 1) & (VCH - 1)))];
          bf16x8_t vf = *reinterpret_cast<bf16x8_t*>(&tv);
#pragma unroll
          for (int ig = 0; ig < 2; ++ig)
            o[cb][ig] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[ig][jb][t], o[cb][ig], 0, 0, 0);
        }
    }

    if (more) store_tile(cur ^ 1);
    __syncthreads();
  }

  // ---- normalise and store: lane owns query column lr, channels 8q + 4lh + e ----
#pragma unroll
  for (int ig = 0; ig < 2; ++ig) {
    const float l = l_run[ig] + __shfl_xor(l_run[ig], 32, 64);   // the two key halves of the query
    const float inv = 1.0f / l;
    const int qrow = q0 + ig * 32 + lr;
    if (qrow < a.r) {
      bf16_t* op = a.o + (int64_t)qrow * d + head * HD;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          u32x2_t pk = {pack_bf16x2_hw(o[cb][ig][4 * q] * inv, o[cb][ig][4 * q + 1] * inv),
                        pack_bf16x2_hw(o[cb][ig][4 * q + 2] * inv, o[cb][ig][4 * q + 3] * inv)};
          *reinterpret_cast<u32x2_t*>(op + cb * 32 + 8 * q + 4 * lh) = pk;
        }
    }
  }
}

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attention_general_kernel(AttnArgs a, int n_qblocks, int n_blocks,
                                                                       int per_xcd) {
  // each XCD (consecutive workgroup ids round-robin over 8 XCDs) gets a contiguous range of heads
  int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= n_blocks) return;
  const int head = logical / n_qblocks, qb = logical % n_qblocks;
  __shared__ u32x4_t sK[2 * BKV * HD / 8];
  __shared__ u32x4_t sV[2 * HD * BKV / 8];
  attention_general<HD, NW>(a, head, qb * (NW * 64) + (threadIdx.x >> 6) * 64, a.q_scale, sK, sV);
}

// ------------------------------------------------------------------------------------------
// head_dim 64: pipelined, reference-free exponentials, general path as fallback
// ------------------------------------------------------------------------------------------
constexpr int TILE = 512;   // 16-byte chunks per 64-key K or V^T tile at head_dim 64

template <int I> using IC = std::integral_constant<int, I>;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// buffer resource words: base address, no stride, byte count, raw 32-bit data format
__device__ __forceinline__ u32x4_t make_rsrc_words(const void* p, uint32_t bytes) {
  const uint64_t addr = (uint64_t)p;
  u32x4_t r = {(uint32_t)addr, (uint32_t)(addr >> 32) & 0xffffu, bytes, 0x00020000u};
  r[0] = __builtin_amdgcn_readfirstlane(r[0]); r[1] = __builtin_amdgcn_readfirstlane(r[1]);
  r[2] = __builtin_amdgcn_readfirstlane(r[2]); r[3] = __builtin_amdgcn_readfirstlane(r[3]);
  return r;
}

// 16 bytes per lane from a buffer straight into LDS at lds_base + 16*lane; bytes past the end
// of the buffer arrive as zero.  The compiler's own builtin for this instruction makes every
// later LDS read wait for the load, so it is issued by hand and waited for explicitly with
// vmcnt(0) before the barrier that publishes the tile.  Nothing else in this kernel uses m0.
__device__ __forceinline__ void direct_lds_load(u32x4_t rsrc, uint32_t lds_base, uint32_t voffset) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_base), "v"(voffset), "s"(rsrc) : "memory");
}

// Split of the last, partly filled round of workgroups along the keys.  Block slots
// 0 .. full_items-1 are whole work items; every later slot is cut into `split` key ranges whose
// unnormalised outputs and row sums (the reference-free form needs no common maximum, so they
// simply add) go to a workspace, one block of PART_FLOATS floats per range, in accumulator
// order; the fix-up kernel adds them, checks the row sums, normalises and stores.
struct KeySplit {
  int32_t full_items;
  int32_t split;       // key ranges per remaining slot (1: none)
  float* ws;
};
constexpr int PART_FLOATS = 256 * 66;      // per thread: 64 output values and 2 row sums

template <int NW>
__device__ __forceinline__ void attention_finish(const AttnArgs& a, int head, int q0, int wave, int lane,
                                                 floatx16_t (&o)[2][2], const float (&l)[2], char* lds);

// One more workgroup took the running-maximum path.  Kept out of line: inlined, these few
// instructions change the register allocation of the whole kernel, key loop included.
__device__ __attribute__((noinline)) void count_fallback(uint32_t* counter) {
  if (threadIdx.x == 0 && counter != nullptr) atomicAdd(counter, 1u);
}

template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void attention_hd64_kernel(AttnArgs a, int n_qblocks, int n_blocks,
                                                                    int per_xcd, KeySplit ks) {
  constexpr int HD = 64;
  constexpr int NL = 8 / NW;              // 1 KB wave-loads per wave per tile (K and V^T each)
  static_assert(8 % NW == 0, "waves must divide the 8 wave-loads of a tile");

  int slot = blockIdx.x, chunk = 0, n_chunks = 1;
  if (slot >= ks.full_items) {
    const int rr = slot - ks.full_items;
    slot = ks.full_items + rr / ks.split;
    chunk = rr - (rr / ks.split) * ks.split;
    n_chunks = ks.split;
  }
  int logical = (slot % 8) * per_xcd + slot / 8;
  if (logical >= n_blocks) return;
  const int head = logical / n_qblocks, qb = logical % n_qblocks;
  const int d = a.n_heads * HD;
  // this item's keys: whole 64-key tiles [t_begin, t_end) of the problem; the last range also takes the ragged tail
  const int tiles_all = a.n_keys / BKV;
  const int t_begin = (int)((int64_t)chunk * tiles_all / n_chunks);
  const int t_end = (int)((int64_t)(chunk + 1) * tiles_all / n_chunks);
  const int n_keys = (chunk == n_chunks - 1) ? a.n_keys - t_begin * BKV : (t_end - t_begin) * BKV;
  const bf16_t* kbase = a.k + (int64_t)t_begin * BKV * d;
  const bf16_t* vtbase = a.vt + (int64_t)t_begin * BKV;

  __shared__ u32x4_t skv[2][3][TILE];            // K tiles, then V^T tiles, three rotating buffers each
  u32x4_t (&sK)[3][TILE] = skv[0];
  u32x4_t (&sV)[3][TILE] = skv[1];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: lives in a scalar register
  const int lr = lane & 31, lh = lane >> 5;
  const int q0 = qb * (NW * 64) + wave * 64;

  // Q fragments (B operand): lane holds query q0 + ig*32 + lr, channels 16s + 8*lh .. +7
  bf16x8_t qf[2][4];
#pragma unroll
  for (int ig = 0; ig < 2; ++ig) {
    int qrow = min(q0 + ig * 32 + lr, a.r - 1);
    const u32x4_t* qp = reinterpret_cast<const u32x4_t*>(a.q + (int64_t)qrow * d + head * HD);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      u32x4_t t = qp[2 * s + lh];
      if (a.q_scale != 1.0f) {
#pragma unroll
        for (int i = 0; i < 4; ++i) t[i] = pack_bf16x2_hw(unpack_lo(t[i]) * a.q_scale, unpack_hi(t[i]) * a.q_scale);
      }
      qf[ig][s] = *reinterpret_cast<bf16x8_t*>(&t);
    }
  }

  // ---- staging: wave-load j (of 8) fills tile rows 8j..8j+7; lane l -> row 8j + l/8 and LDS
  //      chunk slot l%8, which holds the row's logical chunk (l%8) ^ ((row>>1)&7) ----
  const uint32_t k_bytes = (uint32_t)((int64_t)n_keys * d * 2 - head * HD * 2);
  const uint32_t v_bytes = (uint32_t)(((int64_t)d - head * HD) * a.ld_vt * 2 - (int64_t)t_begin * BKV * 2);
  const u32x4_t rsK = make_rsrc_words(kbase + head * HD, k_bytes);
  const u32x4_t rsV = make_rsrc_words(vtbase + (int64_t)head * HD * a.ld_vt, v_bytes);
  // LDS byte address of this wave's first 1 KB slot in buffer 0 (wave-uniform)
  const uint32_t lds_k0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lds_ptr_t)&sK[0][64 * wave]);
  const uint32_t lds_v0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lds_ptr_t)&sV[0][64 * wave]);
  uint32_t k_voff[NL], v_voff[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int row = 8 * (wave + NW * i) + (lane >> 3);
    const int c = (lane & 7) ^ ((row >> 1) & 7);
    k_voff[i] = (uint32_t)row * (uint32_t)(d * 2) + c * 16;
    v_voff[i] = (uint32_t)row * (uint32_t)(a.ld_vt * 2) + c * 16;
  }
  const uint32_t k_tile_bytes = (uint32_t)(BKV * d * 2), v_tile_bytes = BKV * 2;
  auto gload_k = [&](int tile, int buf) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      direct_lds_load(rsK, lds_k0 + (uint32_t)(buf * TILE + 64 * NW * i) * 16, k_voff[i] + (uint32_t)tile * k_tile_bytes);
  };
  auto gload_v = [&](int tile, int buf) {
#pragma unroll
    for (int i = 0; i < NL; ++i)
      direct_lds_load(rsV, lds_v0 + (uint32_t)(buf * TILE + 64 * NW * i) * 16, v_voff[i] + (uint32_t)tile * v_tile_bytes);
  };

  // ---- fragment read offsets (chunks) ----
  const int kperm = (lr & ~12) | ((lr & 4) << 1) | ((lr & 8) >> 1);   // K row read as MFMA row lr
  int k_fo[4], v_fo[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    k_fo[s] = kperm * 8 + ((2 * s + lh) ^ ((kperm >> 1) & 7));   // + jb*256
    v_fo[s] = lr * 8 + ((2 * s + lh) ^ ((lr >> 1) & 7));         // index 2*jb + t; + cb*256
  }

  floatx16_t o[2][2];              // [cb][ig]; cleared after the prologue, which does not touch it
  float la[2] = {0.f, 0.f}, lb[2] = {0.f, 0.f};   // two partial row sums per query group

  floatx16_t s0[2], s1[2];         // scores of the even / odd 32-key block, [ig]
  bf16x8_t p0[2][2], p1[2][2];     // their probabilities as PV operands, [ig][t]
  bf16x8_t kfr[4], vfr[4];         // K fragments [ks] and V^T fragments [2*cb + t] of the block in flight

  auto read_k = [&](int kb, int jb) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      u32x4_t t = sK[kb][jb * 256 + k_fo[ks]];
      kfr[ks] = *reinterpret_cast<bf16x8_t*>(&t);
    }
  };
  auto read_v = [&](int vb, int jb) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        u32x4_t tv = sV[vb][cb * 256 + v_fo[2 * jb + t]];
        vfr[2 * cb + t] = *reinterpret_cast<bf16x8_t*>(&tv);
      }
  };
  auto qk = [&](floatx16_t (&sd)[2]) {
#pragma unroll
    for (int ig = 0; ig < 2; ++ig)
#pragma unroll
      for (int e = 0; e < 16; ++e) sd[ig][e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int ig = 0; ig < 2; ++ig)
        sd[ig] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[ks], qf[ig][ks], sd[ig], 0, 0, 0);
  };
  // probabilities of accumulator values 8h .. 8h+7 (the keys of PV k-half t = h)
  auto sm_half = [&](floatx16_t (&ss)[2], bf16x8_t (&pd)[2][2], int h) {
#pragma unroll
    for (int ig = 0; ig < 2; ++ig) {
      uint32_t pk[4];
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        float x0 = __builtin_amdgcn_exp2f(ss[ig][8 * h + 2 * e2]);
        float x1 = __builtin_amdgcn_exp2f(ss[ig][8 * h + 2 * e2 + 1]);
        la[ig] += x0;
        lb[ig] += x1;
        pk[e2] = pack_bf16x2_hw(x0, x1);
      }
      u32x4_t t = {pk[0], pk[1], pk[2], pk[3]};
      pd[ig][h] = *reinterpret_cast<bf16x8_t*>(&t);
    }
  };
  auto pv = [&](bf16x8_t (&ps)[2][2]) {
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ig = 0; ig < 2; ++ig)
          o[cb][ig] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[2 * cb + t], ps[ig][t], o[cb][ig], 0, 0, 0);
  };
  // half a step = 8 MFMAs, 16 exponentials, 24 other VALU instructions, 4 fragment reads
  auto sched_half = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // LDS read
      __builtin_amdgcn_sched_group_barrier(0x400, 4, 0);   // exp
      __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);   // VALU
    }
  };

  const int ntf = n_keys / BKV;           // full key tiles; 32-key blocks 0 .. 2*ntf-1
  if (ntf > 0) {
    // ---- prologue: scores of blocks 0 and 1, probabilities of block 0 ----
    gload_k(0, 0); gload_v(0, 0); gload_k(1, 1); gload_v(1, 1); gload_k(2, 2);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    read_k(0, 0);
    qk(s0);
    __builtin_amdgcn_sched_barrier(0);
    read_k(0, 1);
    __builtin_amdgcn_sched_barrier(0);
    qk(s1);
    sm_half(s0, p0, 0);
    sm_half(s0, p0, 1);
    __builtin_amdgcn_sched_barrier(0);
    read_k(1, 0); read_v(0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int ig = 0; ig < 2; ++ig)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[cb][ig][e] = 0.f;
  if (ntf > 0) {
    // Iteration `tile` (buffer index P = tile % 3): on entry the fragments hold K tile+1 block 0
    // and V^T tile block 0, s1 the scores of block 2*tile+1, p0 the probabilities of block 2*tile.
    // K tile t lives in sK[t % 3], V^T tile t in sV[t % 3]; the loads issued here fill the buffers
    // whose last readers finished before this iteration's barrier, and are first read after the
    // next one.
    auto iter = [&](auto PAR, int tile) {
      constexpr int P = decltype(PAR)::value;
      constexpr int P1 = (P + 1) % 3, P2 = (P + 2) % 3;
      __builtin_amdgcn_s_waitcnt(0x0f70);           // vmcnt(0): this wave's LDS fills have landed
      __syncthreads();
      gload_k(tile + 3, P); gload_v(tile + 2, P2);
      __builtin_amdgcn_sched_barrier(0);
      // scores of block 2*tile+2, probabilities of block 2*tile+1, PV of block 2*tile
      qk(s0);
      sm_half(s1, p1, 0);
      read_k(P1, 1);
      sched_half();
      __builtin_amdgcn_sched_barrier(0);
      pv(p0);
      sm_half(s1, p1, 1);
      read_v(P, 1);
      sched_half();
      __builtin_amdgcn_sched_barrier(0);
      // scores of block 2*tile+3, probabilities of block 2*tile+2, PV of block 2*tile+1
      qk(s1);
      sm_half(s0, p0, 0);
      read_k(P2, 0);
      sched_half();
      __builtin_amdgcn_sched_barrier(0);
      pv(p1);
      sm_half(s0, p0, 1);
      read_v(P1, 0);
      sched_half();
      __builtin_amdgcn_sched_barrier(0);
    };
    const int n_iter = ntf - 1;
    int tile = 0;
    for (; tile + 3 <= n_iter; tile += 3) {
      iter(IC<0>{}, tile);
      iter(IC<1>{}, tile + 1);
      iter(IC<2>{}, tile + 2);
    }
    int rem = 0;
    if (tile < n_iter) { iter(IC<0>{}, tile); ++tile; rem = 1; }
    if (tile < n_iter) { iter(IC<1>{}, tile); ++tile; rem = 2; }
    // ---- drain: tile = ntf-1 in buffer `rem`; the fragments hold its V^T block 0 ----
    auto drain = [&](auto PAR) {
      constexpr int P = decltype(PAR)::value;
      sm_half(s1, p1, 0);
      sm_half(s1, p1, 1);
      pv(p0);
      __builtin_amdgcn_sched_barrier(0);
      read_v(P, 1);
      __builtin_amdgcn_sched_barrier(0);
      pv(p1);
    };
    if (rem == 0) drain(IC<0>{}); else if (rem == 1) drain(IC<1>{}); else drain(IC<2>{});
  }

  // ---- ragged tail: keys ntf*64 .. n_keys-1 (K rows past the end arrive as zero and are masked) ----
  const int n_tail = n_keys - ntf * BKV;
  if (n_tail > 0) {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    gload_k(ntf, 0); gload_v(ntf, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
#pragma unroll
    for (int jb = 0; jb < 2; ++jb) {
      read_k(0, jb); read_v(0, jb);
      qk(s0);
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = jb * 32 + 16 * (g >> 1) + 8 * lh + 4 * (g & 1) + e;
          if (j >= n_tail) { s0[0][4 * g + e] = -INFINITY; s0[1][4 * g + e] = -INFINITY; }
        }
      sm_half(s0, p0, 0);
      sm_half(s0, p0, 1);
      pv(p0);
    }
  }

  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): no LDS fill of this wave is still in flight

  // ---- row sums ----
  // (the lane index is taken from the hardware again here: every VGPR is in use inside the loop, and a
  //  value that is only needed after it would be parked in scratch memory and fetched back)
  int lane_after;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(lane_after));
  const int tid_after = wave * 64 + lane_after;
  float l[2];
#pragma unroll
  for (int ig = 0; ig < 2; ++ig) {
    l[ig] = la[ig] + lb[ig];
    l[ig] += __shfl_xor(l[ig], 32, 64);   // the two key halves of the query
  }
  if (n_chunks > 1) {
    // partial result of a key range: 1 KB per store instruction, contiguous over the workgroup
    float* part = ks.ws + ((size_t)(slot - ks.full_items) * ks.split + chunk) * PART_FLOATS;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int ig = 0; ig < 2; ++ig)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          floatx4_t v = {o[cb][ig][4 * q], o[cb][ig][4 * q + 1], o[cb][ig][4 * q + 2], o[cb][ig][4 * q + 3]};
          *reinterpret_cast<floatx4_t*>(part + (((cb * 2 + ig) * 4 + q) * 256 + tid_after) * 4) = v;
        }
    part[64 * 256 + tid_after] = l[0];
    part[65 * 256 + tid_after] = l[1];
    return;
  }
  // were the scores inside the range of the reference-free form?
  const int bad = !(l[0] >= 0x1p-80f && l[0] <= 0x1p80f) | !(l[1] >= 0x1p-80f && l[1] <= 0x1p80f);
  if (__syncthreads_or(bad)) {
    count_fallback(a.fallback_count);
    attention_general<HD, NW>(a, head, q0, a.q_scale, &sK[0][0], &sV[0][0]);
    return;
  }
  attention_finish<NW>(a, head, q0, wave, lane_after, o, l, reinterpret_cast<char*>(&skv[0][0][0]));
}

// Adds up the key ranges of a split query block (one workgroup per block, same thread -> element
// mapping as the main kernel), then finishes it like an unsplit one.
template <int NW>
__global__ __launch_bounds__(NW * 64, 2) void attention_hd64_fixup_kernel(AttnArgs a, int n_qblocks, int n_blocks,
                                                                          int per_xcd, KeySplit ks) {
  constexpr int HD = 64;
  const int slot = ks.full_items + blockIdx.x;
  const int logical = (slot % 8) * per_xcd + slot / 8;
  if (logical >= n_blocks) return;
  const int head = logical / n_qblocks, qb = logical % n_qblocks;
  __shared__ u32x4_t skv[2][3][TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int q0 = qb * (NW * 64) + wave * 64;
  floatx16_t o[2][2];
  float l[2] = {0.f, 0.f};
#pragma unroll
  for (int cb = 0; cb < 2; ++cb)
#pragma unroll
    for (int ig = 0; ig < 2; ++ig)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[cb][ig][e] = 0.f;
  const float* part = ks.ws + (size_t)blockIdx.x * ks.split * PART_FLOATS;
  for (int c = 0; c < ks.split; ++c, part += PART_FLOATS) {
    floatx4_t v[16];
#pragma unroll
    for (int x = 0; x < 16; ++x) v[x] = __builtin_nontemporal_load(reinterpret_cast<const floatx4_t*>(part + (x * 256 + tid) * 4));
#pragma unroll
    for (int x = 0; x < 16; ++x)
#pragma unroll
      for (int e = 0; e < 4; ++e) o[x >> 3][(x >> 2) & 1][4 * (x & 3) + e] += v[x][e];
    l[0] += part[64 * 256 + tid];
    l[1] += part[65 * 256 + tid];
  }
  const int bad = !(l[0] >= 0x1p-80f && l[0] <= 0x1p80f) | !(l[1] >= 0x1p-80f && l[1] <= 0x1p80f);
  if (__syncthreads_or(bad)) {
    count_fallback(a.fallback_count);
    attention_general<HD, NW>(a, head, q0, a.q_scale, &skv[0][0][0], &skv[1][0][0]);
    return;
  }
  attention_finish<NW>(a, head, q0, wave, lane, o, l, reinterpret_cast<char*>(&skv[0][0][0]));
}

template <int NW>
__device__ __forceinline__ void attention_finish(const AttnArgs& a, int head, int q0, int wave, int lane,
                                                 floatx16_t (&o)[2][2], const float (&l)[2], char* lds) {
  constexpr int HD = 64;
  const int d = a.n_heads * HD;
  const int lr = lane & 31, lh = lane >> 5;
  // ---- normalise; the wave's 64 x 64 block goes through LDS (the K/V buffers are idle now: every
  //      wave passed the barrier above after its last fragment read) so that each query's 128-byte
  //      output row leaves as one full cache line: lane owns query column lr, channels 8q + 4lh + e ----
  constexpr int OST = 136;                       // staging row stride in bytes (128 + 8: conflict-free 8-byte writes)
  static_assert(NW * 64 * OST <= 2 * 3 * TILE * 16, "output staging must fit the K/V buffers");
  char* stage = lds + wave * (64 * OST);
#pragma unroll
  for (int ig = 0; ig < 2; ++ig) {
    const float inv = 1.0f / l[ig];
#pragma unroll
    for (int cb = 0; cb < 2; ++cb)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u32x2_t pk = {pack_bf16x2_hw(o[cb][ig][4 * q] * inv, o[cb][ig][4 * q + 1] * inv),
                      pack_bf16x2_hw(o[cb][ig][4 * q + 2] * inv, o[cb][ig][4 * q + 3] * inv)};
        *reinterpret_cast<u32x2_t*>(stage + (ig * 32 + lr) * OST + (cb * 32 + 8 * q + 4 * lh) * 2) = pk;
      }
  }
  // 64 rows x 8 pieces of 16 bytes; the wave reads back only what it wrote itself
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int row = it * 8 + (lane >> 3), piece = lane & 7;
    const u32x2_t lo = *reinterpret_cast<const u32x2_t*>(stage + row * OST + piece * 16);
    const u32x2_t hi = *reinterpret_cast<const u32x2_t*>(stage + row * OST + piece * 16 + 8);
    const int qrow = q0 + row;
    if (qrow < a.r) {
      u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
      *reinterpret_cast<u32x4_t*>(a.o + (int64_t)qrow * d + head * HD + piece * 8) = v;
    }
  }
}

template <int HD, int NW>
hipError_t launch_cfg(const AttnArgs& a, hipStream_t st) {
  int n_qblocks = (a.r + NW * 64 - 1) / (NW * 64);
  int n_blocks = n_qblocks * a.n_heads;
  int per_xcd = (n_blocks + 7) / 8;
  if (HD == 64) {
    // The chip runs 512 of these workgroups at a time (two per CU).  The n_rem blocks of the last
    // round are cut into s key ranges so that the round takes ceil(n_rem*s/512)/s of a block's
    // time (plus about two key tiles of pipeline fill per range); s minimises that.
    KeySplit ks;
    const int slots = per_xcd * 8;
    ks.full_items = slots / 512 * 512;
    ks.split = 1;
    ks.ws = a.split_ws;
    const int n_rem = slots - ks.full_items;
    const int key_tiles = a.n_keys / BKV;
    if (a.split_ws != nullptr && n_rem > 0) {
      const int s_max = (int)std::min<size_t>((size_t)std::min(key_tiles / 16, 16),
                                              a.split_ws_bytes / ((size_t)n_rem * PART_FLOATS * sizeof(float)));
      double best = 1.0;
      for (int sp = 2; sp <= s_max; ++sp) {
        const double t = (double)((n_rem * sp + 511) / 512) / sp * (1.0 + 2.0 * sp / key_tiles) + 0.004 * sp;
        if (t < best - 0.02) { best = t; ks.split = sp; }
      }
    }
    if (ks.split == 1) ks.full_items = slots;
    const int n_split = slots - ks.full_items;
    hipLaunchKernelGGL((attention_hd64_kernel<NW>), dim3(ks.full_items + n_split * ks.split), dim3(NW * 64), 0, st, a,
                       n_qblocks, n_blocks, per_xcd, ks);
    if (n_split > 0)
      hipLaunchKernelGGL((attention_hd64_fixup_kernel<NW>), dim3(n_split), dim3(NW * 64), 0, st, a, n_qblocks,
                         n_blocks, per_xcd, ks);
  } else
    hipLaunchKernelGGL((attention_general_kernel<HD, NW>), dim3(per_xcd * 8), dim3(NW * 64), 0, st, a, n_qblocks,
                       n_blocks, per_xcd);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.r <= 0 || a.n_keys <= 0) return hipSuccess;
  if (a.ld_vt % 64 != 0 || a.ld_vt < a.n_keys) return hipErrorInvalidValue;
  // K and V^T are addressed with 32-bit byte offsets
  if (((int64_t)a.n_keys + 4 * BKV) * a.n_heads * a.head_dim * 2 >= ((int64_t)1 << 32) ||
      (int64_t)a.n_heads * a.head_dim * a.ld_vt * 2 >= ((int64_t)1 << 32))
    return hipErrorInvalidValue;
  if (a.head_dim == 64) return launch_cfg<64, 4>(a, st);
  if (a.head_dim == 32) return launch_cfg<32, 4>(a, st);
  return hipErrorInvalidValue;
}
