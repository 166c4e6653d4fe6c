// Flash-style attention of refreshed queries against the full cached K/V
// (FullAttn of Eq. 2 evaluated on the selected rows of Eq. 3): O = softmax(Q K^T / sqrt(hd)) V
// per head, never materialising the score matrix.
//
// Layout: Q [r, H*hd] and K [N, H*hd] row-major, V transposed [H*hd, ld_vt] (key index
// contiguous), O [r, H*hd].
//
// One workgroup = NW waves x 64 queries of one head.  Keys are walked in tiles of 64 staged
// through LDS (K tile [64 keys][hd], V^T tile [hd][64 keys], 16-byte chunks XOR-swizzled so
// that ds_read_b128 fragment reads are bank-conflict free), double-buffered with register
// prefetch.  Per tile a wave computes S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (A = K rows,
// B = Q rows held in registers for the whole kernel), so every lane owns one query column:
// its 32 accumulator values are 32 different keys of the same query, and the row max / row
// sum of the online softmax are in-lane reductions plus one exchange with lane^32.
// exp2 is used with the 1/sqrt(hd)*log2(e) scale folded into one FMA; probabilities are
// rounded to bf16 by the hardware pack conversion and summed with v_dot2 on the rounded values.  P^T goes straight
// from the accumulators (rounded to bf16) into the B operand of O^T += V^T P^T: the K rows
// are read in a permuted order (bits 2 and 3 of the row index swapped) so that the eight
// k-slots a lane feeds to one PV MFMA are eight consecutive keys, which makes the V^T
// fragment a single 16-byte LDS read.
#include "hero_device.h"
#include "hero_kernels.h"

namespace {

constexpr int BKV = 64;   // keys per tile

template <int HD, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attention_kernel(AttnArgs a, int n_qblocks, int n_blocks,
                                                               int per_xcd, float scale_log2e) {
  constexpr int T = NW * 64;
  constexpr int KCH = HD / 8;             // 16-byte chunks per K-tile row
  constexpr int VCH = BKV / 8;            // 16-byte chunks per V^T-tile row
  constexpr int KS = HD / 16;             // k-steps of the QK^T MFMA
  constexpr int CB = HD / 32;             // 32-row blocks of O^T
  constexpr int NKL = BKV * KCH / T;      // K chunks per thread per tile
  constexpr int NVL = HD * VCH / T;       // V^T chunks per thread per tile
  static_assert(BKV * KCH % T == 0 && HD * VCH % T == 0, "tile/threads mismatch");
  constexpr int K_TILE = BKV * KCH, V_TILE = HD * VCH;   // in 16-byte chunks

  // each XCD (consecutive workgroup ids round-robin over 8 XCDs) gets a contiguous range of heads
  int logical = (blockIdx.x % 8) * per_xcd + blockIdx.x / 8;
  if (logical >= n_blocks) return;
  const int head = logical / n_qblocks, qb = logical % n_qblocks;
  const int d = a.n_heads * HD;

  __shared__ u32x4_t sK[2][K_TILE];
  __shared__ u32x4_t sV[2][V_TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 31, lh = lane >> 5;
  const int q0 = qb * (NW * 64) + wave * 64;

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
    for (int i = 0; i < NKL; ++i) sK[buf][k_off[i]] = rk[i];
#pragma unroll
    for (int i = 0; i < NVL; ++i) sV[buf][v_off[i]] = rv[i];
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
        u32x4_t t = sK[cur][row * KCH + ((2 * ks + lh) ^ ((row >> 1) & (KCH - 1)))];
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
      typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
      const bf16x2_t ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
      for (int jb = 0; jb < 2; ++jb) {
        uint32_t pk[8];
#pragma unroll
        for (int e2 = 0; e2 < 8; ++e2) {
          float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[jb][ig][2 * e2], scale_log2e, -m_ref));
          float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[jb][ig][2 * e2 + 1], scale_log2e, -m_ref));
          pk[e2] = pack_bf16x2_hw(p0, p1);
          // the row sum uses the rounded probabilities, exactly what multiplies V
          psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pk[e2]), ones, psum, false);
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
          u32x4_t tv = sV[cur][row * VCH + ((4 * jb + 2 * t + lh) ^ ((row >> 1) & (VCH - 1)))];
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
hipError_t launch_cfg(const AttnArgs& a, hipStream_t st) {
  int n_qblocks = (a.r + NW * 64 - 1) / (NW * 64);
  int n_blocks = n_qblocks * a.n_heads;
  int per_xcd = (n_blocks + 7) / 8;
  float scale_log2e = 1.4426950408889634f / sqrtf((float)HD);
  hipLaunchKernelGGL((attention_kernel<HD, NW>), dim3(per_xcd * 8), dim3(NW * 64), 0, st, a, n_qblocks,
                     n_blocks, per_xcd, scale_log2e);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.r <= 0 || a.n_keys <= 0) return hipSuccess;
  if (a.ld_vt % 64 != 0 || a.ld_vt < a.n_keys) return hipErrorInvalidValue;
  if (a.head_dim == 64) return launch_cfg<64, 4>(a, st);
  if (a.head_dim == 32) return launch_cfg<32, 4>(a, st);
  return hipErrorInvalidValue;
}
