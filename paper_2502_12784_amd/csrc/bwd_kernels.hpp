// Attention backward for gfx950 (paper Sec. 3.3, Eq. 4), three kernels on one stream:
//
//   mha_bwd_dot_kernel  : D_i = sum_k dO_ik O_ik                 (the paper's "dPsum")
//   mha_bwd_dkdv_kernel : one workgroup per tile of 128 keys, loops over query tiles,
//                         recomputes P = exp(S - LSE), accumulates dV = P^T dO and
//                         dK = scale * dS^T Q in registers, writes them once (as in Sec. 3.3,
//                         where each thread block owns a slice of dK and dV).
//   mha_bwd_dq_kernel   : one workgroup per tile of 128 queries, loops over key tiles,
//                         recomputes P and dS and accumulates dQ = scale * dS K in registers.
//
// The paper adds every block's dQ contribution into HBM with atomic adds.  Here dQ has its
// own pass with the forward's loop structure instead: it costs two recomputed contractions
// (7 executed for 5 counted) but needs no fp32 dQ buffer to zero and convert, no atomics, and
// gives bitwise reproducible gradients.
//
// Register layouts follow mma_gfx950.hpp.  In the dK/dV kernel the score tile is computed as
// S = Q K^T (lane = key column, registers = query rows) so that P and dS, packed to 16 bits,
// are directly the B operands of dV^T = dO^T P and dK^T = Q^T dS; the dO^T / Q^T operands
// come from the row-major LDS tiles through transposing reads.  In the dQ kernel everything
// is transposed as in the forward (lane = query column), so LSE_i and D_i are per-lane
// scalars and dS^T is directly the B operand of dQ^T = K^T dS^T.
#pragma once
#include "fwd_kernel.hpp"
#include "mma_gfx950.hpp"

namespace spark {

// ---------------------------------------------------------------------------------------
// D = rowsum(dO o O).  One thread per 16-byte chunk of a row; D/8 neighbouring lanes share a
// row and reduce with shuffles.  Pure streaming: reads two tensors, writes BH*N floats.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void mha_bwd_dot_kernel(const T* __restrict__ O,
                                                         const T* __restrict__ dO,
                                                         float* __restrict__ Dout, int64_t rows) {
  using v8 = typename Frag<T>::v8;
  constexpr int CPR = D / 8;
  const int64_t chunk = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t row = chunk / CPR;
  float acc = 0.f;
  if (row < rows) {
    const v8 a = *reinterpret_cast<const v8*>(O + chunk * 8);
    const v8 b = *reinterpret_cast<const v8*>(dO + chunk * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += (float)a[i] * (float)b[i];
  }
#pragma unroll
  for (int off = CPR / 2; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
  if (row < rows && (threadIdx.x % CPR) == 0) Dout[row] = acc;
}

// ---------------------------------------------------------------------------------------
// Shared pieces
// ---------------------------------------------------------------------------------------

// Copy ROWS x D 16-bit elements (rows r0.., clamped to N-1) from a row-major global matrix
// into registers, 16 bytes per thread per step, and from registers into a padded LDS tile.
template <int D, int ROWS, typename T>
static __device__ __forceinline__ void tile_g2r(const T* __restrict__ base, int r0, int N, int tid,
                                                u32x4 (&reg)[ROWS * (D / 8) / 256]) {
  constexpr int CPR = D / 8;
#pragma unroll
  for (int i = 0; i < ROWS * CPR / 256; ++i) {
    const int c = tid + 256 * i;
    const int row = c / CPR, cc = c % CPR;
    int grow = r0 + row;
    grow = grow < N ? grow : N - 1;
    reg[i] = *reinterpret_cast<const u32x4*>(base + (size_t)grow * D + cc * 8);
  }
}

template <int D, int ROWS, int STRIDE>
static __device__ __forceinline__ void tile_r2s(SPARK_LDS char* dst, int tid,
                                                const u32x4 (&reg)[ROWS * (D / 8) / 256]) {
  constexpr int CPR = D / 8;
#pragma unroll
  for (int i = 0; i < ROWS * CPR / 256; ++i) {
    const int c = tid + 256 * i;
    const int row = c / CPR, cc = c % CPR;
    lds_write(dst, row * STRIDE + cc * 16, reg[i]);
  }
}

// Write a wave's transposed accumulator (D x 32, lane = column) times `mul` as 32 rows of D
// 16-bit values: through the wave's LDS slice `ob`, then 16-byte row stores for rows < N.
template <typename T, int D, int OSTR>
static __device__ __forceinline__ void store_transposed(const f32x16 (&acc)[D / 32], float mul,
                                                        SPARK_LDS char* ob, T* __restrict__ out,
                                                        int row0, int N, int lane) {
  using v4 = typename Frag<T>::v4;
  constexpr int CPR = D / 8;
  constexpr int RPP = 64 / CPR;
  const int g = lane >> 5, c32 = lane & 31;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      v4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (T)(acc[dt][r4 * 4 + e] * mul);
      lds_write(ob, c32 * OSTR + (dt * 32 + 8 * r4 + 4 * g) * 2, pk);
    }
#pragma unroll
  for (int p = 0; p < 32 / RPP; ++p) {
    const int row = p * RPP + lane / CPR, cc = lane % CPR;
    const u32x4 v = lds_read16<u32x4>(ob, row * OSTR + cc * 16);
    if (row0 + row < N) *reinterpret_cast<u32x4*>(out + (size_t)(row0 + row) * D + cc * 8) = v;
  }
}

// A-operand (32 rows of the TRANSPOSE of a row-major LDS tile, 16 k-slots) for d-tile `dt`:
// k-slot (g, j) is tile row  rbase + 8*(j/4) + 4g + (j%4)  (the order of packed C registers).
template <typename T, int STRIDE>
static __device__ __forceinline__ typename Frag<T>::v8 read_transposed(SPARK_LDS const char* tile,
                                                                      int rbase, int dt, int lane) {
  using v8 = typename Frag<T>::v8;
  using v4 = typename Frag<T>::v4;
  const int g = lane >> 5, c32 = lane & 31, i16 = lane & 15;
  const int row0 = rbase + 4 * g + (i16 >> 2);
  const int col = dt * 32 + (c32 & 16) + 4 * (i16 & 3);
  const v4 lo = lds_read_tr8<v4>(tile, row0 * STRIDE + col * 2);
  const v4 hi = lds_read_tr8<v4>(tile, (row0 + 8) * STRIDE + col * 2);
  return join4<v8, v4>(lo, hi);
}

// ---------------------------------------------------------------------------------------
// dK, dV
// ---------------------------------------------------------------------------------------
template <int D> struct BwdKvCfg {
  static constexpr int BN = 128;  // keys per workgroup (32 per wave)
  static constexpr int BM = 64;   // query rows per LDS stage (two 32-row steps)
  static constexpr int STR = D * 2 + 16;
  static constexpr int TILE = BM * STR;  // one of Q, dO
  static constexpr int STAT = 2 * BM * 4;  // LSE*log2(e) and D of the stage's rows
  static constexpr int STAGE = 2 * TILE + STAT;
  static constexpr int OSTR = D * 2 + 16;
  static constexpr int SMEM = 2 * STAGE;
  static_assert(4 * 32 * OSTR <= SMEM, "epilogue staging must fit");
};

template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(256) void mha_bwd_dkdv_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Dws,
    T* __restrict__ dK, T* __restrict__ dV, int N, int nkt, float scale, float scale_log2) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using C = BwdKvCfg<D>;
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int NLD = C::BM * (D / 8) / 256;

  extern __shared__ __attribute__((aligned(16))) char smem_generic[];
  SPARK_LDS char* smem = (SPARK_LDS char*)smem_generic;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31;

  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / nkt;
  const int kt = logical - head * nkt;  // causal: low key tiles (most queries) come first

  const size_t head_off = (size_t)head * N * D;
  const T* Qh = Q + head_off;
  const T* dOh = dO + head_off;
  const float* LSEh = LSE + (size_t)head * N;
  const float* Dh = Dws + (size_t)head * N;

  const int k0w = kt * C::BN + wave * 32;  // first key of this wave
  const int krow = k0w + c32;
  const int krow_c = krow < N ? krow : N - 1;

  v8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *reinterpret_cast<const v8*>(K + head_off + (size_t)krow_c * D + ks * 16 + g * 8);
    vf[ks] = *reinterpret_cast<const v8*>(V + head_off + (size_t)krow_c * D + ks * 16 + g * 8);
  }

  f32x16 dk[DT], dv[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }

  const int ns = (N + C::BM - 1) / C::BM;              // query stages in the sequence
  const int s_begin = CAUSAL ? (kt * C::BN) / C::BM : 0;  // queries before the tile's first key see none of it

  u32x4 qreg[NLD], doreg[NLD];
  float statreg = 0.f;
  auto load_stage = [&](int m) {
    tile_g2r<D, C::BM>(Qh, m * C::BM, N, tid, qreg);
    tile_g2r<D, C::BM>(dOh, m * C::BM, N, tid, doreg);
    if (tid < 2 * C::BM) {
      const int row = m * C::BM + (tid & (C::BM - 1));
      if (tid < C::BM)  // rows past the end get LSE = +inf so that P = 0 there
        statreg = row < N ? LSEh[row] * 1.4426950408889634f : INFINITY;
      else
        statreg = row < N ? Dh[row] : 0.f;
    }
  };
  auto store_stage = [&](int buf) {
    SPARK_LDS char* sb = smem + buf * C::STAGE;
    tile_r2s<D, C::BM, C::STR>(sb, tid, qreg);
    tile_r2s<D, C::BM, C::STR>(sb + C::TILE, tid, doreg);
    if (tid < 2 * C::BM) lds_write(sb + 2 * C::TILE, tid * 4, statreg);
  };

  if (s_begin < ns) {
    load_stage(s_begin);
    store_stage(0);
  }
  __syncthreads();

  for (int m = s_begin; m < ns; ++m) {
    const int buf = (m - s_begin) & 1;
    if (m + 1 < ns) load_stage(m + 1);

    SPARK_LDS const char* qb = smem + buf * C::STAGE;
    SPARK_LDS const char* dob = qb + C::TILE;
    SPARK_LDS const char* stb = dob + C::TILE;

#pragma unroll
    for (int sub = 0; sub < C::BM / 32; ++sub) {
      const int q0s = m * C::BM + sub * 32;
      if (CAUSAL && q0s + 31 < k0w) continue;  // every query here precedes every key of the wave
      if (q0s >= N) continue;

      f32x16 s, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int off = (sub * 32 + c32) * C::STR + ks * 32 + g * 16;
        const v8 qa = lds_read16<v8>(qb, off);
        s = F::mfma(qa, kf[ks], s);
        const v8 da = lds_read16<v8>(dob, off);
        dp = F::mfma(da, vf[ks], dp);
      }

      float p[16], ds[16];
      const bool need_mask = CAUSAL && q0s < k0w + 31;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int qoff = sub * 32 + 8 * r4 + 4 * g;
        const f32x4 l4 = lds_read16<f32x4>(stb, qoff * 4);
        const f32x4 d4 = lds_read16<f32x4>(stb, (C::BM + qoff) * 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = r4 * 4 + e;
          float pe = __builtin_amdgcn_exp2f(s[r] * scale_log2 - l4[e]);
          if (need_mask && krow > m * C::BM + qoff + e) pe = 0.f;
          p[r] = pe;
          ds[r] = pe * (dp[r] - d4[e]);
        }
      }

#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const v8 pf = pack8<T>(&p[kk * 8]);
        const v8 dsf = pack8<T>(&ds[kk * 8]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const v8 doT = read_transposed<T, C::STR>(dob, sub * 32 + 16 * kk, dt, lane);
          dv[dt] = F::mfma(doT, pf, dv[dt]);
          const v8 qT = read_transposed<T, C::STR>(qb, sub * 32 + 16 * kk, dt, lane);
          dk[dt] = F::mfma(qT, dsf, dk[dt]);
        }
      }
    }

    if (m + 1 < ns) store_stage(buf ^ 1);
    __syncthreads();
  }

  SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
  store_transposed<T, D, C::OSTR>(dk, scale, ob, dK + head_off, k0w, N, lane);
  store_transposed<T, D, C::OSTR>(dv, 1.0f, ob, dV + head_off, k0w, N, lane);
}

// ---------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------
template <int D> struct BwdQCfg {
  static constexpr int BM = 128;  // query rows per workgroup (32 per wave)
  static constexpr int BN = 64;   // keys per iteration
  static constexpr int STR = D * 2 + 16;
  static constexpr int TILE = BN * STR;  // one of K, V
  static constexpr int STAGE = 2 * TILE;
  static constexpr int OSTR = D * 2 + 16;
  static constexpr int SMEM = 2 * STAGE;
  static_assert(4 * 32 * OSTR <= SMEM, "epilogue staging must fit");
};

template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(256) void mha_bwd_dq_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ Dws,
    T* __restrict__ dQ, int N, int nqt, float scale, float scale_log2) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using C = BwdQCfg<D>;
  constexpr int KS = D / 16, DT = D / 32;
  constexpr int NLD = C::BN * (D / 8) / 256;

  extern __shared__ __attribute__((aligned(16))) char smem_generic[];
  SPARK_LDS char* smem = (SPARK_LDS char*)smem_generic;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31;

  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / nqt;
  const int rank = logical - head * nqt;
  const int qt = CAUSAL ? nqt - 1 - rank : rank;

  const size_t head_off = (size_t)head * N * D;
  const T* Kh = K + head_off;
  const T* Vh = V + head_off;

  const int q0 = qt * C::BM + wave * 32;
  const int qrow = q0 + c32;
  const int qrow_c = qrow < N ? qrow : N - 1;

  v8 qf[KS], dof[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *reinterpret_cast<const v8*>(Q + head_off + (size_t)qrow_c * D + ks * 16 + g * 8);
    dof[ks] = *reinterpret_cast<const v8*>(dO + head_off + (size_t)qrow_c * D + ks * 16 + g * 8);
  }
  const float lse2 = LSE[(size_t)head * N + qrow_c] * 1.4426950408889634f;
  const float Dq = Dws[(size_t)head * N + qrow_c];

  int kv_end = N;
  if (CAUSAL) {
    const int lim = (qt + 1) * C::BM;
    kv_end = lim < N ? lim : N;
  }
  const int nt = (kv_end + C::BN - 1) / C::BN;

  u32x4 kreg[NLD], vreg[NLD];
  f32x16 dq[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;

  tile_g2r<D, C::BN>(Kh, 0, N, tid, kreg);
  tile_g2r<D, C::BN>(Vh, 0, N, tid, vreg);
  tile_r2s<D, C::BN, C::STR>(smem, tid, kreg);
  tile_r2s<D, C::BN, C::STR>(smem + C::TILE, tid, vreg);
  __syncthreads();

  for (int j = 0; j < nt; ++j) {
    const int buf = j & 1;
    if (j + 1 < nt) {
      tile_g2r<D, C::BN>(Kh, (j + 1) * C::BN, N, tid, kreg);
      tile_g2r<D, C::BN>(Vh, (j + 1) * C::BN, N, tid, vreg);
    }
    const int k0 = j * C::BN;
    if (!CAUSAL || k0 <= q0 + 31) {
      SPARK_LDS const char* kb = smem + buf * C::STAGE;
      SPARK_LDS const char* vb = kb + C::TILE;

      f32x16 s[2], dp[2];
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[mt][r] = 0.f; dp[mt][r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
          const int off = (mt * 32 + c32) * C::STR + ks * 32 + g * 16;
          const v8 ka = lds_read16<v8>(kb, off);
          s[mt] = F::mfma(ka, qf[ks], s[mt]);
          const v8 va = lds_read16<v8>(vb, off);
          dp[mt] = F::mfma(va, dof[ks], dp[mt]);
        }
      }

      float ds[32];
      const bool need_mask = (CAUSAL && k0 + C::BN - 1 > q0) || (k0 + C::BN > N);
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float pe = __builtin_amdgcn_exp2f(s[mt][r] * scale_log2 - lse2);
          if (need_mask) {
            const int key = k0 + mt * 32 + 8 * (r / 4) + 4 * g + (r % 4);
            const bool ok = key < N && (!CAUSAL || key <= qrow);
            if (!ok) pe = 0.f;
          }
          ds[mt * 16 + r] = pe * (dp[mt][r] - Dq);
        }

#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const v8 dsf = pack8<T>(&ds[kk * 8]);
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const v8 kT = read_transposed<T, C::STR>(kb, 16 * kk, dt, lane);
          dq[dt] = F::mfma(kT, dsf, dq[dt]);
        }
      }
    }
    if (j + 1 < nt) {
      tile_r2s<D, C::BN, C::STR>(smem + (buf ^ 1) * C::STAGE, tid, kreg);
      tile_r2s<D, C::BN, C::STR>(smem + (buf ^ 1) * C::STAGE + C::TILE, tid, vreg);
    }
    __syncthreads();
  }

  SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
  store_transposed<T, D, C::OSTR>(dq, scale, ob, dQ + head_off, q0, N, lane);
}

}  // namespace spark
