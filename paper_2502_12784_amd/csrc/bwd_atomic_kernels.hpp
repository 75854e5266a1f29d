// Attention backward as the paper builds it (Sec. 3.3): ONE fused kernel in which every workgroup
// owns a slice of dK and dV, accumulates them on chip, and adds its contribution to dQ into HBM
// with atomic adds in every iteration; five contractions are executed for five counted.
//
//   mha_bwd_prep_kernel        : D_i = sum_k dO_ik O_ik (the paper's "dPsum"), LSE * log2(e), and the
//                                fp32 dQ accumulator cleared (a fill kernel, not a memset, so that
//                                the sequence can be captured in a HIP graph).
//   mha_bwd_fused_atomic_kernel: one workgroup per tile of 128 keys (32 per wave); per stage of 64
//                                queries: S = Q K^T and dP = dO V^T on the matrix cores,
//                                P = exp(S - LSE), dS = P o (dP - D), dV += P^T dO, dK += dS^T Q in
//                                registers; dS goes through LDS to all four waves, which form
//                                dQ_stage = dS K (64 x d, each wave one 32-column slice) and add it to
//                                the fp32 accumulator with global_atomic_add_f32.
//   mha_bwd_dq_convert_kernel  : dQ = scale * accumulator, rounded once to 16 bits.
//
// This variant exists to be measured against the two-kernel backward of bwd_kernels.hpp (separate
// deterministic dQ pass, seven contractions executed).  On MI355X it loses: the chip retires fp32
// atomic adds at about 1.3 TB/s of operand bytes (one 128-byte line per ~25 clocks and L2 channel,
// measured with this kernel's exact access pattern and nothing else running), and with 128 keys
// per workgroup every element of dQ receives N/128 adds: 2.2 GB for N = 4096, d = 128, 64 heads,
// causal, i.e. 1.7 ms of atomic traffic against 0.4 ms for the whole separate dQ pass.  The fused
// kernel is therefore written for clarity, not software-pipelined like the dK/dV kernel: its
// run time is set by the atomic units whatever the rest does.  Results differ from run to run in
// the last bits of dQ (the order of the adds is not fixed); dK and dV are reproducible.
#pragma once
#include "mma_gfx950.hpp"
#include "tiles_gfx950.hpp"

namespace spark {

// ---------------------------------------------------------------------------------------
// D, LSE * log2(e), and clearing of the dQ accumulator.  16 lanes per query row, 8 elements each.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void mha_bwd_prep_kernel(const T* __restrict__ O, const T* __restrict__ dO,
                                                           const float* __restrict__ LSE,
                                                           float* __restrict__ Dout, float* __restrict__ LSE2out,
                                                           float* __restrict__ dQacc, TensorMap mo, TensorMap mdo,
                                                           int H, int Nq, int dh, long long rows) {
  using v8 = typename Frag<T>::v8;
  const long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);  // flat (head, query) index
  const int part = threadIdx.x & 15;
  const bool live = row < rows;
  const long long r = live ? row : rows - 1;
  const int head = (int)(r / Nq), q = (int)(r - (long long)head * Nq);
  float acc = 0.f;
  if (part * 8 < dh) {
    const v8 o = *reinterpret_cast<const v8*>(O + head_base(mo, head, H) + (size_t)q * (size_t)mo.row + part * 8);
    const v8 g = *reinterpret_cast<const v8*>(dO + head_base(mdo, head, H) + (size_t)q * (size_t)mdo.row + part * 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc = __builtin_fmaf((float)o[i], (float)g[i], acc);
    if (live) {
      f32x4* z = reinterpret_cast<f32x4*>(dQacc + (size_t)r * dh + part * 8);
      z[0] = f32x4{0.f, 0.f, 0.f, 0.f};
      z[1] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
#pragma unroll
  for (int m = 8; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 16);
  if (live && part == 0) {
    Dout[r] = acc;
    LSE2out[r] = LSE[r] * 1.4426950408889634f;
  }
}

// dQ = scale * accumulator -> 16 bits; one lane per 8 elements.
template <typename T>
__global__ __launch_bounds__(256) void mha_bwd_dq_convert_kernel(const float* __restrict__ dQacc, T* __restrict__ dQ,
                                                                 TensorMap mdq, int H, int Nq, int dh, float scale,
                                                                 long long chunks) {
  using v8 = typename Frag<T>::v8;
  const long long c = (long long)blockIdx.x * 256 + threadIdx.x;
  if (c >= chunks) return;
  const int cpr = dh >> 3;
  const long long row = c / cpr;
  const int part = (int)(c - row * cpr);
  const int head = (int)(row / Nq), q = (int)(row - (long long)head * Nq);
  const f32x4* src = reinterpret_cast<const f32x4*>(dQacc + (size_t)row * dh + part * 8);
  const f32x4 a = src[0], b = src[1];
  v8 out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[i] = (T)(a[i] * scale);
    out[4 + i] = (T)(b[i] * scale);
  }
  *reinterpret_cast<v8*>(dQ + head_base(mdq, head, H) + (size_t)q * (size_t)mdq.row + part * 8) = out;
}

// ---------------------------------------------------------------------------------------
// The fused kernel.  LDS: [K tile 128 x D | 2 stage slots (Q 64 x D, dO 64 x D) | statistics of the
// two slots | dS exchange, 2 (stage parity) x 2 (32-query step) x 128 keys x 32 queries, 16 bit].
// ---------------------------------------------------------------------------------------
template <int D> struct BwdAtomicCfg {
  static constexpr int BN = 128, BM = 64;
  static constexpr int ROWB = D * 2;
  static constexpr int KTILE = BN * ROWB;
  static constexpr int TILE = BM * ROWB;
  static constexpr int STAGE = 2 * TILE;
  static constexpr int STAT = 2 * BM * 4;
  static constexpr int SLOT0 = KTILE;
  static constexpr int STAT0 = SLOT0 + 2 * STAGE;
  static constexpr int DSX0 = STAT0 + 2 * STAT;
  static constexpr int DSX_STEP = BN * 32 * 2;  // one 32-query step: 128 key rows of 64 bytes
  static constexpr int SMEM = DSX0 + 4 * DSX_STEP;
  static constexpr int OSTR = D * 2 + 16;
  static_assert(4 * 32 * OSTR <= SMEM, "epilogue staging must fit");
};

template <typename T, int D, bool CAUSAL>
__global__ __launch_bounds__(256, 1) void mha_bwd_fused_atomic_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const float* __restrict__ LSE2, const float* __restrict__ Dws, float* __restrict__ dQacc,
    T* __restrict__ dK, T* __restrict__ dV, TensorMap mq, TensorMap mk, TensorMap mv, TensorMap mdo,
    TensorMap mdk, TensorMap mdv, int H, int Nq, int Nk, int dh, int nkt, float scale) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using v4 = typename F::v4;
  using C = BwdAtomicCfg<D>;
  constexpr int KS = D / 16, DT = D / 32;

  SPARK_LDS char* const smem = lds_origin();
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31, i16 = lane & 15;

  const int items = causal_items<CAUSAL>(nkt);  // causal: key tiles (p, nkt-1-p) are paired
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / items;
  const int item = logical - head * items;

  const T* Vh = V + head_base(mv, head, H);
  const BufView kview(K + head_base(mk, head, H), head_span_bytes(mk, Nk, dh));
  const BufView qview(Q + head_base(mq, head, H), head_span_bytes(mq, Nq, dh));
  const BufView doview(dO + head_base(mdo, head, H), head_span_bytes(mdo, Nq, dh));
  const BufView lview(LSE2 + (size_t)head * Nq, (uint32_t)Nq * 4), dview(Dws + (size_t)head * Nq, (uint32_t)Nq * 4);
  const uint32_t k_row_bytes = (uint32_t)mk.row * 2, q_row_bytes = (uint32_t)mq.row * 2,
                 do_row_bytes = (uint32_t)mdo.row * 2;
  const uint32_t k_lane_src = dma_lane_src<D>(wave, lane, k_row_bytes, dh);
  const uint32_t q_lane_src = dma_lane_src<D>(wave, lane, q_row_bytes, dh);
  const uint32_t do_lane_src = dma_lane_src<D>(wave, lane, do_row_bytes, dh);
  const float scale_log2 = scale * 1.4426950408889634f;
  float* const acc_head = dQacc + (size_t)head * Nq * dh;
  const SwzLane<D> off(lane);

  for (int rep = 0; rep < (CAUSAL ? 2 : 1); ++rep) {
    const int kt = CAUSAL ? (rep == 0 ? item : nkt - 1 - item) : item;  // the long tile first
    if (CAUSAL && rep == 1) {
      if (kt == item) break;  // odd tile count: the middle tile has no partner
      __syncthreads();        // the first tile's epilogue is done with the LDS
    }
    const int k0w = kt * C::BN + wave * 32;
    const int krow = k0w + c32;  // this lane's key
    const int krow_c = krow < Nk ? krow : Nk - 1;
    const int ns = (Nq + C::BM - 1) / C::BM;
    const int s_begin = CAUSAL ? (kt * C::BN) / C::BM : 0;

    auto fetch_stage = [&](int m, int slot) {
      SPARK_LDS char* sb = smem + C::SLOT0 + slot * C::STAGE;
      tile_dma<D, C::BM>(qview, m * C::BM, sb, wave, q_lane_src, q_row_bytes);
      tile_dma<D, C::BM>(doview, m * C::BM, sb + C::TILE, wave, do_lane_src, do_row_bytes);
      SPARK_LDS char* st = smem + C::STAT0 + slot * C::STAT;
      if (wave == 0) lview.load4_to_lds(st, lane * 4, (uint32_t)m * C::BM * 4);
      if (wave == 1) dview.load4_to_lds(st + C::BM * 4, lane * 4, (uint32_t)m * C::BM * 4);
    };

    // K tile into LDS (rows past the end of the keys arrive as zeros: they add nothing to dQ);
    // the wave's own K and V rows as MFMA fragments in registers
    tile_dma<D, C::BN>(kview, kt * C::BN, smem, wave, k_lane_src, k_row_bytes);
    fetch_stage(s_begin, 0);
    v8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      vf[ks] = load_row_chunk<v8>(Vh + (size_t)krow_c * (size_t)mv.row, ks * 16 + g * 8, dh);
    wait_vmem_all();
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kf[ks] = lds_read16<v8>(smem, off.row[ks] + wave * 32 * C::ROWB);

    f32x16 dk[DT], dv[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }

    for (int m = s_begin; m < ns; ++m) {
      const int slot = (m - s_begin) & 1;
      if (m + 1 < ns) fetch_stage(m + 1, slot ^ 1);  // everybody left that slot before the last barrier
      SPARK_LDS const char* qb = smem + C::SLOT0 + slot * C::STAGE;
      SPARK_LDS const char* dob = qb + C::TILE;
      SPARK_LDS char* dsx = smem + C::DSX0 + slot * 2 * C::DSX_STEP;

#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int q0 = m * C::BM + sub * 32;
        // S = Q K^T and dP = dO V^T: lane = key column, registers = query rows
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const v8 aq = lds_read16<v8>(qb, off.row[ks] + sub * 32 * C::ROWB);
          const v8 ag = lds_read16<v8>(dob, off.row[ks] + sub * 32 * C::ROWB);
          s = F::mfma(aq, kf[ks], s);
          dp = F::mfma(ag, vf[ks], dp);
        }
        // P = exp(S - LSE), dS = P o (dP - D); register r is query row 8 (r/4) + 4g + (r%4)
        float p[16], ds[16];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int so = C::STAT0 + slot * C::STAT + (sub * 32 + 8 * r4 + 4 * g) * 4;
          const f32x4 l = lds_read16<f32x4>(smem, so), dd = lds_read16<f32x4>(smem, so + C::BM * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * r4 + e;
            float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -l[e]));
            const int qi = q0 + 8 * r4 + 4 * g + e;
            if (krow >= Nk || (CAUSAL && krow > qi)) pe = 0.f;
            p[r] = pe;
            ds[r] = pe * (dp[r] - dd[e]);
          }
        }
        const v8 pf[2] = {pack8<T>(&p[0]), pack8<T>(&p[8])};
        const v8 dsf[2] = {pack8<T>(&ds[0]), pack8<T>(&ds[8])};
        // dV^T += dO^T P and dK^T += Q^T dS (operands by transposing reads of the same tiles)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk)
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            const int o = (sub * 32 + kk * 16) * C::ROWB;
            dv[dt] = F::mfma(read_tr_pair<T>(dob, off.tr[0][dt] + o, off.tr[1][dt] + o), pf[kk], dv[dt]);
            dk[dt] = F::mfma(read_tr_pair<T>(qb, off.tr[0][dt] + o, off.tr[1][dt] + o), dsf[kk], dk[dt]);
          }
        // dS to the other waves: row = key (64 bytes: 32 queries), the lane's 16 queries are four
        // runs of four: elements 4x .. 4x+3 of dsf[kk] are queries 16 kk + 8 x + 4g + (0..3)
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const u32x4 w = __builtin_bit_cast(u32x4, dsf[kk]);
#pragma unroll
          for (int x = 0; x < 2; ++x)
            lds_write(dsx, sub * C::DSX_STEP + (wave * 32 + c32) * 64 + (16 * kk + 8 * x + 4 * g) * 2,
                      u32x2{w[2 * x], w[2 * x + 1]});
        }
      }
      wait_vmem_all();  // the next stage has landed
      __syncthreads();  // ... and every wave's dS of this stage is in LDS

      // dQ_stage = dS K: 2 steps x DT column slices of 32, dealt to the four waves.  Both operands
      // by transposing reads: A = dS (lane = query row, k = keys) from the exchange buffer,
      // B = K (lane = column, k = keys) from the K tile; k-slot (g, j) is key 16 step + 8g + j in both.
#pragma unroll
      for (int u = wave; u < 2 * DT; u += 4) {
        const int sub = u / DT, dt = u % DT;
        f32x16 dq;
#pragma unroll
        for (int r = 0; r < 16; ++r) dq[r] = 0.f;
#pragma unroll
        for (int st = 0; st < C::BN / 16; ++st) {
          const int key = st * 16 + 8 * g + (i16 >> 2);
          const int a_off = sub * C::DSX_STEP + key * 64 + ((c32 >> 4) * 16 + 4 * (i16 & 3)) * 2;
          const v4 a_lo = lds_read_tr8<v4>(dsx, a_off), a_hi = lds_read_tr8<v4>(dsx, a_off + 4 * 64);
          const int chunk = dt * 4 + ((c32 >> 4) << 1) + ((i16 & 3) >> 1);
          const v4 b_lo = lds_read_tr8<v4>(smem, swz_off<D>(key, chunk) + (i16 & 1) * 8);
          const v4 b_hi = lds_read_tr8<v4>(smem, swz_off<D>(key + 4, chunk) + (i16 & 1) * 8);
          dq = F::mfma(join4<v8, v4>(a_lo, a_hi), join4<v8, v4>(b_lo, b_hi), dq);
        }
        // lane = column dt*32 + c32, register r = query row 8 (r/4) + 4g + (r%4): 32 lanes add to 128
        // contiguous bytes of one row of the accumulator
        const int col = dt * 32 + c32;
        if (col < dh) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = m * C::BM + sub * 32 + 8 * (r / 4) + 4 * g + (r % 4);
            if (qi < Nq) unsafeAtomicAdd(acc_head + (size_t)qi * dh + col, dq[r]);
          }
        }
      }
      // no barrier here: the next stage writes the exchange buffer of the other parity, and the one
      // after that is separated from these reads by the barrier that ends the next stage
    }
    __syncthreads();  // all dQ reads of the K tile and the exchange buffer are done

    SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
    store_transposed<T, D, C::OSTR>(dk, scale, ob, dK + head_base(mdk, head, H), k0w, Nk, lane, (size_t)mdk.row, dh);
    store_transposed<T, D, C::OSTR>(dv, 1.0f, ob, dV + head_base(mdv, head, H), k0w, Nk, lane, (size_t)mdv.row, dh);
  }  // rep
}

}  // namespace spark
