// Fused attention forward for gfx950: S = scale*Q K^T, online row softmax, O = P V, LSE saved.
//
// Structure (paper Sec. 3.2): one workgroup owns one tile of 128 query rows of one (batch,
// head) and loops over tiles of 64 keys; per iteration it computes the score tile on the
// matrix cores, updates the running row max / row sum (Sec. 3.2.1, Eq. 3), rescales the O
// accumulator by exp(m_pre - m_cur), and accumulates P V on the matrix cores.  O is written
// once at the end, so HBM sees three reads and one write.
//
// What is specific to CDNA4 here:
//   * Each of the 4 waves owns 32 query rows.  The score tile is computed TRANSPOSED,
//     S^T = K Q^T (keys on the MFMA M axis, queries on the N axis), so a lane owns ONE query
//     column and its 32 accumulator registers are 32 of the tile's 64 keys.  Row max and row
//     sum are then in-lane reductions plus one exchange with the lane 32 positions away
//     (the counterpart of the paper's shuffle step for fp32 accumulators).
//   * O is accumulated transposed as well, O^T = V^T P^T.  The packed accumulator registers
//     of S^T are directly the B operand of that MFMA (see mma_gfx950.hpp), and the V^T
//     operand comes from the row-major V tile in LDS through transposing LDS reads.  P never
//     touches LDS or HBM (the paper's Sec. 3.2.2 layout transform becomes register renaming).
//   * K/V tiles are double-buffered in LDS and arrive there by direct global->LDS loads (no
//     staging registers, no LDS store instructions); tile j+1 is requested before the
//     arithmetic of tile j and awaited before the one barrier that ends the iteration.
//   * The tiles are unpadded and XOR-swizzled (tiles_gfx950.hpp) so that the 16-byte row reads
//     of K and the 4-row transposing reads of V both spread over all banks.
//   * Each 64-key tile runs as two 32-key online-softmax steps whose VALU work is interleaved,
//     in program order, with the MFMAs of the other half (a wave issues in order); LDS operand
//     reads are issued several MFMAs ahead and pinned there with scheduler fences.
//   * Workgroups of 4 waves (128 queries, two per CU) or of 8 waves (256 queries, one per CU):
//     with 8 waves each K/V tile that is brought into LDS serves twice as many MFMAs (measured
//     -4 % at d = 128 on long sequences, +2 % at d = 64); the host picks per problem.  The 8-wave
//     form has the CU's LDS to itself: it holds two stages of two tiles each, requests tiles two
//     at a time and meets at a barrier every second iteration only (PAIR).
//   * Causal: the loop ends at the diagonal, only diagonal tiles are masked, waves skip tiles
//     wholly above their rows, and a workgroup takes the complementary pair of query tiles
//     (nqt-1-p, p) so every workgroup carries the same amount of work.
#pragma once
#include "dropout_gfx950.hpp"
#include "mma_gfx950.hpp"
#include "tiles_gfx950.hpp"

namespace spark {

// PAIR: the K/V buffers hold two stages of TWO 64-key tiles each instead of two single tiles: tiles
// are requested two at a time and the workgroup meets at a barrier every second iteration only.
template <int D, int NW = 4, bool PAIR = false> struct FwdCfg {
  static constexpr int BM = 32 * NW;  // query rows per workgroup (32 per wave)
  static constexpr int BN = 64;   // keys per iteration
  static constexpr int ROWB = D * 2;      // bytes per (swizzled, unpadded) row
  static constexpr int TILE = BN * ROWB;  // one of K, V
  static constexpr int STAGE = 2 * TILE;  // power of two: the buffer is switched by one XOR
  static constexpr int OSTR = D * 2 + 16;  // epilogue staging row stride
  static constexpr int SLOTS = PAIR ? 4 : 2;  // tiles resident or in flight
  static constexpr int SMEM = SLOTS * STAGE > NW * 32 * OSTR ? SLOTS * STAGE : NW * 32 * OSTR;  // tiles / epilogue
  static_assert((STAGE & (STAGE - 1)) == 0, "XOR buffer switch");
};

template <typename T, int D, bool CAUSAL, bool DROP, int NW = 4, bool PAIR = false>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void mha_fwd_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    T* __restrict__ O, float* __restrict__ LSE, TensorMap mq, TensorMap mk, TensorMap mv,
    TensorMap mo, int H, int Nq, int Nk, int dh, int nqt, float scale_log2, Dropout dr) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using v4 = typename F::v4;
  using C = FwdCfg<D, NW, PAIR>;
  constexpr int KS = D / 16;   // k-steps of the score contraction
  constexpr int DT = D / 32;   // 32-row tiles of O^T
  constexpr int CPR = D / 8;   // 16-byte chunks per row

  SPARK_LDS char* const smem = lds_origin();

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31;
  const uint32_t k_row_bytes = (uint32_t)mk.row * 2, v_row_bytes = (uint32_t)mv.row * 2;
  const uint32_t k_lane_src = dma_lane_src<D>(wave & 3, lane, k_row_bytes, dh);
  const uint32_t v_lane_src = dma_lane_src<D>(wave & 3, lane, v_row_bytes, dh);

  // Work items.  Non-causal: one query tile per workgroup.  Causal: a workgroup takes the pair
  // of tiles (nqt-1-p, p), whose loop lengths add up to the same total for every p, so that
  // all workgroups carry equal work and the launch has no tail of long tiles.
  const int items = causal_items<CAUSAL>(nqt);
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / items;
  const int item = logical - head * items;

  // Nq query rows and Nk key rows per head (equal for self-attention; causal needs them equal)
  const T* Qh = Q + head_base(mq, head, H);
  const T* Kh = K + head_base(mk, head, H);
  const T* Vh = V + head_base(mv, head, H);

  for (int rep = 0; rep < (CAUSAL ? 2 : 1); ++rep) {
    const int qt = CAUSAL ? (rep == 0 ? nqt - 1 - item : item) : item;
    if (CAUSAL && rep == 1) {
      if (qt == nqt - 1 - item) break;  // odd tile count: the middle tile has no partner
      __syncthreads();                  // the first tile's epilogue is done with the LDS
    }

    const int q0 = qt * C::BM + wave * 32;  // first query row of this wave
    const int qrow = q0 + c32;              // this lane's query row
    const int qrow_c = qrow < Nq ? qrow : Nq - 1;

    v8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[ks] = load_row_chunk<v8>(Qh + (size_t)qrow_c * (size_t)mq.row, ks * 16 + g * 8, dh);

    int kv_end = Nk;
    if (CAUSAL) {
      const int lim = (qt + 1) * C::BM;
      kv_end = lim < Nk ? lim : Nk;
    }
    const int nt = (kv_end + C::BN - 1) / C::BN;

    // K / V tiles: global -> LDS directly; rows past the end of the sequence arrive as zeros.
    const BufView kview(Kh, head_span_bytes(mk, Nk, dh)), vview(Vh, head_span_bytes(mv, Nk, dh));
    auto fetch_tile = [&](int j, int buf) {  // four waves move a tile
      if (NW > 4 && wave >= 4) return;
      tile_dma<D, C::BN>(kview, j * C::BN, smem + buf * C::STAGE, wave, k_lane_src, k_row_bytes);
      tile_dma<D, C::BN>(vview, j * C::BN, smem + buf * C::STAGE + C::TILE, wave, v_lane_src, v_row_bytes);
    };
    SwzLane<D> off(lane);  // read offsets of the current buffer; switched by one XOR each

    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;
    // reference of the row's exponentials (log2 domain).  Finite, so that a masked score (-inf)
    // minus the reference is -inf and not NaN before the first valid key has set it.
    float m_run = -1e30f;
    float l_run = 0.f;        // running row sum over this lane's keys only (halves merged at the end)

    fetch_tile(0, 0);
    if (PAIR && nt > 1) fetch_tile(1, 1);
    // The Q fragments must have arrived before the loop: otherwise the waits for them would sit
    // inside the loop body.
    wait_vmem_all();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
    __syncthreads();

    // One iteration, compiled twice: MASKED for tiles that the diagonal or the end of the keys
    // crosses, and without any mask arithmetic for all the others (left to a run-time flag, the
    // compiler evaluates the mask predicate for every score of every tile).
    auto iteration = [&](const int j, auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      if (PAIR) {  // at the start of a pair: the next pair, into the slots everybody left before the last barrier
        if ((j & 1) == 0) {
          if (j + 2 < nt) fetch_tile(j + 2, (j + 2) & 3);
          if (j + 3 < nt) fetch_tile(j + 3, (j + 3) & 3);
        }
      } else {
        const int buf = j & 1;
        if (j + 1 < nt) fetch_tile(j + 1, buf ^ 1);  // everybody left that buffer before the last barrier
      }

      const int k0 = j * C::BN;
      // wave-uniform: skip tiles entirely above the diagonal (they are among the masked ones)
      if (!MASKED || !CAUSAL || k0 <= q0 + 31) {
        SPARK_LDS const char* kb = smem;  // + off.* (which carry the buffer bit)
        SPARK_LDS const char* vb = smem + C::TILE;

        // The 64-key tile is processed as two 32-key halves, each its own online-softmax step,
        // so that the VALU work of one half sits between the MFMAs of the other:
        //   S_0                   (MFMA)
        //   S_1       ||  softmax of half 0   (an MFMA, then a few VALU instructions, ...)
        //   O += P_0 V_0  ||  softmax of half 1
        //   O += P_1 V_1
        // A wave issues in order, so the VALU instructions must be placed between the MFMAs in
        // program order; the fences keep the scheduler from regrouping them.  K fragments are read
        // 8 reads ahead, V^T fragments one 16-key step ahead.
        f32x16 s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[mt][r] = 0.f;
        constexpr int GPH = KS / 4;  // groups of 4 k-steps per half
        v8 kf[2][4];
        auto load_kgroup = [&](int gi) {  // gi = half * GPH + group
          const int half = gi / GPH, ks0 = 4 * (gi % GPH);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            kf[gi & 1][e] = lds_read16<v8>(kb, off.row[ks0 + e] + half * 32 * C::ROWB);
        };
        v8 vf[2][DT];
        auto load_vgroup = [&](int kk) {
          const int o = kk * 16 * C::ROWB;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
            vf[kk & 1][dt] = read_tr_pair<T>(vb, off.tr[0][dt] + o, off.tr[1][dt] + o);
        };

        float t[32];
        // raw scores of one half -> t, masked
        auto load_half = [&](int h) {
#pragma unroll
          for (int r = 0; r < 16; ++r) t[h * 16 + r] = s[h][r];
          if (MASKED) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = k0 + h * 32 + 8 * (r / 4) + 4 * g + (r % 4);
              const bool ok = key < Nk && (!CAUSAL || key <= qrow);
              if (!ok) t[h * 16 + r] = -INFINITY;
            }
          }
        };
        // Online softmax (Eq. 3) with a lazy reference point.  P is formed against the current
        // reference m_run straight away, WITHOUT computing the row maximum first; the row sum of the
        // result (needed anyway) tells whether the reference was too low: if no lane's partial sum
        // exceeds 2^8, no P exceeds 2^8 either, which fp32 sums and the 16-bit MFMA operand hold
        // without loss, and the reference stays (the final O = acc / l and LSE = m + log l do not
        // depend on it).  Otherwise (the first tile, and afterwards only when a row's maximum grows
        // by more than ~2^8) the maximum is computed after all, the reference moved there, the
        // accumulators rescaled by exp(m_pre - m_cur) as in Eq. 3, and the half's P formed again.
        // Returns the rescale factor.
        auto renorm = [&](int h) {
          load_half(h);  // raw scores again (they are still in the accumulators)
          float mx = t[h * 16];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(mx, t[h * 16 + r]);
          mx = half_pair_max(mx) * scale_log2;  // scale > 0 commutes with the maximum
          const float m_new = fmaxf(m_run, mx);
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
          m_run = m_new;
          l_run *= alpha;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
          return alpha;
        };
        // Dropout acts on P after the row sums are taken: dropped entries become zero in the
        // operand of O += P V; the survivors' factor 1/(1-p) is applied once, to O, at the end.
        auto drop_half = [&](int h) {
          uint32_t kb[4];
          keep_bytes_query_lane(dr, head, qrow, k0 + 32 * h, lane, kb);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if (!keep_reg(kb, r, dr.thr)) t[h * 16 + r] = 0.f;
            // the select stays on the fp32 value: moved behind the conversion it would split every
            // packed two-value conversion into single ones plus a merge
            asm volatile("" : "+v"(t[h * 16 + r]));
          }
        };
        float rs0 = 0.f, rs1 = 0.f;  // this lane's sums of P over the two halves
        auto exp_elem = [&](int i, float& rs) {
          t[i] = __builtin_amdgcn_exp2f(__builtin_fmaf(t[i], scale_log2, -m_run));
          rs += t[i];
          // materialise here, between the MFMAs around this call: nothing uses the values before the
          // end of the phase, and the compiler otherwise moves the arithmetic there
          asm volatile("" : "+v"(t[i]), "+v"(rs));
        };

        // ---- S_0 ----
        load_kgroup(0);
        load_kgroup(1);
        sched_fence();
#pragma unroll
        for (int gi = 0; gi < GPH; ++gi) {
#pragma unroll
          for (int e = 0; e < 4; ++e) s[0] = F::mfma(kf[gi & 1][e], qf[4 * gi + e], s[0]);
          if (gi + 2 < 2 * GPH) load_kgroup(gi + 2);
          sched_fence();
        }
        load_vgroup(0);
        sched_fence();

        load_half(0);
        // ---- S_1  ||  exponentials of half 0 ----
        constexpr int EPU = 16 / KS;  // elements per MFMA
#pragma unroll
        for (int gi = GPH; gi < 2 * GPH; ++gi) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            s[1] = F::mfma(kf[gi & 1][e], qf[4 * (gi - GPH) + e], s[1]);
#pragma unroll
            for (int x = 0; x < EPU; ++x) exp_elem(((gi - GPH) * 4 + e) * EPU + x, rs0);
            sched_fence();
          }
          if (gi + 2 < 2 * GPH) load_kgroup(gi + 2);
          if (gi == GPH) load_vgroup(1);
          sched_fence();
        }
        if (__any(!(rs0 <= 256.0f))) {  // also true for inf / NaN
          renorm(0);
          rs0 = 0.f;
#pragma unroll
          for (int i = 0; i < 16; ++i) exp_elem(i, rs0);
        }
        load_half(1);
        v8 pf[4];
        if (DROP) drop_half(0);
        pf[0] = pack8<T>(&t[0]);
        pf[1] = pack8<T>(&t[8]);
        sched_fence();
        // ---- O^T += V_0^T P_0^T  ||  exponentials of half 1 ----
        constexpr int EPV = 16 / (2 * DT);  // elements per MFMA
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            o[dt] = F::mfma(vf[kk & 1][dt], pf[kk], o[dt]);
#pragma unroll
            for (int x = 0; x < EPV; ++x) exp_elem(16 + (kk * DT + dt) * EPV + x, rs1);
            sched_fence();
          }
          load_vgroup(kk + 2);
          sched_fence();
        }
        if (__any(!(rs1 <= 256.0f))) {  // P_0 V_0 is in the accumulators already and is rescaled with them
          rs0 *= renorm(1);
          rs1 = 0.f;
#pragma unroll
          for (int i = 16; i < 32; ++i) exp_elem(i, rs1);
        }
        l_run += rs0 + rs1;
        if (DROP) drop_half(1);
        pf[2] = pack8<T>(&t[16]);
        pf[3] = pack8<T>(&t[24]);
        sched_fence();
        // ---- O^T += V_1^T P_1^T ----
#pragma unroll
        for (int kk = 2; kk < 4; ++kk) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) o[dt] = F::mfma(vf[kk & 1][dt], pf[kk], o[dt]);
          sched_fence();
        }
      }

      // next slot: 0 -> 1 -> 2 -> 3 -> 0 with PAIR (XOR with STAGE, then with 3 STAGE), else 0 <-> 1
      const int flip = PAIR && (j & 1) ? 3 * C::STAGE : C::STAGE;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) off.row[ks] ^= flip;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) off.tr[h][dt] ^= flip;
      if (!PAIR || (j & 1) || j + 1 >= nt) {
        wait_vmem_all();  // the next tile (pair) has landed: requested at the top of this iteration (pair)
        __syncthreads();
      }
    };
    // Tiles [0, n_plain) end within the keys and, if causal, at or below the diagonal for every
    // row of this wave.  The split differs between the waves of a workgroup; the number of
    // iterations, and with it the number of barriers, does not.
    int n_plain = Nk / C::BN;
    if (CAUSAL && (q0 + 1) / C::BN < n_plain) n_plain = (q0 + 1) / C::BN;
    if (n_plain > nt) n_plain = nt;
    int j = 0;
    for (; j < n_plain; ++j) iteration(j, std::false_type{});
    for (; j < nt; ++j) iteration(j, std::true_type{});

    // Epilogue: normalise, round once, transpose through this wave's LDS slice, store rows.
    l_run = half_pair_sum(l_run);
    const float inv = (DROP ? dr.rescale : 1.0f) / l_run;
    SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        v4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (T)(o[dt][r4 * 4 + e] * inv);
        lds_write(ob, c32 * C::OSTR + (dt * 32 + 8 * r4 + 4 * g) * 2, pk);
      }
    T* Oh = O + head_base(mo, head, H);
    constexpr int RPP = 64 / CPR;  // rows per pass of the wave
#pragma unroll
    for (int p = 0; p < 32 / RPP; ++p) {
      const int row = p * RPP + lane / CPR, cc = lane % CPR;
      const u32x4 v = lds_read16<u32x4>(ob, row * C::OSTR + cc * 16);
      if (q0 + row < Nq && cc * 8 < dh)
        *reinterpret_cast<u32x4*>(Oh + (size_t)(q0 + row) * (size_t)mo.row + cc * 8) = v;
    }
    if (g == 0 && qrow < Nq)
      LSE[(size_t)head * Nq + qrow] = (m_run + __builtin_amdgcn_logf(l_run)) * 0.6931471805599453f;
  }  // rep
}

}  // namespace spark
