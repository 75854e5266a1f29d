// Attention backward for gfx950 (paper Sec. 3.3, Eq. 4), two kernels on one stream, in this order:
//
//   mha_bwd_dq_kernel        : one workgroup per tile of 128 queries; first forms
//                              D_i = sum_k dO_ik O_ik (the paper's "dPsum") for its rows from the
//                              fragments it loads anyway and writes D and LSE*log2(e) to the
//                              workspace, then loops over key tiles, recomputes P and dS and
//                              accumulates dQ = scale * dS K.
//   mha_bwd_dkdv_pipe_kernel : one workgroup per tile of 128 keys, loops over query tiles,
//                              recomputes P = exp(S - LSE), accumulates dV = P^T dO and
//                              dK = scale * dS^T Q in registers, writes them once (as in
//                              Sec. 3.3, where each thread block owns a slice of dK and dV).
//                              Software-pipelined inside the wave.  Reads D and LSE*log2(e) from
//                              the workspace.
//
// The paper adds every block's dQ contribution into HBM with atomic adds.  Here dQ has its
// own pass with the forward's loop structure instead: it costs two recomputed contractions
// (7 executed for 5 counted) but needs no fp32 dQ buffer to zero and convert, no atomics, and
// gives bitwise reproducible gradients.  Both variants exist and were timed on the same inputs
// (the atomic one is in bwd_atomic_kernels.hpp): with 128 keys per workgroup it adds N/128 fp32
// values per dQ element, 2.2 GB for N = 4096, d = 128, 64 heads, causal; MI355X performs
// device-scope atomics at the memory side, at 1.3 TB/s, so that variant takes 1.76 ms where these
// two kernels take 0.95 ms.
//
// Register layouts follow mma_gfx950.hpp.  In the dK/dV kernels the score tile is computed as
// S = Q K^T (lane = key column, registers = query rows) so that P and dS, packed to 16 bits,
// are directly the B operands of dV^T = dO^T P and dK^T = Q^T dS; the dO^T / Q^T operands
// come from the row-major LDS tiles through transposing reads.  In the dQ kernel everything
// is transposed as in the forward (lane = query column), so LSE_i and D_i are per-lane
// scalars and dS^T is directly the B operand of dQ^T = K^T dS^T.
#pragma once
#include "dropout_gfx950.hpp"
#include "mma_gfx950.hpp"
#include "tiles_gfx950.hpp"

namespace spark {

// ---------------------------------------------------------------------------------------
// dK, dV: software-pipelined.
//
// At d = 128 the accumulators (dK^T, dV^T: 128 registers) and the resident K / V fragments
// (64) leave room for one wave per SIMD only, so nothing but the wave itself can hide its
// softmax arithmetic and LDS latency.  (At d = 64 two workgroups share a CU and the same
// schedule still pays: measured 9 % faster on causal N = 8192 than an unpipelined loop.)  A wave issues in order, and an MFMA occupies the matrix
// core for ~34 cycles while the wave can issue about half a dozen other instructions; so the
// loop is skewed by one 32-query step and written as units of {one MFMA, a few VALU / LDS
// instructions}:
//   region 1:  scores of step i+1 (MFMA)   ||  second half of P, dS of step i      (VALU)
//   region 2:  dV, dK of step i   (MFMA)   ||  first half of P, dS of step i+1     (VALU)
// Because step i+1 may lie in the next 64-query stage, stages live in a ring of three LDS
// slots: stage m+1 is resident while stage m is processed, and stage m+2 is being written by
// direct global->LDS loads (no staging registers, no LDS store instructions).  No step is
// skipped: blocks above the causal diagonal are masked to zero (first two stages of a workgroup
// only); rows past the end of the sequence read as zeros (Q = dO = 0), so they add nothing.
// ---------------------------------------------------------------------------------------
template <int D> struct BwdKvPipeCfg {
  static constexpr int BN = 128, BM = 64, SLOTS = 3;
  static constexpr int ROWB = D * 2;
  static constexpr int TILE = BM * ROWB;
  static constexpr int STAGE = 2 * TILE;
  static constexpr int STAT = 2 * BM * 4;  // LSE*log2(e) and D of the stage's rows
  static constexpr int OSTR = D * 2 + 16;
  static constexpr int STAT0 = SLOTS * STAGE;  // LDS = [slot 0..2 | stat 0..2]
  static constexpr int SMEM = SLOTS * STAGE + SLOTS * STAT;
  static_assert(4 * 32 * OSTR <= SLOTS * STAGE, "epilogue staging must fit");
};

template <typename T, int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, (D == 64 && !DROP) ? 2 : 1) void mha_bwd_dkdv_pipe_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ LSE2, const float* __restrict__ Dws,
    T* __restrict__ dK, T* __restrict__ dV, TensorMap mq, TensorMap mk, TensorMap mv, TensorMap mdo,
    TensorMap mdk, TensorMap mdv, int H, int Nq, int Nk, int dh, int nkt, float scale, Dropout dr) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using C = BwdKvPipeCfg<D>;
  constexpr int KS = D / 16, DT = D / 32;

  SPARK_LDS char* const smem = lds_origin();

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31;

  const int items = causal_items<CAUSAL>(nkt);  // causal: key tiles (p, nkt-1-p) are paired
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / items;
  const int item = logical - head * items;

  const T* Kh = K + head_base(mk, head, H);
  const T* Vh = V + head_base(mv, head, H);
  const BufView qview(Q + head_base(mq, head, H), head_span_bytes(mq, Nq, dh));
  const BufView doview(dO + head_base(mdo, head, H), head_span_bytes(mdo, Nq, dh));
  const uint32_t q_row_bytes = (uint32_t)mq.row * 2, do_row_bytes = (uint32_t)mdo.row * 2;
  const BufView lview(LSE2 + (size_t)head * Nq, (uint32_t)Nq * 4), dview(Dws + (size_t)head * Nq, (uint32_t)Nq * 4);
  const uint32_t q_lane_src = dma_lane_src<D>(wave, lane, q_row_bytes, dh);
  const uint32_t do_lane_src = dma_lane_src<D>(wave, lane, do_row_bytes, dh);
  const float scale_log2 = scale * 1.4426950408889634f;

  for (int rep = 0; rep < (CAUSAL ? 2 : 1); ++rep) {
    const int kt = CAUSAL ? (rep == 0 ? item : nkt - 1 - item) : item;  // the long tile first
    if (CAUSAL && rep == 1) {
      if (kt == item) break;  // odd tile count: the middle tile has no partner
      __syncthreads();        // the first tile's epilogue is done with the LDS
    }
    const int k0w = kt * C::BN + wave * 32;
    const int krow = k0w + c32;
    const int krow_c = krow < Nk ? krow : Nk - 1;

    v8 kf[KS], vf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = load_row_chunk<v8>(Kh + (size_t)krow_c * (size_t)mk.row, ks * 16 + g * 8, dh);
      vf[ks] = load_row_chunk<v8>(Vh + (size_t)krow_c * (size_t)mv.row, ks * 16 + g * 8, dh);
    }

    f32x16 dk[DT], dv[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }

    const int ns = (Nq + C::BM - 1) / C::BM;
    const int s_begin = CAUSAL ? (kt * C::BN) / C::BM : 0;

    const SwzLane<D> lane_off(lane);  // offsets inside slot 0
    const int lane_stat = C::STAT0 + 16 * g;

    // global -> LDS slot, asynchronously (completion is awaited with wait_vmem_all + barrier)
    auto fetch_stage = [&](int m, int slot) {
      SPARK_LDS char* sb = smem + slot * C::STAGE;
      tile_dma<D, C::BM>(qview, m * C::BM, sb, wave, q_lane_src, q_row_bytes);
      tile_dma<D, C::BM>(doview, m * C::BM, sb + C::TILE, wave, do_lane_src, do_row_bytes);
      // 64 floats of LSE*log2(e) (wave 0) and of D (wave 1): 4 bytes per lane
      SPARK_LDS char* st = smem + C::STAT0 + slot * C::STAT;
      if (wave == 0) lview.load4_to_lds(st, lane * 4, (uint32_t)m * C::BM * 4);
      if (wave == 1) dview.load4_to_lds(st + C::BM * 4, lane * 4, (uint32_t)m * C::BM * 4);
    };

    // LDS read offsets of the step whose scores are being formed (row reads, statistics) ...
    int rowA[KS], statA;
    // ... and of the step whose dV / dK are being accumulated (transposing reads)
    int trC[2][DT];
    auto point_A = [&](int slot) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) rowA[ks] = lane_off.row[ks] + slot * C::STAGE;
      statA = lane_stat + slot * C::STAT;
    };
    auto point_C = [&](int slot) {
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) trC[h][dt] = lane_off.tr[h][dt] + slot * C::STAGE;
    };

    v8 fa[2][4];
    auto load_agroup = [&](int gi, int sub) {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        fa[gi & 1][2 * e] = lds_read16<v8>(smem, rowA[2 * gi + e] + sub * 32 * C::ROWB);
        fa[gi & 1][2 * e + 1] = lds_read16<v8>(smem + C::TILE, rowA[2 * gi + e] + sub * 32 * C::ROWB);
      }
    };
    // statistics of 8 of the 16 query rows a lane holds (half = 0: registers 0..7, 1: 8..15) of the
    // step rowA / statA point at
    auto load_stats = [&](f32x4 (&l)[2], f32x4 (&d)[2], int sub, int half) {
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const int o = statA + (sub * 32 + 8 * (2 * half + x)) * 4;
        l[x] = lds_read16<f32x4>(smem, o);
        if (DROP) d[x] = lds_read16<f32x4>(smem, o + C::BM * 4);
      }
    };
    // The workspace holds -D.  Without dropout dS = P o (dP - D) needs no subtraction: the dP
    // accumulator of a step starts from -D of its 16 query rows instead of from zero (the four
    // 16-byte reads below deliver them in exactly the accumulator's row order), so the MFMAs
    // themselves leave dP - D there.  (Under dropout the mask must act on dP alone, so the
    // accumulator starts from zero and -D is added afterwards.)
    auto dp_start = [&](int sub) {
      f32x16 c;
      if (DROP) {
#pragma unroll
        for (int r = 0; r < 16; ++r) c[r] = 0.f;
      } else {
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const f32x4 v = lds_read16<f32x4>(smem, statA + (sub * 32 + 8 * x) * 4 + C::BM * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) c[4 * x + e] = v[e];
        }
      }
      return c;
    };
    constexpr int NG = KS / 2;
    constexpr int NTG = 2 * (DT / 2);
    constexpr int E1 = 8 / (2 * NG);  // softmax elements per pair of score MFMAs in region 1
    v8 ft[2][4];
    // half e of transposed-fragment group tg (one dO^T and one Q^T operand: four reads); issued in
    // halves so that no MFMA slot carries more than a few LDS reads
    auto load_thalf = [&](int tg, int sub, int e) {
      const int kk = tg / (DT / 2), dt0 = 2 * (tg % (DT / 2));
      const int o = sub * 32 * C::ROWB + kk * 16 * C::ROWB;
      ft[tg & 1][2 * e] = read_tr_pair<T>(smem + C::TILE, trC[0][dt0 + e] + o, trC[1][dt0 + e] + o);
      ft[tg & 1][2 * e + 1] = read_tr_pair<T>(smem, trC[0][dt0 + e] + o, trC[1][dt0 + e] + o);
    };

    // One element of P and dS from finished scores: the unit of VALU work that is placed between
    // MFMAs.  r8 = register index within the half (0..7).
    // Under dropout (kb: the step's decision bytes) the dV operand is the dropped P, and
    // dS = r P o (M o dPraw - D (1-p)): the workspace holds D (1-p), r goes into the final scales.
    auto softmax_elem = [&](const f32x16& s, const f32x16& dp, int half, int r8, const f32x4 (&l)[2],
                            const f32x4 (&d)[2], int q0s, bool mask, const uint32_t (&kb)[4], float* p,
                            float* ds, uint32_t (&pk_p)[4], uint32_t (&pk_ds)[4]) {
      const int r = 8 * half + r8;
      float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(s[r], scale_log2, -l[r8 >> 2][r8 & 3]));
      if (mask) pe = krow > q0s + 8 * (r / 4) + 4 * g + (r % 4) ? 0.f : pe;
      if (DROP) {
        const bool keep = keep_reg(kb, r, dr.thr);
        p[r8] = keep ? pe : 0.f;
        asm volatile("" : "+v"(p[r8]));  // keeps the select in front of the packed conversion
        ds[r8] = pe * ((keep ? dp[r] : 0.f) + d[r8 >> 2][r8 & 3]);  // d holds -D (1-p)
      } else {
        p[r8] = pe;
        ds[r8] = pe * dp[r];  // the accumulator started from -D
      }
      // materialise dS here, between the MFMAs around this call: it is not used before the packing
      // at the end of the region, and the compiler would otherwise move its arithmetic there,
      // where no MFMA hides it
      asm volatile("" : "+v"(ds[r8]));
      if (r8 & 1) {  // a pair is complete: convert it now
        pk_p[r8 >> 1] = pack2<T>(p[r8 - 1], p[r8]);
        pk_ds[r8 >> 1] = pack2<T>(ds[r8 - 1], ds[r8]);
      }
    };
    uint32_t kbCur[4] = {0, 0, 0, 0}, kbNew[4] = {0, 0, 0, 0};  // decision bytes of the current / next step

    // ---- prologue: stages s_begin and s_begin+1 resident, scores of the first step formed ----
    fetch_stage(s_begin, 0);
    if (s_begin + 1 < ns) fetch_stage(s_begin + 1, 1);
    wait_vmem_all();
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(kf[ks]), "+v"(vf[ks]));
    __syncthreads();

    point_A(0);
    point_C(0);
    f32x16 sX, dpX, sY, dpY;
    f32x4 lL[2], dL[2], lH[2], dH[2];  // statistics: first half of the next step / second half of the current
#pragma unroll
    for (int r = 0; r < 16; ++r) sX[r] = 0.f;
    dpX = dp_start(0);
    load_agroup(0, 0);
    load_agroup(1, 0);
    load_stats(lL, dL, 0, 0);
#pragma unroll
    for (int gi = 0; gi < NG; ++gi) {
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        sX = F::mfma(fa[gi & 1][2 * e], kf[2 * gi + e], sX);
        dpX = F::mfma(fa[gi & 1][2 * e + 1], vf[2 * gi + e], dpX);
      }
      if (gi + 2 < NG) load_agroup(gi + 2, 0);
      sched_fence();
    }
    // At D = 128 every step requests the first two fragment groups of its successor half-way through
    // its own dV / dK region, so that no step starts by waiting for LDS (C4 backward -3 %); here
    // those of step (s_begin, 1).  At D = 64 the longer live ranges cost spills (+1 ... +3 %) and the
    // request stays at the start of the step that uses it.
    constexpr bool EARLY = D == 128;
    if (EARLY) {
      load_agroup(0, 1);
      load_agroup(1, 1);
    }
    // With more than 256 registers per lane the MFMAs deliver the scores in accumulation registers,
    // which the VALU reaches through one v_accvgpr_read per element.  Such a read co-issues with
    // executing MFMAs as long as none of them writes the register read (measured), so each element
    // is read where its softmax arithmetic sits, between the MFMAs of the following regions; the
    // two score buffers X / Y alternate so that the one being read is never the one being formed.
    // P / dS operands of the current step: registers 0..7 (pfL, dsfL) are formed one region
    // early, registers 8..15 (pfH, dsfH) while the next step's scores are on the matrix cores.
    v8 pfL, dsfL;
    {
      float p[8], ds[8];
      uint32_t pk_p[4], pk_ds[4];
      if (DROP) keep_bytes_key_lane(dr, head, krow, s_begin * C::BM, lane, kbCur);
#pragma unroll
      for (int r = 0; r < 8; ++r)
        softmax_elem(sX, dpX, 0, r, lL, dL, s_begin * C::BM, CAUSAL, kbCur, p, ds, pk_p, pk_ds);
      pfL = join_pairs<T>(pk_p);
      dsfL = join_pairs<T>(pk_ds);
    }
    load_stats(lH, dH, 0, 1);

    // One stage: steps (m, 0) and (m, 1).  On entry sX / dpX hold the scores of (m, 0), pfL / dsfL
    // their first half and lH / dH the statistics of their second half; rowA and trC point at
    // stage m.  On exit the same holds for (m+1, 0).
    auto stage = [&](int m, int slot, bool mask) {
      const int slot1 = slot == 2 ? 0 : slot + 1;
      const int slot2 = slot1 == 2 ? 0 : slot1 + 1;
      // stage m+2 goes into the slot that stage m-1 used; everybody left it before the last barrier
      if (m + 2 < ns) fetch_stage(m + 2, slot2);

      // One step.  cur: scores complete, first half of P / dS packed.  new: the step after it
      // (sub_new inside the stage rowA / statA point at).
      auto step = [&](f32x16& s_new, f32x16& dp_new, int sub_new, int q0_new, const f32x16& s_cur,
                      const f32x16& dp_cur, int sub_cur, int q0_cur, auto&& request_next) {
        // ---- region 1: scores of the next step  ||  second half of P, dS of the current step ----
        float p[8], ds[8];
        uint32_t pk_p[4], pk_ds[4];
        // dropout decisions of the next step: the ten generator rounds ride in the MFMA slots below
        Philox rng;
        if (DROP) rng = keep_key_lane_begin(dr, head, krow, q0_new, lane);
        load_stats(lL, dL, sub_new, 0);
        load_thalf(0, sub_cur, 0);
#pragma unroll
        for (int i = 0; i < 4 * NG; ++i) {
          const int gi = i / 4, e = (i / 2) & 1;
          if ((i & 1) == 0)
            s_new = F::mfma(fa[gi & 1][2 * e], kf[2 * gi + e], s_new);
          else
            dp_new = F::mfma(fa[gi & 1][2 * e + 1], vf[2 * gi + e], dp_new);
          if ((i & 3) == 3 && gi + 2 < NG) load_agroup(gi + 2, sub_new);
          if (i == 1) load_thalf(0, sub_cur, 1);
          if (i == 2 * NG) load_thalf(1, sub_cur, 0);
          if (i == 2 * NG + 1) load_thalf(1, sub_cur, 1);
          if (i & 1) {
#pragma unroll
            for (int x = 0; x < E1; ++x) softmax_elem(s_cur, dp_cur, 1, (i / 2) * E1 + x, lH, dH, q0_cur, mask, kbCur, p, ds, pk_p, pk_ds);
          }
          if (DROP) {
#pragma unroll
            for (int round = i * 10 / (4 * NG); round < (i + 1) * 10 / (4 * NG); ++round)
              philox_round(rng, dr.key0, dr.key1, round);
          }
          sched_fence();
        }
        if (DROP) keep_key_lane_finish(rng, lane, kbNew);
        const v8 pfH = join_pairs<T>(pk_p), dsfH = join_pairs<T>(pk_ds);
        load_stats(lH, dH, sub_new, 1);
        sched_fence();
        sched_fence();
        // ---- region 2: dV, dK of the current step  ||  first half of P, dS of the next step ----
#pragma unroll
        for (int tg = 0; tg < NTG; ++tg) {
          const int kk = tg / (DT / 2), dt0 = 2 * (tg % (DT / 2));
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            dv[dt0 + e] = F::mfma(ft[tg & 1][2 * e], kk ? pfH : pfL, dv[dt0 + e]);
            dk[dt0 + e] = F::mfma(ft[tg & 1][2 * e + 1], kk ? dsfH : dsfL, dk[dt0 + e]);
            softmax_elem(s_new, dp_new, 0, (8 / NTG) * tg + e, lL, dL, q0_new, mask, kbNew, p, ds, pk_p, pk_ds);
            if (8 / NTG > 2)
              softmax_elem(s_new, dp_new, 0, (8 / NTG) * tg + 2 + e, lL, dL, q0_new, mask, kbNew, p, ds, pk_p, pk_ds);
            if (tg + 2 < NTG) load_thalf(tg + 2, sub_cur, e);  // into the operands just used
            sched_fence();
          }
          // the fragment buffers are free since region 1 ended; one group per slot keeps the number
          // of LDS reads in flight under the 15 the wave's counter can track
          if (EARLY && tg == NTG / 2 - 1) request_next(0);
          if (EARLY && tg == NTG / 2) request_next(1);
          sched_fence();
        }
        pfL = join_pairs<T>(pk_p);
        dsfL = join_pairs<T>(pk_ds);
        // materialise here: otherwise this arithmetic sinks to its use in the next step and
        // runs there with no MFMA to hide it
        asm volatile("" : "+v"(pfL), "+v"(dsfL));
        if (DROP) {
#pragma unroll
          for (int a = 0; a < 4; ++a) kbCur[a] = kbNew[a];
        }
      };

      // (m, 1) scores  ||  (m, 0) softmax; then (m, 0) dV / dK
#pragma unroll
      for (int r = 0; r < 16; ++r) sY[r] = 0.f;
      dpY = dp_start(1);  // statA points at stage m here
      auto request_B = [&](int part) {
        if (part != 1) point_A(slot1);  // stage m+1 has been resident since the end of stage m-1
        if (part != 1) load_agroup(0, 0);
        if (part != 0) load_agroup(1, 0);
      };
      auto request_A = [&](int part) {
        if (part != 1) load_agroup(0, 1);
        if (part != 0) load_agroup(1, 1);
      };
      if (!EARLY) request_A(2);
      sched_fence();
      step(sY, dpY, 1, m * C::BM + 32, sX, dpX, 0, m * C::BM, request_B);
      // (m+1, 0) scores  ||  (m, 1) softmax; then (m, 1) dV / dK
#pragma unroll
      for (int r = 0; r < 16; ++r) sX[r] = 0.f;
      if (!EARLY) request_B(2);
      dpX = dp_start(0);  // statA points at stage m + 1 by now (request_B moved it)
      sched_fence();
      step(sX, dpX, 0, (m + 1) * C::BM, sY, dpY, 1, m * C::BM + 32, request_A);

      point_C(slot1);
      wait_vmem_all();  // stage m+2 has landed (it was requested a whole stage ago)
      __syncthreads();
    };

    int m = s_begin, slot = 0;
    if (CAUSAL) {  // the diagonal crosses the first two stages only
      const int m_end = s_begin + 2 < ns ? s_begin + 2 : ns;
      for (; m < m_end; ++m) {
        stage(m, slot, true);
        slot = slot == 2 ? 0 : slot + 1;
      }
    }
    for (; m < ns; ++m) {
      stage(m, slot, false);
      slot = slot == 2 ? 0 : slot + 1;
    }

    SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
    store_transposed<T, D, C::OSTR>(dk, DROP ? scale * dr.rescale : scale, ob, dK + head_base(mdk, head, H), k0w,
                                    Nk, lane, (size_t)mdk.row, dh);
    store_transposed<T, D, C::OSTR>(dv, DROP ? dr.rescale : 1.0f, ob, dV + head_base(mdv, head, H), k0w, Nk,
                                    lane, (size_t)mdv.row, dh);
  }  // rep
}

// ---------------------------------------------------------------------------------------
// dQ
// ---------------------------------------------------------------------------------------
template <int D> struct BwdQCfg {
  static constexpr int BM = 128;  // query rows per workgroup (32 per wave)
  // keys per iteration: 32 at D = 128 keeps the kernel within 256 registers, so that two
  // workgroups share a CU and one hides the other's softmax arithmetic and LDS latency
  static constexpr int BN = D == 128 ? 32 : 64;
  static constexpr int ROWB = D * 2;
  static constexpr int TILE = BN * ROWB;  // one of K, V (swizzled, unpadded)
  static constexpr int STAGE = 2 * TILE;  // power of two: the buffer is switched by one XOR
  static constexpr int OSTR = D * 2 + 16;
  static constexpr int SMEM = 2 * STAGE > 4 * 32 * OSTR ? 2 * STAGE : 4 * 32 * OSTR;  // tiles / epilogue
  static_assert((STAGE & (STAGE - 1)) == 0, "XOR buffer switch");
};

template <typename T, int D, bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void mha_bwd_dq_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ O, const T* __restrict__ dO, const float* __restrict__ LSE,
    float* __restrict__ Dout, float* __restrict__ LSE2out, T* __restrict__ dQ, TensorMap mq, TensorMap mk,
    TensorMap mv, TensorMap mo, TensorMap mdo, TensorMap mdq, int H, int Nq, int Nk, int dh, int nqt, float scale,
    float scale_log2, Dropout dr) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  using C = BwdQCfg<D>;
  constexpr int KS = D / 16, DT = D / 32;

  SPARK_LDS char* const smem = lds_origin();

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int g = lane >> 5, c32 = lane & 31;

  const int items = causal_items<CAUSAL>(nqt);  // causal: query tiles (nqt-1-p, p) are paired
  const int logical = xcd_contiguous(blockIdx.x, gridDim.x);
  const int head = logical / items;
  const int item = logical - head * items;

  const T* Qh = Q + head_base(mq, head, H);
  const T* dOh = dO + head_base(mdo, head, H);
  const T* Oh = O + head_base(mo, head, H);
  const BufView kview(K + head_base(mk, head, H), head_span_bytes(mk, Nk, dh));
  const BufView vview(V + head_base(mv, head, H), head_span_bytes(mv, Nk, dh));
  const uint32_t k_row_bytes = (uint32_t)mk.row * 2, v_row_bytes = (uint32_t)mv.row * 2;
  const uint32_t k_lane_src = dma_lane_src<D>(wave, lane, k_row_bytes, dh);
  const uint32_t v_lane_src = dma_lane_src<D>(wave, lane, v_row_bytes, dh);
  // K / V tiles go global -> LDS directly (no staging registers, no LDS store instructions);
  // completion is awaited with wait_vmem_all + barrier at the end of the iteration before use.
  auto fetch_tile = [&](int j, int buf) {
    tile_dma<D, C::BN>(kview, j * C::BN, smem + buf * C::STAGE, wave, k_lane_src, k_row_bytes);
    tile_dma<D, C::BN>(vview, j * C::BN, smem + buf * C::STAGE + C::TILE, wave, v_lane_src, v_row_bytes);
  };

  for (int rep = 0; rep < (CAUSAL ? 2 : 1); ++rep) {
    const int qt = CAUSAL ? (rep == 0 ? nqt - 1 - item : item) : item;  // the long tile first
    if (CAUSAL && rep == 1) {
      if (qt == nqt - 1 - item) break;  // odd tile count: the middle tile has no partner
      __syncthreads();                  // the first tile's epilogue is done with the LDS
    }
    const int q0 = qt * C::BM + wave * 32;
    const int qrow = q0 + c32;
    const int qrow_c = qrow < Nq ? qrow : Nq - 1;

    v8 qf[KS], dof[KS], of[KS];  // of: the row of O, needed for D only
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = load_row_chunk<v8>(Qh + (size_t)qrow_c * (size_t)mq.row, ks * 16 + g * 8, dh);
      dof[ks] = load_row_chunk<v8>(dOh + (size_t)qrow_c * (size_t)mdo.row, ks * 16 + g * 8, dh);
      of[ks] = load_row_chunk<v8>(Oh + (size_t)qrow_c * (size_t)mo.row, ks * 16 + g * 8, dh);
    }
    float lse2 = LSE[(size_t)head * Nq + qrow_c];

    int kv_end = Nk;
    if (CAUSAL) {
      const int lim = (qt + 1) * C::BM;
      kv_end = lim < Nk ? lim : Nk;
    }
    const int nt = (kv_end + C::BN - 1) / C::BN;

    SwzLane<D> off(lane);  // read offsets of the current buffer; switched by one XOR each

    f32x16 dq[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;

    fetch_tile(0, 0);
    wait_vmem_all();  // Q / dO / O fragments and LSE are in registers before the loop
    // D_i = sum_k dO_ik O_ik (the paper's "dPsum"): a lane holds half of its query's row, the lane
    // 32 further on the other half.  Under dropout dS = r P o (M o dPraw - D (1-p)), so D is kept
    // multiplied by the keep probability.  The dK/dV kernel runs after this one and reads D and
    // LSE * log2(e) from the workspace.
    float Dq = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int i = 0; i < 8; ++i) Dq = __builtin_fmaf((float)of[ks][i], (float)dof[ks][i], Dq);
    Dq = half_pair_sum(Dq) * (DROP ? dr.keep_prob : 1.0f);
    lse2 *= 1.4426950408889634f;
    if (g == 0 && qrow < Nq) {
      Dout[(size_t)head * Nq + qrow] = -Dq;  // negated: the dK/dV kernel starts its dP accumulators from it
      LSE2out[(size_t)head * Nq + qrow] = lse2;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]), "+v"(dof[ks]));
    asm volatile("" : "+v"(lse2), "+v"(Dq));
    // Without dropout dS = P o (dP - D) needs no subtraction: every dP accumulator starts from -D
    // (one value per lane here: lane = query), handed to the first MFMA as its addend.  That costs 16
    // registers for the whole loop; at D = 128 the kernel has none to spare (the causal one would
    // spill, measured +4 %), so only D = 64 does it (dQ kernel -2 ... -3 %).
    constexpr bool FOLD_D = !DROP && D == 64;
    f32x16 dneg;
#pragma unroll
    for (int r = 0; r < 16; ++r) dneg[r] = -Dq;
    if (FOLD_D) asm volatile("" : "+v"(dneg));
    __syncthreads();

    // One iteration, compiled twice: MASKED for tiles that the diagonal or the end of the keys
    // crosses, and without any mask arithmetic for all the others.
    auto iteration = [&](const int j, auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
      const int buf = j & 1;
      if (j + 1 < nt) fetch_tile(j + 1, buf ^ 1);  // everybody left that buffer before the last barrier
      const int k0 = j * C::BN;
      // wave-uniform: skip tiles entirely above the diagonal (they are among the masked ones)
      if (!MASKED || !CAUSAL || k0 <= q0 + 31) {
        SPARK_LDS const char* kb = smem;  // + off.* (which carry the buffer bit)
        SPARK_LDS const char* vb = smem + C::TILE;

        // S^T = K Q^T first, then dP^T = V dO^T (lane = query column, registers = keys), so that
        // P = exp2(S c - LSE) can be formed under the MFMAs of dP, and the second half of dS under
        // the first MFMAs of dQ.  A wave issues in order: what overlaps is decided by program
        // order, so the arithmetic is placed between the MFMAs by hand, pinned by empty asm
        // statements (the compiler would move it to its first use) and scheduling fences.
        // Row fragments (step i < KS: K at k-step i; step i >= KS: V at k-step i - KS) are read
        // four steps ahead of their MFMAs.
        constexpr int MT = C::BN / 32;  // 32-key blocks per tile
        f32x16 s[MT], dp[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
          for (int r = 0; r < 16; ++r) { s[mt][r] = 0.f; dp[mt][r] = 0.f; }
          if (FOLD_D) dp[mt] = dneg;
        }
        constexpr int AHEAD = 4;
        v8 fa[AHEAD][MT];
        auto load_step = [&](int i) {
          const int ks = i < KS ? i : i - KS;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            fa[i % AHEAD][mt] = lds_read16<v8>(i < KS ? kb : vb, off.row[ks] + mt * 32 * C::ROWB);
        };
        // Dropout: dS = r P o (M o dPraw - D (1-p)); the workspace holds D (1-p) and the factor r
        // goes into the final scale of dQ.
        uint32_t keep[MT][4];
        if (DROP) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) keep_bytes_query_lane(dr, head, qrow, k0 + 32 * mt, lane, keep[mt]);
        }
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) load_step(i);
        sched_fence();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) s[mt] = F::mfma(fa[ks % AHEAD][mt], qf[ks], s[mt]);
          load_step(ks + AHEAD);  // KS >= AHEAD: always a valid step
          sched_fence();
        }

        float pe[16 * MT];
        auto p_elem = [&](int e) {  // e = mt * 16 + r
          const int mt = e / 16, r = e % 16;
          float x = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mt][r], scale_log2, -lse2));
          if (MASKED) {
            const int key = k0 + mt * 32 + 8 * (r / 4) + 4 * g + (r % 4);
            const bool ok = key < Nk && (!CAUSAL || key <= qrow);
            if (!ok) x = 0.f;
          }
          pe[e] = x;
          asm volatile("" : "+v"(pe[e]));
        };
        // K^T fragments, one group per 16-key step of dQ; the first two groups are requested in
        // the second half of the dP phase, when the row fragments have all been requested (one
        // burst of all of them would exceed the 15 LDS reads a wave can have in flight)
        constexpr int NKK = C::BN / 16;
        v8 ft[2][DT];
        auto load_tgroup = [&](int kk) {
          const int o = kk * 16 * C::ROWB;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
            ft[kk & 1][dt] = read_tr_pair<T>(kb, off.tr[0][dt] + o, off.tr[1][dt] + o);
        };
        constexpr int EPM = 16 / KS;  // P elements per MFMA of dP
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            dp[mt] = F::mfma(fa[(KS + ks) % AHEAD][mt], dof[ks], dp[mt]);
#pragma unroll
            for (int x = 0; x < EPM; ++x) p_elem(mt * 16 + ks * EPM + x);
            sched_fence();
          }
          if (KS + ks + AHEAD < 2 * KS) load_step(KS + ks + AHEAD);
          if (ks == KS - AHEAD) load_tgroup(0);
          if (ks == KS - AHEAD / 2) load_tgroup(1);
          sched_fence();
        }

        float ds[16 * MT];
        auto ds_elem = [&](int e) {
          const int mt = e / 16, r = e % 16;
          if (FOLD_D) {
            ds[e] = pe[e] * dp[mt][r];  // the accumulator started from -D
          } else {
            const float dpe = DROP && !keep_reg(keep[mt], r, dr.thr) ? 0.f : dp[mt][r];
            ds[e] = pe[e] * (dpe - Dq);
          }
          asm volatile("" : "+v"(ds[e]));
        };
        // dQ^T += K^T dS^T, 16 keys per step; step kk uses elements 8 kk .. 8 kk + 7.  Those of
        // step 0 are formed up front, those of step kk + 1 under the MFMAs of step kk.
        v8 dsf[NKK];
#pragma unroll
        for (int x = 0; x < 8; ++x) ds_elem(x);
        dsf[0] = pack8<T>(&ds[0]);
        sched_fence();
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) {
            dq[dt] = F::mfma(ft[kk & 1][dt], dsf[kk], dq[dt]);
            if (kk + 1 < NKK) {
#pragma unroll
              for (int x = 0; x < 8 / DT; ++x) ds_elem(8 * (kk + 1) + dt * (8 / DT) + x);
            }
            sched_fence();
          }
          if (kk + 1 < NKK) {
            dsf[kk + 1] = pack8<T>(&ds[8 * (kk + 1)]);
            asm volatile("" : "+v"(dsf[kk + 1]));
          }
          if (kk + 2 < NKK) load_tgroup(kk + 2);
          sched_fence();
        }
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) off.row[ks] ^= C::STAGE;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) off.tr[h][dt] ^= C::STAGE;
      wait_vmem_all();  // the next tile has landed (requested at the top of the iteration)
      __syncthreads();
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

    SPARK_LDS char* ob = smem + wave * 32 * C::OSTR;
    store_transposed<T, D, C::OSTR>(dq, DROP ? scale * dr.rescale : scale, ob, dQ + head_base(mdq, head, H), q0,
                                    Nq, lane, (size_t)mdq.row, dh);
  }  // rep
}

}  // namespace spark
