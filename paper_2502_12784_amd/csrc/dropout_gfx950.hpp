// Attention dropout for the fused kernels on gfx950: the keep/drop decisions are regenerated
// inside every kernel from a counter-based generator, so the forward and the two backward
// kernels see the same mask without storing it (paper Sec. 4.2: the backward repeats the
// forward's dropout; Sec. 4.1: rate 0.1 in every measurement).
//
// Definition of the mask (the library's own; the paper does not give one).  The decision for
// entry (head h, query i, key j) is one byte of the output of Philox4x32 with 10 rounds
// (Salmon, Moraes, Dror, Shaw, SC'11):
//   x = Philox(counter = (j / 4, i / 4, h, offset), key = (seed low word, seed high word))
//   u = byte (j mod 4) of x[i mod 4];   keep iff u >= thr;   survivors scaled by 256 / (256 - thr)
// One call therefore covers a block of 4 queries x 4 keys.  In the MFMA accumulator layout a
// lane holds, per 32 x 32 block, four strips of four consecutive rows of one column: four 1 x 4
// (or 4 x 1) pieces of four different calls.  The four lanes of a quad hold the complementary
// pieces of the same four calls, so each lane evaluates one call and the quad exchanges the
// words with DPP quad broadcasts: one generator call per 16 entries, none wasted.
#pragma once
#include <stdint.h>

namespace spark {

struct Dropout {
  uint32_t key0, key1;  // seed, low and high word
  uint32_t offset;      // counter word 3: distinguishes calls that share a seed
  uint32_t thr;         // drop iff byte < thr (0..255)
  float keep_prob;      // (256 - thr) / 256
  float rescale;        // 256 / (256 - thr)
};

// Philox4x32-10, one round at a time so that a kernel can place the rounds between its MFMAs.
// The key schedule (key + round * Weyl constant) is uniform across the wave: scalar registers.
struct Philox {
  uint32_t c0, c1, c2, c3;
};
static __device__ __forceinline__ void philox_round(Philox& s, uint32_t key0, uint32_t key1, int round) {
  const uint32_t k0 = key0 + (uint32_t)round * 0x9E3779B9u, k1 = key1 + (uint32_t)round * 0xBB67AE85u;
  const uint64_t p0 = (uint64_t)0xD2511F53u * s.c0;
  const uint64_t p1 = (uint64_t)0xCD9E8D57u * s.c2;
  const uint32_t n0 = (uint32_t)(p1 >> 32) ^ s.c1 ^ k0;
  const uint32_t n2 = (uint32_t)(p0 >> 32) ^ s.c3 ^ k1;
  s.c1 = (uint32_t)p1;
  s.c3 = (uint32_t)p0;
  s.c0 = n0;
  s.c2 = n2;
}
static __device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                     uint32_t k0, uint32_t k1, uint32_t (&out)[4]) {
  Philox s{c0, c1, c2, c3};
#pragma unroll
  for (int round = 0; round < 10; ++round) philox_round(s, k0, k1, round);
  out[0] = s.c0; out[1] = s.c1; out[2] = s.c2; out[3] = s.c3;
}

// value of `v` in lane A of this lane's quad (all four lanes must be active)
template <int A>
static __device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, A * 0x55, 0xF, 0xF, true);
}

// 4 x 4 transpose inside every quad: on return x[a] holds what lane a of the quad had in x[w],
// w = this lane's position in the quad.  Two butterfly steps (partner lane w^1, then w^2), each
// exchanging the two words that differ in that bit: 4 DPP moves and 12 selects.
static __device__ __forceinline__ void quad_transpose(uint32_t (&x)[4], int w) {
  const bool odd = w & 1, upper = w & 2;
#pragma unroll
  for (int k = 0; k < 4; k += 2) {  // words k, k+1 <-> lane bit 0
    const uint32_t send = odd ? x[k] : x[k + 1];
    const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)send, 0xB1, 0xF, 0xF, true);  // quad_perm [1,0,3,2]
    x[k] = odd ? recv : x[k];
    x[k + 1] = odd ? x[k + 1] : recv;
  }
#pragma unroll
  for (int k = 0; k < 2; ++k) {  // words k, k+2 <-> lane bit 1
    const uint32_t send = upper ? x[k] : x[k + 2];
    const uint32_t recv = (uint32_t)__builtin_amdgcn_mov_dpp((int)send, 0x4E, 0xF, 0xF, true);  // quad_perm [2,3,0,1]
    x[k] = upper ? recv : x[k];
    x[k + 2] = upper ? x[k + 2] : recv;
  }
}

// Lane = query column (S^T layouts of the forward and dQ kernels).  The lane's query is
// `qrow` (qrow mod 4 == lane mod 4) and it holds keys kblk + 8a + 4g + b of the 32-key block
// starting at kblk (a multiple of 32), g = lane / 32.  kb[a] receives the four decision bytes of
// strip a: byte b belongs to accumulator register 4a + b.
static __device__ __forceinline__ void keep_bytes_query_lane(const Dropout& dr, int head, int qrow,
                                                             int kblk, int lane, uint32_t (&kb)[4]) {
  const int w = lane & 3, g = lane >> 5;
  uint32_t x[4];
  philox4x32_10((uint32_t)((kblk >> 2) + 2 * w + g), (uint32_t)(qrow >> 2), (uint32_t)head, dr.offset,
                dr.key0, dr.key1, x);  // this lane evaluates the call of strip a = w
  // strip a needs word (query mod 4) = w of the call that lane a of the quad evaluated
  quad_transpose(x, w);
#pragma unroll
  for (int a = 0; a < 4; ++a) kb[a] = x[a];
}

// Lane = key column (S layouts of the dK/dV kernel).  The lane's key is `krow`
// (krow mod 4 == lane mod 4) and it holds queries qblk + 8a + 4g + b of the 32-query block
// starting at qblk (a multiple of 32).  kb[a] as above: byte b belongs to register 4a + b.
// In three parts (counter, ten rounds of philox_round, exchange) so that the kernel can spread
// the rounds over its MFMA slots; keep_bytes_key_lane runs them back to back.
static __device__ __forceinline__ Philox keep_key_lane_begin(const Dropout& dr, int head, int krow, int qblk,
                                                             int lane) {
  const int w = lane & 3, g = lane >> 5;  // this lane evaluates the call of strip a = w
  return Philox{(uint32_t)(krow >> 2), (uint32_t)((qblk >> 2) + 2 * w + g), (uint32_t)head, dr.offset};
}
static __device__ __forceinline__ void keep_key_lane_finish(const Philox& s, int lane, uint32_t (&kb)[4]);
static __device__ __forceinline__ void keep_bytes_key_lane(const Dropout& dr, int head, int krow,
                                                           int qblk, int lane, uint32_t (&kb)[4]) {
  Philox s = keep_key_lane_begin(dr, head, krow, qblk, lane);
#pragma unroll
  for (int round = 0; round < 10; ++round) philox_round(s, dr.key0, dr.key1, round);
  keep_key_lane_finish(s, lane, kb);
}
static __device__ __forceinline__ void keep_key_lane_finish(const Philox& s, int lane, uint32_t (&kb)[4]) {
  const int w = lane & 3;
  const uint32_t x[4] = {s.c0, s.c1, s.c2, s.c3};
  // byte (key mod 4) of each of the four words (queries) of a call, gathered into one word
  const uint32_t sel_lo = 0x0c0c0400u + 0x0101u * (uint32_t)w;  // v_perm: bytes {w of S1, w of S0, 0, 0}
  auto own_col = [&](uint32_t x0, uint32_t x1, uint32_t x2, uint32_t x3) {
    const uint32_t lo = __builtin_amdgcn_perm(x1, x0, sel_lo);  // byte0 = x0[w], byte1 = x1[w]
    const uint32_t hi = __builtin_amdgcn_perm(x3, x2, sel_lo);  // byte0 = x2[w], byte1 = x3[w]
    return lo | (hi << 16);
  };
  kb[0] = own_col(quad_bcast<0>(x[0]), quad_bcast<0>(x[1]), quad_bcast<0>(x[2]), quad_bcast<0>(x[3]));
  kb[1] = own_col(quad_bcast<1>(x[0]), quad_bcast<1>(x[1]), quad_bcast<1>(x[2]), quad_bcast<1>(x[3]));
  kb[2] = own_col(quad_bcast<2>(x[0]), quad_bcast<2>(x[1]), quad_bcast<2>(x[2]), quad_bcast<2>(x[3]));
  kb[3] = own_col(quad_bcast<3>(x[0]), quad_bcast<3>(x[1]), quad_bcast<3>(x[2]), quad_bcast<3>(x[3]));
}

// decision for accumulator register r (0..15) from the bytes of its strip
static __device__ __forceinline__ bool keep_reg(const uint32_t (&kb)[4], int r, uint32_t thr) {
  return ((kb[r >> 2] >> (8 * (r & 3))) & 0xFFu) >= thr;
}

// The keep mask itself, one byte per entry (1 = keep), [B*H][Nq][Nk]: one thread per 4 x 4 block.
__global__ void dropout_mask_kernel(unsigned char* __restrict__ M, int Nq, int Nk, int qblocks,
                                    int kblocks, long long total_blocks, Dropout dr) {
  const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= total_blocks) return;
  const int jb = (int)(t % kblocks);
  const long long rest = t / kblocks;
  const int ib = (int)(rest % qblocks);
  const int h = (int)(rest / qblocks);
  uint32_t x[4];
  philox4x32_10((uint32_t)jb, (uint32_t)ib, (uint32_t)h, dr.offset, dr.key0, dr.key1, x);
  for (int r = 0; r < 4; ++r) {
    const int i = 4 * ib + r;
    if (i >= Nq) break;
    for (int c = 0; c < 4; ++c) {
      const int j = 4 * jb + c;
      if (j >= Nk) break;
      M[((size_t)h * Nq + i) * Nk + j] = ((x[r] >> (8 * c)) & 0xFFu) >= dr.thr ? 1 : 0;
    }
  }
}

}  // namespace spark
