// Self-check of the register layouts every kernel here is written against (mma_gfx950.hpp):
// the operand and accumulator layout of the 32x32x16 MFMA, the reuse of packed accumulator
// registers as the operand of a second MFMA (the register-renaming form of the paper's
// Sec. 3.2.2 layout transform), and what a transposing LDS read delivers.  One wave computes
// small integer matrix products THROUGH those layouts and writes the results as plain row-major
// matrices, which a test compares with the same products computed on the host: a layout that
// differs from the documented one gives a different matrix.
#pragma once
#include "mma_gfx950.hpp"

namespace spark {

// Test patterns: small integers, exact in fp16 and bf16 (also after one 32-term product sum).
static __host__ __device__ __forceinline__ int probe_a1(int i, int k) { return (i * 37 + k * 11 + (i * k) % 7) % 3 - 1; }
static __host__ __device__ __forceinline__ int probe_b1(int k, int j) { return (k * 29 + j * 13 + (k * j) % 5) % 5 - 2; }
static __host__ __device__ __forceinline__ int probe_a2(int m, int r) { return (m * 17 + r * 7 + (m * r) % 11) % 7 - 3; }

// out[0 .. 1023]    C1 = A1 B1, 32 x 32 row-major; A1 is 32 x 16, B1 is 16 x 32
// out[1024 .. 2047] C2 = A2 C1, 32 x 32 row-major; A2 is 32 x 32.  C1 is never rearranged: its
//                   accumulator registers 8h .. 8h+7, packed to 16 bits, are used as the B operand
//                   of MFMA h, and A2 is gathered in the matching row order krow(h, g, j).
// out[2048 .. 2303] transposing LDS read of a 16-row x 64-column tile of 16-bit words holding
//                   X[r][c] = 64 r + c: lane l addresses X[4 (l/16) .. ][..] as documented and
//                   writes the four words it receives to out[2048 + 4 l .. + 3] (as numbers).
template <typename T>
__global__ __launch_bounds__(64) void layout_probe_kernel(float* __restrict__ out) {
  using F = Frag<T>;
  using v8 = typename F::v8;
  extern __shared__ __attribute__((aligned(16))) char probe_smem[];
  SPARK_LDS char* const smem = lds_origin();
  const int lane = threadIdx.x, g = lane >> 5, c32 = lane & 31;

  // A: lane holds row l % 32, k-slots 8g .. 8g+7.  B: lane holds column l % 32, same k-slots.
  v8 a1, b1;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    a1[j] = (T)(float)probe_a1(c32, 8 * g + j);
    b1[j] = (T)(float)probe_b1(8 * g + j, c32);
  }
  f32x16 c1;
#pragma unroll
  for (int r = 0; r < 16; ++r) c1[r] = 0.f;
  c1 = F::mfma(a1, b1, c1);
  // C: lane holds column l % 32; register r holds row 8 (r/4) + 4g + (r%4)
#pragma unroll
  for (int r = 0; r < 16; ++r) out[(8 * (r / 4) + 4 * g + (r % 4)) * 32 + c32] = c1[r];

  f32x16 c2;
#pragma unroll
  for (int r = 0; r < 16; ++r) c2[r] = 0.f;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float half[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) half[j] = c1[8 * h + j];
    const v8 b2 = pack8<T>(half);
    v8 a2;
#pragma unroll
    for (int j = 0; j < 8; ++j) a2[j] = (T)(float)probe_a2(c32, 16 * h + 8 * (j / 4) + 4 * g + (j % 4));
    c2 = F::mfma(a2, b2, c2);
  }
#pragma unroll
  for (int r = 0; r < 16; ++r) out[1024 + (8 * (r / 4) + 4 * g + (r % 4)) * 32 + c32] = c2[r];

  // transposing read: tile of 16 rows x 64 columns of 16-bit words, row-major, 128 bytes per row
  for (int i = lane; i < 16 * 64; i += 64) lds_write<uint16_t>(smem, i * 2, (uint16_t)i);
  __syncthreads();
  // group of 16 lanes q = l / 16 reads rows 4q .. 4q+3 at columns 16 .. 31: lane j of the group
  // addresses X[4q + j/4][16 + 4 (j%4)]; lane i of the group then holds X[4q + t][16 + i], t = 0..3
  const int q = lane >> 4, j16 = lane & 15;
  const i16x4 w = lds_read_tr8<i16x4>(smem, ((4 * q + (j16 >> 2)) * 64 + 16 + 4 * (j16 & 3)) * 2);
#pragma unroll
  for (int t = 0; t < 4; ++t) out[2048 + 4 * lane + t] = (float)(uint16_t)w[t];
}

}  // namespace spark
