// Wave64 MFMA fragments and LDS helpers for gfx950 (CDNA4).
//
// Operand layout of v_mfma_f32_32x32x16_{f16,bf16}, C[32x32] += A[32x16] * B[16x32], for lane
// l (0..63) with g = l / 32:
//   A : lane holds row    l % 32, k-slots 8g .. 8g+7   (8 x 16-bit, 4 VGPRs)
//   B : lane holds column l % 32, k-slots 8g .. 8g+7
//   C : lane holds column l % 32; register r (0..15) holds row 8*(r/4) + 4g + (r%4)
// A contraction is invariant under one permutation applied to the k-slots of both operands.
// The kernels use this: registers 8h..8h+7 (h = 0, 1) of a C tile, packed to 16 bits, are
// directly a B (or A) operand whose k-slot (g, j) means row
//     krow(h, g, j) = 16h + 8*(j/4) + 4g + (j%4)
// of that tile, provided the other operand is gathered with the same row order.  This is the
// CDNA4 counterpart of the paper's warp-level C->A layout transform (Sec. 3.2.2): the
// probabilities never leave registers between the two contractions.
//
// ds_read_b64_tr_b16 (transposing LDS read): within each group of 16 lanes, lane i receives
// element (i % 4) of the 4 x 16-bit words addressed by lanes 4t + i/4, t = 0..3.  For a
// row-major tile X[row][col], lane j of the group addressing X[r0 + j/4][c0 + 4*(j%4)] makes
// lane i receive X[r0 + t][c0 + i], t = 0..3: a column of four consecutive rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace spark {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define SPARK_LDS __attribute__((address_space(3)))

template <typename T> struct Frag;

template <> struct Frag<_Float16> {
  typedef f16x8 v8;
  typedef f16x4 v4;
  static __device__ __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

template <> struct Frag<__bf16> {
  typedef bf16x8 v8;
  typedef bf16x4 v4;
  static __device__ __forceinline__ f32x16 mfma(v8 a, v8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};

// Start of the workgroup's LDS as a compile-time constant.  These kernels use dynamically sized LDS
// only, so their segment starts at LDS address 0 (the host refuses to launch a kernel whose code
// object reports static LDS).  With a symbolic origin the compiler adds the origin to every read
// address in the loops (one VALU instruction per LDS read); with a constant one the tile, sub-tile
// and k-step displacements all go into the immediate field of the DS instruction.
static __device__ __forceinline__ SPARK_LDS char* lds_origin() {
  return reinterpret_cast<SPARK_LDS char*>(0u);
}

// 16-byte LDS read / typed LDS write at a byte offset from the start of the workgroup's LDS.
template <typename V8>
static __device__ __forceinline__ V8 lds_read16(SPARK_LDS const char* smem, int byte_off) {
  return *reinterpret_cast<SPARK_LDS const V8*>(smem + byte_off);
}

template <typename V>
static __device__ __forceinline__ void lds_write(SPARK_LDS char* smem, int byte_off, V v) {
  *reinterpret_cast<SPARK_LDS V*>(smem + byte_off) = v;
}

// Transposing 8-byte LDS read (see the header comment); returns 4 x 16-bit.
template <typename V4>
static __device__ __forceinline__ V4 lds_read_tr8(SPARK_LDS const char* smem, int byte_off) {
  i16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((SPARK_LDS i16x4*)(smem + byte_off));
  return __builtin_bit_cast(V4, v);
}

template <typename V8, typename V4>
static __device__ __forceinline__ V8 join4(V4 lo, V4 hi) {
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Pack 8 fp32 values to 16-bit (round to nearest even) as one MFMA operand.
template <typename T>
static __device__ __forceinline__ typename Frag<T>::v8 pack8(const float* x) {
  typename Frag<T>::v8 r;
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = (T)x[i];
  return r;
}

// Two fp32 values to one register of two 16-bit values (one packed conversion), and four such
// registers as one MFMA operand: for kernels that convert each pair as soon as it exists, between
// MFMAs, instead of all eight values at the end of a phase.
template <typename T>
static __device__ __forceinline__ uint32_t pack2(float a, float b) {
  typedef T v2 __attribute__((ext_vector_type(2)));
  v2 r;
  r[0] = (T)a;
  r[1] = (T)b;
  uint32_t u = __builtin_bit_cast(uint32_t, r);
  asm volatile("" : "+v"(u));
  return u;
}
template <typename T>
static __device__ __forceinline__ typename Frag<T>::v8 join_pairs(const uint32_t (&u)[4]) {
  const u32x4 v = {u[0], u[1], u[2], u[3]};
  return __builtin_bit_cast(typename Frag<T>::v8, v);
}

// Reductions over the two lanes l and l^32 (the two halves of a wave), result in both lanes.
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of its
// second; called with (x, x) it returns {x of the lower-half lane, x of the upper-half lane} in
// both lanes, without going through LDS.
static __device__ __forceinline__ float half_pair_max(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (uint32_t)r[0]), __builtin_bit_cast(float, (uint32_t)r[1]));
}
static __device__ __forceinline__ float half_pair_sum(float x) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// Raw buffer view of one row-major [rows][D] 16-bit matrix.  Loads whose 16 bytes do not lie
// inside the matrix return zeros instead of faulting, so ragged tiles need no address clamps,
// and the per-tile part of the address is a scalar offset (no vector address arithmetic in the
// main loops).  The matrix must be smaller than 4 GiB.
struct BufView {
  u32x4 desc;  // buffer descriptor: base, base_hi | stride 0, bytes, flags
  __device__ __forceinline__ BufView(const void* base, uint32_t bytes) {
    const uint64_t a = reinterpret_cast<uint64_t>(base);
    desc[0] = (uint32_t)a;
    desc[1] = (uint32_t)(a >> 32) & 0xffffu;
    desc[2] = bytes;
    desc[3] = 0x00020000u;
  }
  // Direct global->LDS load (no registers): lane l of the wave writes its 16 (or 4) bytes at
  // LDS byte address dst + 16 l (4 l); dst must be wave-uniform.  Out-of-range lanes write
  // zeros.  Completion is counted by vmcnt.
  //
  // Issued as inline assembly on purpose: for the builtin form the compiler cannot tell which
  // LDS bytes the load writes and puts a full vmcnt(0) wait in front of every later LDS read,
  // which would expose the whole global-memory latency.  The caller therefore owns the
  // synchronisation: wait_vmem_all() followed by a workgroup barrier before anyone reads the
  // destination.  (The compiler's own vmcnt waits stay correct: loads return in order, so
  // extra outstanding loads can only make such a wait longer, never shorter.)  The LDS
  // destination travels in M0; it is handed over as an input operand bound to that register, so
  // the compiler writes M0 itself and knows its value is consumed here: any use of M0 of its
  // own (another LDS-DMA, GWS or relative-index instruction) is ordered around it correctly.
  //
  // The s_nop in front of the load is a hazard guard, not padding.  The hardware needs five wait
  // states between a VALU instruction that writes an SGPR (v_readfirstlane, v_readlane restoring a
  // spilled SGPR) and a vector memory instruction that reads it, and one between a write of M0 and
  // an LDS-DMA instruction.  The compiler inserts such waits for instructions it emits itself, but
  // it cannot see that this assembly text is a memory instruction reading the descriptor, the
  // offset and M0: whenever it chose to compute or restore one of them through the VALU right in
  // front of the statement, the load took a stale value (observed: a wave-dependent tile offset
  // gave wrong tiles; with the guard the same code is correct).  s_nop 4 supplies the five wait
  // states unconditionally; measured cost: none (within +-0.5 % on every kernel).
  __device__ __forceinline__ void load16_to_lds(SPARK_LDS char* dst, uint32_t lane_off, uint32_t tile_off) const {
    asm volatile("s_nop 4\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "{m0}"(__builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst)), "v"(lane_off), "s"(desc),
                   "s"(__builtin_amdgcn_readfirstlane(tile_off))
                 : "memory");
  }
  __device__ __forceinline__ void load4_to_lds(SPARK_LDS char* dst, uint32_t lane_off, uint32_t tile_off) const {
    asm volatile("s_nop 4\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :
                 : "{m0}"(__builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst)), "v"(lane_off), "s"(desc),
                   "s"(__builtin_amdgcn_readfirstlane(tile_off))
                 : "memory");
  }
};

// Nothing may be moved across this point by the instruction scheduler.
static __device__ __forceinline__ void sched_fence() { __builtin_amdgcn_sched_barrier(0); }

// s_waitcnt vmcnt(0): every outstanding global/buffer load of this wave has returned.
static __device__ __forceinline__ void wait_vmem_all() { __builtin_amdgcn_s_waitcnt(0x0F70); }

}  // namespace spark
