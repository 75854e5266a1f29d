// Stand-alone microbenchmark: what does the per-MFMA instruction mix of each attention loop cost on
// this GPU when it runs as a straight-line loop, with no barriers, no global loads, no masks and no
// prologue?  That figure is the floor a kernel with that mix can reach; the kernels are compared with
// it instead of with the nominal MFMA peak alone, which real (non-constant) operands do not reach:
// the part lowers its clock under the power draw of toggling data.
//
// One "slot" = one v_mfma_f32_32x32x16 plus the VALU and LDS instructions the loop issues per MFMA:
//   forward element  : v_fma (scale, subtract reference), v_exp, v_add (row sum), half a v_cvt_pk
//   backward element : v_fma, v_exp, v_mul (dS = P * dP; the -D is folded into the accumulator), one v_cvt_pk
//   LDS read         : one 16-byte read whose result is an MFMA operand 8 slots later
// The VALU instructions read accumulator values written two MFMAs earlier, as the kernels do.
// Mix per kernel (32x32 score block, wave):  forward: 2d/16 MFMAs, 16 elements;  dK/dV: 4d/16 MFMAs, 16
// elements;  dQ: 3d/16 MFMAs, 16 elements.
//
// Build: hipcc --offload-arch=gfx950 -O3 (see build.py); run without arguments on the GPU.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef float f32x16 __attribute__((ext_vector_type(16)));
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
template <typename T> struct Tr;
template <> struct Tr<_Float16> {
  typedef _Float16 v8 __attribute__((ext_vector_type(8)));
  typedef _Float16 v2 __attribute__((ext_vector_type(2)));
  static __device__ f32x16 mfma(v8 a, v8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }
  static const char* name() { return "fp16"; }
};
template <> struct Tr<__bf16> {
  typedef __bf16 v8 __attribute__((ext_vector_type(8)));
  typedef __bf16 v2 __attribute__((ext_vector_type(2)));
  static __device__ f32x16 mfma(v8 a, v8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
  static const char* name() { return "bf16"; }
};
// NV2: softmax elements per TWO MFMAs.  KIND 0: forward element, 1: backward element.  NL2: LDS reads per
// two MFMAs.  WPS: waves per SIMD (workgroups of 4 waves, WPS per CU).
template <typename T, int NV2, int KIND, int NL2, int WPS>
__global__ __launch_bounds__(256, WPS) void mix_kernel(const typename Tr<T>::v8* ops, float* out, int iters) {
  typedef typename Tr<T>::v8 v8;
  typedef typename Tr<T>::v2 v2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  for (int i = threadIdx.x; i < 2048; i += 256) ((v8*)smem)[i] = ops[i % 4096];
  __syncthreads();
  v8 a[8], b[8];
  for (int i = 0; i < 8; ++i) {
    a[i] = ops[(threadIdx.x * 16 + i) % 4096];
    b[i] = ops[(threadIdx.x * 16 + 8 + i) % 4096];
  }
  f32x16 acc[4];
  for (int j = 0; j < 4; ++j)
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.f;
  float x[16], rs = 0.f;
  unsigned pk[8];
  for (int i = 0; i < 16; ++i) x[i] = (float)a[i & 7][i >> 3] * 0.01f;
  for (int i = 0; i < 8; ++i) pk[i] = 0;
  const int lane_off = (threadIdx.x & 63) * 16 + (threadIdx.x >> 6) * 4096;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      acc[u & 3] = Tr<T>::mfma(a[u & 7], b[(u * 3) & 7], acc[u & 3]);
#pragma unroll
      for (int l = 0; l < (NL2 + (u & 1)) / 2; ++l) {
        const int slot = (u + l + 4) & 7;
        v8 v = *(const v8*)(smem + lane_off + ((u + l) & 3) * 1024 + (it & 1) * 16384);
        if ((u + l) & 1) b[slot] = v; else a[slot] = v;
      }
#pragma unroll
      for (int q = 0; q < (NV2 + (u & 1)) / 2; ++q) {
        const int i = ((u * NV2) / 2 + q) & 15;
        const float s = acc[(u + 2) & 3][i];  // written two MFMAs ago
        const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(s, 0.18f, -3.0f));
        if (KIND == 0) {
          rs += p;
          if (i & 1) {
            v2 h = {(T)x[i - 1], (T)p};
            pk[i >> 1] ^= __builtin_bit_cast(unsigned, h);
            asm volatile("" : "+v"(pk[i >> 1]), "+v"(rs));
          } else {
            x[i] = p;
            asm volatile("" : "+v"(x[i]), "+v"(rs));
          }
        } else {
          const float d = p * acc[(u + 3) & 3][i];
          v2 h = {(T)p, (T)d};
          pk[i >> 1] ^= __builtin_bit_cast(unsigned, h);
          asm volatile("" : "+v"(pk[i >> 1]));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = rs;
  for (int j = 0; j < 4; ++j)
    for (int i = 0; i < 16; ++i) s += acc[j][i];
  for (int i = 0; i < 16; ++i) s += x[i];
  for (int i = 0; i < 8; ++i) s += (float)pk[i] + (float)a[i][0] + (float)b[i][1];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}
template <typename T, int NV2, int KIND, int NL2, int WPS>
void run(const void* ops, float* out, hipEvent_t e0, hipEvent_t e1, const char* what) {
  auto kern = mix_kernel<T, NV2, KIND, NL2, WPS>;
  CK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
  const int wgs = 256 * WPS, iters = 6000;
  kern<<<wgs, 256, 65536>>>((const typename Tr<T>::v8*)ops, out, 20000);  // lets the clock settle
  float best = 1e9;
  for (int rep = 0; rep < 3; ++rep) {
    CK(hipEventRecord(e0));
    kern<<<wgs, 256, 65536>>>((const typename Tr<T>::v8*)ops, out, iters);
    CK(hipEventRecord(e1));
    CK(hipEventSynchronize(e1));
    float ms;
    CK(hipEventElapsedTime(&ms, e0, e1));
    if (ms < best) best = ms;
  }
  const double per = best * 1e6 / (iters * 16.0) / WPS;
  printf("%s  %-52s waves/SIMD %d: %6.2f ns per MFMA and SIMD = %5.0f TFLOP/s executed on 1024 SIMDs\n", Tr<T>::name(), what,
         WPS, per, 1024 * 32768.0 / per / 1e3);
}
template <typename T> void all(const void* ops, float* out, hipEvent_t e0, hipEvent_t e1) {
  run<T, 0, 0, 0, 1>(ops, out, e0, e1, "MFMA only");
  run<T, 0, 0, 0, 2>(ops, out, e0, e1, "MFMA only");
  run<T, 2, 0, 3, 2>(ops, out, e0, e1, "forward d=128: 1 fwd element + 1.5 LDS reads per MFMA");
  run<T, 4, 0, 3, 3>(ops, out, e0, e1, "forward d=64:  2 fwd elements + 1.5 LDS reads per MFMA");
  run<T, 1, 1, 4, 1>(ops, out, e0, e1, "dK/dV d=128:   0.5 bwd element + 2 LDS reads per MFMA");
  run<T, 2, 1, 4, 2>(ops, out, e0, e1, "dK/dV d=64:    1 bwd element + 2 LDS reads per MFMA");
  run<T, 1, 1, 3, 2>(ops, out, e0, e1, "dQ d=128:      0.5 (kernel: 0.67) bwd element + 1.5 LDS");
  run<T, 3, 1, 3, 2>(ops, out, e0, e1, "dQ d=64:       1.5 (kernel: 1.33) bwd elements + 1.5 LDS");
}
int main() {
  const size_t n = 4096 * 8;
  void* ops;
  float* out;
  CK(hipMalloc(&ops, n * 2));
  CK(hipMalloc(&out, 256 * 3 * 256 * 4));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  printf("operands: uniform random in [-1, 1]; one slot = one v_mfma_f32_32x32x16 (32768 flop)\n");
  {
    std::vector<_Float16> f(n);
    for (size_t i = 0; i < n; ++i) f[i] = (_Float16)((rand() % 2001 - 1000) / 1000.0f);
    CK(hipMemcpy(ops, f.data(), n * 2, hipMemcpyHostToDevice));
  }
  all<_Float16>(ops, out, e0, e1);
  {
    std::vector<__bf16> f(n);
    for (size_t i = 0; i < n; ++i) f[i] = (__bf16)((rand() % 2001 - 1000) / 1000.0f);
    CK(hipMemcpy(ops, f.data(), n * 2, hipMemcpyHostToDevice));
  }
  all<__bf16>(ops, out, e0, e1);
  return 0;
}
