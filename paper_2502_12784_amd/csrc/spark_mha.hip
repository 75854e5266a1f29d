// C ABI of the fused MHA library: argument validation and kernel dispatch (host side).
// The operations are defined in include/spark_mha.h.
#include "../../include/spark_mha.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <atomic>

#include "bwd_atomic_kernels.hpp"
#include "bwd_kernels.hpp"
#include "fwd_kernel.hpp"
#include "layout_probe.hpp"

// Scratch memory of spark_mha_bwd_static: the backward's workspace (D and LSE * log2(e)) for callers
// that cannot allocate.  One copy per GPU, at its own address on each, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress, never a device address.
#define SPARK_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[SPARK_STATIC_SCRATCH_BYTES];

namespace {

using namespace spark;

// Device address of `scratch` on the current device, looked up once per device with that device
// current and kept; nullptr if the runtime cannot resolve it.
void* static_scratch_ptr() {
  static std::atomic<void*> ptrs[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  void* p = ptrs[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  ptrs[dev].store(p, std::memory_order_release);  // every thread resolves the same address
  return p;
}

// hipGetLastError() == hipSuccess, and with SPARK_MHA_DEBUG set in the environment the runtime's own
// description of a failure on stderr (the C ABI itself only returns SPARK_ERR_LAUNCH).
bool launch_ok(const char* what) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return true;
  static const bool verbose = getenv("SPARK_MHA_DEBUG") != nullptr;
  if (verbose) fprintf(stderr, "spark_mha: %s: %s\n", what, hipGetErrorString(e));
  return false;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Everything one problem is made of; the entry points fill it and hand it to the launchers.
struct Problem {
  int B, H, Nq, Nk, d;
  float scale;
  int causal;
  int dtype;
  int thr;  // dropout threshold, 0 = no dropout
  unsigned long long seed;
  unsigned offset;
  // element strides of the [B,H,N,d] tensors
  TensorMap mq, mk, mv, mo, mdo, mdq, mdk, mdv;
  hipStream_t st;
};

TensorMap contiguous(int H, int N, int d) {
  return TensorMap{(long long)H * N * d, (long long)N * d, (long long)d};
}

// Nq queries attend to Nk keys; self-attention passes the same N twice.
int check_common(int B, int H, int Nq, int Nk, int d, float scale, int causal, int dtype) {
  if (dtype != SPARK_F16 && dtype != SPARK_BF16) return SPARK_ERR_DTYPE;
  if (B < 1 || H < 1 || Nq < 1 || Nk < 1) return SPARK_ERR_SHAPE;
  if (causal && Nq != Nk) return SPARK_ERR_SHAPE;  // the mask is defined for a square S only
  if (d < 8 || d > 128 || (d & 7)) return SPARK_ERR_SHAPE;  // rows of 16-byte chunks, tiles up to 128 wide
  if (!isfinite(scale) || !(scale > 0.f)) return SPARK_ERR_SHAPE;
  const int64_t bh = (int64_t)B * H;
  const int64_t nmax = Nq > Nk ? Nq : Nk;
  const int64_t tiles64 = (nmax + 63) / 64;
  if (bh * tiles64 >= (int64_t)1 << 31) return SPARK_ERR_SHAPE;
  // 31-bit byte offsets inside one head, including the rows a ragged last tile reaches past N
  if ((nmax + 256) * d * 2 >= (int64_t)1 << 31) return SPARK_ERR_SHAPE;
  return SPARK_OK;
}

// A strided tensor is usable if rows hold d contiguous elements, every stride keeps 16-byte
// alignment, and one head's rows span less than 4 GiB (the kernels address a head through a
// 32-bit buffer descriptor).
// An output tensor must in addition give every (batch, head) its own rows: a zero batch or head stride
// (a broadcast, fine for an input) would make all those workgroups store to the same memory.
int check_strides(const spark_strides_t* s, int N, int d, TensorMap* out, bool is_output = false, int B = 1,
                  int H = 1) {
  if (!s) return SPARK_ERR_NULL;
  if (s->batch < 0 || s->head < 0 || s->row < d) return SPARK_ERR_SHAPE;
  if (is_output && ((B > 1 && s->batch == 0) || (H > 1 && s->head == 0))) return SPARK_ERR_SHAPE;
  if ((s->batch | s->head | s->row) & 7) return SPARK_ERR_ALIGN;
  // 31-bit byte offsets inside one head, including the rows a ragged last tile reaches past N
  // (offsets from 2^31 on are how the kernels mark chunks that must read as zeros)
  if ((int64_t)(N + 256) * s->row * 2 >= (int64_t)1 << 31) return SPARK_ERR_SHAPE;
  *out = TensorMap{s->batch, s->head, s->row};
  return SPARK_OK;
}

// Dropout rate -> 8-bit threshold: an entry is dropped iff its random byte < thr, i.e. with
// probability thr / 256.  -1 if the rate is not a number in [0, 255.5/256).
int drop_threshold(float p_drop) {
  if (!(p_drop >= 0.f) || !(p_drop < 1.f)) return -1;
  const int thr = (int)floorf(p_drop * 256.0f + 0.5f);
  return thr <= 255 ? thr : -1;
}

Dropout make_dropout(int thr, unsigned long long seed, unsigned offset) {
  Dropout dr;
  dr.key0 = (uint32_t)seed;
  dr.key1 = (uint32_t)(seed >> 32);
  dr.offset = offset;
  dr.thr = (uint32_t)thr;
  dr.keep_prob = (float)(256 - thr) / 256.0f;
  dr.rescale = 256.0f / (float)(256 - thr);
  return dr;
}

template <typename KernelT>
int set_smem(KernelT kernel, int bytes) {
  // The kernels address LDS from 0 (lds_origin): that holds only without static LDS in front.
  hipFuncAttributes fa;
  if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel)) != hipSuccess || fa.sharedSizeBytes != 0) {
    if (getenv("SPARK_MHA_DEBUG")) fprintf(stderr, "spark_mha: kernel attributes unavailable or static LDS present\n");
    return SPARK_ERR_LAUNCH;
  }
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess && getenv("SPARK_MHA_DEBUG"))
    fprintf(stderr, "spark_mha: hipFuncSetAttribute(%d bytes of LDS): %s\n", bytes, hipGetErrorString(e));
  return e == hipSuccess ? SPARK_OK : SPARK_ERR_LAUNCH;
}

// set_smem once per kernel and device: the attribute belongs to the function on the current
// device, so a process that drives several GPUs needs it on each of them.  `done` holds one bit
// per device ordinal; a failure is not remembered, the next call tries again.
template <typename KernelT>
int ensure_smem(KernelT kernel, int bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) return SPARK_ERR_LAUNCH;
  if (dev < 64 && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return SPARK_OK;
  const int rc = set_smem(kernel, bytes);
  if (rc == SPARK_OK && dev < 64) done.fetch_or(uint64_t(1) << dev, std::memory_order_release);
  return rc;
}

// Workgroups of 8 waves (256 query rows, one per CU) instead of 4 (128 rows, two per CU): each
// K/V tile brought into LDS then serves twice as many MFMAs.  Pays at d = 128 when the wider
// tiles still give every CU at least two workgroups and the loop over the keys is long enough
// to outweigh running one workgroup per CU with nothing to overlap its prologue and epilogue
// (measured on the grid of Sec. 4.1, hidden size 2048: -5 ... -7 % from 2048 keys on, +7 ... +10 %
// at 512, equal at 1024; at d = 64 it costs 2 %).
template <bool CAUSAL>
bool wide_workgroups(const Problem& p) {
  const int64_t tiles = (p.Nq + 255) / 256;
  return p.d > 64 && p.Nk >= 2048 && (int64_t)p.B * p.H * causal_items<CAUSAL>((int)tiles) >= 512;
}

template <typename T, int D, bool CAUSAL, bool DROP, int NW, bool PAIR = false>
int launch_fwd_nw(const Problem& p, const void* Q, const void* K, const void* V, void* O, float* LSE) {
  using C = FwdCfg<D, NW, PAIR>;
  auto kernel = mha_fwd_kernel<T, D, CAUSAL, DROP, NW, PAIR>;
  static std::atomic<uint64_t> ready{0};
  const int attr = ensure_smem(kernel, C::SMEM, ready);
  if (attr != SPARK_OK) return attr;
  const int BH = p.B * p.H;
  const int nqt = (p.Nq + C::BM - 1) / C::BM;
  const float scale_log2 = p.scale * 1.4426950408889634f;
  hipLaunchKernelGGL(kernel, dim3((unsigned)(BH * causal_items<CAUSAL>(nqt))), dim3(64 * NW), C::SMEM, p.st,
                     static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                     static_cast<T*>(O), LSE, p.mq, p.mk, p.mv, p.mo, p.H, p.Nq, p.Nk, p.d, nqt, scale_log2,
                     make_dropout(p.thr, p.seed, p.offset));
  return launch_ok("forward kernel") ? SPARK_OK : SPARK_ERR_LAUNCH;
}

template <typename T, int D, bool CAUSAL, bool DROP>
int launch_fwd(const Problem& p, const void* Q, const void* K, const void* V, void* O, float* LSE) {
  if constexpr (D == 128) {
    // ... with the K/V tiles requested two at a time and one barrier every second iteration (the
    // workgroup has the CU's LDS to itself): another -1 ... -3 % on the forward.
    if (wide_workgroups<CAUSAL>(p)) return launch_fwd_nw<T, D, CAUSAL, DROP, 8, true>(p, Q, K, V, O, LSE);
  }
  return launch_fwd_nw<T, D, CAUSAL, DROP, 4>(p, Q, K, V, O, LSE);
}

template <typename T, int D, bool CAUSAL, bool DROP>
int launch_bwd(const Problem& p, const void* Q, const void* K, const void* V, const void* O,
               const float* LSE, const void* dO, void* dQ, void* dK, void* dV, float* Dws,
               void* const* ev) {
  const T* q = static_cast<const T*>(Q);
  const T* k = static_cast<const T*>(K);
  const T* v = static_cast<const T*>(V);
  const T* o = static_cast<const T*>(O);
  const T* dout = static_cast<const T*>(dO);
  const int BH = p.B * p.H;
  const Dropout dr = make_dropout(p.thr, p.seed, p.offset);
  float* LSE2ws = Dws + (size_t)BH * p.Nq;  // second half of the workspace: LSE * log2(e)
  // optional profiling marks between the kernels (spark_mha_bwd_marked)
  auto mark = [&](int i) {
    return !ev || hipEventRecord(static_cast<hipEvent_t>(ev[i]), p.st) == hipSuccess;
  };

  if (!mark(0)) return SPARK_ERR_LAUNCH;
  {  // dQ: one workgroup per tile of 128 queries (8-wave workgroups measured 3 % slower here).
     // Also writes D = rowsum(dO o O) and LSE * log2(e) for the dK/dV kernel.
    using C = BwdQCfg<D>;
    auto kernel = mha_bwd_dq_kernel<T, D, CAUSAL, DROP>;
    static std::atomic<uint64_t> ready{0};
    const int attr = ensure_smem(kernel, C::SMEM, ready);
    if (attr != SPARK_OK) return attr;
    const int nqt = (p.Nq + C::BM - 1) / C::BM;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(BH * causal_items<CAUSAL>(nqt))), dim3(256), C::SMEM, p.st,
                       q, k, v, o, dout, LSE, Dws, LSE2ws, static_cast<T*>(dQ), p.mq, p.mk, p.mv, p.mo,
                       p.mdo, p.mdq, p.H, p.Nq, p.Nk, p.d, nqt, p.scale, p.scale * 1.4426950408889634f, dr);
    if (!launch_ok("dQ kernel") || !mark(1)) return SPARK_ERR_LAUNCH;
  }
  {  // dK, dV: one workgroup per tile of 128 keys, software-pipelined
    using C = BwdKvPipeCfg<D>;
    auto kernel = mha_bwd_dkdv_pipe_kernel<T, D, CAUSAL, DROP>;
    static std::atomic<uint64_t> ready{0};
    const int attr = ensure_smem(kernel, C::SMEM, ready);
    if (attr != SPARK_OK) return attr;
    const int nkt = (p.Nk + C::BN - 1) / C::BN;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(BH * causal_items<CAUSAL>(nkt))), dim3(256), C::SMEM, p.st,
                       q, k, v, dout, LSE2ws, Dws, static_cast<T*>(dK), static_cast<T*>(dV), p.mq, p.mk,
                       p.mv, p.mdo, p.mdk, p.mdv, p.H, p.Nq, p.Nk, p.d, nkt, p.scale, dr);
    if (!launch_ok("dK/dV kernel") || !mark(2)) return SPARK_ERR_LAUNCH;
  }
  return SPARK_OK;
}

size_t workspace_bytes(int B, int H, int Nq) { return 2 * (size_t)B * H * Nq * sizeof(float); }
size_t workspace_bytes_stats(int B, int H, int Nq) { return workspace_bytes(B, H, Nq); }

// The paper's own backward (Sec. 3.3): prepare (D, LSE * log2(e), cleared fp32 dQ accumulator), one
// fused kernel that adds dQ contributions with atomics, conversion of the accumulator to dQ.
size_t atomic_dq_offset(int B, int H, int Nq) { return (workspace_bytes_stats(B, H, Nq) + 255) & ~(size_t)255; }

template <typename T, int D, bool CAUSAL>
int launch_bwd_atomic(const Problem& p, const void* Q, const void* K, const void* V, const void* O,
                      const float* LSE, const void* dO, void* dQ, void* dK, void* dV, void* workspace) {
  const int BH = p.B * p.H;
  const long long rows = (long long)BH * p.Nq;
  float* Dws = static_cast<float*>(workspace);
  float* LSE2ws = Dws + rows;
  float* dQacc = reinterpret_cast<float*>(static_cast<char*>(workspace) + atomic_dq_offset(p.B, p.H, p.Nq));
  hipLaunchKernelGGL(mha_bwd_prep_kernel<T>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, p.st,
                     static_cast<const T*>(O), static_cast<const T*>(dO), LSE, Dws, LSE2ws, dQacc, p.mo, p.mdo,
                     p.H, p.Nq, p.d, rows);
  if (hipGetLastError() != hipSuccess) return SPARK_ERR_LAUNCH;
  {
    using C = BwdAtomicCfg<D>;
    auto kernel = mha_bwd_fused_atomic_kernel<T, D, CAUSAL>;
    static std::atomic<uint64_t> ready{0};
    const int attr = ensure_smem(kernel, C::SMEM, ready);
    if (attr != SPARK_OK) return attr;
    const int nkt = (p.Nk + C::BN - 1) / C::BN;
    hipLaunchKernelGGL(kernel, dim3((unsigned)(BH * causal_items<CAUSAL>(nkt))), dim3(256), C::SMEM, p.st,
                       static_cast<const T*>(Q), static_cast<const T*>(K), static_cast<const T*>(V),
                       static_cast<const T*>(dO), LSE2ws, Dws, dQacc, static_cast<T*>(dK), static_cast<T*>(dV),
                       p.mq, p.mk, p.mv, p.mdo, p.mdk, p.mdv, p.H, p.Nq, p.Nk, p.d, nkt, p.scale);
    if (hipGetLastError() != hipSuccess) return SPARK_ERR_LAUNCH;
  }
  const long long chunks = rows * (p.d >> 3);
  hipLaunchKernelGGL(mha_bwd_dq_convert_kernel<T>, dim3((unsigned)((chunks + 255) / 256)), dim3(256), 0, p.st,
                     dQacc, static_cast<T*>(dQ), p.mdq, p.H, p.Nq, p.d, p.scale, chunks);
  return hipGetLastError() == hipSuccess ? SPARK_OK : SPARK_ERR_LAUNCH;
}

// Expand the (dtype, d, causal, dropout) runtime tuple into a template instantiation.
#define SPARK_DISPATCH_CD(FN, T, D, ...)                                                    \
  do {                                                                                      \
    if (p.causal) return p.thr ? FN<T, D, true, true>(__VA_ARGS__)                          \
                               : FN<T, D, true, false>(__VA_ARGS__);                        \
    return p.thr ? FN<T, D, false, true>(__VA_ARGS__) : FN<T, D, false, false>(__VA_ARGS__); \
  } while (0)
#define SPARK_DISPATCH(FN, ...)                                              \
  do {                                                                       \
    if (p.dtype == SPARK_F16) {                                              \
      if (p.d <= 64) SPARK_DISPATCH_CD(FN, _Float16, 64, __VA_ARGS__);       \
      SPARK_DISPATCH_CD(FN, _Float16, 128, __VA_ARGS__);                     \
    }                                                                        \
    if (p.d <= 64) SPARK_DISPATCH_CD(FN, __bf16, 64, __VA_ARGS__);           \
    SPARK_DISPATCH_CD(FN, __bf16, 128, __VA_ARGS__);                         \
  } while (0)

// Shape, scale, dtype and dropout checks common to forward and backward; fills `p` with
// contiguous strides (the strided entry points overwrite them afterwards).
int make_problem(Problem* p, int B, int H, int Nq, int Nk, int d, float scale, int causal, int thr,
                 unsigned long long seed, unsigned offset, spark_dtype_t dtype, void* stream) {
  const int rc = check_common(B, H, Nq, Nk, d, scale, causal, (int)dtype);
  if (rc != SPARK_OK) return rc;
  if (thr < 0) return SPARK_ERR_SHAPE;
  p->B = B; p->H = H; p->Nq = Nq; p->Nk = Nk; p->d = d;
  p->scale = scale;
  p->causal = causal != 0;
  p->dtype = (int)dtype;
  p->thr = thr;
  p->seed = seed;
  p->offset = offset;
  p->mq = p->mo = p->mdo = p->mdq = contiguous(H, Nq, d);
  p->mk = p->mv = p->mdk = p->mdv = contiguous(H, Nk, d);
  p->st = static_cast<hipStream_t>(stream);
  return SPARK_OK;
}

int run_fwd(const Problem& p, const void* Q, const void* K, const void* V, void* O, float* LSE) {
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE))
    return SPARK_ERR_ALIGN;
  SPARK_DISPATCH(launch_fwd, p, Q, K, V, O, LSE);
}

int run_bwd(const Problem& p, const void* Q, const void* K, const void* V, const void* O,
            const float* LSE, const void* dO, void* dQ, void* dK, void* dV, void* workspace,
            size_t ws_bytes, void* const* ev) {
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE) ||
      !aligned16(dO) || !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return SPARK_ERR_ALIGN;
  if (ws_bytes < workspace_bytes(p.B, p.H, p.Nq)) return SPARK_ERR_WORKSPACE;
  float* Dws = static_cast<float*>(workspace);
  SPARK_DISPATCH(launch_bwd, p, Q, K, V, O, LSE, dO, dQ, dK, dV, Dws, ev);
}

}  // namespace

extern "C" {

int spark_mha_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B, int H,
                  int N, int d, float scale, int causal, spark_dtype_t dtype, void* stream) {
  return spark_mha_cross_fwd(Q, K, V, O, LSE, B, H, N, N, d, scale, causal, dtype, stream);
}

int spark_mha_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                        int H, int Nq, int Nk, int d, float scale, int causal,
                        spark_dtype_t dtype, void* stream) {
  return spark_mha_dropout_fwd(Q, K, V, O, LSE, B, H, Nq, Nk, d, scale, causal, 0.0f, 0, 0, dtype,
                               stream);
}

int spark_mha_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int B,
                          int H, int Nq, int Nk, int d, float scale, int causal, float p_drop,
                          unsigned long long seed, unsigned offset, spark_dtype_t dtype,
                          void* stream) {
  if (!Q || !K || !V || !O || !LSE) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, drop_threshold(p_drop), seed,
                              offset, dtype, stream);
  if (rc != SPARK_OK) return rc;
  return run_fwd(p, Q, K, V, O, LSE);
}

int spark_mha_strided_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const spark_strides_t* sQ, const spark_strides_t* sK,
                          const spark_strides_t* sV, const spark_strides_t* sO, int B, int H, int Nq,
                          int Nk, int d, float scale, int causal, float p_drop,
                          unsigned long long seed, unsigned offset, spark_dtype_t dtype,
                          void* stream) {
  if (!Q || !K || !V || !O || !LSE) return SPARK_ERR_NULL;
  Problem p;
  int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, drop_threshold(p_drop), seed, offset,
                        dtype, stream);
  if (rc != SPARK_OK) return rc;
  if ((rc = check_strides(sQ, Nq, d, &p.mq)) != SPARK_OK) return rc;
  if ((rc = check_strides(sK, Nk, d, &p.mk)) != SPARK_OK) return rc;
  if ((rc = check_strides(sV, Nk, d, &p.mv)) != SPARK_OK) return rc;
  if ((rc = check_strides(sO, Nq, d, &p.mo, true, B, H)) != SPARK_OK) return rc;
  return run_fwd(p, Q, K, V, O, LSE);
}

size_t spark_mha_cross_bwd_workspace_bytes(int B, int H, int Nq, int Nk, int d,
                                           spark_dtype_t dtype) {
  if (check_common(B, H, Nq, Nk, d, 1.0f, 0, (int)dtype) != SPARK_OK) return 0;
  return workspace_bytes(B, H, Nq);  // D and LSE*log2(e), fp32 [B,H,Nq] each
}

size_t spark_mha_bwd_workspace_bytes(int B, int H, int N, int d, spark_dtype_t dtype) {
  return spark_mha_cross_bwd_workspace_bytes(B, H, N, N, d, dtype);
}

int spark_mha_bwd(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                  const void* dO, void* dQ, void* dK, void* dV, void* workspace,
                  size_t workspace_bytes, int B, int H, int N, int d, float scale, int causal,
                  spark_dtype_t dtype, void* stream) {
  return spark_mha_cross_bwd(Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, B, H, N, N,
                             d, scale, causal, dtype, stream);
}

int spark_mha_cross_bwd(const void* Q, const void* K, const void* V, const void* O,
                        const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                        void* workspace, size_t workspace_bytes, int B, int H, int Nq, int Nk,
                        int d, float scale, int causal, spark_dtype_t dtype, void* stream) {
  return spark_mha_dropout_bwd(Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, B, H, Nq,
                               Nk, d, scale, causal, 0.0f, 0, 0, dtype, stream);
}

int spark_mha_dropout_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                          void* workspace, size_t workspace_bytes, int B, int H, int Nq, int Nk,
                          int d, float scale, int causal, float p_drop, unsigned long long seed,
                          unsigned offset, spark_dtype_t dtype, void* stream) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !workspace) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, drop_threshold(p_drop), seed,
                              offset, dtype, stream);
  if (rc != SPARK_OK) return rc;
  return run_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, nullptr);
}

int spark_mha_strided_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                          const spark_strides_t* sQ, const spark_strides_t* sK,
                          const spark_strides_t* sV, const spark_strides_t* sO,
                          const spark_strides_t* sdO, const spark_strides_t* sdQ,
                          const spark_strides_t* sdK, const spark_strides_t* sdV, void* workspace,
                          size_t workspace_bytes, int B, int H, int Nq, int Nk, int d, float scale,
                          int causal, float p_drop, unsigned long long seed, unsigned offset,
                          spark_dtype_t dtype, void* stream) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !workspace) return SPARK_ERR_NULL;
  Problem p;
  int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, drop_threshold(p_drop), seed, offset,
                        dtype, stream);
  if (rc != SPARK_OK) return rc;
  if ((rc = check_strides(sQ, Nq, d, &p.mq)) != SPARK_OK) return rc;
  if ((rc = check_strides(sK, Nk, d, &p.mk)) != SPARK_OK) return rc;
  if ((rc = check_strides(sV, Nk, d, &p.mv)) != SPARK_OK) return rc;
  if ((rc = check_strides(sO, Nq, d, &p.mo)) != SPARK_OK) return rc;
  if ((rc = check_strides(sdO, Nq, d, &p.mdo)) != SPARK_OK) return rc;
  if ((rc = check_strides(sdQ, Nq, d, &p.mdq, true, B, H)) != SPARK_OK) return rc;
  if ((rc = check_strides(sdK, Nk, d, &p.mdk, true, B, H)) != SPARK_OK) return rc;
  if ((rc = check_strides(sdV, Nk, d, &p.mdv, true, B, H)) != SPARK_OK) return rc;
  return run_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, nullptr);
}

int spark_mha_bwd_marked(const void* Q, const void* K, const void* V, const void* O,
                         const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                         void* workspace, size_t workspace_bytes, int B, int H, int N, int d,
                         float scale, int causal, spark_dtype_t dtype, void* stream,
                         void* const events[3]) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !workspace) return SPARK_ERR_NULL;
  if (!events || !events[0] || !events[1] || !events[2]) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, N, N, d, scale, causal, 0, 0, 0, dtype, stream);
  if (rc != SPARK_OK) return rc;
  return run_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, events);
}

size_t spark_mha_bwd_static_max_rows(void) { return SPARK_STATIC_SCRATCH_BYTES / (2 * sizeof(float)); }

int spark_mha_bwd_static(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                         const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N, int d,
                         float scale, int causal, spark_dtype_t dtype, void* stream) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, N, N, d, scale, causal, 0, 0, 0, dtype, stream);
  if (rc != SPARK_OK) return rc;
  if (workspace_bytes(B, H, N) > SPARK_STATIC_SCRATCH_BYTES) return SPARK_ERR_WORKSPACE;
  void* ws = static_scratch_ptr();
  if (!ws) return SPARK_ERR_LAUNCH;
  return run_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, ws, SPARK_STATIC_SCRATCH_BYTES, nullptr);
}

size_t spark_mha_bwd_atomic_workspace_bytes(int B, int H, int Nq, int Nk, int d, spark_dtype_t dtype) {
  if (check_common(B, H, Nq, Nk, d, 1.0f, 0, (int)dtype) != SPARK_OK) return 0;
  return atomic_dq_offset(B, H, Nq) + (size_t)B * H * Nq * d * sizeof(float);
}

int spark_mha_bwd_atomic(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                         const void* dO, void* dQ, void* dK, void* dV, void* workspace,
                         size_t workspace_bytes, int B, int H, int Nq, int Nk, int d, float scale,
                         int causal, spark_dtype_t dtype, void* stream) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !workspace) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, 0, 0, 0, dtype, stream);
  if (rc != SPARK_OK) return rc;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(LSE) ||
      !aligned16(dO) || !aligned16(dQ) || !aligned16(dK) || !aligned16(dV) || !aligned16(workspace))
    return SPARK_ERR_ALIGN;
  // the two elementwise kernels are gridded over rows / 16 and over 8-element chunks / 256
  if (((int64_t)B * H * Nq + 15) / 16 >= (int64_t)1 << 31 ||
      ((int64_t)B * H * Nq * (d >> 3) + 255) / 256 >= (int64_t)1 << 31)
    return SPARK_ERR_SHAPE;
  if (workspace_bytes < spark_mha_bwd_atomic_workspace_bytes(B, H, Nq, Nk, d, dtype)) return SPARK_ERR_WORKSPACE;
#define SPARK_ATOMIC_CD(T, D)                                                                          \
  return p.causal ? launch_bwd_atomic<T, D, true>(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace)       \
                  : launch_bwd_atomic<T, D, false>(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace)
  if (p.dtype == SPARK_F16) {
    if (p.d <= 64) SPARK_ATOMIC_CD(_Float16, 64);
    SPARK_ATOMIC_CD(_Float16, 128);
  }
  if (p.d <= 64) SPARK_ATOMIC_CD(__bf16, 64);
  SPARK_ATOMIC_CD(__bf16, 128);
#undef SPARK_ATOMIC_CD
}

int spark_mha_dropout_bwd_marked(const void* Q, const void* K, const void* V, const void* O,
                                 const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                                 void* workspace, size_t workspace_bytes, int B, int H, int Nq, int Nk,
                                 int d, float scale, int causal, float p_drop, unsigned long long seed,
                                 unsigned offset, spark_dtype_t dtype, void* stream,
                                 void* const events[3]) {
  if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV || !workspace) return SPARK_ERR_NULL;
  if (!events || !events[0] || !events[1] || !events[2]) return SPARK_ERR_NULL;
  Problem p;
  const int rc = make_problem(&p, B, H, Nq, Nk, d, scale, causal, drop_threshold(p_drop), seed,
                              offset, dtype, stream);
  if (rc != SPARK_OK) return rc;
  return run_bwd(p, Q, K, V, O, LSE, dO, dQ, dK, dV, workspace, workspace_bytes, events);
}

int spark_dropout_threshold(float p_drop) { return drop_threshold(p_drop); }

int spark_dropout_mask(unsigned char* M, int B, int H, int Nq, int Nk, float p_drop,
                       unsigned long long seed, unsigned offset, void* stream) {
  if (!M) return SPARK_ERR_NULL;
  if (B < 1 || H < 1 || Nq < 1 || Nk < 1) return SPARK_ERR_SHAPE;
  const int thr = drop_threshold(p_drop);
  if (thr < 0) return SPARK_ERR_SHAPE;
  const int qblocks = (Nq + 3) / 4, kblocks = (Nk + 3) / 4;
  const long long total = (long long)B * H * qblocks * kblocks;
  if (total >= ((long long)1 << 31) * 256) return SPARK_ERR_SHAPE;
  const unsigned grid = (unsigned)((total + 255) / 256);
  hipLaunchKernelGGL(dropout_mask_kernel, dim3(grid), dim3(256), 0, static_cast<hipStream_t>(stream),
                     M, Nq, Nk, qblocks, kblocks, total, make_dropout(thr, seed, offset));
  return hipGetLastError() == hipSuccess ? SPARK_OK : SPARK_ERR_LAUNCH;
}

int spark_layout_probe(float* out, spark_dtype_t dtype, void* stream) {
  if (!out) return SPARK_ERR_NULL;
  if (dtype != SPARK_F16 && dtype != SPARK_BF16) return SPARK_ERR_DTYPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (dtype == SPARK_F16)
    hipLaunchKernelGGL(layout_probe_kernel<_Float16>, dim3(1), dim3(64), 16 * 64 * 2, st, out);
  else
    hipLaunchKernelGGL(layout_probe_kernel<__bf16>, dim3(1), dim3(64), 16 * 64 * 2, st, out);
  return hipGetLastError() == hipSuccess ? SPARK_OK : SPARK_ERR_LAUNCH;
}

const char* spark_status_str(int status) {
  switch (status) {
    case SPARK_OK: return "ok";
    case SPARK_ERR_NULL: return "a required pointer is NULL";
    case SPARK_ERR_SHAPE:
      return "unsupported shape, scale, dropout rate or stride (need B,H,N >= 1, d a multiple of 8 with "
             "8 <= d <= 128, finite scale > 0, Nq == Nk if causal, 0 <= p_drop < 0.998, row stride >= d, "
             "nonzero batch/head strides for outputs, sizes within the documented limits)";
    case SPARK_ERR_DTYPE: return "unsupported dtype (need SPARK_F16 or SPARK_BF16)";
    case SPARK_ERR_ALIGN: return "a pointer or stride is not 16-byte aligned";
    case SPARK_ERR_WORKSPACE:
      return "workspace smaller than spark_mha_bwd_workspace_bytes(), or B*H*N above "
             "spark_mha_bwd_static_max_rows() for spark_mha_bwd_static";
    case SPARK_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
  }
}

}  // extern "C"
