/*
 * spark_mha.h -- C ABI of the fused multi-head-attention library for MI355X (gfx950).
 *
 * Two operations, each enqueued on a caller-provided HIP stream, each in a self-attention
 * form (one sequence length N), a cross-attention form (Nq queries, Nk keys/values) and a
 * form with attention dropout:
 *
 *   spark_mha_fwd : O = softmax(scale * Q K^T [+ causal mask]) V, and the row
 *                   statistic LSE that the backward needs.
 *                   (paper Sec. 2.1 Eq. 1; fused single-kernel scheme of Sec. 3.2;
 *                   online softmax of Sec. 3.2.1 Eq. 2-3.  The scale multiplies
 *                   the logits before the softmax.)
 *   spark_mha_bwd : dQ, dK, dV from dO, recomputing P = exp(S - LSE) instead of
 *                   storing it (paper Sec. 3.3 Eq. 4, with dK = dS^T Q and
 *                   dS = P o (dP - D), D = rowsum(dO o O), the paper's "dPsum").
 *
 * Conventions common to every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises; it only enqueues kernels on
 *     `stream` (a hipStream_t passed as void*; NULL means the default stream).
 *     The work runs on the calling thread's current device, which must be the device that
 *     `stream` and all pointers belong to; each device is set up on its first call.
 *   - Q, K, V, O, dO, dQ, dK, dV have shape [B, H, N, d], contiguous, d fastest,
 *     element type `dtype` (IEEE fp16 or bfloat16).  LSE has shape [B, H, N],
 *     fp32.  Pointers must be 16-byte aligned.  Inputs and outputs must not
 *     alias each other.
 *   - Supported: d a multiple of 8 with 8 <= d <= 128 (the paper's own sizes are 64 and 128,
 *     Sec. 4.1; the kernels are built for rows of 64 and of 128 elements, and a smaller d runs in
 *     the next wider one with the missing columns read as zeros, so d = 96 costs what d = 128
 *     costs); any N >= 1; B, H >= 1; scale finite and > 0; causal is a flag (0 = all keys,
 *     nonzero = masked).  Size limits: B*H*ceil(N/64) < 2^31 and (N + 256)*d*2 < 2^31.  Anything
 *     else returns SPARK_ERR_SHAPE; nothing is silently mis-computed.
 *   - causal != 0: query i attends to keys j <= i (Sec. 2.1, masked MHA).
 *   - The spark_mha_cross_* entry points take Nq query rows and Nk key/value rows (Sec. 2.1:
 *     the decoder's second attention layer attends to the encoder output, so S of Eq. 1 is
 *     Nq x Nk there).  Q, O, dO, dQ are then [B, H, Nq, d]; K, V, dK, dV are [B, H, Nk, d];
 *     LSE is [B, H, Nq].  Nq, Nk >= 1, each under the limits stated for N.  The causal
 *     mask is defined for Nq == Nk only: causal != 0 with Nq != Nk returns SPARK_ERR_SHAPE.
 *     spark_mha_fwd / spark_mha_bwd are exactly the cross forms with Nq = Nk = N.
 *   - Arithmetic: both contractions run on fp16/bf16 MFMA with fp32
 *     accumulation; the softmax statistics, P before packing, the O
 *     accumulator, LSE, D and dS before packing are fp32 (Sec. 3.2.1: softmax in
 *     16 bits is not accurate enough).  Results are rounded once to `dtype`.
 *   - Every argument is validated before anything is enqueued: a call that
 *     returns an error has no side effect.  Launch failures reported by the
 *     runtime are returned as SPARK_ERR_LAUNCH.
 *   - Thread safety: the entry points keep no mutable global state other than a
 *     one-time per-process kernel-attribute setup; concurrent calls on different
 *     streams are allowed as long as their output buffers differ.
 */
#ifndef SPARK_MHA_H_
#define SPARK_MHA_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SPARK_F16 = 0, SPARK_BF16 = 1 } spark_dtype_t;

typedef enum {
  SPARK_OK = 0,
  SPARK_ERR_NULL = -1,      /* a required pointer is NULL */
  SPARK_ERR_SHAPE = -2,     /* B, H or N < 1; d not a multiple of 8 in 8..128; a size limit exceeded;
                               scale not finite or <= 0; causal with Nq != Nk; invalid p_drop; row
                               stride < d, a head spanning 2 GiB or more, or an output tensor with a
                               zero batch (B > 1) or head (H > 1) stride */
  SPARK_ERR_DTYPE = -3,     /* dtype is neither SPARK_F16 nor SPARK_BF16 */
  SPARK_ERR_ALIGN = -4,     /* a pointer, or a stride in bytes, is not a multiple of 16 */
  SPARK_ERR_WORKSPACE = -5, /* workspace too small (see spark_mha_bwd_workspace_bytes) */
  SPARK_ERR_LAUNCH = -6     /* the HIP runtime refused a launch */
} spark_status_t;

/*
 * Forward (paper Sec. 3.2, Eq. 1-3).
 *   Q, K, V : in,  device, [B,H,N,d] dtype
 *   O       : out, device, [B,H,N,d] dtype, fully overwritten
 *   LSE     : out, device, [B,H,N] fp32: natural-log log-sum-exp over the allowed
 *             keys of the scaled logits, LSE_i = ln sum_j exp(scale * q_i . k_j).
 *             (This is the row statistic the paper's Sec. 3.3 calls "LES" and
 *             uses as Exp(S_ij - L_i).)
 * Returns SPARK_OK or a negative spark_status_t.
 */
int spark_mha_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                  int B, int H, int N, int d, float scale, int causal,
                  spark_dtype_t dtype, void* stream);

/*
 * Bytes of device workspace spark_mha_bwd needs for this problem (holds
 * -D, D = rowsum(dO o O), and LSE * log2(e), fp32 [B,H,N] each).  Returns 0 for invalid shapes.
 */
size_t spark_mha_bwd_workspace_bytes(int B, int H, int N, int d, spark_dtype_t dtype);

/*
 * Backward (paper Sec. 3.3, Eq. 4).
 *   Q, K, V, O, dO : in,  device, [B,H,N,d] dtype   (O, LSE as written by spark_mha_fwd)
 *   LSE            : in,  device, [B,H,N] fp32
 *   dQ, dK, dV     : out, device, [B,H,N,d] dtype, fully overwritten (no need to zero)
 *   workspace      : device scratch of at least spark_mha_bwd_workspace_bytes(...)
 *                    bytes, 16-byte aligned; contents on return are unspecified.
 * Enqueues, in order on `stream`: the dQ kernel (one workgroup per query tile; a
 * separate deterministic pass in place of the paper's atomic adds into HBM; it
 * also forms D for its rows and leaves it in the workspace) and the dK/dV kernel
 * (one workgroup per key/value tile, accumulating dK and dV on chip as in Sec. 3.3).
 */
int spark_mha_bwd(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                  const void* dO, void* dQ, void* dK, void* dV,
                  void* workspace, size_t workspace_bytes,
                  int B, int H, int N, int d, float scale, int causal,
                  spark_dtype_t dtype, void* stream);

/*
 * spark_mha_bwd with profiling marks: identical work, and additionally records the caller's
 * three HIP events (hipEvent_t handles, host array) on `stream`: events[0] before the dQ
 * kernel, events[1] after it, events[2] after the dK/dV kernel.  The caller creates, reads and
 * destroys the events.  SPARK_ERR_NULL if any is NULL.
 */
int spark_mha_bwd_marked(const void* Q, const void* K, const void* V, const void* O,
                         const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                         void* workspace, size_t workspace_bytes,
                         int B, int H, int N, int d, float scale, int causal,
                         spark_dtype_t dtype, void* stream, void* const events[3]);

/*
 * The backward exactly as the paper builds it (Sec. 3.3): ONE fused kernel whose workgroups each own a
 * slice of dK and dV, accumulate them on chip, and add their contributions to dQ into HBM with fp32
 * atomic adds in every iteration (five contractions executed for five counted), preceded by a
 * kernel that forms D = rowsum(dO o O) and clears the fp32 dQ accumulator and followed by one that
 * scales and rounds the accumulator to dQ.  Same arguments, layouts and error codes as
 * spark_mha_cross_bwd (no dropout); the workspace additionally holds the accumulator:
 * spark_mha_bwd_atomic_workspace_bytes(...) = two fp32 [B,H,Nq] arrays, padded to 256 bytes, plus
 * fp32 [B,H,Nq,d].  dK and dV are reproducible bit for bit; dQ differs from run to run in its
 * last bits, because the order of the atomic adds is not fixed (several results are correct).
 * Provided for comparison: on MI355X it is the slower variant (the chip retires fp32 atomic adds at
 * about 1.3 TB/s, and every element of dQ receives Nk/128 of them), so spark_mha_bwd and the
 * other entry points use the separate deterministic dQ pass.
 */
size_t spark_mha_bwd_atomic_workspace_bytes(int B, int H, int Nq, int Nk, int d, spark_dtype_t dtype);

int spark_mha_bwd_atomic(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                         const void* dO, void* dQ, void* dK, void* dV,
                         void* workspace, size_t workspace_bytes,
                         int B, int H, int Nq, int Nk, int d, float scale, int causal,
                         spark_dtype_t dtype, void* stream);

/*
 * spark_mha_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same kernels,
 * same results bit for bit as spark_mha_bwd (self-attention, no dropout); the workspace (D and
 * LSE * log2(e), 2 * B*H*N floats) is a fixed array inside the library's device image instead of
 * an argument.  The call allocates and frees nothing and makes no allocating runtime call.
 *   - Limit: B*H*N <= spark_mha_bwd_static_max_rows() (1 Mi rows: 8 MiB of scratch per GPU, held
 *     by each GPU the library runs on until the process ends); larger problems return
 *     SPARK_ERR_WORKSPACE and enqueue nothing.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap in time
 *     (different streams, or several host threads) race on it and must be serialised by the
 *     caller.  Calls on the same stream are ordered and safe.  Nothing in the array needs to
 *     start at zero: every row a call reads was written by that call's first kernel.
 *   - Arguments, layouts and error codes otherwise as for spark_mha_bwd; SPARK_ERR_LAUNCH also if
 *     the runtime cannot resolve the array's device address.
 */
int spark_mha_bwd_static(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                         const void* dO, void* dQ, void* dK, void* dV,
                         int B, int H, int N, int d, float scale, int causal,
                         spark_dtype_t dtype, void* stream);

/* Largest B*H*N spark_mha_bwd_static accepts. */
size_t spark_mha_bwd_static_max_rows(void);

/*
 * Cross-attention forward: Eq. 1 with S = scale * Q K^T of shape Nq x Nk (Sec. 2.1, second
 * attention layer of the decoder); same kernel, arithmetic and guarantees as spark_mha_fwd.
 *   Q       : in,  device, [B,H,Nq,d] dtype
 *   K, V    : in,  device, [B,H,Nk,d] dtype
 *   O       : out, device, [B,H,Nq,d] dtype, fully overwritten
 *   LSE     : out, device, [B,H,Nq] fp32
 */
int spark_mha_cross_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                        int B, int H, int Nq, int Nk, int d, float scale, int causal,
                        spark_dtype_t dtype, void* stream);

/* Workspace bytes of spark_mha_cross_bwd: two fp32 [B,H,Nq] arrays.  0 for invalid shapes. */
size_t spark_mha_cross_bwd_workspace_bytes(int B, int H, int Nq, int Nk, int d,
                                           spark_dtype_t dtype);

/*
 * Cross-attention backward (Sec. 3.3, Eq. 4 with an Nq x Nk score matrix).
 *   Q, O, dO   : in,  device, [B,H,Nq,d] dtype;   K, V : in, device, [B,H,Nk,d] dtype
 *   LSE        : in,  device, [B,H,Nq] fp32 (as written by spark_mha_cross_fwd)
 *   dQ         : out, device, [B,H,Nq,d] dtype;   dK, dV : out, device, [B,H,Nk,d] dtype
 *   workspace  : at least spark_mha_cross_bwd_workspace_bytes(...) bytes, 16-byte aligned
 * Same kernels, order and guarantees as spark_mha_bwd.
 */
int spark_mha_cross_bwd(const void* Q, const void* K, const void* V, const void* O,
                        const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                        void* workspace, size_t workspace_bytes,
                        int B, int H, int Nq, int Nk, int d, float scale, int causal,
                        spark_dtype_t dtype, void* stream);

/*
 * Attention dropout (paper Sec. 4.1: every measurement runs with a dropout rate of 0.1;
 * Sec. 4.2: the backward applies the forward's dropout again so that the two agree).  The paper
 * fixes neither where the mask acts nor how it is drawn; this library drops entries of P after
 * the softmax, independently, and scales the survivors by 1/(1-p):
 *   O = (r M o P) V,  dV = (r M o P)^T dO,  dP = r M o (dO V^T),  dS = P o (dP - D),
 * with LSE unchanged.  The mask is never stored: every kernel regenerates it from
 * (seed, offset).  The decision for (head h = b*H + head index, query i, key j) is
 *   x = Philox4x32-10(counter = (j/4, i/4, h, offset), key = (seed & 0xffffffff, seed >> 32))
 *   u = byte (j mod 4) of x[i mod 4] (byte 0 least significant);  keep iff u >= thr
 * where thr = spark_dropout_threshold(p_drop) = floor(256 p_drop + 1/2): the rate is realised
 * to 8 bits (0.1 -> 26/256), and r = 256 / (256 - thr) matches the realised rate exactly.
 * p_drop must satisfy 0 <= p_drop and thr <= 255, else SPARK_ERR_SHAPE; thr = 0 runs the
 * kernels without dropout.  A forward and its backward must be given the same
 * (p_drop, seed, offset); use a new offset (or seed) for every attention call whose mask
 * should differ.  Everything else is as for spark_mha_cross_fwd / spark_mha_cross_bwd.
 */
int spark_mha_dropout_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          int B, int H, int Nq, int Nk, int d, float scale, int causal,
                          float p_drop, unsigned long long seed, unsigned offset,
                          spark_dtype_t dtype, void* stream);

int spark_mha_dropout_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                          void* workspace, size_t workspace_bytes,
                          int B, int H, int Nq, int Nk, int d, float scale, int causal,
                          float p_drop, unsigned long long seed, unsigned offset,
                          spark_dtype_t dtype, void* stream);

/*
 * spark_mha_dropout_bwd with profiling marks (see spark_mha_bwd_marked): identical work, plus the
 * caller's three HIP events recorded on `stream` before the dQ kernel, after it, and after the
 * dK/dV kernel.
 */
int spark_mha_dropout_bwd_marked(const void* Q, const void* K, const void* V, const void* O,
                                 const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                                 void* workspace, size_t workspace_bytes,
                                 int B, int H, int Nq, int Nk, int d, float scale, int causal,
                                 float p_drop, unsigned long long seed, unsigned offset,
                                 spark_dtype_t dtype, void* stream, void* const events[3]);

/* The 8-bit threshold a dropout rate is realised with (see above), or -1 if p_drop is invalid. */
int spark_dropout_threshold(float p_drop);

/*
 * Writes the keep mask the dropout kernels use, for inspection and testing:
 *   M : out, device, [B,H,Nq,Nk] bytes, 1 = keep, 0 = drop.  No alignment requirement.
 */
int spark_dropout_mask(unsigned char* M, int B, int H, int Nq, int Nk, float p_drop,
                       unsigned long long seed, unsigned offset, void* stream);

/*
 * Strided tensors: the most general forms.  Every [B,H,N,d] tensor gets its own element strides
 * for the batch, head and row (sequence) indices; the d elements of a row stay contiguous.  A
 * projection output laid out [B,N,H,d] is {N*H*d, d, H*d}; the contiguous default of the other
 * entry points is {H*N*d, N*d, d}.  Requirements per tensor: row >= d; batch, head >= 0; all
 * three multiples of 8 elements (16 bytes), else SPARK_ERR_ALIGN; (N + 256) * row * 2 < 2^31 bytes
 * (one head is addressed with 32-bit offsets), else SPARK_ERR_SHAPE; a NULL strides pointer is
 * SPARK_ERR_NULL.  A zero batch or head stride broadcasts an INPUT over that index; for an output
 * (O, dQ, dK, dV) it would make every (batch, head) store to the same rows and is refused with
 * SPARK_ERR_SHAPE when B > 1 (batch) or H > 1 (head).  Other overlaps of output tensors with
 * themselves or anything else are not checked and must not occur.  LSE and the workspace are always
 * contiguous [B,H,Nq].  Cross-attention (Nq, Nk) and dropout (p_drop, seed, offset; p_drop = 0
 * for none) as in the entry points above; same kernels, same guarantees.
 */
typedef struct {
  long long batch, head, row; /* element strides; d is contiguous */
} spark_strides_t;

int spark_mha_strided_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE,
                          const spark_strides_t* sQ, const spark_strides_t* sK,
                          const spark_strides_t* sV, const spark_strides_t* sO,
                          int B, int H, int Nq, int Nk, int d, float scale, int causal,
                          float p_drop, unsigned long long seed, unsigned offset,
                          spark_dtype_t dtype, void* stream);

int spark_mha_strided_bwd(const void* Q, const void* K, const void* V, const void* O,
                          const float* LSE, const void* dO, void* dQ, void* dK, void* dV,
                          const spark_strides_t* sQ, const spark_strides_t* sK,
                          const spark_strides_t* sV, const spark_strides_t* sO,
                          const spark_strides_t* sdO, const spark_strides_t* sdQ,
                          const spark_strides_t* sdK, const spark_strides_t* sdV,
                          void* workspace, size_t workspace_bytes,
                          int B, int H, int Nq, int Nk, int d, float scale, int causal,
                          float p_drop, unsigned long long seed, unsigned offset,
                          spark_dtype_t dtype, void* stream);

/*
 * Hardware self-check of the register layouts the kernels are written against (wave64
 * 32x32x16 MFMA operands and accumulators, packed accumulator registers reused as the operand
 * of a second MFMA -- the register form of the paper's Sec. 3.2.2 layout transform -- and the
 * transposing LDS read).  One wave computes fixed small-integer products through those layouts.
 *   out : out, device, 2304 floats:
 *         [0, 1024)    C1 = A1 B1 (32x32, row-major), A1[i][k] = (37i + 11k + (ik mod 7)) mod 3 - 1
 *                      for k < 16, B1[k][j] = (29k + 13j + (kj mod 5)) mod 5 - 2;
 *         [1024, 2048) C2 = A2 C1, A2[m][r] = (17m + 7r + (mr mod 11)) mod 7 - 3, r < 32;
 *         [2048, 2304) lane l = 16q + i of the wave, words t = 0..3: X[4q + t][16 + i] of the
 *                      tile X[r][c] = 64r + c.
 * All values are exact in both dtypes, so the expected output is exact.  Returns SPARK_OK,
 * SPARK_ERR_NULL, SPARK_ERR_DTYPE or SPARK_ERR_LAUNCH.
 */
int spark_layout_probe(float* out, spark_dtype_t dtype, void* stream);

/* Static, NUL-terminated description of a status code. */
const char* spark_status_str(int status);

#ifdef __cplusplus
}
#endif
#endif /* SPARK_MHA_H_ */
