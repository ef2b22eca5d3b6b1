// Internal: launchers of the layer's HIP kernels.  All pointers are device pointers, all
// matrices row-major; element type is float or bf16 (SSDT_F32 / SSDT_BF16) with fp32
// arithmetic and accumulation throughout.  Every reduction runs in a fixed order, so results
// do not depend on addresses or timing.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

#include "ssdt.h"

namespace ssdt {
namespace k {

enum Epi {
  EPI_NONE = 0,    // C = acc
  EPI_BIAS,        // C = acc + bias
  EPI_BIAS_ACT,    // u = acc + bias; C = u (skipped when C is null); C2 = act(u)
  EPI_BIAS_RESID,  // C = acc + bias + resid
  EPI_ACTBWD       // C = acc * act'(aux)   (aux = pre-activation for GELU, activation output for ReLU)
};

// C[M,N] = sum_k A(m,k) B(k,n)   with   A(m,k) = transA ? A[k*lda+m] : A[m*lda+k]
//                                       B(k,n) = transB ? B[n*ldb+k] : B[k*ldb+n]
struct Gemm {
  int M = 0, N = 0, K = 0;
  const void *A = nullptr;
  long lda = 0;
  bool transA = false;
  const void *B = nullptr;
  long ldb = 0;
  bool transB = false;
  void *C = nullptr;
  long ldc = 0;
  int epi = EPI_NONE;
  const void *bias = nullptr;   // [N] or null (then treated as 0)
  const void *resid = nullptr;  // [M, ldr]
  long ldr = 0;
  void *C2 = nullptr;           // [M, ldc]
  const void *aux = nullptr;    // [M, ldc]
  int act = SSDT_ACT_GELU;
  int dtype = SSDT_F32;
  void *colsum = nullptr;       // [N] or null: sum over k of B(k, n), taken from the operand fragments while they pass
                                // through the registers.  Only gemm_mfma_km_bf16 can do this; every other path
                                // returns hipErrorNotSupported (nothing launched) when it is set.
  bool colsum_accumulate = false;  // add to what colsum holds
  void *scratch = nullptr;      // optional: room for transposed copies of operands (bf16 fast path)
  size_t scratch_bytes = 0;
};
hipError_t gemm(const Gemm &g, hipStream_t s);
hipError_t gemm_generic(const Gemm &g, hipStream_t s);  // the FMA kernel, any shape (gemm() falls back to it)
extern int g_force_waves;                               // 0 = choose; > 0 pins the tile rows per workgroup-order group
extern int g_attn_kb;                                   // 0 = choose; 1 pins the register-staged key-side attention backward
extern int g_force_tile;                                // 0 = choose; 128 / 256 pin the matrix-core tile
// scratch bytes gemm() can make use of for this problem (0 for fp32)
// Leading dimension of the K-contiguous scratch copy of a GEMM operand: rows that are a multiple of 32 KiB
// long get 128 bytes of padding (measured 4-6 % on the N = 8192, K = 32768 shapes of the layer, where unpadded
// rows raised the kernel's L2 miss rate from 20 % to 34 %; neutral on the other shapes).
inline long nt_copy_ld(int K) { return ((long)K * 2) % 32768 == 0 ? (long)K + 64 : (long)K; }
size_t gemm_scratch_bytes(int M, int N, int K, bool transA, bool transB, int dtype);
size_t gemm_nt_scratch_bytes(int M, int N, int K, bool transA, bool transB, int dtype);  // gemm_mfma_bf16's own need

// Row norm over H.  kind = SSDT_NORM_*.  mean may be null for RMSNorm.
hipError_t norm_fwd(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int rows,
                    int H, float eps, int kind, int dtype, hipStream_t s);
// dx = (resid ? resid : 0) + norm-backward(dy); dgamma/dbeta by a two-stage column reduction
// through `partial` (fp32, colreduce_partial_floats(rows, H) elements).
hipError_t norm_bwd(const void *dy, const void *x, const float *mean, const float *rstd, const void *gamma,
                    const void *resid, void *dx, void *dgamma, void *dbeta, float *partial, int rows, int H, int kind,
                    int dtype, bool accumulate, hipStream_t s);
// out[n] = sum_m a[m, n]  (bias gradients), same two-stage scheme
hipError_t colsum(const void *a, long lda, void *out, float *partial, int rows, int cols, int dtype, bool accumulate,
                  hipStream_t s);
// w <- w - lr * g, elementwise in fp32, stored in the tensors' type
hipError_t sgd_update(void *w, const void *g, size_t n, float lr, int dtype, hipStream_t s);
size_t colreduce_partial_floats(int rows, int cols);

struct Attn {
  int B = 0, A = 0, Sq = 0, Sk = 0, d = 0;
  float scale = 1.f;
  int mask = SSDT_MASK_NONE;
  const int32_t *kv_len = nullptr;  // [B], key-padding mask only
  int dtype = SSDT_F32;
  const void *q = nullptr, *k = nullptr, *v = nullptr;  // rows b*S + i, head h at columns h*d
  long ldq = 0, ldk = 0, ldv = 0;
  void *o = nullptr;
  long ldo = 0;
  float *lse = nullptr;  // [B, A, Sq]
  // backward only
  const void *dout = nullptr;
  long lddo = 0;
  void *dq = nullptr, *dk = nullptr, *dv = nullptr;
  long lddq = 0, lddk = 0, lddv = 0;
  float *delta = nullptr;  // scratch, 2 x [B, A, Sq] floats (the second half holds lse in base-2 units for the matrix-core backward)
};
hipError_t attn_fwd(const Attn &a, hipStream_t s);
hipError_t attn_bwd(const Attn &a, hipStream_t s);
// the one-wavefront-per-row kernels, any shape (attn_fwd / attn_bwd fall back to them)
hipError_t attn_fwd_generic(const Attn &a, hipStream_t s);
hipError_t attn_bwd_generic(const Attn &a, hipStream_t s);
hipError_t attn_delta(const Attn &a, hipStream_t s);  // delta[b,h,i] = sum_c o[i,c] dout[i,c]

// out[c, r] = in[r, c]
hipError_t transpose(const void *in, long ldi, void *out, long ldo, int rows, int cols, int dtype, hipStream_t s);
// bf16 only: out[c, r] = in[r, c] and sums[c] (+)= sum_r in[r, c] in one pass over `in`; `partial` as for colsum.
// hipErrorNotSupported (nothing launched) when the extents or alignments do not fit the kernel.
hipError_t transpose_colsum(const void *in, long ldi, void *out, long ldo, int rows, int cols, void *sums, float *partial,
                            bool accumulate, hipStream_t s);
// y += x  (elementwise, n elements)
hipError_t add_inplace(void *y, const void *x, size_t n, int dtype, hipStream_t s);

// 16-byte-vectorised bf16 row kernels; return hipErrorNotSupported when the shape / alignment does not fit
hipError_t norm_fwd_vec(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int rows,
                        int H, float eps, int kind, hipStream_t s);
hipError_t norm_bwd_dx_vec(const void *dy, const void *x, const float *mean, const float *rstd, const void *gamma,
                           const void *resid, void *dx, int rows, int H, int kind, hipStream_t s);
hipError_t attn_delta_vec(const void *o, long ldo, const void *dout, long lddo, float *delta, int B, int Sq, int A, int d,
                          hipStream_t s);
hipError_t colreduce1_vec(const void *a, long lda, const void *x, const float *mean, const float *rstd, int kind,
                          float *partial, int rows, int cols, int chunks, bool norm, hipStream_t s);

// fast paths (bf16 on the matrix cores); return hipErrorNotSupported when the shape does not fit
hipError_t gemm_mfma_bf16(const Gemm &g, hipStream_t s);
hipError_t gemm_mfma_km_bf16(const Gemm &g, hipStream_t s);  // reads k-major operands as stored; no scratch
bool gemm_km_fits(int M, int N, int K, bool transA, bool transB, int dtype);  // shape conditions of that kernel
extern int g_km_stagger;  // stages between the K-loop starts of neighbouring XCDs (-100 = by shape)
extern int g_km_pf;       // stages that the L2 prefetch runs ahead (-1 = by shape, 0 = none)
extern int g_km_mode;  // 0 = off, 1 = for problems with a k-major operand (default), 2 = also for the NT form
hipError_t attn_fwd_mfma_bf16(const Attn &a, hipStream_t s);
hipError_t attn_bwd_mfma_bf16(const Attn &a, hipStream_t s);

}  // namespace k
}  // namespace ssdt
