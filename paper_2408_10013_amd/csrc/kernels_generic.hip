// Generic kernels of the layer, templated on the storage type (float / bf16), fp32 math.
//
//  - gemm_generic: LDS-tiled FMA matrix multiply for any transposition and any shape; the
//    fp32 path of the layer and the fallback of the bf16 path for shapes the matrix-core
//    kernel does not take.
//  - attn_*_generic: one wavefront per query (or key) row with an online softmax; exact
//    -inf masking; used for fp32 and for head sizes / lengths the fused kernel does not take.
//  - norm forward/backward (one wavefront per row), deterministic two-stage column
//    reductions for bias and gain gradients, transpose, add.
//
// The operations are the textbook definitions of the transformer layer the paper's
// Sec. 2.1 names (attention block, MLP block, norms, residuals).
#include "dev.h"
#include "kernels.h"
#include "prof.h"

namespace ssdt {
namespace k {

#define SSDT_LAUNCH_CHECK() do { hipError_t e_ = hipGetLastError(); if (e_ != hipSuccess) return e_; } while (0)

// ------------------------------------------------------------------------------------------
// GEMM
// ------------------------------------------------------------------------------------------
struct GemmP {
  int M, N, K;
  const void *A, *B;
  void *C, *C2;
  const void *bias, *resid, *aux;
  long lda, ldb, ldc, ldr;
  int transA, transB, epi, act;
};

template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_k(GemmP p) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const T *A = (const T *)p.A, *B = (const T *)p.B;
  int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < p.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = tid + i * 256, m, kk;
      if (!p.transA) { kk = idx & 15; m = idx >> 4; } else { m = idx & 63; kk = idx >> 6; }
      int gm = m0 + m, gk = k0 + kk;
      float v = 0.f;
      if (gm < p.M && gk < p.K) v = ld(A + (p.transA ? (long)gk * p.lda + gm : (long)gm * p.lda + gk));
      As[kk][m] = v;
      int n;
      if (!p.transB) { n = idx & 63; kk = idx >> 6; } else { kk = idx & 15; n = idx >> 4; }
      int gn = n0 + n;
      gk = k0 + kk;
      v = 0.f;
      if (gn < p.N && gk < p.K) v = ld(B + (p.transB ? (long)gn * p.ldb + gk : (long)gk * p.ldb + gn));
      Bs[kk][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  T *C = (T *)p.C, *C2 = (T *)p.C2;
  const T *bias = (const T *)p.bias, *resid = (const T *)p.resid, *aux = (const T *)p.aux;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= p.N) continue;
      float v = acc[i][j];
      if (bias && p.epi != EPI_NONE && p.epi != EPI_ACTBWD) v += ld(bias + n);
      long o = (long)m * p.ldc + n;
      switch (p.epi) {
        case EPI_BIAS_ACT:
          if (C) st(C + o, v);
          st(C2 + o, p.act == SSDT_ACT_GELU ? gelu_f(v) : fmaxf(v, 0.f));
          break;
        case EPI_BIAS_RESID:
          st(C + o, v + ld(resid + (long)m * p.ldr + n));
          break;
        case EPI_ACTBWD: {
          float u = ld(aux + o);
          st(C + o, v * (p.act == SSDT_ACT_GELU ? gelu_grad_f(u) : (u > 0.f ? 1.f : 0.f)));
          break;
        }
        default:
          st(C + o, v);
      }
    }
  }
}

hipError_t gemm_generic(const Gemm &g, hipStream_t s) {
  GemmP p{g.M, g.N, g.K, g.A, g.B, g.C, g.C2, g.bias, g.resid, g.aux, g.lda, g.ldb, g.ldc, g.ldr,
          g.transA, g.transB, g.epi, g.act};
  dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
  prof::Scope ps(prof::GEMM_GENERIC, 2.0 * g.M * g.N * g.K, 0, s);
  if (g.dtype == SSDT_F32) hipLaunchKernelGGL(gemm_generic_k<float>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(gemm_generic_k<bf16>, grid, dim3(256), 0, s, p);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t gemm(const Gemm &g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (g.colsum) return gemm_mfma_km_bf16(g, s);  // the only kernel with that by-product
  if (g.dtype == SSDT_BF16) {
    hipError_t e = gemm_mfma_km_bf16(g, s);  // operands taken as stored, also k-major ones
    if (e != hipErrorNotSupported) return e;
    e = gemm_mfma_bf16(g, s);                // K-contiguous form, other operands through transposed copies
    if (e != hipErrorNotSupported) return e;
  }
  return gemm_generic(g, s);
}

// ------------------------------------------------------------------------------------------
// norms
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void norm_fwd_k(const T *x, const T *gamma, const T *beta, T *y, float *mean,
                                                  float *rstd, int rows, int H, float eps, int kind) {
  int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T *xr = x + (long)row * H;
  float mu = 0.f;
  if (kind == SSDT_NORM_LAYERNORM) {
    float sum = 0.f;
    for (int c = lane; c < H; c += 64) sum += ld(xr + c);
    mu = wave_sum(sum) / (float)H;
  }
  float sq = 0.f;
  for (int c = lane; c < H; c += 64) {
    float dlt = ld(xr + c) - mu;
    sq += dlt * dlt;
  }
  float r = 1.f / sqrtf(wave_sum(sq) / (float)H + eps);
  T *yr = y + (long)row * H;
  for (int c = lane; c < H; c += 64) {
    float v = (ld(xr + c) - mu) * r * ld(gamma + c);
    if (beta) v += ld(beta + c);
    st(yr + c, v);
  }
  if (lane == 0) {
    if (mean) mean[row] = mu;
    rstd[row] = r;
  }
}

hipError_t norm_fwd(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int rows,
                    int H, float eps, int kind, int dtype, hipStream_t s) {
  if (dtype == SSDT_BF16) {
    hipError_t e = norm_fwd_vec(x, gamma, beta, y, mean, rstd, rows, H, eps, kind, s);
    if (e != hipErrorNotSupported) return e;
  }
  dim3 grid((rows + 3) / 4);
  prof::Scope ps(prof::NORM_FWD, 0, 2.0 * rows * H * (dtype == SSDT_F32 ? 4 : 2), s);
  if (dtype == SSDT_F32)
    hipLaunchKernelGGL(norm_fwd_k<float>, grid, dim3(256), 0, s, (const float *)x, (const float *)gamma,
                       (const float *)beta, (float *)y, mean, rstd, rows, H, eps, kind);
  else
    hipLaunchKernelGGL(norm_fwd_k<bf16>, grid, dim3(256), 0, s, (const bf16 *)x, (const bf16 *)gamma,
                       (const bf16 *)beta, (bf16 *)y, mean, rstd, rows, H, eps, kind);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

template <typename T>
__global__ __launch_bounds__(256) void norm_bwd_dx_k(const T *dy, const T *x, const float *mean, const float *rstd,
                                                     const T *gamma, const T *resid, T *dx, int rows, int H, int kind) {
  int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const T *xr = x + (long)row * H, *dyr = dy + (long)row * H;
  float mu = (kind == SSDT_NORM_LAYERNORM) ? mean[row] : 0.f, r = rstd[row];
  float s1 = 0.f, s2 = 0.f;
  for (int c = lane; c < H; c += 64) {
    float dh = ld(dyr + c) * ld(gamma + c);
    float xh = (ld(xr + c) - mu) * r;
    s1 += dh;
    s2 += dh * xh;
  }
  float c1 = (kind == SSDT_NORM_LAYERNORM) ? wave_sum(s1) / (float)H : 0.f;
  float c2 = wave_sum(s2) / (float)H;
  for (int c = lane; c < H; c += 64) {
    float dh = ld(dyr + c) * ld(gamma + c);
    float xh = (ld(xr + c) - mu) * r;
    float v = r * (dh - c1 - xh * c2);
    if (resid) v += ld(resid + (long)row * H + c);
    st(dx + (long)row * H + c, v);
  }
}

static inline int colreduce_chunks(int rows) {
  int c = rows / 128;
  return c < 1 ? 1 : (c > 64 ? 64 : c);
}
size_t colreduce_partial_floats(int rows, int cols) { return (size_t)2 * colreduce_chunks(rows) * cols; }

// Stage 1: block (cx, chunk) sums 128 columns over its chunk of rows.  NORM: g += a*xhat, b += a.
template <typename T, bool NORM>
__global__ __launch_bounds__(256) void colreduce1_k(const T *a, long lda, const T *x, const float *mean,
                                                    const float *rstd, int kind, float *partial, int rows, int cols,
                                                    int rows_per_chunk) {
  __shared__ float sg[4][128], sb[4][128];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int c0 = blockIdx.x * 128 + lane * 2;
  int r0 = blockIdx.y * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);
  float g0 = 0.f, g1 = 0.f, b0 = 0.f, b1 = 0.f;
  for (int r = r0 + w; r < r1; r += 4) {
    float mu = 0.f, rs = 1.f;
    if (NORM) {
      mu = (kind == SSDT_NORM_LAYERNORM) ? mean[r] : 0.f;
      rs = rstd[r];
    }
    if (c0 < cols) {
      float v = ld(a + (long)r * lda + c0);
      b0 += v;
      if (NORM) g0 += v * (ld(x + (long)r * lda + c0) - mu) * rs;
    }
    if (c0 + 1 < cols) {
      float v = ld(a + (long)r * lda + c0 + 1);
      b1 += v;
      if (NORM) g1 += v * (ld(x + (long)r * lda + c0 + 1) - mu) * rs;
    }
  }
  sg[w][lane * 2] = g0; sg[w][lane * 2 + 1] = g1;
  sb[w][lane * 2] = b0; sb[w][lane * 2 + 1] = b1;
  __syncthreads();
  if (threadIdx.x < 128) {
    int c = blockIdx.x * 128 + threadIdx.x;
    if (c < cols) {
      float g = ((sg[0][threadIdx.x] + sg[1][threadIdx.x]) + sg[2][threadIdx.x]) + sg[3][threadIdx.x];
      float b = ((sb[0][threadIdx.x] + sb[1][threadIdx.x]) + sb[2][threadIdx.x]) + sb[3][threadIdx.x];
      size_t chunks = gridDim.y;
      partial[(size_t)blockIdx.y * cols + c] = b;
      if (NORM) partial[(chunks + blockIdx.y) * cols + c] = g;
    }
  }
}

template <typename T>
__global__ void colreduce2_k(const float *partial, int chunks, int cols, T *out_b, T *out_g, int accumulate) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= cols) return;
  float b = 0.f, g = 0.f;
  for (int k = 0; k < chunks; ++k) b += partial[(size_t)k * cols + c];
  if (out_b) st(out_b + c, accumulate ? ld(out_b + c) + b : b);
  if (out_g) {
    for (int k = 0; k < chunks; ++k) g += partial[(size_t)(chunks + k) * cols + c];
    st(out_g + c, accumulate ? ld(out_g + c) + g : g);
  }
}

template <typename T>
static hipError_t colreduce(const T *a, long lda, const T *x, const float *mean, const float *rstd, int kind,
                            T *out_g, T *out_b, float *partial, int rows, int cols, bool norm, bool accumulate,
                            hipStream_t s) {
  int chunks = colreduce_chunks(rows);
  int rpc = (rows + chunks - 1) / chunks;
  dim3 grid((cols + 127) / 128, chunks);
  prof::Scope ps(prof::COLREDUCE, 0, (norm ? 2.0 : 1.0) * rows * cols * sizeof(T), s);
  hipError_t ev = sizeof(T) == 2 ? colreduce1_vec(a, lda, x, mean, rstd, kind, partial, rows, cols, chunks, norm, s) : hipErrorNotSupported;
  if (ev != hipErrorNotSupported && ev != hipSuccess) return ev;
  if (ev == hipErrorNotSupported) {
    if (norm) hipLaunchKernelGGL((colreduce1_k<T, true>), grid, dim3(256), 0, s, a, lda, x, mean, rstd, kind, partial, rows, cols, rpc);
    else hipLaunchKernelGGL((colreduce1_k<T, false>), grid, dim3(256), 0, s, a, lda, x, mean, rstd, kind, partial, rows, cols, rpc);
  }
  SSDT_LAUNCH_CHECK();
  hipLaunchKernelGGL(colreduce2_k<T>, dim3((cols + 255) / 256), dim3(256), 0, s, (const float *)partial, chunks, cols, out_b, out_g,
                     accumulate ? 1 : 0);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t norm_bwd(const void *dy, const void *x, const float *mean, const float *rstd, const void *gamma,
                    const void *resid, void *dx, void *dgamma, void *dbeta, float *partial, int rows, int H, int kind,
                    int dtype, bool accumulate, hipStream_t s) {
  dim3 grid((rows + 3) / 4);
  hipError_t ev = dtype == SSDT_BF16 ? norm_bwd_dx_vec(dy, x, mean, rstd, gamma, resid, dx, rows, H, kind, s) : hipErrorNotSupported;
  if (ev != hipErrorNotSupported && ev != hipSuccess) return ev;
  if (ev == hipErrorNotSupported) {
    prof::Scope ps(prof::NORM_BWD, 0, (resid ? 4.0 : 3.0) * rows * H * (dtype == SSDT_F32 ? 4 : 2), s);
    if (dtype == SSDT_F32)
      hipLaunchKernelGGL(norm_bwd_dx_k<float>, grid, dim3(256), 0, s, (const float *)dy, (const float *)x, mean, rstd,
                         (const float *)gamma, (const float *)resid, (float *)dx, rows, H, kind);
    else
      hipLaunchKernelGGL(norm_bwd_dx_k<bf16>, grid, dim3(256), 0, s, (const bf16 *)dy, (const bf16 *)x, mean, rstd,
                         (const bf16 *)gamma, (const bf16 *)resid, (bf16 *)dx, rows, H, kind);
  }
  SSDT_LAUNCH_CHECK();
  if (dtype == SSDT_F32)
    return colreduce<float>((const float *)dy, H, (const float *)x, mean, rstd, kind, (float *)dgamma, (float *)dbeta,
                            partial, rows, H, true, accumulate, s);
  return colreduce<bf16>((const bf16 *)dy, H, (const bf16 *)x, mean, rstd, kind, (bf16 *)dgamma, (bf16 *)dbeta, partial,
                         rows, H, true, accumulate, s);
}

hipError_t colsum(const void *a, long lda, void *out, float *partial, int rows, int cols, int dtype, bool accumulate,
                  hipStream_t s) {
  if (dtype == SSDT_F32)
    return colreduce<float>((const float *)a, lda, nullptr, nullptr, nullptr, 0, nullptr, (float *)out, partial, rows,
                            cols, false, accumulate, s);
  return colreduce<bf16>((const bf16 *)a, lda, nullptr, nullptr, nullptr, 0, nullptr, (bf16 *)out, partial, rows, cols,
                         false, accumulate, s);
}

// ------------------------------------------------------------------------------------------
// attention, one wavefront per row
// ------------------------------------------------------------------------------------------
struct AttnP {
  int B, A, Sq, Sk, d, mask;
  float scale;
  const int32_t *kv_len;
  const void *q, *k, *v, *dout;
  void *o, *dq, *dk, *dv;
  float *lse, *delta;
  long ldq, ldk, ldv, ldo, lddo, lddq, lddk, lddv;
};

__device__ __forceinline__ int key_limit(const AttnP &p, int b, int i) {
  int lim = p.Sk;
  if (p.mask == SSDT_MASK_CAUSAL) lim = min(lim, i + 1);
  if (p.mask == SSDT_MASK_KEYPAD && p.kv_len) lim = min(lim, max(0, p.kv_len[b]));
  return lim;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_generic_k(AttnP p) {
  __shared__ float sq[4][128];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  bool active = i < p.Sq;
  const T *q = (const T *)p.q + (long)(b * p.Sq + (active ? i : 0)) * p.ldq + h * p.d;
  const T *kb = (const T *)p.k + (long)b * p.Sk * p.ldk + h * p.d;
  const T *vb = (const T *)p.v + (long)b * p.Sk * p.ldv + h * p.d;
  for (int c = lane; c < p.d; c += 64) sq[w][c] = ld(q + c);
  __syncthreads();
  if (!active) return;
  int lim = key_limit(p, b, i);
  float m = -INFINITY, l = 0.f, acc0 = 0.f, acc1 = 0.f;
  for (int j0 = 0; j0 < lim; j0 += 64) {
    int j = j0 + lane;
    float s = -INFINITY;
    if (j < lim) {
      const T *kr = kb + (long)j * p.ldk;
      float dot = 0.f;
      for (int c = 0; c < p.d; ++c) dot = fmaf(sq[w][c], ld(kr + c), dot);
      s = dot * p.scale;
    }
    float mn = fmaxf(m, wave_max(s));
    float pj = (j < lim) ? expf(s - mn) : 0.f;
    float corr = (m == -INFINITY) ? 0.f : expf(m - mn);
    l = l * corr + wave_sum(pj);
    acc0 *= corr;
    acc1 *= corr;
    int cnt = min(64, lim - j0);
    for (int jj = 0; jj < cnt; ++jj) {
      float pp = __shfl(pj, jj, 64);
      const T *vr = vb + (long)(j0 + jj) * p.ldv;
      if (lane < p.d) acc0 = fmaf(pp, ld(vr + lane), acc0);
      if (lane + 64 < p.d) acc1 = fmaf(pp, ld(vr + lane + 64), acc1);
    }
    m = mn;
  }
  T *o = (T *)p.o + (long)(b * p.Sq + i) * p.ldo + h * p.d;
  float inv = l > 0.f ? 1.f / l : 0.f;
  if (lane < p.d) st(o + lane, acc0 * inv);
  if (lane + 64 < p.d) st(o + lane + 64, acc1 * inv);
  if (lane == 0) p.lse[((long)b * p.A + h) * p.Sq + i] = l > 0.f ? m + logf(l) : -INFINITY;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_delta_k(AttnP p) {
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  if (i >= p.Sq) return;
  const T *o = (const T *)p.o + (long)(b * p.Sq + i) * p.ldo + h * p.d;
  const T *dO = (const T *)p.dout + (long)(b * p.Sq + i) * p.lddo + h * p.d;
  float s = 0.f;
  for (int c = lane; c < p.d; c += 64) s += ld(o + c) * ld(dO + c);
  s = wave_sum(s);
  if (lane == 0) p.delta[((long)b * p.A + h) * p.Sq + i] = s;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dq_generic_k(AttnP p) {
  __shared__ float sq[4][128], sdo[4][128];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  bool active = i < p.Sq;
  long row = (long)b * p.Sq + (active ? i : 0);
  const T *q = (const T *)p.q + row * p.ldq + h * p.d;
  const T *dO = (const T *)p.dout + row * p.lddo + h * p.d;
  const T *kb = (const T *)p.k + (long)b * p.Sk * p.ldk + h * p.d;
  const T *vb = (const T *)p.v + (long)b * p.Sk * p.ldv + h * p.d;
  for (int c = lane; c < p.d; c += 64) {
    sq[w][c] = ld(q + c);
    sdo[w][c] = ld(dO + c);
  }
  __syncthreads();
  if (!active) return;
  int lim = key_limit(p, b, i);
  long si = ((long)b * p.A + h) * p.Sq + i;
  float lse = p.lse[si], dl = p.delta[si];
  float acc0 = 0.f, acc1 = 0.f;
  for (int j0 = 0; j0 < lim; j0 += 64) {
    int j = j0 + lane;
    float ds = 0.f;
    if (j < lim && lse != -INFINITY) {
      const T *kr = kb + (long)j * p.ldk, *vr = vb + (long)j * p.ldv;
      float dot = 0.f, dp = 0.f;
      for (int c = 0; c < p.d; ++c) {
        dot = fmaf(sq[w][c], ld(kr + c), dot);
        dp = fmaf(sdo[w][c], ld(vr + c), dp);
      }
      ds = expf(dot * p.scale - lse) * (dp - dl);
    }
    int cnt = min(64, lim - j0);
    for (int jj = 0; jj < cnt; ++jj) {
      float dd = __shfl(ds, jj, 64);
      const T *kr = kb + (long)(j0 + jj) * p.ldk;
      if (lane < p.d) acc0 = fmaf(dd, ld(kr + lane), acc0);
      if (lane + 64 < p.d) acc1 = fmaf(dd, ld(kr + lane + 64), acc1);
    }
  }
  T *dq = (T *)p.dq + row * p.lddq + h * p.d;
  if (lane < p.d) st(dq + lane, acc0 * p.scale);
  if (lane + 64 < p.d) st(dq + lane + 64, acc1 * p.scale);
}

template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_dkv_generic_k(AttnP p) {
  __shared__ float sk[4][128], sv[4][128];
  int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int j = blockIdx.x * 4 + w, h = blockIdx.y, b = blockIdx.z;
  bool active = j < p.Sk;
  long row = (long)b * p.Sk + (active ? j : 0);
  const T *kr = (const T *)p.k + row * p.ldk + h * p.d;
  const T *vr = (const T *)p.v + row * p.ldv + h * p.d;
  for (int c = lane; c < p.d; c += 64) {
    sk[w][c] = ld(kr + c);
    sv[w][c] = ld(vr + c);
  }
  __syncthreads();
  if (!active) return;
  bool key_valid = !(p.mask == SSDT_MASK_KEYPAD && p.kv_len && j >= p.kv_len[b]);
  int istart = (p.mask == SSDT_MASK_CAUSAL) ? j : 0;
  float dk0 = 0.f, dk1 = 0.f, dv0 = 0.f, dv1 = 0.f;
  const T *qb = (const T *)p.q + (long)b * p.Sq * p.ldq + h * p.d;
  const T *dob = (const T *)p.dout + (long)b * p.Sq * p.lddo + h * p.d;
  if (key_valid) {
    for (int i0 = istart; i0 < p.Sq; i0 += 64) {
      int i = i0 + lane;
      float pp = 0.f, ds = 0.f;
      if (i < p.Sq) {
        long si = ((long)b * p.A + h) * p.Sq + i;
        float lse = p.lse[si];
        if (lse != -INFINITY) {
          const T *qr = qb + (long)i * p.ldq, *dr = dob + (long)i * p.lddo;
          float dot = 0.f, dp = 0.f;
          for (int c = 0; c < p.d; ++c) {
            dot = fmaf(ld(qr + c), sk[w][c], dot);
            dp = fmaf(ld(dr + c), sv[w][c], dp);
          }
          pp = expf(dot * p.scale - lse);
          ds = pp * (dp - p.delta[si]);
        }
      }
      int cnt = min(64, p.Sq - i0);
      for (int ii = 0; ii < cnt; ++ii) {
        float p1 = __shfl(pp, ii, 64), d1 = __shfl(ds, ii, 64);
        const T *qr = qb + (long)(i0 + ii) * p.ldq, *dr = dob + (long)(i0 + ii) * p.lddo;
        if (lane < p.d) {
          dv0 = fmaf(p1, ld(dr + lane), dv0);
          dk0 = fmaf(d1, ld(qr + lane), dk0);
        }
        if (lane + 64 < p.d) {
          dv1 = fmaf(p1, ld(dr + lane + 64), dv1);
          dk1 = fmaf(d1, ld(qr + lane + 64), dk1);
        }
      }
    }
  }
  T *dk = (T *)p.dk + row * p.lddk + h * p.d, *dv = (T *)p.dv + row * p.lddv + h * p.d;
  if (lane < p.d) {
    st(dk + lane, dk0 * p.scale);
    st(dv + lane, dv0);
  }
  if (lane + 64 < p.d) {
    st(dk + lane + 64, dk1 * p.scale);
    st(dv + lane + 64, dv1);
  }
}

static AttnP to_p(const Attn &a) {
  return AttnP{a.B, a.A, a.Sq, a.Sk, a.d, a.mask, a.scale, a.kv_len, a.q, a.k, a.v, a.dout, a.o, a.dq, a.dk, a.dv,
               a.lse, a.delta, a.ldq, a.ldk, a.ldv, a.ldo, a.lddo, a.lddq, a.lddk, a.lddv};
}

hipError_t attn_fwd(const Attn &a, hipStream_t s) {
  if (a.d > 128 || a.d <= 0) return hipErrorInvalidValue;
  if (a.mask == SSDT_MASK_CAUSAL && a.Sq != a.Sk) return hipErrorInvalidValue;
  if (a.dtype == SSDT_BF16) {
    hipError_t e = attn_fwd_mfma_bf16(a, s);
    if (e != hipErrorNotSupported) return e;
  }
  return attn_fwd_generic(a, s);
}

static double attn_flops(const Attn &a) {
  return 4.0 * a.B * a.A * (double)a.Sq * a.Sk * a.d * (a.mask == SSDT_MASK_CAUSAL ? 0.5 : 1.0);
}

hipError_t attn_fwd_generic(const Attn &a, hipStream_t s) {
  prof::Scope ps(prof::ATTN_FWD, attn_flops(a), 0, s);
  AttnP p = to_p(a);
  dim3 grid((a.Sq + 3) / 4, a.A, a.B);
  if (a.dtype == SSDT_F32) hipLaunchKernelGGL(attn_fwd_generic_k<float>, grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(attn_fwd_generic_k<bf16>, grid, dim3(256), 0, s, p);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t attn_bwd(const Attn &a, hipStream_t s) {
  if (a.d > 128 || a.d <= 0 || !a.delta) return hipErrorInvalidValue;
  if (a.mask == SSDT_MASK_CAUSAL && a.Sq != a.Sk) return hipErrorInvalidValue;
  if (a.dtype == SSDT_BF16) {
    hipError_t e = attn_bwd_mfma_bf16(a, s);
    if (e != hipErrorNotSupported) return e;
  }
  return attn_bwd_generic(a, s);
}

hipError_t attn_delta(const Attn &a, hipStream_t s) {
  AttnP p = to_p(a);
  if (a.dtype == SSDT_BF16) {
    hipError_t e = attn_delta_vec(a.o, a.ldo, a.dout, a.lddo, a.delta, a.B, a.Sq, a.A, a.d, s);
    if (e != hipErrorNotSupported) return e;
  }
  dim3 gq((a.Sq + 3) / 4, a.A, a.B);
  if (a.dtype == SSDT_F32) hipLaunchKernelGGL(attn_delta_k<float>, gq, dim3(256), 0, s, p);
  else hipLaunchKernelGGL(attn_delta_k<bf16>, gq, dim3(256), 0, s, p);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t attn_bwd_generic(const Attn &a, hipStream_t s) {
  prof::Scope ps(prof::ATTN_BWD, 2 * attn_flops(a), 0, s);
  AttnP p = to_p(a);
  dim3 gq((a.Sq + 3) / 4, a.A, a.B), gk((a.Sk + 3) / 4, a.A, a.B);
  if (a.dtype == SSDT_F32) {
    hipLaunchKernelGGL(attn_delta_k<float>, gq, dim3(256), 0, s, p);
    hipLaunchKernelGGL(attn_bwd_dq_generic_k<float>, gq, dim3(256), 0, s, p);
    hipLaunchKernelGGL(attn_bwd_dkv_generic_k<float>, gk, dim3(256), 0, s, p);
  } else {
    hipLaunchKernelGGL(attn_delta_k<bf16>, gq, dim3(256), 0, s, p);
    hipLaunchKernelGGL(attn_bwd_dq_generic_k<bf16>, gq, dim3(256), 0, s, p);
    hipLaunchKernelGGL(attn_bwd_dkv_generic_k<bf16>, gk, dim3(256), 0, s, p);
  }
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

// ------------------------------------------------------------------------------------------
// transpose, add
// ------------------------------------------------------------------------------------------
template <typename U>
__global__ __launch_bounds__(256) void transpose_k(const U *in, long ldi, U *out, long ldo, int rows, int cols) {
  __shared__ U tile[64][65];
  int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  for (int r = ty; r < 64; r += 4)
    if (r0 + r < rows && c0 + tx < cols) tile[r][tx] = in[(long)(r0 + r) * ldi + c0 + tx];
  __syncthreads();
  for (int c = ty; c < 64; c += 4)
    if (c0 + c < cols && r0 + tx < rows) out[(long)(c0 + c) * ldo + r0 + tx] = tile[tx][c];
}

// 16-bit elements, extents multiples of 64, 16-byte aligned rows: each wavefront moves a 64x64 tile with
// 16-byte accesses only and no LDS.  Lane (rb, cb) = (lane / 8, lane % 8) reads the 8x8 block at rows
// 8 rb.., columns 8 cb.. (eight lanes cover one 128-byte line of each row), transposes it in registers and
// writes it as rows 8 cb.., columns 8 rb.. of the output (again eight lanes per 128-byte line).
typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
__global__ __launch_bounds__(256) void transpose16_k(const uint16_t *in, long ldi, uint16_t *out, long ldo, int rows, int cols) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r0 = (blockIdx.y * 2 + (wave >> 1)) * 64, c0 = (blockIdx.x * 2 + (wave & 1)) * 64;
  if (r0 >= rows || c0 >= cols) return;
  const int rb = lane >> 3, cb = lane & 7;
  const uint16_t *src = in + (long)(r0 + rb * 8) * ldi + c0 + cb * 8;
  uint32_t v[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const u32x4_nt q = __builtin_nontemporal_load((const u32x4_nt *)(src + i * ldi));
    v[i][0] = q.x; v[i][1] = q.y; v[i][2] = q.z; v[i][3] = q.w;
  }
  uint16_t *dst = out + (long)(c0 + cb * 8) * ldo + r0 + rb * 8;
#pragma unroll
  for (int j = 0; j < 8; ++j) {  // output row j of the block = column j of the input block
    uint32_t o[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint32_t a = v[2 * k][j >> 1], b = v[2 * k + 1][j >> 1];
      o[k] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
    }
    const u32x4_nt w = {o[0], o[1], o[2], o[3]};
    __builtin_nontemporal_store(w, (u32x4_nt *)(dst + j * ldo));
  }
}

// The transposed copy and the column sums of a bf16 matrix in one pass over it (the weight-gradient product needs
// dY transposed, the bias gradient is dY's column sums): a wavefront walks a 64-column strip of one row chunk in
// 64x64 tiles, moving each tile as transpose16_k does and adding its rows into eight per-lane column sums; the next
// tile's loads are issued before the current tile's stores, so that waiting for them never waits for a store.  At
// the end the eight lanes that share a column block are added in a fixed order and the chunk's sums go to
// partial[chunk][column] (stage 2 of the column reduction finishes the job).
__global__ __launch_bounds__(256) void transpose_colsum16_k(const uint16_t *in, long ldi, uint16_t *out, long ldo, int rows,
                                                            int cols, float *partial, int rows_per_chunk) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c0 = (blockIdx.x * 4 + wave) * 64;
  if (c0 >= cols) return;
  const int rb = lane >> 3, cb = lane & 7;
  const int r_begin = blockIdx.y * rows_per_chunk, r_end = min(rows, r_begin + rows_per_chunk);
  float acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) acc[j] = 0.f;
  u32x4_nt v[8], nv[8];
  const uint16_t *src = in + (long)(r_begin + rb * 8) * ldi + c0 + cb * 8;
  if (r_begin < r_end) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_nontemporal_load((const u32x4_nt *)(src + i * ldi));
  }
  for (int r0 = r_begin; r0 < r_end; r0 += 64) {
    src += 64 * ldi;
    if (r0 + 64 < r_end) {
#pragma unroll
      for (int i = 0; i < 8; ++i) nv[i] = __builtin_nontemporal_load((const u32x4_nt *)(src + i * ldi));
    }
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] += __uint_as_float(v[i][k] << 16);
        acc[2 * k + 1] += __uint_as_float(v[i][k] & 0xffff0000u);
      }
    uint16_t *dst = out + (long)(c0 + cb * 8) * ldo + r0 + rb * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t a = v[2 * k][j >> 1], b = v[2 * k + 1][j >> 1];
        o[k] = (j & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
      }
      const u32x4_nt w = {o[0], o[1], o[2], o[3]};
      __builtin_nontemporal_store(w, (u32x4_nt *)(dst + j * ldo));
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = nv[i];
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    acc[j] += __shfl_xor(acc[j], 8, 64);
    acc[j] += __shfl_xor(acc[j], 16, 64);
    acc[j] += __shfl_xor(acc[j], 32, 64);
  }
  if (rb == 0) {
    float *dst = partial + (size_t)blockIdx.y * cols + c0 + cb * 8;
    *(float4 *)dst = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *(float4 *)(dst + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
}

hipError_t transpose_colsum(const void *in, long ldi, void *out, long ldo, int rows, int cols, void *sums, float *partial,
                            bool accumulate, hipStream_t s) {
  const int chunks = colreduce_chunks(rows);
  if (rows % 64 || cols % 64 || ldi % 8 || ldo % 8 || ((uintptr_t)in | (uintptr_t)out | (uintptr_t)partial) % 16 || rows % chunks ||
      (rows / chunks) % 64)
    return hipErrorNotSupported;
  {
    prof::Scope ps(prof::TRANSPOSE, 0, 2.0 * rows * cols * 2, s);
    hipLaunchKernelGGL(transpose_colsum16_k, dim3((cols / 64 + 3) / 4, chunks), dim3(256), 0, s, (const uint16_t *)in, ldi,
                       (uint16_t *)out, ldo, rows, cols, partial, rows / chunks);
    SSDT_LAUNCH_CHECK();
  }
  prof::Scope ps(prof::COLREDUCE, 0, 4.0 * chunks * cols, s);
  hipLaunchKernelGGL(colreduce2_k<bf16>, dim3((cols + 255) / 256), dim3(256), 0, s, (const float *)partial, chunks, cols,
                     (bf16 *)sums, (bf16 *)nullptr, accumulate ? 1 : 0);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

hipError_t transpose(const void *in, long ldi, void *out, long ldo, int rows, int cols, int dtype, hipStream_t s) {
  dim3 grid((cols + 63) / 64, (rows + 63) / 64);
  prof::Scope ps(prof::TRANSPOSE, 0, 2.0 * rows * cols * (dtype == SSDT_F32 ? 4 : 2), s);
  if (dtype != SSDT_F32 && rows % 64 == 0 && cols % 64 == 0 && ldi % 8 == 0 && ldo % 8 == 0 &&
      ((uintptr_t)in | (uintptr_t)out) % 16 == 0) {
    hipLaunchKernelGGL(transpose16_k, dim3((cols + 127) / 128, (rows + 127) / 128), dim3(256), 0, s, (const uint16_t *)in, ldi,
                       (uint16_t *)out, ldo, rows, cols);
    SSDT_LAUNCH_CHECK();
    return hipSuccess;
  }
  if (dtype == SSDT_F32)
    hipLaunchKernelGGL(transpose_k<uint32_t>, grid, dim3(256), 0, s, (const uint32_t *)in, ldi, (uint32_t *)out, ldo, rows, cols);
  else
    hipLaunchKernelGGL(transpose_k<uint16_t>, grid, dim3(256), 0, s, (const uint16_t *)in, ldi, (uint16_t *)out, ldo, rows, cols);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

template <typename T>
__global__ void sgd_update_k(T *w, const T *g, size_t n, float lr) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) st(w + i, fmaf(-lr, ld(g + i), ld(w + i)));
}
// bf16, 16 bytes per access
__global__ void sgd_update_bf16x8_k(uint4 *w, const uint4 *g, size_t n8, float lr) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n8; i += stride) {
    uint4 a = w[i];
    const uint4 b = g[i];
    uint32_t *pa = (uint32_t *)&a;
    const uint32_t *pb = (const uint32_t *)&b;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const float w0 = bf2f((uint16_t)(pa[t] & 0xffff)), w1 = bf2f((uint16_t)(pa[t] >> 16));
      const float g0 = bf2f((uint16_t)(pb[t] & 0xffff)), g1 = bf2f((uint16_t)(pb[t] >> 16));
      pa[t] = pack_bf2(fmaf(-lr, g0, w0), fmaf(-lr, g1, w1));
    }
    w[i] = a;
  }
}

hipError_t sgd_update(void *w, const void *g, size_t n, float lr, int dtype, hipStream_t s) {
  if (n == 0) return hipSuccess;
  prof::Scope ps(prof::ADD, 0, 3.0 * n * (dtype == SSDT_F32 ? 4 : 2), s);
  if (dtype == SSDT_BF16 && n % 8 == 0 && (((uintptr_t)w | (uintptr_t)g) & 15) == 0) {
    size_t blocks = std::min<size_t>((n / 8 + 255) / 256, 16384);
    hipLaunchKernelGGL(sgd_update_bf16x8_k, dim3((unsigned)blocks), dim3(256), 0, s, (uint4 *)w, (const uint4 *)g, n / 8, lr);
  } else {
    size_t blocks = std::min<size_t>((n + 255) / 256, 65536);
    if (dtype == SSDT_F32) hipLaunchKernelGGL(sgd_update_k<float>, dim3((unsigned)blocks), dim3(256), 0, s, (float *)w, (const float *)g, n, lr);
    else hipLaunchKernelGGL(sgd_update_k<bf16>, dim3((unsigned)blocks), dim3(256), 0, s, (bf16 *)w, (const bf16 *)g, n, lr);
  }
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

template <typename T>
__global__ void add_inplace_k(T *y, const T *x, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) st(y + i, ld(y + i) + ld(x + i));
}

hipError_t add_inplace(void *y, const void *x, size_t n, int dtype, hipStream_t s) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  if (blocks == 0) return hipSuccess;
  prof::Scope ps(prof::ADD, 0, 3.0 * n * (dtype == SSDT_F32 ? 4 : 2), s);
  if (dtype == SSDT_F32) hipLaunchKernelGGL(add_inplace_k<float>, dim3((unsigned)blocks), dim3(256), 0, s, (float *)y, (const float *)x, n);
  else hipLaunchKernelGGL(add_inplace_k<bf16>, dim3((unsigned)blocks), dim3(256), 0, s, (bf16 *)y, (const bf16 *)x, n);
  SSDT_LAUNCH_CHECK();
  return hipSuccess;
}

}  // namespace k
}  // namespace ssdt
