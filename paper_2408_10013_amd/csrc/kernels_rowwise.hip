// HBM-bound row kernels for bf16 storage, 16 bytes per lane per access: norm forward and
// backward with the row held in registers (each byte of the row is read from memory once),
// and the first stage of the deterministic column reductions (bias / gain / shift gradients).
// Same arithmetic and the same fixed reduction orders as the generic kernels; chosen when the
// width is a multiple of 8 elements, rows are 16-byte aligned and (for the norms) H <= 8192.
#include "dev.h"
#include "kernels.h"
#include "prof.h"

namespace ssdt {
namespace k {

__device__ __forceinline__ void unpack8(const uint4 &v, float *f) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}
__device__ __forceinline__ uint4 pack8(const float *f) {
  return make_uint4(pack_bf2(f[0], f[1]), pack_bf2(f[2], f[3]), pack_bf2(f[4], f[5]), pack_bf2(f[6], f[7]));
}

template <int NCH>
__global__ __launch_bounds__(256) void norm_fwd_vec_k(const uint16_t *x, const uint16_t *gamma, const uint16_t *beta,
                                                      uint16_t *y, float *mean, float *rstd, int rows, int H, float eps,
                                                      int kind) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nch = H >> 3;
  const uint4 *xr = (const uint4 *)(x + (long)row * H);
  uint4 v[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    v[i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
  }
  float mu = 0.f;
  if (kind == SSDT_NORM_LAYERNORM) {
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      float f[8];
      unpack8(v[i], f);
#pragma unroll
      for (int t = 0; t < 8; ++t) sum += f[t];
    }
    mu = wave_sum(sum) / (float)H;
  }
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    if (i * 64 + lane < nch) {
      float f[8];
      unpack8(v[i], f);
#pragma unroll
      for (int t = 0; t < 8; ++t) { float d = f[t] - mu; sq += d * d; }
    }
  }
  const float r = 1.f / sqrtf(wave_sum(sq) / (float)H + eps);
  uint4 *yr = (uint4 *)(y + (long)row * H);
  const uint4 *g4 = (const uint4 *)gamma, *b4 = (const uint4 *)beta;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    if (c < nch) {
      float f[8], g[8], o[8];
      unpack8(v[i], f);
      unpack8(g4[c], g);
#pragma unroll
      for (int t = 0; t < 8; ++t) o[t] = (f[t] - mu) * r * g[t];
      if (beta) {
        float b[8];
        unpack8(b4[c], b);
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] += b[t];
      }
      yr[c] = pack8(o);
    }
  }
  if (lane == 0) {
    if (mean) mean[row] = mu;
    rstd[row] = r;
  }
}

template <int NCH>
__global__ __launch_bounds__(256) void norm_bwd_dx_vec_k(const uint16_t *dy, const uint16_t *x, const float *mean,
                                                         const float *rstd, const uint16_t *gamma, const uint16_t *resid,
                                                         uint16_t *dx, int rows, int H, int kind) {
  // the gain vector is shared by the block's four rows and read twice per row: staged in LDS once (read from global
  // memory chunk by chunk, every one of its 2 x NCH loads was a full round trip in front of the arithmetic)
  __shared__ uint4 g4[NCH * 64];
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int nch = H >> 3;
  for (int c = threadIdx.x; c < nch; c += 256) g4[c] = ((const uint4 *)gamma)[c];
  __syncthreads();
  if (row >= rows) return;
  const uint4 *xr = (const uint4 *)(x + (long)row * H), *dyr = (const uint4 *)(dy + (long)row * H);
  const float mu = (kind == SSDT_NORM_LAYERNORM) ? mean[row] : 0.f, r = rstd[row];
  uint4 vx[NCH], vd[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    vx[i] = c < nch ? xr[c] : make_uint4(0, 0, 0, 0);
    vd[i] = c < nch ? dyr[c] : make_uint4(0, 0, 0, 0);
  }
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    if (c < nch) {
      float fx[8], fd[8], g[8];
      unpack8(vx[i], fx);
      unpack8(vd[i], fd);
      unpack8(g4[c], g);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float dh = fd[t] * g[t], xh = (fx[t] - mu) * r;
        s1 += dh;
        s2 += dh * xh;
      }
    }
  }
  const float c1 = (kind == SSDT_NORM_LAYERNORM) ? wave_sum(s1) / (float)H : 0.f;
  const float c2 = wave_sum(s2) / (float)H;
  uint4 *dxr = (uint4 *)(dx + (long)row * H);
  // the residual-branch gradient: all of its loads go out before the first result is stored (loads issued between
  // stores are waited for one at a time, and this kernel is nothing but memory latency)
  uint4 vr[NCH];
  if (resid) {
    const uint4 *rr = (const uint4 *)(resid + (long)row * H);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = i * 64 + lane;
      vr[i] = c < nch ? rr[c] : make_uint4(0, 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    if (c < nch) {
      float fx[8], fd[8], g[8], o[8];
      unpack8(vx[i], fx);
      unpack8(vd[i], fd);
      unpack8(g4[c], g);
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const float dh = fd[t] * g[t], xh = (fx[t] - mu) * r;
        o[t] = r * (dh - c1 - xh * c2);
      }
      if (resid) {
        float q[8];
        unpack8(vr[i], q);
#pragma unroll
        for (int t = 0; t < 8; ++t) o[t] += q[t];
      }
      vx[i] = pack8(o);
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = i * 64 + lane;
    if (c < nch) dxr[c] = vx[i];
  }
}

// Stage 1 of a column reduction: block (cx, chunk) sums 512 columns over its chunk of rows, the 4
// wavefronts taking every 4th row, then adds the 4 partial sums in a fixed order.
typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
template <bool NORM>
__global__ __launch_bounds__(256) void colreduce1_vec_k(const uint16_t *a, long lda, const uint16_t *x, const float *mean,
                                                        const float *rstd, int kind, float *partial, int rows, int cols,
                                                        int rows_per_chunk) {
  __shared__ float sg[NORM ? 4 : 1][512], sb[4][512];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c0 = blockIdx.x * 512 + lane * 8;
  const int r0 = blockIdx.y * rows_per_chunk, r1 = min(rows, r0 + rows_per_chunk);
  float g[8], b[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) g[t] = b[t] = 0.f;
  if (c0 < cols) {
    for (int r = r0 + w; r < r1; r += 4) {
      float v[8];
      // streamed once, and usually underneath a GEMM on the other stream: keep it out of the L2's way
      const u32x4_nt q = __builtin_nontemporal_load((const u32x4_nt *)(a + (long)r * lda + c0));
      unpack8(make_uint4(q.x, q.y, q.z, q.w), v);
#pragma unroll
      for (int t = 0; t < 8; ++t) b[t] += v[t];
      if (NORM) {
        const float mu = (kind == SSDT_NORM_LAYERNORM) ? mean[r] : 0.f, rs = rstd[r];
        float xv[8];
        unpack8(*(const uint4 *)(x + (long)r * lda + c0), xv);
#pragma unroll
        for (int t = 0; t < 8; ++t) g[t] += v[t] * (xv[t] - mu) * rs;
      }
    }
  }
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    sb[w][lane * 8 + t] = b[t];
    if (NORM) sg[w][lane * 8 + t] = g[t];
  }
  __syncthreads();
  const size_t chunks = gridDim.y;
  for (int i = threadIdx.x; i < 512; i += 256) {
    const int c = blockIdx.x * 512 + i;
    if (c < cols) {
      partial[(size_t)blockIdx.y * cols + c] = ((sb[0][i] + sb[1][i]) + sb[2][i]) + sb[3][i];
      if (NORM) partial[(chunks + blockIdx.y) * cols + c] = ((sg[0][i] + sg[1][i]) + sg[2][i]) + sg[3][i];
    }
  }
}

// delta[b, h, i] = sum_c o[b, i, h, c] dout[b, i, h, c] for bf16 rows that hold the heads side by side (head size a
// power of two between 8 and 512): one wavefront per token walks the row of o and of dout with 16-byte loads
// (d/8 lanes per head), multiplies, and adds the lanes of a head together.
__global__ __launch_bounds__(256) void attn_delta_vec_k(const uint16_t *o, long ldo, const uint16_t *dO, long lddo, float *delta,
                                                        long rows, int Sq, int A, int d) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const long row = (long)blockIdx.x * 4 + w;  // b * Sq + i
  if (row >= rows) return;
  const int b = (int)(row / Sq), i = (int)(row % Sq), H = A * d, lph = d >> 3;
  o += row * ldo;
  dO += row * lddo;
  for (int c = lane * 8; c < H; c += 512) {
    const u32x4_nt a = __builtin_nontemporal_load((const u32x4_nt *)(o + c));
    const uint4 g = *(const uint4 *)(dO + c);  // read again by the backward kernels that follow
    float x[8], y[8];
    unpack8(make_uint4(a.x, a.y, a.z, a.w), x);
    unpack8(g, y);
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) s = fmaf(x[t], y[t], s);
    for (int m = 1; m < lph; m <<= 1) s += __shfl_xor(s, m, 64);
    if ((lane & (lph - 1)) == 0) delta[((long)b * A + c / d) * Sq + i] = s;
  }
}

static int pick_nch(int H) {
  const int need = (H / 8 + 63) / 64;
  for (int n : {1, 2, 4, 8, 16})
    if (need <= n) return n;
  return 0;
}
static bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }

hipError_t norm_fwd_vec(const void *x, const void *gamma, const void *beta, void *y, float *mean, float *rstd, int rows,
                        int H, float eps, int kind, hipStream_t s) {
  const int nch = (H % 8 == 0) ? pick_nch(H) : 0;
  if (!nch || !al16(x) || !al16(y) || !al16(gamma) || (beta && !al16(beta))) return hipErrorNotSupported;
  prof::Scope ps(prof::NORM_FWD, 0, 2.0 * rows * H * 2, s);
  dim3 grid((rows + 3) / 4);
#define SSDT_GO(N) hipLaunchKernelGGL(norm_fwd_vec_k<N>, grid, dim3(256), 0, s, (const uint16_t *)x, (const uint16_t *)gamma, \
                                      (const uint16_t *)beta, (uint16_t *)y, mean, rstd, rows, H, eps, kind)
  switch (nch) { case 1: SSDT_GO(1); break; case 2: SSDT_GO(2); break; case 4: SSDT_GO(4); break; case 8: SSDT_GO(8); break; default: SSDT_GO(16); }
#undef SSDT_GO
  return hipGetLastError();
}

hipError_t norm_bwd_dx_vec(const void *dy, const void *x, const float *mean, const float *rstd, const void *gamma,
                           const void *resid, void *dx, int rows, int H, int kind, hipStream_t s) {
  const int nch = (H % 8 == 0) ? pick_nch(H) : 0;
  if (!nch || !al16(x) || !al16(dy) || !al16(dx) || !al16(gamma) || (resid && !al16(resid))) return hipErrorNotSupported;
  prof::Scope ps(prof::NORM_BWD, 0, (resid ? 4.0 : 3.0) * rows * H * 2, s);
  dim3 grid((rows + 3) / 4);
#define SSDT_GO(N) hipLaunchKernelGGL(norm_bwd_dx_vec_k<N>, grid, dim3(256), 0, s, (const uint16_t *)dy, (const uint16_t *)x, mean, rstd, \
                                      (const uint16_t *)gamma, (const uint16_t *)resid, (uint16_t *)dx, rows, H, kind)
  switch (nch) { case 1: SSDT_GO(1); break; case 2: SSDT_GO(2); break; case 4: SSDT_GO(4); break; case 8: SSDT_GO(8); break; default: SSDT_GO(16); }
#undef SSDT_GO
  return hipGetLastError();
}

hipError_t attn_delta_vec(const void *o, long ldo, const void *dout, long lddo, float *delta, int B, int Sq, int A, int d,
                          hipStream_t s) {
  const int lph = d / 8;
  if (d % 8 || lph < 1 || lph > 64 || (lph & (lph - 1)) || ldo % 8 || lddo % 8 || !al16(o) || !al16(dout)) return hipErrorNotSupported;
  const long rows = (long)B * Sq;
  hipLaunchKernelGGL(attn_delta_vec_k, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, (const uint16_t *)o, ldo,
                     (const uint16_t *)dout, lddo, delta, rows, Sq, A, d);
  return hipGetLastError();
}

hipError_t colreduce1_vec(const void *a, long lda, const void *x, const float *mean, const float *rstd, int kind,
                          float *partial, int rows, int cols, int chunks, bool norm, hipStream_t s) {
  if (cols % 8 || lda % 8 || !al16(a) || (norm && !al16(x))) return hipErrorNotSupported;
  const int rpc = (rows + chunks - 1) / chunks;
  dim3 grid((cols + 511) / 512, chunks);
  if (norm) hipLaunchKernelGGL(colreduce1_vec_k<true>, grid, dim3(256), 0, s, (const uint16_t *)a, lda, (const uint16_t *)x, mean, rstd, kind, partial, rows, cols, rpc);
  else hipLaunchKernelGGL(colreduce1_vec_k<false>, grid, dim3(256), 0, s, (const uint16_t *)a, lda, (const uint16_t *)x, mean, rstd, kind, partial, rows, cols, rpc);
  return hipGetLastError();
}

}  // namespace k
}  // namespace ssdt
