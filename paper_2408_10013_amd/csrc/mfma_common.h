// Shared by the matrix-core GEMM kernels: the kernel argument block, the workgroup-id -> tile map and the
// epilogues (bias, activation, residual, activation derivative) with their staged, 16-byte-wide output path.
#pragma once
#include "dev.h"
#include "kernels.h"

namespace ssdt {
namespace k {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef int v4i_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void_t;

struct NtP {
  int M, N, K;
  const uint16_t *A, *Bt;
  long lda, ldb, ldc, ldr;
  uint16_t *C, *C2;
  const uint16_t *bias, *resid, *aux;
  int act, tiles_m, tiles_n, gm;
  uint16_t *colsum;  // gemm_km256_k: if set, colsum[n] (+)= sum over k of the second operand (k, n), n = 0..N-1
  int colsum_acc;    //               nonzero: added to what colsum holds
  int stagger;  // gemm_km256_k: the workgroups of XCD x start their K loop x * stagger stages in (0 = all at stage 0)
  int pf;       // gemm_km256_k: stages that the L2 prefetch runs ahead of the loads (0 = none)
};

__device__ __forceinline__ void unpack4(uint2 v, float *f) {
  f[0] = bf2f((uint16_t)(v.x & 0xffff)); f[1] = bf2f((uint16_t)(v.x >> 16));
  f[2] = bf2f((uint16_t)(v.y & 0xffff)); f[3] = bf2f((uint16_t)(v.y >> 16));
}
__device__ __forceinline__ uint2 pack4(const float *f) { return make_uint2(pack_bf2(f[0], f[1]), pack_bf2(f[2], f[3])); }

// workgroup id -> tile: compact per XCD, then grouped along M (p.gm tile rows per group)
__device__ __forceinline__ void tile_of(const NtP &p, int pid, int *tile_m, int *tile_n) {
  const int nt = p.tiles_m * p.tiles_n;
  if ((nt & 7) == 0) pid = (pid & 7) * (nt >> 3) + (pid >> 3);
  const int GM = p.gm;
  const int width = GM * p.tiles_n, group = pid / width, first_m = group * GM;
  const int gsz = min(p.tiles_m - first_m, GM);
  *tile_m = first_m + (pid % width) % gsz;
  *tile_n = (pid % width) / gsz;
}

// One 32x32 accumulator block: this lane holds row m and columns n + g*8 + 0..3, g = 0..3
// (n already includes the lane's half offset).
template <int EPI>
__device__ __forceinline__ void epilogue_block(const NtP &p, const f32x16_t &acc, int m, int n) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int nn = n + g * 8;
    float v[4] = {acc[g * 4 + 0], acc[g * 4 + 1], acc[g * 4 + 2], acc[g * 4 + 3]};
    if (EPI != EPI_NONE && EPI != EPI_ACTBWD && p.bias) {
      float b[4];
      unpack4(*(const uint2 *)(p.bias + nn), b);
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] += b[t];
    }
    const long o = (long)m * p.ldc + nn;
    if (EPI == EPI_BIAS_ACT) {
      if (p.C) *(uint2 *)(p.C + o) = pack4(v);
      float a[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) a[t] = p.act == SSDT_ACT_GELU ? gelu_f(v[t]) : fmaxf(v[t], 0.f);
      *(uint2 *)(p.C2 + o) = pack4(a);
    } else if (EPI == EPI_BIAS_RESID) {
      float r[4];
      unpack4(*(const uint2 *)(p.resid + (long)m * p.ldr + nn), r);
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] += r[t];
      *(uint2 *)(p.C + o) = pack4(v);
    } else if (EPI == EPI_ACTBWD) {
      float u[4];
      unpack4(*(const uint2 *)(p.aux + o), u);
#pragma unroll
      for (int t = 0; t < 4; ++t) v[t] *= p.act == SSDT_ACT_GELU ? gelu_grad_f(u[t]) : (u[t] > 0.f ? 1.f : 0.f);
      *(uint2 *)(p.C + o) = pack4(v);
    } else {
      *(uint2 *)(p.C + o) = pack4(v);
    }
  }
}

__device__ __forceinline__ void unpack8f(const uint4 &v, float *f) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xffff0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xffff0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xffff0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xffff0000u);
}

// Epilogue of a 64x64 fp32 sub-tile through LDS: the accumulators are written in MFMA layout and
// read back row-major, so that every global access (bias, residual, activation input, outputs) is
// 16 bytes per lane with 8 lanes covering 128 contiguous bytes of a row.  `st` is this wavefront's
// private 64 x 68 float staging area; m_base / n_base are the sub-tile's origin.
constexpr int kEpiLd = 68;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
// Streaming accesses of the epilogue: every output line is written once and read by a later kernel only after
// far more than an L2's worth of other data, residual and activation inputs are read once.  Marked
// non-temporal they do not displace the operand panels the other workgroups of the XCD are sharing
// (measured: +3-4 % on a whole 32768 x 8192 x 8192 GEMM; the stores alone cost 7 % when left cacheable).
__device__ __forceinline__ void store8_nt(uint16_t *dst, const float *v) {
  const u32x4_t q = {pack_bf2(v[0], v[1]), pack_bf2(v[2], v[3]), pack_bf2(v[4], v[5]), pack_bf2(v[6], v[7])};
  __builtin_nontemporal_store(q, (u32x4_t *)dst);
}
// The residual / activation-input rows of one 64x64 sub-tile (eight row passes), fetched before anything is
// stored: a load issued after a store is waited for together with that store (loads and stores share one
// in-order counter), which made every row pass of those epilogues a full round trip.
template <int EPI>
__device__ __forceinline__ void epilogue_fetch(const NtP &p, int m_base, int n_base, int lane, u32x4_t (&in)[8]) {
  if (EPI != EPI_BIAS_RESID && EPI != EPI_ACTBWD) return;
  const int n = n_base + (lane & 7) * 8;
#pragma unroll
  for (int pass = 0; pass < 8; ++pass) {
    const int m = m_base + pass * 8 + (lane >> 3);
    const uint16_t *src = EPI == EPI_BIAS_RESID ? p.resid + (long)m * p.ldr + n : p.aux + (long)m * p.ldc + n;
    in[pass] = __builtin_nontemporal_load((const u32x4_t *)src);
  }
}

// Second half of the staged epilogue: a 64x64 fp32 sub-tile sits row-major (leading dimension kEpiLd) in this
// wavefront's staging area `st`; apply the epilogue (inputs already in `in`) and store it, 16 bytes per lane per
// access.
template <int EPI>
__device__ __forceinline__ void epilogue_rows(const NtP &p, const float *st, int m_base, int n_base, int lane,
                                              const u32x4_t (&in)[8]) {
  const int col0 = (lane & 7) * 8, n = n_base + col0;
  float b[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) b[t] = 0.f;
  if (EPI != EPI_NONE && EPI != EPI_ACTBWD && p.bias) unpack8f(*(const uint4 *)(p.bias + n), b);
#pragma unroll
  for (int pass = 0; pass < 8; ++pass) {
    const int row = pass * 8 + (lane >> 3), m = m_base + row;
    const float4 lo = *(const float4 *)(st + row * kEpiLd + col0), hi = *(const float4 *)(st + row * kEpiLd + col0 + 4);
    float v[8] = {lo.x + b[0], lo.y + b[1], lo.z + b[2], lo.w + b[3], hi.x + b[4], hi.y + b[5], hi.z + b[6], hi.w + b[7]};
    const long o = (long)m * p.ldc + n;
    if (EPI == EPI_BIAS_ACT) {
      if (p.C) store8_nt(p.C + o, v);
      if (p.act == SSDT_ACT_GELU) {
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = gelu_f(v[t]);
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = fmaxf(v[t], 0.f);
      }
      store8_nt(p.C2 + o, v);
    } else {
      if (EPI == EPI_BIAS_RESID) {
        float r[8];
        unpack8f(make_uint4(in[pass].x, in[pass].y, in[pass].z, in[pass].w), r);
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] += r[t];
      } else if (EPI == EPI_ACTBWD) {
        float u[8];
        unpack8f(make_uint4(in[pass].x, in[pass].y, in[pass].z, in[pass].w), u);
        if (p.act == SSDT_ACT_GELU) {
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] *= gelu_grad_f(u[t]);
        } else {
#pragma unroll
          for (int t = 0; t < 8; ++t) v[t] = u[t] > 0.f ? v[t] : 0.f;
        }
      }
      store8_nt(p.C + o, v);
    }
  }
}

}  // namespace k
}  // namespace ssdt
