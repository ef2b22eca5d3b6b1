// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
// The kernel computes C[M,N] = A[M,K] . Bt[N,K]^T with both operands contiguous along K
// ("NT"), which is the form the MFMA operand registers want (8 consecutive K per lane).
// Other transpositions are brought to this form by a transpose into caller scratch.
//
// Work decomposition: one workgroup of 4 wavefronts per BMxBN tile of C, each wavefront
// owning a (BM/2)x(BN/2) quadrant as a grid of 32x32 MFMA blocks; K is walked in steps of 64
// through a double-buffered LDS tile (rows padded by 16 bytes so that the 128-bit operand
// reads of 16 consecutive lanes fall on distinct banks).  Global loads of step k+1 are issued
// before the MFMAs of step k and written to the other LDS buffer after them, so one barrier
// per step suffices.  The MFMA is issued with the Bt fragment as its first operand, which
// leaves every lane with 4 consecutive columns of one row of C: epilogue traffic is 8-byte.
// Workgroup ids are remapped so that the ids one XCD receives (id mod 8) cover a compact
// block of tiles, and tiles are visited in groups of rows for L2 reuse.
#include "dev.h"
#include "kernels.h"

namespace ssdt {
namespace k {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

struct NtP {
  int M, N, K;
  const uint16_t *A, *Bt;
  long lda, ldb, ldc, ldr;
  uint16_t *C, *C2;
  const uint16_t *bias, *resid, *aux;
  int act, tiles_m, tiles_n;
};

constexpr int kBK = 64;
constexpr int kLDK = kBK + 8;  // padded LDS row, in elements

__device__ __forceinline__ void unpack4(uint2 v, float *f) {
  f[0] = bf2f((uint16_t)(v.x & 0xffff)); f[1] = bf2f((uint16_t)(v.x >> 16));
  f[2] = bf2f((uint16_t)(v.y & 0xffff)); f[3] = bf2f((uint16_t)(v.y >> 16));
}
__device__ __forceinline__ uint2 pack4(const float *f) { return make_uint2(pack_bf2(f[0], f[1]), pack_bf2(f[2], f[3])); }

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_nt_k(NtP p) {
  constexpr int WTM = BM / 2, WTN = BN / 2, TM = WTM / 32, TN = WTN / 32;
  constexpr int CHA = BM * kBK / 8 / 256, CHB = BN * kBK / 8 / 256;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int STAGE = (BM + BN) * kLDK;  // elements per LDS buffer: A tile then B tile

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  // workgroup id -> tile: compact per XCD, then grouped along M
  int pid = blockIdx.x;
  const int nt = p.tiles_m * p.tiles_n;
  if ((nt & 7) == 0) pid = (pid & 7) * (nt >> 3) + (pid >> 3);
  constexpr int GM = 8;
  const int width = GM * p.tiles_n, group = pid / width, first_m = group * GM;
  const int gsz = min(p.tiles_m - first_m, GM);
  const int tile_m = first_m + (pid % width) % gsz, tile_n = (pid % width) / gsz;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const uint16_t *Ag = p.A + (long)m0 * p.lda, *Bg = p.Bt + (long)n0 * p.ldb;
  // each thread moves CHA + CHB 16-byte chunks per K step: chunk c covers row c/8, k-offset (c%8)*8
  const int ld_row = tid >> 3, ld_kc = (tid & 7) * 8;
  const uint16_t *ag = Ag + (long)ld_row * p.lda + ld_kc, *bg = Bg + (long)ld_row * p.ldb + ld_kc;
  const long a_step = 32 * p.lda, b_step = 32 * p.ldb;  // 256 threads cover 32 rows per chunk index
  uint16_t *s_st = smem + ld_row * kLDK + ld_kc;
  uint4 ra[CHA], rb[CHB];
#define SSDT_GLOAD(kt)                                                                   \
  {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < CHA; ++i) ra[i] = *(const uint4 *)(ag + i * a_step + (kt) * kBK); \
    _Pragma("unroll") for (int i = 0; i < CHB; ++i) rb[i] = *(const uint4 *)(bg + i * b_step + (kt) * kBK); \
  }
#define SSDT_SSTORE(buf)                                                                 \
  {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < CHA; ++i) *(uint4 *)(s_st + (buf) * STAGE + i * 32 * kLDK) = ra[i]; \
    _Pragma("unroll") for (int i = 0; i < CHB; ++i) *(uint4 *)(s_st + (buf) * STAGE + BM * kLDK + i * 32 * kLDK) = rb[i]; \
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int frag_off = (lane & 31) * kLDK + (lane >> 5) * 8;
  const uint16_t *a_frag = smem + (wm * WTM) * kLDK + frag_off;
  const uint16_t *b_frag = smem + BM * kLDK + (wn * WTN) * kLDK + frag_off;
#define SSDT_COMPUTE(buf)                                                                \
  {                                                                                      \
    _Pragma("unroll") for (int kk = 0; kk < kBK / 16; ++kk) {                            \
      bf16x8_t af[TM], bfr[TN];                                                          \
      _Pragma("unroll") for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8_t *)(a_frag + (buf) * STAGE + i * 32 * kLDK + kk * 16); \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8_t *)(b_frag + (buf) * STAGE + j * 32 * kLDK + kk * 16); \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                     \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                   \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0); \
    }                                                                                    \
  }

  const int nk = p.K / kBK;
  SSDT_GLOAD(0);
  SSDT_SSTORE(0);
  __syncthreads();
  int cur = 0;
  for (int kt = 1; kt < nk; ++kt) {
    SSDT_GLOAD(kt);
    SSDT_COMPUTE(cur);
    SSDT_SSTORE(cur ^ 1);
    __syncthreads();
    cur ^= 1;
  }
  SSDT_COMPUTE(cur);
#undef SSDT_GLOAD
#undef SSDT_SSTORE
#undef SSDT_COMPUTE

  // epilogue: lane holds row m = (lane & 31), columns n = g*8 + (lane >> 5)*4 + 0..3 of each block
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WTM + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * WTN + j * 32 + g * 8 + (lane >> 5) * 4;
        float v[4] = {acc[i][j][g * 4 + 0], acc[i][j][g * 4 + 1], acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]};
        if (EPI != EPI_NONE && EPI != EPI_ACTBWD && p.bias) {
          float b[4];
          unpack4(*(const uint2 *)(p.bias + n), b);
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] += b[t];
        }
        const long o = (long)m * p.ldc + n;
        if (EPI == EPI_BIAS_ACT) {
          if (p.C) *(uint2 *)(p.C + o) = pack4(v);
          float a[4];
#pragma unroll
          for (int t = 0; t < 4; ++t) a[t] = p.act == SSDT_ACT_GELU ? gelu_f(v[t]) : fmaxf(v[t], 0.f);
          *(uint2 *)(p.C2 + o) = pack4(a);
        } else if (EPI == EPI_BIAS_RESID) {
          float r[4];
          unpack4(*(const uint2 *)(p.resid + (long)m * p.ldr + n), r);
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
  }
}

template <int BM, int BN, int EPI>
static hipError_t launch_nt(const NtP &p, hipStream_t s) {
  constexpr size_t smem = (size_t)2 * (BM + BN) * kLDK * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_nt_k<BM, BN, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_nt_k<BM, BN, EPI>), dim3(p.tiles_m * p.tiles_n), dim3(256), smem, s, p);
  return hipGetLastError();
}

template <int BM, int BN>
static hipError_t launch_nt_epi(int epi, const NtP &p, hipStream_t s) {
  switch (epi) {
    case EPI_NONE: return launch_nt<BM, BN, EPI_NONE>(p, s);
    case EPI_BIAS: return launch_nt<BM, BN, EPI_BIAS>(p, s);
    case EPI_BIAS_ACT: return launch_nt<BM, BN, EPI_BIAS_ACT>(p, s);
    case EPI_BIAS_RESID: return launch_nt<BM, BN, EPI_BIAS_RESID>(p, s);
    case EPI_ACTBWD: return launch_nt<BM, BN, EPI_ACTBWD>(p, s);
  }
  return hipErrorInvalidValue;
}

static inline size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }
static inline bool al8(const void *p) { return ((uintptr_t)p & 7) == 0; }

size_t gemm_scratch_bytes(int M, int N, int K, bool transA, bool transB, int dtype) {
  if (dtype != SSDT_BF16) return 0;
  size_t b = 0;
  if (transA) b += up((size_t)M * K * 2, 256);
  if (!transB) b += up((size_t)N * K * 2, 256);
  return b;
}

int g_force_tile = 0;  // test hook: 0 = choose, 128 or 256

hipError_t gemm_mfma_bf16(const Gemm &g, hipStream_t s) {
  if (g.dtype != SSDT_BF16) return hipErrorNotSupported;
  if (g.M % 128 || g.N % 128 || g.K % kBK) return hipErrorNotSupported;
  if (g.ldc % 4 || !al8(g.C) || (g.C2 && !al8(g.C2)) || (g.bias && !al8(g.bias)) || (g.aux && !al8(g.aux)) ||
      (g.resid && (!al8(g.resid) || g.ldr % 4)))
    return hipErrorNotSupported;
  if (g.epi == EPI_BIAS_ACT && !g.C2) return hipErrorInvalidValue;
  if (g.epi == EPI_BIAS_RESID && !g.resid) return hipErrorInvalidValue;
  if (g.epi == EPI_ACTBWD && !g.aux) return hipErrorInvalidValue;
  size_t need = gemm_scratch_bytes(g.M, g.N, g.K, g.transA, g.transB, g.dtype);
  if (need && (!g.scratch || g.scratch_bytes < need || !al16(g.scratch))) return hipErrorNotSupported;
  const uint16_t *A = (const uint16_t *)g.A, *Bt = (const uint16_t *)g.B;
  long lda = g.lda, ldb = g.ldb;
  char *sc = (char *)g.scratch;
  if (g.transA) {  // stored [K, M] -> [M, K]
    hipError_t e = transpose(g.A, g.lda, sc, g.K, g.K, g.M, SSDT_BF16, s);
    if (e != hipSuccess) return e;
    A = (const uint16_t *)sc;
    lda = g.K;
    sc += up((size_t)g.M * g.K * 2, 256);
  }
  if (!g.transB) {  // stored [K, N] -> [N, K]
    hipError_t e = transpose(g.B, g.ldb, sc, g.K, g.K, g.N, SSDT_BF16, s);
    if (e != hipSuccess) return e;
    Bt = (const uint16_t *)sc;
    ldb = g.K;
  }
  if (!al16(A) || !al16(Bt) || lda % 8 || ldb % 8) return hipErrorNotSupported;
  NtP p{g.M, g.N, g.K, A, Bt, lda, ldb, g.ldc, g.ldr, (uint16_t *)g.C, (uint16_t *)g.C2, (const uint16_t *)g.bias,
        (const uint16_t *)g.resid, (const uint16_t *)g.aux, g.act, 0, 0};
  bool big = (g.M % 256 == 0) && (g.N % 256 == 0) && ((long)(g.M / 256) * (g.N / 256) >= 256);
  if (g_force_tile == 128) big = false;
  if (g_force_tile == 256 && g.M % 256 == 0 && g.N % 256 == 0) big = true;
  if (big) {
    p.tiles_m = g.M / 256; p.tiles_n = g.N / 256;
    return launch_nt_epi<256, 256>(g.epi, p, s);
  }
  p.tiles_m = g.M / 128; p.tiles_n = g.N / 128;
  return launch_nt_epi<128, 128>(g.epi, p, s);
}

}  // namespace k
}  // namespace ssdt
