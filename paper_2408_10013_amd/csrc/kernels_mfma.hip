// bf16 GEMM on the CDNA4 matrix cores, fp32 accumulation.
//
// Both kernels compute C[M,N] = A[M,K] . Bt[N,K]^T with the two operands contiguous along K
// ("NT"), the form the MFMA operand registers want (8 consecutive K per lane).  Other
// transpositions are brought to this form by a transpose into caller scratch.
//
// gemm_nt256_k -- the workhorse, one workgroup of 8 wavefronts per 256x256 tile of C, each
//   wavefront owning 128x64 as 8x4 blocks of v_mfma_f32_16x16x32_bf16 (128 accumulator
//   registers, two wavefronts per SIMD).  That MFMA shape because the part is power-limited: a
//   loop of nothing but MFMAs on random operands sustains about 11 % more FLOP/s (at a higher
//   clock) in it than in 32x32x16.  K is walked in stages of 64 through two 64 KiB LDS buffers
//   filled by direct global-to-LDS loads (no staging registers, no LDS store instructions): a
//   row of a stage is one whole 128-byte cache line, so the L2-to-L1 path moves no byte twice.
//   The 16-byte chunk c of row r is kept at slot c ^ ((r >> 1) & 7), which makes the 128-bit
//   operand reads of 16 consecutive rows fall on distinct banks without padding (the loader
//   applies the permutation on the global side, since a direct load writes LDS linearly by
//   lane).  Loads, LDS reads and all waiting are written out (inline assembly, explicit
//   `s_waitcnt`): see the kernel for the schedule.
// gemm_nt128_k -- 128x128 tiles, 4 wavefronts, v_mfma_f32_32x32x16_bf16, register-staged
//   double-buffered LDS; for problems too small to fill 256 compute units with 256x256 tiles.
//
// The MFMA is issued with the Bt fragment as its first operand, which leaves every lane with 4
// consecutive columns of one row of C.  Workgroup ids are remapped so that the ids one XCD
// receives (id mod 8) cover a compact block of tiles, and tiles are visited in groups of rows,
// for L2 reuse.
#include "dev.h"
#include "kernels.h"
#include "mfma_common.h"
#include "prof.h"

namespace ssdt {
namespace k {

constexpr int kBM2 = 256, kBN2 = 256, kBK2 = 64;
constexpr int kStage2 = (kBM2 + kBN2) * kBK2;  // elements per stage: A rows then Bt rows, 128 bytes each

__device__ __forceinline__ bf16x8_t as_bf(v4i_t v) {
  union { v4i_t a; bf16x8_t b; } u;
  u.a = v;
  return u.b;
}
#define SSDT_DSR(dst, addr, off) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(off))

// ------------------------------------------------------------------------------------------
// 256x256 tile, 8 wavefronts, v_mfma_f32_16x16x32_bf16, two 64-wide LDS stages of direct
// global-to-LDS loads, operand fragments streamed through the registers
// ------------------------------------------------------------------------------------------
// A stage (64 of K for all 512 rows, 64 KiB) is consumed as two 32-wide steps; a wavefront's 128x64 part of
// the tile is 8 blocks of 16 rows of A against 4 blocks of 16 rows of Bt.
//  * The A fragments of a step live in ONE register set that is refilled block by block as soon as the MFMAs
//    of a block have been issued; the Bt fragments live in two sets that alternate per step.  LDS reads are
//    thereby spread evenly over the MFMAs, every fragment is requested a whole step before it is used, and
//    one `s_waitcnt lgkmcnt(11)` in front of a block's MFMAs is all the waiting there is: when block i of a
//    step is about to start, the reads issued after the fragment it needs are always the 7 - i remaining
//    refills of the previous step, the 4 Bt reads at the head of this step and the i refills of this step.
//  * All reads of a stage have been issued by the end of its first step.  The single barrier per stage
//    therefore sits after the first block of the second step (behind an `lgkmcnt(0)`: nobody reads the
//    stage any more); behind it the next stage, whose loads were waited for just before, may be read, and
//    the stage after next is loaded over the current one, two loads per block behind the first MFMAs of
//    blocks 1..4 (measured against one load per block and against four per block: +0.6 % and +1.5 %).
//    Those loads have the rest of the step and the whole first step of the next stage to land.
//  * Loop control is peeled (steady state, second-to-last, last stage), the loads take their base from
//    scalar registers: the steady-state loop contains no vector ALU instruction except four address adds.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
constexpr unsigned kStageBytes2 = kStage2 * 2;

#define SSDT_WAITL(N, X) asm volatile("s_waitcnt lgkmcnt(" #N ")\n\ts_nop 0" : "+v"(X))

template <int EPI>
__global__ __launch_bounds__(512) void gemm_nt256_k(NtP p) {
  constexpr int MB = 8, NB = 4, NT = 512, NWN = 4, LJ = 2048 / NT, RJ = NT / 8;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave / NWN, wn = wave % NWN;
  int tile_m, tile_n;
  tile_of(p, blockIdx.x, &tile_m, &tile_n);
  const int m0 = tile_m * kBM2, n0 = tile_n * kBN2;

  // loader: thread t fills 16-byte positions j*NT + t of A and of Bt, j = 0..LJ-1: row j*RJ + t/8, slot t%8,
  // which holds global chunk (t%8) ^ ((row >> 1) & 7); 8 consecutive lanes fetch one 128-byte line.  A load is
  // `global_load_lds_dwordx4 voff, s[base]`: the base (tile and stage) sits in scalar registers and advances by
  // scalar adds, the per-lane part is a 32-bit byte offset that never changes; M0 (the LDS destination of the
  // wavefront's 1 KiB) is set in the same statement (M0 cannot be named as a clobber; nothing else in this kernel
  // uses it: LDS instructions need no M0 here and there is no other direct-to-LDS load).  No instruction offset
  // on the load: it would be added to the LDS address as well as to the global one.
  const int lrow = tid >> 3, lchunk = (tid & 7) ^ ((lrow >> 1) & 7);
  unsigned voa[LJ], vob[LJ];
#pragma unroll
  for (int j = 0; j < LJ; ++j) {
    voa[j] = (unsigned)((lrow + j * RJ) * (int)p.lda + lchunk * 8) * 2u;
    vob[j] = (unsigned)((lrow + j * RJ) * (int)p.ldb + lchunk * 8) * 2u;
  }
  const char *pa = (const char *)(p.A + (long)m0 * p.lda), *pb = (const char *)(p.Bt + (long)n0 * p.ldb);  // stage 0 of the tile
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  unsigned sb_c = lds0 + wave * 1024;  // LDS byte address of this wavefront's 1 KiB in the current stage's buffer
// a load of the stage PTR points at into the LDS buffer whose wavefront base is SB
#define SSDT_LD(SB, PTR, VOFF, LDSOFF)                                                                     \
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"                         \
               :: "s"(SB), "v"(VOFF), "s"(PTR), "n"(LDSOFF) : "memory", "scc")
#define SSDT_LDA(SB, PA, j) SSDT_LD(SB, PA, voa[j], (j) * NT * 16)
#define SSDT_LDB(SB, PB, j) SSDT_LD(SB, PB, vob[j], kBM2 * kBK2 * 2 + (j) * NT * 16)

  f32x4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int nk = p.K / kBK2;
  SSDT_LDA(sb_c, pa, 0); SSDT_LDB(sb_c, pb, 0); SSDT_LDA(sb_c, pa, 1); SSDT_LDB(sb_c, pb, 1);
  SSDT_LDA(sb_c, pa, 2); SSDT_LDB(sb_c, pb, 2); SSDT_LDA(sb_c, pa, 3); SSDT_LDB(sb_c, pb, 3);
  if (nk > 1) {
    const unsigned sb1 = sb_c + kStageBytes2;
    const char *pa1 = pa + kBK2 * 2, *pb1 = pb + kBK2 * 2;
    SSDT_LDA(sb1, pa1, 0); SSDT_LDB(sb1, pb1, 0); SSDT_LDA(sb1, pa1, 1); SSDT_LDB(sb1, pb1, 1);
    SSDT_LDA(sb1, pa1, 2); SSDT_LDB(sb1, pb1, 2); SSDT_LDA(sb1, pa1, 3); SSDT_LDB(sb1, pb1, 3);
  }
  pa += 2 * kBK2 * 2; pb += 2 * kBK2 * 2;  // from here on: the stage after next

  // fragment addresses: lane l reads row (l & 15) of a 16-row block, 16-byte chunk 4*kk + (l >> 4) of step kk
  const int lr = lane & 15, lq = lane >> 4, lp = lr >> 1;
  const unsigned arow = lds0 + (wm * 128 + lr) * 128, brow = lds0 + kBM2 * 128 + (wn * NB * 16 + lr) * 128;
  // *_n: step 0 of the NEXT stage's buffer, *_c: step 1 of the CURRENT stage's buffer
  unsigned aA_n = arow + ((lq ^ lp) * 16), aB_n = brow + ((lq ^ lp) * 16);
  unsigned aA_c = arow + (((4 | lq) ^ lp) * 16), aB_c = brow + (((4 | lq) ^ lp) * 16);
  v4i_t A0, A1, A2, A3, A4, A5, A6, A7, B[2][NB];

#define SSDT_RDB(SET, addr)                                                                               \
  {                                                                                                       \
    SSDT_DSR(B[SET][0], addr, 0); SSDT_DSR(B[SET][1], addr, 2048); SSDT_DSR(B[SET][2], addr, 4096);       \
    SSDT_DSR(B[SET][3], addr, 6144);                                                                      \
  }
// MFMAs j = J0..J1-1 of block I (row block I of A against Bt set SET), fenced so that nothing moves across
#define SSDT_MF(I, AI, SET, J0, J1)                                                                       \
  {                                                                                                       \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
    _Pragma("unroll") for (int j = J0; j < J1; ++j)                                                       \
      acc[I][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf(B[SET][j]), as_bf(AI), acc[I][j], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                                    \
  }
// Bt set SET must be complete before its first use; tie it to the wait in front of block 0
#define SSDT_TIEB(SET) asm volatile("" : "+v"(B[SET][0]), "+v"(B[SET][1]), "+v"(B[SET][2]), "+v"(B[SET][3]))
// first step of a stage: block I on set 0, then refill AI with the block's fragment of the second step
#define SSDT_EVEN(I, AI)                                                                                  \
  {                                                                                                       \
    SSDT_WAITL(11, AI);                                                                                   \
    if (I == 0) SSDT_TIEB(0);                                                                             \
    SSDT_MF(I, AI, 0, 0, NB);                                                                             \
    SSDT_DSR(AI, aA_c, I * 2048);                                                                         \
  }
// second step, blocks 1..7: block I on set 1 with the loads L0, L1 of the stage after next slotted in behind
// its first MFMAs (a load is three scalar-side instructions, which fit behind one MFMA), then the refill of
// AI from the next stage
#define SSDT_ODD(MORE, MORE2, I, AI, L0, L1)                                                              \
  {                                                                                                       \
    SSDT_MF(I, AI, 1, 0, 1);                                                                              \
    if (MORE2) { L0; }                                                                                    \
    SSDT_MF(I, AI, 1, 1, 2);                                                                              \
    if (MORE2) { L1; }                                                                                    \
    SSDT_MF(I, AI, 1, 2, NB);                                                                             \
    if (MORE) SSDT_DSR(AI, aA_n, I * 2048);                                                               \
  }
// One stage.  MORE / MORE2 (literals): a next stage / a stage after next exists.
#define SSDT_STAGE(MORE, MORE2)                                                                           \
  {                                                                                                       \
    SSDT_RDB(1, aB_c);                                                                                    \
    SSDT_EVEN(0, A0); SSDT_EVEN(1, A1); SSDT_EVEN(2, A2); SSDT_EVEN(3, A3);                               \
    SSDT_EVEN(4, A4); SSDT_EVEN(5, A5); SSDT_EVEN(6, A6); SSDT_EVEN(7, A7);                               \
    SSDT_WAITL(7, A0);                                                                                    \
    SSDT_TIEB(1);                                                                                         \
    SSDT_MF(0, A0, 1, 0, NB);                                                                             \
    /* every read of the current stage has returned to this wavefront */                                  \
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_nop 0" : "+v"(A1), "+v"(A2), "+v"(A3), "+v"(A4), "+v"(A5), "+v"(A6), "+v"(A7)); \
    if (MORE) {                                                                                           \
      __builtin_amdgcn_s_waitcnt(0xF70); /* vmcnt(0): this wavefront's part of the next stage has landed */ \
      __builtin_amdgcn_s_barrier();      /* so has everyone's, and nobody reads the current stage any more */ \
      SSDT_RDB(0, aB_n);                                                                                  \
      SSDT_DSR(A0, aA_n, 0);                                                                              \
    }                                                                                                     \
    SSDT_ODD(MORE, MORE2, 1, A1, SSDT_LDA(sb_c, pa, 0), SSDT_LDB(sb_c, pb, 0));                           \
    SSDT_ODD(MORE, MORE2, 2, A2, SSDT_LDA(sb_c, pa, 1), SSDT_LDB(sb_c, pb, 1));                           \
    SSDT_ODD(MORE, MORE2, 3, A3, SSDT_LDA(sb_c, pa, 2), SSDT_LDB(sb_c, pb, 2));                           \
    SSDT_ODD(MORE, MORE2, 4, A4, SSDT_LDA(sb_c, pa, 3), SSDT_LDB(sb_c, pb, 3));                           \
    SSDT_ODD(MORE, MORE2, 5, A5, , );                                                                     \
    SSDT_ODD(MORE, MORE2, 6, A6, , );                                                                     \
    SSDT_ODD(MORE, MORE2, 7, A7, , );                                                                     \
    aA_c += delta; aB_c += delta; aA_n -= delta; aB_n -= delta; sb_c += delta;                            \
    delta = -delta;                                                                                       \
    pa += kBK2 * 2; pb += kBK2 * 2;                                                                       \
  }

  // vmcnt(2*LJ): stage 0 has landed (stage 1 may still be on its way)
  if (nk > 1) __builtin_amdgcn_s_waitcnt(0xF70 | 8); else __builtin_amdgcn_s_waitcnt(0xF70);
  __builtin_amdgcn_s_barrier();
  SSDT_RDB(0, aB_n);
  SSDT_DSR(A0, aA_n, 0); SSDT_DSR(A1, aA_n, 2048); SSDT_DSR(A2, aA_n, 4096); SSDT_DSR(A3, aA_n, 6144);
  SSDT_DSR(A4, aA_n, 8192); SSDT_DSR(A5, aA_n, 10240); SSDT_DSR(A6, aA_n, 12288); SSDT_DSR(A7, aA_n, 14336);
  aA_n += kStageBytes2; aB_n += kStageBytes2;
  int delta = (int)kStageBytes2, st = 0;
  for (; st + 2 < nk; ++st) SSDT_STAGE(true, true);
  if (st + 1 < nk) SSDT_STAGE(true, false);
  SSDT_STAGE(false, false);
#undef SSDT_LD
#undef SSDT_LDA
#undef SSDT_LDB
#undef SSDT_RDB
#undef SSDT_MF
#undef SSDT_TIEB
#undef SSDT_EVEN
#undef SSDT_ODD
#undef SSDT_STAGE
  // epilogue through LDS (free now), two 64x64 sub-tiles of the wavefront's 128x64: lane l of block (i, j) holds
  // row i*16 + (l & 15), columns j*16 + (l >> 4)*4 + 0..3
  u32x4_t ein[MB / 4][8];  // residual / activation-input rows of both sub-tiles, on their way before the first store
#pragma unroll
  for (int I = 0; I < MB / 4; ++I) epilogue_fetch<EPI>(p, m0 + wm * 128 + I * 64, n0 + wn * 64, lane, ein[I]);
  __builtin_amdgcn_s_barrier();  // every wavefront has finished reading the last stage
  float *stg = (float *)smem + wave * (64 * kEpiLd);
#pragma unroll
  for (int I = 0; I < MB / 4; ++I) {
#pragma unroll
    for (int il = 0; il < 4; ++il)
#pragma unroll
      for (int jl = 0; jl < 4; ++jl) {
        const f32x4_t a = acc[I * 4 + il][jl];
        *(float4 *)(stg + (il * 16 + lr) * kEpiLd + jl * 16 + lq * 4) = make_float4(a[0], a[1], a[2], a[3]);
      }
    epilogue_rows<EPI>(p, stg, m0 + wm * 128 + I * 64, n0 + wn * 64, lane, ein[I]);
  }
}

// ------------------------------------------------------------------------------------------
// 128x128 tile, 4 wavefronts, register-staged double-buffered LDS (rows padded by 16 bytes)
// ------------------------------------------------------------------------------------------
constexpr int kBK = 64;
constexpr int kLDK = kBK + 8;

template <int EPI>
__global__ __launch_bounds__(256) void gemm_nt128_k(NtP p) {
  constexpr int BM = 128, BN = 128, WTM = 64, WTN = 64, TM = 2, TN = 2;
  constexpr int STAGE = (BM + BN) * kLDK;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  int tile_m, tile_n;
  tile_of(p, blockIdx.x, &tile_m, &tile_n);
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  // each thread moves 4 + 4 16-byte chunks per K step: rows ld_row + 32 i, k-offset ld_kc
  const int ld_row = tid >> 3, ld_kc = (tid & 7) * 8;
  const uint16_t *ag = p.A + (long)(m0 + ld_row) * p.lda + ld_kc, *bg = p.Bt + (long)(n0 + ld_row) * p.ldb + ld_kc;
  const long a_step = 32 * p.lda, b_step = 32 * p.ldb;
  uint16_t *s_st = smem + ld_row * kLDK + ld_kc;
  uint4 ra0, ra1, ra2, ra3, rb0, rb1, rb2, rb3;
#define SSDT_GLOAD(kt)                                                                                 \
  {                                                                                                    \
    const long ko_ = (long)(kt) * kBK;                                                                 \
    ra0 = *(const uint4 *)(ag + ko_); ra1 = *(const uint4 *)(ag + a_step + ko_);                       \
    ra2 = *(const uint4 *)(ag + 2 * a_step + ko_); ra3 = *(const uint4 *)(ag + 3 * a_step + ko_);      \
    rb0 = *(const uint4 *)(bg + ko_); rb1 = *(const uint4 *)(bg + b_step + ko_);                       \
    rb2 = *(const uint4 *)(bg + 2 * b_step + ko_); rb3 = *(const uint4 *)(bg + 3 * b_step + ko_);      \
  }
#define SSDT_SSTORE(buf)                                                                               \
  {                                                                                                    \
    uint16_t *d_ = s_st + (buf) * STAGE;                                                               \
    *(uint4 *)(d_) = ra0; *(uint4 *)(d_ + 32 * kLDK) = ra1; *(uint4 *)(d_ + 64 * kLDK) = ra2; *(uint4 *)(d_ + 96 * kLDK) = ra3; \
    d_ += BM * kLDK;                                                                                   \
    *(uint4 *)(d_) = rb0; *(uint4 *)(d_ + 32 * kLDK) = rb1; *(uint4 *)(d_ + 64 * kLDK) = rb2; *(uint4 *)(d_ + 96 * kLDK) = rb3; \
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
#define SSDT_COMPUTE(buf)                                                                              \
  {                                                                                                    \
    _Pragma("unroll") for (int kk = 0; kk < kBK / 16; ++kk) {                                          \
      bf16x8_t af[TM], bfr[TN];                                                                        \
      _Pragma("unroll") for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8_t *)(a_frag + (buf) * STAGE + i * 32 * kLDK + kk * 16); \
      _Pragma("unroll") for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8_t *)(b_frag + (buf) * STAGE + j * 32 * kLDK + kk * 16); \
      _Pragma("unroll") for (int i = 0; i < TM; ++i)                                                   \
        _Pragma("unroll") for (int j = 0; j < TN; ++j)                                                 \
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);      \
    }                                                                                                  \
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
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
      epilogue_block<EPI>(p, acc[i][j], m0 + wm * WTM + i * 32 + (lane & 31), n0 + wn * WTN + j * 32 + (lane >> 5) * 4);
}

template <int EPI>
static hipError_t launch256(const NtP &p, hipStream_t s) {
  constexpr size_t stg = (size_t)8 * 64 * kEpiLd * 4, stages = (size_t)2 * kStage2 * 2, smem = stg > stages ? stg : stages;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_nt256_k<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  prof::Scope ps(prof::GEMM_MFMA_256, 2.0 * p.M * p.N * p.K, 0, s);
  hipLaunchKernelGGL((gemm_nt256_k<EPI>), dim3(p.tiles_m * p.tiles_n), dim3(512), smem, s, p);
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch128(const NtP &p, hipStream_t s) {
  constexpr size_t smem = (size_t)2 * (128 + 128) * kLDK * 2;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_nt128_k<EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  prof::Scope ps(prof::GEMM_MFMA_128, 2.0 * p.M * p.N * p.K, 0, s);
  hipLaunchKernelGGL((gemm_nt128_k<EPI>), dim3(p.tiles_m * p.tiles_n), dim3(256), smem, s, p);
  return hipGetLastError();
}

int g_force_tile = 0;   // test hook: 0 = choose, 128 or 256
int g_force_waves = 0;  // test hook: > 0 pins the tile rows per group of the workgroup order

static hipError_t launch_epi(bool big, int epi, const NtP &p, hipStream_t s) {
#define SSDT_CASE(E) case E: return big ? launch256<E>(p, s) : launch128<E>(p, s);
  switch (epi) {
    SSDT_CASE(EPI_NONE)
    SSDT_CASE(EPI_BIAS)
    SSDT_CASE(EPI_BIAS_ACT)
    SSDT_CASE(EPI_BIAS_RESID)
    SSDT_CASE(EPI_ACTBWD)
  }
#undef SSDT_CASE
  return hipErrorInvalidValue;
}

static inline size_t up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool al16(const void *p) { return ((uintptr_t)p & 15) == 0; }
static inline bool al8(const void *p) { return ((uintptr_t)p & 7) == 0; }

// what gemm_mfma_bf16 itself needs: room for a K-contiguous copy of every operand that is not stored that way
size_t gemm_nt_scratch_bytes(int M, int N, int K, bool transA, bool transB, int dtype) {
  if (dtype != SSDT_BF16) return 0;
  size_t b = 0;
  if (transA) b += up((size_t)M * nt_copy_ld(K) * 2, 256);
  if (!transB) b += up((size_t)N * nt_copy_ld(K) * 2, 256);
  return b;
}
// what gemm() can make use of: nothing where the kernel that reads operands as stored takes the problem
size_t gemm_scratch_bytes(int M, int N, int K, bool transA, bool transB, int dtype) {
  if (gemm_km_fits(M, N, K, transA, transB, dtype)) return 0;
  return gemm_nt_scratch_bytes(M, N, K, transA, transB, dtype);
}


hipError_t gemm_mfma_bf16(const Gemm &g, hipStream_t s) {
  if (g.dtype != SSDT_BF16 || g.colsum) return hipErrorNotSupported;
  if (g.M % 128 || g.N % 128 || g.K % kBK) return hipErrorNotSupported;
  if (g.ldc % 4 || !al8(g.C) || (g.C2 && !al8(g.C2)) || (g.bias && !al8(g.bias)) || (g.aux && !al8(g.aux)) ||
      (g.resid && (!al8(g.resid) || g.ldr % 4)))
    return hipErrorNotSupported;
  if (g.epi == EPI_BIAS_ACT && !g.C2) return hipErrorInvalidValue;
  if (g.epi == EPI_BIAS_RESID && !g.resid) return hipErrorInvalidValue;
  if (g.epi == EPI_ACTBWD && !g.aux) return hipErrorInvalidValue;
  size_t need = gemm_nt_scratch_bytes(g.M, g.N, g.K, g.transA, g.transB, g.dtype);
  if (need && (!g.scratch || g.scratch_bytes < need || !al16(g.scratch))) return hipErrorNotSupported;
  const uint16_t *A = (const uint16_t *)g.A, *Bt = (const uint16_t *)g.B;
  long lda = g.lda, ldb = g.ldb;
  char *sc = (char *)g.scratch;
  const long ldk = nt_copy_ld(g.K);
  if (g.transA) {  // stored [K, M] -> [M, K]
    hipError_t e = transpose(g.A, g.lda, sc, ldk, g.K, g.M, SSDT_BF16, s);
    if (e != hipSuccess) return e;
    A = (const uint16_t *)sc;
    lda = ldk;
    sc += up((size_t)g.M * ldk * 2, 256);
  }
  if (!g.transB) {  // stored [K, N] -> [N, K]
    hipError_t e = transpose(g.B, g.ldb, sc, ldk, g.K, g.N, SSDT_BF16, s);
    if (e != hipSuccess) return e;
    Bt = (const uint16_t *)sc;
    ldb = ldk;
  }
  if (!al16(A) || !al16(Bt) || lda % 8 || ldb % 8) return hipErrorNotSupported;
  NtP p{g.M, g.N, g.K, A, Bt, lda, ldb, g.ldc, g.ldr, (uint16_t *)g.C, (uint16_t *)g.C2, (const uint16_t *)g.bias,
        (const uint16_t *)g.resid, (const uint16_t *)g.aux, g.act, 0, 0, 8, nullptr, 0, 0};
  const bool epi16 = g.ldc % 8 == 0 && al16(g.C) && (!g.C2 || al16(g.C2)) && (!g.bias || al16(g.bias)) &&
                     (!g.aux || al16(g.aux)) && (!g.resid || (al16(g.resid) && g.ldr % 8 == 0));
  // the large-tile kernel addresses a tile's 256 rows with 32-bit byte offsets
  const bool fits256 = epi16 && g.M % 256 == 0 && g.N % 256 == 0 && lda < (1L << 22) && ldb < (1L << 22);
  bool big = fits256 && (long)(g.M / 256) * (g.N / 256) >= 256;
  if (g_force_tile == 128) big = false;
  if (g_force_tile == 256 && fits256) big = true;
  const int t = big ? 256 : 128;
  p.tiles_m = g.M / t;
  p.tiles_n = g.N / t;
  // tile rows per group of the workgroup order: the 32 workgroups an XCD runs side by side then cover 4 x 8 or
  // 8 x 4 tiles; measured 1-5 % apart on the layer's shapes, the better one depends on which extent is longer,
  // and on whether Bt's rows are a multiple of 32 KiB apart (a stored weight that cannot be padded: then fewer
  // Bt panels side by side is better, 1311 -> 1372 TFLOP/s on 32768 x 8192 x 32768)
  p.gm = g_force_waves > 0 ? g_force_waves : ((ldb * 2) % 32768 == 0 ? 8 : (p.tiles_m >= p.tiles_n ? 4 : 8));
  return launch_epi(big, g.epi, p, s);
}

}  // namespace k
}  // namespace ssdt
