// bf16 GEMM on the CDNA4 matrix cores for operands that are contiguous along the OTHER dimension
// ("k-major": element (k, i) at k * ld + i), fp32 accumulation.
//
// The layer stores weights as [in, out] and activations as [tokens, features].  The forward
// product x W therefore has its second operand k-major, and the weight gradient in^T dY has both
// operands k-major (the contraction runs over tokens).  The MFMA wants 8 consecutive k per lane;
// gemm_nt256_k gets them with one 128-bit LDS read from K-contiguous rows, and k-major operands
// used to be brought to that form by a transpose into scratch memory first.  This kernel reads
// k-major operands as they are: a stage of 64 k-rows x 256 columns goes to LDS by direct
// global-to-LDS loads (a row of the stage is 512 contiguous bytes), and the operand fragments are
// fetched with the transposing LDS read ds_read_b64_tr_b16, two per fragment: a group of 16 lanes
// reads a block of 4 k-rows x 16 columns and every lane receives one column's 4 values.
//
// Same tile shape, wavefront layout, accumulator layout, epilogues and workgroup order as
// gemm_nt256_k (256 x 256 per workgroup of 8 wavefronts, each 128 x 64 as 8 x 4 blocks of
// v_mfma_f32_16x16x32_bf16), so the two kernels give bit-identical results on transposed copies of
// the same data.  Differences:
//   * LDS holds [A buffer 0 | A buffer 1 | B buffer 0 | B buffer 1], 32 KiB each, and the stage loop
//     is unrolled by two, so that every LDS address is a per-lane constant plus an instruction
//     offset (below 64 KiB) and no address is updated in the loop.
//   * A k-major row of 512 bytes is kept with its 32-byte units permuted: unit u of k-row k sits at
//     u ^ ((k & 3) | ((k >> 3) & 1) << 2).  One transposing read has its first 32 lanes on k-rows
//     {0..3, 8..11} (or {4..7, 12..15}) of a 16-row group at one column unit; the key sends those
//     eight rows to eight different 32-byte bank groups.  The key of the row a lane reads depends on
//     the lane only, so each 16-column block has its own address register.
//   * LDS reads are compiler-visible (no inline assembly): the compiler computes every
//     `s_waitcnt lgkmcnt` from the program order, which scheduling fences pin to the order written
//     here.  The direct-to-LDS loads and the barrier are still written out, with `vmcnt` waits by hand.
//   * Only wavefronts 4-7 load (a stage's 16 instructions in one burst behind the barrier), no two LDS
//     reads are issued back to back, and instantiations for long K end the burst with an L2 prefetch
//     (see the loader and the two halves of the stage below).
#include "dev.h"
#include "kernels.h"
#include "mfma_common.h"
#include "prof.h"

namespace ssdt {
namespace k {

typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) v4i_t lds_v4i_t;
typedef __attribute__((address_space(3))) char lds_char_t;

constexpr int kTile = 256, kStageK = 64;
constexpr unsigned kBuf = 32768;            // one operand's stage: 256 x 64 bf16 either way round
constexpr unsigned kLdsB = 2 * kBuf;        // B buffers behind the two A buffers

#define SSDT_FENCE __builtin_amdgcn_sched_barrier(0)

// 8 bf16 of an MFMA operand from a k-major stage: `at` addresses this lane's 8 bytes of k-row group 0 of the
// 16-column block, `off` selects buffer and 32-wide step; the second read is 4 k-rows (4 x 512 bytes) further.
__device__ __forceinline__ bf16x8_t frag_km(const lds_char_t *at, unsigned off) {
  const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(at + off));
  const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(at + off + 2048));
  union { struct { s16x4_t a, b; } s; bf16x8_t v; } u;
  u.s.a = lo;
  u.s.b = hi;
  return u.v;
}
// the same from a K-contiguous stage (rows of 128 bytes, 16-byte chunks swizzled as in gemm_nt256_k)
__device__ __forceinline__ bf16x8_t frag_nt(const lds_char_t *at, unsigned off) {
  union { v4i_t a; bf16x8_t v; } u;
  u.a = *(const lds_v4i_t *)(at + off);
  return u.v;
}

// W = wavefronts per workgroup: 8, each 128 x 64 of the tile, two per SIMD.  (A form with 4, each 128 x 128 with the
// accumulators in the AGPRs and the loads issued one by one between the MFMAs, a third fewer LDS reads per MFMA, ran
// within 1 % of this one on every shape, alone and in the layer, in both generations of this kernel: not built.)
template <int EPI, bool AKM, bool BKM, int W, bool CS, bool PF>
__global__ __launch_bounds__(W * 64) void gemm_km256_k(NtP p) {
  static_assert(W == 8, "two wavefronts per SIMD");
  constexpr int MB = 8, NB = 4;
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 2, wn = wave & 3;
  int tile_m, tile_n;
  tile_of(p, blockIdx.x, &tile_m, &tile_n);
  const int m0 = tile_m * kTile, n0 = tile_n * kTile;

  // ---- loader -------------------------------------------------------------------------------------------------
  // Only the second four wavefronts load, all of a stage in one burst right behind the barrier: 8 instructions of
  // 16 bytes per lane for each operand.  The two wavefronts of a SIMD do not alternate: the one launched first gets
  // the matrix pipe whenever it can use it, so it runs through its stage and then waits at the barrier while the
  // other catches up (cycle stamps: about 1100 of a stage's 2800 cycles at the barrier for wavefronts 0-3, under 100
  // for 4-7).  A load instruction occupies the address unit of the compute unit for 16 cycles, and a wavefront that
  // cannot hand over a load cannot issue the MFMAs behind it either, so loads belong to the wavefronts that are
  // waiting for the pipe anyway, and the ones that own the pipe have none.
  // Loader thread t (0..255) and instruction j fill, per operand,
  //   K-contiguous: 16-byte position j*256 + t = (row j*32 + t/8, slot t%8), slot holds global chunk (t%8) ^ ((row >> 1) & 7);
  //   k-major: k-row 16*(j/2) + 4*(j%2) + (t/32)%4 + 8*(t/128), 16-byte half t%2 of 32-byte unit (t%32)/2, which holds
  //            global unit ((t%32)/2) ^ key(k-row); rows are dealt so that the key is t/32 whatever j is, and the two
  //            rows of a wavefront are neighbours (its 1 KiB of LDS is contiguous).
  const bool loader = wave >= 4;
  const int lt = tid - 256, lw = wave - 4;  // loader thread / wavefront index (meaningful if loader)
  unsigned voa, vob, lda_dst, ldb_dst;                    // per-lane global byte offset; this wavefront's LDS offset
  {
    const int lrow = lt >> 3, lchunk = (lt & 7) ^ ((lrow >> 1) & 7);
    const int c = lt & 31, b = lt >> 5, key = b, kr = (b & 3) + 8 * (b >> 2);
    const unsigned km_dst = (unsigned)(2 * (lw & 1) + 8 * (lw >> 1)) * 512, nt_dst = (unsigned)lw * 1024;
    voa = AKM ? (unsigned)(kr * (int)p.lda) * 2u + ((c >> 1) ^ key) * 32 + (c & 1) * 16 : (unsigned)(lrow * (int)p.lda + lchunk * 8) * 2u;
    vob = BKM ? (unsigned)(kr * (int)p.ldb) * 2u + ((c >> 1) ^ key) * 32 + (c & 1) * 16 : (unsigned)(lrow * (int)p.ldb + lchunk * 8) * 2u;
    lda_dst = AKM ? km_dst : nt_dst;
    ldb_dst = BKM ? km_dst : nt_dst;
  }
  const char *pa = (const char *)(AKM ? p.A + m0 : p.A + (long)m0 * p.lda);    // stage 0 of the tile
  const char *pb = (const char *)(BKM ? p.Bt + n0 : p.Bt + (long)n0 * p.ldb);
  const long sa = AKM ? (long)kStageK * p.lda * 2 : kStageK * 2, sb = BKM ? (long)kStageK * p.ldb * 2 : kStageK * 2;
  // global byte offset from instruction j to j + 1, j even / odd: 32 rows (K-contiguous), or 4 / 12 k-rows (k-major: the
  // instructions start at k-rows 0, 4, 16, 20, 32, ...); the same in LDS bytes
  const unsigned ga0 = (unsigned)((AKM ? 4 : 32) * p.lda * 2), ga1 = (unsigned)((AKM ? 12 : 32) * p.lda * 2);
  const unsigned gb0 = (unsigned)((BKM ? 4 : 32) * p.ldb * 2), gb1 = (unsigned)((BKM ? 12 : 32) * p.ldb * 2);
  constexpr unsigned la0 = AKM ? 4 * 512 : 4096, la1 = AKM ? 12 * 512 : 4096, lb0 = BKM ? 4 * 512 : 4096, lb1 = BKM ? 12 * 512 : 4096;
  const unsigned lds0 = (unsigned)(uintptr_t)smem;
  const unsigned wa = lds0 + lda_dst, wb = lds0 + kLdsB + ldb_dst;
  const int nk = p.K / kStageK;  // even, >= 2 (checked by the launcher)
  const long wrap_a = (long)nk * sa, wrap_b = (long)nk * sb;
  int cur = 0, left = 0;         // stage at pa / pb; stages the loop still loads after that one
  const int is_loader = wave >> 2;  // (plain scalar arithmetic: a select here may end up in a vector register)
  // L2 prefetch (instantiations with PF; p.pf > 0: stages ahead).  The 32 workgroups that an XCD runs side by side (p.gm tile rows x 32 / p.gm
  // tile columns) share 12 operand panels; whoever asks first for a line of a stage waits for memory, a fifth of all
  // requests.  With p.pf every loading wavefront ends its burst with one more load, 4 bytes per lane into a dump area
  // of LDS, at lines of the stage p.pf stages further on: wavefronts 4 and 5 a half each of this workgroup's share of
  // its A panel (1 / sharers of the panel), 6 and 7 the same of its B panel, 96 lines per workgroup and stage, so that
  // the XCD's workgroups together touch every line once (lanes beyond the share repeat addresses).  Loads return in
  // order, so the wait before the barrier can leave this last one outstanding: it has two stages to come back.  The
  // sharing pattern only decides which lines are touched early: every address lies inside this workgroup's own panels
  // and K range whatever the grid looks like (past the end of the K loop the touch stays on the stage being loaded).
  const int pfd = PF ? p.pf : 0;
  const bool pt_is_a = lw < 2;
  unsigned vot = 0;
  if (PF) {
    const int gm = p.gm, nsa = 32 / gm;
    const int per = pt_is_a ? kTile / nsa : kTile / gm, nl = per / 2;
    const int line = (pt_is_a ? tile_n % nsa : tile_m % gm) * per + (lw & 1) * nl + lane % nl;
    const bool km = pt_is_a ? AKM : BKM;
    const int ld = (int)(pt_is_a ? p.lda : p.ldb);
    vot = km ? (unsigned)((line >> 2) * ld) * 2u + (line & 3) * 128 : (unsigned)(line * ld) * 2u;
  }
  const unsigned wdump = lds0 + 4 * kBuf + wave * 256;  // 256 bytes per wavefront behind the stage buffers
  const long dsa = (long)pfd * sa, dsb = (long)pfd * sb;
// One instruction pair (A, B) of the burst: 16 bytes per lane straight to LDS, M0 = LDS address of the wavefront's
// 1 KiB, global address = scalar base + per-lane byte offset (no instruction offset: it would be added to the LDS
// address too).  The scalar add between the write of M0 and the load is the wait state that pair needs; the per-lane
// offset moves on to the next instruction's rows behind the load (an address register is read when the load issues).
#define SSDT_LD2(LA, LB, GA, GB)                                                                           \
  "s_mov_b32 m0, %[ta]\n\ts_add_u32 %[ta], %[ta], %[" #LA "]\n\tglobal_load_lds_dwordx4 %[va], %[pa]\n\t"     \
  "v_add_u32 %[va], %[" #GA "], %[va]\n\t"                                                                \
  "s_mov_b32 m0, %[tb]\n\ts_add_u32 %[tb], %[tb], %[" #LB "]\n\tglobal_load_lds_dwordx4 %[vb], %[pb]\n\t"     \
  "v_add_u32 %[vb], %[" #GB "], %[vb]\n\t"
// The whole stage at pa / pb into buffer BUF, by the loading wavefronts only.  One statement with its own branch: a
// branch the compiler knows of splits the hand-scheduled loop into blocks, and the register allocation that comes out
// of that spills fragments.
#define SSDT_LOAD_STAGE_ASM(BUF, TOUCH, ...)                                                               \
    asm volatile("s_cmp_eq_u32 %[ld], 0\n\ts_cbranch_scc1 .Lssdt_noload_%=\n\t"                            \
                 "s_add_u32 %[ta], %[wa], %[ba]\n\ts_add_u32 %[tb], %[wb], %[bb]\n\t"                       \
                 "v_mov_b32 %[va], %[voa]\n\tv_mov_b32 %[vb], %[vob]\n\t"                                   \
                 SSDT_LD2(la0, lb0, ga0, gb0) SSDT_LD2(la1, lb1, ga1, gb1) SSDT_LD2(la0, lb0, ga0, gb0)      \
                 SSDT_LD2(la1, lb1, ga1, gb1) SSDT_LD2(la0, lb0, ga0, gb0) SSDT_LD2(la1, lb1, ga1, gb1)      \
                 SSDT_LD2(la0, lb0, ga0, gb0) SSDT_LD2(la1, lb1, ga1, gb1)                                   \
                 TOUCH                                                                                     \
                 ".Lssdt_noload_%=:"                                                                       \
                 : [ta] "=&s"(ta_), [tb] "=&s"(tb_), [va] "=&v"(va_), [vb] "=&v"(vb_)                      \
                 : [ld] "s"(is_loader), [wa] "s"(wa), [wb] "s"(wb), [ba] "n"((BUF) * kBuf), [bb] "n"((BUF) * kBuf), \
                   [pa] "s"(pa), [pb] "s"(pb), [voa] "v"(voa), [vob] "v"(vob), [ga0] "s"(ga0), [ga1] "s"(ga1), \
                   [gb0] "s"(gb0), [gb1] "s"(gb1), [la0] "n"(la0), [la1] "n"(la1), [lb0] "n"(lb0), [lb1] "n"(lb1) \
                   __VA_ARGS__                                                                             \
                 : "memory", "scc")
#define SSDT_LOAD_STAGE(BUF)                                                                               \
  {                                                                                                        \
    unsigned ta_, tb_, va_, vb_;                                                                           \
    if constexpr (PF) {                                                                                    \
      /* the touched stage: p.pf on from the one at pa / pb if the loop gets that far, else that one */    \
      const bool far_ = left >= pfd, wr_ = cur + pfd >= nk;                                                 \
      const char *pt_ = pt_is_a ? pa + (far_ ? dsa - (wr_ ? wrap_a : 0) : 0) : pb + (far_ ? dsb - (wr_ ? wrap_b : 0) : 0); \
      SSDT_LOAD_STAGE_ASM(BUF, "s_mov_b32 m0, %[dump]\n\ts_nop 0\n\tglobal_load_lds_dword %[vot], %[pt]\n\t",   \
                          , [dump] "s"(wdump), [vot] "v"(vot), [pt] "s"(pt_));                             \
    } else {                                                                                               \
      SSDT_LOAD_STAGE_ASM(BUF, "", );                                                                      \
    }                                                                                                      \
  }

  // ---- fragment addresses ---------------------------------------------------------------------------------
  const int lr = lane & 15, lq = lane >> 4;
  // K-contiguous: lane reads row lr of a 16-row block, chunk 4*step + lq, swizzled by (row >> 1) & 7
  const unsigned nt_c0 = ((lq ^ (lr >> 1)) * 16), nt_c1 = (((4 | lq) ^ (lr >> 1)) * 16);
  // k-major: lane supplies k-row 8*lq + lr/4 (+4 for the second read), bytes 8*(lr%4).. of the block's 32-byte unit
  const int kkey = (lr >> 2) | ((lq & 1) << 2);
  const unsigned km_row = (unsigned)(8 * lq + (lr >> 2)) * 512 + 8 * (lr & 3);
  const lds_char_t *aA[AKM ? MB : 2], *aB[BKM ? NB : 2];
  if (AKM) {
#pragma unroll
    for (int i = 0; i < MB; ++i) aA[i] = (const lds_char_t *)(uintptr_t)(lds0 + km_row + (unsigned)((wm * 8 + i) ^ kkey) * 32);
  } else {
    aA[0] = (const lds_char_t *)(uintptr_t)(lds0 + (wm * 128 + lr) * 128 + nt_c0);
    aA[1] = (const lds_char_t *)(uintptr_t)(lds0 + (wm * 128 + lr) * 128 + nt_c1);
  }
  if (BKM) {
#pragma unroll
    for (int j = 0; j < NB; ++j) aB[j] = (const lds_char_t *)(uintptr_t)(lds0 + kLdsB + km_row + (unsigned)((wn * NB + j) ^ kkey) * 32);
  } else {
    aB[0] = (const lds_char_t *)(uintptr_t)(lds0 + kLdsB + (wn * NB * 16 + lr) * 128 + nt_c0);
    aB[1] = (const lds_char_t *)(uintptr_t)(lds0 + kLdsB + (wn * NB * 16 + lr) * 128 + nt_c1);
  }
  // fragment of 16-row block i (of A) / j (of B) for 32-wide step `step` of the stage in buffer `buf`
  auto rdA = [&](int i, int step, int buf) -> bf16x8_t {
    if constexpr (AKM) return frag_km(aA[i], buf * kBuf + step * 16384);
    else return frag_nt(aA[step], buf * kBuf + i * 2048);
  };
  auto rdB = [&](int j, int step, int buf) -> bf16x8_t {
    if constexpr (BKM) return frag_km(aB[j], buf * kBuf + step * 16384);
    else return frag_nt(aB[step], buf * kBuf + j * 2048);
  };

  f32x4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  bf16x8_t Af[MB], Bf[2][NB];

  // One stage (64 of K) is two 32-wide steps.  The A fragments live in one register set that is refilled block by
  // block as soon as a block's MFMAs have been issued; the B fragments in two sets that alternate per step.  All reads
  // of a stage have been issued by the end of its first step, so the stage's one barrier sits behind the first block
  // of the second step: after it the other buffer (the next stage, whose loads were waited for just before) may be
  // read, and the loading wavefronts bring the stage after next in over this one.  The code is written as the two
  // halves either side of that barrier, and the loop is cut there, where no LDS read is outstanding (with the cut at
  // the stage boundary the compiler, which does not carry its count of outstanding reads around a loop, waited for
  // all of them at the head of every iteration).
  auto mfma_block = [&](int i, int set, int j0, int j1) {
    SSDT_FENCE;
#pragma unroll
    for (int j = j0; j < j1; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Bf[set][j], Af[i], acc[i][j], 0, 0, 0);
    SSDT_FENCE;
  };
// LDS reads are never issued back to back: the command queue of the LDS takes a few, and a wavefront that cannot
// hand over a read cannot issue the MFMAs behind it either.  With the five reads that used to follow the barrier in
// one group, and the four at the end of the stage, that queue was full in 18 % of all cycles (SQ_LDS_CMD_FIFO_FULL
// against SQ_BUSY_CYCLES; 0.6 % now).  Every read below has at least one MFMA of its own wavefront in front of it.
// First half of the stage in buffer BUF: step 0 and the first block of step 1, then the barrier.  On entry Af[0..7]
// and Bf[0][0..3] hold (or are about to receive) the fragments of step 0; the B fragments of step 1 are read here,
// one in each of the first four blocks, the A fragments of step 1 block by block behind their last use.
// waits for every LDS read and for all loads but the last N (N = WITH in the instantiations with touches, else WITHOUT)
#define SSDT_WAIT_LOADS(WITH, WITHOUT)                                                                     \
  {                                                                                                        \
    if constexpr (PF) asm volatile("s_waitcnt vmcnt(" WITH ") lgkmcnt(0)" ::: "memory");                   \
    else asm volatile("s_waitcnt vmcnt(" WITHOUT ") lgkmcnt(0)" ::: "memory");                             \
  }
#define SSDT_KM_HEAD(BUF, MORE, SUM)                                                                       \
  {                                                                                                        \
    _Pragma("unroll") for (int i = 0; i < MB; ++i) {                                                       \
      mfma_block(i, 0, 0, 2);                                                                              \
      if (i < NB) Bf[1][i] = rdB(i, 1, BUF);                                                               \
      mfma_block(i, 0, 2, NB);                                                                             \
      if (SUM && i == 0) sum_block(0);                                                                     \
      Af[i] = rdA(i, 1, BUF);                                                                              \
    }                                                                                                      \
    mfma_block(0, 1, 0, NB);                                                                               \
    if (SUM) sum_block(1);                                                                                 \
    if (MORE) {                                                                                            \
      /* every LDS read of this stage has returned, this wavefront's part of the next stage has landed */  \
      SSDT_WAIT_LOADS("1", "0");                                                                           \
      __builtin_amdgcn_s_barrier();                                                                        \
      asm volatile("" ::: "memory");                                                                       \
      SSDT_FENCE;                                                                                          \
    }                                                                                                      \
  }
// Second half: the loads of the stage after next into buffer BUF, then the rest of step 1 out of the registers
// while step 0 of the next stage (buffer BUF ^ 1) is read: its B fragments and the first A fragment inside the first
// blocks, the other A fragments block by block.  MORE / MORE2: a next stage / a stage after next exists.
#define SSDT_KM_TAIL(BUF, MORE, MORE2)                                                                     \
  {                                                                                                        \
    if (MORE2) {                                                                                           \
      SSDT_FENCE;                                                                                          \
      SSDT_LOAD_STAGE(BUF);                                                                                \
      SSDT_FENCE;                                                                                          \
    }                                                                                                      \
    _Pragma("unroll") for (int i = 1; i < MB; ++i) {                                                       \
      mfma_block(i, 1, 0, 1);                                                                              \
      if (MORE && i <= NB) Bf[0][i - 1] = rdB(i - 1, 0, (BUF) ^ 1);                                        \
      mfma_block(i, 1, 1, 3);                                                                              \
      if (MORE && i == 1) Af[0] = rdA(0, 0, (BUF) ^ 1);                                                    \
      mfma_block(i, 1, 3, NB);                                                                             \
      if (MORE) Af[i] = rdA(i, 0, (BUF) ^ 1);                                                              \
    }                                                                                                      \
    pa += sa; pb += sb; --left;                                                                            \
    if (++cur == nk) { cur = 0; pa -= wrap_a; pb -= wrap_b; }                                              \
  }

  // The K loop may start at a stage other than 0 and wrap around (every workgroup of an XCD at the same stage, so
  // that they still share their panels in the L2; the XCDs apart from each other).
  const int s0 = __builtin_amdgcn_readfirstlane((int)((blockIdx.x & 7) * p.stagger) % nk) & ~1;
  pa += (long)s0 * sa; pb += (long)s0 * sb;
  cur = s0; left = nk - 1;
  SSDT_LOAD_STAGE(0);
  pa += sa; pb += sb; --left;
  if (++cur == nk) { cur = 0; pa -= wrap_a; pb -= wrap_b; }
  SSDT_LOAD_STAGE(1);
  pa += sa; pb += sb; --left;  // from here on: the stage after next
  if (++cur == nk) { cur = 0; pa -= wrap_a; pb -= wrap_b; }
  // stage 0 has landed (stage 1, a loader's last 16 loads, and the two touches may still be on their way)
  SSDT_WAIT_LOADS("18", "16");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  SSDT_FENCE;
#pragma unroll
  for (int j = 0; j < NB; ++j) Bf[0][j] = rdB(j, 0, 0);
#pragma unroll
  for (int i = 0; i < MB; ++i) Af[i] = rdA(i, 0, 0);
  SSDT_FENCE;
// the whole K loop; SUM (literal): also the column sums of the second operand
#define SSDT_KM_LOOP(SUM)                                                                                  \
  {                                                                                                        \
    SSDT_KM_HEAD(0, true, SUM);                                                                            \
    for (int st = 0; st + 4 <= nk; st += 2) {                                                              \
      SSDT_KM_TAIL(0, true, true);                                                                         \
      SSDT_KM_HEAD(1, true, SUM);                                                                          \
      SSDT_KM_TAIL(1, true, true);                                                                         \
      SSDT_KM_HEAD(0, true, SUM);                                                                          \
    }                                                                                                      \
    SSDT_KM_TAIL(0, true, false);                                                                          \
    SSDT_KM_HEAD(1, false, SUM);                                                                           \
    SSDT_KM_TAIL(1, false, false);                                                                         \
  }
  // Column sums of the second operand (the bias gradient when this is a weight-gradient product: sum over tokens of
  // dY), as a by-product: a block of rows of ones is multiplied in, one more MFMA per fragment of the second operand,
  // by the wavefronts of the first tile row that hold distinct fragments; every row of the result is the sum, and a
  // fixed order of additions makes it reproducible.  The loop exists twice so that the others do not pay for the test.
  if (CS && tile_m == 0 && wm == 0) {
    f32x4_t accs[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) accs[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    union { unsigned w[4]; bf16x8_t v; } ones;
    ones.w[0] = ones.w[1] = ones.w[2] = ones.w[3] = 0x3F803F80u;  // 1.0 eight times
    auto sum_block = [&](int set) {
      SSDT_FENCE;
#pragma unroll
      for (int j = 0; j < NB; ++j) accs[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Bf[set][j], ones.v, accs[j], 0, 0, 0);
      SSDT_FENCE;
    };
    SSDT_KM_LOOP(true);
    if (lr == 0) {  // this lane: row 0 of each block, columns j*16 + lq*4 + 0..3
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        uint16_t *o = p.colsum + n0 + wn * NB * 16 + j * 16 + lq * 4;
        float v[4] = {accs[j][0], accs[j][1], accs[j][2], accs[j][3]};
        if (p.colsum_acc) {
          float old[4];
          unpack4(*(const uint2 *)o, old);
#pragma unroll
          for (int t = 0; t < 4; ++t) v[t] += old[t];
        }
        *(uint2 *)o = pack4(v);
      }
    }
  } else {
    auto sum_block = [&](int) {};
    SSDT_KM_LOOP(false);
  }
#undef SSDT_KM_LOOP
#undef SSDT_KM_HEAD
#undef SSDT_KM_TAIL
#undef SSDT_LOAD_STAGE
#undef SSDT_LOAD_STAGE_ASM
#undef SSDT_WAIT_LOADS
#undef SSDT_LD2

  // epilogue through LDS (free now), 64x64 sub-tiles of the wavefront's part, one column of sub-tiles at a time:
  // lane l of block (i, j) holds row i*16 + (l & 15), columns j*16 + (l >> 4)*4 + 0..3
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // (vmcnt: the last touch, whose dump area the staging area covers)
  __builtin_amdgcn_s_barrier();  // every wavefront has finished reading the last stage
  asm volatile("" ::: "memory");
  float *stg = (float *)smem + wave * (64 * kEpiLd);
#pragma unroll
  for (int J = 0; J < NB / 4; ++J) {
    const int nb = n0 + wn * NB * 16 + J * 64;
    u32x4_t ein[MB / 4][8];  // residual / activation-input rows, all requested before the first store
#pragma unroll
    for (int I = 0; I < MB / 4; ++I) epilogue_fetch<EPI>(p, m0 + wm * 128 + I * 64, nb, lane, ein[I]);
#pragma unroll
    for (int I = 0; I < MB / 4; ++I) {
#pragma unroll
      for (int il = 0; il < 4; ++il)
#pragma unroll
        for (int jl = 0; jl < 4; ++jl) {
          const f32x4_t a = acc[I * 4 + il][J * 4 + jl];
          *(float4 *)(stg + (il * 16 + lr) * kEpiLd + jl * 16 + lq * 4) = make_float4(a[0], a[1], a[2], a[3]);
        }
      epilogue_rows<EPI>(p, stg, m0 + wm * 128 + I * 64, nb, lane, ein[I]);
    }
  }
}

int g_km_stagger = -100;  // test hook: stages between the K-loop starting points of neighbouring XCDs (-100 = by shape, -1 = K/8, -2 = K/16)

template <int EPI, bool AKM, bool BKM, int W, bool CS, bool PF>
static hipError_t launch_km_pf(const NtP &p, hipStream_t s) {
  constexpr size_t stg = (size_t)W * 64 * kEpiLd * 4, stages = (size_t)4 * kBuf, smem = stg > stages ? stg : stages;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_km256_k<EPI, AKM, BKM, W, CS, PF>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  prof::Scope ps(prof::GEMM_MFMA_KM, 2.0 * p.M * p.N * p.K, 0, s);
  hipLaunchKernelGGL((gemm_km256_k<EPI, AKM, BKM, W, CS, PF>), dim3(p.tiles_m * p.tiles_n), dim3(W * 64), smem, s, p);
  return hipGetLastError();
}

// the prefetching instantiation exists for the forms whose first operand is K-contiguous (prefetch_for)
template <int EPI, bool AKM, bool BKM, int W, bool CS>
static hipError_t launch_km(const NtP &p, hipStream_t s) {
  if constexpr (!AKM && !CS) {
    if (p.pf > 0) return launch_km_pf<EPI, AKM, BKM, W, CS, true>(p, s);
  }
  return launch_km_pf<EPI, AKM, BKM, W, CS, false>(p, s);
}

template <bool AKM, bool BKM>
static hipError_t launch_km_epi(int epi, const NtP &p, hipStream_t s) {
// (W = 4, one wavefront of 128 x 128 per SIMD with the accumulators in the AGPRs, was measured too: within 1 % of
// W = 8 on every shape of the layer, so only the latter is built.)
#define SSDT_CASE(E) case E: return launch_km<E, AKM, BKM, 8, false>(p, s);
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

int g_km_pf = -1;   // test hook: stages that the L2 prefetch runs ahead of the loads (-1 = by shape, 0 = none)
int g_km_mode = 1;  // test hook: 0 = never use this kernel, 1 = for k-major operands, 2 = also for the NT form

// Shape part of the conditions below: what a caller can know before it has pointers (workspace sizing, the choice
// between this kernel and transposed copies).
// Staggered K loops pay where many column tiles share a short K (measured on 32768 x N x 8192: +4 % at N = 24576
// and 32768, nothing at N = 8192; with K = 32768 nothing or a small loss): there all XCDs sweep the same B panels
// at the same K offset, and starting them K/8 apart spreads those reads over the memory channels.
static int stagger_for(int N, int K) {
  if (g_km_stagger != -100) return g_km_stagger >= 0 ? g_km_stagger : (K / kStageK) / (4 << -g_km_stagger);
  const int nk = K / kStageK;
  return (nk <= 128 && N / kTile >= 64) ? nk / 8 : 0;
}

// L2 prefetch distance by shape (0 = none).  It pays where the first operand is K-contiguous with rows far apart, i.e.
// a long K (sustained, alone: 32768 x 8192 x 24576 K-contiguous +7 %, the forward product with K = 32768 +4 %), costs
// 2 % at K = 8192 (the touches take the address unit's time and there is less latency to hide), and is a wash on the
// weight gradients, both of whose operands are k-major (-0.4 to +2 %).  Where both operands are K-contiguous with rows
// a multiple of 32 KiB apart (32768 x 8192 x 32768) it is 5 % faster alone but doubles the bytes fetched (lines touched
// early are evicted again before their stage: such rows share few L2 sets) and gives nothing in the layer: not used,
// and that product stays with gemm_nt256_k.  One stage ahead is as good as two or three and fetches least.
static int prefetch_for(int K, bool akm, bool bkm) {
  if (g_km_pf >= 0) return g_km_pf;
  if (!bkm && (K * 2) % 32768 == 0) return 0;
  return (!akm && K >= 16384) ? 1 : 0;
}

bool gemm_km_fits(int M, int N, int K, bool transA, bool transB, int dtype) {
  if (dtype != SSDT_BF16 || g_km_mode == 0) return false;
  if (M % kTile || N % kTile || K % (2 * kStageK) || K < 2 * kStageK) return false;
  if ((long)(M / kTile) * (N / kTile) < 256) return false;
  // the K-contiguous form stays with gemm_nt256_k unless this kernel's staggered K loop or its prefetch pays for the shape
  if (!transA && transB && g_km_mode < 2 && stagger_for(N, K) == 0 && prefetch_for(K, false, false) == 0) return false;
  return true;
}

// Takes the problem if it fits (hipErrorNotSupported otherwise, nothing launched): bf16, M and N multiples of 256 with
// at least 256 tiles, K a multiple of 128, 16-byte aligned operands and epilogue tensors.
hipError_t gemm_mfma_km_bf16(const Gemm &g, hipStream_t s) {
  if (!gemm_km_fits(g.M, g.N, g.K, g.transA, g.transB, g.dtype)) return hipErrorNotSupported;
  const bool akm = g.transA, bkm = !g.transB;
  auto al16 = [](const void *q) { return ((uintptr_t)q & 15) == 0; };
  if (!al16(g.A) || !al16(g.B) || g.lda % 8 || g.ldb % 8 || g.lda >= (1L << 22) || g.ldb >= (1L << 22)) return hipErrorNotSupported;
  if (g.ldc % 8 || !al16(g.C) || (g.C2 && !al16(g.C2)) || (g.bias && !al16(g.bias)) || (g.aux && !al16(g.aux)) ||
      (g.resid && (!al16(g.resid) || g.ldr % 8)))
    return hipErrorNotSupported;
  if (g.epi == EPI_BIAS_ACT && !g.C2) return hipErrorInvalidValue;
  if (g.epi == EPI_BIAS_RESID && !g.resid) return hipErrorInvalidValue;
  if (g.epi == EPI_ACTBWD && !g.aux) return hipErrorInvalidValue;
  if (g.colsum && ((uintptr_t)g.colsum & 7)) return hipErrorNotSupported;
  // a k-major tile row is 512 contiguous bytes at column m0 / n0: the leading dimension must hold whole tiles
  if ((akm && g.lda < g.M) || (bkm && g.ldb < g.N)) return hipErrorInvalidValue;
  NtP p{g.M, g.N, g.K, (const uint16_t *)g.A, (const uint16_t *)g.B, g.lda, g.ldb, g.ldc, g.ldr, (uint16_t *)g.C,
        (uint16_t *)g.C2, (const uint16_t *)g.bias, (const uint16_t *)g.resid, (const uint16_t *)g.aux, g.act,
        g.M / kTile, g.N / kTile, 8, (uint16_t *)g.colsum, g.colsum_accumulate ? 1 : 0, 0};
  p.stagger = stagger_for(g.N, g.K);
  p.gm = g_force_waves > 0 ? g_force_waves : (p.tiles_m >= p.tiles_n ? 4 : 8);
  p.pf = (!akm && !g.colsum && (p.gm & (p.gm - 1)) == 0 && p.gm <= 32) ? prefetch_for(g.K, akm, bkm) : 0;
  if (g.colsum) {  // by-product of the weight-gradient form only
    if (!(akm && bkm)) return hipErrorNotSupported;
    if (g.epi == EPI_NONE) return launch_km<EPI_NONE, true, true, 8, true>(p, s);
    if (g.epi == EPI_BIAS_RESID) return launch_km<EPI_BIAS_RESID, true, true, 8, true>(p, s);
    return hipErrorNotSupported;
  }
  if (akm && bkm) return launch_km_epi<true, true>(g.epi, p, s);
  if (bkm) return launch_km_epi<false, true>(g.epi, p, s);
  if (akm) return launch_km_epi<true, false>(g.epi, p, s);
  return launch_km_epi<false, false>(g.epi, p, s);
}

}  // namespace k
}  // namespace ssdt
