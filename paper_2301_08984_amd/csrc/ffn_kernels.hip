// Kernels of the co-sharded feed-forward operator: one bf16 MFMA GEMM with fused epilogues, and a
// fixed-order column sum for the bias gradients.
#include "ffn_kernels.h"

#include "mfma_common.h"

namespace ssa {
namespace {

constexpr int GBK = 32;  // contraction depth of one stage
constexpr float GELU_C0 = 0.7978845608028654f, GELU_C1 = 0.044715f;

// gelu(z) = z (1 - r), r = 1 / (1 + exp(2u)), u = C0 (z + C1 z^3)   [0.5 (1 + tanh u) = 1 - r]
// gelu'(z) = (1 - r) (1 + 2 z r u'(z)), u'(z) = C0 (1 + 3 C1 z^2)      [1 - tanh^2 u = 4 r (1 - r)]
template <bool GRAD>
__device__ inline void gelu4(const float (&z)[4], float (&h)[4], float (&d)[4]) {
  constexpr float K0 = 2.f * LOG2E * GELU_C0, K1 = K0 * GELU_C1;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float z2 = z[e] * z[e];
    const float r = __builtin_amdgcn_rcpf(1.f + fast_exp2(z[e] * fmaf(z2, K1, K0)));
    const float s = 1.f - r;
    h[e] = z[e] * s;
    if (GRAD) d[e] = s * fmaf(2.f * z[e] * r, fmaf(z2, 3.f * GELU_C0 * GELU_C1, GELU_C0), 1.f);
  }
}
template <bool GRAD>
__device__ inline void relu4(const float (&z)[4], float (&h)[4], float (&d)[4]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    h[e] = fmaxf(z[e], 0.f);
    if (GRAD) d[e] = z[e] > 0.f ? 1.f : 0.f;
  }
}
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
// four fp32 -> four bf16 (round to nearest even, the hardware conversion)
__device__ inline uint2 pack4(const float (&y)[4]) {
  union { bf16x2 v; uint32_t u; } a, b;
  a.v = __builtin_convertvector(f32x2{y[0], y[1]}, bf16x2);
  b.v = __builtin_convertvector(f32x2{y[2], y[3]}, bf16x2);
  return uint2{a.u, b.u};
}
__device__ inline void unpack4(uint2 u, float (&y)[4]) {
  y[0] = __uint_as_float(u.x << 16); y[1] = __uint_as_float(u.x & 0xffff0000u);
  y[2] = __uint_as_float(u.y << 16); y[3] = __uint_as_float(u.y & 0xffff0000u);
}

// Work-group -> tile.  Work-groups go to the 8 XCDs round-robin in launch order and each XCD has its
// own L2: work-group b becomes logical index (b % 8) * (tiles / 8) + b / 8, so an XCD works on a
// contiguous range of logical indices, and logical indices walk the tile grid in bands of four
// tile rows, down the band's rows first: the tiles an XCD runs at a time share a few row panels of
// A and column panels of B.
struct TilePos { int mt, nt; };
__device__ inline TilePos tile_pos(int mtiles, int ntiles) {
  const int tiles = mtiles * ntiles;
  const int b = blockIdx.x, xcd = b % 8, idx = b / 8;
  const int id = xcd * (tiles / 8) + min(xcd, tiles % 8) + idx;
  constexpr int BAND = 4;
  const int per_band = BAND * ntiles, band = id / per_band, in_band = id % per_band;
  const int rows = min(BAND, mtiles - band * BAND);
  TilePos t;
  t.mt = band * BAND + in_band % rows;
  t.nt = in_band / rows;
  return t;
}

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
constexpr uint32_t OUTSIDE = 0x7ffffff0u;  // a lane offset past every descriptor's extent: the load returns zeros

// One operand of a 16 KS deep contraction stage (KS = 16-wide contraction steps per stage), 64 F
// rows (of A) or columns (of B) -- "rho" below; F = 32-wide fragments per wavefront -- fetched from
// global memory straight into LDS, 16 bytes per lane, 1 KB per wavefront instruction, F KS / 2
// instructions per wavefront.  Bounds-checked buffer loads (the whole offset is the lane offset,
// the only part the hardware range-checks): everything outside the matrix lands as zeros.  The LDS
// image is swizzled at 16-byte granularity by choosing WHICH global chunk a lane fetches for its
// fixed LDS slot, so that the fragment reads below are free of bank conflicts:
//   TR = false (contraction index contiguous in memory): LDS row = rho, 32 KS bytes = 2 KS chunks;
//        chunk c of row rho sits at slot c ^ ((rho >> 2) & 3) (KS = 2), c ^ ((rho >> 1) & 7) (KS = 4)
//   TR = true  (rho contiguous in memory): LDS row = k, 128 F bytes = 8 F chunks; chunk c of row k
//        sits at slot c ^ (4 * (k & 3))
// With KS = 2 a row of a contraction-contiguous operand is half a cache line per stage, and the
// compute unit's load path then moves whole lines for half the bytes: KS = 4 for such operands.
template <bool TR, int F, int KS>
struct Stager {
  static constexpr int BYTES = 2048 * F * KS, NI = F * KS / 2, BK = 16 * KS;
  const char* base;      // start of the next stage to fetch
  int64_t step;          // bytes from one stage to the next
  int left;              // bytes from `base` to the end of the matrix (meaningful while k0 < ktot)
  int k0, kcur, ktot;
  uint32_t lane_off[NI]; // lane offset of instruction t inside a stage (OUTSIDE if its rho are not in the matrix)
  int klimit[2];         // !TR: the lane's chunk (even / odd instruction) is inside the contraction range while k0 <= klimit
  __amdgpu_buffer_rsrc_t rs;
  __device__ void init(const uint16_t* base_, int64_t ld, int rho_tot, int ktot_, int rho0, int lane, int w) {
    base = (const char*)base_;
    const uint32_t ld2 = (uint32_t)ld * 2u;
    ktot = ktot_;
    k0 = kcur = 0;
    klimit[0] = klimit[1] = 0;
    if (!TR) {
      constexpr int CPR = 2 * KS, RPI = 64 / CPR;  // chunks per LDS row, rows per instruction
      step = 2 * BK;
      left = (int)(((int64_t)(rho_tot - 1) * ld + ktot_) * 2);
#pragma unroll
      for (int t = 0; t < NI; ++t) {
        const int row = RPI * (w * NI + t) + lane / CPR;
        const int c = (lane % CPR) ^ (KS == 2 ? (row >> 2) & 3 : (row >> 1) & 7);
        lane_off[t] = (uint32_t)(rho0 + row) * ld2 + 16u * c;
        if (t < 2) klimit[t] = ktot_ - 8 * c - 8;  // the chunk depends on the parity of t only
      }
    } else {
      constexpr int LPR = 8 * F, RPI = 64 / LPR;  // lanes per LDS row, rows per instruction
      step = (int64_t)BK * ld * 2;
      left = (int)(((int64_t)(ktot_ - 1) * ld + rho_tot) * 2);
#pragma unroll
      for (int t = 0; t < NI; ++t) {
        const int krow = RPI * (w * NI + t) + lane / LPR;
        const int c = (lane % LPR) ^ (4 * (krow & 3));
        lane_off[t] = rho0 + 8 * c + 8 <= rho_tot ? (uint32_t)krow * ld2 + (uint32_t)(rho0 + 8 * c) * 2u : OUTSIDE;
      }
    }
  }
  // Scalar work once per stage, stages in ascending order: a descriptor that starts at the stage's
  // first contraction index and ends with the matrix, so the lane offsets are the same for every
  // stage, and is empty for stages past the end of the contraction (they load zeros).
  __device__ void begin_stage() {
    rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, k0 < ktot ? left : 0, 0x00020000);
    kcur = k0;
    base += step;
    left -= (int)step;
    k0 += BK;
  }
  // instruction t (0..NI-1) of the stage -> LDS at `dst` (this operand's part of a stage buffer)
  __device__ void issue(char* dst, int w, int t) const {
    const bool ok = TR || kcur <= klimit[t & 1];
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void*)(dst + (w * NI + t) * 1024), 16, ok ? lane_off[t] : OUTSIDE, 0, 0, 0);
  }
};

// Fragment addresses of one operand for one wavefront (`wr` = which half of the tile's rho).
// A fragment is 32 rho x 16 k, lane (r = lane % 32, hl = lane / 32) holding rho = r, k = 8 hl .. 8 hl + 7.
template <bool TR, int F, int KS>
struct FragReader {
  uint32_t a0;
  uint32_t blk[TR ? F : 1];
  __device__ void init(int lane, int wr) {
    const int r = lane & 31, hl = lane >> 5;
    if (!TR) {
      const int sw = KS == 2 ? (r >> 2) & 3 : (r >> 1) & 7;
      a0 = (uint32_t)(32 * F * wr + r) * (32u * KS) + (uint32_t)((hl ^ sw) << 4);
      blk[0] = 0;
    } else {
      const int i = lane & 15, bk = lane >> 4, kk = 8 * (bk >> 1) + (i >> 2);
      a0 = (uint32_t)kk * (128u * F) + 32u * (bk & 1) + 8u * (i & 3);
#pragma unroll
      for (int f = 0; f < F; ++f) blk[f] = (uint32_t)(((F * wr + f) ^ ((i >> 2) & 3)) << 6);
    }
  }
  // fragment f (rho = 32 F wr + 32 f ..) of contraction step ks of the stage at `op`
  __device__ bf16x8 read(const char* op, int f, int ks) const {
    if (!TR) {
      return *(const bf16x8*)(op + ((a0 ^ (uint32_t)(ks << 5)) + (uint32_t)f * (1024u * KS)));
    } else {
      const char* p = op + (a0 + blk[f] + (uint32_t)ks * (2048u * F));
      union { s16x4 h[2]; bf16x8 v; } o;
      o.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
      o.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 512 * F));
      return o.v;
    }
  }
};

// slot of item `i` when `n` items are dealt out evenly over `slots` slots; how many come before `slot`
constexpr int slot_of(int i, int n, int slots) { return i * slots / n; }
constexpr int items_before(int slot, int n, int slots) {
  int c = 0;
  for (int i = 0; i < n; ++i) c += slot_of(i, n, slots) < slot ? 1 : 0;
  return c;
}

// ---------------------------------------------------------------------------
// C[M,N] = A B with bf16 operands and fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//   AT = false: A[m][k] at A + m*lda + k      AT = true: A[k][m] at A + k*lda + m
//   BT = false: B[k][n] at B + k*ldb + n      BT = true: B[n][k] at B + n*ldb + k
// Four wavefronts, 2 x 2, each with 32 FI x 32 FJ of the result in accumulation registers; a stage
// is KS contraction steps of 16 deep; NS stage buffers form a ring:
//   FI = 4, FJ = 2, KS = 2, NS = 3: 256 x 128 tile, 72 KB of LDS and 128 accumulation registers:
//        two work-groups per compute unit, which overlap each other's prologue, epilogue and
//        barriers.  For products whose operands are both read transposed.
//   FI = 4, FJ = 2, KS = 4, NS = 3: 144 KB of LDS, one work-group per compute unit, half as many
//        barriers per MFMA.  For products with a contraction-contiguous operand (see Stager).
//   FI = FJ = 4, KS = 2, NS = 4: 256 x 256 tile, 256 accumulation registers (half the LDS reads and
//        loads per MFMA of the others); not instantiated: the feed-forward shapes have too few such
//        tiles to go round.
// Stages travel global -> LDS directly, NS - 1 stages ahead of the multiplication, the load
// instructions spread evenly between the MFMAs (the compute unit's load path moves 64 bytes per
// cycle, of which the kernel needs 32 to 48), and one barrier per stage, issued with half a step of
// MFMAs still to go so the matrix cores keep busy across it.  Operands whose contraction index is
// not contiguous in memory are read from LDS with the transposed read.
// The matrix cores are fed B fragments as their row operand and A fragments as their column
// operand, so a lane ends up with one row m and runs of four consecutive columns n.
// The contraction runs in ascending k, 16 at a time, whatever the tile position or shape: with
// EPI_ACC the accumulator starts from the fp32 partial result of the previous chunks, so a sum
// cut into chunks at multiples of 16 is the same sum.
// ---------------------------------------------------------------------------
template <bool AT, bool BT, int EPI, int FI, int FJ, int KS>
__global__ __launch_bounds__(256, (FI * FJ <= 8 && KS == 2) ? 2 : 1) void gemm_kernel(GemmArgs g) {
  constexpr int NS = FI * FJ <= 8 ? 3 : 4;  // stage buffers
  constexpr int GBM = 64 * FI, GBN = 64 * FJ;
  using StageA = Stager<AT, FI, KS>;
  using StageB = Stager<!BT, FJ, KS>;
  constexpr int A_BYTES = StageA::BYTES, STAGE_BYTES = StageA::BYTES + StageB::BYTES;
  constexpr int NM = FI * FJ, SLOTS = KS * NM;             // MFMAs per contraction step / per stage
  constexpr int LA = StageA::NI, NL = LA + StageB::NI;     // loads per stage (per wavefront): A first
  constexpr int NR = FI + FJ;                              // fragment reads per step
  constexpr int BAR = SLOTS - NM / 2;                      // the barrier sits before this slot
  // the stage buffers are separate arrays: the compiler then knows that a load into one does not
  // feed a read of another, and does not wait for it
  __shared__ __attribute__((aligned(1024))) char stage0[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char stage1[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char stage2[STAGE_BYTES];
  __shared__ __attribute__((aligned(1024))) char stage3[NS == 4 ? STAGE_BYTES : 16];
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 31, hl = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w >> 1, wn = w & 1;
  const int mtiles = (g.M + GBM - 1) / GBM, ntiles = (g.N + GBN - 1) / GBN;
  const TilePos tp = tile_pos(mtiles, ntiles);
  const int m0 = tp.mt * GBM, n0 = tp.nt * GBN;

  StageA sa;
  StageB sb;
  sa.init(g.A, g.lda, g.M, g.K, m0, lane, w);
  sb.init(g.B, g.ldb, g.N, g.K, n0, lane, w);
  FragReader<AT, FI, KS> ra;
  FragReader<!BT, FJ, KS> rb;
  ra.init(lane, wm);
  rb.init(lane, wn);

  // acc[j][i]: row m0 + 32 FI wm + 32 i + r, columns n0 + 32 FJ wn + 32 j + key_of(v, hl).
  // The fp32 partial result between chunks lives in the workspace in the order the registers hold
  // it (tile, wavefront, (j, i, quad), lane): 1 KB per wavefront instruction, fully coalesced.
  f32x16 acc[FJ][FI];
  f32x4* frag32 = nullptr;
  if (EPI == EPI_ACC) frag32 = (f32x4*)g.acc32 + ((int64_t)(tp.mt * ntiles + tp.nt) * 4 + w) * (NM * 4 * 64) + lane;
  if (EPI == EPI_ACC && g.accumulate) {
#pragma unroll
    for (int j = 0; j < FJ; ++j)
#pragma unroll
      for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = frag32[((j * FI + i) * 4 + q) * 64];
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[j][i][4 * q + e] = v[e];
        }
  } else {
#pragma unroll
    for (int j = 0; j < FJ; ++j)
#pragma unroll
      for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][i][v] = 0.f;
  }

  // the stage count is rounded up to a multiple of the ring: stages past the end load zeros and add nothing
  const int nk = (g.K + 16 * KS - 1) / (16 * KS), nkr = (nk + NS - 1) / NS * NS;
  bf16x8 fa[2][FI], fb[2][FJ];  // fragments of the contraction step being multiplied and of the next one
  // fragment reads of one contraction step in the order of their first use: B 0, A 0 .. FI-1, B 1 .. FJ-1
  auto read_item = [&](const char* st, int item, int ks, int set) {
    if (item == 0) fb[set][0] = rb.read(st + A_BYTES, 0, ks);
    else if (item <= FI) fa[set][item - 1] = ra.read(st, item - 1, ks);
    else fb[set][item - FI] = rb.read(st + A_BYTES, item - FI, ks);
  };
  // One stage: multiply `cur` (the fragments of its first step are in registers), fetch the stage
  // NS - 1 ahead into `ldst` (the buffer of the stage before `cur`, free since the last barrier),
  // and, once the stage after `cur` has landed for every wavefront, read the fragments of its
  // first step from `nxt`.  KS NM slots of one MFMA each; the other instructions are dealt out over
  // the slots (loads evenly over the stage, the fragments of the next step over a step, in the
  // order of their first use) and the scheduler is told to keep every slot together: the matrix
  // cores stall as soon as the instructions between two MFMAs take longer to issue than one MFMA
  // takes to run.
  auto stage = [&](const char* cur, const char* nxt, char* ldst) {
    sa.begin_stage();
    sb.begin_stage();
#pragma unroll
    for (int s = 0; s < SLOTS; ++s) {
      const int ks = s / NM, x = s % NM, j = x / FI, i = x % FI;
      if (s == BAR) {
        // all but the youngest loads are done: the next stage is in LDS (this wavefront's part), and
        // so are this wavefront's reads of `cur`.  A bare barrier: __syncthreads() would wait for
        // every load in flight.
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((NS - 3) * NL + items_before(BAR, NL, SLOTS)) : "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      }
      acc[j][i] = mfma(fb[ks & 1][j], fa[ks & 1][i], acc[j][i]);
#pragma unroll
      for (int l = 0; l < NL; ++l)
        if (s == slot_of(l, NL, SLOTS)) {
          if (l < LA) sa.issue(ldst, w, l);
          else sb.issue(ldst + A_BYTES, w, l - LA);
        }
      if (ks + 1 < KS) {  // fragments of the next step of this stage
#pragma unroll
        for (int item = 0; item < NR; ++item)
          if (x == 1 + slot_of(item, NR, NM - 2)) read_item(cur, item, ks + 1, (ks + 1) & 1);
      } else if (s >= BAR) {  // fragments of the first step of the next stage
#pragma unroll
        for (int item = 0; item < NR; ++item)
          if (s - BAR == slot_of(item, NR, NM / 2)) read_item(nxt, item, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  auto fetch_all = [&](char* dst) {
    sa.begin_stage();
    sb.begin_stage();
#pragma unroll
    for (int t = 0; t < LA; ++t) sa.issue(dst, w, t);
#pragma unroll
    for (int t = 0; t < NL - LA; ++t) sb.issue(dst + A_BYTES, w, t);
  };
  fetch_all(stage0);
  fetch_all(stage1);
  if (NS == 4) fetch_all(stage2);
  if constexpr (EPI == EPI_ACC16) {
   if (g.accumulate) {
    // The partial sum of the earlier chunks is the output itself (bf16): read as whole rows (64 FJ
    // contiguous bytes per row), widened, and turned into the register layout through a piece of
    // LDS of the wavefront's own -- the epilogue's path backwards.  The pieces lie in the third stage
    // buffer, which no load targets before the barrier that ends the prologue.
    constexpr int TLD = 128 * FJ + 16, LPR = 8 * FJ, RPI = 64 / LPR;
    static_assert(NS == 3 && 4 * 32 * TLD <= STAGE_BYTES, "accumulator staging does not fit");
    char* tb = stage2 + w * (32 * TLD);
    const int c4 = 4 * (lane % LPR), rsub = lane / LPR;
    const int n = n0 + wn * 32 * FJ + c4;
#pragma unroll
    for (int i = 0; i < FI; ++i) {
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int row = RPI * it + rsub, m = m0 + wm * 32 * FI + 32 * i + row;
        float x[4] = {0.f, 0.f, 0.f, 0.f};
        if (m < g.M && n < g.N) unpack4(*(const uint2*)(g.out + (int64_t)m * g.ldo + n), x);
        *(f32x4*)(tb + row * TLD + c4 * 4) = f32x4{x[0], x[1], x[2], x[3]};
      }
#pragma unroll
      for (int j = 0; j < FJ; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const f32x4 v = *(const f32x4*)(tb + r * TLD + (32 * j + 8 * q + 4 * hl) * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[j][i][4 * q + e] = v[e];
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
   }
  }
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"((NS - 2) * NL) : "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
#pragma unroll
  for (int item = 0; item < NR; ++item) read_item(stage0, item, 0, 0);
  for (int kt = 0; kt < nkr; kt += NS) {
    if (NS == 4) {
      stage(stage0, stage1, stage3);
      stage(stage1, stage2, stage0);
      stage(stage2, stage3, stage1);
      stage(stage3, stage0, stage2);
    } else {
      stage(stage0, stage1, stage2);
      stage(stage1, stage2, stage0);
      stage(stage2, stage0, stage1);
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");

  if (EPI == EPI_ACC && !g.last) {
#pragma unroll
    for (int j = 0; j < FJ; ++j)
#pragma unroll
      for (int i = 0; i < FI; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          frag32[((j * FI + i) * 4 + q) * 64] =
              f32x4{acc[j][i][4 * q], acc[j][i][4 * q + 1], acc[j][i][4 * q + 2], acc[j][i][4 * q + 3]};
  } else {
    // Epilogue through LDS, one 32-row block of the wavefront's part at a time: the registers hold
    // one row and scattered column quads per lane; written to a piece of stage buffer of the
    // wavefront's own (rows padded by 16 bytes: conflict-free both ways) and read back as whole
    // rows, 8 FJ lanes x 4 columns, so that every global access of the epilogue is 64 FJ
    // contiguous bytes per row.  Everybody's loads have landed and everybody has left the main loop
    // before a buffer is reused.
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    constexpr int TLD = 128 * FJ + 16, LPR = 8 * FJ, RPI = 64 / LPR;
    static_assert(32 * TLD <= (NS == 4 ? STAGE_BYTES : STAGE_BYTES / 2), "epilogue staging does not fit");
    char* tb = NS == 4 ? (w == 0 ? stage0 : w == 1 ? stage1 : w == 2 ? stage2 : stage3)
                       : (w == 0 ? stage0 : w == 1 ? stage1 : w == 2 ? stage2 : stage0 + STAGE_BYTES / 2);
    const int c4 = 4 * (lane % LPR), rsub = lane / LPR;
    const int n = n0 + wn * 32 * FJ + c4;
    float bias[4] = {0.f, 0.f, 0.f, 0.f};
    if ((EPI == EPI_ACT || EPI == EPI_ACC || EPI == EPI_ACC16) && g.bias && n < g.N) unpack4(*(const uint2*)(g.bias + n), bias);
#pragma unroll
    for (int i = 0; i < FI; ++i) {
#pragma unroll
      for (int j = 0; j < FJ; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q)
          *(f32x4*)(tb + r * TLD + (32 * j + 8 * q + 4 * hl) * 4) =
              f32x4{acc[j][i][4 * q], acc[j][i][4 * q + 1], acc[j][i][4 * q + 2], acc[j][i][4 * q + 3]};
#pragma unroll
      for (int it = 0; it < 32 / RPI; ++it) {
        const int row = RPI * it + rsub, m = m0 + wm * 32 * FI + 32 * i + row;
        const f32x4 v = *(const f32x4*)(tb + row * TLD + c4 * 4);
        if (m >= g.M || n >= g.N) continue;
        float x[4] = {v[0] + bias[0], v[1] + bias[1], v[2] + bias[2], v[3] + bias[3]};
        uint16_t* orow = g.out + (int64_t)m * g.ldo + n;
        if (EPI == EPI_ACT) {
          float h[4], d[4];
          if (g.out2) {
            if (g.act == 0) relu4<true>(x, h, d); else gelu4<true>(x, h, d);
            *(uint2*)(g.out2 + (int64_t)m * g.ldo + n) = pack4(d);
          } else {
            if (g.act == 0) relu4<false>(x, h, d); else gelu4<false>(x, h, d);
          }
          *(uint2*)orow = pack4(h);
        } else if (EPI == EPI_MUL) {
          float mu[4];
          unpack4(*(const uint2*)(g.mul + (int64_t)m * g.ldm + n), mu);
#pragma unroll
          for (int e = 0; e < 4; ++e) x[e] *= mu[e];
          *(uint2*)orow = pack4(x);
        } else {
          *(uint2*)orow = pack4(x);
        }
      }
    }
  }
}

// out[n] = sum over m of A[m][n], fp32, fixed order: a work-group takes 64 columns; 32 row groups
// per column (rows g, g+32, .. summed in ascending order, 16-byte loads of 8 columns), then the 32
// partial sums in ascending g.  N is a multiple of 8 and A + n 16-byte aligned for n % 8 == 0.
__global__ __launch_bounds__(256) void colsum_kernel(const uint16_t* A, int64_t lda, int M, int N, uint16_t* out) {
  __shared__ float part[32][65];
  const int cl = threadIdx.x & 7, rg = threadIdx.x >> 3;
  const int n = blockIdx.x * 64 + cl * 8;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (n < N) {
    const uint16_t* col = A + n;
#pragma unroll 4
    for (int m = rg; m < M; m += 32) {
      const u32x4 v = *(const u32x4*)(col + (int64_t)m * lda);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[2 * e] += __uint_as_float(v[e] << 16);
        s[2 * e + 1] += __uint_as_float(v[e] & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][cl * 8 + e] = s[e];
  __syncthreads();
  const int c = threadIdx.x;
  if (c < 64 && blockIdx.x * 64 + c < N) {
    float t = part[0][c];
#pragma unroll
    for (int g = 1; g < 32; ++g) t += part[g][c];
    out[blockIdx.x * 64 + c] = f2bf(t);
  }
}

// Explicit instantiations: the host compiler emits the launch stub of the first implicit
// instantiation only.
#define SS_GEMM_INST(a, b, e, fi, fj, ks) template __global__ void gemm_kernel<a, b, e, fi, fj, ks>(GemmArgs);
#define SS_GEMM_INST4(a, b, fi, fj, ks) \
  SS_GEMM_INST(a, b, 0, fi, fj, ks) SS_GEMM_INST(a, b, 1, fi, fj, ks) SS_GEMM_INST(a, b, 2, fi, fj, ks) SS_GEMM_INST(a, b, 3, fi, fj, ks)
SS_GEMM_INST4(false, false, 4, 2, 4)
SS_GEMM_INST4(false, true, 4, 2, 4)
SS_GEMM_INST4(true, false, 4, 2, 2)
SS_GEMM_INST(false, false, 4, 4, 2, 4) SS_GEMM_INST(false, true, 4, 4, 2, 4)
// 128 x 128 tiles for products that are not accumulated over chunks, when the large tiles are few
SS_GEMM_INST(false, false, 0, 2, 2, 4) SS_GEMM_INST(false, false, 1, 2, 2, 4) SS_GEMM_INST(false, false, 3, 2, 2, 4)
SS_GEMM_INST(false, true, 0, 2, 2, 4) SS_GEMM_INST(false, true, 1, 2, 2, 4) SS_GEMM_INST(false, true, 3, 2, 2, 4)
SS_GEMM_INST(true, false, 0, 2, 2, 4) SS_GEMM_INST(true, false, 1, 2, 2, 4) SS_GEMM_INST(true, false, 3, 2, 2, 4)
#undef SS_GEMM_INST4
#undef SS_GEMM_INST

template <bool AT, bool BT, int EPI, int FI, int FJ, int KS>
hipError_t launch_one(const GemmArgs& g, hipStream_t st) {
  const int tiles = ((g.M + 64 * FI - 1) / (64 * FI)) * ((g.N + 64 * FJ - 1) / (64 * FJ));
  gemm_kernel<AT, BT, EPI, FI, FJ, KS><<<tiles, 256, 0, st>>>(g);
  return hipGetLastError();
}

// For an accumulated product the tile shape depends on the operand layouts only, never on the
// sizes: every chunk must cut its fp32 partial result into the same tiles.  The other products may
// choose: an output element is the same chain of MFMA steps whatever tile it falls into, so when
// fewer than 160 of the 256 x 128 tiles exist (k = 4 on the GPT-3 share: 96) they take 128 x 128
// tiles, twice as many work-groups at 4/3 of the operand traffic per flop.
template <bool AT, bool BT>
hipError_t launch_epi(const GemmArgs& g, int epi, hipStream_t st) {
  constexpr int FI = 4, FJ = 2, KS = AT ? 2 : 4;
  if (epi != EPI_ACC && epi != EPI_ACC16 && (int64_t)((g.M + 255) / 256) * ((g.N + 127) / 128) < 160) {
    switch (epi) {
      case EPI_ACT: return launch_one<AT, BT, EPI_ACT, 2, 2, 4>(g, st);
      case EPI_MUL: return launch_one<AT, BT, EPI_MUL, 2, 2, 4>(g, st);
      default: return launch_one<AT, BT, EPI_STORE, 2, 2, 4>(g, st);
    }
  }
  switch (epi) {
    case EPI_ACT: return launch_one<AT, BT, EPI_ACT, FI, FJ, KS>(g, st);
    case EPI_MUL: return launch_one<AT, BT, EPI_MUL, FI, FJ, KS>(g, st);
    case EPI_ACC: return launch_one<AT, BT, EPI_ACC, FI, FJ, KS>(g, st);
    case EPI_ACC16:
      if constexpr (AT) return hipErrorInvalidValue;  // the accumulated products read A untransposed
      else return launch_one<AT, BT, EPI_ACC16, FI, FJ, KS>(g, st);
    default: return launch_one<AT, BT, EPI_STORE, FI, FJ, KS>(g, st);
  }
}

}  // namespace

size_t gemm_acc_bytes(int M, int N) {
  // whole tiles; no tile is larger than 256 x 256
  return (size_t)((M + 255) / 256) * ((N + 255) / 256) * 256 * 256 * sizeof(float);
}

hipError_t launch_gemm(const GemmArgs& g, bool at, bool bt, int epi, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (!at && !bt) return launch_epi<false, false>(g, epi, st);
  if (!at && bt) return launch_epi<false, true>(g, epi, st);
  if (at && !bt) return launch_epi<true, false>(g, epi, st);
  return hipErrorInvalidValue;  // A^T B^T is not needed by the feed-forward operator
}

hipError_t launch_colsum(const void* A, int64_t lda, int M, int N, void* out, hipStream_t st) {
  colsum_kernel<<<(N + 63) / 64, 256, 0, st>>>((const uint16_t*)A, lda, M, N, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace ssa
