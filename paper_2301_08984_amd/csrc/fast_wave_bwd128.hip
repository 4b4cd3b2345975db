// dQ, dK and dV for small shares at head size 128, two wavefronts per SIMD.
//
// With one wavefront per SIMD the backward is bound by instruction issue: a lone wavefront gets an
// issue slot every few cycles and every wait for LDS or a matrix result is dead time.  A
// key-stationary wavefront that accumulates both dK and dV at D = 128 needs 128 accumulation
// registers plus 64 of stationary K and V fragments and cannot share a SIMD.  Here every work-group
// produces ONE of the three gradients for one 32-row block, so that it fits 256 registers and 66 KB
// of LDS and two work-groups (eight wavefronts) share a compute unit, each filling the other's waits:
//   dQ block: 32 queries stationary (Q, dO fragments), wavefronts split the keys:
//             dP^T = V dO^T, S^T = K Q^T, dS^T, dQ^T += K^T dS^T
//   dV block: 32 keys stationary (K fragments): S = Q K^T, P, dV^T += dO^T P
//   dK block: 32 keys stationary (K, V fragments): dP = dO V^T, S, dS, dK^T += Q^T dS
// The scores are formed three times instead of twice; the matrix cores have the room.
// Every wavefront streams its own 32-row sub-tiles from memory straight into two private LDS tiles
// (wave_dma.h), so the loop has no barrier and no LDS store.  A tile is refilled as soon as its last
// fragment has been read: the tile that is needed first in a step is also done with first, so each
// load has between half a step and a whole step to arrive.  The four partial sums of a block are
// folded through LDS as a fixed binary tree.
#include "wave_dma.h"

namespace ssa {
namespace {

constexpr int W2_NG = 4;                          // wavefronts per work-group
constexpr int W2_SLOT_B = 2 * W_TILE_B + 512;     // two tiles and the statistics of 32 queries
constexpr int W2_MERGE_B = W2_NG * 64 * 4 * 4 * 16;
constexpr int W2_LDS_B = W2_NG * W2_SLOT_B > W2_MERGE_B ? W2_NG * W2_SLOT_B : W2_MERGE_B;

// fold of the four wavefronts' partial sums (acc[db] in accumulator layout) and store of the block's
// rows `row` (lane = row) to `out`, scaled: wavefront w folds and stores the 32-column blocks w, w+4, ..
// No load into LDS may be under way.
template <int DB>
__device__ __forceinline__ void w2_merge_store(f32x16 (&acc)[DB], char* smem, int grp, int lane, int hl, bool live,
                                               uint16_t* out_row, float scale) {
  constexpr int WSLOT = 64 * 4 * DB;  // f32x4 units per wavefront
  f32x4* mb = (f32x4*)smem;
  __syncthreads();
  f32x4* my = mb + (size_t)grp * WSLOT + lane;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g)
      my[(4 * db + g) * 64] = f32x4{acc[db][4 * g], acc[db][4 * g + 1], acc[db][4 * g + 2], acc[db][4 * g + 3]};
  __syncthreads();
  if (!live) return;
  for (int db = grp; db < DB; db += W2_NG) {
    uint2 o[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 x[W2_NG];
#pragma unroll
      for (int w = 0; w < W2_NG; ++w) x[w] = mb[(size_t)w * WSLOT + (4 * db + g) * 64 + lane];
#pragma unroll
      for (int st = W2_NG / 2; st >= 1; st >>= 1)
#pragma unroll
        for (int w = 0; w < st; ++w) x[w] += x[w + st];
      o[g] = pack4_bf16(x[0][0], x[0][1], x[0][2], x[0][3], scale);
    }
    store_row32(out_row + 32 * db, o, hl, true);
  }
}

// ---------------------------------------------------------------------------
// dQ block.  Tile 0: K (operand reads, then transposed reads), tile 1: V (operand reads).
// ---------------------------------------------------------------------------
template <bool CAUSAL>
__device__ __forceinline__ void dq2_block(const KP& p, char* smem, int rank, int by, int bz_) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, SUB = 32, NG = W2_NG;
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* t0 = smem + grp * W2_SLOT_B;
  char* t1 = t0 + W_TILE_B;
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int qb = CAUSAL ? nsub - 1 - rank : rank;
  const int q0 = qb * SUB, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float c1 = p.scale * LOG2E;
  const uint32_t ss2 = (uint32_t)p.ss * 2u, dss2 = (uint32_t)p.do_ss * 2u;
  const uint32_t slice = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  const uint32_t dslice = (uint32_t)(((int64_t)(p.S - 1) * p.do_ss + D) * 2);
  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;

  uint32_t goff[8], ka[8], va[2][4];
  w_lane_offsets(goff, ss2, lane);
  w_nat_addr(ka, t0, r, hl);
  w_tr_addr(va, t0, lane);

  // stationary Q and dO fragments, through the two tiles
  u32x4 qf[KS], gf[KS];
  {
    uint32_t goff_g[8];
    w_lane_offsets(goff_g, dss2, lane);
    w_fetch(t0, Qb, (uint32_t)q0 * ss2, slice, goff);
    w_fetch(t1, dOb, (uint32_t)q0 * dss2, dslice, goff_g);
    W_VMCNT(0);
    w_nat_issue<0>(qf, ka);
    w_nat_issue<W_TILE_B>(gf, ka);
    w_nat_wait(qf);
    w_nat_wait(gf);
  }
  if (n > 0) {  // in this order: V(j0), K(j0)
    w_fetch(t1, Vb, (uint32_t)(j0 * SUB) * ss2, slice, goff);
    w_fetch(t0, Kb, (uint32_t)(j0 * SUB) * ss2, slice, goff);
  }
  const float nlse2 = -p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // step i: on their way, in this order: V(j), K(j)
  for (int i = 0; i < n; ++i) {
    const int j = j0 + i * NG;
    const uint32_t next = (uint32_t)(min(j + NG, jlast) * SUB) * ss2;
    f32x16 sa, pa;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
    {
      u32x4 fv[KS];
      W_VMCNT(8);  // V(j) has landed
      w_nat_issue<W_TILE_B>(fv, ka);
      w_nat_wait(fv);
      w_fetch(t1, Vb, next, slice, goff);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) pa = mfma(w_frag(fv[ks]), w_frag(gf[ks]), pa);
    }
    {
      u32x4 fk[KS];
      W_VMCNT(8);  // K(j) has landed
      w_nat_issue<0>(fk, ka);
      w_nat_wait(fk);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sa = mfma(w_frag(fk[ks]), w_frag(qf[ks]), sa);
    }
    // the transposed fragments of K arrive under the arithmetic on the scores
    u32x2 kt[2][2 * DB];
    w_tr_issue<0>(kt, va);
    if ((j * SUB + SUB > p.S) || (CAUSAL && j * SUB + SUB - 1 > q0)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = j * SUB + key_of(v, hl);
        const bool dead = key >= p.S || (CAUSAL && key > q);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    bf16x8 df[2];
    {
      float ds[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) ds[v] = fast_exp2(fmaf(sa[v], c1, nlse2)) * (pa[v] - delta);
      df[0] = pack8(&ds[0]);
      df[1] = pack8(&ds[8]);
    }
    w_tr_wait(kt);
    w_fetch(t0, Kb, next, slice, goff);
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(w_frag2(kt[hb][2 * db], kt[hb][2 * db + 1]), df[hb], acc[db]);
  }
  W_VMCNT(0);  // the tiles are about to be reused by the merge
  w2_merge_store<DB>(acc, smem, grp, lane, hl, q < p.S, (uint16_t*)p.dQ + base + (int64_t)q * p.ss, p.scale);
}

// ---------------------------------------------------------------------------
// dV block (WHICH = 0): tile 0: Q (operand reads), tile 1: dO (transposed reads)
// dK block (WHICH = 1): tile 1: dO (operand reads), tile 0: Q (operand reads, then transposed reads)
// ---------------------------------------------------------------------------
template <bool CAUSAL, int WHICH>
__device__ __forceinline__ void kv2_block(const KP& p, char* smem, int rank, int by, int bz_) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, SUB = 32, QG = W2_NG;
  constexpr bool DK = WHICH == 1;
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  char* t0 = smem + grp * W2_SLOT_B;
  char* t1 = t0 + W_TILE_B;
  // statistics of the step's 32 queries: -lse * log2(e), then Delta
  const uint32_t st_w = (uint32_t)(size_t)(w_lds_void*)(t0 + 2 * W_TILE_B) + 4u * lane;
  const uint32_t st_r = (uint32_t)(size_t)(w_lds_void*)(t0 + 2 * W_TILE_B) + 16u * hl;
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int k0 = rank * 32, key = k0 + r;
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
  const uint32_t ss2 = (uint32_t)p.ss * 2u, dss2 = (uint32_t)p.do_ss * 2u;
  const uint32_t slice = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  const uint32_t dslice = (uint32_t)(((int64_t)(p.S - 1) * p.do_ss + D) * 2);

  uint32_t goff[8], ka[8], va[2][4];
  w_lane_offsets(goff, ss2, lane);
  w_nat_addr(ka, t0, r, hl);
  w_tr_addr(va, t0, lane);
  // the lane offsets of dO differ from those of Q by (row in the sub-tile) * (difference of the row
  // strides): a lane part and a uniform part per instruction
  const uint32_t gd = (uint32_t)(lane >> 4) * (dss2 - ss2);
  auto fetch_do = [&](char* tile, uint32_t boff) {
    uint32_t g[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) g[t] = goff[t] + gd + (uint32_t)(4 * t) * (dss2 - ss2);
    w_fetch(tile, dOb, boff, dslice, g);
  };

  // stationary K (and V) fragments, through the two tiles
  u32x4 kf[KS], vf[KS];  // vf: dK block only
  w_fetch(t0, Kb, (uint32_t)k0 * ss2, slice, goff);
  if (DK) w_fetch(t1, Vb, (uint32_t)k0 * ss2, slice, goff);
  W_VMCNT(0);
  w_nat_issue<0>(kf, ka);
  w_nat_wait(kf);
  if (DK) {
    w_nat_issue<W_TILE_B>(vf, ka);
    w_nat_wait(vf);
  }
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
  const float c1 = p.scale * LOG2E;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int first = CAUSAL ? k0 / SUB : 0;
  const int j0 = first + grp;
  const int n = j0 < nsub ? (nsub - 1 - j0) / QG + 1 : 0;
  const int jlast = j0 + (n - 1) * QG;
  // lanes 0..31 fetch the LSE of query j * 32 + r, lanes 32..63 its Delta
  float pstat = 0.f;
  auto stat_load = [&](int j) {
    const int i = min(j * SUB + r, p.S - 1);
    pstat = hl == 0 ? lse_b[i] : (DK ? dl_b[i] : 0.f);
  };
  // every step: the tile used first ("early"), the statistics, the tile used last ("late"), in this order
  if (n > 0) {
    if (DK) fetch_do(t1, (uint32_t)(j0 * SUB) * dss2); else w_fetch(t0, Qb, (uint32_t)(j0 * SUB) * ss2, slice, goff);
    stat_load(j0);
    if (DK) w_fetch(t0, Qb, (uint32_t)(j0 * SUB) * ss2, slice, goff); else fetch_do(t1, (uint32_t)(j0 * SUB) * dss2);
  }
  for (int i = 0; i < n; ++i) {
    const int j = j0 + i * QG;
    const int jn = min(j + QG, jlast);
    f32x16 sa, pa;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
    W_VMCNT(8);  // the early tile of this step (and its statistics) have landed, the late tile may be under way
    if (DK) {
      u32x4 fg[KS];
      w_nat_issue<W_TILE_B>(fg, ka);
      w_nat_wait(fg);
      fetch_do(t1, (uint32_t)(jn * SUB) * dss2);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) pa = mfma(w_frag(fg[ks]), w_frag(vf[ks]), pa);
    } else {
      u32x4 fq[KS];
      w_nat_issue<0>(fq, ka);
      w_nat_wait(fq);
      w_fetch(t0, Qb, (uint32_t)(jn * SUB) * ss2, slice, goff);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sa = mfma(w_frag(fq[ks]), w_frag(kf[ks]), sa);
    }
    // this step's statistics -> LDS (the previous step's have been read), the next step's -> register
    asm volatile("ds_write_b32 %0, %1" ::"v"(st_w), "v"(hl == 0 ? -pstat * LOG2E : pstat) : "memory");
    stat_load(jn);
    if (DK) {
      u32x4 fq[KS];
      W_VMCNT(9);  // the late tile (Q) has landed
      w_nat_issue<0>(fq, ka);
      w_nat_wait(fq);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sa = mfma(w_frag(fq[ks]), w_frag(kf[ks]), sa);
    }
    // the transposed fragments of the late tile arrive under the arithmetic on the scores
    u32x2 tf[2][2 * DB];
    if (DK) {
      w_tr_issue<0>(tf, va);
    } else {
      W_VMCNT(9);  // the late tile (dO) has landed
      w_tr_issue<W_TILE_B>(tf, va);
    }
    if ((j * SUB + SUB > p.S) || (k0 + 32 > p.S) || (CAUSAL && j * SUB < k0 + 31)) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int qi = j * SUB + key_of(v, hl);
        const bool dead = qi >= p.S || key >= p.S || (CAUSAL && key > qi);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    bf16x8 of[2];  // P (dV block) or dS (dK block) as packed operands
    {
      float x[16];
      u32x4 l4[4];
      asm volatile("ds_read_b128 %0, %4\n\tds_read_b128 %1, %4 offset:32\n\tds_read_b128 %2, %4 offset:64\n\t"
                   "ds_read_b128 %3, %4 offset:96\n\ts_waitcnt lgkmcnt(0)"
                   : "=&v"(l4[0]), "=&v"(l4[1]), "=&v"(l4[2]), "=&v"(l4[3])
                   : "v"(st_r)
                   : "memory");
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * g + e] = fast_exp2(fmaf(sa[4 * g + e], c1, __uint_as_float(l4[g][e])));
      if (DK) {
        u32x4 d4[4];
        asm volatile("ds_read_b128 %0, %4 offset:128\n\tds_read_b128 %1, %4 offset:160\n\tds_read_b128 %2, %4 offset:192\n\t"
                     "ds_read_b128 %3, %4 offset:224\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(d4[0]), "=&v"(d4[1]), "=&v"(d4[2]), "=&v"(d4[3])
                     : "v"(st_r)
                     : "memory");
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) x[4 * g + e] *= pa[4 * g + e] - __uint_as_float(d4[g][e]);
      }
      of[0] = pack8(&x[0]);
      of[1] = pack8(&x[8]);
    }
    // dK += Q^T dS, dV += dO^T P; the late tile is refilled
    w_tr_wait(tf);
    if (DK) w_fetch(t0, Qb, (uint32_t)(jn * SUB) * ss2, slice, goff);
    else fetch_do(t1, (uint32_t)(jn * SUB) * dss2);
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(w_frag2(tf[hb][2 * db], tf[hb][2 * db + 1]), of[hb], acc[db]);
  }
  W_VMCNT(0);  // the tiles are about to be reused by the merge
  uint16_t* out = (uint16_t*)(DK ? p.dK : p.dV) + base + (int64_t)key * p.ss;
  w2_merge_store<DB>(acc, smem, grp, lane, hl, key < p.S, out, DK ? p.scale : 1.f);
}

// One launch: position pos of a (row, head) unit is the dK block (pos % 3 == 0), the dV block (1) or
// the dQ block (2) of rank pos / 3, heaviest first over the whole launch.
template <bool CAUSAL>
__global__ __launch_bounds__(64 * W2_NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_wave3_kernel(KP p) {
  __shared__ __attribute__((aligned(1024))) char smem[W2_LDS_B];
  const int units = gridDim.y * gridDim.z;
  const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int pos = lin / units, unit = lin % units;
  const int by = unit % gridDim.y, bz_ = unit / gridDim.y;
  const int kind = pos % 3, rank = pos / 3;
  if (kind == 0) kv2_block<CAUSAL, 1>(p, smem, rank, by, bz_);
  else if (kind == 1) kv2_block<CAUSAL, 0>(p, smem, rank, by, bz_);
  else dq2_block<CAUSAL>(p, smem, rank, by, bz_);
}

}  // namespace

hipError_t launch_fast_bwd_wave3(const KP& p, hipStream_t st) {
  const dim3 g(3 * ((p.S + 31) / 32), p.h1 - p.h0, p.b1 - p.b0);
  if (p.mask_kind == 1) bwd_wave3_kernel<true><<<g, 64 * W2_NG, 0, st>>>(p);
  else bwd_wave3_kernel<false><<<g, 64 * W2_NG, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace ssa
