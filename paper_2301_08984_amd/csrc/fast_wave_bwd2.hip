// dQ, dK and dV for small shares at head size 128, two wavefronts per SIMD.
//
// With one wavefront per SIMD the backward is bound by instruction issue: a lone wavefront gets an
// issue slot every few cycles and every wait for LDS or a matrix result is dead time (measured:
// matrix cores 17 %, LDS 28 %, vector ALUs 22 % busy, none of them overlapping).  A key-stationary
// wavefront that accumulates both dK and dV at D = 128 needs 128 accumulation registers plus 64 of
// stationary K and V fragments and cannot share a SIMD.  Here every work-group produces ONE of the
// three gradients for one 32-row block, so that it fits 256 registers and 78 KB of LDS and two
// work-groups (eight wavefronts) share a compute unit, each filling the other's waits:
//   dQ block: 32 queries stationary (Q, dO fragments), wavefronts split the keys:
//             S^T = K Q^T, dP^T = V dO^T, dS^T, dQ^T += K^T dS^T
//   dV block: 32 keys stationary (K fragments): S = Q K^T, P, dV^T += dO^T P
//   dK block: 32 keys stationary (K, V fragments): S, dP = dO V^T, dS, dK^T += Q^T dS
// The scores are formed three times instead of twice; the matrix cores have the room.
// Every wavefront stages its own 32-row sub-tiles (global -> registers -> one private LDS slot ->
// operand reads; the next sub-tile waits in registers), so the loop has no barrier.  The four partial
// sums of a block are folded through LDS as a fixed binary tree.
#include "wave_common.h"

namespace ssa {
namespace {

constexpr int W2_NG = 4;  // wavefronts per work-group

template <int D>
constexpr int w2_lds_elems() {
  constexpr int SLOT = 2 * 32 * (D + 24) + 2 * 2 * 32, MERGE = W2_NG * 64 * 4 * (D / 32) * 8;
  return W2_NG * SLOT > MERGE ? W2_NG * SLOT : MERGE;
}

// fold of the four wavefronts' partial sums (acc[db] in accumulator layout) and store of the block's
// rows `row` (lane = row) to `out`, scaled: wavefront w folds and stores the 32-column blocks w, w+4, ..
template <int DB>
__device__ __forceinline__ void w2_merge_store(f32x16 (&acc)[DB], uint16_t* smem, int grp, int lane, int hl, bool live,
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
// dQ block
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL>
__device__ __forceinline__ void dq2_block(const KP& p, uint16_t* smem, int rank, int by, int bz_) {
  constexpr int KS = D / 16, DB = D / 32, SUB = 32, CPT = D / 16, NG = W2_NG;
  constexpr int LD = D + 24;  // K is read both ways; V shares the pad
  constexpr int MAT = SUB * LD, SLOT = 2 * MAT + 2 * 2 * 32;
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint16_t* sK = smem + grp * SLOT;
  uint16_t* sV = sK + MAT;
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
  const uint32_t loff = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.ss + 8u * (lane % (D / 8))) * 2u;
  const uint32_t loff_g = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.do_ss + 8u * (lane % (D / 8))) * 2u;
  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;

  u32x4 pk[CPT], pv[CPT];
  bf16x8 qf[KS], gf[KS];
  {
    u32x4 pq[CPT], pg[CPT];
    sub_load<D>(pq, Qb, p.ss, p.S, q0, loff);
    sub_load<D>(pg, dOb, p.do_ss, p.S, q0, loff_g);
    if (n > 0) {
      sub_load<D>(pk, Kb, p.ss, p.S, j0 * SUB, loff);
      sub_load<D>(pv, Vb, p.ss, p.S, j0 * SUB, loff);
    }
    sub_store<D, LD>(sK, pq, lane);
    sub_store<D, LD>(sV, pg, lane);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = lds_nat<LD>(sK, r, ks, hl);
      gf[ks] = lds_nat<LD>(sV, r, ks, hl);
    }
  }
  const float nlse2 = -p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  for (int i = 0; i < n; ++i) {
    const int j = j0 + i * NG;
    // sub-tile j: registers -> LDS (the reads of the previous sub-tile precede these writes in the
    // wavefront's LDS queue); sub-tile j+NG starts its way from memory
    sub_store<D, LD>(sK, pk, lane);
    sub_store<D, LD>(sV, pv, lane);
    sub_load<D>(pk, Kb, p.ss, p.S, min(j + NG, jlast) * SUB, loff);
    sub_load<D>(pv, Vb, p.ss, p.S, min(j + NG, jlast) * SUB, loff);
    f32x16 sa, pa;
    {
      bf16x8 fk[KS], fv[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        fk[ks] = lds_nat<LD>(sK, r, ks, hl);
        fv[ks] = lds_nat<LD>(sV, r, ks, hl);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa = mfma(fk[ks], qf[ks], sa);
        pa = mfma(fv[ks], gf[ks], pa);
      }
    }
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
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      bf16x8 kt_[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) kt_[db] = lds_tr<LD>(sK, 16 * hb, 32 * db, lane);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(kt_[db], df[hb], acc[db]);
    }
  }
  w2_merge_store<DB>(acc, smem, grp, lane, hl, q < p.S, (uint16_t*)p.dQ + base + (int64_t)q * p.ss, p.scale);
}

// ---------------------------------------------------------------------------
// dV block (WHICH = 0) and dK block (WHICH = 1)
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL, int WHICH>
__device__ __forceinline__ void kv2_block(const KP& p, uint16_t* smem, int rank, int by, int bz_) {
  constexpr int KS = D / 16, DB = D / 32, SUB = 32, CPT = D / 16, QG = W2_NG;
  constexpr int LD = D + 24;
  constexpr int MAT = SUB * LD, SLOT = 2 * MAT + 2 * 2 * 32;
  constexpr bool DK = WHICH == 1;
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint16_t* tq = smem + grp * SLOT;
  uint16_t* tg = tq + MAT;
  float* sstat = (float*)(tq + 2 * MAT);  // -lse * log2(e) for the 32 queries, then Delta
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int k0 = rank * 32, key = k0 + r;
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;

  bf16x8 kf[KS], vf[DK ? KS : 1];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *(const bf16x8*)(Kb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
    if (DK) vf[ks] = *(const bf16x8*)(Vb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
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
  const uint32_t loff_q = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.ss + 8u * (lane % (D / 8))) * 2u;
  const uint32_t loff_g = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.do_ss + 8u * (lane % (D / 8))) * 2u;
  u32x4 pq[CPT], pg[CPT];
  float pstat = 0.f;
  auto gload = [&](int j) {
    sub_load<D>(pq, Qb, p.ss, p.S, j * SUB, loff_q);
    sub_load<D>(pg, dOb, p.do_ss, p.S, j * SUB, loff_g);
    const int i = min(j * SUB + r, p.S - 1);
    pstat = hl == 0 ? lse_b[i] : (DK ? dl_b[i] : 0.f);
  };
  if (n > 0) gload(j0);
  for (int i = 0; i < n; ++i) {
    const int j = j0 + i * QG;
    sub_store<D, LD>(tq, pq, lane);
    sub_store<D, LD>(tg, pg, lane);
    sstat[lane] = hl == 0 ? -pstat * LOG2E : pstat;
    gload(min(j + QG, jlast));
    f32x16 sa, pa;
    {
      bf16x8 fq[KS], fg[DK ? KS : 1];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        fq[ks] = lds_nat<LD>(tq, r, ks, hl);
        if (DK) fg[ks] = lds_nat<LD>(tg, r, ks, hl);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa = mfma(fq[ks], kf[ks], sa);
        if (DK) pa = mfma(fg[ks], vf[ks], pa);
      }
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
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 l4 = *(const f32x4*)(sstat + 8 * g + 4 * hl);
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * g + e] = fast_exp2(fmaf(sa[4 * g + e], c1, l4[e]));
        if (DK) {
          const f32x4 d4 = *(const f32x4*)(sstat + 32 + 8 * g + 4 * hl);
#pragma unroll
          for (int e = 0; e < 4; ++e) x[4 * g + e] *= pa[4 * g + e] - d4[e];
        }
      }
      of[0] = pack8(&x[0]);
      of[1] = pack8(&x[8]);
    }
    const uint16_t* tt = DK ? tq : tg;  // dK += Q^T dS, dV += dO^T P
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      bf16x8 tf[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) tf[db] = lds_tr<LD>(tt, 16 * hb, 32 * db, lane);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(tf[db], of[hb], acc[db]);
    }
  }
  uint16_t* out = (uint16_t*)(DK ? p.dK : p.dV) + base + (int64_t)key * p.ss;
  w2_merge_store<DB>(acc, smem, grp, lane, hl, key < p.S, out, DK ? p.scale : 1.f);
}

// One launch: position pos of a (row, head) unit is the dK block (pos % 3 == 0), the dV block (1) or
// the dQ block (2) of rank pos / 3, heaviest first over the whole launch.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(64 * W2_NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void bwd_wave3_kernel(KP p) {
  __shared__ __attribute__((aligned(16))) uint16_t smem[w2_lds_elems<D>()];
  const int units = gridDim.y * gridDim.z;
  const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int pos = lin / units, unit = lin % units;
  const int by = unit % gridDim.y, bz_ = unit / gridDim.y;
  const int kind = pos % 3, rank = pos / 3;
  if (kind == 0) kv2_block<D, CAUSAL, 1>(p, smem, rank, by, bz_);
  else if (kind == 1) kv2_block<D, CAUSAL, 0>(p, smem, rank, by, bz_);
  else dq2_block<D, CAUSAL>(p, smem, rank, by, bz_);
}

}  // namespace

hipError_t launch_fast_bwd_wave3(const KP& p, hipStream_t st) {
  const dim3 g(3 * ((p.S + 31) / 32), p.h1 - p.h0, p.b1 - p.b0);
  if (p.mask_kind == 1) bwd_wave3_kernel<128, true><<<g, 64 * W2_NG, 0, st>>>(p);
  else bwd_wave3_kernel<128, false><<<g, 64 * W2_NG, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace ssa
