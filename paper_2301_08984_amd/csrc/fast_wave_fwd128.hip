// Forward / recompute kernel for small shares at head size 128: the query-stationary wavefronts of
// fast_wave_fwd.hip with the K and V sub-tiles fetched from memory straight into LDS (wave_dma.h).
//
// One tile per wavefront and operand: the fragments of a sub-tile are read into registers, then the
// tile is refilled, so a sub-tile has one whole step to arrive.
#include "wave_dma.h"

namespace ssa {
namespace {

constexpr int W_NG = 4;  // wavefronts per work-group

template <bool BIAS, bool CAUSAL, bool RECOMP>
__global__ __launch_bounds__(64 * W_NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_wave128_kernel(KP p) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, SUB = 32, NG = W_NG;
  constexpr int TILE_B = W_TILE_B;
  constexpr int SLOT_B = 2 * TILE_B;                 // K, then V
  constexpr int MSLOT = 64 * (4 * DB + 1);           // f32x4 units one wavefront hands over in the merge
  constexpr int MERGE_B = NG * MSLOT * 16 + 4 * 32 * (DB < NG ? DB : NG);  // hand-over area + partial Delta
  constexpr int LDS_B = NG * SLOT_B > MERGE_B ? NG * SLOT_B : MERGE_B;
  __shared__ __attribute__((aligned(1024))) char smem[LDS_B];
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: scalar registers
  char* sK = smem + grp * SLOT_B;
  char* sV = sK + TILE_B;
  const BlockId blk = heavy_first_block_id();
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int qb = CAUSAL ? nsub - 1 - blk.x : blk.x;  // late query blocks see the most keys under a causal mask
  const int q0 = qb * SUB, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* bias_row = BIAS ? (const uint16_t*)p.bias + ((int64_t)h * p.S + qc) * p.S : nullptr;
  const float c1 = p.scale * LOG2E;

  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;  // key sub-tiles with a visible key
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;
  auto jc = [&](int j) { return min(j, jlast); };  // past the wavefront's last sub-tile: fetch it again

  uint32_t goff[8], ka[8], va[2][4];
  w_lane_offsets(goff, (uint32_t)p.ss * 2u, lane);
  w_nat_addr(ka, sK, r, hl);
  w_tr_addr(va, sV, lane);
  const uint32_t ss2 = (uint32_t)p.ss * 2u;
  const uint32_t slice_bytes = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  auto fetch = [&](char* tile, const uint16_t* src, int row0) { w_fetch(tile, src, (uint32_t)row0 * ss2, slice_bytes, goff); };

  uint2 bzn[4], bzc[4];  // bias slices of the next sub-tile / of the one about to be used
  auto bload = [&](int j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) bzn[g] = *(const uint2*)(bias_row + min(j * SUB + 8 * g + 4 * hl, p.S - 4));
  };

  // Q fragments through the (still unused) V tile, beside the first K sub-tile
  u32x4 qf[KS], fk[KS];
  u32x2 vfr[2][2 * DB];
  fetch(sV, Qb, q0);
  if (n > 0) fetch(sK, Kb, j0 * SUB);
  if (BIAS && n > 0) bload(j0);
  W_VMCNT(0);
  w_nat_issue<TILE_B>(qf, ka);
  w_nat_wait(qf);
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;

  // S^T = K Q^T with the fragments in fk: lane = query, registers = keys
  auto stage_s = [&](f32x16& sa) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sa[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sa = mfma(w_frag(fk[ks]), w_frag(qf[ks]), sa);
  };
  // online softmax of one 32-key block, first half: bias, mask, row maximum, running maximum
  auto softmax_max = [&](int k0, f32x16& sa, const uint2* bz, bool edge) {
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 u = bz[g];
        // natural units here; the change to base 2 rides on the subtraction of the maximum
        sa[4 * g + 0] = fmaf(sa[4 * g + 0], p.scale, __uint_as_float(u.x << 16));
        sa[4 * g + 1] = fmaf(sa[4 * g + 1], p.scale, __uint_as_float(u.x & 0xffff0000u));
        sa[4 * g + 2] = fmaf(sa[4 * g + 2], p.scale, __uint_as_float(u.y << 16));
        sa[4 * g + 3] = fmaf(sa[4 * g + 3], p.scale, __uint_as_float(u.y & 0xffff0000u));
      }
    }
    if (edge) {  // uniform; touches the scores only
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = k0 + key_of(v, hl);
        const bool dead = key >= p.S || (CAUSAL && key > q);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    float rmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, sa[v]);
    rmax *= BIAS ? LOG2E : c1;  // the running maximum is kept in base-2 units; scale > 0 on this path
    rmax = half_max(rmax);
    // the running maximum is raised only when exceeded by more than 2^8, so the O rescale is
    // skipped on most sub-tiles; probabilities stay below 2^8, harmless in fp32/bf16 range
    if (__builtin_amdgcn_ballot_w64(rmax > m + 8.f) != 0) {
      const float mn = fmaxf(m, rmax);
      const float alpha = fast_exp2(m - mn);
      m = mn;
      l *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] *= alpha;
    }
  };
  // second half: P = exp2(s - m) as packed bf16 operands, row sum
  auto softmax_exp = [&](const f32x16& sa, bf16x8 (&pf)[2]) {
    float lsum = 0.f;
    float pr[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      pr[v] = fast_exp2(fmaf(sa[v], BIAS ? LOG2E : c1, -m));
      lsum += pr[v];
    }
    l += lsum;
    pf[0] = pack8(&pr[0]);
    pf[1] = pack8(&pr[8]);
  };
  // O^T += V^T P^T with the fragments in vfr
  auto stage_pv = [&](const bf16x8 (&pf)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(w_frag2(vfr[t][2 * db], vfr[t][2 * db + 1]), pf[t], oacc[db]);
  };

  if (n > 0) {
    f32x16 sc, sn;
    w_nat_issue<0>(fk, ka);
    w_nat_wait(fk);
    fetch(sK, Kb, jc(j0 + NG) * SUB);
    fetch(sV, Vb, j0 * SUB);
    stage_s(sc);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
    }
    // step i: scores of sub-tile j are in sc; on their way, in this order: K(j+NG), V(j)
    for (int i = 0; i < n; ++i) {
      const int j = j0 + i * NG;
      // K(j+NG) has landed (V(j) may still be under way): fragments out under the row maxima, slot refilled
      if (BIAS) W_VMCNT(0); else W_VMCNT(8);
      w_nat_issue<0>(fk, ka);
      softmax_max(j * SUB, sc, bzc, (j * SUB + SUB > p.S) || (CAUSAL && j * SUB + SUB - 1 > q0));
      if (BIAS) bload(jc(j + NG));
      w_nat_wait(fk);
      fetch(sK, Kb, jc(j + 2 * NG) * SUB);
      stage_s(sn);
      // V(j) has landed (K(j+2NG) under way): fragments out under the exponentials
      if (BIAS) W_VMCNT(0); else W_VMCNT(8);
      w_tr_issue<0>(vfr, va);
      bf16x8 pf[2];
      softmax_exp(sc, pf);
      w_tr_wait(vfr);
      fetch(sV, Vb, jc(j + NG) * SUB);
      stage_pv(pf);
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
      }
      sc = sn;
    }
    W_VMCNT(0);  // the slots are about to be reused by the merge
  }

  {
    // every wavefront hands over its partial (O, m, l) through LDS; each then folds the statistics
    // with the same fixed binary tree ((g0+g2)+(g1+g3) for NG = 4), which also yields the weights
    // of every tree node, and wavefront w folds, normalises and stores the 32-column output blocks
    // w, w+NG, ...
    f32x4* mb = (f32x4*)smem;
    float* dpart = (float*)(mb + NG * MSLOT);  // [DB][32] partial Delta per output block (recompute)
    __syncthreads();
    f32x4* my = mb + (size_t)grp * MSLOT + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        my[(4 * db + g) * 64] = f32x4{oacc[db][4 * g], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]};
    my[4 * DB * 64] = f32x4{m, l, 0.f, 0.f};
    __syncthreads();
    float mm[NG], ll[NG];
#pragma unroll
    for (int w = 0; w < NG; ++w) {
      const f32x4 ml = mb[(size_t)w * MSLOT + 4 * DB * 64 + lane];
      mm[w] = ml[0];
      ll[w] = ml[1];
    }
    float a0s[NG], a1s[NG];  // tree weights, entry st + w: node w and its partner w + st at level st
#pragma unroll
    for (int st = NG / 2; st >= 1; st >>= 1)
#pragma unroll
      for (int w = 0; w < st; ++w) {
        const float mn = fmaxf(mm[w], mm[w + st]);
        const float a0 = fast_exp2(mm[w] - mn), a1 = fast_exp2(mm[w + st] - mn);
        a0s[st + w] = a0;
        a1s[st + w] = a1;
        ll[w] = ll[w] * a0 + ll[w + st] * a1;
        mm[w] = mn;
      }
    m = mm[0];
    l = half_sum(ll[0]);
    const float inv = 1.f / l;
    float part = 0.f;
    bool mine = false;
    for (int db = grp; db < DB; db += NG) {
      mine = true;
      f32x16 o;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 x[NG];
#pragma unroll
        for (int w = 0; w < NG; ++w) x[w] = mb[(size_t)w * MSLOT + (4 * db + g) * 64 + lane];
#pragma unroll
        for (int st = NG / 2; st >= 1; st >>= 1)
#pragma unroll
          for (int w = 0; w < st; ++w)
#pragma unroll
            for (int e = 0; e < 4; ++e) x[w][e] = x[w][e] * a0s[st + w] + x[w + st][e] * a1s[st + w];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[4 * g + e] = x[0][e];
      }
      if (q < p.S) part += fwd_epilogue_block<RECOMP>(p, o, db, inv, b, h, q, hl, base, 0.f);
    }
    const float lse = (m + log2f(l)) * LN2;
    if (!RECOMP) {
      if (grp == 0 && hl == 0 && q < p.S && p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
      return;
    }
    // recompute: Delta = sum over the output blocks of the partial row sums, in block order
    part = half_sum(part);
    if (mine && hl == 0) dpart[grp * 32 + r] = part;  // DB <= NG: wavefront w owns block w
    __syncthreads();
    if (grp == 0 && hl == 0 && q < p.S) {
      float dl = 0.f;
#pragma unroll
      for (int db = 0; db < (DB < NG ? DB : NG); ++db) dl += dpart[db * 32 + r];
      p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + q] = dl;
      if (p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
    }
  }
}

template <bool RECOMP>
hipError_t fwd_wave128_r(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 31) / 32, p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) fwd_wave128_kernel<true, true, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else if (bias) fwd_wave128_kernel<true, false, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else if (causal) fwd_wave128_kernel<false, true, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else fwd_wave128_kernel<false, false, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fast_fwd_wave128(const KP& p, bool recompute, hipStream_t st) {
  return recompute ? fwd_wave128_r<true>(p, st) : fwd_wave128_r<false>(p, st);
}

}  // namespace ssa
