// Forward / recompute kernel for small shares: query-stationary wavefronts that never wait for each
// other inside the loop.
#include "wave_common.h"

namespace ssa {
namespace {

// ---------------------------------------------------------------------------
// forward / recompute when the share has too few query blocks to fill the chip with
// 128-query work-groups.  A work-group owns one 32-query block; its NG wavefronts all
// hold the block's Q fragments and split the keys: wavefront g takes the 32-key
// sub-tiles g, g+NG, ...  Every wavefront stages its own sub-tiles of K and V
// (global -> registers -> its private LDS slot -> operand reads), so the loop has no
// barrier: the wavefronts drift apart and one's softmax arithmetic and staging overlaps
// the others' matrix products (two wavefronts share each SIMD).  The slot holds one K
// and one V sub-tile: K of sub-tile j+1 is consumed (scores, one step ahead) before V
// of sub-tile j, so K runs two sub-tiles ahead in registers and one ahead in LDS, V one
// ahead in registers.  The NG partial results (O, m, l) are folded through LDS as a
// fixed binary tree, so the result does not depend on timing.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, bool RECOMP, int NG>
__global__ __launch_bounds__(64 * NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_wave_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, SUB = 32, CPT = D / 16;
  constexpr int LDK = D + 8, LDV = D + 16;  // row pads chosen for conflict-free b128 / transpose reads
  constexpr int SLOT = SUB * LDK + SUB * LDV;
  constexpr int MSLOT = 64 * (4 * DB + 1);  // f32x4 units one wavefront hands over in the merge
  constexpr int MERGE = NG * MSLOT * 8 + 2 * 32 * (DB < NG ? DB : NG);  // hand-over area + partial Delta, uint16 units
  constexpr int LDS_ELEMS = NG * SLOT > MERGE ? NG * SLOT : MERGE;
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: scalar registers
  uint16_t* sK = smem + grp * SLOT;
  uint16_t* sV = sK + SUB * LDK;
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
  const uint32_t loff = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.ss + 8u * (lane % (D / 8))) * 2u;

  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;  // key sub-tiles with a visible key
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;
  auto jc = [&](int j) { return min(j, jlast); };  // past the wavefront's last sub-tile: fetch it again

  u32x4 pk[CPT], pv[CPT];
  uint2 bzn[4], bzc[4];  // bias slices of the next sub-tile / of the one about to be used
  auto bload = [&](int j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) bzn[g] = *(const uint2*)(bias_row + min(j * SUB + 8 * g + 4 * hl, p.S - 4));
  };

  // Q fragments: fetched coalesced, passed through the (still unused) K buffer
  bf16x8 qf[KS];
  {
    u32x4 pq[CPT];
    sub_load<D>(pq, Qb, p.ss, p.S, q0, loff);
    if (n > 0) {
      sub_load<D>(pk, Kb, p.ss, p.S, j0 * SUB, loff);
      sub_load<D>(pv, Vb, p.ss, p.S, j0 * SUB, loff);
      if (BIAS) bload(j0);
    }
    sub_store<D, LDK>(sK, pq, lane);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = lds_nat<LDK>(sK, r, ks, hl);
  }
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;

  // S^T = K Q^T of the sub-tile in the K buffer: lane = query, registers = keys
  auto stage_s = [&](f32x16& sa) {
    bf16x8 fk[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fk[ks] = lds_nat<LDK>(sK, r, ks, hl);
#pragma unroll
    for (int v = 0; v < 16; ++v) sa[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sa = mfma(fk[ks], qf[ks], sa);
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
      rescale_acc<DB>(oacc, alpha);
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
  // O^T += V^T P^T with the sub-tile in the V buffer
  auto stage_pv = [&](const bf16x8 (&pf)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      bf16x8 vf[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) vf[db] = lds_tr<LDV>(sV, 16 * t, 32 * db, lane);
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(vf[db], pf[t], oacc[db]);
    }
  };

  if (n > 0) {
    f32x16 sc, sn;
    // K(j0) -> LDS -> scores; then K(j0+NG) -> LDS with K(j0+2NG) in flight, V(j0) -> LDS with V(j0+NG) in flight
    sub_store<D, LDK>(sK, pk, lane);
    sub_load<D>(pk, Kb, p.ss, p.S, jc(j0 + NG) * SUB, loff);
    stage_s(sc);
    sub_store<D, LDK>(sK, pk, lane);
    sub_load<D>(pk, Kb, p.ss, p.S, jc(j0 + 2 * NG) * SUB, loff);
    sub_store<D, LDV>(sV, pv, lane);
    sub_load<D>(pv, Vb, p.ss, p.S, jc(j0 + NG) * SUB, loff);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
    }
    // step i: scores of sub-tile j are in sc, V(j) and K(j+NG) are in LDS, K(j+2NG) and V(j+NG) in registers
    for (int i = 0; i < n; ++i) {
      const int j = j0 + i * NG;
      softmax_max(j * SUB, sc, bzc, (j * SUB + SUB > p.S) || (CAUSAL && j * SUB + SUB - 1 > q0));
      // from here on the step is one straight-line block: the next scores run on the matrix cores
      // under the exponentials of the current ones
      if (BIAS) bload(jc(j + NG));
      stage_s(sn);
      sub_store<D, LDK>(sK, pk, lane);
      sub_load<D>(pk, Kb, p.ss, p.S, jc(j + 3 * NG) * SUB, loff);
      bf16x8 pf[2];
      softmax_exp(sc, pf);
      stage_pv(pf);
      sub_store<D, LDV>(sV, pv, lane);
      sub_load<D>(pv, Vb, p.ss, p.S, jc(j + 2 * NG) * SUB, loff);
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
      }
      sc = sn;
    }
  }

  if (NG > 1) {
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
    return;
  }
  if (q >= p.S) return;
  fwd_epilogue<DB, RECOMP>(p, oacc, m, l, b, h, q, hl, base);
}

template <int D, bool RECOMP>
hipError_t fwd_wave_r(const KP& p, hipStream_t st) {
  constexpr int NG = 4;
  const dim3 g((p.S + 31) / 32, p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) fwd_wave_kernel<D, true, true, RECOMP, NG><<<g, 64 * NG, 0, st>>>(p);
  else if (bias) fwd_wave_kernel<D, true, false, RECOMP, NG><<<g, 64 * NG, 0, st>>>(p);
  else if (causal) fwd_wave_kernel<D, false, true, RECOMP, NG><<<g, 64 * NG, 0, st>>>(p);
  else fwd_wave_kernel<D, false, false, RECOMP, NG><<<g, 64 * NG, 0, st>>>(p);
  return hipGetLastError();
}
template <int D>
hipError_t fwd_wave_d(const KP& p, bool recompute, hipStream_t st) {
  return recompute ? fwd_wave_r<D, true>(p, st) : fwd_wave_r<D, false>(p, st);
}
}  // namespace

hipError_t launch_fast_fwd_wave(const KP& p, bool recompute, hipStream_t st) {
  switch (p.D) {
    case 32: return fwd_wave_d<32>(p, recompute, st);
    case 64: return fwd_wave_d<64>(p, recompute, st);
    case 128: return launch_fast_fwd_wave128(p, recompute, st);
    default: return hipErrorInvalidValue;
  }
}
}  // namespace ssa
