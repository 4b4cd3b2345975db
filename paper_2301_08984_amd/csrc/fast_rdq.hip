// Recompute pass and dQ in one kernel, for shares whose kernels are bound by the vector arithmetic
// per score element (head size 32: two matrix steps against ten vector instructions per element).
#include "mfma_common.h"

namespace ssa {
namespace {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

// ---------------------------------------------------------------------------
// A query block walks its keys once and leaves O (for Delta, the gate gradient and the pre-gated
// dO copy), the softmax statistics AND dQ, instead of once for the statistics and once more for dQ
// with the same scores, bias additions and exponentials.  dQ needs Delta = sum_j P_ij dP_ij, which
// is only known after the last key; with the unnormalised probabilities p~ of the online softmax
//     dQ_i = scale / l * ( sum_j (p~_ij dP_ij) K_j  -  Delta' * sum_j p~_ij K_j ),   l = sum_j p~_ij,
// so two products are accumulated (A1 with p~ dP, A2 with p~) and combined at the end.  The
// two terms cancel where a row is peaked (dS -> 0), so Delta' must be the mean the matrix cores
// actually formed: Delta' = sum_j bf16(p~ dP) / sum_j bf16(p~), both sums over the SAME rounded
// operands that went into A1 and A2 (a one-hot row then gives A1 - Delta' A2 = 0 up to the rounding
// of one division; with the mean of the unrounded values the error of such rows is 2^-9 |dP| |K|).
// The packed operands are summed pairwise by v_dot2c_f32_bf16 against (1, 1): half an instruction
// per element and sum.  l' = sum_j bf16(p~) also normalises O and gives the LSE, so the row sum
// costs no separate addition.  The other backward kernels use Delta = rowsum(dO * O) from the
// epilogue as before.
//
// Work-group: four wavefronts of 32 queries sharing 64-key K / V tiles (two buffers, one barrier per
// tile), as the forward kernel for large shares; K and V are both read as stored (scores, dP) and
// transposed (A1 / A2, O).  A tile is taken as two 32-key blocks, each a complete online-softmax
// step: that and 32-bit buffer offsets keep a wavefront within 168 registers, and three wavefronts
// per SIMD overlap the vector and matrix work better than a longer software pipeline does with two
// (measured on the triangle shape: 141 against 158 us per launch).
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(BIAS && CAUSAL ? 2 : 3, BIAS && CAUSAL ? 2 : 3))) void rdq_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, NT = 256, BM = 128;
  constexpr int LDT = D + 24;  // conflict-free for b128 and transposed reads
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  constexpr int TILE_ELEMS = 2 * BN * LDT;
  constexpr int KV_ELEMS = 2 * TILE_ELEMS;
  constexpr int BIAS_ELEMS = BIAS ? BIAS_TILE_ELEMS * 4 : 0;  // one parked bias tile per wavefront
  __shared__ __attribute__((aligned(16))) uint16_t smem[KV_ELEMS + BIAS_ELEMS];
  const int tid = threadIdx.x;
  const int lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const BlockId blk = xcd_block_id(BIAS && bias_rows_first(gridDim.y, p.S));
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * BM;  // long (late) causal blocks first
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  BiasTile bt;
  if (BIAS)
    bt.init((const uint16_t*)p.bias + (int64_t)h * p.S * p.S, q0, p.S, smem + KV_ELEMS + w * BIAS_TILE_ELEMS, lane);

  // Q and the gradient with respect to the un-gated output, in operand layout.  Gated: dO = dY * gate,
  // rounded to bf16 with the arithmetic of the epilogue, which writes the same values for the later kernels
  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    const int64_t at = base + (int64_t)qc * p.ss + 16 * ks + 8 * hl;
    qf[ks] = *(const bf16x8*)((const uint16_t*)p.Q + at);
    const u32x4 dy = *(const u32x4*)((const uint16_t*)p.dY + at);
    if (p.gated) {
      const u32x4 gg = *(const u32x4*)((const uint16_t*)p.G + at);
      union { uint16_t s[8]; bf16x8 v; } o;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float go = (e & 1) ? __uint_as_float(dy[e >> 1] & 0xffff0000u) : __uint_as_float(dy[e >> 1] << 16);
        const float gl = (e & 1) ? __uint_as_float(gg[e >> 1] & 0xffff0000u) : __uint_as_float(gg[e >> 1] << 16);
        const float gt = fast_rcp(1.f + fast_exp2(-gl * LOG2E));
        o.s[e] = f2bf(go * gt);
      }
      gf[ks] = o.v;
    } else {
      union { u32x4 u; bf16x8 v; } o;
      o.u = dy;
      gf[ks] = o.v;
    }
  }
  union { uint32_t u; bf16x2 v; } one_pair;
  one_pair.u = 0x3f803f80u;
  const bf16x2 ones2 = one_pair.v;
  f32x16 oacc[DB], a1[DB], a2[DB];
  float lsum = 0.f, dsum = 0.f;  // this half-wave's part of l' and delta'
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { oacc[db][v] = 0.f; a1[db][v] = 0.f; a2[db][v] = 0.f; }
  float m = -1e30f;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + BM, p.S) + BN - 1) / BN);
  int wtiles = ntiles;  // tiles holding at least one key visible to this wavefront
  if (CAUSAL) wtiles = min(ntiles, (min(q0 + 32, p.S) + BN - 1) / BN);
  if (q0 >= p.S) wtiles = 0;

  // K / V tiles are fetched with buffer loads whose descriptor starts at the tile and ends with the
  // (row, head) slice: the lane offsets never change, and rows past S - 1 arrive as zeros (their
  // scores are masked, their dP is 0 * 0).  The slice is shorter than 2 GiB (checked on the host).
  const uint32_t ss2 = (uint32_t)p.ss * 2u;
  const uint32_t slice = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);
  uint32_t goff[CPT];
#pragma unroll
  for (int c = 0; c < CPT; ++c) {
    const int idx = tid + c * NT;
    goff[c] = (uint32_t)(idx / CPR) * ss2 + (uint32_t)(idx % CPR) * 16u;
  }
  u32x4 pk[CPT], pv[CPT];
  auto gload = [&](int kt) {
    const uint32_t boff = (uint32_t)(kt * BN) * ss2;  // kt * BN < S
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)Kb + boff), 0, (int)(slice - boff), 0x00020000);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)Vb + boff), 0, (int)(slice - boff), 0x00020000);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      pk[c] = __builtin_amdgcn_raw_buffer_load_b128(rk, goff[c], 0, 0);
      pv[c] = __builtin_amdgcn_raw_buffer_load_b128(rv, goff[c], 0, 0);
    }
  };
  auto stage = [&](uint16_t* dK) {
    uint16_t* dV = dK + BN * LDT;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(dK + row * LDT + col) = pk[c];
      *(u32x4*)(dV + row * LDT + col) = pv[c];
    }
  };
  // one 32-key block of a tile (K at sK, V behind it): scores and dP, online softmax, the three products and the sums
  auto block = [&](const uint16_t* sK, int kb, int k0) {
    const uint16_t* sV = sK + BN * LDT;
    f32x16 sa, pa;
    {
      bf16x8 fk[KS], fv[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        fk[ks] = lds_nat<LDT>(sK, 32 * kb + r, ks, hl);
        fv[ks] = lds_nat<LDT>(sV, 32 * kb + r, ks, hl);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa = mfma(fk[ks], qf[ks], sa);
        pa = mfma(fv[ks], gf[ks], pa);
      }
    }
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 u = bt.read(r, 32 * kb + 8 * g + 4 * hl);
        // natural units here; the change to base 2 rides on the subtraction of the maximum below
        sa[4 * g + 0] = fmaf(sa[4 * g + 0], p.scale, __uint_as_float(u.x << 16));
        sa[4 * g + 1] = fmaf(sa[4 * g + 1], p.scale, __uint_as_float(u.x & 0xffff0000u));
        sa[4 * g + 2] = fmaf(sa[4 * g + 2], p.scale, __uint_as_float(u.y << 16));
        sa[4 * g + 3] = fmaf(sa[4 * g + 3], p.scale, __uint_as_float(u.y & 0xffff0000u));
      }
    }
    if ((k0 + 32 > p.S) || (CAUSAL && k0 + 31 > q0)) {
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
    // the running maximum is raised only when exceeded by more than 2^8, so the rescale is skipped
    // on most blocks; probabilities stay below 2^8, harmless in fp32/bf16 range
    if (__builtin_amdgcn_ballot_w64(rmax > m + 8.f) != 0) {
      const float mn = fmaxf(m, rmax);
      const float alpha = fast_exp2(m - mn);
      m = mn;
      lsum *= alpha;
      dsum *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) { oacc[db][v] *= alpha; a1[db][v] *= alpha; a2[db][v] *= alpha; }
    }
    bf16x8 pf[2], df[2];
    {
      float pr[16], dp[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        pr[v] = fast_exp2(fmaf(sa[v], BIAS ? LOG2E : c1, -m));
        dp[v] = pr[v] * pa[v];
      }
      pf[0] = pack8(&pr[0]);
      pf[1] = pack8(&pr[8]);
      df[0] = pack8(&dp[0]);
      df[1] = pack8(&dp[8]);
    }
    // the sums run over the rounded operands
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      union { bf16x8 v; bf16x2 h[4]; } a, c;
      a.v = pf[j];
      c.v = df[j];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        lsum = __builtin_amdgcn_fdot2_f32_bf16(a.h[e], ones2, lsum, false);
        dsum = __builtin_amdgcn_fdot2_f32_bf16(c.h[e], ones2, dsum, false);
      }
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      bf16x8 vt[DB], kt[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        vt[db] = lds_tr<LDT>(sV, 32 * kb + 16 * j, 32 * db, lane);
        kt[db] = lds_tr<LDT>(sK, 32 * kb + 16 * j, 32 * db, lane);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        oacc[db] = mfma(vt[db], pf[j], oacc[db]);
        a2[db] = mfma(kt[db], pf[j], a2[db]);
        a1[db] = mfma(kt[db], df[j], a1[db]);
      }
    }
  };
  auto tile = [&](const uint16_t* sK, int k0) {
    block(sK, 0, k0);
    block(sK, 1, k0 + 32);
  };

  // two tile buffers and one barrier per tile: while a tile is multiplied the next one is already in
  // registers; it is written to the other buffer after the multiplication, which every wavefront
  // finished reading before the previous barrier
  if (ntiles > 0) {
    gload(0);
    if (BIAS) bt.load(0);
    stage(smem);
    if (BIAS) bt.park(lane);
    if (1 < ntiles) {
      gload(1);
      if (BIAS) bt.load(1);
    }
  }
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    uint16_t* cK = smem + (kt & 1) * TILE_ELEMS;
    uint16_t* nK = smem + ((kt + 1) & 1) * TILE_ELEMS;
    if (kt < wtiles) tile(cK, kt * BN);
    if (kt + 1 < ntiles) {
      stage(nK);
      if (BIAS) bt.park(lane);
      if (kt + 2 < ntiles) {
        gload(kt + 2);
        if (BIAS) bt.load(kt + 2);
      }
    }
    __syncthreads();
  }
  if (q >= p.S) return;
  const float l = half_sum(lsum);
  const float inv = 1.f / l;
  const float dmean = half_sum(dsum) * inv;
  const float f = p.scale * inv;
  uint16_t* out = (uint16_t*)p.dQ + base + (int64_t)q * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 o[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      o[g] = pack4_bf16(fmaf(-dmean, a2[db][4 * g], a1[db][4 * g]), fmaf(-dmean, a2[db][4 * g + 1], a1[db][4 * g + 1]),
                        fmaf(-dmean, a2[db][4 * g + 2], a1[db][4 * g + 2]),
                        fmaf(-dmean, a2[db][4 * g + 3], a1[db][4 * g + 3]), f);
    store_row32(out + 32 * db, o, hl, true);
  }
  fwd_epilogue_rowsum<DB, true>(p, oacc, m, l, b, h, q, hl, base);
}

template <int D>
hipError_t rdq_launch(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 127) / 128, p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) rdq_fast_kernel<D, true, true><<<g, 256, 0, st>>>(p);
  else if (bias) rdq_fast_kernel<D, true, false><<<g, 256, 0, st>>>(p);
  else if (causal) rdq_fast_kernel<D, false, true><<<g, 256, 0, st>>>(p);
  else rdq_fast_kernel<D, false, false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fast_recompute_dq(const KP& p, hipStream_t st) { return rdq_launch<32>(p, st); }

}  // namespace ssa
