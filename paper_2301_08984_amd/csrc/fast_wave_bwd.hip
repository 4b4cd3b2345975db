// dQ and dK/dV for small shares, one launch: wavefronts that never wait for each other inside the loop.
#include "wave_common.h"

namespace ssa {
namespace {

// ---------------------------------------------------------------------------
// dQ for small shares, same organisation: a work-group owns one 32-query block, its NG
// wavefronts hold the block's Q and dO fragments, LSE and Delta, and split the keys.
// Per step S^T = K Q^T and dP^T = V dO^T of the next sub-tile run on the matrix cores
// while the vector ALUs turn the current ones into dS; then dQ^T += K^T dS^T.
// The NG partial sums are added through LDS as a fixed binary tree.
// ---------------------------------------------------------------------------
template <int D, int NG>
constexpr int dq_wave_lds_elems() {
  constexpr int SLOT = 2 * (32 * (D + 24) + 32 * (D + 8)), MERGE = NG * 64 * 4 * (D / 32) * 8;
  return NG * SLOT > MERGE ? NG * SLOT : MERGE;
}
template <int D, bool BIAS, bool CAUSAL, int NG>
__device__ __forceinline__ void dq_wave_block(const KP& p, uint16_t* smem, int rank, int by, int bz_) {
  constexpr int KS = D / 16, DB = D / 32, SUB = 32, CPT = D / 16;
  constexpr int LDK = D + 24, LDV = D + 8;  // K is also read transposed: D + 24 is conflict-free both ways
  constexpr int BUF = SUB * LDK + SUB * LDV;
  constexpr int SLOT = 2 * BUF;
  constexpr int MSLOT = 64 * 4 * DB;
  static_assert(NG * SLOT <= dq_wave_lds_elems<D, NG>() && NG * 64 * 4 * DB * 8 <= dq_wave_lds_elems<D, NG>(), "LDS size");
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: scalar registers
  uint16_t* slot = smem + grp * SLOT;
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int qb = CAUSAL ? nsub - 1 - rank : rank;  // rank 0 = the block that sees the most keys
  const int q0 = qb * SUB, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const uint16_t* bias_row = BIAS ? (const uint16_t*)p.bias + ((int64_t)h * p.S + qc) * p.S : nullptr;
  const float c1 = p.scale * LOG2E;
  const uint32_t loff = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.ss + 8u * (lane % (D / 8))) * 2u;
  const uint32_t loff_g = ((uint32_t)(lane / (D / 8)) * (uint32_t)p.do_ss + 8u * (lane % (D / 8))) * 2u;

  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;

  u32x4 pk[CPT], pv[CPT];
  uint2 bzn[4], bzc[4];
  auto gload = [&](int j) {
    sub_load<D>(pk, Kb, p.ss, p.S, j * SUB, loff);
    sub_load<D>(pv, Vb, p.ss, p.S, j * SUB, loff);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzn[g] = *(const uint2*)(bias_row + min(j * SUB + 8 * g + 4 * hl, p.S - 4));
    }
  };
  auto lstore = [&](int buf) {
    sub_store<D, LDK>(slot + buf * BUF, pk, lane);
    sub_store<D, LDV>(slot + buf * BUF + SUB * LDK, pv, lane);
  };

  // Q and dO fragments: fetched coalesced, passed through the (still unused) second buffer
  bf16x8 qf[KS], gf[KS];
  {
    u32x4 pq[CPT], pg[CPT];
    sub_load<D>(pq, Qb, p.ss, p.S, q0, loff);
    sub_load<D>(pg, dOb, p.do_ss, p.S, q0, loff_g);
    if (n > 0) gload(j0);
    sub_store<D, LDK>(slot + BUF, pq, lane);
    sub_store<D, LDV>(slot + BUF + SUB * LDK, pg, lane);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = lds_nat<LDK>(slot + BUF, r, ks, hl);
      gf[ks] = lds_nat<LDV>(slot + BUF + SUB * LDK, r, ks, hl);
    }
  }
  const float nlse2 = -p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  auto stage_a = [&](int buf, f32x16& sa, f32x16& pa) {
    const uint16_t* sK = slot + buf * BUF;
    const uint16_t* sV = sK + SUB * LDK;
    bf16x8 fk[KS], fv[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fk[ks] = lds_nat<LDK>(sK, r, ks, hl);
      fv[ks] = lds_nat<LDV>(sV, r, ks, hl);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sa = mfma(fk[ks], qf[ks], sa);
      pa = mfma(fv[ks], gf[ks], pa);
    }
  };
  auto stage_v = [&](const f32x16& sa, const f32x16& pa, const uint2* bz, bf16x8 (&df)[2]) {
    float pe[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      float bl[4] = {nlse2, nlse2, nlse2, nlse2};
      if (BIAS) {
        bl[0] = fmaf(__uint_as_float(bz[g].x << 16), LOG2E, nlse2);
        bl[1] = fmaf(__uint_as_float(bz[g].x & 0xffff0000u), LOG2E, nlse2);
        bl[2] = fmaf(__uint_as_float(bz[g].y << 16), LOG2E, nlse2);
        bl[3] = fmaf(__uint_as_float(bz[g].y & 0xffff0000u), LOG2E, nlse2);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) pe[4 * g + e] = fast_exp2(fmaf(sa[4 * g + e], c1, bl[e]));
    }
    float ds[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) ds[v] = pe[v] * (pa[v] - delta);
    df[0] = pack8(&ds[0]);
    df[1] = pack8(&ds[8]);
  };
  auto stage_b = [&](int buf, const bf16x8 (&df)[2]) {
    const uint16_t* sK = slot + buf * BUF;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      bf16x8 kt_[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) kt_[db] = lds_tr<LDK>(sK, 16 * hb, 32 * db, lane);
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(kt_[db], df[hb], acc[db]);
    }
  };

  if (n > 0) {
    f32x16 sc, pc, sn, pn;
    lstore(0);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
    }
    gload(min(j0 + NG, jlast));
    stage_a(0, sc, pc);
    // one step: sub-tile j sits in LDS buffer `buf` with its products in (sc, pc); the registers hold
    // sub-tile j+NG (clamped to the wavefront's last one), which moves to the other buffer and is
    // multiplied into (sn, pn) while the vector ALUs work on (sc, pc)
    for (int i = 0; i < n; ++i) {
      const int j = j0 + i * NG, buf = i & 1;
      uint2 bz[4];
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) { bz[g] = bzc[g]; bzc[g] = bzn[g]; }
      }
      if ((j * SUB + SUB > p.S) || (CAUSAL && j * SUB + SUB - 1 > q0)) {
        // uniform; masked scores become -inf (P = 0) before anything else, so that the rest of the
        // step is one straight-line block
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = j * SUB + key_of(v, hl);
          const bool dead = key >= p.S || (CAUSAL && key > q);
          sc[v] = dead ? -INFINITY : sc[v];
        }
      }
      lstore(buf ^ 1);
      gload(min(j + 2 * NG, jlast));
      stage_a(buf ^ 1, sn, pn);
      bf16x8 df[2];
      stage_v(sc, pc, bz, df);
      stage_b(buf, df);
      sc = sn;
      pc = pn;
    }
  }

  // one 32-column block of the row, 16 bytes per lane and store (both lanes of a row are active)
  auto store_q = [&](int db, const uint2 (&o)[4]) {
    store_row32((uint16_t*)p.dQ + base + (int64_t)q * p.ss + 32 * db, o, hl, true);
  };
  if (NG > 1) {
    // every wavefront hands over its partial sums through LDS; wavefront w then folds and stores
    // the 32-column output blocks w, w+NG, ...: a fixed binary tree over the wavefronts
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
    if (q >= p.S) return;
    for (int db = grp; db < DB; db += NG) {
      uint2 o[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 x[NG];
#pragma unroll
        for (int w = 0; w < NG; ++w) x[w] = mb[(size_t)w * WSLOT + (4 * db + g) * 64 + lane];
#pragma unroll
        for (int st = NG / 2; st >= 1; st >>= 1)
#pragma unroll
          for (int w = 0; w < st; ++w) x[w] += x[w + st];
        o[g] = pack4_bf16(x[0][0], x[0][1], x[0][2], x[0][3], p.scale);
      }
      store_q(db, o);
    }
    return;
  }
  if (q >= p.S) return;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 o[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      o[g] = pack4_bf16(acc[db][4 * g], acc[db][4 * g + 1], acc[db][4 * g + 2], acc[db][4 * g + 3], p.scale);
    store_q(db, o);
  }
}

// ---------------------------------------------------------------------------
// dK, dV when the share has too few key blocks to fill the chip with key-stationary
// work-groups.  A work-group owns one 32-key block; its QG wavefronts all hold that
// block's K and V fragments and split the queries: wavefront g takes the 32-query
// sub-tiles first+g, first+g+QG, ...  Every wavefront stages its own sub-tiles
// (global -> registers -> its private double-buffered LDS slot -> operand reads), so
// the loop has no barrier: the wavefronts drift apart and one's vector-ALU and
// staging work overlaps the others' matrix products.  Per step the scores of the
// next sub-tile run on the matrix cores while the vector ALUs turn the current
// scores into P and dS, then the gradient products of the current sub-tile follow.
// The QG partial sums of dK and dV are folded through LDS as a fixed binary tree
// ((g0+g2)+(g1+g3) for QG = 4), so the result does not depend on timing.
// ---------------------------------------------------------------------------
template <int D, int QG>
constexpr int dkdv_wave_lds_elems() {
  constexpr int SLOT = 4 * 32 * (D + 24) + 2 * 2 * 2 * 32, MERGE = QG * 64 * 8 * (D / 32) * 8;
  return QG * SLOT > MERGE ? QG * SLOT : MERGE;
}
template <int D, bool BIAS, bool CAUSAL, int QG>
__device__ __forceinline__ void dkdv_wave_block(const KP& p, uint16_t* smem, int rank, int by, int bz_) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 24, SUB = 32;  // read both ways: conflict-free for b128 and transposed reads
  constexpr int CPR = D / 8, CPT = SUB * CPR / 64;
  constexpr int MAT = SUB * LD;                  // uint16 elements of one staged matrix
  constexpr int SLOT = 4 * MAT + 2 * 2 * 2 * SUB;  // two buffers of (Q, dO) + two of (lse, delta) as floats
  constexpr int MERGE = QG * 64 * 8 * DB * 8;  // uint16 units of the hand-over area
  static_assert(QG * SLOT <= dkdv_wave_lds_elems<D, QG>() && MERGE <= dkdv_wave_lds_elems<D, QG>(), "LDS size");
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: scalar registers
  uint16_t* slot = smem + grp * SLOT;
  float* sstat = (float*)(slot + 4 * MAT);
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int k0 = rank * 32, key = k0 + r;  // rank 0 = the key block that sees the most queries under a causal mask
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
  const uint16_t* biasT_row = BIAS ? (const uint16_t*)p.biasT + ((int64_t)h * p.S + kc) * p.S : nullptr;

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *(const bf16x8*)(Kb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
    vf[ks] = *(const bf16x8*)(Vb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }
  const float c1 = p.scale * LOG2E;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int first = CAUSAL ? k0 / SUB : 0;  // queries before the block's first key see none of it
  const int j0 = first + grp;               // this wavefront's sub-tiles: j0, j0+QG, ... < nsub
  const int n = j0 < nsub ? (nsub - 1 - j0) / QG + 1 : 0;
  const int jlast = j0 + (n - 1) * QG;

  const uint32_t loff_q = ((uint32_t)(lane / CPR) * (uint32_t)p.ss + 8u * (lane % CPR)) * 2u;
  const uint32_t loff_g = ((uint32_t)(lane / CPR) * (uint32_t)p.do_ss + 8u * (lane % CPR)) * 2u;
  u32x4 pq[CPT], pg[CPT];
  float pstat = 0.f;
  uint2 bzn[4], bzc[4];  // bias slices of the sub-tile in the registers / of the one about to be used
  auto gload = [&](int j) {
    sub_load<D>(pq, Qb, p.ss, p.S, j * SUB, loff_q);
    sub_load<D>(pg, dOb, p.do_ss, p.S, j * SUB, loff_g);
    const int i = min(j * SUB + r, p.S - 1);
    pstat = hl == 0 ? lse_b[i] : dl_b[i];
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzn[g] = *(const uint2*)(biasT_row + min(j * SUB + 8 * g + 4 * hl, p.S - 4));
    }
  };
  auto lstore = [&](int buf) {
    uint16_t* tq = slot + buf * 2 * MAT;
    uint16_t* tg = tq + MAT;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = lane + c * 64, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(tq + row * LD + col) = pq[c];
      *(u32x4*)(tg + row * LD + col) = pg[c];
    }
    // lanes 0..31: -LSE in the exp2 domain, lanes 32..63: Delta (arithmetic at store time, not on the in-flight load)
    sstat[buf * 2 * SUB + lane] = hl == 0 ? -pstat * LOG2E : pstat;
  };
  // scores and dP of the sub-tile staged in `buf`
  auto stage_a = [&](int buf, f32x16& sa, f32x16& pa) {
    const uint16_t* tq = slot + buf * 2 * MAT;
    const uint16_t* tg = tq + MAT;
    bf16x8 fq[KS], fg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fq[ks] = lds_nat<LD>(tq, r, ks, hl);
      fg[ks] = lds_nat<LD>(tg, r, ks, hl);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sa = mfma(fq[ks], kf[ks], sa);
      pa = mfma(fg[ks], vf[ks], pa);
    }
  };
  // P and dS as packed bf16 operands
  auto stage_v = [&](int buf, const f32x16& sa, const f32x16& pa, const uint2* bz, bf16x8 (&pf)[2],
                     bf16x8 (&df)[2]) {
    const float* tl = sstat + buf * 2 * SUB;
    const float* td = tl + SUB;
    float pr[16], ds[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 l4 = *(const f32x4*)(tl + 8 * g + 4 * hl);
      float bl[4] = {0.f, 0.f, 0.f, 0.f};
      if (BIAS) {
        const uint2 u = bz[g];
        bl[0] = __uint_as_float(u.x << 16) * LOG2E; bl[1] = __uint_as_float(u.x & 0xffff0000u) * LOG2E;
        bl[2] = __uint_as_float(u.y << 16) * LOG2E; bl[3] = __uint_as_float(u.y & 0xffff0000u) * LOG2E;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) pr[4 * g + e] = fast_exp2(fmaf(sa[4 * g + e], c1, BIAS ? bl[e] + l4[e] : l4[e]));
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 d4 = *(const f32x4*)(td + 8 * g + 4 * hl);
#pragma unroll
      for (int e = 0; e < 4; ++e) ds[4 * g + e] = pr[4 * g + e] * (pa[4 * g + e] - d4[e]);
    }
    pf[0] = pack8(&pr[0]); pf[1] = pack8(&pr[8]);
    df[0] = pack8(&ds[0]); df[1] = pack8(&ds[8]);
  };
  // dV += dO^T P, dK += Q^T dS
  auto stage_b = [&](int buf, const bf16x8 (&pf)[2], const bf16x8 (&df)[2]) {
    const uint16_t* tq = slot + buf * 2 * MAT;
    const uint16_t* tg = tq + MAT;
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      bf16x8 tg_[DB], tq_[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tg_[db] = lds_tr<LD>(tg, 16 * hb, 32 * db, lane);
        tq_[db] = lds_tr<LD>(tq, 16 * hb, 32 * db, lane);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dv[db] = mfma(tg_[db], pf[hb], dv[db]);
        dk[db] = mfma(tq_[db], df[hb], dk[db]);
      }
    }
  };

  if (n > 0) {
    f32x16 sc, pc, sn, pn;
    gload(j0);
    lstore(0);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
    }
    gload(min(j0 + QG, jlast));
    stage_a(0, sc, pc);
    // one step: sub-tile j sits in LDS buffer `buf` with its scores in (sc, pc); the registers hold
    // sub-tile j+QG (clamped to the wavefront's last one), which moves to the other buffer and has
    // its scores computed into (sn, pn) while the vector ALUs work on (sc, pc)
    for (int i = 0; i < n; ++i) {
      const int j = j0 + i * QG, buf = i & 1;
      uint2 bz[4];
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) { bz[g] = bzc[g]; bzc[g] = bzn[g]; }
      }
      if ((j * SUB + SUB > p.S) || (k0 + 32 > p.S) || (CAUSAL && j * SUB < k0 + 31)) {
        // uniform; masked scores become -inf (P = 0) before anything else, so that the rest of the
        // step is one straight-line block
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int i = j * SUB + key_of(v, hl);
          const bool dead = i >= p.S || key >= p.S || (CAUSAL && key > i);
          sc[v] = dead ? -INFINITY : sc[v];
        }
      }
      lstore(buf ^ 1);
      gload(min(j + 2 * QG, jlast));
      bf16x8 pf[2], df[2];
      stage_a(buf ^ 1, sn, pn);
      stage_v(buf, sc, pc, bz, pf, df);
      stage_b(buf, pf, df);
      sc = sn;
      pc = pn;
    }
  }

  // one 32-column block of the row, 16 bytes per lane and store (both lanes of a row are active)
  auto store_kv = [&](int db, const uint2 (&a)[4], const uint2 (&c)[4]) {
    store_row32((uint16_t*)p.dK + base + (int64_t)key * p.ss + 32 * db, a, hl, true);
    store_row32((uint16_t*)p.dV + base + (int64_t)key * p.ss + 32 * db, c, hl, true);
  };
  if (QG > 1) {
    // every wavefront hands over its partial sums through LDS; wavefront w then folds and stores
    // the 32-column output blocks w, w+QG, ...  The fold is a fixed binary tree over the
    // wavefronts ((g0+g2)+(g1+g3) for QG = 4), so the result does not depend on timing.
    constexpr int WSLOT = 64 * 8 * DB;  // f32x4 units per wavefront
    f32x4* mb = (f32x4*)smem;
    __syncthreads();
    f32x4* my = mb + (size_t)grp * WSLOT + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        my[(8 * db + g) * 64] = f32x4{dk[db][4 * g], dk[db][4 * g + 1], dk[db][4 * g + 2], dk[db][4 * g + 3]};
        my[(8 * db + 4 + g) * 64] = f32x4{dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3]};
      }
    __syncthreads();
    if (key >= p.S) return;
    for (int db = grp; db < DB; db += QG) {
      uint2 a[4], c[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 xk[QG], xv[QG];
#pragma unroll
        for (int w = 0; w < QG; ++w) {
          xk[w] = mb[(size_t)w * WSLOT + (8 * db + g) * 64 + lane];
          xv[w] = mb[(size_t)w * WSLOT + (8 * db + 4 + g) * 64 + lane];
        }
#pragma unroll
        for (int st = QG / 2; st >= 1; st >>= 1)
#pragma unroll
          for (int w = 0; w < st; ++w) { xk[w] += xk[w + st]; xv[w] += xv[w + st]; }
        a[g] = pack4_bf16(xk[0][0], xk[0][1], xk[0][2], xk[0][3], p.scale);
        c[g] = pack4_bf16(xv[0][0], xv[0][1], xv[0][2], xv[0][3], 1.f);
      }
      store_kv(db, a, c);
    }
    return;
  }
  if (key >= p.S) return;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 a[4], c[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      a[g] = pack4_bf16(dk[db][4 * g], dk[db][4 * g + 1], dk[db][4 * g + 2], dk[db][4 * g + 3], p.scale);
      c[g] = pack4_bf16(dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3], 1.f);
    }
    store_kv(db, a, c);
  }
}

// ---------------------------------------------------------------------------
// One launch for dQ and dK/dV.  Both only read what the recompute pass left (LSE, Delta, dO) and
// each alone leaves compute units idle behind its longest chain, so their work-groups share one
// grid: position pos of a (row, head) unit is the dK/dV block of rank pos/2 (even pos) or the dQ
// block of rank pos/2 (odd pos), heaviest first over the whole launch, and the light work-groups
// of one fill in behind the heavy ones of the other.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL>
__global__ __launch_bounds__(256) void bwd_wave_kernel(KP p) {
  constexpr int NG = 4;
  constexpr int LDS_ELEMS = dq_wave_lds_elems<D, NG>() > dkdv_wave_lds_elems<D, NG>() ? dq_wave_lds_elems<D, NG>()
                                                                                       : dkdv_wave_lds_elems<D, NG>();
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int units = gridDim.y * gridDim.z;
  const int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int pos = lin / units, unit = lin % units;
  const int by = unit % gridDim.y, bz_ = unit / gridDim.y;
  if ((pos & 1) == 0) dkdv_wave_block<D, BIAS, CAUSAL, NG>(p, smem, pos >> 1, by, bz_);
  else dq_wave_block<D, BIAS, CAUSAL, NG>(p, smem, pos >> 1, by, bz_);
}

template <int D>
hipError_t bwd_wave_d(const KP& p, hipStream_t st) {
  const dim3 g(2 * ((p.S + 31) / 32), p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) bwd_wave_kernel<D, true, true><<<g, 256, 0, st>>>(p);
  else if (bias) bwd_wave_kernel<D, true, false><<<g, 256, 0, st>>>(p);
  else if (causal) bwd_wave_kernel<D, false, true><<<g, 256, 0, st>>>(p);
  else bwd_wave_kernel<D, false, false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fast_bwd_wave(const KP& p, hipStream_t st) {
  switch (p.D) {
    case 32: return bwd_wave_d<32>(p, st);
    case 64: return bwd_wave_d<64>(p, st);
    case 128: return bwd_wave_d<128>(p, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace ssa
