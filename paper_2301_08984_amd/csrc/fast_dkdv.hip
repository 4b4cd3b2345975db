// Specialised dK/dV and bias-gradient kernels, and the bias transpose (see the comments above each).
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

// ---------------------------------------------------------------------------
// dK, dV (optional dense bf16 bias read from its transposed copy, optional causal mask).  Each wavefront
// keeps a 32-key block of K and V and both gradient accumulators in registers and
// walks the queries in 32-row sub-blocks with a software pipeline: while the vector
// ALUs turn the scores of sub-block j into P and dS, the matrix cores already
// produce the scores of sub-block j+1 and consume P/dS of sub-block j-1.
// Q / dO tiles (64 rows) are double-buffered in LDS, one barrier per tile; the next
// tile travels global -> registers meanwhile.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, int NW, bool SLICE32>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(D <= 32 ? (BIAS && CAUSAL ? 2 : 3) : 1, D <= 32 ? (BIAS && CAUSAL ? 2 : 3) : 1))) void dkdv_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 24, NT = 64 * NW, BK = 32 * NW;  // tiles read both ways
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  __shared__ __attribute__((aligned(16))) uint16_t sQ[2][BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sG[2][BN * LD];
  __shared__ __attribute__((aligned(16))) float sL[2][BN];
  __shared__ __attribute__((aligned(16))) float sD[2][BN];
  __shared__ __attribute__((aligned(16))) uint16_t sBias[BIAS ? NW * BIAS_TILE_ELEMS : 8];  // one parked tile per wavefront
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const BlockId blk = xcd_block_id(BIAS && bias_rows_first(gridDim.y, p.S));
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int kblk = blk.x * BK;  // early key blocks see the most queries under a causal mask
  const int k0 = kblk + 32 * w, key = k0 + r;
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
  // bias comes from the transposed copy biasT[h][key][query], so that a lane (= key) finds four
  // consecutive queries in 8 bytes
  BiasTile bt;
  if (BIAS) bt.init((const uint16_t*)p.biasT + (int64_t)h * p.S * p.S, k0, p.S, sBias + w * BIAS_TILE_ELEMS, lane);
  auto bload = [&](int qt) { bt.load(qt); };

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
  const int ntiles = (p.S + BN - 1) / BN;
  const int first = CAUSAL ? kblk / BN : 0;  // queries before the block's first key see none of it

  u32x4 pq[CPT], pg[CPT];
  float pstat = 0.f;
  // SLICE32: the (row, head) slices of Q and dO are shorter than 2 GiB (decided on the host).  The
  // tiles are then fetched with buffer loads whose descriptor starts at the tile and ends with the
  // slice: lane offsets that never change (no 64-bit address per load), and rows past S - 1 arrive as
  // zeros: their scores are masked, and their dS is P * (0 - Delta) with P = 0.
  uint32_t goq[SLICE32 ? CPT : 1], gog[SLICE32 ? CPT : 1];
  if (SLICE32) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT;
      goq[c] = (uint32_t)(idx / CPR) * ((uint32_t)p.ss * 2u) + (uint32_t)(idx % CPR) * 16u;
      gog[c] = (uint32_t)(idx / CPR) * ((uint32_t)p.do_ss * 2u) + (uint32_t)(idx % CPR) * 16u;
    }
  }
  auto gload = [&](int qt) {
    if (SLICE32) {
      const uint32_t bq = (uint32_t)(qt * BN) * ((uint32_t)p.ss * 2u), bg = (uint32_t)(qt * BN) * ((uint32_t)p.do_ss * 2u);
      const uint32_t nq = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2), ng = (uint32_t)(((int64_t)(p.S - 1) * p.do_ss + D) * 2);
      const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)Qb + bq), 0, (int)(nq - bq), 0x00020000);
      const __amdgpu_buffer_rsrc_t rg = __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)dOb + bg), 0, (int)(ng - bg), 0x00020000);
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        pq[c] = __builtin_amdgcn_raw_buffer_load_b128(rq, goq[c], 0, 0);
        pg[c] = __builtin_amdgcn_raw_buffer_load_b128(rg, gog[c], 0, 0);
      }
    } else {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int idx = tid + c * NT, row = min(qt * BN + idx / CPR, p.S - 1), col = (idx % CPR) * 8;
        pq[c] = *(const u32x4*)(Qb + (int64_t)row * p.ss + col);
        pg[c] = *(const u32x4*)(dOb + (int64_t)row * p.do_ss + col);
      }
    }
    if (tid < 2 * BN) {
      const int i = min(qt * BN + (tid & (BN - 1)), p.S - 1);
      pstat = tid < BN ? lse_b[i] : dl_b[i];  // LSE is scaled when stored to LDS, not on the in-flight load
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(&sQ[buf][row * LD + col]) = pq[c];
      *(u32x4*)(&sG[buf][row * LD + col]) = pg[c];
    }
    if (tid < BN) sL[buf][tid] = -pstat * LOG2E;  // stored negated: one fused multiply-add per score
    else if (tid < 2 * BN) sD[buf][tid - BN] = pstat;
  };
  // scores and dP of one 32-query sub-block
  auto stage_a = [&](const uint16_t* tq, const uint16_t* tg, int sub, f32x16& sa, f32x16& pa) {
    bf16x8 fq[KS], fg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      fq[ks] = lds_nat<LD>(tq, 32 * sub + r, ks, hl);
      fg[ks] = lds_nat<LD>(tg, 32 * sub + r, ks, hl);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sa = mfma(fq[ks], kf[ks], sa);
      pa = mfma(fg[ks], vf[ks], pa);
    }
  };
  // P and dS of one sub-block, as packed bf16 operands
  auto stage_v = [&](const float* tl, const float* td, int i0, int sub, const f32x16& sa, const f32x16& pa,
                     const uint2* bz, bf16x8 (&pf)[2], bf16x8 (&df)[2], auto edge_tag) {
    constexpr bool edge = decltype(edge_tag)::value;
    float pr[16], ds[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4 l4 = *(const f32x4*)(tl + 32 * sub + 8 * g + 4 * hl);
      const f32x4 d4 = *(const f32x4*)(td + 32 * sub + 8 * g + 4 * hl);
      float bl[4] = {0.f, 0.f, 0.f, 0.f};
      if (BIAS) {
        const uint2 u = bz[4 * sub + g];
        bl[0] = __uint_as_float(u.x << 16); bl[1] = __uint_as_float(u.x & 0xffff0000u);
        bl[2] = __uint_as_float(u.y << 16); bl[3] = __uint_as_float(u.y & 0xffff0000u);
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        // with a bias: natural units first, the change to base 2 rides on the subtraction of the LSE
        float pe = BIAS ? fast_exp2(fmaf(fmaf(sa[4 * g + e], p.scale, bl[e]), LOG2E, l4[e]))
                        : fast_exp2(fmaf(sa[4 * g + e], c1, l4[e]));
        if (edge) {
          const int i = i0 + 32 * sub + 8 * g + 4 * hl + e;
          const bool dead = i >= p.S || key >= p.S || (CAUSAL && key > i);
          pe = dead ? 0.f : pe;
        }
        pr[4 * g + e] = pe;
        ds[4 * g + e] = pe * (pa[4 * g + e] - d4[e]);
      }
    }
    pf[0] = pack8(&pr[0]); pf[1] = pack8(&pr[8]);
    df[0] = pack8(&ds[0]); df[1] = pack8(&ds[8]);
  };
  // dV += dO^T P, dK += Q^T dS for one sub-block
  auto stage_b = [&](const uint16_t* tq, const uint16_t* tg, int sub, const bf16x8 (&pf)[2], const bf16x8 (&df)[2]) {
#pragma unroll
    for (int hb = 0; hb < 2; ++hb) {
      bf16x8 tg_[DB], tq_[DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tg_[db] = lds_tr<LD>(tg, 32 * sub + 16 * hb, 32 * db, lane);
        tq_[db] = lds_tr<LD>(tq, 32 * sub + 16 * hb, 32 * db, lane);
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        dv[db] = mfma(tg_[db], pf[hb], dv[db]);
        dk[db] = mfma(tq_[db], df[hb], dk[db]);
      }
    }
  };

  if (first < ntiles) {
    gload(first);
    lstore(first & 1);
    if (first + 1 < ntiles) gload(first + 1);
    if (BIAS) bload(first);
  }
  for (int qt = first; qt < ntiles; ++qt) {
    const int i0 = qt * BN;
    __syncthreads();
    if (qt + 1 < ntiles) lstore((qt + 1) & 1);
    if (qt + 2 < ntiles) gload(qt + 2);
    if (BIAS) {
      bt.park(lane);
      if (qt + 1 < ntiles) bload(qt + 1);
    }
    if (k0 >= p.S || (CAUSAL && i0 + BN - 1 < k0)) continue;  // no visible pair for this wavefront
    const uint16_t* tq = sQ[qt & 1];
    const uint16_t* tg = sG[qt & 1];
    const float* tl = sL[qt & 1];
    const float* td = sD[qt & 1];
    const bool edge = (i0 + BN > p.S) || (k0 + 32 > p.S) || (CAUSAL && i0 < k0 + 31);
    // one straight-line block per tile: A0 | A1 with V0 | B0 with V1 | B1, where A = scores and dP
    // on the matrix cores, V = P and dS on the vector ALUs, B = gradient products
    uint2 bz[8];
    if (BIAS && D > 32) {
#pragma unroll
      for (int j = 0; j < 8; ++j) bz[j] = bt.read(r, 8 * j + 4 * hl);
    }
    auto tile = [&](auto edge_tag) {
      // D = 128: keeps the 32 operand reads inside this block; they are common to both variants of
      // the tile and would otherwise all be hoisted above the branch, out of reach of the schedule
      // below, where their 128 registers push the transposed operands into the accumulation file
      // (measured: 929 -> 785 us on the long-sequence GPT share; smaller D is faster without)
      if (D >= 128) asm volatile("" ::: "memory");
      if constexpr (D <= 32) {
        // Head size 32: the vector arithmetic binds, not the matrix cores.  One sub-block at a time
        // keeps the wavefront within 168 registers, and the third wavefront per SIMD overlaps more
        // than the pipeline below does with two
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
          f32x16 sa, pa;
          bf16x8 pf[2], df[2];
          if (BIAS) {
#pragma unroll
            for (int g = 0; g < 4; ++g) bz[4 * sub + g] = bt.read(r, 32 * sub + 8 * g + 4 * hl);
          }
          stage_a(tq, tg, sub, sa, pa);
          stage_v(tl, td, i0, sub, sa, pa, bz, pf, df, edge_tag);
          stage_b(tq, tg, sub, pf, df);
        }
        return;
      }
      f32x16 sa0, pa0, sa1, pa1;
      bf16x8 pf0[2], df0[2], pf1[2], df1[2];
      stage_a(tq, tg, 0, sa0, pa0);
      stage_a(tq, tg, 1, sa1, pa1);
      stage_v(tl, td, i0, 0, sa0, pa0, bz, pf0, df0, edge_tag);
      stage_b(tq, tg, 0, pf0, df0);
      stage_v(tl, td, i0, 1, sa1, pa1, bz, pf1, df1, edge_tag);
      stage_b(tq, tg, 1, pf1, df1);
      // A0
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
      for (int j = 0; j < 2 * KS - 4; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
      // A1 with V0
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
      for (int j = 0; j < 2 * KS; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
      }
      // B0 with V1
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      for (int j = 0; j < 4 * DB; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
      }
      // B1
      __builtin_amdgcn_sched_group_barrier(0x100, 8, 0);
      for (int j = 0; j < 4 * DB; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
      }
    };
    if (edge) tile(std::true_type{});
    else tile(std::false_type{});
  }
  if (key >= p.S) return;
  uint16_t* oK = (uint16_t*)p.dK + base + (int64_t)key * p.ss;
  uint16_t* oV = (uint16_t*)p.dV + base + (int64_t)key * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 a[4], c[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      a[g] = pack4_bf16(dk[db][4 * g], dk[db][4 * g + 1], dk[db][4 * g + 2], dk[db][4 * g + 3], p.scale);
      c[g] = pack4_bf16(dv[db][4 * g], dv[db][4 * g + 1], dv[db][4 * g + 2], dv[db][4 * g + 3], 1.f);
    }
    store_row32(oK + 32 * db, a, hl, true);
    store_row32(oV + 32 * db, c, hl, true);
  }
}

// ---------------------------------------------------------------------------
// bias gradient, LDS-tiled: a work-group owns a 64-query x 64-key tile of one head (four
// wavefronts, 32x32 each, lane = query) and walks rows in order; every row's Q, dO, K, V
// slices of the tile are fetched once per work-group with fully coalesced loads, staged in
// double-buffered LDS, and read by the four wavefronts (a quarter of the cache-line traffic of
// per-wavefront fetches).  When one head's tiles are too few to fill the chip the rows are
// cut into groups of p.sm_gw consecutive global rows (grid z): each (group, tile) sums its
// rows in order into a partial kept in the workspace, resumed when a chunk boundary cuts the
// group, and the groups are summed in index order afterwards, so the result never depends
// on k.  With a single group the sum continues directly in the output.
// ---------------------------------------------------------------------------
// At D = 32 four work-groups fill a compute unit exactly (4 x 40 KB of LDS, 128 registers per lane),
// which is also what a 1024 x 1024 head needs for all its tiles to be resident at once; the per-row
// statistics therefore live in the padding of the Q tile's rows instead of arrays of their own.
// HP = 2 (D = 32, heads side by side in memory): eight wavefronts cover the same tile of two
// neighbouring heads, whose row slices are fetched together as 128 contiguous bytes: whole cache
// lines instead of halves, at twice the bytes per cycle through the load path.
template <int D, bool CAUSAL, int HP>
__global__ __launch_bounds__(256 * HP)
__attribute__((amdgpu_waves_per_eu(D <= 32 ? 4 : 1, D <= 32 ? 4 : (D <= 64 ? 2 : 1))))
void dbias_tile_kernel(KP p) {
  constexpr int KS = D / 16, LD = D + 8, CPR = D / 8;
  constexpr int CPT = 64 * CPR / 256;  // 16-byte chunks per thread per tensor tile
  static_assert(HP == 1 || CPT == 1, "two heads per work-group: D = 32 only");
  __shared__ __attribute__((aligned(16))) uint16_t sT[2][4][HP][64 * LD];  // Q, dO, K, V
  const int tid = threadIdx.x, lane = tid & 63, w = (tid >> 6) & 3, hsel = tid >> 8, r = lane & 31, hl = lane >> 5;
  const int Hc = (p.h1 - p.h0) / HP;  // head groups
  // consecutive tiles (same head, neighbouring query tiles, all key tiles) run on one XCD, so a
  // row's Q/dO/K/V slices are fetched into few L2s instead of all eight
  const BlockId blk = xcd_block_id();
  const int hA = p.h0 + (blk.z % Hc) * HP;  // first head of the work-group
  const int h = hA + hsel;
  const int q0t = blk.y * 64, k0t = blk.x * 64;
  const int wq = w >> 1, wk = w & 1;
  const int q0 = q0t + 32 * wq, k0 = k0t + 32 * wk;
  const int q = q0 + r, qc = min(q, p.S - 1);
  // rows of this work-group: the chunk, or the part of one row group inside the chunk
  int bfirst = p.b0, blast = p.b1;
  float* dst;
  bool resume;
  if (p.sm_partial) {
    const int g = p.b0 / p.sm_gw + blk.z / Hc;
    bfirst = max(g * p.sm_gw, p.b0);
    blast = min((g + 1) * p.sm_gw, p.b1);
    dst = p.sm_partial + ((int64_t)((g - p.sm_g0) % p.sm_ring) * p.sm_hs + (h - p.sm_h0)) * p.S * p.S + (int64_t)qc * p.S;
    resume = max(g * p.sm_gw, p.share_b0) < p.b0;
  } else {
    dst = p.dbias_acc + ((int64_t)h * p.S + qc) * p.S;
    resume = p.dbias_accumulate != 0;
  }
  if (bfirst >= blast) return;
  const bool skip = CAUSAL && k0t > q0t + 63;  // whole tile above the diagonal: gradient is zero
  float acc[16], bz[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int k = min(k0 + key_of(v, hl), p.S - 1);
    acc[v] = (resume && !skip) ? dst[k] : 0.f;
    bz[v] = bf2f(((const uint16_t*)p.bias)[((int64_t)h * p.S + qc) * p.S + k]) * LOG2E;
  }
  const float c1 = p.scale * LOG2E;
  if (!skip) {
    // staging: thread -> (tensor-tile row, 16-byte chunk); Q/dO rows q0t.., K/V rows k0t..
    u32x4 pre[4][CPT];
    float pstat = 0.f;
    // HP = 1: thread t takes the chunks t, t + 256, ... of its head's tile rows.  HP = 2: the two heads'
    // slices of a row are 2 * CPR consecutive chunks (stride_h == D); thread t takes chunk t of them.
    auto chunk = [&](int c, int& hh, int& row, int& col) {
      const int idx = HP == 1 ? tid + c * 256 : tid;
      row = idx / (CPR * HP);
      hh = HP == 1 ? 0 : (idx % (CPR * HP)) / CPR;
      col = (idx % CPR) * 8;
    };
    auto gload = [&](int b) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        int hh, row, col;
        chunk(c, hh, row, col);
        const int rq = min(q0t + row, p.S - 1), rk = min(k0t + row, p.S - 1);
        const int hc = HP == 1 ? h : hA;  // HP = 2: addressed from the first head, hh * D columns on
        const int64_t ba = (int64_t)b * p.sb + (int64_t)hc * p.sh + hh * D + col;
        pre[0][c] = *(const u32x4*)((const uint16_t*)p.Q + ba + (int64_t)rq * p.ss);
        pre[1][c] = *(const u32x4*)((const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(hc - p.do_h0) * p.do_sh + (int64_t)rq * p.do_ss + hh * D + col);
        pre[2][c] = *(const u32x4*)((const uint16_t*)p.K + ba + (int64_t)rk * p.ss);
        pre[3][c] = *(const u32x4*)((const uint16_t*)p.V + ba + (int64_t)rk * p.ss);
      }
      if (tid < 128 * HP) {
        const int hs = hA + tid / 128, i = min(q0t + (tid & 63), p.S - 1);
        pstat = (tid & 64) == 0 ? p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(hs - p.lse_h0) * p.lse_sh + i]
                                : p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(hs - p.dl_h0) * p.dl_sh + i];
      }
    };
    auto lstore = [&](int buf) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        int hh, row, col;
        chunk(c, hh, row, col);
#pragma unroll
        for (int t = 0; t < 4; ++t) *(u32x4*)(&sT[buf][t][hh][row * LD + col]) = pre[t][c];
      }
      // LSE (base 2) and Delta of query i: the two floats after the D elements of row i of the Q tile
      if (tid < 128 * HP) {
        float* st = (float*)(&sT[buf][0][tid / 128][(tid & 63) * LD + D]);
        if ((tid & 64) == 0) st[0] = pstat * LOG2E;
        else st[1] = pstat;
      }
    };
    gload(bfirst);
    lstore(bfirst & 1);
    if (bfirst + 1 < blast) gload(bfirst + 1);
    for (int b = bfirst; b < blast; ++b) {
      const int buf = b & 1;  // by global row parity: a row always takes the same path
      __syncthreads();
      if (b + 1 < blast) lstore(buf ^ 1);
      if (b + 2 < blast) gload(b + 2);
      f32x16 sa, pa;
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa = mfma(lds_nat<LD>(sT[buf][2][hsel], 32 * wk + r, ks, hl), lds_nat<LD>(sT[buf][0][hsel], 32 * wq + r, ks, hl), sa);
        pa = mfma(lds_nat<LD>(sT[buf][3][hsel], 32 * wk + r, ks, hl), lds_nat<LD>(sT[buf][1][hsel], 32 * wq + r, ks, hl), pa);
      }
      const float2 st2 = *(const float2*)(&sT[buf][0][hsel][(32 * wq + r) * LD + D]);
      const float lse2 = st2.x, dlt = st2.y;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const float e = fast_exp2(fmaf(sa[v], c1, bz[v] - lse2));
        float t = pa[v] - dlt;
        if (CAUSAL) t = k0 + key_of(v, hl) > q ? 0.f : t;
        acc[v] = __builtin_fmaf(e, t, acc[v]);
      }
    }
  }
  if (q < p.S && !(skip && resume)) {
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int kb = k0 + 8 * g + 4 * hl;
      if (kb + 3 < p.S) *(f32x4*)(dst + kb) = f32x4{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
      else for (int e = 0; e < 4; ++e) if (kb + e < p.S) dst[kb + e] = acc[4 * g + e];
    }
  }
}

// biasT[h][j][i] = bias[h][i][j] (bf16), 32x32 tiles through LDS; heads [h0,h1)
__global__ __launch_bounds__(256) void bias_transpose_kernel(const uint16_t* src, uint16_t* dst, int S, int h0) {
  __shared__ uint16_t t[32][33];
  const int h = h0 + blockIdx.z, i0 = blockIdx.y * 32, j0 = blockIdx.x * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int y = ty; y < 32; y += 8)
    if (i0 + y < S && j0 + tx < S) t[y][tx] = src[((int64_t)h * S + i0 + y) * S + j0 + tx];
  __syncthreads();
  for (int y = ty; y < 32; y += 8)
    if (j0 + y < S && i0 + tx < S) dst[((int64_t)h * S + j0 + y) * S + i0 + tx] = t[tx][y];
}


template <int D, int NW, bool SLICE32>
void dkdv_fast_launch(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 32 * NW - 1) / (32 * NW), p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) dkdv_fast_kernel<D, true, true, NW, SLICE32><<<g, 64 * NW, 0, st>>>(p);
  else if (bias) dkdv_fast_kernel<D, true, false, NW, SLICE32><<<g, 64 * NW, 0, st>>>(p);
  else if (causal) dkdv_fast_kernel<D, false, true, NW, SLICE32><<<g, 64 * NW, 0, st>>>(p);
  else dkdv_fast_kernel<D, false, false, NW, SLICE32><<<g, 64 * NW, 0, st>>>(p);
}
template <int D>
hipError_t dkdv_d(const KP& p, hipStream_t st) {
  // head size 32 runs three wavefronts per SIMD and has no registers to spare for 64-bit addresses
  const int64_t lim = 1ll << 31;
  const bool slice32 = D <= 32 && ((int64_t)(p.S - 1) * p.ss + D) * 2 < lim && ((int64_t)(p.S - 1) * p.do_ss + D) * 2 < lim;
  if (slice32) dkdv_fast_launch<D, 4, D <= 32>(p, st);
  else dkdv_fast_launch<D, 4, false>(p, st);
  return hipGetLastError();
}
template <int D>
hipError_t dbias_d(const KP& p, hipStream_t st) {
  {  // callers guarantee S > 64 and S a multiple of 4 (fast_ok)
    int ng = 1;
    if (p.sm_partial) ng = (p.b1 - 1) / p.sm_gw - p.b0 / p.sm_gw + 1;
    const int heads = p.h1 - p.h0;
    const int64_t tiles = (int64_t)((p.S + 63) / 64) * ((p.S + 63) / 64);
    if (D == 32 && heads % 2 == 0 && p.sh == D && p.do_sh == D && tiles * (heads / 2) * ng >= 512) {
      // neighbouring heads are 64 bytes apart: two per work-group, if that still leaves two
      // work-groups per compute unit
      dim3 g((p.S + 63) / 64, (p.S + 63) / 64, heads / 2 * ng);
      if (p.mask_kind == 1) dbias_tile_kernel<D <= 32 ? D : 32, true, 2><<<g, 512, 0, st>>>(p);
      else dbias_tile_kernel<D <= 32 ? D : 32, false, 2><<<g, 512, 0, st>>>(p);
      return hipGetLastError();
    }
    dim3 g((p.S + 63) / 64, (p.S + 63) / 64, heads * ng);
    if (p.mask_kind == 1) dbias_tile_kernel<D, true, 1><<<g, 256, 0, st>>>(p);
    else dbias_tile_kernel<D, false, 1><<<g, 256, 0, st>>>(p);
    return hipGetLastError();
  }
}

}  // namespace

#define SS_FAST_DISPATCH_D(fn, ...)               \
  switch (p.D) {                                  \
    case 32: return fn<32>(__VA_ARGS__);          \
    case 64: return fn<64>(__VA_ARGS__);          \
    case 128: return fn<128>(__VA_ARGS__);        \
    default: return hipErrorInvalidValue;         \
  }
hipError_t launch_fast_dkdv(const KP& p, hipStream_t st) {
  // large shares at head size 128 without a bias: one gradient per work-group, tiles straight into LDS
  if (p.D == 128 && p.bias_kind == 0 && wg_shape(p) == WG_4x1) return launch_fast_kv128(p, st);
  SS_FAST_DISPATCH_D(dkdv_d, p, st)
}
hipError_t launch_fast_dbias(const KP& p, hipStream_t st) { SS_FAST_DISPATCH_D(dbias_d, p, st) }

hipError_t launch_bias_transpose(const void* bias, void* biasT, int S, int h0, int h1, hipStream_t st) {
  dim3 g((S + 31) / 32, (S + 31) / 32, h1 - h0);
  bias_transpose_kernel<<<g, 256, 0, st>>>((const uint16_t*)bias, (uint16_t*)biasT, S, h0);
  return hipGetLastError();
}

}  // namespace ssa
