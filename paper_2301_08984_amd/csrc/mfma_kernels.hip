// bf16 MFMA attention kernels for gfx950 (CDNA4), head sizes 32 / 64 / 128.
//
// Orientation.  Every kernel keeps the index that softmax statistics belong to
// (the query) on the LANE axis of the 32x32 MFMA accumulator wherever it can:
//   forward / dQ : S^T = K Q^T   -> acc[key][query], lane = query, registers = keys
//                  O^T = V^T P^T,  dQ^T = K^T dS^T  (B operand = the accumulator
//                  registers, converted to bf16 in place; no shuffles, no LDS trip)
//   dK/dV        : S = Q K^T     -> acc[query][key], lane = key, registers = queries
//                  dV^T = dO^T P,  dK^T = Q^T dS
// Row max / row sum are then in-lane reductions plus one exchange between the
// two 32-lane halves (v_permlane32_swap).
//
// MFMA v_mfma_f32_32x32x16_bf16 layouts (lane l, r = l%32, hl = l/32):
//   A[m][k]: lane holds m = r,  k = 8*hl + 0..7      B[k][n]: lane holds n = r, k = 8*hl + 0..7
//   C[m][n]: lane holds n = r,  register v holds m = 8*(v/4) + 4*hl + v%4
// An accumulator block is reused as the B operand of the next product with its
// registers 8t..8t+7 as the eight k-slots; the matching A operand is read from a
// row-major LDS tile with ds_read_b64_tr_b16 (transpose read) in the same row order.
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

// cooperative copy of a [BN x D] tile (rows row0.., zero past `rows_valid`) into LDS
template <int D, int LD, int NT>
__device__ inline void stage_tile(uint16_t* dst, const uint16_t* src, int64_t row_stride, int row0,
                                  int rows_total, int tid) {
  constexpr int CPR = D / 8;  // 16-byte chunks per row
  constexpr int CH = BN * CPR;
#pragma unroll
  for (int c = tid; c < CH; c += NT) {
    const int row = c / CPR, col = (c % CPR) * 8;
    u32x4 v = u32x4{0, 0, 0, 0};
    if (row0 + row < rows_total) v = *(const u32x4*)(src + (int64_t)(row0 + row) * row_stride + col);
    *(u32x4*)(dst + row * LD + col) = v;
  }
}

struct BiasCtx {
  const int* cidx;     // LDS: c[i] = y_i*(2*win_w-1) + x_i        (RELPOS)
  const float* table;  // LDS: this head's table                    (RELPOS)
  int c0;              // (win_h-1)*(2*win_w-1) + (win_w-1)
};

// additive bias of pairs (q, kbase..kbase+3), already multiplied by log2(e)
__device__ inline void bias4(const KP& p, const BiasCtx& bc, int h, int q, int kbase, float* out) {
  if (p.bias_kind == 1) {
    const int64_t off = ((int64_t)h * p.S + q) * p.S + kbase;
    if ((p.S & 3) == 0 && kbase + 3 < p.S) {
      if (p.bias_bf16) {
        const uint2 u = *(const uint2*)((const uint16_t*)p.bias + off);
        out[0] = __uint_as_float(u.x << 16) * LOG2E; out[1] = __uint_as_float(u.x & 0xffff0000u) * LOG2E;
        out[2] = __uint_as_float(u.y << 16) * LOG2E; out[3] = __uint_as_float(u.y & 0xffff0000u) * LOG2E;
      } else {
        const float4 f = *(const float4*)((const float*)p.bias + off);
        out[0] = f.x * LOG2E; out[1] = f.y * LOG2E; out[2] = f.z * LOG2E; out[3] = f.w * LOG2E;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        out[e] = 0.f;
        if (kbase + e < p.S)
          out[e] = (p.bias_bf16 ? bf2f(((const uint16_t*)p.bias)[off + e]) : ((const float*)p.bias)[off + e]) * LOG2E;
      }
    }
  } else if (p.bias_kind == 2) {
    const int cq = bc.cidx[q] + bc.c0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = min(kbase + e, p.S - 1);
      out[e] = bc.table[cq - bc.cidx[k]] * LOG2E;
    }
  } else {
    out[0] = out[1] = out[2] = out[3] = 0.f;
  }
}
// single pair (used where registers run over queries)
__device__ inline float bias1(const KP& p, const BiasCtx& bc, int h, int q, int k) {
  if (p.bias_kind == 1) {
    const int64_t off = ((int64_t)h * p.S + q) * p.S + k;
    return (p.bias_bf16 ? bf2f(((const uint16_t*)p.bias)[off]) : ((const float*)p.bias)[off]) * LOG2E;
  } else if (p.bias_kind == 2) {
    return bc.table[bc.cidx[q] + bc.c0 - bc.cidx[k]] * LOG2E;
  }
  return 0.f;
}

// fills the RELPOS lookup tables of head h (no-op otherwise); caller syncs afterwards
__device__ inline void relpos_setup(const KP& p, int h, int* cidx, float* table, int tid, int nt, BiasCtx& bc) {
  bc.cidx = cidx; bc.table = table; bc.c0 = 0;
  if (p.bias_kind != 2) return;
  const int R = (2 * p.win_h - 1) * (2 * p.win_w - 1);
  for (int i = tid; i < p.S; i += nt) cidx[i] = (i / p.win_w) * (2 * p.win_w - 1) + (i % p.win_w);
  for (int r = tid; r < R; r += nt)
    table[r] = p.bias_bf16 ? bf2f(((const uint16_t*)p.bias)[(int64_t)h * R + r]) : ((const float*)p.bias)[(int64_t)h * R + r];
  bc.c0 = (p.win_h - 1) * (2 * p.win_w - 1) + (p.win_w - 1);
}

// ---------------------------------------------------------------------------
// forward, and the backward's recompute pass (RECOMP): one 32-query block per
// wavefront, NW wavefronts per work-group share the staged K/V tiles.  This is the
// all-features kernel (any bias / mask kind, decided at run time).
// ---------------------------------------------------------------------------
template <int D, int NW, bool RECOMP>
__global__ __launch_bounds__(NW * 64) void mfma_fwd_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 8, NT = NW * 64;
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;  // 16-byte chunks per row / per thread per tile
  __shared__ __attribute__((aligned(16))) uint16_t sK[BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sV[2][BN * LD];
  __shared__ int s_cidx[MAX_RELPOS_S];
  __shared__ float s_table[MAX_RELPOS_R];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const int qblk = (gridDim.x - 1 - blockIdx.x) * (32 * NW);  // long (late) causal blocks first
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  BiasCtx bc;
  relpos_setup(p, h, s_cidx, s_table, tid, NT, bc);
  const int32_t* rid = p.mask_kind == 2 ? p.region + (int64_t)(b % p.mask_period) * p.S : nullptr;
  const int my_rid = rid ? rid[qc] : 0;

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qf[ks] = q < p.S ? *(const bf16x8*)(Qb + (int64_t)q * p.ss + 16 * ks + 8 * hl) : zero8();
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (p.mask_kind == 1) ntiles = min(ntiles, (min(qblk + 32 * NW, p.S) + BN - 1) / BN);
  // tiles that hold at least one key visible to this wavefront
  int wtiles = ntiles;
  if (p.mask_kind == 1) wtiles = min(ntiles, (min(q0 + 32, p.S) + BN - 1) / BN);
  if (q0 >= p.S) wtiles = 0;
  const bool has_bias = p.bias_kind != 0;

  // software pipeline: tile kt+2 travels global->registers while tile kt+1 sits in LDS and its
  // scores are produced by the matrix cores, and tile kt goes through softmax and the PV product
  u32x4 pk[CPT], pv[CPT];
  auto gload = [&](int kt) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = kt * BN + idx / CPR, col = (idx % CPR) * 8;
      pk[c] = u32x4{0, 0, 0, 0};
      pv[c] = u32x4{0, 0, 0, 0};
      if (row < p.S) {
        pk[c] = *(const u32x4*)(Kb + (int64_t)row * p.ss + col);
        pv[c] = *(const u32x4*)(Vb + (int64_t)row * p.ss + col);
      }
    }
  };
  auto lstore = [&](uint16_t* dV) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(sK + row * LD + col) = pk[c];
      *(u32x4*)(dV + row * LD + col) = pv[c];
    }
  };
  auto scores = [&](f32x16 (&sa)[2]) {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) sa[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) sa[kb] = mfma(lds_nat<LD>(sK, 32 * kb + r, ks, hl), qf[ks], sa[kb]);
    }
  };

  gload(0);
  lstore(sV[0]);
  if (ntiles > 1) gload(1);
  __syncthreads();
  f32x16 scur[2], snext[2];
  if (wtiles > 0) scores(scur);
  __syncthreads();
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BN;
    if (kt + 1 < ntiles) lstore(sV[(kt + 1) & 1]);
    if (kt + 2 < ntiles) gload(kt + 2);
    __syncthreads();
    if (kt < wtiles) {
      if (kt + 1 < wtiles) scores(snext);
      // does this tile need per-element masking?  (tail keys, the causal diagonal, region ids)
      const bool edge = (k0 + BN > p.S) || (p.mask_kind == 1 && k0 + BN - 1 > q0) || p.mask_kind == 2;
      float rmax = -INFINITY;
      if (has_bias || edge) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int kbase = k0 + 32 * kb + 8 * g + 4 * hl;
            float bz[4];
            bias4(p, bc, h, qc, kbase, bz);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int key = kbase + e;
              float x = fmaf(scur[kb][4 * g + e], c1, bz[e]);
              if (edge) {
                bool dead = key >= p.S;
                if (p.mask_kind == 1) dead = dead || key > q;
                if (p.mask_kind == 2) dead = dead || rid[min(key, p.S - 1)] != my_rid;
                x = dead ? -INFINITY : x;
              }
              scur[kb][4 * g + e] = x;
              rmax = fmaxf(rmax, x);
            }
          }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, scur[kb][v]);
        rmax *= c1;
      }
      rmax = half_max(rmax);
      // the running maximum is only raised when it is exceeded by more than 2^8: probabilities
      // then stay below 2^8 in bf16/fp32 range and the O rescale is skipped on most tiles
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
      float lsum = 0.f;
      if (has_bias || edge) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            scur[kb][v] = fast_exp2(scur[kb][v] - m);
            lsum += scur[kb][v];
          }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            scur[kb][v] = fast_exp2(fmaf(scur[kb][v], c1, -m));
            lsum += scur[kb][v];
          }
      }
      l += lsum;
      const uint16_t* tv = sV[kt & 1];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
          float tmp[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) tmp[e] = scur[kb][8 * hb + e];
          const bf16x8 pf = pack8(tmp);
#pragma unroll
          for (int db = 0; db < DB; ++db)
            oacc[db] = mfma(lds_tr<LD>(tv, 32 * kb + 16 * hb, 32 * db, lane), pf, oacc[db]);
        }
      scur[0] = snext[0];
      scur[1] = snext[1];
    }
    __syncthreads();
  }
  fwd_epilogue<DB, RECOMP>(p, oacc, m, l, b, h, q, hl, base);
}

// ---------------------------------------------------------------------------
// dQ: same decomposition as the forward; Q and dO fragments stay in registers
// ---------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void mfma_dq_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 8, NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t sK[BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sV[BN * LD];
  __shared__ int s_cidx[MAX_RELPOS_S];
  __shared__ float s_table[MAX_RELPOS_R];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const int qblk = (gridDim.x - 1 - blockIdx.x) * (32 * NW);
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  BiasCtx bc;
  relpos_setup(p, h, s_cidx, s_table, tid, NT, bc);
  const int32_t* rid = p.mask_kind == 2 ? p.region + (int64_t)(b % p.mask_period) * p.S : nullptr;
  const int my_rid = rid ? rid[qc] : 0;

  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = q < p.S ? *(const bf16x8*)(Qb + (int64_t)q * p.ss + 16 * ks + 8 * hl) : zero8();
    gf[ks] = q < p.S ? *(const bf16x8*)(dOb + (int64_t)q * p.do_ss + 16 * ks + 8 * hl) : zero8();
  }
  const float lse2 = p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (p.mask_kind == 1) ntiles = min(ntiles, (min(qblk + 32 * NW, p.S) + BN - 1) / BN);
  for (int kt = 0; kt < ntiles; ++kt) {
    const int k0 = kt * BN;
    __syncthreads();
    stage_tile<D, LD, NT>(sK, Kb, p.ss, k0, p.S, tid);
    stage_tile<D, LD, NT>(sV, Vb, p.ss, k0, p.S, tid);
    __syncthreads();
    if (q0 >= p.S || (p.mask_kind == 1 && k0 > q0 + 31)) continue;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc = mfma(lds_nat<LD>(sK, 32 * kb + r, ks, hl), qf[ks], sacc);
        pacc = mfma(lds_nat<LD>(sV, 32 * kb + r, ks, hl), gf[ks], pacc);
      }
      float ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int kbase = k0 + 32 * kb + 8 * g + 4 * hl;
        float bz[4];
        bias4(p, bc, h, qc, kbase, bz);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int key = kbase + e;
          bool dead = key >= p.S;
          if (p.mask_kind == 1) dead = dead || key > q;
          if (p.mask_kind == 2) dead = dead || rid[min(key, p.S - 1)] != my_rid;
          const float pr = fast_exp2(fmaf(sacc[4 * g + e], c1, bz[e]) - lse2);
          ds[4 * g + e] = dead ? 0.f : pr * (pacc[4 * g + e] - delta);
        }
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const bf16x8 df = pack8(&ds[8 * hb]);
#pragma unroll
        for (int db = 0; db < DB; ++db)
          acc[db] = mfma(lds_tr<LD>(sK, 32 * kb + 16 * hb, 32 * db, lane), df, acc[db]);
      }
    }
  }
  if (q >= p.S) return;
  uint16_t* out = (uint16_t*)p.dQ + base + (int64_t)q * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = 32 * db + 8 * g + 4 * hl;
      uint2 o;
      o.x = (uint32_t)f2bf(acc[db][4 * g] * p.scale) | ((uint32_t)f2bf(acc[db][4 * g + 1] * p.scale) << 16);
      o.y = (uint32_t)f2bf(acc[db][4 * g + 2] * p.scale) | ((uint32_t)f2bf(acc[db][4 * g + 3] * p.scale) << 16);
      *(uint2*)(out + d0) = o;
    }
}

// ---------------------------------------------------------------------------
// dK, dV: one 32-key block per wavefront, K and V fragments in registers,
// Q and dO tiles staged in LDS and read both ways (natural and transposed)
// ---------------------------------------------------------------------------
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void mfma_dkdv_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 8, NT = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t sQ[BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sG[BN * LD];
  __shared__ float s_lse[BN], s_delta[BN];
  __shared__ int s_cidx[MAX_RELPOS_S];
  __shared__ float s_table[MAX_RELPOS_R];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.y, b = p.b0 + blockIdx.z;
  const int kblk = blockIdx.x * (32 * NW);  // early key blocks see the most queries under a causal mask
  const int k0 = kblk + 32 * w, key = k0 + r;
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
  BiasCtx bc;
  relpos_setup(p, h, s_cidx, s_table, tid, NT, bc);
  const int32_t* rid = p.mask_kind == 2 ? p.region + (int64_t)(b % p.mask_period) * p.S : nullptr;
  const int my_rid = rid ? rid[kc] : 0;

  bf16x8 kf[KS], vf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = key < p.S ? *(const bf16x8*)(Kb + (int64_t)key * p.ss + 16 * ks + 8 * hl) : zero8();
    vf[ks] = key < p.S ? *(const bf16x8*)(Vb + (int64_t)key * p.ss + 16 * ks + 8 * hl) : zero8();
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }
  const float c1 = p.scale * LOG2E;

  const int ntiles = (p.S + BN - 1) / BN;
  const int first = p.mask_kind == 1 ? kblk / BN : 0;  // queries before the block's first key see none of it
  for (int qt = first; qt < ntiles; ++qt) {
    const int i0 = qt * BN;
    __syncthreads();
    stage_tile<D, LD, NT>(sQ, Qb, p.ss, i0, p.S, tid);
    stage_tile<D, LD, NT>(sG, dOb, p.do_ss, i0, p.S, tid);
    if (tid < BN) {
      const int i = min(i0 + tid, p.S - 1);
      s_lse[tid] = lse_b[i] * LOG2E;
      s_delta[tid] = dl_b[i];
    }
    __syncthreads();
    if (k0 >= p.S || (p.mask_kind == 1 && i0 + BN - 1 < k0)) continue;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 sacc, pacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sacc = mfma(lds_nat<LD>(sQ, 32 * qb + r, ks, hl), kf[ks], sacc);
        pacc = mfma(lds_nat<LD>(sG, 32 * qb + r, ks, hl), vf[ks], pacc);
      }
      float pr[16], ds[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int il = 32 * qb + key_of(v, hl);
        const int i = i0 + il;
        const int ic = min(i, p.S - 1);
        bool dead = i >= p.S || key >= p.S;
        if (p.mask_kind == 1) dead = dead || key > i;
        if (p.mask_kind == 2) dead = dead || rid[ic] != my_rid;
        const float x = fmaf(sacc[v], c1, bias1(p, bc, h, ic, kc)) - s_lse[il];
        const float e = dead ? 0.f : fast_exp2(x);
        pr[v] = e;
        ds[v] = e * (pacc[v] - s_delta[il]);
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const bf16x8 pf = pack8(&pr[8 * hb]);
        const bf16x8 df = pack8(&ds[8 * hb]);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          dv[db] = mfma(lds_tr<LD>(sG, 32 * qb + 16 * hb, 32 * db, lane), pf, dv[db]);
          dk[db] = mfma(lds_tr<LD>(sQ, 32 * qb + 16 * hb, 32 * db, lane), df, dk[db]);
        }
      }
    }
  }
  if (key >= p.S) return;
  uint16_t* oK = (uint16_t*)p.dK + base + (int64_t)key * p.ss;
  uint16_t* oV = (uint16_t*)p.dV + base + (int64_t)key * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int d0 = 32 * db + 8 * g + 4 * hl;
      uint2 a, c;
      a.x = (uint32_t)f2bf(dk[db][4 * g] * p.scale) | ((uint32_t)f2bf(dk[db][4 * g + 1] * p.scale) << 16);
      a.y = (uint32_t)f2bf(dk[db][4 * g + 2] * p.scale) | ((uint32_t)f2bf(dk[db][4 * g + 3] * p.scale) << 16);
      c.x = (uint32_t)f2bf(dv[db][4 * g]) | ((uint32_t)f2bf(dv[db][4 * g + 1]) << 16);
      c.y = (uint32_t)f2bf(dv[db][4 * g + 2]) | ((uint32_t)f2bf(dv[db][4 * g + 3]) << 16);
      *(uint2*)(oK + d0) = a;
      *(uint2*)(oV + d0) = c;
    }
}

// ---------------------------------------------------------------------------
// bias gradient (dense accumulator): each wavefront owns one 32x32 block of
// (query, key) pairs of one head and walks the chunk's rows b in order, adding
// dS to fp32 registers; a later chunk continues from the stored value, so the
// sum is taken in the same order whatever k is.  acc[query][key]: lane = key, so
// stores run along the contiguous key axis.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void mfma_dbias_kernel(KP p) {
  constexpr int KS = D / 16;
  __shared__ int s_cidx[MAX_RELPOS_S];
  __shared__ float s_table[MAX_RELPOS_R];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.z;
  const int i0 = blockIdx.y * 32;
  const int k0 = (blockIdx.x * 4 + w) * 32;
  BiasCtx bc;
  relpos_setup(p, h, s_cidx, s_table, tid, 256, bc);
  __syncthreads();
  if (k0 >= p.S) return;
  if (p.mask_kind == 1 && k0 > i0 + 31) {  // block entirely above the diagonal: gradient is zero
    if (!p.dbias_accumulate) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = i0 + key_of(v, hl), key = k0 + r;
        if (i < p.S && key < p.S) p.dbias_acc[((int64_t)h * p.S + i) * p.S + key] = 0.f;
      }
    }
    return;
  }
  const int key = k0 + r, kc = min(key, p.S - 1);
  const int qa = min(i0 + r, p.S - 1);  // row this lane supplies to the A operands
  float acc[16], bz[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = min(i0 + key_of(v, hl), p.S - 1);
    acc[v] = p.dbias_accumulate ? p.dbias_acc[((int64_t)h * p.S + i) * p.S + kc] : 0.f;
    bz[v] = bias1(p, bc, h, i, kc);
  }
  const float c1 = p.scale * LOG2E;
  for (int b = p.b0; b < p.b1; ++b) {
    const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
    const uint16_t* Qr = (const uint16_t*)p.Q + base + (int64_t)qa * p.ss;
    const uint16_t* Kr = (const uint16_t*)p.K + base + (int64_t)kc * p.ss;
    const uint16_t* Vr = (const uint16_t*)p.V + base + (int64_t)kc * p.ss;
    const uint16_t* Gr = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh + (int64_t)qa * p.do_ss;
    const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
    const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
    const int32_t* rid = p.mask_kind == 2 ? p.region + (int64_t)(b % p.mask_period) * p.S : nullptr;
    const int my_rid = rid ? rid[kc] : 0;
    f32x16 sacc, pacc;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sacc[v] = 0.f; pacc[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = 16 * ks + 8 * hl;
      sacc = mfma(*(const bf16x8*)(Qr + c), *(const bf16x8*)(Kr + c), sacc);
      pacc = mfma(*(const bf16x8*)(Gr + c), *(const bf16x8*)(Vr + c), pacc);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int i = i0 + key_of(v, hl), ic = min(i, p.S - 1);
      bool dead = false;
      if (p.mask_kind == 1) dead = key > i;
      if (p.mask_kind == 2) dead = rid[ic] != my_rid;
      const float e = fast_exp2(fmaf(sacc[v], c1, bz[v]) - lse_b[ic] * LOG2E);
      acc[v] += dead ? 0.f : e * (pacc[v] - dl_b[ic]);
    }
  }
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int i = i0 + key_of(v, hl);
    if (i < p.S && key < p.S) p.dbias_acc[((int64_t)h * p.S + i) * p.S + key] = acc[v];
  }
}

template <int D>
hipError_t fwd_d(const KP& p, bool recompute, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (p.S <= 64) {
    dim3 g((p.S + 63) / 64, Hc, Bc);
    if (recompute) mfma_fwd_kernel<D, 2, true><<<g, 128, 0, st>>>(p);
    else mfma_fwd_kernel<D, 2, false><<<g, 128, 0, st>>>(p);
  } else {
    dim3 g((p.S + 127) / 128, Hc, Bc);
    if (recompute) mfma_fwd_kernel<D, 4, true><<<g, 256, 0, st>>>(p);
    else mfma_fwd_kernel<D, 4, false><<<g, 256, 0, st>>>(p);
  }
  return hipGetLastError();
}
template <int D>
hipError_t dq_d(const KP& p, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (p.S <= 64) mfma_dq_kernel<D, 2><<<dim3((p.S + 63) / 64, Hc, Bc), 128, 0, st>>>(p);
  else mfma_dq_kernel<D, 4><<<dim3((p.S + 127) / 128, Hc, Bc), 256, 0, st>>>(p);
  return hipGetLastError();
}
template <int D>
hipError_t dkdv_d(const KP& p, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (p.S <= 64) mfma_dkdv_kernel<D, 2><<<dim3((p.S + 63) / 64, Hc, Bc), 128, 0, st>>>(p);
  else mfma_dkdv_kernel<D, 4><<<dim3((p.S + 127) / 128, Hc, Bc), 256, 0, st>>>(p);
  return hipGetLastError();
}
template <int D>
hipError_t dbias_d(const KP& p, hipStream_t st) {
  dim3 g((p.S + 127) / 128, (p.S + 31) / 32, p.h1 - p.h0);
  mfma_dbias_kernel<D><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

bool mfma_supported(const KP& p, bool bf16) {
  if (!bf16) return false;
  if (p.D != 32 && p.D != 64 && p.D != 128) return false;
  if (p.bias_kind == 2 && (p.S > MAX_RELPOS_S || (2 * p.win_h - 1) * (2 * p.win_w - 1) > MAX_RELPOS_R)) return false;
  if ((p.S + 31) / 32 > 65535) return false;
  return true;
}

#define SS_DISPATCH_D(fn, ...)                    \
  switch (p.D) {                                  \
    case 32: return fn<32>(__VA_ARGS__);          \
    case 64: return fn<64>(__VA_ARGS__);          \
    case 128: return fn<128>(__VA_ARGS__);        \
    default: return hipErrorInvalidValue;         \
  }

// the specialised kernels (one translation unit each) serve what fast_ok() accepts; the
// all-feature kernels above serve the rest
hipError_t launch_mfma_fwd(const KP& p, bool recompute, hipStream_t st) {
  if (fast_ok(p)) return launch_fast_fwd(p, recompute, st);
  SS_DISPATCH_D(fwd_d, p, recompute, st)
}
hipError_t launch_mfma_dq(const KP& p, hipStream_t st) {
  if (fast_ok(p)) return launch_fast_dq(p, st);
  SS_DISPATCH_D(dq_d, p, st)
}
hipError_t launch_mfma_dkdv(const KP& p, hipStream_t st) {
  if (fast_ok(p)) return launch_fast_dkdv(p, st);
  SS_DISPATCH_D(dkdv_d, p, st)
}
hipError_t launch_mfma_dbias(const KP& p, hipStream_t st) {
  if (fast_ok(p) && p.bias_kind == 1) return launch_fast_dbias(p, st);
  SS_DISPATCH_D(dbias_d, p, st)
}

bool mfma_wants_bias_transpose(const KP& p) { return fast_ok(p) && p.bias_kind == 1; }
// small shares with long rows: dQ and dK/dV share one launch
bool mfma_fuses_dq_dkdv(const KP& p) { return fast_ok(p) && wg_shape(p) == WG_2x4; }
hipError_t launch_mfma_dq_dkdv(const KP& p, hipStream_t st) {
  // head size 128 without a bias: one gradient per work-group, two work-groups per compute unit
  if (p.D == 128 && p.bias_kind == 0) return launch_fast_bwd_wave3(p, st);
  return launch_fast_bwd_wave(p, st);
}
// head size 32 on the large-share work-group shape: the vector arithmetic per score element binds, and
// the recompute pass and dQ share all of it
bool mfma_fuses_recompute_dq(const KP& p) {
  if (!fast_ok(p) || p.D != 32 || wg_shape(p) != WG_4x1) return false;
  return ((int64_t)(p.S - 1) * p.ss + p.D) * 2 < (1ll << 31);  // the kernel addresses a (row, head) slice with 32-bit offsets
}
hipError_t launch_mfma_recompute_dq(const KP& p, hipStream_t st) { return launch_fast_recompute_dq(p, st); }
int mfma_dbias_group_rows(const KP& p) { return dbias_group_rows(p); }

}  // namespace ssa
