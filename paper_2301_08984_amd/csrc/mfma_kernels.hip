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
// forward / recompute, specialised at compile time on the presence of a dense bf16
// bias and of the causal mask.  The inner loop is straight-line code: loads are
// clamped instead of guarded, and tiles that need no per-element masking (all keys
// below the causal diagonal and inside S) take a path without compares.
//
// NG = 2 doubles the work-group to eight wavefronts: group g takes the key tiles
// kt = g, g+2, ... with its own LDS tiles and its own (O, m, l); the two partial
// softmax results are merged through LDS at the end.  Two wavefronts then share
// every SIMD, so one's softmax arithmetic overlaps the other's matrix products,
// and the serial chain of key tiles per wavefront is half as long.  It is chosen
// from the size of the whole share, never from the chunk, so results do not
// depend on k.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, bool RECOMP, int NG>
__global__ __launch_bounds__(256 * NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, NT = 256;
  constexpr int LDK = D + 8, LDV = D + 16;  // row pads chosen for conflict-free b128 / transpose reads
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  constexpr int TILE_ELEMS = BN * LDK + BN * LDV;
  constexpr int MERGE_ELEMS = NG > 1 ? 256 * (16 * DB + 2) * 2 : 0;  // in uint16 units
  constexpr int LDS_ELEMS = NG * TILE_ELEMS > MERGE_ELEMS ? NG * TILE_ELEMS : MERGE_ELEMS;
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int tid = threadIdx.x & 255, grp = threadIdx.x >> 8;
  const int lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  uint16_t* sK = smem + grp * TILE_ELEMS;
  uint16_t* sV = sK + BN * LDK;
  const BlockId blk = xcd_block_id();
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * 128;  // long (late) causal blocks first
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* bias_row = BIAS ? (const uint16_t*)p.bias + ((int64_t)h * p.S + qc) * p.S : nullptr;

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(Qb + (int64_t)qc * p.ss + 16 * ks + 8 * hl);
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + 128, p.S) + BN - 1) / BN);
  int wtiles = ntiles;  // tiles holding at least one key visible to this wavefront
  if (CAUSAL) wtiles = min(ntiles, (min(q0 + 32, p.S) + BN - 1) / BN);
  if (q0 >= p.S) wtiles = 0;

  u32x4 pk[CPT], pv[CPT];
  auto gload = [&](int kt) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = min(kt * BN + idx / CPR, p.S - 1), col = (idx % CPR) * 8;
      pk[c] = *(const u32x4*)(Kb + (int64_t)row * p.ss + col);
      pv[c] = *(const u32x4*)(Vb + (int64_t)row * p.ss + col);
    }
  };
  if (grp < ntiles) gload(grp);
  const int nit = (ntiles + NG - 1) / NG;
  for (int it = 0; it < nit; ++it) {
    const int kt = it * NG + grp;
    const int k0 = kt * BN;
    __syncthreads();
    if (kt < ntiles) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
        *(u32x4*)(sK + row * LDK + col) = pk[c];
        *(u32x4*)(sV + row * LDV + col) = pv[c];
      }
      if (kt + NG < ntiles) gload(kt + NG);
    }
    __syncthreads();
    if (kt >= wtiles) continue;
    uint2 bz[8];
    if (BIAS) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g)
          bz[4 * kb + g] = *(const uint2*)(bias_row + min(k0 + 32 * kb + 8 * g + 4 * hl, p.S - 4));
    }
    f32x16 sa[2];
    {
      // operand reads run ahead of the matrix cores; the two score blocks alternate so that
      // consecutive MFMAs never wait on each other's accumulator
      bf16x8 fa[KS], fb[KS];
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        fa[ks] = lds_nat<LDK>(sK, r, ks, hl);
        fb[ks] = lds_nat<LDK>(sK, 32 + r, ks, hl);
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[0][v] = 0.f; sa[1][v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa[0] = mfma(fa[ks], qf[ks], sa[0]);
        sa[1] = mfma(fb[ks], qf[ks], sa[1]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
      for (int j = 0; j < 2 * KS - 4; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
    }
    const bool edge = (k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0);
    if (BIAS) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint2 u = bz[4 * kb + g];
          sa[kb][4 * g + 0] = fmaf(sa[kb][4 * g + 0], c1, __uint_as_float(u.x << 16) * LOG2E);
          sa[kb][4 * g + 1] = fmaf(sa[kb][4 * g + 1], c1, __uint_as_float(u.x & 0xffff0000u) * LOG2E);
          sa[kb][4 * g + 2] = fmaf(sa[kb][4 * g + 2], c1, __uint_as_float(u.y << 16) * LOG2E);
          sa[kb][4 * g + 3] = fmaf(sa[kb][4 * g + 3], c1, __uint_as_float(u.y & 0xffff0000u) * LOG2E);
        }
    }
    if (edge) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int key = k0 + 32 * kb + key_of(v, hl);
          const bool dead = key >= p.S || (CAUSAL && key > q);
          sa[kb][v] = dead ? -INFINITY : sa[kb][v];
        }
    }
    float rmax = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, sa[kb][v]);
    if (!BIAS) rmax *= c1;  // scale > 0 on this path
    rmax = half_max(rmax);
    // the running maximum is raised only when exceeded by more than 2^8, so the O rescale is
    // skipped on most tiles; probabilities stay below 2^8, harmless in fp32/bf16 range
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
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        sa[kb][v] = BIAS ? fast_exp2(sa[kb][v] - m) : fast_exp2(fmaf(sa[kb][v], c1, -m));
        lsum += sa[kb][v];
      }
    l += lsum;
    {
      bf16x8 pf[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float tmp[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) tmp[e] = sa[j >> 1][8 * (j & 1) + e];
        pf[j] = pack8(tmp);
      }
      // V^T fragments of step j+1 are fetched while step j multiplies
      bf16x8 vf[2][DB];
#pragma unroll
      for (int db = 0; db < DB; ++db) vf[0][db] = lds_tr<LDV>(sV, 0, 32 * db, lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j + 1 < 4) {
#pragma unroll
          for (int db = 0; db < DB; ++db) vf[(j + 1) & 1][db] = lds_tr<LDV>(sV, 16 * (j + 1), 32 * db, lane);
        }
#pragma unroll
        for (int db = 0; db < DB; ++db) oacc[db] = mfma(vf[j & 1][db], pf[j], oacc[db]);
      }
      __builtin_amdgcn_sched_group_barrier(0x100, 2 * DB, 1);
#pragma unroll
      for (int j = 0; j < 3 * DB; ++j) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
      }
      __builtin_amdgcn_sched_group_barrier(0x008, DB, 1);
    }
  }
  if (NG > 1) {
    // merge the two groups' partial softmax results; group 1 hands (O, m, l) to group 0
    float* mb = (float*)smem + (size_t)tid * (16 * DB + 2);
    __syncthreads();
    if (grp == 1) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) mb[16 * db + v] = oacc[db][v];
      mb[16 * DB] = m;
      mb[16 * DB + 1] = l;
    }
    __syncthreads();
    if (grp == 1) return;
    const float m1 = mb[16 * DB], l1 = mb[16 * DB + 1];
    const float mn = fmaxf(m, m1);
    const float a0 = fast_exp2(m - mn), a1 = fast_exp2(m1 - mn);
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[db][v] = oacc[db][v] * a0 + mb[16 * db + v] * a1;
    l = l * a0 + l1 * a1;
    m = mn;
  }
  if (q >= p.S) return;
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
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)b * p.do_sb + (int64_t)h * p.do_sh;
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
  const float lse2 = p.lse[(int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)b * p.dl_sb + (int64_t)h * p.dl_sh + qc];
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
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)b * p.do_sb + (int64_t)h * p.do_sh;
  const float* lse_b = p.lse + (int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)b * p.dl_sb + (int64_t)h * p.dl_sh;
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
// dQ, specialised like the forward (dense bf16 bias / causal at compile time, NG key-tile
// groups).  Q and dO fragments stay in registers; per 32-key block the scores and dP come
// from the matrix cores, dS from the vector ALUs, and dQ^T += K^T dS^T reads the same K
// tile transposed.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, int NG>
__global__ __launch_bounds__(256 * NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void dq_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, NT = 256;
  constexpr int LDK = D + 16, LDV = D + 8;
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  constexpr int TILE_ELEMS = BN * LDK + BN * LDV;
  constexpr int MERGE_ELEMS = NG > 1 ? 256 * (16 * DB) * 2 : 0;
  constexpr int LDS_ELEMS = NG * TILE_ELEMS > MERGE_ELEMS ? NG * TILE_ELEMS : MERGE_ELEMS;
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int tid = threadIdx.x & 255, grp = threadIdx.x >> 8;
  const int lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  uint16_t* sK = smem + grp * TILE_ELEMS;
  uint16_t* sV = sK + BN * LDK;
  const BlockId blk = xcd_block_id();
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * 128;
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)b * p.do_sb + (int64_t)h * p.do_sh;
  const uint16_t* bias_row = BIAS ? (const uint16_t*)p.bias + ((int64_t)h * p.S + qc) * p.S : nullptr;

  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *(const bf16x8*)(Qb + (int64_t)qc * p.ss + 16 * ks + 8 * hl);
    gf[ks] = *(const bf16x8*)(dOb + (int64_t)qc * p.do_ss + 16 * ks + 8 * hl);
  }
  const float lse2 = p.lse[(int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)b * p.dl_sb + (int64_t)h * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + 128, p.S) + BN - 1) / BN);
  int wtiles = ntiles;
  if (CAUSAL) wtiles = min(ntiles, (min(q0 + 32, p.S) + BN - 1) / BN);
  if (q0 >= p.S) wtiles = 0;

  u32x4 pk[CPT], pv[CPT];
  auto gload = [&](int kt) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = min(kt * BN + idx / CPR, p.S - 1), col = (idx % CPR) * 8;
      pk[c] = *(const u32x4*)(Kb + (int64_t)row * p.ss + col);
      pv[c] = *(const u32x4*)(Vb + (int64_t)row * p.ss + col);
    }
  };
  if (grp < ntiles) gload(grp);
  const int nit = (ntiles + NG - 1) / NG;
  for (int it = 0; it < nit; ++it) {
    const int kt = it * NG + grp;
    const int k0 = kt * BN;
    __syncthreads();
    if (kt < ntiles) {
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
        *(u32x4*)(sK + row * LDK + col) = pk[c];
        *(u32x4*)(sV + row * LDV + col) = pv[c];
      }
      if (kt + NG < ntiles) gload(kt + NG);
    }
    __syncthreads();
    if (kt >= wtiles) continue;
    const bool edge = (k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      uint2 bz[4];
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          bz[g] = *(const uint2*)(bias_row + min(k0 + 32 * kb + 8 * g + 4 * hl, p.S - 4));
      }
      f32x16 sa, pa;
      {
        bf16x8 fk[KS], fv[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          fk[ks] = lds_nat<LDK>(sK, 32 * kb + r, ks, hl);
          fv[ks] = lds_nat<LDV>(sV, 32 * kb + r, ks, hl);
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sa = mfma(fk[ks], qf[ks], sa);
          pa = mfma(fv[ks], gf[ks], pa);
        }
      }
      float ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float bl[4] = {0.f, 0.f, 0.f, 0.f};
        if (BIAS) {
          bl[0] = __uint_as_float(bz[g].x << 16) * LOG2E; bl[1] = __uint_as_float(bz[g].x & 0xffff0000u) * LOG2E;
          bl[2] = __uint_as_float(bz[g].y << 16) * LOG2E; bl[3] = __uint_as_float(bz[g].y & 0xffff0000u) * LOG2E;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float pe = fast_exp2(fmaf(sa[4 * g + e], c1, bl[e] - lse2));
          if (edge) {
            const int key = k0 + 32 * kb + 8 * g + 4 * hl + e;
            const bool dead = key >= p.S || (CAUSAL && key > q);
            pe = dead ? 0.f : pe;
          }
          ds[4 * g + e] = pe * (pa[4 * g + e] - delta);
        }
      }
#pragma unroll
      for (int hb = 0; hb < 2; ++hb) {
        const bf16x8 df = pack8(&ds[8 * hb]);
        bf16x8 kt_[DB];
#pragma unroll
        for (int db = 0; db < DB; ++db) kt_[db] = lds_tr<LDK>(sK, 32 * kb + 16 * hb, 32 * db, lane);
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[db] = mfma(kt_[db], df, acc[db]);
      }
    }
  }
  if (NG > 1) {
    float* mb = (float*)smem + (size_t)tid * (16 * DB);
    __syncthreads();
    if (grp == 1) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) mb[16 * db + v] = acc[db][v];
    }
    __syncthreads();
    if (grp == 1) return;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] += mb[16 * db + v];
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
// dK, dV (optional dense bf16 bias read from its transposed copy, optional causal mask).  Each wavefront
// keeps a 32-key block of K and V and both gradient accumulators in registers and
// walks the queries in 32-row sub-blocks with a software pipeline: while the vector
// ALUs turn the scores of sub-block j into P and dS, the matrix cores already
// produce the scores of sub-block j+1 and consume P/dS of sub-block j-1.
// Q / dO tiles (64 rows) are double-buffered in LDS, one barrier per tile; the next
// tile travels global -> registers meanwhile.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL>
__global__ __launch_bounds__(256) void dkdv_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, LD = D + 16, NT = 256;
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  __shared__ __attribute__((aligned(16))) uint16_t sQ[2][BN * LD];
  __shared__ __attribute__((aligned(16))) uint16_t sG[2][BN * LD];
  __shared__ __attribute__((aligned(16))) float sL[2][BN];
  __shared__ __attribute__((aligned(16))) float sD[2][BN];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const BlockId blk = xcd_block_id();
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int kblk = blk.x * 128;  // early key blocks see the most queries under a causal mask
  const int k0 = kblk + 32 * w, key = k0 + r;
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)b * p.do_sb + (int64_t)h * p.do_sh;
  const float* lse_b = p.lse + (int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)b * p.dl_sb + (int64_t)h * p.dl_sh;
  // transposed bias copy: biasT[h][key][query], four consecutive queries per 8-byte load
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
  const int ntiles = (p.S + BN - 1) / BN;
  const int first = CAUSAL ? kblk / BN : 0;  // queries before the block's first key see none of it

  u32x4 pq[CPT], pg[CPT];
  float pstat = 0.f;
  auto gload = [&](int qt) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = min(qt * BN + idx / CPR, p.S - 1), col = (idx % CPR) * 8;
      pq[c] = *(const u32x4*)(Qb + (int64_t)row * p.ss + col);
      pg[c] = *(const u32x4*)(dOb + (int64_t)row * p.do_ss + col);
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
    if (tid < BN) sL[buf][tid] = pstat * LOG2E;
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
        bl[0] = __uint_as_float(u.x << 16) * LOG2E; bl[1] = __uint_as_float(u.x & 0xffff0000u) * LOG2E;
        bl[2] = __uint_as_float(u.y << 16) * LOG2E; bl[3] = __uint_as_float(u.y & 0xffff0000u) * LOG2E;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float pe = fast_exp2(fmaf(sa[4 * g + e], c1, bl[e] - l4[e]));
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
  }
  for (int qt = first; qt < ntiles; ++qt) {
    const int i0 = qt * BN;
    __syncthreads();
    if (qt + 1 < ntiles) lstore((qt + 1) & 1);
    if (qt + 2 < ntiles) gload(qt + 2);
    if (k0 >= p.S || (CAUSAL && i0 + BN - 1 < k0)) continue;  // no visible pair for this wavefront
    const uint16_t* tq = sQ[qt & 1];
    const uint16_t* tg = sG[qt & 1];
    const float* tl = sL[qt & 1];
    const float* td = sD[qt & 1];
    const bool edge = (i0 + BN > p.S) || (k0 + 32 > p.S) || (CAUSAL && i0 < k0 + 31);
    // one straight-line block per tile: A0 | A1 with V0 | B0 with V1 | B1, where A = scores and dP
    // on the matrix cores, V = P and dS on the vector ALUs, B = gradient products
    uint2 bz[8];
    if (BIAS) {
#pragma unroll
      for (int j = 0; j < 8; ++j) bz[j] = *(const uint2*)(biasT_row + min(i0 + 8 * j + 4 * hl, p.S - 4));
    }
    auto tile = [&](auto edge_tag) {
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
    const uint16_t* Gr = (const uint16_t*)p.dO + (int64_t)b * p.do_sb + (int64_t)h * p.do_sh + (int64_t)qa * p.do_ss;
    const float* lse_b = p.lse + (int64_t)b * p.lse_sb + (int64_t)h * p.lse_sh;
    const float* dl_b = p.delta + (int64_t)b * p.dl_sb + (int64_t)h * p.dl_sh;
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

// ---------------------------------------------------------------------------
// bias gradient, specialised (dense bf16 bias, no region mask): one wavefront owns a
// 32-key x 32-query block of one head, keeps the bias and the running sum in registers
// (lane = query, registers = keys) and walks the chunk's rows in order; the operands
// of row b+1 are fetched while row b is computed.  Continuing from the stored value
// on later chunks keeps the order of additions independent of k.
// ---------------------------------------------------------------------------
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) void dbias_fast_kernel(KP p) {
  constexpr int KS = D / 16;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const BlockId blk = xcd_block_id();  // one head's blocks share an XCD: its rows are fetched into one L2
  const int h = p.h0 + blk.z;
  const int q0 = blk.y * 32;
  const int k0 = (blk.x * 4 + w) * 32;
  if (k0 >= p.S) return;
  const int q = q0 + r, qc = min(q, p.S - 1);
  const int kr = min(k0 + r, p.S - 1);  // key row this lane supplies to the A operands
  float* dst = p.dbias_acc + ((int64_t)h * p.S + qc) * p.S;
  if (CAUSAL && k0 > q0 + 31) {  // block entirely above the diagonal: gradient is zero
    if (!p.dbias_accumulate && q < p.S) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int kb = k0 + 8 * g + 4 * hl;
        if (kb + 3 < p.S) *(f32x4*)(dst + kb) = f32x4{0.f, 0.f, 0.f, 0.f};
        else for (int e = 0; e < 4; ++e) if (kb + e < p.S) dst[kb + e] = 0.f;
      }
    }
    return;
  }
  float acc[16], bz[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int k = min(k0 + key_of(v, hl), p.S - 1);
    acc[v] = p.dbias_accumulate ? dst[k] : 0.f;
    bz[v] = bf2f(((const uint16_t*)p.bias)[((int64_t)h * p.S + qc) * p.S + k]) * LOG2E;
  }
  const float c1 = p.scale * LOG2E;
  const int64_t row_q = (int64_t)h * p.sh + (int64_t)qc * p.ss;
  const int64_t row_k = (int64_t)h * p.sh + (int64_t)kr * p.ss;
  const int64_t row_g = (int64_t)h * p.do_sh + (int64_t)qc * p.do_ss;
  const int64_t st_off = (int64_t)h * p.lse_sh + qc, dl_off = (int64_t)h * p.dl_sh + qc;
  constexpr int NS = D <= 32 ? 4 : 2;  // operand slots: rows b+1 .. b+NS-1 are in flight while row b is computed
  bf16x8 fq[NS][KS], fk[NS][KS], fv[NS][KS], fg[NS][KS];
  float lse2[NS], dlt[NS];
  auto fetch = [&](int b, int slot) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = 16 * ks + 8 * hl;
      fq[slot][ks] = *(const bf16x8*)((const uint16_t*)p.Q + (int64_t)b * p.sb + row_q + c);
      fk[slot][ks] = *(const bf16x8*)((const uint16_t*)p.K + (int64_t)b * p.sb + row_k + c);
      fv[slot][ks] = *(const bf16x8*)((const uint16_t*)p.V + (int64_t)b * p.sb + row_k + c);
      fg[slot][ks] = *(const bf16x8*)((const uint16_t*)p.dO + (int64_t)b * p.do_sb + row_g + c);
    }
    lse2[slot] = p.lse[(int64_t)b * p.lse_sb + st_off];  // scaled at use: no arithmetic on in-flight loads
    dlt[slot] = p.delta[(int64_t)b * p.dl_sb + dl_off];
  };
  auto step = [&](int slot, bool valid) {
    const float lse2s = lse2[slot] * LOG2E;
    f32x16 sa, pa;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      sa = mfma(fk[slot][ks], fq[slot][ks], sa);
      pa = mfma(fv[slot][ks], fg[slot][ks], pa);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float e = fast_exp2(fmaf(sa[v], c1, bz[v] - lse2s));
      float t = valid ? pa[v] - dlt[slot] : 0.f;
      if (CAUSAL) t = k0 + key_of(v, hl) > q ? 0.f : t;
      // one explicit fused multiply-add; a padding row contributes e * 0
      acc[v] = __builtin_fmaf(e, t, acc[v]);
    }
  };
  // rows are taken in groups of NS aligned to multiples of NS of the global row index, row b
  // always using slot b % NS: a given row passes through the same copy of the arithmetic whatever
  // the chunk boundaries are; rows of a group outside the chunk are padding rows of weight zero
  const int bs = p.b0 - p.b0 % NS;
  auto clampb = [&](int b) { return min(max(b, p.b0), p.b1 - 1); };
#pragma unroll
  for (int s_ = 0; s_ < NS - 1; ++s_) fetch(clampb(bs + s_), s_);
  for (int b = bs; b < p.b1; b += NS) {
#pragma unroll
    for (int s_ = 0; s_ < NS; ++s_) {
      fetch(clampb(b + s_ + NS - 1), (s_ + NS - 1) % NS);
      step(s_, b + s_ >= p.b0 && b + s_ < p.b1);
    }
  }
  if (q < p.S) {
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

// the specialised kernels serve: no bias or a dense bf16 bias with S % 4 == 0; no mask or the
// causal mask; a positive scale; more than one 64-key tile's worth of rows
inline bool fast_ok(const KP& p) {
  if (p.S <= 64 || !(p.scale > 0.f) || p.mask_kind == 2 || p.bias_kind == 2) return false;
  if (p.bias_kind == 1 && (!p.bias_bf16 || (p.S & 3))) return false;
  return true;
}

// eight-wavefront work-groups (two key-tile groups) when the whole share offers fewer
// work-groups than two per compute unit and there are enough key tiles to split
inline bool use_two_groups(const KP& p) {
  const int64_t wgs = (int64_t)((p.S + 127) / 128) * p.share_units;
  return wgs < 512 && p.S >= 512;
}

template <int D, bool RECOMP, int NG>
void fwd_fast_launch(const KP& p, dim3 g, hipStream_t st) {
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) fwd_fast_kernel<D, true, true, RECOMP, NG><<<g, 256 * NG, 0, st>>>(p);
  else if (bias) fwd_fast_kernel<D, true, false, RECOMP, NG><<<g, 256 * NG, 0, st>>>(p);
  else if (causal) fwd_fast_kernel<D, false, true, RECOMP, NG><<<g, 256 * NG, 0, st>>>(p);
  else fwd_fast_kernel<D, false, false, RECOMP, NG><<<g, 256 * NG, 0, st>>>(p);
}

template <int D>
hipError_t fwd_d(const KP& p, bool recompute, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (fast_ok(p)) {
    dim3 g((p.S + 127) / 128, Hc, Bc);
    if (use_two_groups(p)) {
      if (recompute) fwd_fast_launch<D, true, 2>(p, g, st);
      else fwd_fast_launch<D, false, 2>(p, g, st);
    } else {
      if (recompute) fwd_fast_launch<D, true, 1>(p, g, st);
      else fwd_fast_launch<D, false, 1>(p, g, st);
    }
    return hipGetLastError();
  }
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
template <int D, int NG>
void dq_fast_launch(const KP& p, dim3 g, hipStream_t st) {
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) dq_fast_kernel<D, true, true, NG><<<g, 256 * NG, 0, st>>>(p);
  else if (bias) dq_fast_kernel<D, true, false, NG><<<g, 256 * NG, 0, st>>>(p);
  else if (causal) dq_fast_kernel<D, false, true, NG><<<g, 256 * NG, 0, st>>>(p);
  else dq_fast_kernel<D, false, false, NG><<<g, 256 * NG, 0, st>>>(p);
}

template <int D>
hipError_t dq_d(const KP& p, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (fast_ok(p)) {
    dim3 g((p.S + 127) / 128, Hc, Bc);
    if (use_two_groups(p)) dq_fast_launch<D, 2>(p, g, st);
    else dq_fast_launch<D, 1>(p, g, st);
    return hipGetLastError();
  }
  if (p.S <= 64) mfma_dq_kernel<D, 2><<<dim3((p.S + 63) / 64, Hc, Bc), 128, 0, st>>>(p);
  else mfma_dq_kernel<D, 4><<<dim3((p.S + 127) / 128, Hc, Bc), 256, 0, st>>>(p);
  return hipGetLastError();
}
template <int D>
hipError_t dkdv_d(const KP& p, hipStream_t st) {
  const int Hc = p.h1 - p.h0, Bc = p.b1 - p.b0;
  if (fast_ok(p)) {
    dim3 g((p.S + 127) / 128, Hc, Bc);
    const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
    if (bias && causal) dkdv_fast_kernel<D, true, true><<<g, 256, 0, st>>>(p);
    else if (bias) dkdv_fast_kernel<D, true, false><<<g, 256, 0, st>>>(p);
    else if (causal) dkdv_fast_kernel<D, false, true><<<g, 256, 0, st>>>(p);
    else dkdv_fast_kernel<D, false, false><<<g, 256, 0, st>>>(p);
    return hipGetLastError();
  }
  if (p.S <= 64) mfma_dkdv_kernel<D, 2><<<dim3((p.S + 63) / 64, Hc, Bc), 128, 0, st>>>(p);
  else mfma_dkdv_kernel<D, 4><<<dim3((p.S + 127) / 128, Hc, Bc), 256, 0, st>>>(p);
  return hipGetLastError();
}
template <int D>
hipError_t dbias_d(const KP& p, hipStream_t st) {
  if (fast_ok(p) && p.bias_kind == 1) {
    dim3 g((p.S + 127) / 128, (p.S + 31) / 32, p.h1 - p.h0);
    if (p.mask_kind == 1) dbias_fast_kernel<D, true><<<g, 256, 0, st>>>(p);
    else dbias_fast_kernel<D, false><<<g, 256, 0, st>>>(p);
    return hipGetLastError();
  }
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

hipError_t launch_mfma_fwd(const KP& p, bool recompute, hipStream_t st) { SS_DISPATCH_D(fwd_d, p, recompute, st) }
hipError_t launch_mfma_dq(const KP& p, hipStream_t st) { SS_DISPATCH_D(dq_d, p, st) }
hipError_t launch_mfma_dkdv(const KP& p, hipStream_t st) { SS_DISPATCH_D(dkdv_d, p, st) }
hipError_t launch_mfma_dbias(const KP& p, hipStream_t st) { SS_DISPATCH_D(dbias_d, p, st) }

bool mfma_wants_bias_transpose(const KP& p) { return fast_ok(p) && p.bias_kind == 1; }

hipError_t launch_bias_transpose(const void* bias, void* biasT, int S, int h0, int h1, hipStream_t st) {
  dim3 g((S + 31) / 32, (S + 31) / 32, h1 - h0);
  bias_transpose_kernel<<<g, 256, 0, st>>>((const uint16_t*)bias, (uint16_t*)biasT, S, h0);
  return hipGetLastError();
}

}  // namespace ssa
