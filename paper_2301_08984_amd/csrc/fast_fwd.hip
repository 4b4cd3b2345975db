// Specialised forward / recompute kernel (see the comment above the kernel).
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

// ---------------------------------------------------------------------------
// forward / recompute, specialised at compile time on the presence of a dense bf16
// bias and of the causal mask.  The inner loop is straight-line code: loads are
// clamped instead of guarded, and tiles that need no per-element masking (all keys
// below the causal diagonal and inside S) take a path without compares.
//
// A work-group is QW query wavefronts (32 queries each) times NG key-tile groups:
// group g takes the key tiles kt = g, g+NG, ... with its own LDS tiles and its own
// (O, m, l); the partial softmax results are merged through LDS at the end, in
// group order.  With NG > 1 two wavefronts share every SIMD, so one's softmax
// arithmetic overlaps the other's matrix products, and the serial chain of key
// tiles per wavefront is NG times shorter; small shares use fewer query wavefronts
// and more groups so that more compute units get a work-group.  The shape is
// chosen from the size of the whole share, never from the chunk, so results do
// not depend on k.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, bool RECOMP, int QW, int NG>
__global__ __launch_bounds__(64 * QW * NG) __attribute__((amdgpu_waves_per_eu(D <= 32 ? (BIAS && (CAUSAL || NG > 1) ? 3 : 4) : 2, D <= 32 ? (BIAS && (CAUSAL || NG > 1) ? 3 : 4) : 2))) void fwd_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, NT = 64 * QW, BM = 32 * QW;
  constexpr int LDK = D + 8, LDV = D + 16;  // row pads chosen for conflict-free b128 / transpose reads
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  constexpr int TILE_ELEMS = BN * LDK + BN * LDV;
  constexpr bool DBUF = D <= 64;  // two tile buffers per group where LDS is plentiful
  constexpr int NBUF = DBUF ? 2 : 1;
  constexpr int MERGE_ELEMS = NT * (16 * DB + 2) * 2 * (NG - 1);  // in uint16 units
  constexpr int BIAS_ELEMS = BIAS ? BIAS_TILE_ELEMS * QW * NG : 0;  // one parked bias tile per wavefront
  constexpr int KV_ELEMS = NG * NBUF * TILE_ELEMS;
  constexpr int LDS_ELEMS = KV_ELEMS + BIAS_ELEMS > MERGE_ELEMS ? KV_ELEMS + BIAS_ELEMS : MERGE_ELEMS;
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int tid = threadIdx.x % NT, grp = threadIdx.x / NT;
  const int lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  uint16_t* sK = smem + grp * NBUF * TILE_ELEMS;
  uint16_t* sV = sK + BN * LDK;
  const BlockId blk = xcd_block_id(BIAS && bias_rows_first(gridDim.y, p.S));
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * BM;  // long (late) causal blocks first
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  BiasTile bt;
  if (BIAS)
    bt.init((const uint16_t*)p.bias + (int64_t)h * p.S * p.S, q0, p.S,
            smem + KV_ELEMS + (threadIdx.x >> 6) * BIAS_TILE_ELEMS, lane);

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
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + BM, p.S) + BN - 1) / BN);
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
  // the bias slice of the next tile travels with the next K/V tile
  auto bload = [&](int kt) { bt.load(kt); };
  auto bpark = [&]() { bt.park(lane); };  // read back by the next tile()
  if (grp < ntiles) {
    gload(grp);
    if (BIAS) bload(grp);
  }
  // one key tile: scores, online softmax, value product (tile in LDS at sK / sV, bias slice bz)
  auto tile = [&](const uint16_t* sK, const uint16_t* sV, int k0) {
    f32x16 sa[2];
    uint2 bz[8];
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
    if (BIAS) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g) bz[4 * kb + g] = bt.read(r, 32 * kb + 8 * g + 4 * hl);
    }
    const bool edge = (k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0);
    if (BIAS) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint2 u = bz[4 * kb + g];
          // natural units here; the change to base 2 rides on the subtraction of the maximum below
          sa[kb][4 * g + 0] = fmaf(sa[kb][4 * g + 0], p.scale, __uint_as_float(u.x << 16));
          sa[kb][4 * g + 1] = fmaf(sa[kb][4 * g + 1], p.scale, __uint_as_float(u.x & 0xffff0000u));
          sa[kb][4 * g + 2] = fmaf(sa[kb][4 * g + 2], p.scale, __uint_as_float(u.y << 16));
          sa[kb][4 * g + 3] = fmaf(sa[kb][4 * g + 3], p.scale, __uint_as_float(u.y & 0xffff0000u));
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
    rmax *= BIAS ? LOG2E : c1;  // the running maximum is kept in base-2 units; scale > 0 on this path
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
        sa[kb][v] = fast_exp2(fmaf(sa[kb][v], BIAS ? LOG2E : c1, -m));
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
  
  };
  auto stage = [&](uint16_t* dK, uint16_t* dV) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(dK + row * LDK + col) = pk[c];
      *(u32x4*)(dV + row * LDV + col) = pv[c];
    }
  };
  const int nit = (ntiles + NG - 1) / NG;
  if (DBUF) {
    // two tile buffers per group and one barrier per tile: while a tile is multiplied the next one
    // is already in registers; it is written to the other buffer after the multiplication, which
    // every wavefront finished reading before the previous barrier
    if (grp < ntiles) {
      stage(sK, sV);
      if (BIAS) bpark();
      if (grp + NG < ntiles) {
        gload(grp + NG);
        if (BIAS) bload(grp + NG);
      }
    }
    __syncthreads();
    for (int it = 0; it < nit; ++it) {
      const int kt = it * NG + grp;
      uint16_t* cK = sK + (it & 1) * TILE_ELEMS;
      uint16_t* nK = sK + ((it + 1) & 1) * TILE_ELEMS;
      if (kt < wtiles) tile(cK, cK + BN * LDK, kt * BN);
      if (kt + NG < ntiles) {
        stage(nK, nK + BN * LDK);
        if (BIAS) bpark();
        if (kt + 2 * NG < ntiles) {
          gload(kt + 2 * NG);
          if (BIAS) bload(kt + 2 * NG);
        }
      }
      __syncthreads();
    }
  } else {
    for (int it = 0; it < nit; ++it) {
      const int kt = it * NG + grp;
      __syncthreads();
      if (kt < ntiles) {
        stage(sK, sV);
        if (BIAS) bpark();
        if (kt + NG < ntiles) {
          gload(kt + NG);
          if (BIAS) bload(kt + NG);
        }
      }
      __syncthreads();
      if (kt < wtiles) tile(sK, sV, kt * BN);
    }
  }
  if (NG > 1) {
    // merge the groups' partial softmax results: groups 1.. hand (O, m, l) to group 0, which folds
    // them in group order
    constexpr int SLOT = NT * (16 * DB + 2);
    float* mb = (float*)smem + (size_t)tid * (16 * DB + 2);
    __syncthreads();
    if (grp > 0) {
      float* my = mb + (size_t)(grp - 1) * SLOT;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) my[16 * db + v] = oacc[db][v];
      my[16 * DB] = m;
      my[16 * DB + 1] = l;
    }
    __syncthreads();
    if (grp > 0) return;
#pragma unroll
    for (int g = 1; g < NG; ++g) {
      const float* o = mb + (size_t)(g - 1) * SLOT;
      const float m1 = o[16 * DB], l1 = o[16 * DB + 1];
      const float mn = fmaxf(m, m1);
      const float a0 = fast_exp2(m - mn), a1 = fast_exp2(m1 - mn);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[db][v] = oacc[db][v] * a0 + o[16 * db + v] * a1;
      l = l * a0 + l1 * a1;
      m = mn;
    }
  }
  if (q >= p.S) return;
  fwd_epilogue<DB, RECOMP>(p, oacc, m, l, b, h, q, hl, base);
}

template <int D, bool RECOMP, int QW, int NG>
void fwd_fast_launch(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 32 * QW - 1) / (32 * QW), p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) fwd_fast_kernel<D, true, true, RECOMP, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else if (bias) fwd_fast_kernel<D, true, false, RECOMP, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else if (causal) fwd_fast_kernel<D, false, true, RECOMP, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else fwd_fast_kernel<D, false, false, RECOMP, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
}

template <int D, bool RECOMP>
hipError_t fwd_r(const KP& p, hipStream_t st) {
  switch (wg_shape(p)) {
    case WG_4x2: fwd_fast_launch<D, RECOMP, 4, 2>(p, st); break;
    default: fwd_fast_launch<D, RECOMP, 4, 1>(p, st); break;
  }
  return hipGetLastError();
}
template <int D>
hipError_t fwd_d(const KP& p, bool recompute, hipStream_t st) {
  return recompute ? fwd_r<D, true>(p, st) : fwd_r<D, false>(p, st);
}

}  // namespace

#define SS_FAST_DISPATCH_D(fn, ...)               \
  switch (p.D) {                                  \
    case 32: return fn<32>(__VA_ARGS__);          \
    case 64: return fn<64>(__VA_ARGS__);          \
    case 128: return fn<128>(__VA_ARGS__);        \
    default: return hipErrorInvalidValue;         \
  }
hipError_t launch_fast_fwd(const KP& p, bool recompute, hipStream_t st) {
  // small shares: 32-query work-groups whose wavefronts split the keys
  if (wg_shape(p) == WG_2x4) return launch_fast_fwd_wave(p, recompute, st);
  // large shares at head size 128 without a bias: tiles straight into LDS
  if (p.D == 128 && p.bias_kind == 0 && wg_shape(p) == WG_4x1) return launch_fast_fwd128(p, recompute, st);
  SS_FAST_DISPATCH_D(fwd_d, p, recompute, st)
}

}  // namespace ssa
