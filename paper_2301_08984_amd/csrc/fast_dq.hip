// Specialised dQ kernel (see the comment above the kernel).
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

// ---------------------------------------------------------------------------
// dQ, specialised like the forward (dense bf16 bias / causal at compile time, NG key-tile
// groups).  Q and dO fragments stay in registers; per 32-key block the scores and dP come
// from the matrix cores, dS from the vector ALUs, and dQ^T += K^T dS^T reads the same K
// tile transposed.
// ---------------------------------------------------------------------------
template <int D, bool BIAS, bool CAUSAL, int QW, int NG>
// D = 32 needs 100 - 140 registers: three (with a bias) or four wavefronts per SIMD instead of two
__global__ __launch_bounds__(64 * QW * NG)
__attribute__((amdgpu_waves_per_eu(D <= 32 ? (BIAS ? 3 : 4) : 2, D <= 32 ? (BIAS ? 3 : 4) : 2))) void dq_fast_kernel(KP p) {
  constexpr int KS = D / 16, DB = D / 32, NT = 64 * QW, BM = 32 * QW;
  constexpr int LDK = D + 24, LDV = D + 8;  // K is read both ways: D + 24 is conflict-free for b128 and transposed reads
  constexpr int CPR = D / 8, CPT = BN * CPR / NT;
  constexpr int TILE_ELEMS = BN * LDK + BN * LDV;
  constexpr int MERGE_ELEMS = NT * (16 * DB) * 2 * (NG - 1);
  constexpr int BIAS_ELEMS = BIAS ? BIAS_TILE_ELEMS * QW * NG : 0;  // one parked bias tile per wavefront
  constexpr int KV_ELEMS = NG * TILE_ELEMS;
  constexpr int LDS_ELEMS = KV_ELEMS + BIAS_ELEMS > MERGE_ELEMS ? KV_ELEMS + BIAS_ELEMS : MERGE_ELEMS;
  __shared__ __attribute__((aligned(16))) uint16_t smem[LDS_ELEMS];
  const int tid = threadIdx.x % NT, grp = threadIdx.x / NT;
  const int lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  uint16_t* sK = smem + grp * TILE_ELEMS;
  uint16_t* sV = sK + BN * LDK;
  const BlockId blk = xcd_block_id(BIAS && bias_rows_first(gridDim.y, p.S));
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * BM;
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  BiasTile bt;
  if (BIAS)
    bt.init((const uint16_t*)p.bias + (int64_t)h * p.S * p.S, q0, p.S,
            smem + KV_ELEMS + (threadIdx.x >> 6) * BIAS_TILE_ELEMS, lane);

  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *(const bf16x8*)(Qb + (int64_t)qc * p.ss + 16 * ks + 8 * hl);
    gf[ks] = *(const bf16x8*)(dOb + (int64_t)qc * p.do_ss + 16 * ks + 8 * hl);
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
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + BM, p.S) + BN - 1) / BN);
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
  // the bias slice of the next tile travels with the next K/V tile
  auto bload = [&](int kt) { bt.load(kt); };
  if (grp < ntiles) {
    gload(grp);
    if (BIAS) bload(grp);
  }
  const int nit = (ntiles + NG - 1) / NG;
  for (int it = 0; it < nit; ++it) {
    const int kt = it * NG + grp;
    const int k0 = kt * BN;
    __syncthreads();
    if (kt < ntiles) {
      if (BIAS) bt.park(lane);
#pragma unroll
      for (int c = 0; c < CPT; ++c) {
        const int idx = tid + c * NT, row = idx / CPR, col = (idx % CPR) * 8;
        *(u32x4*)(sK + row * LDK + col) = pk[c];
        *(u32x4*)(sV + row * LDV + col) = pv[c];
      }
      if (kt + NG < ntiles) {
        gload(kt + NG);
        if (BIAS) bload(kt + NG);
      }
    }
    __syncthreads();
    if (kt >= wtiles) continue;
    const bool edge = (k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      uint2 bz[4];
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
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) bz[g] = bt.read(r, 32 * kb + 8 * g + 4 * hl);
      }
      float ds[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float bl[4] = {0.f, 0.f, 0.f, 0.f};
        if (BIAS) {
          bl[0] = __uint_as_float(bz[g].x << 16); bl[1] = __uint_as_float(bz[g].x & 0xffff0000u);
          bl[2] = __uint_as_float(bz[g].y << 16); bl[3] = __uint_as_float(bz[g].y & 0xffff0000u);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // with a bias: natural units first, the change to base 2 rides on the subtraction of the LSE
          float pe = BIAS ? fast_exp2(fmaf(fmaf(sa[4 * g + e], p.scale, bl[e]), LOG2E, -lse2))
                          : fast_exp2(fmaf(sa[4 * g + e], c1, -lse2));
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
    // groups 1.. hand their partial dQ to group 0, which adds them in group order
    constexpr int SLOT = NT * 16 * DB;
    float* mb = (float*)smem + (size_t)tid * (16 * DB);
    __syncthreads();
    if (grp > 0) {
      float* my = mb + (size_t)(grp - 1) * SLOT;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) my[16 * db + v] = acc[db][v];
    }
    __syncthreads();
    if (grp > 0) return;
#pragma unroll
    for (int g = 1; g < NG; ++g)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[db][v] += mb[(size_t)(g - 1) * SLOT + 16 * db + v];
  }
  if (q >= p.S) return;
  uint16_t* out = (uint16_t*)p.dQ + base + (int64_t)q * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 o[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      o[g] = pack4_bf16(acc[db][4 * g], acc[db][4 * g + 1], acc[db][4 * g + 2], acc[db][4 * g + 3], p.scale);
    store_row32(out + 32 * db, o, hl, true);
  }
}

template <int D, int QW, int NG>
void dq_fast_launch(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 32 * QW - 1) / (32 * QW), p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) dq_fast_kernel<D, true, true, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else if (bias) dq_fast_kernel<D, true, false, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else if (causal) dq_fast_kernel<D, false, true, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
  else dq_fast_kernel<D, false, false, QW, NG><<<g, 64 * QW * NG, 0, st>>>(p);
}

template <int D>
hipError_t dq_d(const KP& p, hipStream_t st) {
  switch (wg_shape(p)) {
    case WG_4x2: dq_fast_launch<D, 4, 2>(p, st); break;
    default: dq_fast_launch<D, 4, 1>(p, st); break;
  }
  return hipGetLastError();
}

}  // namespace

#define SS_FAST_DISPATCH_D(fn, ...)               \
  switch (p.D) {                                  \
    case 32: return fn<32>(__VA_ARGS__);          \
    case 64: return fn<64>(__VA_ARGS__);          \
    case 128: return fn<128>(__VA_ARGS__);        \
    default: return hipErrorInvalidValue;         \
  }
hipError_t launch_fast_dq(const KP& p, hipStream_t st) {
  // large shares at head size 128 without a bias: tiles straight into LDS
  if (p.D == 128 && p.bias_kind == 0 && wg_shape(p) == WG_4x1) return launch_fast_dq128(p, st);
  SS_FAST_DISPATCH_D(dq_d, p, st)
}

}  // namespace ssa
