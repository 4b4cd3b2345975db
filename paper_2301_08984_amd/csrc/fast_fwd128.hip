// Forward / recompute kernel for large shares at head size 128 without a bias: the 128-query
// work-group of fast_fwd.hip (four wavefronts of 32 queries that share every 64-key K / V tile) with
// the tiles fetched from memory straight into LDS (wave_dma.h).
//
// The register-staged kernel spends, per tile and wavefront, about 50 vector instructions on load
// addresses, 16 `ds_write_b128`, 64 staging registers and two barriers, and its single tile buffer
// keeps loads, stores and arithmetic from overlapping.  Here a tile is 32 `buffer_load ... lds`
// (8 per wavefront, lane offsets that never change), the tiles alternate between two buffers and
// one barrier per tile does both jobs: "tile kt has landed for everybody" and "everybody is done
// with the other buffer", after which the loads of tile kt + 1 start and have a whole step to land.
#include "wave_dma.h"

#include <type_traits>

namespace ssa {
namespace {

constexpr int F_STAGE_B = 4 * W_TILE_B;  // K rows 0..31, K rows 32..63, V rows 0..31, V rows 32..63

template <bool CAUSAL, bool RECOMP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_fast128_kernel(KP p) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, BM = 128, BN = 64;
  __shared__ __attribute__((aligned(1024))) char smem[2 * F_STAGE_B];
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const BlockId blk = xcd_block_id(false);
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * BM;  // long (late) causal blocks first
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + BM, p.S) + BN - 1) / BN);
  int wtiles = ntiles;  // tiles holding at least one key visible to this wavefront
  if (CAUSAL) wtiles = min(ntiles, (min(q0 + 32, p.S) + BN - 1) / BN);
  if (q0 >= p.S) wtiles = 0;

  // this wavefront's share of a tile: load instructions 2w and 2w+1 of each of its four sub-tiles
  const uint32_t ss2 = (uint32_t)p.ss * 2u;
  const uint32_t slice = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  uint32_t goff[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int rho = 4 * (2 * w + u) + (lane >> 4);
    goff[u] = (uint32_t)rho * ss2 + 16u * (uint32_t)((lane & 15) ^ w_sw(rho));
  }
  auto fetch_tile = [&](char* stage, int kt) {
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const int row0 = kt * BN + 32 * (sub & 1);
      // a sub-tile past the last row: an empty descriptor, zeros arrive
      const uint32_t boff = row0 < p.S ? (uint32_t)row0 * ss2 : slice;
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          (void*)((const char*)(sub < 2 ? Kb : Vb) + boff), 0, (int)(slice - boff), 0x00020000);
#pragma unroll
      for (int u = 0; u < 2; ++u)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (w_lds_void*)(stage + sub * W_TILE_B + (2 * w + u) * 1024), 16,
                                                 goff[u], 0, 0, 0);
    }
  };
  uint32_t ka[8], va[2][4];
  w_nat_addr(ka, smem, r, hl);
  w_tr_addr(va, smem, lane);

  fetch_tile(smem, 0);
  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) qf[ks] = *(const bf16x8*)(Qb + (int64_t)qc * p.ss + 16 * ks + 8 * hl);
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;

  // one key tile in the stage buffer SB bytes into LDS: scores, online softmax, value product
  auto tile = [&](auto sb, int k0) {
    constexpr int SB = decltype(sb)::value;
    f32x16 sa[2];
    {
      u32x4 fa[KS], fb[KS];
      w_nat_issue<SB>(fa, ka);
      w_nat_issue<SB + W_TILE_B>(fb, ka);
      w_nat_wait(fa);
      w_nat_wait(fb);
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[0][v] = 0.f; sa[1][v] = 0.f; }
      // the two score blocks alternate so that consecutive MFMAs never wait on each other's accumulator
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa[0] = mfma(w_frag(fa[ks]), qf[ks], sa[0]);
        sa[1] = mfma(w_frag(fb[ks]), qf[ks], sa[1]);
      }
    }
    // the transposed fragments of the first half of V arrive under the softmax arithmetic
    u32x2 vt[2][2 * DB];
    w_tr_issue<SB + 2 * W_TILE_B>(vt, va);
    if ((k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0)) {
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
    rmax *= c1;  // the running maximum is kept in base-2 units; scale > 0 on this path
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
    bf16x8 pf[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      float pr[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        pr[v] = fast_exp2(fmaf(sa[kb][v], c1, -m));
        lsum += pr[v];
      }
      pf[2 * kb] = pack8(&pr[0]);
      pf[2 * kb + 1] = pack8(&pr[8]);
    }
    l += lsum;
    w_tr_wait(vt);
    // ... and those of the second half under the products with the first
    u32x2 vu[2][2 * DB];
    w_tr_issue<SB + 3 * W_TILE_B>(vu, va);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(w_frag2(vt[t][2 * db], vt[t][2 * db + 1]), pf[t], oacc[db]);
    w_tr_wait(vu);
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(w_frag2(vu[t][2 * db], vu[t][2 * db + 1]), pf[2 + t], oacc[db]);
  };
  // step kt: tile kt is on its way into buffer kt % 2
  auto step = [&](auto sb, int kt) {
    constexpr int SB = decltype(sb)::value;
    W_VMCNT(0);  // this wavefront's part of tile kt has landed
    __builtin_amdgcn_s_barrier();  // ... everybody's; and everybody is done with the other buffer
    asm volatile("" ::: "memory");
    if (kt + 1 < ntiles) fetch_tile(smem + (F_STAGE_B - SB), kt + 1);
    if (kt < wtiles) tile(sb, kt * BN);
  };
  int kt = 0;
  for (; kt + 1 < ntiles; kt += 2) {
    step(std::integral_constant<int, 0>{}, kt);
    step(std::integral_constant<int, F_STAGE_B>{}, kt + 1);
  }
  if (kt < ntiles) step(std::integral_constant<int, 0>{}, kt);
  if (q >= p.S) return;
  fwd_epilogue<DB, RECOMP>(p, oacc, m, l, b, h, q, hl, base);
}

}  // namespace

hipError_t launch_fast_fwd128(const KP& p, bool recompute, hipStream_t st) {
  const dim3 g((p.S + 127) / 128, p.h1 - p.h0, p.b1 - p.b0);
  const bool causal = p.mask_kind == 1;
  if (recompute) {
    if (causal) fwd_fast128_kernel<true, true><<<g, 256, 0, st>>>(p);
    else fwd_fast128_kernel<false, true><<<g, 256, 0, st>>>(p);
  } else {
    if (causal) fwd_fast128_kernel<true, false><<<g, 256, 0, st>>>(p);
    else fwd_fast128_kernel<false, false><<<g, 256, 0, st>>>(p);
  }
  return hipGetLastError();
}

}  // namespace ssa
