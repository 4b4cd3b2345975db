// dQ for large shares at head size 128 without a bias: the 128-query work-group of fast_dq.hip with
// the K / V tiles fetched from memory straight into two LDS buffers (wave_dma.h, and the header of
// fast_fwd128.hip for the buffer scheme).  Q and dO fragments stay in registers; per 32-key block
// the scores and dP come from the matrix cores, dS from the vector ALUs, and dQ^T += K^T dS^T reads
// the same K sub-tile transposed.
#include "wave_dma.h"

#include <type_traits>

namespace ssa {
namespace {

constexpr int Q_STAGE_B = 4 * W_TILE_B;  // K rows 0..31, K rows 32..63, V rows 0..31, V rows 32..63

template <bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void dq_fast128_kernel(KP p) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, BM = 128, BN = 64;
  __shared__ __attribute__((aligned(1024))) char smem[2 * Q_STAGE_B];
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const BlockId blk = xcd_block_id(false);
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int qblk = (gridDim.x - 1 - blk.x) * BM;
  const int q0 = qblk + 32 * w, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float c1 = p.scale * LOG2E;

  int ntiles = (p.S + BN - 1) / BN;
  if (CAUSAL) ntiles = min(ntiles, (min(qblk + BM, p.S) + BN - 1) / BN);
  int wtiles = ntiles;
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
  bf16x8 qf[KS], gf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    qf[ks] = *(const bf16x8*)(Qb + (int64_t)qc * p.ss + 16 * ks + 8 * hl);
    gf[ks] = *(const bf16x8*)(dOb + (int64_t)qc * p.do_ss + 16 * ks + 8 * hl);
  }
  const float nlse2 = -p.lse[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + qc] * LOG2E;
  const float delta = p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + qc];
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // one 32-key half (K sub-tile KO bytes, V sub-tile VO bytes into LDS) of a tile
  auto half = [&](auto ko, auto vo, int k0, bool edge) {
    constexpr int KO = decltype(ko)::value, VO = decltype(vo)::value;
    f32x16 sa, pa;
    {
      u32x4 fk[KS], fv[KS];
      w_nat_issue<KO>(fk, ka);
      w_nat_issue<VO>(fv, ka);
      w_nat_wait(fk);
      w_nat_wait(fv);
#pragma unroll
      for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sa = mfma(w_frag(fk[ks]), qf[ks], sa);
        pa = mfma(w_frag(fv[ks]), gf[ks], pa);
      }
    }
    // the transposed fragments of K arrive under the arithmetic on the scores
    u32x2 kt_[2][2 * DB];
    w_tr_issue<KO>(kt_, va);
    if (edge) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = k0 + key_of(v, hl);
        const bool dead = key >= p.S || (CAUSAL && key > q);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    bf16x8 df[2];
    {
      float ds[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) ds[v] = fast_exp2(fmaf(sa[v], c1, nlse2)) * (pa[v] - delta);
      df[0] = pack8(&ds[0]);
      df[1] = pack8(&ds[8]);
    }
    w_tr_wait(kt_);
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(w_frag2(kt_[hb][2 * db], kt_[hb][2 * db + 1]), df[hb], acc[db]);
  };
  // step kt: tile kt is on its way into buffer kt % 2
  auto step = [&](auto sb, int kt) {
    constexpr int SB = decltype(sb)::value;
    W_VMCNT(0);  // this wavefront's part of tile kt has landed
    __builtin_amdgcn_s_barrier();  // ... everybody's; and everybody is done with the other buffer
    asm volatile("" ::: "memory");
    if (kt + 1 < ntiles) fetch_tile(smem + (Q_STAGE_B - SB), kt + 1);
    if (kt < wtiles) {
      const int k0 = kt * BN;
      const bool edge = (k0 + BN > p.S) || (CAUSAL && k0 + BN - 1 > q0);
      half(std::integral_constant<int, SB>{}, std::integral_constant<int, SB + 2 * W_TILE_B>{}, k0, edge);
      half(std::integral_constant<int, SB + W_TILE_B>{}, std::integral_constant<int, SB + 3 * W_TILE_B>{}, k0 + 32, edge);
    }
  };
  int kt = 0;
  for (; kt + 1 < ntiles; kt += 2) {
    step(std::integral_constant<int, 0>{}, kt);
    step(std::integral_constant<int, Q_STAGE_B>{}, kt + 1);
  }
  if (kt < ntiles) step(std::integral_constant<int, 0>{}, kt);
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

}  // namespace

hipError_t launch_fast_dq128(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 127) / 128, p.h1 - p.h0, p.b1 - p.b0);
  if (p.mask_kind == 1) dq_fast128_kernel<true><<<g, 256, 0, st>>>(p);
  else dq_fast128_kernel<false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace ssa
