// dK and dV for large shares at head size 128 without a bias, one gradient per work-group.
//
// The key-stationary kernel of fast_dkdv.hip keeps both accumulators (128 registers) and the K and V
// fragments of its 32 keys in one wavefront, needs more than 400 registers and so runs one wavefront
// per SIMD.  Here a work-group of four wavefronts (32 keys each) produces dK (S = Q K^T, dP = dO V^T,
// dS, dK^T += Q^T dS) or dV (S, P, dV^T += dO^T P) for its 128 keys, fits 256 registers and 65 KB of
// LDS, and two work-groups share a compute unit; both kinds are one launch (position 2r is the dK
// group of key block r, 2r + 1 its dV group; early key blocks see the most queries under a causal
// mask and come first).  The scores are formed twice; the matrix cores have the room.
// The 64-query tiles of Q and dO go from memory straight into two LDS buffers (wave_dma.h, and the
// header of fast_fwd128.hip for the buffer scheme); the statistics of a tile's queries travel
// through a register of the first two wavefronts into the buffer's tail.
#include "wave_dma.h"

#include <type_traits>

namespace ssa {
namespace {

constexpr int KV_STAGE_B = 4 * W_TILE_B + 512;  // Q rows 0..31, 32..63, dO rows 0..31, 32..63, -lse2[64], Delta[64]

template <bool CAUSAL, int WHICH>  // WHICH = 1: dK, 0: dV
__device__ __forceinline__ void kv_fast128_block(const KP& p, char* smem, int rank, int by, int bz_) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, BK = 128, BN = 64;
  constexpr bool DK = WHICH == 1;
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int h = p.h0 + by, b = p.b0 + bz_;
  const int kblk = rank * BK;
  const int k0 = kblk + 32 * w, key = k0 + r;
  const int kc = min(key, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* dOb = (const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh;
  const float* lse_b = p.lse + (int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh;
  const float* dl_b = p.delta + (int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh;
  const float c1 = p.scale * LOG2E;
  const int ntiles = (p.S + BN - 1) / BN;
  const int first = CAUSAL ? kblk / BN : 0;  // queries before the block's first key see none of it

  // this wavefront's share of a tile: load instructions 2w and 2w+1 of each of its four sub-tiles
  const uint32_t ss2 = (uint32_t)p.ss * 2u, dss2 = (uint32_t)p.do_ss * 2u;
  const uint32_t slice = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  const uint32_t dslice = (uint32_t)(((int64_t)(p.S - 1) * p.do_ss + D) * 2);
  uint32_t goff[2], goff_g[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int rho = 4 * (2 * w + u) + (lane >> 4);
    const uint32_t c16 = 16u * (uint32_t)((lane & 15) ^ w_sw(rho));
    goff[u] = (uint32_t)rho * ss2 + c16;
    goff_g[u] = (uint32_t)rho * dss2 + c16;
  }
  // lanes of the first two wavefronts carry the statistics of the tile's queries: wavefront 0 the
  // LSE of query lane, wavefront 1 its Delta (dK only)
  float pstat = 0.f;
  auto fetch_tile = [&](char* stage, int qt) {
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const int row0 = qt * BN + 32 * (sub & 1);
      const bool q_ = sub < 2;
      // a sub-tile past the last row: an empty descriptor, zeros arrive
      const uint32_t boff = row0 < p.S ? (uint32_t)row0 * (q_ ? ss2 : dss2) : (q_ ? slice : dslice);
      const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
          (void*)((const char*)(q_ ? Qb : dOb) + boff), 0, (int)((q_ ? slice : dslice) - boff), 0x00020000);
#pragma unroll
      for (int u = 0; u < 2; ++u)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (w_lds_void*)(stage + sub * W_TILE_B + (2 * w + u) * 1024), 16,
                                                 q_ ? goff[u] : goff_g[u], 0, 0, 0);
    }
    if (w == 0) pstat = lse_b[min(qt * BN + lane, p.S - 1)];
    if (DK && w == 1) pstat = dl_b[min(qt * BN + lane, p.S - 1)];
  };
  uint32_t ka[8], va[2][4];
  w_nat_addr(ka, smem, r, hl);
  w_tr_addr(va, smem, lane);
  const uint32_t st_w = (uint32_t)(size_t)(w_lds_void*)(smem + 4 * W_TILE_B) + 256u * w + 4u * lane;  // w < 2
  const uint32_t st_r = (uint32_t)(size_t)(w_lds_void*)(smem + 4 * W_TILE_B) + 16u * hl;

  if (first < ntiles) fetch_tile(smem, first);
  bf16x8 kf[KS], vf[KS];  // vf: dK only
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    kf[ks] = *(const bf16x8*)(Kb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
    if (DK) vf[ks] = *(const bf16x8*)(Vb + (int64_t)kc * p.ss + 16 * ks + 8 * hl);
  }
  f32x16 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // one 32-query half of a tile: Q sub-tile QO bytes, dO sub-tile GO bytes, statistics SO bytes into LDS
  auto half = [&](auto qo, auto go, auto so, int i0, bool edge) {
    constexpr int QO = decltype(qo)::value, GO = decltype(go)::value, SO = decltype(so)::value;
    f32x16 sa, pa;
#pragma unroll
    for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
    {
      u32x4 fq[KS];
      w_nat_issue<QO>(fq, ka);
      if (DK) {
        u32x4 fg[KS];
        w_nat_issue<GO>(fg, ka);
        w_nat_wait(fq);
        w_nat_wait(fg);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          sa = mfma(w_frag(fq[ks]), kf[ks], sa);
          pa = mfma(w_frag(fg[ks]), vf[ks], pa);
        }
      } else {
        w_nat_wait(fq);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) sa = mfma(w_frag(fq[ks]), kf[ks], sa);
      }
    }
    // dK += Q^T dS, dV += dO^T P: the transposed fragments arrive under the arithmetic on the scores
    u32x2 tf[2][2 * DB];
    w_tr_issue<DK ? QO : GO>(tf, va);
    if (edge) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int qi = i0 + key_of(v, hl);
        const bool dead = qi >= p.S || key >= p.S || (CAUSAL && key > qi);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    bf16x8 of[2];  // P (dV) or dS (dK) as packed operands
    {
      float x[16];
      u32x4 l4[4];
      asm volatile("ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\tds_read_b128 %2, %4 offset:%7\n\t"
                   "ds_read_b128 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
                   : "=&v"(l4[0]), "=&v"(l4[1]), "=&v"(l4[2]), "=&v"(l4[3])
                   : "v"(st_r), "n"(SO), "n"(SO + 32), "n"(SO + 64), "n"(SO + 96)
                   : "memory");
#pragma unroll
      for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * g + e] = fast_exp2(fmaf(sa[4 * g + e], c1, __uint_as_float(l4[g][e])));
      if (DK) {
        u32x4 d4[4];
        asm volatile("ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\tds_read_b128 %2, %4 offset:%7\n\t"
                     "ds_read_b128 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
                     : "=&v"(d4[0]), "=&v"(d4[1]), "=&v"(d4[2]), "=&v"(d4[3])
                     : "v"(st_r), "n"(SO + 256), "n"(SO + 288), "n"(SO + 320), "n"(SO + 352)
                     : "memory");
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < 4; ++e) x[4 * g + e] *= pa[4 * g + e] - __uint_as_float(d4[g][e]);
      }
      of[0] = pack8(&x[0]);
      of[1] = pack8(&x[8]);
    }
    w_tr_wait(tf);
#pragma unroll
    for (int hb = 0; hb < 2; ++hb)
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] = mfma(w_frag2(tf[hb][2 * db], tf[hb][2 * db + 1]), of[hb], acc[db]);
  };
  // step qt: tile qt is on its way into buffer (qt - first) % 2, its statistics are in `pstat`
  auto step = [&](auto sb, int qt) {
    constexpr int SB = decltype(sb)::value;
    if (w < (DK ? 2 : 1))
      asm volatile("ds_write_b32 %0, %1 offset:%2" ::"v"(st_w), "v"(w == 0 ? -pstat * LOG2E : pstat), "n"(SB) : "memory");
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // this wavefront's part of tile qt has landed
    __builtin_amdgcn_s_barrier();  // ... everybody's; and everybody is done with the other buffer
    asm volatile("" ::: "memory");
    if (qt + 1 < ntiles) fetch_tile(smem + (KV_STAGE_B - SB), qt + 1);
    const int i0 = qt * BN;
    if (k0 >= p.S || (CAUSAL && i0 + BN - 1 < k0)) return;  // no visible pair for this wavefront
    const bool edge = (i0 + BN > p.S) || (k0 + 32 > p.S) || (CAUSAL && i0 < k0 + 31);
    half(std::integral_constant<int, SB>{}, std::integral_constant<int, SB + 2 * W_TILE_B>{},
         std::integral_constant<int, SB>{}, i0, edge);
    half(std::integral_constant<int, SB + W_TILE_B>{}, std::integral_constant<int, SB + 3 * W_TILE_B>{},
         std::integral_constant<int, SB + 128>{}, i0 + 32, edge);
  };
  int qt = first;
  for (; qt + 1 < ntiles; qt += 2) {
    step(std::integral_constant<int, 0>{}, qt);
    step(std::integral_constant<int, KV_STAGE_B>{}, qt + 1);
  }
  if (qt < ntiles) step(std::integral_constant<int, 0>{}, qt);
  if (key >= p.S) return;
  uint16_t* out = (uint16_t*)(DK ? p.dK : p.dV) + base + (int64_t)key * p.ss;
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    uint2 o[4];
#pragma unroll
    for (int g = 0; g < 4; ++g)
      o[g] = pack4_bf16(acc[db][4 * g], acc[db][4 * g + 1], acc[db][4 * g + 2], acc[db][4 * g + 3], DK ? p.scale : 1.f);
    store_row32(out + 32 * db, o, hl, true);
  }
}

template <bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void kv_fast128_kernel(KP p) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * KV_STAGE_B];
  const BlockId blk = xcd_block_id(false);
  if (blk.x & 1) kv_fast128_block<CAUSAL, 0>(p, smem, blk.x >> 1, blk.y, blk.z);
  else kv_fast128_block<CAUSAL, 1>(p, smem, blk.x >> 1, blk.y, blk.z);
}

}  // namespace

hipError_t launch_fast_kv128(const KP& p, hipStream_t st) {
  const dim3 g(2 * ((p.S + 127) / 128), p.h1 - p.h0, p.b1 - p.b0);
  if (p.mask_kind == 1) kv_fast128_kernel<true><<<g, 256, 0, st>>>(p);
  else kv_fast128_kernel<false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace ssa
