// Whole-sequence-in-registers attention kernels for short sequences (S <= 64) with
// head size 32, bf16: the shape of window attention (7x7 = 49 tokens per window).
//
// One wavefront owns one (row b, head h) pair at a time and keeps its entire
// padded 64x64 score matrix in MFMA accumulators, so the softmax is exact in one
// pass, nothing is rescaled, and the backward needs no separate recompute pass,
// no Delta pass and no O: Delta_i = sum_j P_ij dP_ij is taken from registers.
// The backward is ONE kernel per chunk: pass 1 (lane = query) yields LSE, Delta
// and dQ; pass 2 (lane = key) re-derives P from LSE and yields dK, dV and the
// bias-gradient contribution.
//
// Bias gradient.  Rows are grouped by GW consecutive global row indices.  A
// wavefront walks one group in row order, summing dS into registers, and stores
// the group's partial sum [S,S] to the workspace; a group cut by a chunk boundary
// is continued from the stored partial by the next chunk, so the order of
// additions never depends on k.  After the last chunk the partials are summed
// over groups in index order (dense gradient), and for a relative-position table
// gathered per table entry in a fixed order.
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

constexpr int SD = 32;        // head size
constexpr int SLD = SD + 8;   // LDS row stride of the per-wave tiles (elements)
constexpr int BLD = 68;       // LDS row stride of the bias tile (elements)
constexpr int FWD_ROWS_PER_WAVE = 8;

struct WaveLds {
  uint16_t t0[64 * SLD];  // forward: V ; backward: K
  uint16_t t1[64 * SLD];  // forward: K ; backward: dO
  uint16_t t2[64 * SLD];  // Q (forward: then the output block)
  float lse2[64];
  float delta[64];
  int rid[64];
};

// builds bias[q][k] (raw bf16 value; -inf where the pair can never be attended: padding,
// causal) for head h with 256 threads; caller syncs.  The 16 entries of a thread are fetched first
// and stored afterwards, so that the gathers are in flight together (one after the other they cost
// every work-group several microseconds before its first row).
__device__ inline void build_bias_tile(const KP& p, int h, uint16_t* tile, int tid) {
  const int R = (2 * p.win_h - 1) * (2 * p.win_w - 1);
  uint16_t v[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int idx = tid + i * 256, q = idx >> 6, k = idx & 63;
    const bool dead = q >= p.S || k >= p.S || (p.mask_kind == 1 && k > q);
    int64_t off = 0;
    if (p.bias_kind == 1) {
      off = ((int64_t)h * p.S + min(q, p.S - 1)) * p.S + min(k, p.S - 1);
    } else if (p.bias_kind == 2) {
      const int qq = min(q, p.S - 1), kk = min(k, p.S - 1);
      const int yq = qq / p.win_w, xq = qq - yq * p.win_w, yk = kk / p.win_w, xk = kk - yk * p.win_w;
      off = (int64_t)h * R + (yq - yk + p.win_h - 1) * (2 * p.win_w - 1) + (xq - xk + p.win_w - 1);
    }
    uint16_t x = 0;
    if (p.bias_kind != 0) x = p.bias_bf16 ? ((const uint16_t*)p.bias)[off] : f2bf(((const float*)p.bias)[off]);
    v[i] = dead ? (uint16_t)0xff80 : x;  // -inf
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int idx = tid + i * 256;
    tile[(idx >> 6) * BLD + (idx & 63)] = v[i];
  }
}

// a [<=64 x 32] activation slice in whole row segments: lane l takes the 16-byte chunk l % 4 of rows
// l / 4 + 16 c (rows past S - 1 repeat the last row; their scores are masked by the bias tile)
__device__ inline void load_rows(const uint16_t* base, int64_t row_stride, int S, int lane, u32x4 (&f)[4]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int row = min((lane >> 2) + 16 * c, S - 1);
    f[c] = *(const u32x4*)(base + (int64_t)row * row_stride + 8 * (lane & 3));
  }
}
// ... into a per-wave LDS tile
__device__ inline void store_rows(uint16_t* t, int lane, const u32x4 (&f)[4]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) *(u32x4*)(t + ((lane >> 2) + 16 * c) * SLD + 8 * (lane & 3)) = f[c];
}
// natural-layout fragment of rows 32*blk.. of a per-wave LDS tile
__device__ inline bf16x8 tile_nat(const uint16_t* t, int blk, int ks, int r, int hl) {
  return *(const bf16x8*)(t + (32 * blk + r) * SLD + 16 * ks + 8 * hl);
}
// orders this wavefront's LDS writes before its following LDS reads
__device__ inline void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// scores of query block qb against both key blocks, lane = query: x = s*c1 + bias*log2e, masked -> -inf
template <bool REGION>
__device__ inline void scores_by_query(const KP& p, const bf16x8 (&kf)[2][2], const bf16x8 (&qf)[2][2], int qb,
                                       const uint16_t* bias_tile, const int* rid, int q, int hl, float c1,
                                       float (&x)[2][16]) {
  const int my_rid = REGION ? rid[q] : 0;
#pragma unroll
  for (int kb = 0; kb < 2; ++kb) {
    f32x16 sa;
#pragma unroll
    for (int v = 0; v < 16; ++v) sa[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) sa = mfma(kf[kb][ks], qf[qb][ks], sa);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int kbase = 32 * kb + 8 * g + 4 * hl;
      const uint2 u = *(const uint2*)(bias_tile + q * BLD + kbase);
      const float bl[4] = {__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                           __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u)};
      int4 rk = {0, 0, 0, 0};
      if (REGION) rk = *(const int4*)(rid + kbase);
      const int rks[4] = {rk.x, rk.y, rk.z, rk.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float t = fmaf(sa[4 * g + e], c1, bl[e] * LOG2E);
        if (REGION) t = rks[e] != my_rid ? -INFINITY : t;
        x[kb][4 * g + e] = t;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// forward: grid (ceil(rows/32), heads); each wavefront takes 8 consecutive rows of one head.
// Global memory is touched only in whole 64-byte row segments (four lanes per segment, 16 rows per
// instruction): the operands pass through the wavefront's LDS tiles on their way into operand
// layout, and the output block goes back through a tile on its way out.  Loading in operand layout
// (one lane = one row, 16 bytes) costs four cache-line lookups per four lanes instead of one, and the
// short-sequence kernels are bound by exactly that.
// ---------------------------------------------------------------------------
template <bool REGION>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void small_fwd_kernel(KP p) {
  __shared__ __attribute__((aligned(16))) uint16_t bias_tile[64 * BLD];
  __shared__ __attribute__((aligned(16))) WaveLds wl[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.y;
  build_bias_tile(p, h, bias_tile, tid);
  __syncthreads();
  WaveLds& L = wl[w];
  const float c1 = p.scale * LOG2E;
  const int bfirst = p.b0 + (blockIdx.x * 4 + w) * FWD_ROWS_PER_WAVE;
  const int blast = min(bfirst + FWD_ROWS_PER_WAVE, p.b1);
  // the operands of row b + 1 are fetched while row b is computed
  u32x4 qn[4], kn[4], vn[4];
  auto fetch = [&](int b) {
    const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
    load_rows((const uint16_t*)p.Q + base, p.ss, p.S, lane, qn);
    load_rows((const uint16_t*)p.K + base, p.ss, p.S, lane, kn);
    load_rows((const uint16_t*)p.V + base, p.ss, p.S, lane, vn);
  };
  if (bfirst < blast) fetch(bfirst);
  for (int b = bfirst; b < blast; ++b) {
    const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
    store_rows(L.t2, lane, qn);
    store_rows(L.t1, lane, kn);
    store_rows(L.t0, lane, vn);
    fetch(min(b + 1, blast - 1));
    // most windows of a shifted-window map lie inside one region: their mask masks nothing, and the
    // row takes the copy of the code without the compare and select per score (uniform branch)
    bool masked = false;
    if (REGION) {
      const int my = p.region[(int64_t)(b % p.mask_period) * p.S + min(lane, p.S - 1)];
      L.rid[lane] = my;
      masked = __builtin_amdgcn_ballot_w64(my != __builtin_amdgcn_readfirstlane(my)) != 0;
    }
    wave_lds_sync();
    bf16x8 qf[2][2], kf[2][2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        qf[blk][ks] = tile_nat(L.t2, blk, ks, r, hl);
        kf[blk][ks] = tile_nat(L.t1, blk, ks, r, hl);
      }
    wave_lds_sync();  // the Q tile is reused for the output below
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int q = 32 * qb + r;
      float x[2][16];
      if (masked) scores_by_query<true>(p, kf, qf, qb, bias_tile, L.rid, q, hl, c1, x);
      else scores_by_query<false>(p, kf, qf, qb, bias_tile, L.rid, q, hl, c1, x);
      float m = -1e30f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, x[kb][v]);
      m = half_max(m);
      float l = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          x[kb][v] = fast_exp2(x[kb][v] - m);
          l += x[kb][v];
        }
      f32x16 oacc;
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[v] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
          oacc = mfma(lds_tr<SLD>(L.t0, 32 * kb + 16 * hb, 0, lane), pack8(&x[kb][8 * hb]), oacc);
      // normalise; the block's output row goes to the (consumed) Q tile, LSE straight to memory
      l = half_sum(l);
      const float inv = 1.f / l;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint2 o;
        o.x = (uint32_t)f2bf(oacc[4 * g] * inv) | ((uint32_t)f2bf(oacc[4 * g + 1] * inv) << 16);
        o.y = (uint32_t)f2bf(oacc[4 * g + 2] * inv) | ((uint32_t)f2bf(oacc[4 * g + 3] * inv) << 16);
        *(uint2*)(L.t2 + q * SLD + 8 * g + 4 * hl) = o;
      }
      if (q < p.S && hl == 0 && p.lse_out)
        p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = (m + log2f(l)) * LN2;
    }
    wave_lds_sync();
    // Y rows leave as whole 64-byte segments
    {
      uint16_t* Yb = (uint16_t*)p.Y + base;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int row = (lane >> 2) + 16 * c;
        const u32x4 o = *(const u32x4*)(L.t2 + row * SLD + 8 * (lane & 3));
        if (row < p.S) *(u32x4*)(Yb + (int64_t)row * p.ss + 8 * (lane & 3)) = o;
      }
    }
    wave_lds_sync();  // the next row's tile stores must not overtake this row's reads
  }
}

// ---------------------------------------------------------------------------
// backward: grid (ceil(groups/4), heads); each wavefront takes one group of rows
// ---------------------------------------------------------------------------
template <bool REGION>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void small_bwd_kernel(KP p) {
  __shared__ __attribute__((aligned(16))) uint16_t bias_tile[64 * BLD];
  __shared__ __attribute__((aligned(16))) WaveLds wl[4];
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int h = p.h0 + blockIdx.y;
  build_bias_tile(p, h, bias_tile, tid);
  __syncthreads();
  WaveLds& L = wl[w];
  const float c1 = p.scale * LOG2E;
  const int g = p.b0 / p.sm_gw + blockIdx.x * 4 + w;  // global group index
  const int bfirst = max(g * p.sm_gw, p.b0);
  const int blast = min((g + 1) * p.sm_gw, p.b1);
  if (bfirst >= blast) return;
  // bias-gradient accumulators, lane = key: acc[qb][kb][v] for query 32*qb + key_of(v), key 32*kb + r
  float acc[2][2][16];
  float* part = nullptr;
  if (p.sm_partial) {
    part = p.sm_partial + ((int64_t)((g - p.sm_g0) % p.sm_ring) * p.sm_hs + (h - p.sm_h0)) * p.S * p.S;
    const bool resume = max(g * p.sm_gw, p.share_b0) < p.b0;  // an earlier chunk started this group
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int q = 32 * qb + key_of(v, hl), k = 32 * kb + r;
          acc[qb][kb][v] = (resume && q < p.S && k < p.S) ? part[q * p.S + k] : 0.f;
        }
  }
  for (int b = bfirst; b < blast; ++b) {
    const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
    // K, dO and Q go to this wavefront's LDS tiles (read back both ways), fetched in whole 64-byte
    // row segments; V ends up in registers, in operand layout
    bf16x8 vf[2][2];
    {
      u32x4 tk[4], tg[4], tq[4];
      load_rows((const uint16_t*)p.K + base, p.ss, p.S, lane, tk);
      load_rows((const uint16_t*)p.dO + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)(h - p.do_h0) * p.do_sh, p.do_ss, p.S, lane, tg);
      load_rows((const uint16_t*)p.Q + base, p.ss, p.S, lane, tq);
      u32x4 tv[4];
      load_rows((const uint16_t*)p.V + base, p.ss, p.S, lane, tv);
      // V passes through the Q tile on its way into operand layout
      store_rows(L.t2, lane, tv);
      wave_lds_sync();
#pragma unroll
      for (int blk = 0; blk < 2; ++blk)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) vf[blk][ks] = tile_nat(L.t2, blk, ks, r, hl);
      wave_lds_sync();
      store_rows(L.t0, lane, tk);
      store_rows(L.t1, lane, tg);
      store_rows(L.t2, lane, tq);
    }
    // most windows of a shifted-window map lie inside one region: their mask masks nothing, and the
    // row takes the copy of the code without the compare and select per score (uniform branch)
    bool masked = false;
    if (REGION) {
      const int my = p.region[(int64_t)(b % p.mask_period) * p.S + min(lane, p.S - 1)];
      L.rid[lane] = my;
      masked = __builtin_amdgcn_ballot_w64(my != __builtin_amdgcn_readfirstlane(my)) != 0;
    }
    wave_lds_sync();
    // ---- pass 1, lane = query: exact softmax, Delta, dQ
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int q = 32 * qb + r;
      float x[2][16];
      bf16x8 qf[2][2], gq_[2];
      {
        bf16x8 kf[2][2];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          kf[0][ks] = tile_nat(L.t0, 0, ks, r, hl);
          kf[1][ks] = tile_nat(L.t0, 1, ks, r, hl);
          qf[qb][ks] = tile_nat(L.t2, qb, ks, r, hl);
          gq_[ks] = tile_nat(L.t1, qb, ks, r, hl);
        }
        if (masked) scores_by_query<true>(p, kf, qf, qb, bias_tile, L.rid, q, hl, c1, x);
        else scores_by_query<false>(p, kf, qf, qb, bias_tile, L.rid, q, hl, c1, x);
      }
      float m = -1e30f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) m = fmaxf(m, x[kb][v]);
      m = half_max(m);
      float l = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          x[kb][v] = fast_exp2(x[kb][v] - m);
          l += x[kb][v];
        }
      l = half_sum(l);
      l = q < p.S ? l : 1.f;  // padded queries: keep the statistics finite
      const float inv = 1.f / l;
      f32x16 pa[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) pa[kb][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) pa[kb] = mfma(vf[kb][ks], gq_[ks], pa[kb]);
      }
      float dl = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          x[kb][v] *= inv;
          dl = fmaf(x[kb][v], pa[kb][v], dl);
        }
      dl = half_sum(dl);
      if (hl == 0) {
        L.lse2[q] = m + log2f(l);
        L.delta[q] = dl;
      }
      f32x16 dq;
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[v] = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) x[kb][v] *= (pa[kb][v] - dl);
#pragma unroll
        for (int hb = 0; hb < 2; ++hb)
          dq = mfma(lds_tr<SLD>(L.t0, 32 * kb + 16 * hb, 0, lane), pack8(&x[kb][8 * hb]), dq);
      }
      {
        uint2 o[4];
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          o[gq].x = (uint32_t)f2bf(dq[4 * gq] * p.scale) | ((uint32_t)f2bf(dq[4 * gq + 1] * p.scale) << 16);
          o[gq].y = (uint32_t)f2bf(dq[4 * gq + 2] * p.scale) | ((uint32_t)f2bf(dq[4 * gq + 3] * p.scale) << 16);
        }
        store_row32((uint16_t*)p.dQ + base + (int64_t)min(q, p.S - 1) * p.ss, o, hl, q < p.S);
      }
    }
    wave_lds_sync();  // LSE / Delta written by half of the lanes, read by all
    // ---- pass 2, lane = key: P from LSE, dS, dK, dV, bias-gradient contribution
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const int key = 32 * kb + r;
      const int my_rid = REGION ? L.rid[key] : 0;
      f32x16 dk, dv;
#pragma unroll
      for (int v = 0; v < 16; ++v) { dk[v] = 0.f; dv[v] = 0.f; }
      const bf16x8 kk0 = tile_nat(L.t0, kb, 0, r, hl), kk1 = tile_nat(L.t0, kb, 1, r, hl);
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        f32x16 sa, pa;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sa[v] = 0.f; pa[v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          sa = mfma(tile_nat(L.t2, qb, ks, r, hl), ks == 0 ? kk0 : kk1, sa);
          pa = mfma(tile_nat(L.t1, qb, ks, r, hl), vf[kb][ks], pa);
        }
        float pr[16], ds[16];
        auto probs = [&](auto masked_tag) {
          constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
          for (int gq = 0; gq < 4; ++gq) {
            const int qbase = 32 * qb + 8 * gq + 4 * hl;
            const f32x4 l4 = *(const f32x4*)(L.lse2 + qbase);
            const f32x4 d4 = *(const f32x4*)(L.delta + qbase);
            int4 rq = {0, 0, 0, 0};
            if (MASKED) rq = *(const int4*)(L.rid + qbase);
            const int rqs[4] = {rq.x, rq.y, rq.z, rq.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float bl = bf2f(bias_tile[(qbase + e) * BLD + key]) * LOG2E;
              float t = fmaf(sa[4 * gq + e], c1, bl) - l4[e];
              if (MASKED) t = rqs[e] != my_rid ? -INFINITY : t;
              const float pe = fast_exp2(t);
              pr[4 * gq + e] = pe;
              ds[4 * gq + e] = pe * (pa[4 * gq + e] - d4[e]);
            }
          }
        };
        if (masked) probs(std::true_type{});
        else probs(std::false_type{});
        if (part) {
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[qb][kb][v] += ds[v];
        }
#pragma unroll
        for (int hb = 0; hb < 2; ++hb) {
          dv = mfma(lds_tr<SLD>(L.t1, 32 * qb + 16 * hb, 0, lane), pack8(&pr[8 * hb]), dv);
          dk = mfma(lds_tr<SLD>(L.t2, 32 * qb + 16 * hb, 0, lane), pack8(&ds[8 * hb]), dk);
        }
      }
      {
        uint2 a[4], c[4];
#pragma unroll
        for (int gd = 0; gd < 4; ++gd) {
          a[gd].x = (uint32_t)f2bf(dk[4 * gd] * p.scale) | ((uint32_t)f2bf(dk[4 * gd + 1] * p.scale) << 16);
          a[gd].y = (uint32_t)f2bf(dk[4 * gd + 2] * p.scale) | ((uint32_t)f2bf(dk[4 * gd + 3] * p.scale) << 16);
          c[gd].x = (uint32_t)f2bf(dv[4 * gd]) | ((uint32_t)f2bf(dv[4 * gd + 1]) << 16);
          c[gd].y = (uint32_t)f2bf(dv[4 * gd + 2]) | ((uint32_t)f2bf(dv[4 * gd + 3]) << 16);
        }
        const int64_t krow = base + (int64_t)min(key, p.S - 1) * p.ss;
        store_row32((uint16_t*)p.dK + krow, a, hl, key < p.S);
        store_row32((uint16_t*)p.dV + krow, c, hl, key < p.S);
      }
    }
    wave_lds_sync();  // next row's tile stores after this row's reads
  }
  if (part) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int q = 32 * qb + key_of(v, hl), k = 32 * kb + r;
          if (q < p.S && k < p.S) part[q * p.S + k] = acc[qb][kb][v];
        }
  }
}

// Two-level, fixed-shape sum over groups, done slice by slice as the groups complete.  Level 1 folds
// a slice of `slice` consecutive groups into the slot of the slice's first group (ascending order,
// starting from zero); level 2 adds the slice sums in ascending order to dense[h][i][j].  Which
// groups form a slice depends only on the share, so the additions are the same for every k.
typedef f32x4 f32x4_u __attribute__((aligned(4)));
// The nh heads of one slot are one contiguous run of nh * SS floats: a thread takes four consecutive
// ones (16-byte loads need 4-byte alignment only), each summed over the slice's groups in order.
__global__ __launch_bounds__(256) void group_fold_kernel(float* partial, int ring, int hs, int nh, int SS, int slice,
                                                         int s0, int ngroups) {
  const int64_t n = (int64_t)nh * SS, t = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (t >= n) return;
  const int g0 = (s0 + blockIdx.y) * slice, g1 = min(g0 + slice, ngroups);
  const int64_t gs = (int64_t)hs * SS;
  float* dst = partial + (int64_t)(g0 % ring) * gs + t;
  if (t + 4 <= n) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
    for (int g = g0; g < g1; ++g) {
      const f32x4 v = *(const f32x4_u*)(partial + (int64_t)(g % ring) * gs + t);
#pragma unroll
      for (int e = 0; e < 4; ++e) a[e] += v[e];
    }
    *(f32x4_u*)dst = a;
  } else {
    for (int e = 0; t + e < n; ++e) {
      float a = 0.f;
      for (int g = g0; g < g1; ++g) a += partial[(int64_t)(g % ring) * gs + t + e];
      dst[e] = a;
    }
  }
}
__global__ __launch_bounds__(256) void group_reduce_kernel(const float* partial, float* dense, int ring, int hs,
                                                           int hd0, int nh, int SS, int slice, int s0, int s1,
                                                           int first) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= (int64_t)nh * SS) return;
  const int hh = (int)(t / SS), ij = (int)(t % SS);
  float* out = dense + (int64_t)(hd0 + hh) * SS + ij;
  float a = first ? 0.f : *out;
  for (int s = s0; s < s1; ++s) a += partial[((int64_t)((s * slice) % ring) * hs + hh) * SS + ij];
  *out = a;
}

}  // namespace

bool small_supported(const KP& p, bool bf16) {
  return bf16 && p.D == SD && p.S <= 64 && !p.gated && p.scale > 0.f;
}

hipError_t launch_small_fwd(const KP& p, hipStream_t st) {
  const int rows = p.b1 - p.b0;
  dim3 g((rows + 4 * FWD_ROWS_PER_WAVE - 1) / (4 * FWD_ROWS_PER_WAVE), p.h1 - p.h0);
  if (p.mask_kind == 2) small_fwd_kernel<true><<<g, 256, 0, st>>>(p);
  else small_fwd_kernel<false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

hipError_t launch_small_bwd(const KP& p, hipStream_t st) {
  const int ng = (p.b1 - 1) / p.sm_gw - p.b0 / p.sm_gw + 1;
  dim3 g((ng + 3) / 4, p.h1 - p.h0);
  if (p.mask_kind == 2) small_bwd_kernel<true><<<g, 256, 0, st>>>(p);
  else small_bwd_kernel<false><<<g, 256, 0, st>>>(p);
  return hipGetLastError();
}

hipError_t launch_group_fold(float* partial, float* dense, int ring, int hs, int hd0, int nh, int S, int slice,
                             int s0, int s1, int ngroups, bool first, hipStream_t st) {
  if (s1 <= s0) return hipSuccess;
  const int64_t n = (int64_t)nh * S * S;
  if (slice > 1) {  // a slice of one group is its own sum (0 + x = x exactly)
    group_fold_kernel<<<dim3((unsigned)((n + 1023) / 1024), s1 - s0), 256, 0, st>>>(partial, ring, hs, nh, S * S,
                                                                                    slice, s0, ngroups);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  group_reduce_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(partial, dense, ring, hs, hd0, nh, S * S, slice, s0,
                                                                   s1, first ? 1 : 0);
  return hipGetLastError();
}

}  // namespace ssa
