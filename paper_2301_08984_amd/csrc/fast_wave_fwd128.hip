// Forward / recompute kernel for small shares at head size 128: the query-stationary wavefronts of
// fast_wave_fwd.hip with the K and V sub-tiles fetched from memory straight into LDS.
//
// Measured on the register-staged kernel: the 16 `ds_write_b128` per 32 x 32 tile are its largest
// single cost (LDS takes writes at 76 bytes per cycle and compute unit, a third of its read rate, and
// a wavefront that waits at a store holds back the reads and matrix instructions behind it), the
// 64 staging registers push the Q fragments into accumulation registers (28 copies per tile), and
// every load needs an address add.  Here a sub-tile is 8 `buffer_load ... lds` of 1 KB each: no
// staging registers, no store instructions, lane offsets that never change.
//
// LDS image of a 32-row sub-tile (rows of 256 bytes = 16 chunks of 16 bytes, no padding, since a
// load instruction fills 1 KB = 4 rows contiguously): chunk c of row rho sits at position
// c ^ sw(rho), sw(rho) = ((rho & 3) << 2) | ((rho >> 2) & 3).  The swizzle is applied by choosing
// WHICH chunk a lane fetches for its fixed LDS position.  16 consecutive rows put the same chunk at
// 16 different positions (operand reads of K and Q: no bank conflicts), and 4 consecutive rows put
// a 64-byte group of chunks into 4 different 64-byte bank groups (transposed reads of V).
//
// This file is compiled with the matrix instructions in their vector-register form and uses no
// accumulation registers at all, so that the compiler may give the wavefront all 256 registers as
// vector registers (with any accumulation register in use it splits them 128 / 128 and moves
// operands between the halves, 16 to 44 copies per tile here).
//
// One slot per wavefront and operand: the fragments of a sub-tile are read into registers, then the
// slot is refilled, so a sub-tile has one whole step to arrive.
#include "wave_common.h"

namespace ssa {
namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void w_lds_void;
typedef __attribute__((address_space(3))) s16x4 w_lds_s16x4;
typedef __attribute__((address_space(3))) bf16x8 w_lds_bf16x8;

constexpr int W_NG = 4;  // wavefronts per work-group

__device__ __forceinline__ int w_sw(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

#define W_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
#define W_LGKM0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")

template <bool BIAS, bool CAUSAL, bool RECOMP>
__global__ __launch_bounds__(64 * W_NG) __attribute__((amdgpu_waves_per_eu(2, 2))) void fwd_wave128_kernel(KP p) {
  constexpr int D = 128, KS = D / 16, DB = D / 32, SUB = 32, NG = W_NG;
  constexpr int TILE_B = SUB * D * 2;                // bytes of one sub-tile
  constexpr int SLOT_B = 2 * TILE_B;                 // K, then V
  constexpr int MSLOT = 64 * (4 * DB + 1);           // f32x4 units one wavefront hands over in the merge
  constexpr int MERGE_B = NG * MSLOT * 16 + 4 * 32 * (DB < NG ? DB : NG);  // hand-over area + partial Delta
  constexpr int LDS_B = NG * SLOT_B > MERGE_B ? NG * SLOT_B : MERGE_B;
  __shared__ __attribute__((aligned(1024))) char smem[LDS_B];
  const int lane = threadIdx.x & 63, r = lane & 31, hl = lane >> 5;
  const int grp = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: scalar registers
  char* sK = smem + grp * SLOT_B;
  char* sV = sK + TILE_B;
  const BlockId blk = heavy_first_block_id();
  const int h = p.h0 + blk.y, b = p.b0 + blk.z;
  const int nsub = (p.S + SUB - 1) / SUB;
  const int qb = CAUSAL ? nsub - 1 - blk.x : blk.x;  // late query blocks see the most keys under a causal mask
  const int q0 = qb * SUB, q = q0 + r;
  const int qc = min(q, p.S - 1);
  const int64_t base = (int64_t)b * p.sb + (int64_t)h * p.sh;
  const uint16_t* Qb = (const uint16_t*)p.Q + base;
  const uint16_t* Kb = (const uint16_t*)p.K + base;
  const uint16_t* Vb = (const uint16_t*)p.V + base;
  const uint16_t* bias_row = BIAS ? (const uint16_t*)p.bias + ((int64_t)h * p.S + qc) * p.S : nullptr;
  const float c1 = p.scale * LOG2E;

  const int nj = CAUSAL ? min(nsub, qb + 1) : nsub;  // key sub-tiles with a visible key
  const int j0 = grp;
  const int n = j0 < nj ? (nj - 1 - j0) / NG + 1 : 0;
  const int jlast = j0 + (n - 1) * NG;
  auto jc = [&](int j) { return min(j, jlast); };  // past the wavefront's last sub-tile: fetch it again

  // lane offsets of the 8 load instructions of a sub-tile: instruction t fills LDS rows 4t .. 4t+3,
  // lane l the position l % 16 of row 4t + l / 16
  uint32_t goff[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int rho = 4 * t + (lane >> 4);
    goff[t] = (uint32_t)rho * (uint32_t)p.ss * 2u + 16u * (uint32_t)((lane & 15) ^ w_sw(rho));
  }
  // sub-tile starting at row `row0` of a (row, head) slice -> `slot`.  The descriptor starts at the
  // sub-tile and ends with the slice, so the lane offsets are the same for every sub-tile and rows
  // past S-1 arrive as zeros (the hardware range-checks the lane offset).
  const uint32_t ss2 = (uint32_t)p.ss * 2u;
  const uint32_t slice_bytes = (uint32_t)(((int64_t)(p.S - 1) * p.ss + D) * 2);  // < 2 GiB, checked on the host
  auto fetch = [&](char* slot, const uint16_t* src, int row0) {
    const uint32_t boff = (uint32_t)row0 * ss2;  // row0 < S
    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)src + boff), 0, (int)(slice_bytes - boff), 0x00020000);
#pragma unroll
    for (int t = 0; t < 8; ++t)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (w_lds_void*)(slot + t * 1024), 16, goff[t], 0, 0, 0);
  };
  // The fragment reads are written as assembly: the compiler cannot tell which of the loads under
  // way fills the slot a `ds_read` touches and would wait for all of them (vmcnt(0)) before every
  // read it can see, which would undo the overlap.  A read is split into an issue part and a wait
  // part so that independent arithmetic can be placed between them; the registers are not touched in
  // between (they are outputs of the first and in/outputs of the second).
  // operand fragment ks of the sub-tile in the K slot: row r, chunk 2 ks + hl
  uint32_t ka[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    ka[ks] = (uint32_t)(size_t)(w_lds_void*)sK + (((uint32_t)r * 256u + (uint32_t)((hl ^ w_sw(r)) << 4)) ^ (uint32_t)(ks << 5));
  auto nat_issue = [&](u32x4 (&f)[KS]) {
    asm volatile(
        "ds_read_b128 %0, %8\n\tds_read_b128 %1, %9\n\tds_read_b128 %2, %10\n\tds_read_b128 %3, %11\n\t"
        "ds_read_b128 %4, %12\n\tds_read_b128 %5, %13\n\tds_read_b128 %6, %14\n\tds_read_b128 %7, %15"
        : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(f[4]), "=&v"(f[5]), "=&v"(f[6]), "=&v"(f[7])
        : "v"(ka[0]), "v"(ka[1]), "v"(ka[2]), "v"(ka[3]), "v"(ka[4]), "v"(ka[5]), "v"(ka[6]), "v"(ka[7])
        : "memory");
  };
  auto nat_wait = [&](u32x4 (&f)[KS]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7])
                 :
                 : "memory");
  };
  // transposed fragments of V: lane gets column 32 db + l % 32 of rows 16 t + {0..3, 8..11} + 4 hl,
  // i.e. (as ds_read_b64_tr_b16 wants it) four consecutive elements of row 16 t + 8 half + 4 (bk >> 1) + (i >> 2)
  // at column 32 db + 16 (bk & 1) + 4 (i & 3), with i = l % 16, bk = l / 16
  uint32_t va[2][DB];
  {
    const int i = lane & 15, bk = lane >> 4;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      const int row = 8 * half + 4 * (bk >> 1) + (i >> 2);
      const int lowc = (2 * (bk & 1) + ((i & 3) >> 1)) ^ ((2 * half + (bk >> 1)) & 3);
#pragma unroll
      for (int db = 0; db < DB; ++db)
        va[half][db] = (uint32_t)(size_t)(w_lds_void*)sV + (uint32_t)row * 256u + (uint32_t)((db ^ (i >> 2)) << 6) +
                       (uint32_t)(lowc << 4) + 8u * (i & 1);
    }
  }
  // f[t][2 db + half]
  auto tr_issue = [&](u32x2 (&f)[2][2 * DB]) {
#define W_TR8(OFF)                                                                                                   \
  "ds_read_b64_tr_b16 %0, %8 offset:" #OFF "\n\tds_read_b64_tr_b16 %1, %9 offset:" #OFF "\n\t"                       \
  "ds_read_b64_tr_b16 %2, %10 offset:" #OFF "\n\tds_read_b64_tr_b16 %3, %11 offset:" #OFF "\n\t"                     \
  "ds_read_b64_tr_b16 %4, %12 offset:" #OFF "\n\tds_read_b64_tr_b16 %5, %13 offset:" #OFF "\n\t"                     \
  "ds_read_b64_tr_b16 %6, %14 offset:" #OFF "\n\tds_read_b64_tr_b16 %7, %15 offset:" #OFF
#define W_TR_OPS(T)                                                                                                   \
  : "=&v"(f[T][0]), "=&v"(f[T][1]), "=&v"(f[T][2]), "=&v"(f[T][3]), "=&v"(f[T][4]), "=&v"(f[T][5]), "=&v"(f[T][6]),   \
    "=&v"(f[T][7])                                                                                                    \
  : "v"(va[0][0]), "v"(va[1][0]), "v"(va[0][1]), "v"(va[1][1]), "v"(va[0][2]), "v"(va[1][2]), "v"(va[0][3]),          \
    "v"(va[1][3])                                                                                                     \
  : "memory"
    asm volatile(W_TR8(0) W_TR_OPS(0));
    asm volatile(W_TR8(4096) W_TR_OPS(1));
#undef W_TR8
#undef W_TR_OPS
  };
  auto tr_wait = [&](u32x2 (&f)[2][2 * DB]) {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(f[0][0]), "+v"(f[0][1]), "+v"(f[0][2]), "+v"(f[0][3]), "+v"(f[0][4]), "+v"(f[0][5]), "+v"(f[0][6]),
                   "+v"(f[0][7]), "+v"(f[1][0]), "+v"(f[1][1]), "+v"(f[1][2]), "+v"(f[1][3]), "+v"(f[1][4]), "+v"(f[1][5]),
                   "+v"(f[1][6]), "+v"(f[1][7])
                 :
                 : "memory");
  };
  auto frag = [](const u32x4& x) { union { u32x4 u; bf16x8 v; } c; c.u = x; return c.v; };
  auto frag2 = [](const u32x2& lo, const u32x2& hi) { union { u32x2 h[2]; bf16x8 v; } c; c.h[0] = lo; c.h[1] = hi; return c.v; };

  uint2 bzn[4], bzc[4];  // bias slices of the next sub-tile / of the one about to be used
  auto bload = [&](int j) {
#pragma unroll
    for (int g = 0; g < 4; ++g) bzn[g] = *(const uint2*)(bias_row + min(j * SUB + 8 * g + 4 * hl, p.S - 4));
  };

  // Q fragments through the (still unused) K slot
  u32x4 qf[KS], fk[KS];
  u32x2 vfr[2][2 * DB];
  fetch(sK, Qb, q0);
  if (BIAS && n > 0) bload(j0);
  W_VMCNT(0);
  nat_issue(qf);
  nat_wait(qf);
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[db][v] = 0.f;
  float m = -1e30f, l = 0.f;

  // S^T = K Q^T with the fragments in fk: lane = query, registers = keys
  auto stage_s = [&](f32x16& sa) {
#pragma unroll
    for (int v = 0; v < 16; ++v) sa[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) sa = mfma(frag(fk[ks]), frag(qf[ks]), sa);
  };
  // online softmax of one 32-key block, first half: bias, mask, row maximum, running maximum
  auto softmax_max = [&](int k0, f32x16& sa, const uint2* bz, bool edge) {
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint2 u = bz[g];
        // natural units here; the change to base 2 rides on the subtraction of the maximum
        sa[4 * g + 0] = fmaf(sa[4 * g + 0], p.scale, __uint_as_float(u.x << 16));
        sa[4 * g + 1] = fmaf(sa[4 * g + 1], p.scale, __uint_as_float(u.x & 0xffff0000u));
        sa[4 * g + 2] = fmaf(sa[4 * g + 2], p.scale, __uint_as_float(u.y << 16));
        sa[4 * g + 3] = fmaf(sa[4 * g + 3], p.scale, __uint_as_float(u.y & 0xffff0000u));
      }
    }
    if (edge) {  // uniform; touches the scores only
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = k0 + key_of(v, hl);
        const bool dead = key >= p.S || (CAUSAL && key > q);
        sa[v] = dead ? -INFINITY : sa[v];
      }
    }
    float rmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) rmax = fmaxf(rmax, sa[v]);
    rmax *= BIAS ? LOG2E : c1;  // the running maximum is kept in base-2 units; scale > 0 on this path
    rmax = half_max(rmax);
    // the running maximum is raised only when exceeded by more than 2^8, so the O rescale is
    // skipped on most sub-tiles; probabilities stay below 2^8, harmless in fp32/bf16 range
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
  };
  // second half: P = exp2(s - m) as packed bf16 operands, row sum
  auto softmax_exp = [&](const f32x16& sa, bf16x8 (&pf)[2]) {
    float lsum = 0.f;
    float pr[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      pr[v] = fast_exp2(fmaf(sa[v], BIAS ? LOG2E : c1, -m));
      lsum += pr[v];
    }
    l += lsum;
    pf[0] = pack8(&pr[0]);
    pf[1] = pack8(&pr[8]);
  };
  // O^T += V^T P^T with the fragments in vfr
  auto stage_pv = [&](const bf16x8 (&pf)[2]) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < DB; ++db) oacc[db] = mfma(frag2(vfr[t][2 * db], vfr[t][2 * db + 1]), pf[t], oacc[db]);
  };

  if (n > 0) {
    f32x16 sc, sn;
    fetch(sK, Kb, j0 * SUB);
    W_VMCNT(0);
    nat_issue(fk);
    nat_wait(fk);
    fetch(sK, Kb, jc(j0 + NG) * SUB);
    fetch(sV, Vb, j0 * SUB);
    stage_s(sc);
    if (BIAS) {
#pragma unroll
      for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
    }
    // step i: scores of sub-tile j are in sc; on their way, in this order: K(j+NG), V(j)
    for (int i = 0; i < n; ++i) {
      const int j = j0 + i * NG;
      // K(j+NG) has landed (V(j) may still be under way): fragments out under the row maxima, slot refilled
      if (BIAS) W_VMCNT(0); else W_VMCNT(8);
      nat_issue(fk);
      softmax_max(j * SUB, sc, bzc, (j * SUB + SUB > p.S) || (CAUSAL && j * SUB + SUB - 1 > q0));
      if (BIAS) bload(jc(j + NG));
      nat_wait(fk);
      fetch(sK, Kb, jc(j + 2 * NG) * SUB);
      stage_s(sn);
      // V(j) has landed (K(j+2NG) under way): fragments out under the exponentials
      if (BIAS) W_VMCNT(0); else W_VMCNT(8);
      tr_issue(vfr);
      bf16x8 pf[2];
      softmax_exp(sc, pf);
      tr_wait(vfr);
      fetch(sV, Vb, jc(j + NG) * SUB);
      stage_pv(pf);
      if (BIAS) {
#pragma unroll
        for (int g = 0; g < 4; ++g) bzc[g] = bzn[g];
      }
      sc = sn;
    }
    W_VMCNT(0);  // the slots are about to be reused by the merge
  }

  {
    // every wavefront hands over its partial (O, m, l) through LDS; each then folds the statistics
    // with the same fixed binary tree ((g0+g2)+(g1+g3) for NG = 4), which also yields the weights
    // of every tree node, and wavefront w folds, normalises and stores the 32-column output blocks
    // w, w+NG, ...
    f32x4* mb = (f32x4*)smem;
    float* dpart = (float*)(mb + NG * MSLOT);  // [DB][32] partial Delta per output block (recompute)
    __syncthreads();
    f32x4* my = mb + (size_t)grp * MSLOT + lane;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        my[(4 * db + g) * 64] = f32x4{oacc[db][4 * g], oacc[db][4 * g + 1], oacc[db][4 * g + 2], oacc[db][4 * g + 3]};
    my[4 * DB * 64] = f32x4{m, l, 0.f, 0.f};
    __syncthreads();
    float mm[NG], ll[NG];
#pragma unroll
    for (int w = 0; w < NG; ++w) {
      const f32x4 ml = mb[(size_t)w * MSLOT + 4 * DB * 64 + lane];
      mm[w] = ml[0];
      ll[w] = ml[1];
    }
    float a0s[NG], a1s[NG];  // tree weights, entry st + w: node w and its partner w + st at level st
#pragma unroll
    for (int st = NG / 2; st >= 1; st >>= 1)
#pragma unroll
      for (int w = 0; w < st; ++w) {
        const float mn = fmaxf(mm[w], mm[w + st]);
        const float a0 = fast_exp2(mm[w] - mn), a1 = fast_exp2(mm[w + st] - mn);
        a0s[st + w] = a0;
        a1s[st + w] = a1;
        ll[w] = ll[w] * a0 + ll[w + st] * a1;
        mm[w] = mn;
      }
    m = mm[0];
    l = half_sum(ll[0]);
    const float inv = 1.f / l;
    float part = 0.f;
    bool mine = false;
    for (int db = grp; db < DB; db += NG) {
      mine = true;
      f32x16 o;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 x[NG];
#pragma unroll
        for (int w = 0; w < NG; ++w) x[w] = mb[(size_t)w * MSLOT + (4 * db + g) * 64 + lane];
#pragma unroll
        for (int st = NG / 2; st >= 1; st >>= 1)
#pragma unroll
          for (int w = 0; w < st; ++w)
#pragma unroll
            for (int e = 0; e < 4; ++e) x[w][e] = x[w][e] * a0s[st + w] + x[w + st][e] * a1s[st + w];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[4 * g + e] = x[0][e];
      }
      if (q < p.S) part += fwd_epilogue_block<RECOMP>(p, o, db, inv, b, h, q, hl, base, 0.f);
    }
    const float lse = (m + log2f(l)) * LN2;
    if (!RECOMP) {
      if (grp == 0 && hl == 0 && q < p.S && p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
      return;
    }
    // recompute: Delta = sum over the output blocks of the partial row sums, in block order
    part = half_sum(part);
    if (mine && hl == 0) dpart[grp * 32 + r] = part;  // DB <= NG: wavefront w owns block w
    __syncthreads();
    if (grp == 0 && hl == 0 && q < p.S) {
      float dl = 0.f;
#pragma unroll
      for (int db = 0; db < (DB < NG ? DB : NG); ++db) dl += dpart[db * 32 + r];
      p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + q] = dl;
      if (p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
    }
  }
}

template <bool RECOMP>
hipError_t fwd_wave128_r(const KP& p, hipStream_t st) {
  const dim3 g((p.S + 31) / 32, p.h1 - p.h0, p.b1 - p.b0);
  const bool bias = p.bias_kind == 1, causal = p.mask_kind == 1;
  if (bias && causal) fwd_wave128_kernel<true, true, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else if (bias) fwd_wave128_kernel<true, false, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else if (causal) fwd_wave128_kernel<false, true, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  else fwd_wave128_kernel<false, false, RECOMP><<<g, 64 * W_NG, 0, st>>>(p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_fast_fwd_wave128(const KP& p, bool recompute, hipStream_t st) {
  return recompute ? fwd_wave128_r<true>(p, st) : fwd_wave128_r<false>(p, st);
}

}  // namespace ssa
