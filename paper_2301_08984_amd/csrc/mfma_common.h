// Shared device helpers of the MFMA kernels (gfx950).
//
// MFMA v_mfma_f32_32x32x16_bf16 layouts (lane l, r = l%32, hl = l/32):
//   A[m][k]: lane holds m = r,  k = 8*hl + 0..7      B[k][n]: lane holds n = r, k = 8*hl + 0..7
//   C[m][n]: lane holds n = r,  register v holds m = 8*(v/4) + 4*hl + v%4
// An accumulator block is reused as the B operand of the next product with its
// registers 8t..8t+7 as the eight k-slots; the matching A operand is read from a
// row-major LDS tile with ds_read_b64_tr_b16 (transpose read) in the same row order.
#pragma once
#include "kparams.h"

namespace ssa {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int BN = 64;            // rows of a staged LDS tile
constexpr int MAX_RELPOS_S = 256;
constexpr int MAX_RELPOS_R = 1024;

__device__ inline float bf2f(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
__device__ inline uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // v_exp_f32
// v_rcp_f32 (1 ulp): the gate 1 / (1 + e^-g) is rounded to bf16 right after, and a full division
// costs ten instructions per element
__device__ inline float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
__device__ inline float half_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float half_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// Stores one row of 32 bf16 columns held as "lane = row, group g = columns 8g + 4*hl .. +3" (the
// layout of a 32x32 accumulator block, packed to 8 bytes per group): the two half-waves exchange
// pieces so that every lane writes 16 contiguous bytes twice (columns 8*(2j + hl) .. +7) instead of
// 8 bytes four times, which halves the cache-line lookups of the store.  Both lanes of a row (l and
// l + 32) must be active; `live` masks the stores only.
__device__ inline void store_row32(uint16_t* row_ptr, const uint2 (&a)[4], int hl, bool live) {
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    auto s = __builtin_amdgcn_permlane32_swap(a[2 * j].x, a[2 * j + 1].x, false, false);
    auto t = __builtin_amdgcn_permlane32_swap(a[2 * j].y, a[2 * j + 1].y, false, false);
    if (live) *(u32x4*)(row_ptr + 8 * (2 * j + hl)) = u32x4{s[0], t[0], s[1], t[1]};
  }
}
// four scaled values as packed bf16
__device__ inline uint2 pack4_bf16(float a, float b, float c, float d, float s) {
  uint2 o;
  o.x = (uint32_t)f2bf(a * s) | ((uint32_t)f2bf(b * s) << 16);
  o.y = (uint32_t)f2bf(c * s) | ((uint32_t)f2bf(d * s) << 16);
  return o;
}
// The matching load: every lane fetches 16 contiguous bytes twice and the half-waves exchange pieces,
// so that a[g] ends up holding columns 8g + 4*hl .. +3 of the lane's row.  Both lanes of a row (l and
// l + 32) must be active.
__device__ inline void load_row32(const uint16_t* row_ptr, uint2 (&a)[4], int hl) {
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const u32x4 v = *(const u32x4*)(row_ptr + 8 * (2 * j + hl));
    auto s = __builtin_amdgcn_permlane32_swap(v[0], v[2], false, false);
    auto t = __builtin_amdgcn_permlane32_swap(v[1], v[3], false, false);
    a[2 * j].x = s[0]; a[2 * j].y = t[0];
    a[2 * j + 1].x = s[1]; a[2 * j + 1].y = t[1];
  }
}
__device__ inline f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ inline bf16x8 zero8() {
  union { u32x4 u; bf16x8 v; } z;
  z.u = u32x4{0, 0, 0, 0};
  return z.v;
}
// eight fp32 -> one bf16x8 operand (round to nearest even)
__device__ inline bf16x8 pack8(const float* x) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (__bf16)x[e];
  return o;
}

// Row-major bf16 tile in LDS, `LD` elements per row.
// natural operand: row = r, eight consecutive columns starting at 16*ks + 8*hl
template <int LD>
__device__ inline bf16x8 lds_nat(const uint16_t* t, int row, int ks, int hl) {
  return *(const bf16x8*)(t + row * LD + 16 * ks + 8 * hl);
}
// transposed operand for the product whose k-slots are accumulator registers 8t..8t+7 of a
// 32-row block: lane gets column (cbase + l%32) of rows rbase + {0..3, 8..11} + 4*hl
template <int LD>
__device__ inline bf16x8 lds_tr(const uint16_t* t, int rbase, int cbase, int lane) {
  const int i = lane & 15, bk = lane >> 4;
  const int row = rbase + 4 * (bk >> 1) + (i >> 2);
  const int col = cbase + 16 * (bk & 1) + 4 * (i & 3);
  typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
  union { s16x4 h[2]; bf16x8 v; } o;
  o.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(t + row * LD + col));
  o.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(t + (row + 8) * LD + col));
  return o.v;
}

// Work-groups are handed to the 8 XCDs round-robin in launch order, and each XCD has its own L2.
// This maps the hardware block id to a logical (x, y, z) such that blocks with consecutive
// logical ids (same head and row, neighbouring tiles: the ones that re-read the same K/V or
// Q/dO) run on the same XCD.  A bijection on [0, gridDim.x*gridDim.y*gridDim.z).
// `z_fast`: z (the row) varies before y (the head), so that the work-groups an XCD runs at one time
// belong to one head and a handful of rows: for kernels with a dense bias whose heads together do
// not fit one L2 (see bias_rows_first), the head's bias then stays in that L2 instead of being
// fetched again for every row, while a row's K/V (or Q/dO) are still shared by neighbouring tiles.
struct BlockId { int x, y, z; };
__device__ inline bool bias_rows_first(int heads, int S) { return (int64_t)heads * S * S * 2 > (4 << 20); }
__device__ inline BlockId xcd_block_id(bool z_fast = false) {
  constexpr int NX = 8;
  const int gx = gridDim.x, gy = gridDim.y;
  const int n = gx * gy * gridDim.z;
  const int lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  const int xcd = lin % NX, idx = lin / NX;
  const int v = xcd * (n / NX) + min(xcd, n % NX) + idx;
  BlockId b;
  b.x = v % gx;
  const int yz = v / gx;
  if (z_fast) {
    b.z = yz % (int)gridDim.z;
    b.y = yz / (int)gridDim.z;
  } else {
    b.y = yz % gy;
    b.z = yz / gy;
  }
  return b;
}

// Dense bias tile of one wavefront: 32 rows (queries, or keys of the transposed copy) by 64 columns.
// A lane of the score tile owns one row and needs 4 consecutive columns at a time, so direct loads
// would touch 64 rows per instruction.  Instead 8 lanes fetch 128 contiguous bytes of one row, 16
// bytes each (8 rows per instruction, 4 instructions per tile, issued one tile ahead: 8-byte loads
// move half as many bytes per cycle through a compute unit's load path, and the bias is two thirds
// of these kernels' load traffic), the tile is parked in a wavefront-private LDS area and read back
// in the layout of the accumulator.  LDS rows are padded to 136 bytes so that the 8-byte reads of 32
// rows fall into distinct banks.  The loads are buffer loads over the head's S x S matrix: a row past
// S - 1 lies past the end and reads as zeros, columns past S - 1 read the next row; both belong to
// scores that are masked or never stored.  S is a multiple of 4 and S * S * 2 bytes at most 2 GiB.
constexpr int BIAS_LD = 68, BIAS_TILE_ELEMS = 32 * BIAS_LD;
struct BiasTile {
  __amdgpu_buffer_rsrc_t rs;  // the head's matrix
  uint16_t* lds;              // the wavefront's area, BIAS_TILE_ELEMS elements
  uint32_t off, rstep;        // byte offset of this lane's chunk in tile 0; bytes between its rows
  u32x4 nxt[4];
  __device__ void init(const uint16_t* head, int row0, int S, uint16_t* area, int lane) {
    rs = __builtin_amdgcn_make_buffer_rsrc((void*)head, 0, (int)((int64_t)S * S * 2), 0x00020000);
    const int first = __builtin_amdgcn_readfirstlane(min(row0, S - 1));
    off = ((uint32_t)(first + (lane >> 3)) * (uint32_t)S + 8u * (lane & 7)) * 2u;
    rstep = 16u * (uint32_t)S;  // 8 rows
    lds = area;
  }
  __device__ void load(int tile) {
#pragma unroll
    for (int c = 0; c < 4; ++c) nxt[c] = __builtin_amdgcn_raw_buffer_load_b128(rs, off + tile * 128 + c * rstep, 0, 0);
  }
  __device__ void park(int lane) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint16_t* d = lds + ((lane >> 3) + 8 * c) * BIAS_LD + 8 * (lane & 7);
      *(uint2*)d = uint2{nxt[c][0], nxt[c][1]};
      *(uint2*)(d + 4) = uint2{nxt[c][2], nxt[c][3]};
    }
  }
  // columns col .. col + 3 (col a multiple of 4) of row r of the parked tile
  __device__ uint2 read(int r, int col) const { return *(const uint2*)(lds + r * BIAS_LD + col); }
};

__device__ inline int key_of(int v, int hl) { return 8 * (v >> 2) + 4 * hl + (v & 3); }

// Forward epilogue for one 32-column block `db` of a query's output (lane = query, registers =
// columns 8g + 4*hl + e, not yet normalised): normalise by `inv`, gate, store Y; recompute
// mode: gate gradient and pre-gated dO copy, and `part` continues this lane's part of
// Delta = rowsum(dO * O).  Rows are read and written 16 bytes per lane (load_row32 / store_row32).
// Both lanes of the row must be active.
template <bool RECOMP>
__device__ inline float fwd_epilogue_block(const KP& p, const f32x16& o16, int db, float inv, int b, int h, int q, int hl,
                                           int64_t base, float part) {
  const int64_t row = base + (int64_t)q * p.ss + 32 * db;
  float o[16], gt[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) o[v] = o16[v] * inv;
  if (p.gated) {
    uint2 gu[4];
    load_row32((const uint16_t*)p.G + row, gu, hl);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const float gl[4] = {__uint_as_float(gu[g].x << 16), __uint_as_float(gu[g].x & 0xffff0000u),
                           __uint_as_float(gu[g].y << 16), __uint_as_float(gu[g].y & 0xffff0000u)};
#pragma unroll
      for (int e = 0; e < 4; ++e) gt[4 * g + e] = fast_rcp(1.f + fast_exp2(-gl[e] * LOG2E));
    }
  }
  if (!RECOMP) {
    if (p.gated) {
#pragma unroll
      for (int v = 0; v < 16; ++v) o[v] *= gt[v];
    }
    uint2 out[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      out[g].x = (uint32_t)f2bf(o[4 * g]) | ((uint32_t)f2bf(o[4 * g + 1]) << 16);
      out[g].y = (uint32_t)f2bf(o[4 * g + 2]) | ((uint32_t)f2bf(o[4 * g + 3]) << 16);
    }
    store_row32((uint16_t*)p.Y + row, out, hl, true);
  } else {
    uint2 du[4];
    load_row32((const uint16_t*)p.dY + row, du, hl);
    float go[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      go[4 * g] = __uint_as_float(du[g].x << 16); go[4 * g + 1] = __uint_as_float(du[g].x & 0xffff0000u);
      go[4 * g + 2] = __uint_as_float(du[g].y << 16); go[4 * g + 3] = __uint_as_float(du[g].y & 0xffff0000u);
    }
    if (p.gated) {
      uint2 o1[4], o2[4];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        uint16_t dg[4], dor[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int v = 4 * g + e;
          dg[e] = f2bf(go[v] * o[v] * gt[v] * (1.f - gt[v]));
          dor[e] = f2bf(go[v] * gt[v]);
          go[v] = bf2f(dor[e]);  // the later kernels read the rounded copy
        }
        o1[g].x = (uint32_t)dg[0] | ((uint32_t)dg[1] << 16); o1[g].y = (uint32_t)dg[2] | ((uint32_t)dg[3] << 16);
        o2[g].x = (uint32_t)dor[0] | ((uint32_t)dor[1] << 16); o2[g].y = (uint32_t)dor[2] | ((uint32_t)dor[3] << 16);
      }
      store_row32((uint16_t*)p.dG + row, o1, hl, true);
      store_row32((uint16_t*)p.dO_out + (int64_t)(b - p.do_b0) * p.do_sb + (int64_t)q * p.do_ss + (int64_t)(h - p.do_h0) * p.do_sh + 32 * db, o2, hl,
                  true);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) part = fmaf(go[v], o[v], part);
  }
  return part;
}

// forward epilogue: normalise, gate, store Y (and LSE); recompute mode: gate gradient,
// pre-gated dO copy, Delta = rowsum(dO*O) and LSE into the workspace.  `l` is the complete row sum.
template <int DB, bool RECOMP>
__device__ inline void fwd_epilogue_rowsum(const KP& p, f32x16 (&oacc)[DB], float m, float l, int b, int h, int q,
                                           int hl, int64_t base) {
  if (q >= p.S) return;
  const float inv = 1.f / l;
  const float lse = (m + log2f(l)) * LN2;
  float part = 0.f;
#pragma unroll
  for (int db = 0; db < DB; ++db) part = fwd_epilogue_block<RECOMP>(p, oacc[db], db, inv, b, h, q, hl, base, part);
  if (!RECOMP) {
    if (p.lse_out && hl == 0) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
  } else {
    part = half_sum(part);
    if (hl == 0) {
      p.delta[(int64_t)(b - p.dl_b0) * p.dl_sb + (int64_t)(h - p.dl_h0) * p.dl_sh + q] = part;
      if (p.lse_out) p.lse_out[(int64_t)(b - p.lse_b0) * p.lse_sb + (int64_t)(h - p.lse_h0) * p.lse_sh + q] = lse;
    }
  }
}
// the same with `l` = each half-wave's part of the row sum
template <int DB, bool RECOMP>
__device__ inline void fwd_epilogue(const KP& p, f32x16 (&oacc)[DB], float m, float l, int b, int h, int q,
                                    int hl, int64_t base) {
  if (q >= p.S) return;
  fwd_epilogue_rowsum<DB, RECOMP>(p, oacc, m, half_sum(l), b, h, q, hl, base);
}

// the specialised kernels serve: no bias or a dense bf16 bias with S % 4 == 0; no mask or the
// causal mask; a positive scale; more than one 64-key tile's worth of rows
inline bool fast_ok(const KP& p) {
  if (p.S <= 64 || !(p.scale > 0.f) || p.mask_kind == 2 || p.bias_kind == 2) return false;
  if (p.bias_kind == 1 && (!p.bias_bf16 || (p.S & 3) || p.S > 32768)) return false;
  return true;
}

// Work-group shape of the forward / dQ kernels: query wavefronts x key-tile groups.  Large shares
// use 4x1 (many independent work-groups per compute unit); when the whole share offers fewer than
// two 128-query work-groups per compute unit the key tiles are split over groups inside the
// work-group (4x2); below one per compute unit (2x4) separate kernels take over whose work-groups
// own 32 queries (forward, dQ) or 32 keys (dK/dV) and whose four wavefronts split the other axis.
// Decided from the share, never from the chunk.
// Rows per group of the tiled bias-gradient kernel: 0 = one group (the sum continues in the output);
// otherwise the share's rows are cut into groups so that about two work-groups per compute unit exist.
inline int dbias_group_rows(const KP& p) {
  if (p.bias_kind != 1 || !fast_ok(p)) return 0;
  const int64_t tiles = (int64_t)((p.S + 63) / 64) * ((p.S + 63) / 64) * p.H;
  return tiles >= 512 ? 0 : 64;
}

enum WgShape { WG_4x1, WG_4x2, WG_2x4 };
inline WgShape wg_shape(const KP& p) {
  const int64_t wgs = (int64_t)((p.S + 127) / 128) * p.share_units;
  if (wgs >= 512 || p.S < 512) return WG_4x1;
  if (wgs >= 256) return WG_4x2;
  // the kernels of the smallest shape address one (row, head) slice with 32-bit buffer offsets
  const int64_t row_stride = p.ss > (int64_t)p.H * p.D ? p.ss : (int64_t)p.H * p.D;
  if (((int64_t)(p.S - 1) * row_stride + p.D) * 2 >= (1ll << 31)) return WG_4x2;
  return WG_2x4;
}

}  // namespace

// specialised kernels, one translation unit each
hipError_t launch_fast_fwd(const KP& p, bool recompute, hipStream_t st);
hipError_t launch_fast_fwd128(const KP& p, bool recompute, hipStream_t st);
hipError_t launch_fast_dq(const KP& p, hipStream_t st);
hipError_t launch_fast_dq128(const KP& p, hipStream_t st);
hipError_t launch_fast_recompute_dq(const KP& p, hipStream_t st);
hipError_t launch_fast_dkdv(const KP& p, hipStream_t st);
hipError_t launch_fast_kv128(const KP& p, hipStream_t st);
hipError_t launch_fast_fwd_wave(const KP& p, bool recompute, hipStream_t st);
hipError_t launch_fast_fwd_wave128(const KP& p, bool recompute, hipStream_t st);
hipError_t launch_fast_bwd_wave(const KP& p, hipStream_t st);
hipError_t launch_fast_bwd_wave3(const KP& p, hipStream_t st);
hipError_t launch_fast_dbias(const KP& p, hipStream_t st);

}  // namespace ssa
