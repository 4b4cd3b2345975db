// Sub-tiles that travel from memory straight into LDS, for the small-share kernels at head size 128.
//
// Measured on the register-staged kernels: the 16 `ds_write_b128` per 32 x 32 tile are their largest
// single cost (LDS takes writes at 76 bytes per cycle and compute unit, a third of its read rate, and
// a wavefront that waits at a store holds back the reads and matrix instructions behind it), the
// 64 staging registers push stationary fragments into accumulation registers (tens of copies per
// tile), and every load needs an address add.  Here a sub-tile is 8 `buffer_load ... lds` of 1 KB
// each: no staging registers, no store instructions, lane offsets that never change.
//
// LDS image of a 32-row sub-tile (rows of 256 bytes = 16 chunks of 16 bytes, no padding, since a
// load instruction fills 1 KB = 4 rows contiguously): chunk c of row rho sits at position
// c ^ sw(rho), sw(rho) = ((rho & 3) << 2) | ((rho >> 2) & 3).  The swizzle is applied by choosing
// WHICH chunk a lane fetches for its fixed LDS position.  16 consecutive rows put the same chunk at
// 16 different positions (operand reads along the rows: no bank conflicts), and 4 consecutive rows
// put a 64-byte group of chunks into 4 different 64-byte bank groups (transposed reads).
//
// The fragment reads are written as assembly: the compiler cannot tell which of the loads under way
// fills the tile a `ds_read` touches and would wait for all of them (vmcnt(0)) before every read it
// can see, which would undo the overlap.  A read is split into an issue part and a wait part; the
// registers are not touched in between (outputs of the first, in/outputs of the second).
//
// Files that include this are compiled with the matrix instructions in their vector-register form
// and use no accumulation registers at all, so that the compiler may give the wavefront all 256
// registers as vector registers (with any accumulation register in use it splits them 128 / 128 and
// moves operands between the halves on every use).
#pragma once
#include "wave_common.h"

namespace ssa {
namespace {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void w_lds_void;

constexpr int W_TILE_B = 32 * 128 * 2;  // bytes of one sub-tile

__device__ __forceinline__ int w_sw(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

#define W_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")

// lane offsets of the 8 load instructions of a sub-tile whose rows are `ss2` bytes apart: instruction
// t fills LDS rows 4t .. 4t+3, lane l the position l % 16 of row 4t + l / 16
__device__ __forceinline__ void w_lane_offsets(uint32_t (&goff)[8], uint32_t ss2, int lane) {
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    const int rho = 4 * t + (lane >> 4);
    goff[t] = (uint32_t)rho * ss2 + 16u * (uint32_t)((lane & 15) ^ w_sw(rho));
  }
}
// Sub-tile starting `boff` bytes into a (row, head) slice of `slice_bytes` bytes -> the tile at
// `tile` (uniform).  The descriptor starts at the sub-tile and ends with the slice, so the lane
// offsets are the same for every sub-tile and rows past the end arrive as zeros (the hardware
// range-checks the lane offset).  boff < slice_bytes < 2 GiB.
__device__ __forceinline__ void w_fetch(char* tile, const void* slice, uint32_t boff, uint32_t slice_bytes,
                                        const uint32_t (&goff)[8]) {
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)slice + boff), 0, (int)(slice_bytes - boff), 0x00020000);
#pragma unroll
  for (int t = 0; t < 8; ++t)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (w_lds_void*)(tile + t * 1024), 16, goff[t], 0, 0, 0);
}
// LDS addresses of the operand fragments ks = 0..7 of the tile at `tile0`: row r, chunk 2 ks + hl
__device__ __forceinline__ void w_nat_addr(uint32_t (&ka)[8], const char* tile0, int r, int hl) {
  const uint32_t a0 = (uint32_t)(size_t)(w_lds_void*)tile0 + (uint32_t)r * 256u + (uint32_t)((hl ^ w_sw(r)) << 4);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) ka[ks] = a0 ^ (uint32_t)(ks << 5);
}
// LDS addresses of the transposed reads of the tile at `tile0`: lane gets column 32 db + l % 32 of
// rows 16 t + {0..3, 8..11} + 4 hl, i.e. (as ds_read_b64_tr_b16 wants it) four consecutive elements
// of row 16 t + 8 half + 4 (bk >> 1) + (i >> 2) at column 32 db + 16 (bk & 1) + 4 (i & 3), with
// i = l % 16, bk = l / 16; va[half][db] is for t = 0, t = 1 is 4096 bytes further on
__device__ __forceinline__ void w_tr_addr(uint32_t (&va)[2][4], const char* tile0, int lane) {
  const int i = lane & 15, bk = lane >> 4;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const int row = 8 * half + 4 * (bk >> 1) + (i >> 2);
    const int lowc = (2 * (bk & 1) + ((i & 3) >> 1)) ^ ((2 * half + (bk >> 1)) & 3);
#pragma unroll
    for (int db = 0; db < 4; ++db)
      va[half][db] = (uint32_t)(size_t)(w_lds_void*)tile0 + (uint32_t)row * 256u + (uint32_t)((db ^ (i >> 2)) << 6) +
                     (uint32_t)(lowc << 4) + 8u * (i & 1);
  }
}
// the eight operand fragments of the tile OFF bytes after the one the addresses were made for
template <int OFF>
__device__ __forceinline__ void w_nat_issue(u32x4 (&f)[8], const uint32_t (&ka)[8]) {
  asm volatile(
      "ds_read_b128 %0, %8 offset:%16\n\tds_read_b128 %1, %9 offset:%16\n\tds_read_b128 %2, %10 offset:%16\n\t"
      "ds_read_b128 %3, %11 offset:%16\n\tds_read_b128 %4, %12 offset:%16\n\tds_read_b128 %5, %13 offset:%16\n\t"
      "ds_read_b128 %6, %14 offset:%16\n\tds_read_b128 %7, %15 offset:%16"
      : "=&v"(f[0]), "=&v"(f[1]), "=&v"(f[2]), "=&v"(f[3]), "=&v"(f[4]), "=&v"(f[5]), "=&v"(f[6]), "=&v"(f[7])
      : "v"(ka[0]), "v"(ka[1]), "v"(ka[2]), "v"(ka[3]), "v"(ka[4]), "v"(ka[5]), "v"(ka[6]), "v"(ka[7]), "n"(OFF)
      : "memory");
}
__device__ __forceinline__ void w_nat_wait(u32x4 (&f)[8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7])
               :
               : "memory");
}
// the sixteen transposed reads of a tile: f[t][2 db + half]
template <int OFF>
__device__ __forceinline__ void w_tr_issue(u32x2 (&f)[2][8], const uint32_t (&va)[2][4]) {
#define W_TR8(N)                                                                                          \
  "ds_read_b64_tr_b16 %0, %8 offset:%" #N "\n\tds_read_b64_tr_b16 %1, %9 offset:%" #N "\n\t"                 \
  "ds_read_b64_tr_b16 %2, %10 offset:%" #N "\n\tds_read_b64_tr_b16 %3, %11 offset:%" #N "\n\t"               \
  "ds_read_b64_tr_b16 %4, %12 offset:%" #N "\n\tds_read_b64_tr_b16 %5, %13 offset:%" #N "\n\t"               \
  "ds_read_b64_tr_b16 %6, %14 offset:%" #N "\n\tds_read_b64_tr_b16 %7, %15 offset:%" #N
#define W_TR_OPS(T, O)                                                                                                \
  : "=&v"(f[T][0]), "=&v"(f[T][1]), "=&v"(f[T][2]), "=&v"(f[T][3]), "=&v"(f[T][4]), "=&v"(f[T][5]), "=&v"(f[T][6]),   \
    "=&v"(f[T][7])                                                                                                    \
  : "v"(va[0][0]), "v"(va[1][0]), "v"(va[0][1]), "v"(va[1][1]), "v"(va[0][2]), "v"(va[1][2]), "v"(va[0][3]),          \
    "v"(va[1][3]), "n"(O)                                                                                             \
  : "memory"
  asm volatile(W_TR8(16) W_TR_OPS(0, OFF));
  asm volatile(W_TR8(16) W_TR_OPS(1, OFF + 4096));
#undef W_TR8
#undef W_TR_OPS
}
__device__ __forceinline__ void w_tr_wait(u32x2 (&f)[2][8]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(f[0][0]), "+v"(f[0][1]), "+v"(f[0][2]), "+v"(f[0][3]), "+v"(f[0][4]), "+v"(f[0][5]), "+v"(f[0][6]),
                 "+v"(f[0][7]), "+v"(f[1][0]), "+v"(f[1][1]), "+v"(f[1][2]), "+v"(f[1][3]), "+v"(f[1][4]), "+v"(f[1][5]),
                 "+v"(f[1][6]), "+v"(f[1][7])
               :
               : "memory");
}
__device__ __forceinline__ bf16x8 w_frag(const u32x4& x) {
  union { u32x4 u; bf16x8 v; } c;
  c.u = x;
  return c.v;
}
__device__ __forceinline__ bf16x8 w_frag2(const u32x2& lo, const u32x2& hi) {
  union { u32x2 h[2]; bf16x8 v; } c;
  c.h[0] = lo;
  c.h[1] = hi;
  return c.v;
}

}  // namespace
}  // namespace ssa
