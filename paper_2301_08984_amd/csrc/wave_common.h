// Helpers shared by the wave kernels (small shares with long rows): block order, bounds-checked
// staging loads, accumulator rescale.
#pragma once
#include "mfma_common.h"

#include <type_traits>

namespace ssa {
namespace {

// Block order of the wave kernels: the heaviest blocks first over the whole launch (block 0 of
// every head and row, then block 1, ...), so that when there are more work-groups than compute
// units the late, light ones fill in behind the early ones.
__device__ inline BlockId heavy_first_block_id() {
  const int units = gridDim.y * gridDim.z;
  const int n = gridDim.x * units;
  int lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  // Between one and two work-groups per compute unit, two resident at a time: the dispatcher deals
  // the first NCU out one per compute unit and then starts over, so work-group p + NCU joins
  // work-group p.  With t counting from the heaviest, the NCU - m heaviest (m = n - NCU) are given
  // the positions that stay alone, and the others are paired medium with light (t = NCU - m + i with
  // t = n - 1 - i), so that every compute unit gets about the same number of sub-tiles.  Only the
  // order of execution depends on this; any order gives the same results.
  constexpr int NCU = 256;
  if (n > NCU && n <= 2 * NCU) {
    const int m = n - NCU;
    lin = lin < m ? NCU - m + lin : lin < NCU ? lin - m : n - 1 - (lin - NCU);
  }
  BlockId b;
  b.x = lin / units;
  b.y = (lin % units) % gridDim.y;
  b.z = (lin % units) / gridDim.y;
  return b;
}

// coalesced fetch of the 32-row sub-tile starting at row `row0` (uniform over the wavefront) of one
// (row, head) slice of a [.., S, .., D] bf16 tensor whose rows are `ss` elements apart: lane l takes
// the 16-byte chunks l, l+64, ... (chunk i = row i / (D/8), columns 8 * (i % (D/8)) ..).  Buffer
// loads with a descriptor over the slice: rows past S-1 return zeros, so the staging needs neither
// clamps nor branches.  The hardware bounds-checks the lane offset only (not the scalar offset), so
// the whole offset is the lane offset: `loff` = ((l / (D/8)) * ss + 8 * (l % (D/8))) * 2 bytes plus
// the chunk's and the sub-tile's row offsets.  The slice spans less than 2 GiB (checked on the host).
template <int D>
__device__ inline void sub_load(u32x4 (&dst)[D / 16], const uint16_t* base, int64_t ss, int S, int row0,
                                uint32_t loff) {
  constexpr int RSTEP = 64 / (D / 8);
  const __amdgpu_buffer_rsrc_t rs =
      __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)(((int64_t)(S - 1) * ss + D) * 2), 0x00020000);
  const uint32_t step = (uint32_t)RSTEP * (uint32_t)ss * 2u;
  const uint32_t off = loff + (uint32_t)row0 * (uint32_t)ss * 2u;
#pragma unroll
  for (int c = 0; c < D / 16; ++c) dst[c] = __builtin_amdgcn_raw_buffer_load_b128(rs, off + c * step, 0, 0);
}
// O accumulators *= alpha, for the rare step on which the running maximum is raised.  Written so that
// the accumulators stay in the accumulation registers on the common path: as ordinary C++ the
// compiler copies all of them to vector registers and back around the branch on every step.
// The wait states cover a matrix operation that may still be writing the accumulators.
template <int DB>
__device__ inline void rescale_acc(f32x16 (&o)[DB], float alpha) {
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    float t[16], tmp;
#pragma unroll
    for (int v = 0; v < 16; ++v) t[v] = o[db][v];
#define SS_RS(i) "v_accvgpr_read_b32 %16, %" #i "\n\tv_mul_f32 %16, %16, %17\n\tv_accvgpr_write_b32 %" #i ", %16\n\t"
    asm volatile("s_nop 15\n\ts_nop 15\n\t" SS_RS(0) SS_RS(1) SS_RS(2) SS_RS(3) SS_RS(4) SS_RS(5) SS_RS(6) SS_RS(7)
                     SS_RS(8) SS_RS(9) SS_RS(10) SS_RS(11) SS_RS(12) SS_RS(13) SS_RS(14) SS_RS(15) "s_nop 7"
                 : "+a"(t[0]), "+a"(t[1]), "+a"(t[2]), "+a"(t[3]), "+a"(t[4]), "+a"(t[5]), "+a"(t[6]), "+a"(t[7]),
                   "+a"(t[8]), "+a"(t[9]), "+a"(t[10]), "+a"(t[11]), "+a"(t[12]), "+a"(t[13]), "+a"(t[14]),
                   "+a"(t[15]), "=&v"(tmp)
                 : "v"(alpha));
#undef SS_RS
#pragma unroll
    for (int v = 0; v < 16; ++v) o[db][v] = t[v];
  }
}

template <int D, int LD>
__device__ inline void sub_store(uint16_t* t, const u32x4 (&src)[D / 16], int lane) {
  constexpr int CPR = D / 8;
#pragma unroll
  for (int c = 0; c < D / 16; ++c) {
    const int idx = lane + c * 64, row = idx / CPR, col = (idx % CPR) * 8;
    *(u32x4*)(t + row * LD + col) = src[c];
  }
}


}  // namespace
}  // namespace ssa
