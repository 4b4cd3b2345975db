// Kernels of the co-sharded feed-forward operator: one bf16 MFMA GEMM with fused epilogues, and a
// fixed-order column sum for the bias gradients.
#include "ffn_kernels.h"

#include "mfma_common.h"

namespace ssa {
namespace {

constexpr int GBM = 256, GBN = 128, GBK = 64;  // work-group tile; four wavefronts, 2 x 2, 128 x 64 each
constexpr float GELU_C0 = 0.7978845608028654f, GELU_C1 = 0.044715f;

// k-slots of one 16-wide contraction step as the transposed LDS read delivers them to half hl of the
// wavefront: {4hl .. 4hl+3, 8+4hl .. 8+4hl+3}.  A k-contiguous operand paired with a transposed one
// is read in the same order, as two 8-byte pieces.
template <int LD>
__device__ inline bf16x8 lds_nat_perm(const uint16_t* t, int row, int ks, int hl) {
  union { uint2 h[2]; bf16x8 v; } o;
  o.h[0] = *(const uint2*)(t + row * LD + 16 * ks + 4 * hl);
  o.h[1] = *(const uint2*)(t + row * LD + 16 * ks + 8 + 4 * hl);
  return o.v;
}

__device__ inline float act_f(float z, int kind) {
  if (kind == 0) return fmaxf(z, 0.f);
  const float u = GELU_C0 * (z + GELU_C1 * z * z * z);
  const float t = 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + fast_exp2(2.f * LOG2E * u));
  return 0.5f * z * (1.f + t);
}
__device__ inline void act_and_grad(float z, int kind, float& h, float& d) {
  if (kind == 0) {
    h = fmaxf(z, 0.f);
    d = z > 0.f ? 1.f : 0.f;
    return;
  }
  const float u = GELU_C0 * (z + GELU_C1 * z * z * z);
  const float t = 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + fast_exp2(2.f * LOG2E * u));
  h = 0.5f * z * (1.f + t);
  d = 0.5f * (1.f + t) + 0.5f * z * (1.f - t * t) * GELU_C0 * (1.f + 3.f * GELU_C1 * z * z);
}

// Stages a ROWS x COLS tile (COLS contiguous in memory, rows `ld` elements apart) starting at
// (r0, c0) of a matrix with rtot x ctot valid elements: thread t takes the 16-byte chunks t, t+256, ..
// Bounds-checked buffer loads: everything outside the matrix reads as zero (the whole offset is the
// lane offset, the only part the hardware range-checks; a column past ctot gets an offset past the
// descriptor's extent).
template <int ROWS, int COLS>
struct TileLoader {
  static constexpr int CPR = COLS / 8, CPT = ROWS * CPR / 256;
  __amdgpu_buffer_rsrc_t rs;
  uint32_t lane_off[CPT];  // (row_in_tile * ld + 8 * chunk_in_row) * 2
  int ccol;                // 8 * chunk_in_row (the same for all of a thread's chunks: 256 % CPR == 0)
  uint32_t ld2;
  int ctot;
  __device__ void init(const uint16_t* base, int64_t ld, int rtot, int ctot_, int tid) {
    rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)(((int64_t)(rtot - 1) * ld + ctot_) * 2), 0x00020000);
    ld2 = (uint32_t)ld * 2u;
    ctot = ctot_;
    ccol = (tid % CPR) * 8;
#pragma unroll
    for (int c = 0; c < CPT; ++c) lane_off[c] = (uint32_t)((tid + c * 256) / CPR) * ld2 + (uint32_t)ccol * 2u;
  }
  __device__ void load(u32x4 (&dst)[CPT], int r0, int c0) const {
    const uint32_t so = (uint32_t)r0 * ld2 + (uint32_t)c0 * 2u;
    const bool inside = c0 + ccol < ctot;
#pragma unroll
    for (int c = 0; c < CPT; ++c)
      dst[c] = __builtin_amdgcn_raw_buffer_load_b128(rs, inside ? lane_off[c] + so : 0x7ffffff0u, 0, 0);
  }
  template <int LD>
  __device__ static void store(uint16_t* t, const u32x4 (&src)[CPT], int tid) {
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
      const int idx = tid + c * 256, row = idx / CPR, col = (idx % CPR) * 8;
      *(u32x4*)(t + row * LD + col) = src[c];
    }
  }
};

// ---------------------------------------------------------------------------
// C[M,N] = A B with bf16 operands and fp32 accumulation on v_mfma_f32_32x32x16_bf16.
//   AT = false: A[m][k] at A + m*lda + k      AT = true: A[k][m] at A + k*lda + m
//   BT = false: B[k][n] at B + k*ldb + n      BT = true: B[n][k] at B + n*ldb + k
// A 256 x 128 tile per work-group, 64-wide contraction stages through LDS (one buffer per operand,
// the next stage travels global -> registers meanwhile; two work-groups per compute unit overlap
// each other's staging).  Operands whose contraction index is not contiguous in memory are read
// from LDS with the transposed read.  The contraction runs in ascending k, 16 at a time, whatever
// the tile position: with EPI_ACC the accumulator starts from the fp32 partial result of the
// previous chunks, so a sum cut into chunks at multiples of 16 is the same sum.
// ---------------------------------------------------------------------------
template <bool AT, bool BT, int EPI>
__global__ __launch_bounds__(256, 2) void gemm_kernel(GemmArgs g) {
  constexpr int LDA = AT ? GBM + 16 : GBK + 8, LDB = BT ? GBK + 8 : GBN + 16;
  constexpr int A_ELEMS = AT ? GBK * LDA : GBM * LDA, B_ELEMS = BT ? GBN * LDB : GBK * LDB;
  __shared__ __attribute__((aligned(16))) uint16_t sA[A_ELEMS];
  __shared__ __attribute__((aligned(16))) uint16_t sB[B_ELEMS];
  using LoadA = TileLoader<AT ? GBK : GBM, AT ? GBM : GBK>;
  using LoadB = TileLoader<BT ? GBN : GBK, BT ? GBK : GBN>;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 31, hl = lane >> 5;
  const int wm = w >> 1, wn = w & 1;
  const int m0 = blockIdx.y * GBM, n0 = blockIdx.x * GBN;

  LoadA la;
  LoadB lb;
  la.init(g.A, g.lda, AT ? g.K : g.M, AT ? g.M : g.K, tid);
  lb.init(g.B, g.ldb, BT ? g.N : g.K, BT ? g.K : g.N, tid);
  u32x4 pa[LoadA::CPT], pb[LoadB::CPT];
  auto gload = [&](int k0) {
    if (AT) la.load(pa, k0, m0); else la.load(pa, m0, k0);
    if (BT) lb.load(pb, n0, k0); else lb.load(pb, k0, n0);
  };

  f32x16 acc[4][2];
  if (EPI == EPI_ACC && g.accumulate) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + wn * 64 + 32 * j + r;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = m0 + wm * 128 + 32 * i + key_of(v, hl);
          acc[i][j][v] = (m < g.M && n < g.N) ? g.acc32[(int64_t)m * g.ld32 + n] : 0.f;
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  }

  const int nk = (g.K + GBK - 1) / GBK;
  gload(0);
  for (int kt = 0; kt < nk; ++kt) {
    __syncthreads();
    LoadA::template store<LDA>(sA, pa, tid);
    LoadB::template store<LDB>(sB, pb, tid);
    if (kt + 1 < nk) gload((kt + 1) * GBK);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < GBK / 16; ++ks) {
      bf16x8 fa[4], fb[2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int mrow = wm * 128 + 32 * i;
        if (AT) fa[i] = lds_tr<LDA>(sA, 16 * ks, mrow, lane);
        else if (!BT) fa[i] = lds_nat_perm<LDA>(sA, mrow + r, ks, hl);
        else fa[i] = lds_nat<LDA>(sA, mrow + r, ks, hl);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int ncol = wn * 64 + 32 * j;
        if (!BT) fb[j] = lds_tr<LDB>(sB, 16 * ks, ncol, lane);
        else if (AT) fb[j] = lds_nat_perm<LDB>(sB, ncol + r, ks, hl);
        else fb[j] = lds_nat<LDB>(sB, ncol + r, ks, hl);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = mfma(fa[i], fb[j], acc[i][j]);
    }
  }

  // epilogue: lane = column n, register v = row m
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn * 64 + 32 * j + r;
    if (n >= g.N) continue;
    float bias = 0.f;
    if ((EPI == EPI_ACT || (EPI == EPI_ACC && g.last)) && g.bias) bias = bf2f(g.bias[n]);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = m0 + wm * 128 + 32 * i + key_of(v, hl);
        if (m >= g.M) continue;
        const float x = acc[i][j][v];
        if (EPI == EPI_ACT) {
          if (g.out2) {
            float h, d;
            act_and_grad(x + bias, g.act, h, d);
            g.out[(int64_t)m * g.ldo + n] = f2bf(h);
            g.out2[(int64_t)m * g.ldo + n] = f2bf(d);
          } else {
            g.out[(int64_t)m * g.ldo + n] = f2bf(act_f(x + bias, g.act));
          }
        } else if (EPI == EPI_MUL) {
          g.out[(int64_t)m * g.ldo + n] = f2bf(x * bf2f(g.mul[(int64_t)m * g.ldm + n]));
        } else if (EPI == EPI_ACC) {
          if (g.last) g.out[(int64_t)m * g.ldo + n] = f2bf(x + bias);
          else g.acc32[(int64_t)m * g.ld32 + n] = x;
        } else {
          g.out[(int64_t)m * g.ldo + n] = f2bf(x);
        }
      }
  }
}

// out[n] = sum over m of A[m][n], fp32, fixed order: a work-group takes 64 columns; 32 row groups
// per column (rows g, g+32, .. summed in ascending order, 16-byte loads of 8 columns), then the 32
// partial sums in ascending g.  N is a multiple of 8 and A + n 16-byte aligned for n % 8 == 0.
__global__ __launch_bounds__(256) void colsum_kernel(const uint16_t* A, int64_t lda, int M, int N, uint16_t* out) {
  __shared__ float part[32][65];
  const int cl = threadIdx.x & 7, rg = threadIdx.x >> 3;
  const int n = blockIdx.x * 64 + cl * 8;
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (n < N) {
    const uint16_t* col = A + n;
#pragma unroll 4
    for (int m = rg; m < M; m += 32) {
      const u32x4 v = *(const u32x4*)(col + (int64_t)m * lda);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        s[2 * e] += __uint_as_float(v[e] << 16);
        s[2 * e + 1] += __uint_as_float(v[e] & 0xffff0000u);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) part[rg][cl * 8 + e] = s[e];
  __syncthreads();
  const int c = threadIdx.x;
  if (c < 64 && blockIdx.x * 64 + c < N) {
    float t = part[0][c];
#pragma unroll
    for (int g = 1; g < 32; ++g) t += part[g][c];
    out[blockIdx.x * 64 + c] = f2bf(t);
  }
}

template <bool AT, bool BT>
hipError_t launch_epi(const GemmArgs& g, int epi, hipStream_t st) {
  const dim3 grid((g.N + GBN - 1) / GBN, (g.M + GBM - 1) / GBM);
  switch (epi) {
    case EPI_ACT: gemm_kernel<AT, BT, EPI_ACT><<<grid, 256, 0, st>>>(g); break;
    case EPI_MUL: gemm_kernel<AT, BT, EPI_MUL><<<grid, 256, 0, st>>>(g); break;
    case EPI_ACC: gemm_kernel<AT, BT, EPI_ACC><<<grid, 256, 0, st>>>(g); break;
    default: gemm_kernel<AT, BT, EPI_STORE><<<grid, 256, 0, st>>>(g); break;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, bool at, bool bt, int epi, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (!at && !bt) return launch_epi<false, false>(g, epi, st);
  if (!at && bt) return launch_epi<false, true>(g, epi, st);
  if (at && !bt) return launch_epi<true, false>(g, epi, st);
  return hipErrorInvalidValue;  // A^T B^T is not needed by the feed-forward operator
}

hipError_t launch_colsum(const void* A, int64_t lda, int M, int N, void* out, hipStream_t st) {
  colsum_kernel<<<(N + 63) / 64, 256, 0, st>>>((const uint16_t*)A, lda, M, N, (uint16_t*)out);
  return hipGetLastError();
}

}  // namespace ssa
