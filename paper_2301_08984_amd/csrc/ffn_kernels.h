// Launchers of the feed-forward kernels (bf16 MFMA GEMM with fused epilogues, column sums).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssa {

enum { EPI_ACT = 0, EPI_MUL = 1, EPI_ACC = 2, EPI_STORE = 3, EPI_ACC16 = 4 };

// C[M,N] = A B (see gemm_kernel for the operand layouts); what happens to C:
//   EPI_ACT   out = act(C + bias[n]) (bf16); out2, if given, = act'(C + bias[n])
//   EPI_MUL   out = C * mul[m][n] (bf16; out may be mul)
//   EPI_ACC   the accumulator starts from acc32 if `accumulate`; then `last` ? out = C + bias[n] (bf16,
//             bias may be NULL) : acc32 = C (fp32, whole tiles in the kernel's own order; see gemm_acc_bytes)
//   EPI_STORE out = C (bf16)
//   EPI_ACC16 the accumulator starts from `out` (bf16, widened) if `accumulate`; out = C + bias[n] (bf16,
//             bias may be NULL): the partial sum between chunks lives in the output itself
struct GemmArgs {
  const uint16_t* A;
  const uint16_t* B;
  int64_t lda, ldb;
  int M, N, K;
  const uint16_t* bias;
  uint16_t* out;
  int64_t ldo;
  uint16_t* out2;
  const uint16_t* mul;
  int64_t ldm;
  float* acc32;  // ceil(M/256) * ceil(N/256) tiles of 256 x 256 fp32, in the kernel's own order
  int accumulate, last, act;
};

// bytes of the fp32 partial-result buffer of an M x N product
size_t gemm_acc_bytes(int M, int N);
hipError_t launch_gemm(const GemmArgs& g, bool a_transposed, bool b_transposed, int epilogue, hipStream_t st);
// out[n] (bf16) = sum over m of A[m][n] (bf16 in, fp32 sum, fixed order)
hipError_t launch_colsum(const void* A, int64_t lda, int M, int N, void* out, hipStream_t st);

}  // namespace ssa
