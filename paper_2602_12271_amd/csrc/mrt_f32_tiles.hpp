// fp32 contractions on the matrix unit for the fp32 kernels (forward fp32 path and backward pass):
// operands stay fp32 in LDS, products are formed by v_mfma_f32_16x16x4_f32, so the arithmetic is
// that of an fp32 dot product (different summation order only).
#pragma once
#include <hip/hip_runtime.h>

namespace mrt {
namespace {

constexpr int kThreads = 1024;
using f32x4 = float __attribute__((ext_vector_type(4)));
constexpr int kWaves = kThreads / 64;

// One 16x16 tile of C += A B over k in [0, K) on the fp32 matrix unit.  A(r, k) and B(k, c) are
// accessors that return 0 outside their operand.  v_mfma_f32_16x16x4_f32: lane i supplies
// A[i % 16][i / 16] and B[i / 16][i % 16] of one 16x4 by 4x16 step and holds
// C[4 * (i / 16) + r][i % 16] in register r.
template <typename FA, typename FB>
__device__ inline f32x4 mma16(FA A, FB B, int K, f32x4 acc, int lane) {
  const int i = lane & 15, q = lane >> 4;
  for (int k0 = 0; k0 < K; k0 += 4)
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(A(i, k0 + q), B(k0 + q, i), acc, 0, 0, 0);
  return acc;
}

// C = A B for an M x N result, its 16x16 tiles dealt to the waves; done(row, col, value) is
// called once per element of C.
template <typename FA, typename FB, typename FD>
__device__ inline void gemm_tiles(int M, int N, int K, FA A, FB B, FD done, int tid) {
  const int wave = tid >> 6, lane = tid & 63, i = lane & 15, q = lane >> 4;
  const int tn = (N + 15) >> 4, tiles = ((M + 15) >> 4) * tn;
  for (int t = wave; t < tiles; t += kWaves) {
    const int r0 = 16 * (t / tn), c0 = 16 * (t % tn);
    const f32x4 acc = mma16([&](int r, int k) { return A(r0 + r, k); },
                            [&](int k, int c) { return B(k, c0 + c); }, K, f32x4{0.f, 0.f, 0.f, 0.f}, lane);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = r0 + 4 * q + r, col = c0 + i;
      if (row < M && col < N) done(row, col, acc[r]);
    }
  }
}


}  // namespace
}  // namespace mrt
