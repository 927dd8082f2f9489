// Gram matrices M_h = W_O^h W_O^hT of the per-head output projection (Eq. mha).
// Weight-only preparation: the indicator needs ||x W_O^h||_2 = sqrt(x M_h x^T) only.
#include "common.hpp"

namespace restkv {

namespace {

// grid (d/16, d/16, Hq), 256 threads = 16x16 outputs; FP64 accumulation over d_model.
__global__ __launch_bounds__(256) void k_gram(int d, int64_t D, const float* __restrict__ w,
                                              float* __restrict__ gram) {
  __shared__ float As[16][65];
  __shared__ float Bs[16][65];
  const int h = blockIdx.z;
  const int a0 = blockIdx.y * 16, b0 = blockIdx.x * 16;
  const int ta = threadIdx.x >> 4, tb = threadIdx.x & 15;
  const float* wh = w + (int64_t)h * d * D;
  double acc = 0.0;
  for (int64_t k0 = 0; k0 < D; k0 += 64) {
    __syncthreads();
    for (int x = threadIdx.x; x < 16 * 64; x += 256) {
      const int r = x >> 6, c = x & 63;
      const int64_t kk = k0 + c;
      As[r][c] = kk < D ? wh[(int64_t)(a0 + r) * D + kk] : 0.f;
      Bs[r][c] = kk < D ? wh[(int64_t)(b0 + r) * D + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < 64; ++c) acc += (double)As[ta][c] * (double)Bs[tb][c];
  }
  gram[((int64_t)h * d + a0 + ta) * d + b0 + tb] = (float)acc;
}

}  // namespace

int launch_gram(const Prob& pb, const float* w_o, int64_t d_model, float* gram, hipStream_t st) {
  RK_LAUNCH(ST_GRAM, st, k_gram, dim3(pb.d / 16, pb.d / 16, pb.Hq), dim3(256), 0, st, pb.d, d_model,
                     w_o, gram);
  return hip_status();
}

}  // namespace restkv
