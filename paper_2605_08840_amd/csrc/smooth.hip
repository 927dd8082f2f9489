// Spatial-temporal smoothing (Sec. 3.3): EMA over the window queries, drift statistic of
// the per-query top-B positions, adaptive window size / shift, shifted box mean.
#include "rowselect.hpp"

namespace restkv {

namespace {

// ema[g,n] by the recursion: first query as is, every later one enters with weight alpha.
// grid (ceil(P/256), Hkv), 256 threads; reads of score are coalesced along n.
__global__ __launch_bounds__(256) void k_ema(Prob pb, const float* __restrict__ score,
                                             float* __restrict__ ema) {
  const int g = blockIdx.y;
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= pb.P) return;
  const float* s = score + (int64_t)g * pb.W * pb.ld + n;
  const float a = pb.alpha, b = 1.0f - pb.alpha;
  float e = s[0];
  for (int i = 1; i < pb.W; ++i) e = a * s[(int64_t)i * pb.ld] + b * e;
  ema[(int64_t)g * pb.ld + n] = e;
}

// Sum of the positions of the top-min(B,P) entries of one (head, query) row of the raw score.
// grid (W, Hkv), SEL_NT threads.
__global__ __launch_bounds__(SEL_NT) void k_row_topk_sum(Prob pb, const float* __restrict__ score,
                                                         unsigned long long* __restrict__ rowsum) {
  __shared__ SelectSmem sm;
  const int i = blockIdx.x, g = blockIdx.y;
  const float* row = score + ((int64_t)g * pb.W + i) * pb.ld;
  const int k = min(pb.B, pb.P);
  uint32_t tau, n_gt, k_eq;
  block_kth_key(row, pb.P, k, sm, tau, n_gt, k_eq);
  unsigned long long acc = 0;
  block_visit_topk(row, pb.P, tau, k_eq, sm, [&](int x, uint32_t) { acc += (unsigned long long)x; });
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.isum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long tot = 0;
    for (int j = 0; j < SEL_NW; ++j) tot += sm.isum[j];
    rowsum[g * pb.W + i] = tot;
  }
}

// Window size and shift from the drift statistic (device function so that every block of
// the box kernel derives the same integers without a host round trip).
__device__ inline void aws_window(const Prob& pb, const unsigned long long* rowsum, int g,
                                  int& w_s, int& gamma, double& d_front, double& d_rear) {
  w_s = pb.base_k; gamma = 0; d_front = 0.0; d_rear = 0.0;
  if (!pb.adaptive) return;
  const int nf = pb.W / 2;
  const double bt = (double)min(pb.B, pb.P);
  unsigned long long sf = 0, sr = 0;
  for (int i = 0; i < pb.W; ++i) {
    const unsigned long long s = rowsum[g * pb.W + i];
    if (i < nf) sf += s; else sr += s;
  }
  d_front = (double)sf / (bt * (double)nf);
  d_rear = (double)sr / (bt * (double)(pb.W - nf));
  const double x = d_front - d_rear;
  const double beta = (double)pb.beta;
  w_s = pb.base_k + 2 * (int)floor(fabs(x) / beta);
  const int f = (int)floor(x / beta);
  gamma = x > 0.0 ? f : f + 1;
}

// final[g,n] = (1/W_s) sum_{j=gamma-half}^{gamma+half} ema[g,n+j], zero outside [0,P).
// grid (ceil(P/256), Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_box(Prob pb, const float* __restrict__ ema,
                                             const unsigned long long* __restrict__ rowsum,
                                             float* __restrict__ fin, int32_t* __restrict__ aws_info,
                                             double* __restrict__ aws_d) {
  const int g = blockIdx.y;
  int w_s, gamma;
  double df, dr;
  aws_window(pb, rowsum, g, w_s, gamma, df, dr);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    if (aws_info) { aws_info[2 * g] = w_s; aws_info[2 * g + 1] = gamma; }
    if (aws_d) { aws_d[2 * g] = df; aws_d[2 * g + 1] = dr; }
  }
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= pb.P) return;
  const float* e = ema + (int64_t)g * pb.ld;
  const int half = w_s / 2;
  const int lo = max(0, n + gamma - half), hi = min(pb.P - 1, n + gamma + half);
  float s = 0.f;
  for (int m = lo; m <= hi; ++m) s += e[m];
  fin[(int64_t)g * pb.ld + n] = s / (float)w_s;
}

}  // namespace

int launch_smooth(const Prob& pb, const float* score, float* ema, float* fin, int32_t* aws_info,
                  double* aws_d, char* ws, const SmoothWs& lay, hipStream_t st) {
  unsigned long long* rowsum = (unsigned long long*)(ws + lay.rowsum);
  float* e = ema ? ema : (float*)(ws + lay.ema);
  const dim3 gl((pb.P + 255) / 256, pb.Hkv);
  RK_LAUNCH(ST_EMA, st, k_ema, gl, dim3(256), 0, st, pb, score, e);
  if (pb.adaptive)
    RK_LAUNCH(ST_ROWTOPK, st, k_row_topk_sum, dim3(pb.W, pb.Hkv), dim3(SEL_NT), 0, st, pb, score, rowsum);
  RK_LAUNCH(ST_BOX, st, k_box, gl, dim3(256), 0, st, pb, e, rowsum, fin, aws_info, aws_d);
  return hip_status();
}

}  // namespace restkv
