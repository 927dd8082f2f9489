// Per-head selection (Sec. 3.3, Eq. topk): top-(B-W) prefix positions in ascending order,
// window positions appended.
#include "rowselect.hpp"

namespace restkv {

namespace {

// grid (Hkv), SEL_NT threads
__global__ __launch_bounds__(SEL_NT) void k_select(Prob pb, const float* __restrict__ fin,
                                                   int32_t* __restrict__ idx) {
  __shared__ SelectSmem sm;
  __shared__ CountSmem cs;
  __shared__ uint32_t buf[SEL_NS];
  const int g = blockIdx.x;
  const float* row = fin + (int64_t)g * pb.ld;
  const int bp = pb.B - pb.W;
  int32_t* out = idx + (int64_t)g * pb.B;
  uint32_t tau, n_gt, k_eq;
  block_kth_key_fast(row, pb.P, bp, sm, cs, buf, tau, n_gt, k_eq);
  block_visit_topk(row, pb.P, tau, k_eq, sm, [&](int x, uint32_t rank) {
    if (rank < (uint32_t)bp) out[rank] = x;
  });
  for (int j = threadIdx.x; j < pb.W; j += SEL_NT) out[bp + j] = pb.P + j;
}

}  // namespace

int launch_select(const Prob& pb, const float* fin, int32_t* idx, hipStream_t st) {
  RK_LAUNCH(ST_SELECT, st, k_select, dim3(pb.Hkv), dim3(SEL_NT), 0, st, pb, fin, idx);
  return hip_status();
}

}  // namespace restkv
