// Gather of the kept K/V rows into the budgeted cache (Sec. 3.3, Eq. topk).
#include "common.hpp"

namespace restkv {

namespace {

// One 16-byte chunk per thread; a row of d elements is `cpr` chunks.  grid (ceil(B*cpr/256), Hkv, 2).
__global__ __launch_bounds__(256) void k_compact(Prob pb, const uint4* __restrict__ k,
                                                 const uint4* __restrict__ v,
                                                 const int32_t* __restrict__ idx,
                                                 uint4* __restrict__ k_out, uint4* __restrict__ v_out,
                                                 int cpr, int64_t sh16, int64_t st16) {
  const int g = blockIdx.y;
  const int x = blockIdx.x * 256 + threadIdx.x;
  if (x >= pb.B * cpr) return;
  const int j = x / cpr, c = x % cpr;
  const int n = idx[(int64_t)g * pb.B + j];
  const bool ok = n >= 0 && n < pb.L;
  const uint4* src = blockIdx.z ? v : k;
  uint4* dst = blockIdx.z ? v_out : k_out;
  uint4 val = make_uint4(0, 0, 0, 0);
  if (ok) val = src[(int64_t)g * sh16 + (int64_t)n * st16 + c];
  dst[((int64_t)g * pb.B + j) * cpr + c] = val;
}

// element-wise fallback for strides that are not multiples of 16 bytes
template <typename T>
__global__ __launch_bounds__(256) void k_compact_elem(Prob pb, const T* __restrict__ k,
                                                      const T* __restrict__ v,
                                                      const int32_t* __restrict__ idx,
                                                      T* __restrict__ k_out, T* __restrict__ v_out) {
  const int g = blockIdx.y;
  const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (x >= (int64_t)pb.B * pb.d) return;
  const int j = (int)(x / pb.d), c = (int)(x % pb.d);
  const int n = idx[(int64_t)g * pb.B + j];
  const bool ok = n >= 0 && n < pb.L;
  const T* src = blockIdx.z ? v : k;
  T* dst = blockIdx.z ? v_out : k_out;
  T val{};
  if (ok) val = src[(int64_t)g * pb.kv_sh + (int64_t)n * pb.kv_st + c];
  dst[((int64_t)g * pb.B + j) * pb.d + c] = val;
}

}  // namespace

int launch_compact(const Prob& pb, const void* k, const void* v, const int32_t* idx, void* k_out,
                   void* v_out, hipStream_t st) {
  const int esz = pb.dtype == RESTKV_F32 ? 4 : 2;
  const int per16 = 16 / esz;
  const bool vec = (pb.kv_sh % per16 == 0) && (pb.kv_st % per16 == 0) &&
                   (((uintptr_t)k | (uintptr_t)v | (uintptr_t)k_out | (uintptr_t)v_out) & 15u) == 0;
  if (vec) {
    const int cpr = pb.d / per16;
    RK_LAUNCH(ST_COMPACT, st, k_compact, dim3((pb.B * cpr + 255) / 256, pb.Hkv, 2), dim3(256), 0, st, pb,
                       (const uint4*)k, (const uint4*)v, idx, (uint4*)k_out, (uint4*)v_out, cpr,
                       pb.kv_sh / per16, pb.kv_st / per16);
  } else if (esz == 4) {
    RK_LAUNCH(ST_COMPACT, st, k_compact_elem<float>, dim3(((int64_t)pb.B * pb.d + 255) / 256, pb.Hkv, 2),
                       dim3(256), 0, st, pb, (const float*)k, (const float*)v, idx, (float*)k_out,
                       (float*)v_out);
  } else {
    RK_LAUNCH(ST_COMPACT, st, k_compact_elem<uint16_t>, dim3(((int64_t)pb.B * pb.d + 255) / 256, pb.Hkv, 2),
                       dim3(256), 0, st, pb, (const uint16_t*)k, (const uint16_t*)v, idx,
                       (uint16_t*)k_out, (uint16_t*)v_out);
  }
  return hip_status();
}

}  // namespace restkv
