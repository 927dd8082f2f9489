// Shared host/device declarations of the ReST-KV eviction library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "restkv.h"

namespace restkv {

// Resolved problem description: parameter block with defaults filled in.
struct Prob {
  int Hq, Hkv, G, d, L, W, P, B, R;   // R = G*W rows (queries) per KV head
  int dtype, causal, base_k, adaptive;
  int ind, gmax, tmode, pmax;          // ablation variant: indicator 0..2, group maximum, temporal 0..2, max pooling
  float scale, alpha, beta;
  int64_t q_sh, q_st, kv_sh, kv_st, ld;
  const int32_t* hb;   // optional per-KV-head budgets (device, [Hkv]); NULL: B for every head
  // optional attention output [Hq,W,d] f32 and log-sum-exp [Hq,W] (natural log) of the window
  // queries from the caller's own attention kernel; NULL: the library's attention pass runs
  const float* ext_out;
  const float* ext_lse;
};

// Fills `out`; returns RESTKV_OK or the error the block deserves.
int resolve(const restkv_params* p, Prob* out);

// ---- scratch layout ---------------------------------------------------------
// All offsets are in bytes from the 256-byte aligned workspace base.
struct ScoreWs {
  int S_simple;          // key splits of the attention pass, FP32 path
  int S_max;             // capacity of the split dimension
  int ldv;               // row stride of vv (P rounded up to 4)
  size_t part_m, part_mx, part_n, part_ref, part_l, part_z;   // [Hq*W*S] , part_z [Hq*W*S*d] f32
  size_t rs_m, rs_l, rs_zz, rs_nstar, rs_istar;   // [Hq*W]
  size_t rs_u;           // [Hq*W*d] f32   u = z M_h
  size_t vv;             // [Hq*ldv] f32   v_n M_h v_n^T
  size_t op;             // [3, Hkv*nwb, d/16, 2, 32, 8] bf16: q, u_hi, u_lo in MFMA operand order
  int nwb;               // blocks of 32 (padded) query rows per KV head in `op`; 0 if unused
  size_t bytes;
};
struct SmoothWs {
  size_t rowsum;         // [Hkv*W] u64 index sums of the per-query top-B
  size_t ema;            // [Hkv*ld] f32 (used when the caller passes ema == NULL)
  size_t thr;            // [Hkv*W] float2 bracket {lo, hi} of each row's top-B threshold
  size_t cnt_hi, sum_hi;          // [Hkv*W] u32 / u64: entries above the bracket, their position sum
  size_t cmask;                   // [Hkv*W, ceil(P/1024), 64] u16: entries inside the bracket, one bit
                                  // string per lane of the scan
  size_t bytes;
};
// extra scratch of the fused score + smoothing call (after the two layouts above)
struct FuseWs {
  int ns;                // sampled prefix keys per row (multiple of 64)
  int nchunks;           // key chunks = workgroups along the keys of the score pass
  int caps;              // capacity of one (row, chunk) candidate slice
  size_t smp;            // [Hkv*W, ns] f32 scores of the sampled keys
  size_t scnt;           // [Hkv*W, nchunks] u32 slice fill counts
  size_t sval, sidx;     // [Hkv*W, nchunks, caps] f32 / i32 candidate slices
  size_t bytes;
};
ScoreWs score_ws(const Prob& pb);
SmoothWs smooth_ws(const Prob& pb);
FuseWs fuse_ws(const Prob& pb);

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// ---- launchers (each returns a RESTKV_* code) ---------------------------------
int launch_gram(const Prob& pb, const float* w_o, int64_t d_model, float* gram, hipStream_t st);
int launch_score_simple(const Prob& pb, const void* q, const void* k, const void* v,
                        const float* gram, float* score, char* ws, const ScoreWs& lay,
                        hipStream_t st);
bool mfma_eligible(const Prob& pb, const void* q, const void* k, const void* v);
int launch_score_mfma(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
                      float* score, char* ws, const ScoreWs& lay, hipStream_t st);
int launch_smooth(const Prob& pb, const float* score, float* ema, float* fin, int32_t* aws_info,
                  double* aws_d, char* ws, const SmoothWs& lay, hipStream_t st);
// Fused score + smoothing (matrix-core path only).  fused_eligible() says whether the shape
// qualifies; score_pass_chunks() is the number of key chunks the score pass will use.
struct FusedPtrs {
  float* smp; int ns;
  float2* thr; uint32_t* cnt_hi; unsigned long long* sum_hi;
  uint32_t* scnt; float* sval; int* sidx; int caps;
  float* ema;
};
bool fused_eligible(const Prob& pb, const void* q, const void* k, const void* v);
int score_pass_chunks(const Prob& pb);
int launch_score_fused(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
                       float* score, char* ws, const ScoreWs& lay, const FusedPtrs& fp, hipStream_t st);
int launch_bracket_samples(const Prob& pb, const float* smp, int ns, float2* thr, uint32_t* cnt_hi,
                           unsigned long long* sum_hi, hipStream_t st);
int launch_smooth_fused_tail(const Prob& pb, const float* score, const float* ema, float* fin,
                             int32_t* aws_info, double* aws_d, char* ws, const SmoothWs& lay,
                             const FusedPtrs& fp, int nchunks, hipStream_t st);
size_t select_ws_bytes(const Prob& pb);
int launch_select(const Prob& pb, const float* fin, int32_t* idx, char* ws, hipStream_t st);
// the same with the library's own static scratch (RESTKV_EWORKSPACE beyond its capacity)
size_t select_static_capacity();
int launch_select_static(const Prob& pb, const float* fin, int32_t* idx, hipStream_t st);
int launch_compact(const Prob& pb, const void* k, const void* v, const int32_t* idx, void* k_out,
                   void* v_out, hipStream_t st);

// Brackets one kernel launch with events when timing is enabled (see timing.hip).
struct StageTimer {
  StageTimer(int stage, hipStream_t st);
  ~StageTimer();
  hipStream_t st_;
  long slot_;
};
enum Stage { ST_GRAM = 0, ST_ATTN, ST_COMBINE, ST_VV, ST_SCORE, ST_EMA, ST_ROWTOPK, ST_BOX, ST_SELECT,
             ST_COMPACT };

#define RK_LAUNCH(stage, st, ...)            \
  do {                                       \
    ::restkv::StageTimer tm_((stage), (st)); \
    hipLaunchKernelGGL(__VA_ARGS__);         \
  } while (0)

inline int hip_status() { return hipGetLastError() == hipSuccess ? RESTKV_OK : RESTKV_EHIP; }

// ---- device helpers -----------------------------------------------------------
struct bf16_t { uint16_t x; };

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16_t v) { return __uint_as_float(((uint32_t)v.x) << 16); }

// Sum over the 64 lanes of a wavefront, result in every lane: rotations inside the 16-lane
// DPP rows, then the two row swaps of gfx950 (no LDS traffic).
__device__ __forceinline__ uint32_t wave_sum(uint32_t x) {
  x += __builtin_amdgcn_update_dpp(0u, x, 0x121, 0xF, 0xF, false);   // row_ror:1
  x += __builtin_amdgcn_update_dpp(0u, x, 0x122, 0xF, 0xF, false);   // row_ror:2
  x += __builtin_amdgcn_update_dpp(0u, x, 0x124, 0xF, 0xF, false);   // row_ror:4
  x += __builtin_amdgcn_update_dpp(0u, x, 0x128, 0xF, 0xF, false);   // row_ror:8
  auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  x = r[0] + r[1];
  r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return r[0] + r[1];
}

// Bit strings of comparison outcomes: for each of two elements x0, x1 (in this order) and each of
// two wave-uniform thresholds, bits = 2 bits + (x > t): one compare, whose outcome an
// add-with-carry shifts in.  Sixteen elements leave element k of a lane at bit 15 - k.
// gfx950 wants two other instructions between a vector instruction that writes a scalar register
// (a compare's outcome) and a vector instruction that reads it: the four compares go first, each
// into its own scalar pair, then the four adds.
__device__ __forceinline__ void shift_in_gt_2x2(uint32_t& hb, uint32_t& lb, float x0, float x1, float thi,
                                                float tlo) {
  unsigned long long c0, c1, c2;
  asm("v_cmp_lt_f32_e64 %2, %7, %5\n\t"
      "v_cmp_lt_f32_e64 %3, %8, %5\n\t"
      "v_cmp_lt_f32_e64 %4, %7, %6\n\t"
      "v_cmp_lt_f32_e32 vcc, %8, %6\n\t"
      "v_addc_co_u32_e64 %0, %2, %0, %0, %2\n\t"
      "v_addc_co_u32_e64 %1, %3, %1, %1, %3\n\t"
      "v_addc_co_u32_e64 %0, %4, %0, %0, %4\n\t"
      "v_addc_co_u32_e32 %1, vcc, %1, %1, vcc"
      : "+v"(hb), "+v"(lb), "=&s"(c0), "=&s"(c1), "=&s"(c2)
      : "v"(x0), "v"(x1), "s"(thi), "s"(tlo)
      : "vcc");
}
// The same distance between the vector instruction that made the thresholds wave-uniform
// (a readfirstlane) and the first compare that reads them.
__device__ __forceinline__ void settle_scalars(float& a, float& b) { asm volatile("s_nop 1" : "+s"(a), "+s"(b)); }

// Budget of KV head g: its own entry of the optional per-head array, held inside (W, B], else B.
__device__ __forceinline__ int head_budget(const Prob& pb, int g) {
  if (!pb.hb) return pb.B;
  return min(max(pb.hb[g], pb.W + 1), pb.B);
}

// Order-preserving map float -> uint32 (larger float <=> larger key; -0 < +0).
__device__ __forceinline__ uint32_t float_key(float f) {
  const uint32_t b = __float_as_uint(f);
  return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

}  // namespace restkv
