// Pieces shared by the FP32 and the MFMA scoring paths: scratch pointers and the kernel
// that merges the key splits of the attention pass into per-query statistics.
#pragma once

#include "common.hpp"

namespace restkv {

struct ScorePtrs {
  float* part_m; float* part_mx; int* part_n; float* part_ref; float* part_l; float* part_z;
  float* rs_m; float* rs_l; float* rs_zz; int* rs_nstar; float* rs_istar; float* rs_u;
  float* vv;
  uint16_t* op;
};

inline ScorePtrs score_ptrs(char* ws, const ScoreWs& lay) {
  ScorePtrs p;
  p.part_m = (float*)(ws + lay.part_m); p.part_mx = (float*)(ws + lay.part_mx);
  p.part_n = (int*)(ws + lay.part_n);
  p.part_ref = (float*)(ws + lay.part_ref); p.part_l = (float*)(ws + lay.part_l);
  p.part_z = (float*)(ws + lay.part_z);
  p.rs_m = (float*)(ws + lay.rs_m); p.rs_l = (float*)(ws + lay.rs_l); p.rs_zz = (float*)(ws + lay.rs_zz);
  p.rs_nstar = (int*)(ws + lay.rs_nstar); p.rs_istar = (float*)(ws + lay.rs_istar);
  p.rs_u = (float*)(ws + lay.rs_u); p.vv = (float*)(ws + lay.vv);
  p.op = (uint16_t*)(ws + lay.op);
  return p;
}

// Per split s and query row the attention pass leaves (all logits in log2 units, scaled):
//   part_m    largest logit seen, -inf if the split saw no key
//   part_mx   logit of the key the split kept OUT of its sums (valid if part_n >= 0)
//   part_n    index of that key, or -1
//   part_ref  reference the sums are relative to
//   part_l    sum over the included keys of 2^(logit - ref)
//   part_z    sum over the included keys of 2^(logit - ref) * v
// A split keeps a key out when, on arrival, it is the largest so far and holds more than half
// of the mass seen so far (always true for a key that ends with more than half of the total).
// part_ref never follows a kept-out key, only keys that are part of the sums (on the matrix-core
// path: exactly the logit of a key that was heavy among the others when it arrived, so that its
// bf16 weight is exact).
// The merge keeps out the excluded key that is the overall maximum (if any) and folds every
// other excluded key back in.  With a key kept out ("champion", weight A* = 1/l):
//   l = 1 + l_rest, z = (v* + z_rest)/l, u = z M_h, zz = u.z, and the champion's indicator
//   in its leave-one-out form I* = A* ||(z_rest/l_rest - v*) W_O||  (Eq. ori with Eq. relation;
//   equals Eq. rec_ei).  Without one, l and z are the plain softmax sums relative to the maximum.
constexpr int CMB_RQ = 4;    // query rows of one head per workgroup of the merge kernel

// Statistics of a caller's own attention kernel as ONE split of the attention pass: the log-sum-exp
// of a row (natural log) is both the reference and the "largest logit", the sum of weights is 1, no
// key is kept out; the caller's attention output [Hq*W, d] then serves as part_z unchanged.
// grid (ceil(rows/256)), 256 threads.  (A template only so that the header can hold it.)
template <int UNUSED>
__global__ __launch_bounds__(256) void k_stats_fill(int rows, const float* __restrict__ lse,
                                                    float* __restrict__ part_m, float* __restrict__ part_mx,
                                                    int* __restrict__ part_n, float* __restrict__ part_ref,
                                                    float* __restrict__ part_l) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  const float m2 = lse[r] * 1.4426950408889634f;
  part_m[r] = m2; part_ref[r] = m2; part_mx[r] = 0.f; part_n[r] = -1; part_l[r] = 1.f;
}

// Merge of the key splits and the per-row quantities of the score pass.
// grid (ceil(W / CMB_RQ), Hq), CMB_RQ * D threads.  For the merge a thread is (row r of the
// group, column c); the per-split scalars of a row are fetched by one thread each and shared
// through LDS.  For u = z M_h (and y = x M_h) a thread is (part p = r of the Gram matrix's rows,
// column c): it holds its D / CMB_RQ Gram entries in registers (loaded first, their latency
// hides behind the merge; every entry is needed by exactly one thread, so the matrix never
// touches LDS) and works on all CMB_RQ rows at once, whose z and x it reads as LDS broadcasts;
// the partial sums of the parts meet in LDS.
template <typename T, int D>
__global__ __launch_bounds__(CMB_RQ * D, 4) void k_attn_combine(Prob pb, const T* __restrict__ v, int S,
                                                             const float* __restrict__ gram,
                                                             const float* __restrict__ part_m,
                                                             const float* __restrict__ part_mx,
                                                             const int* __restrict__ part_n,
                                                             const float* __restrict__ part_ref,
                                                             const float* __restrict__ part_l,
                                                             const float* __restrict__ part_z,
                                                             float* __restrict__ rs_m, float* __restrict__ rs_l,
                                                             float* __restrict__ rs_zz, int* __restrict__ rs_nstar,
                                                             float* __restrict__ rs_istar,
                                                             float* __restrict__ rs_u,
                                                             const T* __restrict__ q, uint16_t* __restrict__ op,
                                                             int log2gp, int nwb, int ngrp) {
  constexpr int NWV = D / 64, SMAX = 64;     // wavefronts per row; capacity of the split dimension
  constexpr int AP = D / CMB_RQ;             // Gram rows per thread
  static_assert(CMB_RQ == 4, "z and x of the group's rows travel as one float4 each");
  __shared__ __attribute__((aligned(16))) float zx[D][2 * CMB_RQ];     // [a][z of the rows | x of the rows]
  __shared__ float up[CMB_RQ][2][CMB_RQ][D];                           // [part][u | y][row][c]
  __shared__ float red[CMB_RQ][NWV][2];
  __shared__ float s_m[CMB_RQ][2], s_mx[CMB_RQ][SMAX], s_l[CMB_RQ][SMAX];
  __shared__ int s_n[CMB_RQ][SMAX + 1];      // [SMAX]: the split that holds the champion, or -1
  __shared__ float s_w[CMB_RQ][SMAX];
  const int h = blockIdx.y, g = h / pb.G;
  const int r = threadIdx.x / D, c = threadIdx.x % D;
  const T* vg = v + (int64_t)g * pb.kv_sh;
  float mreg[AP];
  if (gram) {
    const float* Mh = gram + (int64_t)h * D * D + (int64_t)(r * AP) * D + c;
#pragma unroll
    for (int j = 0; j < AP; ++j) mreg[j] = Mh[j * D];
  }
  // A workgroup walks ngrp groups of CMB_RQ rows with the one set of Gram registers.
  for (int grp = 0; grp < ngrp; ++grp) {
  const int i = (blockIdx.x * ngrp + grp) * CMB_RQ + r;
  if ((blockIdx.x * ngrp + grp) * CMB_RQ >= pb.W) break;      // workgroup-uniform
  const bool live = i < pb.W;
  const int row = h * pb.W + (live ? i : 0);
  const int64_t o = (int64_t)row * S;
  // Per-split scalars: thread c < S of the row's first wavefront owns split c (S <= 64).
  float pm = -INFINITY, pmx = 0.f, pref = 0.f, pl = 0.f;
  int pn = -1;
  if (c < S) {
    pm = part_m[o + c];
    pmx = part_mx[o + c];
    pn = part_n[o + c];
    pref = part_ref[o + c];
    pl = part_l[o + c];
  }
  T qv = T();                    // needed at the very end: its latency hides behind everything else
  if (op) qv = q[(int64_t)h * pb.q_sh + (int64_t)(live ? i : 0) * pb.q_st + c];
  if (c < 64) {
    float M0 = pm;
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) M0 = fmaxf(M0, __shfl_xor(M0, sh, 64));
    // split whose kept-out key is the overall maximum: the earliest one (= lowest key)
    const unsigned long long cand = __ballot(pn >= 0 && pmx == M0);
    const int ss = cand ? __builtin_ctzll(cand) : -1;
    // a split adds to the merged sums if it saw a key and its own sums are not empty; its
    // kept-out key joins them unless it is the overall maximum
    const bool has = pm != -INFINITY && pl > 0.f;
    const bool joins = pm != -INFINITY && pn >= 0 && c != ss;
    // The merged sums are relative to R, the largest logit that is part of them (reference of a
    // split, logit of a joining key), NOT to the overall maximum M0: a kept-out key may be any
    // distance above the rest without the rest's sums underflowing.
    float R = has ? pref : -INFINITY;
    if (joins) R = fmaxf(R, pmx);
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) R = fmaxf(R, __shfl_xor(R, sh, 64));
    s_w[r][c] = has ? exp2f(pref - R) : 0.f;
    s_l[r][c] = has ? pl : 0.f;                    // an empty split's sums may hold anything
    s_mx[r][c] = joins ? exp2f(pmx - R) : 0.f;
    s_n[r][c] = pn;
    if (c == 0) { s_m[r][0] = M0; s_m[r][1] = R == -INFINITY ? 0.f : exp2f(R - M0); s_n[r][SMAX] = ss; }
  }
  __syncthreads();
  const float M = s_m[r][0];
  const int sstar = s_n[r][SMAX];
  const int nstar = sstar >= 0 ? s_n[r][sstar] : -1;

  float lrest = 0.f, zr = 0.f;
  const float* pz = part_z + o * D + c;
  for (int s = 0; s < S; s += 8) {           // sixteen independent loads in flight
    float t[8], tv[8], wk[8], wv[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      const int sk = min(s + k, S - 1);
      const bool in = s + k < S;
      wk[k] = in ? s_w[r][sk] : 0.f;
      wv[k] = in ? s_mx[r][sk] : 0.f;
      t[k] = pz[(int64_t)sk * D];
      // value row of the kept-out key, fetched unconditionally (row 0 when there is none)
      tv[k] = to_float(vg[(int64_t)(wv[k] != 0.f ? s_n[r][sk] : 0) * pb.kv_st + c]);
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      zr = fmaf(wk[k], wk[k] != 0.f ? t[k] : 0.f, zr);
      lrest = fmaf(wk[k], s + k < S ? s_l[r][min(s + k, S - 1)] : 0.f, lrest);
      zr = fmaf(wv[k], tv[k], zr);
      lrest += wv[k];
    }
  }
  // rest -> units of the overall maximum (0 when the rest is below FP32 range next to the kept-out key)
  const float fr = s_m[r][1];
  float l, z, x;
  if (nstar >= 0) {
    const float vstar = to_float(vg[(int64_t)nstar * pb.kv_st + c]);
    l = 1.f + lrest * fr;
    z = (vstar + zr * fr) / l;
    x = lrest > 0.f ? zr / lrest - vstar : 0.f;   // z_without_champion - v_champion
  } else {
    l = lrest * fr;
    z = zr / lrest;
    x = 0.f;
  }
  float u = z, y = x;
  if (pb.ind != 0) {
    // attention-weight and value-norm indicators: no output term (u = 0, zz = 0), no key is
    // evaluated by the leave-one-out form; the score pass then sees sqrt(vv) with vv = 1 or ||v||^2
    u = 0.f; y = 0.f;
  } else if (gram) {
    zx[c][r] = z;
    zx[c][CMB_RQ + r] = x;
    __syncthreads();
    float ua[CMB_RQ], ya[CMB_RQ];
#pragma unroll
    for (int k = 0; k < CMB_RQ; ++k) { ua[k] = 0.f; ya[k] = 0.f; }
#pragma unroll
    for (int j = 0; j < AP; ++j) {
      const float4 z4 = *(const float4*)&zx[r * AP + j][0];
      const float4 x4 = *(const float4*)&zx[r * AP + j][CMB_RQ];
      ua[0] = fmaf(z4.x, mreg[j], ua[0]); ua[1] = fmaf(z4.y, mreg[j], ua[1]);
      ua[2] = fmaf(z4.z, mreg[j], ua[2]); ua[3] = fmaf(z4.w, mreg[j], ua[3]);
      ya[0] = fmaf(x4.x, mreg[j], ya[0]); ya[1] = fmaf(x4.y, mreg[j], ya[1]);
      ya[2] = fmaf(x4.z, mreg[j], ya[2]); ya[3] = fmaf(x4.w, mreg[j], ya[3]);
    }
#pragma unroll
    for (int k = 0; k < CMB_RQ; ++k) { up[r][0][k][c] = ua[k]; up[r][1][k][c] = ya[k]; }
    __syncthreads();
    u = (up[0][0][r][c] + up[1][0][r][c]) + (up[2][0][r][c] + up[3][0][r][c]);
    y = (up[0][1][r][c] + up[1][1][r][c]) + (up[2][1][r][c] + up[3][1][r][c]);
  }
  // zz = u.z and |x|_M^2 = y.x of the row: wavefront sums, then across the row's wavefronts
  float s0 = u * z, s1 = y * x;
#pragma unroll
  for (int sh = 32; sh >= 1; sh >>= 1) { s0 += __shfl_xor(s0, sh, 64); s1 += __shfl_xor(s1, sh, 64); }
  if ((c & 63) == 0) { red[r][c >> 6][0] = s0; red[r][c >> 6][1] = s1; }
  __syncthreads();
  if (live) {
  float zz = 0.f, qx = 0.f;
#pragma unroll
  for (int wv = 0; wv < NWV; ++wv) { zz += red[r][wv][0]; qx += red[r][wv][1]; }
  rs_u[(int64_t)row * D + c] = u;
  if (op) {
    // q, and u split into bf16 high and low parts, in the order the score pass feeds them to the
    // matrix cores: [which][32-row block][d/16][lane half][local row][8], local row =
    // position * Gp + head, so that a wavefront fetches each operand register as one 1 KiB run
    const int head = h - g * pb.G;
    const int log2iw = 5 - log2gp;
    const int wb = i >> log2iw, m_ = ((i & ((1 << log2iw) - 1)) << log2gp) + head;
    const int64_t nb = (int64_t)pb.Hkv * nwb;
    const int64_t inner = ((((int64_t)(g * nwb + wb) * (D / 16) + (c >> 4)) * 2 + ((c >> 3) & 1)) * 32 + m_) * 8 + (c & 7);
    const int64_t plane = nb * (D / 16) * 2 * 32 * 8;
    const uint32_t ub = __float_as_uint(u);
    uint32_t hi = ub + 0x7FFFu + ((ub >> 16) & 1u);          // round to nearest even (u is finite)
    hi &= 0xFFFF0000u;
    const uint32_t lb = __float_as_uint(u - __uint_as_float(hi));
    const uint32_t lo = (lb + 0x7FFFu + ((lb >> 16) & 1u)) >> 16;
    uint16_t qb;
    __builtin_memcpy(&qb, &qv, 2);
    op[inner] = qb;
    op[plane + inner] = (uint16_t)(hi >> 16);
    op[2 * plane + inner] = (uint16_t)lo;
  }
  if (c == 0) {
    rs_m[row] = M;
    rs_l[row] = l;
    rs_zz[row] = zz;
    rs_nstar[row] = pb.ind != 0 ? -1 : nstar;
    rs_istar[row] = sqrtf(fmaxf(qx, 0.f)) / l;      // A* ||(z_rest - v*) W_O||,  A* = 1/l
  }
  }
  __syncthreads();                           // the next group reuses the LDS scalars and sums
  }
}

// launch configuration of k_attn_combine
// groups of CMB_RQ rows per workgroup: one when that already gives plenty of workgroups, more
// (fewer re-reads of the Gram matrix) when there are very many heads
inline int combine_groups(const Prob& pb) {
  const int64_t wgs = (int64_t)pb.Hq * ((pb.W + CMB_RQ - 1) / CMB_RQ);
  int ngrp = (int)(wgs / 2048);
  if (ngrp < 1) ngrp = 1;
  const int all = (pb.W + CMB_RQ - 1) / CMB_RQ;
  return ngrp < all ? ngrp : all;
}
inline dim3 combine_grid(const Prob& pb) {
  const int per = CMB_RQ * combine_groups(pb);
  return dim3((pb.W + per - 1) / per, pb.Hq);
}
template <int D>
inline dim3 combine_block() { return dim3(CMB_RQ * D); }

}  // namespace restkv
