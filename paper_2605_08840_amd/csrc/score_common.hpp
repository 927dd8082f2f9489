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
// A split keeps a key out when, on arrival, it is the largest so far and holds more than 1/9
// of the mass seen so far (always true for a key that ends with more than 1/9 of the total).
// The merge keeps out the excluded key that is the overall maximum (if any) and folds every
// other excluded key back in.  With a key kept out ("champion", weight A* = 1/l):
//   l = 1 + l_rest, z = (v* + z_rest)/l, u = z M_h, zz = u.z, and the champion's indicator
//   in its leave-one-out form I* = A* ||(z_rest/l_rest - v*) W_O||  (Eq. ori with Eq. relation;
//   equals Eq. rec_ei).  Without one, l and z are the plain softmax sums relative to the maximum.
__device__ __forceinline__ float block_sum(float x, float* red, int nthreads) {
  // wavefront reduce, then across wavefronts through LDS
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = x;
  __syncthreads();
  float tot = 0.f;
  for (int j = 0; j < (nthreads + 63) / 64; ++j) tot += red[j];
  return tot;
}

// one block of D threads per query row (global row = h*W + i)
template <typename T, int D>
__global__ __launch_bounds__(D) void k_attn_combine(Prob pb, const T* __restrict__ v, int S,
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
                                                    int log2gp, int nwb) {
  __shared__ float zs[D];
  __shared__ float xs[D];
  __shared__ float red[4];
  const int row = blockIdx.x;               // h*W + i  ==  g*R + r
  const int h = row / pb.W, g = h / pb.G;
  const int c = threadIdx.x;
  const T* vg = v + (int64_t)g * pb.kv_sh;
  const int64_t o = (int64_t)row * S;

  float M = -INFINITY;
  for (int s = 0; s < S; ++s) M = fmaxf(M, part_m[o + s]);
  int sstar = -1;                            // split whose kept-out key is the overall maximum
  for (int s = 0; s < S; ++s)
    if (sstar < 0 && part_n[o + s] >= 0 && part_mx[o + s] == M) sstar = s;   // earliest split = lowest key
  const int nstar = sstar >= 0 ? part_n[o + sstar] : -1;
  float lrest = 0.f, zr = 0.f;
  for (int s = 0; s < S; ++s) {
    const float ms = part_m[o + s];
    if (ms == -INFINITY) continue;
    const float wr = exp2f(part_ref[o + s] - M);   // the split's sums are relative to its reference
    lrest += wr * part_l[o + s];
    zr += wr * part_z[(o + s) * D + c];
    if (s != sstar && part_n[o + s] >= 0) {        // a kept-out key that is not the maximum joins the rest
      const float w = exp2f(part_mx[o + s] - M);
      lrest += w;
      zr += w * to_float(vg[(int64_t)part_n[o + s] * pb.kv_st + c]);
    }
  }
  float l, z, x;
  if (nstar >= 0) {
    const float vstar = to_float(vg[(int64_t)nstar * pb.kv_st + c]);
    l = 1.f + lrest;
    z = (vstar + zr) / l;
    x = lrest > 0.f ? zr / lrest - vstar : 0.f;   // z_without_champion - v_champion
  } else {
    l = lrest;
    z = zr / l;
    x = 0.f;
  }
  zs[c] = z;
  xs[c] = x;
  __syncthreads();
  float u = z, y = x;
  if (gram) {
    const float* Mh = gram + (int64_t)h * D * D;
    u = 0.f; y = 0.f;
    for (int a = 0; a < D; ++a) {
      const float mv = Mh[a * D + c];
      u = fmaf(zs[a], mv, u);
      y = fmaf(xs[a], mv, y);
    }
  }
  const float zz = block_sum(u * z, red, D);
  const float qx = block_sum(y * x, red, D);
  rs_u[(int64_t)row * D + c] = u;
  if (op) {
    // q, and u split into bf16 high and low parts, in the order the score pass feeds them to the
    // matrix cores: [which][32-row block][d/16][lane half][local row][8], local row =
    // position * Gp + head, so that a wavefront fetches each operand register as one 1 KiB run
    const int i = row - h * pb.W, head = h - g * pb.G;
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
    const T qv = q[(int64_t)h * pb.q_sh + (int64_t)i * pb.q_st + c];
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
    rs_nstar[row] = nstar;
    rs_istar[row] = sqrtf(fmaxf(qx, 0.f)) / l;      // A* ||(z_rest - v*) W_O||,  A* = 1/l
  }
}


}  // namespace restkv
