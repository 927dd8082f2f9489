// Reconstruction indicator, plain-FP32 kernels (vector ALU, LDS tiles).
//
// This is the path for float32 inputs (the small configuration) and the
// arithmetic reference shape of the MFMA path: the same four stages, the same
// scratch layout, every product in FP32.
//
//   attn_partial : per key split, online softmax over the visible keys of every
//                  window query; the key with the largest logit so far (the
//                  "champion") is kept OUT of the running sums, so that the sums
//                  hold the attention of all the other keys relative to it.
//   attn_combine : merges the splits; z, u = z M_h, zz = u.z, and the champion's
//                  own indicator from its leave-one-out form (Eq. ori, Eq. relation).
//   vv           : v_n M_h v_n^T for every prefix token and query head.
//   score        : A/(1-A) * sqrt(zz - 2 u.v_n + vv) for all other tokens (Eq. rec_ei),
//                  mean over the query heads of the group.
#include "score_common.hpp"

namespace restkv {

namespace {

constexpr int RB = 16;      // rows (queries) per block
constexpr int TN = 32;      // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;

// max / argmax (lowest key on ties) across the 16 lanes that share a row
__device__ __forceinline__ void argmax16(float& v, int& i) {
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) {
    const float ov = __shfl_xor(v, o, 16);
    const int oi = __shfl_xor(i, o, 16);
    if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
  }
}
__device__ __forceinline__ float sum16(float v) {
#pragma unroll
  for (int o = 8; o >= 1; o >>= 1) v += __shfl_xor(v, o, 16);
  return v;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_partial(Prob pb, const T* __restrict__ q,
                                                      const T* __restrict__ k,
                                                      const T* __restrict__ v, int S,
                                                      float* __restrict__ part_m,
                                                      float* __restrict__ part_mx,
                                                      int* __restrict__ part_n,
                                                      float* __restrict__ part_ref,
                                                      float* __restrict__ part_l,
                                                      float* __restrict__ part_z) {
  __shared__ float Qs[RB][D];
  __shared__ float Ks[TN][D + 1];
  __shared__ float Vs[TN][D];
  __shared__ float Ps[RB][TN];
  constexpr int NC = D / 16;          // value columns per thread

  const int s = blockIdx.x, g = blockIdx.z;
  const int t = threadIdx.x, rl = t >> 4, ln = t & 15;
  const int r = blockIdx.y * RB + rl;            // row inside the KV head
  const bool row_ok = r < pb.R;
  const int hl = row_ok ? r / pb.W : 0, i = row_ok ? r % pb.W : 0;
  const int nvis = pb.causal ? pb.P + i + 1 : pb.L;
  const T* kg = k + (int64_t)g * pb.kv_sh;
  const T* vg = v + (int64_t)g * pb.kv_sh;

  int kps = (pb.L + S - 1) / S;
  kps = (kps + TN - 1) / TN * TN;
  const int kbeg = s * kps;
  const int kend = min(pb.L, kbeg + kps);

  for (int x = t; x < RB * D; x += 256) {
    const int rr = x / D, c = x % D;
    const int rg = blockIdx.y * RB + rr;
    float val = 0.f;
    if (rg < pb.R) {
      const int h = g * pb.G + rg / pb.W;
      val = to_float(q[(int64_t)h * pb.q_sh + (int64_t)(rg % pb.W) * pb.q_st + c]);
    }
    Qs[rr][c] = val;
  }

  const float c2 = pb.scale * LOG2E;
  float m = -INFINITY, ref = -INFINITY, l = 0.f;
  int nstar = -1;
  float acc[NC];
#pragma unroll
  for (int j = 0; j < NC; ++j) acc[j] = 0.f;

  for (int k0 = kbeg; k0 < kend; k0 += TN) {
    __syncthreads();
    for (int x = t; x < TN * D; x += 256) {
      const int kk = x / D, c = x % D;
      const int n = k0 + kk;
      float kv_ = 0.f, vv_ = 0.f;
      if (n < kend) {
        kv_ = to_float(kg[(int64_t)n * pb.kv_st + c]);
        vv_ = to_float(vg[(int64_t)n * pb.kv_st + c]);
      }
      Ks[kk][c] = kv_;
      Vs[kk][c] = vv_;
    }
    __syncthreads();
    float sv[2];
    float tmax = -INFINITY;
    int tidx = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int kk = ln + 16 * j, n = k0 + kk;
      float dot = 0.f;
#pragma unroll 8
      for (int c = 0; c < D; ++c) dot = fmaf(Qs[rl][c], Ks[kk][c], dot);
      const bool vis = n < kend && n < nvis;
      sv[j] = vis ? dot * c2 : -INFINITY;
      if (vis && (sv[j] > tmax)) { tmax = sv[j]; tidx = n; }
    }
    argmax16(tmax, tidx);
    // The sums are relative to `ref`, the largest logit that is part of them; the champion stays
    // out of them and may be any distance above the rest.
    const bool newc = tmax > m;             // the row has a new champion in this tile
    const float mold = m;
    const int nold = nstar;
    if (newc) { m = tmax; nstar = tidx; }
    const bool joins = newc && nold >= 0;   // the previous champion joins the sums
    float tinc = -INFINITY;                 // largest logit joining the sums at this tile
#pragma unroll
    for (int j = 0; j < 2; ++j)
      if (k0 + ln + 16 * j != nstar) tinc = fmaxf(tinc, sv[j]);
#pragma unroll
    for (int o = 8; o >= 1; o >>= 1) tinc = fmaxf(tinc, __shfl_xor(tinc, o, 16));
    if (joins) tinc = fmaxf(tinc, mold);
    if (tinc > ref) {
      const float w = exp2f(ref - tinc);    // ref = -inf (empty sums) gives 0
      l *= w;
#pragma unroll
      for (int j = 0; j < NC; ++j) acc[j] *= w;
      ref = tinc;
    }
    if (joins) {
      const float w = exp2f(mold - ref);
      l += w;
#pragma unroll
      for (int j = 0; j < NC; ++j)
        acc[j] = fmaf(w, to_float(vg[(int64_t)nold * pb.kv_st + ln + 16 * j]), acc[j]);
    }
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int kk = ln + 16 * j, n = k0 + kk;
      const float pj = (n == nstar || sv[j] == -INFINITY) ? 0.f : exp2f(sv[j] - ref);
      Ps[rl][kk] = pj;
      psum += pj;
    }
    l += sum16(psum);
    __syncthreads();
#pragma unroll 4
    for (int kk = 0; kk < TN; ++kk) {
      const float pj = Ps[rl][kk];
#pragma unroll
      for (int j = 0; j < NC; ++j) acc[j] = fmaf(pj, Vs[kk][ln + 16 * j], acc[j]);
    }
  }
  if (row_ok) {
    const int64_t o = ((int64_t)g * pb.R + r) * S + s;
    if (ln == 0) { part_m[o] = m; part_mx[o] = m; part_n[o] = nstar; part_ref[o] = ref; part_l[o] = l; }
#pragma unroll
    for (int j = 0; j < NC; ++j) part_z[o * D + ln + 16 * j] = acc[j];
  }
  (void)hl;
}

// vv[h, n] = v_n M_h v_n^T ; grid (ceil(P/64), Hq), 256 threads
template <typename T, int D>
__global__ __launch_bounds__(256) void k_vv(Prob pb, const T* __restrict__ v,
                                            const float* __restrict__ gram, float* __restrict__ vv,
                                            int ldv) {
  __shared__ float Vs[64][D + 1];
  __shared__ float red[4][64];
  const int h = blockIdx.y, g = h / pb.G;
  const int n0 = blockIdx.x * 64;
  const int t = threadIdx.x, nl = t & 63, part = t >> 6;
  const T* vg = v + (int64_t)g * pb.kv_sh;
  for (int x = t; x < 64 * D; x += 256) {
    const int kk = x / D, c = x % D;
    const int n = n0 + kk;
    Vs[kk][c] = n < pb.P ? to_float(vg[(int64_t)n * pb.kv_st + c]) : 0.f;
  }
  __syncthreads();
  constexpr int CQ = D / 4;
  const int c0 = part * CQ;
  float acc = 0.f;
  if (gram) {
    const float* Mh = gram + (int64_t)h * D * D;
    float y[CQ];
#pragma unroll
    for (int j = 0; j < CQ; ++j) y[j] = 0.f;
    for (int a = 0; a < D; ++a) {
      const float va = Vs[nl][a];
      const float* mr = Mh + a * D + c0;
#pragma unroll
      for (int j = 0; j < CQ; ++j) y[j] = fmaf(va, mr[j], y[j]);
    }
#pragma unroll
    for (int j = 0; j < CQ; ++j) acc = fmaf(y[j], Vs[nl][c0 + j], acc);
  } else {
#pragma unroll
    for (int j = 0; j < CQ; ++j) acc = fmaf(Vs[nl][c0 + j], Vs[nl][c0 + j], acc);
  }
  red[part][nl] = acc;
  __syncthreads();
  if (part == 0 && n0 + nl < pb.P)
    vv[(int64_t)h * ldv + n0 + nl] = red[0][nl] + red[1][nl] + red[2][nl] + red[3][nl];
}

// grid (ceil(P/TN), Hkv), 256 threads
template <typename T, int D>
__global__ __launch_bounds__(256) void k_score(Prob pb, const T* __restrict__ q,
                                               const T* __restrict__ k, const T* __restrict__ v,
                                               const float* __restrict__ rs_m,
                                               const float* __restrict__ rs_l,
                                               const float* __restrict__ rs_zz,
                                               const int* __restrict__ rs_nstar,
                                               const float* __restrict__ rs_istar,
                                               const float* __restrict__ rs_u,
                                               const float* __restrict__ vv, int ldv,
                                               float* __restrict__ score) {
  __shared__ float Qs[RB][D];
  __shared__ float Us[RB][D];
  __shared__ float Ks[TN][D + 1];
  __shared__ float Vs[TN][D + 1];
  const int g = blockIdx.y, n0 = blockIdx.x * TN;
  const int t = threadIdx.x, rl = t >> 4, ln = t & 15;
  const T* kg = k + (int64_t)g * pb.kv_sh;
  const T* vg = v + (int64_t)g * pb.kv_sh;
  for (int x = t; x < TN * D; x += 256) {
    const int kk = x / D, c = x % D;
    const int n = n0 + kk;
    float kv_ = 0.f, vv_ = 0.f;
    if (n < pb.P) {
      kv_ = to_float(kg[(int64_t)n * pb.kv_st + c]);
      vv_ = to_float(vg[(int64_t)n * pb.kv_st + c]);
    }
    Ks[kk][c] = kv_;
    Vs[kk][c] = vv_;
  }
  const float c2 = pb.scale * LOG2E;
  const float invG = 1.0f / (float)pb.G;
  for (int i0 = 0; i0 < pb.W; i0 += RB) {
    const int i = i0 + rl;
    float out[2] = {0.f, 0.f};
    for (int hl = 0; hl < pb.G; ++hl) {
      const int h = g * pb.G + hl;
      __syncthreads();
      for (int x = t; x < RB * D; x += 256) {
        const int rr = x / D, c = x % D;
        const int ii = i0 + rr;
        float qv = 0.f, uv = 0.f;
        if (ii < pb.W) {
          qv = to_float(q[(int64_t)h * pb.q_sh + (int64_t)ii * pb.q_st + c]);
          uv = rs_u[((int64_t)h * pb.W + ii) * D + c];
        }
        Qs[rr][c] = qv;
        Us[rr][c] = uv;
      }
      __syncthreads();
      if (i < pb.W) {
        const int row = h * pb.W + i;
        const float m = rs_m[row], l = rs_l[row], zz = rs_zz[row], istar = rs_istar[row];
        const int nstar = rs_nstar[row];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const int kk = ln + 16 * j, n = n0 + kk;
          if (n >= pb.P) continue;
          float dot = 0.f, cx = 0.f;
#pragma unroll 8
          for (int c = 0; c < D; ++c) {
            dot = fmaf(Qs[rl][c], Ks[kk][c], dot);
            cx = fmaf(Us[rl][c], Vs[kk][c], cx);
          }
          const float e = exp2f(dot * c2 - m);
          const float vvn = vv[(int64_t)h * ldv + n];
          float val;
          if (pb.ind == 0) {
            const float dist2 = zz - 2.f * cx + vvn;
            val = e / (l - e) * sqrtf(fmaxf(dist2, 0.f));
            if (n == nstar) val = istar;
          } else {                             // attention weight, optionally times ||v_n|| (vv = ||v_n||^2 here)
            val = e / l;
            if (pb.ind == 2) val *= sqrtf(vvn);
          }
          out[j] = pb.gmax ? fmaxf(out[j], val) : out[j] + val;
        }
      }
    }
    if (i < pb.W) {
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int n = n0 + ln + 16 * j;
        if (n < pb.P) score[((int64_t)g * pb.W + i) * pb.ld + n] = pb.gmax ? out[j] : out[j] * invG;
      }
    }
  }
}

template <typename T, int D>
int run(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
        float* score, char* ws, const ScoreWs& lay, hipStream_t st) {
  const T* qq = (const T*)q;
  const T* kk = (const T*)k;
  const T* vp = (const T*)v;
  const ScorePtrs w = score_ptrs(ws, lay);
  int S = lay.S_simple;
  if (pb.ind != 0) gram = nullptr;                 // no projection: vv becomes the squared norm of the value row
  const float* part_z = w.part_z;
  if (pb.ext_lse) {
    // the caller's attention output and log-sum-exp stand in for the attention pass: one "split"
    S = 1;
    const int rows = pb.Hq * pb.W;
    RK_LAUNCH(ST_ATTN, st, (k_stats_fill<0>), dim3((rows + 255) / 256), dim3(256), 0, st, rows, pb.ext_lse,
              w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l);
    part_z = pb.ext_out;
  } else {
    RK_LAUNCH(ST_ATTN, st, (k_attn_partial<T, D>), dim3(S, (pb.R + RB - 1) / RB, pb.Hkv), dim3(256), 0, st,
                       pb, qq, kk, vp, S, w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l, w.part_z);
  }
  RK_LAUNCH(ST_COMBINE, st, (k_attn_combine<T, D>), combine_grid(pb), combine_block<D>(), 0, st, pb, vp, S, gram,
            w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l, part_z, w.rs_m, w.rs_l, w.rs_zz, w.rs_nstar,
            w.rs_istar, w.rs_u, (const T*)nullptr, (uint16_t*)nullptr, 0, 0, combine_groups(pb));
  RK_LAUNCH(ST_VV, st, (k_vv<T, D>), dim3((pb.P + 63) / 64, pb.Hq), dim3(256), 0, st, pb, vp, gram, w.vv, lay.ldv);
  RK_LAUNCH(ST_SCORE, st, (k_score<T, D>), dim3((pb.P + TN - 1) / TN, pb.Hkv), dim3(256), 0, st, pb, qq,
                     kk, vp, w.rs_m, w.rs_l, w.rs_zz, w.rs_nstar, w.rs_istar, w.rs_u, w.vv, lay.ldv, score);
  return hip_status();
}

}  // namespace

int launch_score_simple(const Prob& pb, const void* q, const void* k, const void* v,
                        const float* gram, float* score, char* ws, const ScoreWs& lay,
                        hipStream_t st) {
  if (pb.dtype == RESTKV_F32) {
    return pb.d == 64 ? run<float, 64>(pb, q, k, v, gram, score, ws, lay, st)
                      : run<float, 128>(pb, q, k, v, gram, score, ws, lay, st);
  }
  return pb.d == 64 ? run<bf16_t, 64>(pb, q, k, v, gram, score, ws, lay, st)
                    : run<bf16_t, 128>(pb, q, k, v, gram, score, ws, lay, st);
}

}  // namespace restkv
