// Reconstruction indicator on the matrix cores (bf16 inputs, FP32 accumulation), gfx950.
//
// Same four stages and scratch layout as the FP32 path.  Every contraction runs on
// v_mfma_f32_32x32x16_bf16 in the "transposed" orientation: the 32 query rows of a
// wavefront sit on the N side of the MFMA (lane % 32 = query row), the keys (or value
// columns) on the M side.  A lane therefore owns ONE query row and 16 keys per 32x32
// block, so the softmax statistics, the champion bookkeeping and the per-row
// constants of the score are plain per-lane scalars.
//
//   C layout of a 32x32 block:  register j of lane l holds
//       M index = 8*(j/4) + 4*(l/32) + (j%4),   N index = l % 32.
//   A / B operands: lane l holds M (or N) index l % 32 and the 8 consecutive
//       K indices 8*(l/32) .. 8*(l/32)+7 of each 16-wide K step.
//
// Query rows of one KV head are laid out so that a wavefront holds all (padded) Gp
// query heads of 32/Gp window positions; the mean over the group is then a reduction
// across lanes of one wavefront.
#include <limits.h>

#include "score_common.hpp"

namespace restkv {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int TN = 64;                 // keys per LDS tile
constexpr float LOG2E = 1.4426950408889634f;
constexpr float RESCALE_TH = 8.0f;     // log2 units a row maximum may run ahead of its reference

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) {
  union { uint4 u; bf16x8 b; } x;
  x.u = u;
  return x.b;
}
__device__ __forceinline__ float xhalf_max(float x) {   // max with the lane 32 away
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float xhalf_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ int xhalf_min(int x) {
  const auto r = __builtin_amdgcn_permlane32_swap((unsigned)x, (unsigned)x, false, false);
  return min((int)r[0], (int)r[1]);
}
__device__ __forceinline__ float bf16_to_f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// key (or value-column) index of register j of a 32x32 block for this lane half
__device__ __forceinline__ constexpr int cidx(int j, int hf) { return 8 * (j >> 2) + 4 * hf + (j & 3); }

struct RowInfo {
  int hloc, i, h, row;   // head inside the group, window position, query head, global row h*W+i
  bool valid;
};
__device__ __forceinline__ RowInfo row_info(const Prob& pb, int g, int wave_block, int lane, int log2iw) {
  RowInfo r;
  const int rr = lane & 31;
  const int iw = 1 << log2iw;
  r.hloc = rr >> log2iw;
  r.i = wave_block * iw + (rr & (iw - 1));
  r.valid = r.hloc < pb.G && r.i < pb.W;
  r.h = g * pb.G + (r.valid ? r.hloc : 0);
  r.row = r.h * pb.W + (r.valid ? r.i : 0);
  return r;
}

// cooperative global -> register -> LDS copy of one 64-key tile of a [tokens, D] matrix
template <int D, int NTHR>
struct TileRegs {
  static constexpr int CPT = TN * D / 8 / NTHR;     // 16-byte chunks per thread
  uint4 r[CPT];
  __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int64_t stride, int kb, int L) {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int x = threadIdx.x + j * NTHR;
      const int key = x / (D / 8), c8 = x % (D / 8);
      // rows past the end are clamped, not skipped (their keys are masked, their weights zero):
      // unconditional loads keep the prefetch free of branches
      const int n = min(kb + key, L - 1);
      r[j] = *(const uint4*)(base + (int64_t)n * stride + c8 * 8);
    }
  }
  __device__ __forceinline__ void store(uint16_t* lds, int lds_stride) const {
#pragma unroll
    for (int j = 0; j < CPT; ++j) {
      const int x = threadIdx.x + j * NTHR;
      const int key = x / (D / 8), c8 = x % (D / 8);
      *(uint4*)(lds + key * lds_stride + c8 * 8) = r[j];
    }
  }
};

// Compiler-only fence: memory operations are not moved across it.  Placed right after the global
// loads of the next tile so that they are issued BEFORE the tile's matrix work instead of being
// sunk down to the LDS stores that consume them (which would expose the full memory latency).
__device__ __forceinline__ void pin_issue() { asm volatile("" ::: "memory"); }

// ------------------------------------------------------------------------------------------
// Attention pass: per key split, champion-excluded online softmax statistics and A.V sums.
// grid (S, row blocks, Hkv), NW*64 threads.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64) void k_attn_mfma(Prob pb, const uint16_t* __restrict__ q,
                                                       const uint16_t* __restrict__ k,
                                                       const uint16_t* __restrict__ v, int S, int kps,
                                                       int log2iw, ScorePtrs o) {
  constexpr int KS = D / 16, CB = D / 32, KST = D + 8, VST = D + 32, NTHR = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][TN * KST];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][TN * VST];

  const int s = blockIdx.x, g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6, rr = l & 31, hf = l >> 5;
  const RowInfo ri = row_info(pb, g, blockIdx.y * NW + wv, l, log2iw);
  const uint16_t* kg = k + (int64_t)g * pb.kv_sh;
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (ri.valid) u = *(const uint4*)(q + (int64_t)ri.h * pb.q_sh + (int64_t)ri.i * pb.q_st + 16 * ks + 8 * hf);
    qf[ks] = as_bf16x8(u);
  }
  // Split s owns one contiguous key range (a sequential stream per workgroup measured faster
  // than tiles interleaved across the splits).
  const int kbeg = s * kps;
  const int kend = min(pb.L, kbeg + kps);
  const int ntiles = kend > kbeg ? (kend - kbeg + TN - 1) / TN : 0;
  auto tile_key = [&](int t) { return kbeg + t * TN; };
  const int vis_last = (pb.causal && ri.valid) ? pb.P + ri.i : pb.L - 1;
  const float c2 = pb.scale * LOG2E;

  float mall = -INFINITY, mref = -INFINITY, mx = -INFINITY, lsum = 0.f;
  int nx = -1;                       // key kept out of the sums (see below), -1: none
  f32x16 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int j = 0; j < 16; ++j) oacc[cb][j] = 0.f;

  // lane-constant part of the transposing LDS read address of the value tile
  const int s16 = l & 15;
  const int voff = (4 * hf + (s16 >> 2)) * VST + 16 * ((l >> 4) & 1) + 4 * (s16 & 3);

  TileRegs<D, NTHR> tk, tv;
  if (ntiles > 0) {
    tk.load(kg, pb.kv_st, tile_key(0), pb.L);
    tv.load(vg, pb.kv_st, tile_key(0), pb.L);
    tk.store(Ks[0], KST);
    tv.store(Vs[0], VST);
  }
  __syncthreads();

  for (int t = 0; t < ntiles; ++t) {
    const int buf = t & 1;
    const int kb = tile_key(t);
    {
      // the next tile travels through registers while this one is computed (the last iteration
      // re-fetches its own tile: no branch around the loads, nothing reads that copy)
      const int tn = min(t + 1, ntiles - 1);
      tk.load(kg, pb.kv_st, tile_key(tn), pb.L);
      tv.load(vg, pb.kv_st, tile_key(tn), pb.L);
      pin_issue();
    }
    // ---- logits S^T[key, row] = K Q^T ----
    f32x16 sacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int j = 0; j < 16; ++j) sacc[mb][j] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bf16x8 a = as_bf16x8(*(const uint4*)&Ks[buf][(32 * mb + rr) * KST + 16 * ks + 8 * hf]);
        sacc[mb] = MFMA(a, qf[ks], sacc[mb]);
      }
    }
    const bool tile_mask = (kb + TN > kend) || (pb.causal && kb + TN - 1 > pb.P);
    if (tile_mask) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const int n = kb + 32 * mb + cidx(j, hf);
          if (n >= kend || n > vis_last) sacc[mb][j] = -INFINITY;
        }
    }
    float tm = sacc[0][0];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int j = 0; j < 16; ++j) tm = fmaxf(tm, sacc[mb][j]);
    tm = xhalf_max(tm);

    // A key is kept out of the sums only if, on arrival, it is the largest so far AND would
    // hold more than 1/9 of the mass seen so far; such keys are rare after the first tile, so
    // the expensive part of the bookkeeping (index search, folding the previous kept-out key
    // back in) almost never runs.  The reference of the exponentials follows the maximum lazily.
    const bool newmax = tm > mall;
    const bool resc = (tm - mref) * c2 > RESCALE_TH;
    bool excl_here = false;
    if (__ballot(newmax || resc) != 0ull) {
      bool dominant = false;
      if (newmax) {
        const float pstar = __builtin_amdgcn_exp2f((tm - mref) * c2);      // inf on the first tile
        float total = xhalf_sum(lsum);
        if (nx >= 0) total += __builtin_amdgcn_exp2f((mx - mref) * c2);
        dominant = pstar * 8.0f > total;
      }
      if (__ballot(dominant) != 0ull) {
        int cand = INT_MAX;
        if (dominant) {
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j)
              if (sacc[mb][j] == tm) cand = min(cand, kb + 32 * mb + cidx(j, hf));
        }
        cand = xhalf_min(cand);
        if (dominant) {
          if (nx >= 0) {             // the key kept out so far joins the running sums
            const float w = __builtin_amdgcn_exp2f((mx - mref) * c2);
            if (hf == 0) lsum += w;
            const uint16_t* vr = vg + (int64_t)nx * pb.kv_st;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
              for (int jq = 0; jq < 4; ++jq) {
                const uint2 u = *(const uint2*)(vr + 32 * cb + 8 * jq + 4 * hf);
                oacc[cb][4 * jq + 0] += w * __uint_as_float(u.x << 16);
                oacc[cb][4 * jq + 1] += w * __uint_as_float(u.x & 0xFFFF0000u);
                oacc[cb][4 * jq + 2] += w * __uint_as_float(u.y << 16);
                oacc[cb][4 * jq + 3] += w * __uint_as_float(u.y & 0xFFFF0000u);
              }
          }
          mx = tm;
          nx = cand;
        }
        excl_here = true;
      }
      if (resc) {
        const float f = __builtin_amdgcn_exp2f((mref - tm) * c2);   // first tile: 2^-inf = 0
        lsum *= f;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
          for (int j = 0; j < 16; ++j) oacc[cb][j] *= f;
        mref = tm;
      }
      mall = fmaxf(mall, tm);
    }
    // ---- weights relative to the reference ----
    const float nm = -mref * c2;
    bf16x8 pv[2][2];
    if (excl_here) {                 // wave-uniform: this tile holds a key that is being kept out
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][j], c2, nm));
          if ((kb + 32 * mb + cidx(j, hf)) == nx) p = 0.f;
          lsum += p;
          pv[mb][j >> 3][j & 7] = (__bf16)p;
        }
    } else {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mb][j], c2, nm));
          lsum += p;
          pv[mb][j >> 3][j & 7] = (__bf16)p;
        }
    }
    // ---- O^T[c, row] += V^T P^T ; value operand through the transposing LDS read ----
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int kg2 = 0; kg2 < 2; ++kg2) {
        const int kb16 = 32 * mb + 16 * kg2;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
          const uint16_t* base = &Vs[buf][kb16 * VST + 32 * cb + voff];
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(base));
          const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (__attribute__((address_space(3))) s16x4*)(base + 8 * VST));
          union { s16x8 s; bf16x8 b; } a;
          a.s = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          oacc[cb] = MFMA(a.b, pv[mb][kg2], oacc[cb]);
        }
      }
    pin_issue();                     // ... and their LDS stores stay behind the tile's work
    tk.store(Ks[buf ^ 1], KST);
    tv.store(Vs[buf ^ 1], VST);
    __syncthreads();
  }
  const float ltot = xhalf_sum(lsum);
  if (ri.valid) {
    const int64_t po = (int64_t)ri.row * S + s;
    if (hf == 0) {
      o.part_m[po] = mall * c2;
      o.part_mx[po] = mx * c2;
      o.part_n[po] = nx;
      o.part_ref[po] = ntiles > 0 ? mref * c2 : 0.f;
      o.part_l[po] = ltot;
    }
    float* zp = o.part_z + po * D;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        f32x4 x = {oacc[cb][4 * jq], oacc[cb][4 * jq + 1], oacc[cb][4 * jq + 2], oacc[cb][4 * jq + 3]};
        *(f32x4*)(zp + 32 * cb + 8 * jq + 4 * hf) = x;
      }
  }
}

// ------------------------------------------------------------------------------------------
// vv[h, n] = v_n M_h v_n^T :  Y^T = M_h V^T on the MFMA, then a row dot with v_n.
// A wavefront owns 32 rows of one head's Gram matrix (hi + lo bf16 parts, resident in
// registers for the whole kernel); the value tile in LDS is the B operand shared by all
// wavefronts of the workgroup (HPW heads x D/32 row blocks).  Partial row dots of the D/32
// wavefronts of a head meet in LDS.
// grid (key chunks, ceil(G/HPW), Hkv), HPW*(D/32)*64 threads.
template <int D, int HPW>
__global__ __launch_bounds__(HPW * (D / 32) * 64) void k_vv_mfma(Prob pb, const uint16_t* __restrict__ v,
                                                                 const float* __restrict__ gram,
                                                                 float* __restrict__ vv, int ldv,
                                                                 int tiles_per_wg) {
  constexpr int KS = D / 16, CB = D / 32, KST = D + 8, NW = HPW * CB, NTHR = NW * 64;
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][TN * KST];
  __shared__ float part[2][HPW][CB][TN];
  const int g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6, rr = l & 31, hf = l >> 5;
  const int hw = wv / CB, mb = wv % CB;               // head inside the workgroup, Gram row block
  const int hloc = blockIdx.y * HPW + hw;
  const bool head_ok = hloc < pb.G;
  const int h = g * pb.G + (head_ok ? hloc : 0);
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;

  bf16x8 ahi[KS], alo[KS];
  {
    const float* mrow = gram + ((int64_t)h * D + 32 * mb + rr) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const f32x4 x0 = *(const f32x4*)(mrow + 16 * ks + 8 * hf);
      const f32x4 x1 = *(const f32x4*)(mrow + 16 * ks + 8 * hf + 4);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float f = e < 4 ? x0[e] : x1[e - 4];
        const __bf16 hi = (__bf16)f;
        ahi[ks][e] = hi;
        alo[ks][e] = (__bf16)(f - (float)hi);
      }
    }
  }
  const int NT = (pb.P + TN - 1) / TN;
  const int t0 = blockIdx.x * tiles_per_wg;
  const int t1 = min(NT, t0 + tiles_per_wg);
  if (t0 >= t1) return;

  TileRegs<D, NTHR> tv;
  tv.load(vg, pb.kv_st, t0 * TN, pb.L);
  tv.store(Vs[0], KST);
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int buf = (t - t0) & 1;
    tv.load(vg, pb.kv_st, min(t + 1, t1 - 1) * TN, pb.L);     // unconditional: see pin_issue
    pin_issue();
    f32x16 y[2];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
      for (int j = 0; j < 16; ++j) y[nb][j] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const bf16x8 b = as_bf16x8(*(const uint4*)&Vs[buf][(32 * nb + rr) * KST + 16 * ks + 8 * hf]);
        y[nb] = MFMA(ahi[ks], b, y[nb]);
        y[nb] = MFMA(alo[ks], b, y[nb]);
      }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      float acc = 0.f;
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const uint2 u = *(const uint2*)&Vs[buf][(32 * nb + rr) * KST + 32 * mb + 8 * jq + 4 * hf];
        acc = fmaf(y[nb][4 * jq + 0], __uint_as_float(u.x << 16), acc);
        acc = fmaf(y[nb][4 * jq + 1], __uint_as_float(u.x & 0xFFFF0000u), acc);
        acc = fmaf(y[nb][4 * jq + 2], __uint_as_float(u.y << 16), acc);
        acc = fmaf(y[nb][4 * jq + 3], __uint_as_float(u.y & 0xFFFF0000u), acc);
      }
      acc = xhalf_sum(acc);
      if (hf == 0) part[buf][hw][mb][32 * nb + rr] = acc;
    }
    pin_issue();
    tv.store(Vs[buf ^ 1], KST);
    __syncthreads();
    if (threadIdx.x < HPW * TN) {
      const int hh = threadIdx.x / TN, key = threadIdx.x % TN;
      const int n = t * TN + key;
      const int hl2 = blockIdx.y * HPW + hh;
      if (n < pb.P && hl2 < pb.G) {
        float sum = 0.f;
#pragma unroll
        for (int m2 = 0; m2 < CB; ++m2) sum += part[buf][hh][m2][key];
        vv[(int64_t)(g * pb.G + hl2) * ldv + n] = sum;
      }
    }
  }
}

// vv without a projection: squared norm of the value row.  grid (ceil(P/256), Hkv)
template <int D>
__global__ __launch_bounds__(256) void k_vnorm2(Prob pb, const uint16_t* __restrict__ v,
                                                float* __restrict__ vv, int ldv) {
  const int g = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
  if (n >= pb.P) return;
  const uint16_t* vr = v + (int64_t)g * pb.kv_sh + (int64_t)n * pb.kv_st;
  float acc = 0.f;
#pragma unroll
  for (int c8 = 0; c8 < D / 8; ++c8) {
    const uint4 u = *(const uint4*)(vr + 8 * c8);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = __uint_as_float(w[e] << 16), b = __uint_as_float(w[e] & 0xFFFF0000u);
      acc = fmaf(a, a, acc);
      acc = fmaf(b, b, acc);
    }
  }
  for (int hl = 0; hl < pb.G; ++hl) vv[(int64_t)(g * pb.G + hl) * ldv + n] = acc;
}

// Sum over the lanes that hold the same window position for the GP (padded) heads of the
// group: lanes IW = 32/GP apart inside each 32-lane half.  Rotations inside the 16-lane DPP
// rows cover the strides below 16, a row swap the stride 16.
template <int GP>
__device__ __forceinline__ float group_sum(float x) {
  constexpr int IW = 32 / GP;
#define RK_ROR(n) x += __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x120 + (n), 0xF, 0xF, false))
  if constexpr (IW <= 1) RK_ROR(1);
  if constexpr (IW <= 2) RK_ROR(2);
  if constexpr (IW <= 4) RK_ROR(4);
  if constexpr (IW <= 8) RK_ROR(8);
#undef RK_ROR
  if constexpr (IW <= 16) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  }
  return x;
}

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// ------------------------------------------------------------------------------------------
// Score pass: logits again, cross term u.v_n, closed form, mean over the group.
// grid (key chunks, row blocks, Hkv), NW*64 threads.
//
// Per element (query row r of head h, key n), with everything relative to the row maximum M:
//   e = 2^(s - M) / G,  den = l - G e,  d2 = vv[h,n] - 2 (u.v_n - zz/2),
//   I/G = e * sqrt(d2) / den = e * x * rsq(x * den^2),  x = max(d2, tiny)
// (1/G of the group mean is folded into the exponent, zz/2 into the accumulator's start value).
template <int D, int NW, int GP>
__global__ __launch_bounds__(NW * 64) void k_score_mfma(Prob pb, const uint16_t* __restrict__ q,
                                                        const uint16_t* __restrict__ k,
                                                        const uint16_t* __restrict__ v, ScorePtrs o,
                                                        int ldv, float* __restrict__ score,
                                                        int tiles_per_wg, int vec_store) {
  constexpr int KS = D / 16, KST = D + 8, NTHR = NW * 64, LOG2IW = ilog2(32 / GP);
  __shared__ __attribute__((aligned(16))) uint16_t Ks[2][TN * KST];
  __shared__ __attribute__((aligned(16))) uint16_t Vs[2][TN * KST];
  __shared__ __attribute__((aligned(16))) float vvs[2][GP][TN];

  const int g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6, rr = l & 31, hf = l >> 5;
  const RowInfo ri = row_info(pb, g, blockIdx.y * NW + wv, l, LOG2IW);
  const uint16_t* kg = k + (int64_t)g * pb.kv_sh;
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;

  bf16x8 qf[KS], uhi[KS], ulo[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    uint4 u = make_uint4(0, 0, 0, 0);
    if (ri.valid) u = *(const uint4*)(q + (int64_t)ri.h * pb.q_sh + (int64_t)ri.i * pb.q_st + 16 * ks + 8 * hf);
    qf[ks] = as_bf16x8(u);
    const float* up = o.rs_u + (int64_t)ri.row * D + 16 * ks + 8 * hf;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float f = ri.valid ? up[e] : 0.f;
      const __bf16 hi = (__bf16)f;
      uhi[ks][e] = hi;
      ulo[ks][e] = (__bf16)(f - (float)hi);
    }
  }
  const float c2 = pb.scale * LOG2E;
  const float Gf = (float)pb.G;
  const float nM2 = ri.valid ? -o.rs_m[ri.row] - log2f(Gf) : 0.f;     // e comes out divided by G
  const float lrow = ri.valid ? o.rs_l[ri.row] : INFINITY;           // an idle lane scores exactly 0
  const float nhzz = ri.valid ? -0.5f * o.rs_zz[ri.row] : 0.f;
  const int nstar = ri.valid ? o.rs_nstar[ri.row] : -1;
  const float istar = ri.valid ? o.rs_istar[ri.row] / Gf : 0.f;
  const bool writer = ri.hloc == 0 && ri.i < pb.W;
  float* orow = score + ((int64_t)g * pb.W + (writer ? ri.i : 0)) * pb.ld;

  const int NT = (pb.P + TN - 1) / TN;
  const int t0 = blockIdx.x * tiles_per_wg;
  const int t1 = min(NT, t0 + tiles_per_wg);
  if (t0 >= t1) return;

  // v M v^T of the tile for the heads of the group: GP*TN floats, one float4 per loader thread
  const bool vv_loader = threadIdx.x < GP * (TN / 4);
  const int vv_h = threadIdx.x / (TN / 4), vv_q = threadIdx.x % (TN / 4);
  const float* vv_src = o.vv + (int64_t)(g * pb.G + min(vv_h, pb.G - 1)) * ldv + 4 * vv_q;
  auto load_vv = [&](int kb) {
    f32x4 x = {0.f, 0.f, 0.f, 0.f};
    if (vv_loader && vv_h < pb.G && kb + 4 * vv_q < pb.P) x = *(const f32x4*)(vv_src + kb);
    return x;
  };

  TileRegs<D, NTHR> tk, tv;
  tk.load(kg, pb.kv_st, t0 * TN, pb.L);
  tv.load(vg, pb.kv_st, t0 * TN, pb.L);
  f32x4 vvr = load_vv(t0 * TN);
  tk.store(Ks[0], KST);
  tv.store(Vs[0], KST);
  if (vv_loader) *(f32x4*)&vvs[0][vv_h][4 * vv_q] = vvr;
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const int buf = (t - t0) & 1;
    const int kb = t * TN;
    {
      const int kn = min(t + 1, t1 - 1) * TN;                 // unconditional: see pin_issue
      tk.load(kg, pb.kv_st, kn, pb.L);
      tv.load(vg, pb.kv_st, kn, pb.L);
      vvr = load_vv(kn);
      pin_issue();
    }
    f32x16 sacc[2], cacc[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int j = 0; j < 16; ++j) { sacc[mb][j] = 0.f; cacc[mb][j] = nhzz; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bf16x8 ak = as_bf16x8(*(const uint4*)&Ks[buf][(32 * mb + rr) * KST + 16 * ks + 8 * hf]);
        sacc[mb] = MFMA(ak, qf[ks], sacc[mb]);
        const bf16x8 av = as_bf16x8(*(const uint4*)&Vs[buf][(32 * mb + rr) * KST + 16 * ks + 8 * hf]);
        cacc[mb] = MFMA(av, uhi[ks], cacc[mb]);
        cacc[mb] = MFMA(av, ulo[ks], cacc[mb]);
      }
    // ---- epilogue: values in place of the logits ----
    const float* vvrow = &vvs[buf][ri.hloc < GP ? ri.hloc : 0][0];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const f32x4 vv4 = *(const f32x4*)(vvrow + 32 * mb + 8 * jq + 4 * hf);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int j = 4 * jq + e;
          const float ev = __builtin_amdgcn_exp2f(fmaf(sacc[mb][j], c2, nM2));
          const float den = fmaf(-Gf, ev, lrow);
          const float x = fmaxf(fmaf(-2.f, cacc[mb][j], vv4[e]), 1e-30f);
          sacc[mb][j] = ev * x * __builtin_amdgcn_rsqf(x * den * den);
        }
      }
    if (__ballot(nstar >= kb && nstar < kb + TN) != 0ull) {     // a champion of this wavefront is here
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j)
          if (kb + 32 * mb + cidx(j, hf) == nstar) sacc[mb][j] = istar;
    }
    // ---- mean over the group, store ----
    const bool full = kb + TN <= pb.P;
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const int n0 = kb + 32 * mb + 8 * jq + 4 * hf;
        f32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = group_sum<GP>(sacc[mb][4 * jq + e]);
        if (writer) {
          if (full && vec_store) {
            *(f32x4*)(orow + n0) = out;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (n0 + e < pb.P) orow[n0 + e] = out[e];
          }
        }
      }
    pin_issue();
    tk.store(Ks[buf ^ 1], KST);
    tv.store(Vs[buf ^ 1], KST);
    if (vv_loader) *(f32x4*)&vvs[buf ^ 1][vv_h][4 * vv_q] = vvr;
    __syncthreads();
  }
}

template <int D, int NW>
void launch_attn(const Prob& pb, dim3 grid, hipStream_t st, const uint16_t* q, const uint16_t* k,
                 const uint16_t* v, int S, int kps, int log2iw, const ScorePtrs& w) {
  RK_LAUNCH(ST_ATTN, st, (k_attn_mfma<D, NW>), grid, dim3(NW * 64), 0, st, pb, q, k, v, S, kps,
            log2iw, w);
}

template <int D, int NW>
void launch_pass2(const Prob& pb, int gp, dim3 grid, hipStream_t st, const uint16_t* q, const uint16_t* k,
                  const uint16_t* v, const ScorePtrs& w, int ldv, float* score, int tpw, int vec) {
#define RK_CASE(GPV)                                                                              \
  case GPV:                                                                                       \
    RK_LAUNCH(ST_SCORE, st, (k_score_mfma<D, NW, GPV>), grid, dim3(NW * 64), 0, st, pb, q, k, v, w, \
              ldv, score, tpw, vec);                                                              \
    break;
  switch (gp) {
    RK_CASE(1) RK_CASE(2) RK_CASE(4) RK_CASE(8) RK_CASE(16) RK_CASE(32)
    default: break;
  }
#undef RK_CASE
}

template <int D>
int run_mfma(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
             float* score, char* ws, const ScoreWs& lay, hipStream_t st) {
  const uint16_t* qq = (const uint16_t*)q;
  const uint16_t* kk = (const uint16_t*)k;
  const uint16_t* vp = (const uint16_t*)v;
  const ScorePtrs w = score_ptrs(ws, lay);
  int gp = 1;
  while (gp < pb.G) gp <<= 1;
  const int iw = 32 / gp, log2iw = ilog2(iw);
  const int nwr = (pb.W + iw - 1) / iw;            // wavefronts needed to cover the window
  const int nw = nwr <= 4 ? 4 : 8;
  const int gy = (nwr + nw - 1) / nw;
  // attention pass: about one workgroup per compute unit, whole tiles per split
  int S = 256 / (pb.Hkv * gy);
  const int max_s = (pb.L + TN - 1) / TN;
  if (S > max_s) S = max_s;
  if (S > lay.S_max) S = lay.S_max;
  if (S < 1) S = 1;
  int kps = (pb.L + S - 1) / S;
  kps = (kps + TN - 1) / TN * TN;
  const dim3 g1(S, gy, pb.Hkv);
  if (nw == 4) launch_attn<D, 4>(pb, g1, st, qq, kk, vp, S, kps, log2iw, w);
  else launch_attn<D, 8>(pb, g1, st, qq, kk, vp, S, kps, log2iw, w);
  RK_LAUNCH(ST_COMBINE, st, (k_attn_combine<bf16_t, D>), dim3(pb.Hq * pb.W), dim3(D), 0, st, pb,
            (const bf16_t*)v, S, gram, w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l, w.part_z, w.rs_m,
            w.rs_l, w.rs_zz, w.rs_nstar, w.rs_istar, w.rs_u);
  if (gram) {
    constexpr int HPW = D == 128 ? 2 : 4;
    const int NTv = (pb.P + TN - 1) / TN;
    const int hg = (pb.G + HPW - 1) / HPW;
    int tpv = (int)(((int64_t)NTv * hg * pb.Hkv + 1023) / 1024);
    if (tpv < 1) tpv = 1;
    RK_LAUNCH(ST_VV, st, (k_vv_mfma<D, HPW>), dim3((NTv + tpv - 1) / tpv, hg, pb.Hkv),
              dim3(HPW * (D / 32) * 64), 0, st, pb, vp, gram, w.vv, lay.ldv, tpv);
  } else {
    RK_LAUNCH(ST_VV, st, (k_vnorm2<D>), dim3((pb.P + 255) / 256, pb.Hkv), dim3(256), 0, st, pb, vp,
              w.vv, lay.ldv);
  }
  const int NT = (pb.P + TN - 1) / TN;
  int tpw = (int)(((int64_t)NT * gy * pb.Hkv + 2047) / 2048);
  if (tpw < 1) tpw = 1;
  const dim3 g2((NT + tpw - 1) / tpw, gy, pb.Hkv);
  const int vec = ((pb.ld & 3) == 0 && ((uintptr_t)score & 15u) == 0) ? 1 : 0;
  if (nw == 4) launch_pass2<D, 4>(pb, gp, g2, st, qq, kk, vp, w, lay.ldv, score, tpw, vec);
  else launch_pass2<D, 8>(pb, gp, g2, st, qq, kk, vp, w, lay.ldv, score, tpw, vec);
  return hip_status();
}

}  // namespace

bool mfma_eligible(const Prob& pb, const void* q, const void* k, const void* v) {
  if (pb.dtype != RESTKV_BF16) return false;
  if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v) & 15u) != 0) return false;
  if ((pb.q_sh | pb.q_st | pb.kv_sh | pb.kv_st) & 7) return false;
  if (pb.G > 32) return false;
  return true;
}

int launch_score_mfma(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
                      float* score, char* ws, const ScoreWs& lay, hipStream_t st) {
  return pb.d == 64 ? run_mfma<64>(pb, q, k, v, gram, score, ws, lay, st)
                    : run_mfma<128>(pb, q, k, v, gram, score, ws, lay, st);
}

}  // namespace restkv
