// Reconstruction indicator on the matrix cores (bf16 inputs, FP32 accumulation), gfx950.
//
// Same four stages and scratch layout as the FP32 path: attention pass per key split, merge
// (score_common.hpp), value Gram pass vv, score pass.  Every contraction runs on
// v_mfma_f32_32x32x16_bf16:
//
//   C layout of a 32x32 block:  register j of lane l holds
//       M index = 8*(j/4) + 4*(l/32) + (j%4),   N index = l % 32.
//   A / B operands: lane l holds M (or N) index l % 32 and the 8 consecutive
//       K indices 8*(l/32) .. 8*(l/32)+7 of each 16-wide K step.
//
// The attention pass puts the 32 query rows of a wavefront on the N side (lane % 32 = query
// row, keys or value columns on the M side), so the softmax statistics and the champion
// bookkeeping are per-lane scalars.  The score pass puts the query rows on the M side and the
// keys on the N side, with the heads of a group in consecutive registers, so the mean over
// the group is a few in-lane adds and a store writes 32 consecutive keys of one row.
//
// All three kernels are persistent (about one 8-wavefront workgroup per compute unit walking a
// run of 64-key tiles) and stream their K/V tiles through asynchronous LDS rings (TileRing).
#include <limits.h>

#include <type_traits>

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
constexpr float RESCALE_TH = 8.0f;  // log2 units a row maximum may run ahead of its reference

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

// vv without a projection: squared norm of the value row (1 for the attention-weight
// indicator, which has no value term).  grid (ceil(P/256), Hkv)
template <int D>
__global__ __launch_bounds__(256) void k_vnorm2(Prob pb, const uint16_t* __restrict__ v,
                                                float* __restrict__ vv, int ldv) {
  const int g = blockIdx.y, n = blockIdx.x * 256 + threadIdx.x;
  if (n >= pb.P) return;
  if (pb.ind == 1) {
    for (int hl = 0; hl < pb.G; ++hl) vv[(int64_t)(g * pb.G + hl) * ldv + n] = 1.0f;
    return;
  }
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

constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// ------------------------------------------------------------------------------------------
// Asynchronous tile ring shared by the pipelined kernels.
//
// A 64-key tile of a [tokens, D] bf16 matrix is copied global -> LDS by global_load_lds_dwordx4:
// each wave-instruction moves 1 KiB (64 lanes x 16 B) to consecutive LDS bytes, while every
// lane picks its own global source.  Inside a tile row the 16-byte chunks are permuted by a
// row-dependent XOR (see TileRing) so that the lanes of one LDS read instruction, which walk
// down the rows at a fixed chunk, spread over all banks without padding between the rows.
// The copies are issued from inline asm and waited for with explicit s_waitcnt
// vmcnt(n): a wave's loads retire in order, and a later store can only make the count higher,
// so "count <= number of loads issued after the group" implies that the group has landed.
// One 1 KiB asynchronous copy: lane i moves the 16 bytes at base + voff_i to LDS bytes
// [16 i, 16 i + 16) of lds_dst.  base and lds_dst are wave-uniform.
__device__ __forceinline__ void dma_1k(const void* base, uint32_t voff, void* lds_dst) {
  const uint32_t dst =
      __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)lds_dst);
  const uint64_t sb = (uint64_t)base;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)sb);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(sb >> 32));
  const uint64_t ub = ((uint64_t)hi << 32) | lo;
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(ub), "s"(dst)
               : "memory", "m0");
}
// The same with the LDS byte address given as a number (wave-uniform, like base): nothing of the
// copy's addressing is left to the vector ALU but the lane's own offset.
__device__ __forceinline__ void dma_1k_to(const void* base, uint32_t voff, uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(base), "s"(lds_dst)
               : "memory", "m0");
}
// LDS byte address of a __shared__ object
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// The wavefront's index inside its workgroup as a scalar: what is derived from it (ring slots,
// row blocks, the early / late split) then lives in scalar registers and branches.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }
// KIND 0: tile read as MFMA operand columns (16 rows x one 16-byte chunk per instruction):
//         chunk c of row r sits at chunk position c ^ key, key = (r >> log2(16/CH)) & (CH-1).
// KIND 1: tile read through the transposing 8-byte LDS read (4 rows x 4 consecutive chunks per
//         half wave): the GROUP of four chunks c>>2 sits at group position (c>>2) ^ key,
//         key = r & 3 (D = 128) or (r >> 1) & 1 (D = 64).
template <int D, int KIND = 0>
struct TileRing {
  static constexpr int CH = D / 8;                 // 16-byte chunks per row
  static constexpr int RPI = 64 / CH;              // rows per wave-instruction
  static constexpr int NI = TN / RPI;              // wave-instructions per tile
  static constexpr int SH = CH == 16 ? 0 : 1;      // D = 128: 0, D = 64: 1
  __device__ static __forceinline__ int swz(int r, int c) {
    if constexpr (KIND == 0) return c ^ ((r >> SH) & (CH - 1));
    else return c ^ (((r >> SH) & (CH / 4 - 1)) << 2);
  }
  // offset in uint16 units of chunk c of row r
  __device__ static __forceinline__ int off(int r, int c) { return r * D + (swz(r, c) << 3); }
  // wave wv of NW issues its share of one tile: rows [kb, kb+64) of the matrix at `base`
  // (wave-uniform pointer, row pitch `pitch` bytes), clamped to row L-1.  Byte offsets are 32-bit:
  // the host checks that the matrix of one head spans less than 4 GiB.
  template <int NW>
  __device__ static __forceinline__ void issue(const uint16_t* base, uint32_t pitch, int kb, int L,
                                               uint16_t* lds_tile, int wv, int lane) {
    issue_rows<NW>(base, pitch, [&](int r) { return min(kb + r, L - 1); }, lds_tile, wv, lane);
  }
  // the same with an arbitrary matrix row for every tile row r (row_of(r) must be a valid row)
  template <int NW, typename F>
  __device__ static __forceinline__ void issue_rows(const uint16_t* base, uint32_t pitch, F row_of,
                                                    uint16_t* lds_tile, int wv, int lane) {
    static_assert(NI % NW == 0, "tile instructions must divide over the wavefronts");
#pragma unroll
    for (int j = 0; j < NI / NW; ++j) {
      const int blk = wv * (NI / NW) + j;
      const int r = blk * RPI + lane / CH, cs = lane % CH;
      const uint32_t voff = (uint32_t)row_of(r) * pitch + (uint32_t)(swz(r, cs) * 16);
      dma_1k(base, voff, lds_tile + blk * 512);
    }
  }
  // The fast path for tiles that lie wholly inside the matrix (no row clamp): the lane's byte
  // offsets inside a tile are computed once per kernel (plan), a copy then takes the tile's
  // wave-uniform address (tile_base = base + first row * pitch) and LDS address and no vector
  // arithmetic at all.
  template <int NW>
  __device__ static __forceinline__ void plan(uint32_t pitch, int wv, int lane, uint32_t (&off)[NI / NW]) {
#pragma unroll
    for (int j = 0; j < NI / NW; ++j) {
      const int blk = wv * (NI / NW) + j;
      const int r = blk * RPI + lane / CH, cs = lane % CH;
      off[j] = (uint32_t)r * pitch + (uint32_t)(swz(r, cs) * 16);
    }
  }
  template <int NW>
  __device__ static __forceinline__ void issue_whole(const void* tile_base, const uint32_t (&off)[NI / NW],
                                                     uint32_t lds_tile, int wv) {
#pragma unroll
    for (int j = 0; j < NI / NW; ++j) dma_1k_to(tile_base, off[j], lds_tile + (uint32_t)(wv * (NI / NW) + j) * 1024u);
  }
};
// Workgroup barrier without the full fence of __syncthreads (which would also wait for the
// asynchronous tile copies in flight): the wavefront's own LDS accesses are drained first, the
// copies are accounted for separately with wait_vm.
__device__ __forceinline__ void wg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N == 0 || N == 1 || N == 2 || N == 3 || N == 4 || N == 5 || N == 8, "add the literal");
  if constexpr (N == 1) asm volatile("s_waitcnt vmcnt(1)" ::: "memory");
  if constexpr (N == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if constexpr (N == 2) asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
  if constexpr (N == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  if constexpr (N == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  if constexpr (N == 3) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
  if constexpr (N == 5) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");
}

// ------------------------------------------------------------------------------------------
// vv[h, n] = v_n M_h v_n^T with the symmetric Gram matrix M_h, as  sum_i v_i (T v)_i  with the
// upper triangular T = diag(M) + 2 triu(M, 1): only the 32 x 32 blocks on or above the diagonal
// are multiplied (10 of 16 for D = 128).  Y^T = T V^T runs on the MFMA with T split into bf16
// high and low parts that stay in registers for the whole kernel; row block rb needs the k-steps
// from 2 rb on, so a wavefront takes the row blocks pr and D/32 - 1 - pr of one head: D/16 + 2
// k-steps whatever pr.  The value tiles arrive through a 4-deep asynchronous LDS ring and are
// the B operand shared by all wavefronts; the partial dots of a head's wavefronts meet in LDS.
// A tile has a matrix part (two 32-key halves of 20 MFMAs) and a vector part (the row dots);
// wavefronts 0..3 and 4..7 run them in complementary order (see the loop), so the matrix cores
// stay fed.  The two wavefronts of a head are in the same group.
// grid (key chunks, ceil(G/HPW), Hkv), 512 threads; HPW = 4 heads per workgroup (8 for D = 64).
template <int D>
__global__ __launch_bounds__(512) void k_vv_pipe(Prob pb, const uint16_t* __restrict__ v,
                                                 const float* __restrict__ gram, float* __restrict__ vv,
                                                 int ldv, int tiles_per_wg) {
  constexpr int NW = 8, KS = D / 16, CB = D / 32, WPH = CB / 2, HPW = NW / WPH;
  using Ring = TileRing<D, 0>;
  constexpr int NG = Ring::NI / NW;                 // copies per wavefront and tile
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[4][TN * D];
  __shared__ float part[2][HPW][WPH][TN];
  const int g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6, rr = l & 31, hf = l >> 5;
  const int wvs = wave_index();                     // the same as a scalar, for the copies' addresses
  const int hw = wv / WPH, pr = wv % WPH;           // head inside the workgroup, row block pair
  const int hloc = blockIdx.y * HPW + hw;
  const int h = g * pb.G + (hloc < pb.G ? hloc : 0);
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;
  const uint32_t pitch = (uint32_t)pb.kv_st * 2u;

  const int NT = (pb.P + TN - 1) / TN;
  const int t0 = blockIdx.x * tiles_per_wg;
  const int t1 = min(NT, t0 + tiles_per_wg);
  if (t0 >= t1) return;
  uint32_t voff[NG];
  Ring::template plan<NW>(pitch, wvs, l, voff);
  const uint32_t vs_base = lds_addr(&Vs[0][0]);
  auto issue_tile = [&](int t) {
    const int kb = min(t, t1 - 1) * TN;
    if (kb + TN <= pb.L)
      Ring::template issue_whole<NW>((const char*)vg + (uint64_t)kb * pitch, voff, vs_base + (uint32_t)(t & 3) * (TN * D * 2), wvs);
    else
      Ring::template issue<NW>(vg, pitch, kb, pb.L, Vs[t & 3], wv, l);
  };
  issue_tile(t0);
  issue_tile(t0 + 1);

  auto body = [&](auto prc) {
    constexpr int PR = decltype(prc)::value;
    constexpr int RB0 = PR, RB1 = CB - 1 - PR;      // RB0 <= RB1
    constexpr int N0 = KS - 2 * RB0, N1 = KS - 2 * RB1;
    bf16x8 ahi0[N0], alo0[N0], ahi1[N1], alo1[N1];
    auto load_frag = [&](int rb, int ks, bf16x8& hi8, bf16x8& lo8) {
      const int i = 32 * rb + rr;                    // Gram row of this lane
      const float* mrow = gram + ((int64_t)h * D + i) * D + 16 * ks + 8 * hf;
      const f32x4 x0 = *(const f32x4*)mrow;
      const f32x4 x1 = *(const f32x4*)(mrow + 4);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int j = 16 * ks + 8 * hf + e;
        float f = e < 4 ? x0[e] : x1[e - 4];
        f = j > i ? 2.f * f : (j == i ? f : 0.f);
        const __bf16 hi = (__bf16)f;
        hi8[e] = hi;
        lo8[e] = (__bf16)(f - (float)hi);
      }
    };
#pragma unroll
    for (int a = 0; a < N0; ++a) load_frag(RB0, 2 * RB0 + a, ahi0[a], alo0[a]);
#pragma unroll
    for (int a = 0; a < N1; ++a) load_frag(RB1, 2 * RB1 + a, ahi1[a], alo1[a]);

    // vv of one tile of this wavefront's head: the partial dots of the head's wavefronts meet here
    auto head_sum = [&](int t) {
      if (PR == 0) {
        const int n = t * TN + l;
        if (n < pb.P && hloc < pb.G) {
          float sum = 0.f;
#pragma unroll
          for (int m2 = 0; m2 < WPH; ++m2) sum += part[(t - t0) & 1][hw][m2][l];
          vv[(int64_t)h * ldv + n] = sum;
        }
      }
    };
    f32x16 y0[2], y1[2];
    uint2 vq0[2][4], vq1[2][4];      // the value entries the row dots of a half need (fetched with its operands)
    // matrix quarter: Y^T = T V^T for the 32 keys of half nb of tile t
    auto mat = [&](int nb, int t) {
      const uint16_t* vt = Vs[t & 3];
      __builtin_amdgcn_s_setprio(2);
#pragma unroll
      for (int j = 0; j < 16; ++j) { y0[nb][j] = 0.f; y1[nb][j] = 0.f; }
      // all operand reads of the quarter first: the MFMAs then run back to back instead of one
      // LDS round trip per k-step
      bf16x8 b[N0];
#pragma unroll
      for (int a = 0; a < N0; ++a) b[a] = as_bf16x8(*(const uint4*)&vt[Ring::off(32 * nb + rr, 2 * (2 * RB0 + a) + hf)]);
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        vq0[nb][jq] = *(const uint2*)&vt[Ring::off(32 * nb + rr, 4 * RB0 + jq) + 4 * hf];
        vq1[nb][jq] = *(const uint2*)&vt[Ring::off(32 * nb + rr, 4 * RB1 + jq) + 4 * hf];
      }
#pragma unroll
      for (int ks = 2 * RB0; ks < KS; ++ks) {
        y0[nb] = MFMA(ahi0[ks - 2 * RB0], b[ks - 2 * RB0], y0[nb]);
        if (ks >= 2 * RB1) y1[nb] = MFMA(ahi1[ks - 2 * RB1], b[ks - 2 * RB0], y1[nb]);
        y0[nb] = MFMA(alo0[ks - 2 * RB0], b[ks - 2 * RB0], y0[nb]);
        if (ks >= 2 * RB1) y1[nb] = MFMA(alo1[ks - 2 * RB1], b[ks - 2 * RB0], y1[nb]);
      }
      __builtin_amdgcn_s_setprio(0);
    };
    // vector quarter: row dot with v_n (register j of a block is Gram row 32 rb + 8 (j/4) + 4 hf + j%4)
    auto dot = [&](int nb, int t) {
      float a0[4], a1[4];              // four independent chains per row block
#pragma unroll
      for (int jq = 0; jq < 4; ++jq) {
        const uint2 u0 = vq0[nb][jq], u1 = vq1[nb][jq];
        a0[jq] = y0[nb][4 * jq + 0] * __uint_as_float(u0.x << 16);
        a1[jq] = y1[nb][4 * jq + 0] * __uint_as_float(u1.x << 16);
        a0[jq] = fmaf(y0[nb][4 * jq + 1], __uint_as_float(u0.x & 0xFFFF0000u), a0[jq]);
        a1[jq] = fmaf(y1[nb][4 * jq + 1], __uint_as_float(u1.x & 0xFFFF0000u), a1[jq]);
        a0[jq] = fmaf(y0[nb][4 * jq + 2], __uint_as_float(u0.y << 16), a0[jq]);
        a1[jq] = fmaf(y1[nb][4 * jq + 2], __uint_as_float(u1.y << 16), a1[jq]);
        a0[jq] = fmaf(y0[nb][4 * jq + 3], __uint_as_float(u0.y & 0xFFFF0000u), a0[jq]);
        a1[jq] = fmaf(y1[nb][4 * jq + 3], __uint_as_float(u1.y & 0xFFFF0000u), a1[jq]);
      }
      const float acc0 = (a0[0] + a0[1]) + (a0[2] + a0[3]), acc1 = (a1[0] + a1[1]) + (a1[2] + a1[3]);
      const float acc = xhalf_sum(acc0 + acc1);
      if (hf == 0) part[(t - t0) & 1][hw][PR][32 * nb + rr] = acc;
    };

    // Steps H_t, one tile each, separated by workgroup barriers.  Wavefronts 0..3 run
    //   H_t: matrix(0,t) matrix(1,t) dot(0,t) dot(1,t),
    // wavefronts 4..7 the complementary order, one tile behind with their row dots,
    //   H_t: dot(0,t-1) dot(1,t-1) matrix(0,t) matrix(1,t),
    // so that on every SIMD one wavefront feeds the matrix cores while the other does its vector
    // work.  Tile t is read in H_t only; the copy of tile t+2 is issued at the top of H_t (its
    // slot held tile t-2); a wavefront waits for its share of tile t+1 before the barrier that
    // ends H_t, when only the copy of tile t+2 is younger.  The partial dots of tile t meet in LDS
    // one step after they were written (two buffers).
    const bool late = wv >= NW / 2;
    wait_vm<NG>();           // own share of tile t0 (compiler-issued loads above are older or waited for)
    wg_barrier();
    for (int t = t0; t < t1; ++t) {
      issue_tile(t + 2);     // into the slot of tile t-2
      if (!late) {
        if (t > t0) head_sum(t - 1);
        mat(0, t);
        mat(1, t);
        dot(0, t);
        dot(1, t);
      } else {
        if (t > t0 + 1) head_sum(t - 2);
        if (t > t0) { dot(0, t - 1); dot(1, t - 1); }
        mat(0, t);
        mat(1, t);
      }
      wait_vm<NG>();         // own share of tile t+1 (only the copy of tile t+2 is younger)
      wg_barrier();
    }
    if (late) {
      dot(0, t1 - 1);
      dot(1, t1 - 1);
      if (t1 - 2 >= t0) head_sum(t1 - 2);
    } else {
      head_sum(t1 - 1);
    }
    wg_barrier();
    if (late) head_sum(t1 - 1);
    wait_vm<0>();            // no copy may land in LDS after the workgroup has gone
  };
  if constexpr (WPH == 1) {
    body(std::integral_constant<int, 0>{});
  } else {
    if (pr == 0) body(std::integral_constant<int, 0>{});
    else body(std::integral_constant<int, 1>{});
  }
}

// ------------------------------------------------------------------------------------------
// Attention pass, pipelined: per key split, champion-excluded online softmax statistics and
// A.V sums (outputs: the per-split statistics described in score_common.hpp).
// grid (S, row blocks, Hkv), 512 threads.
//
// K tiles travel through a 3-deep, V tiles through a 4-deep asynchronous LDS ring.  A step t has a
// matrix half (P.V of tile t-1, then Q.K of tile t: 48 MFMAs) and a vector half (softmax
// bookkeeping of tile t).  Every wavefront passes ONE workgroup barrier per step: wavefronts 0..3
// after the vector half, wavefronts 4..7 between the halves, so that the two wavefronts of a SIMD
// alternate between the matrix cores and the vector ALUs without meeting twice per tile.  With
// B_t the barrier of step t: K tile t and V tile t-1 are read between B_t-1 and B_t+1 at the
// latest by the matrix halves of step t (early wavefronts: before B_t, late ones: before their
// B_t too); the copy of tile t+2 is issued at the top of step t, after B_t-1, into the K slot of
// tile t-1 and the V slot of tile t-2, both last read by a matrix half that precedes B_t-1; every
// wavefront waits for its share of tile t+1 (only tile t+2 is younger) before its B_t, the first
// barrier after which tile t+1 is read.
template <int D>
__global__ __launch_bounds__(512) void k_attn_pipe(Prob pb, const uint16_t* __restrict__ q,
                                                   const uint16_t* __restrict__ k,
                                                   const uint16_t* __restrict__ v, int S, int kps,
                                                   int log2iw, ScorePtrs o) {
  constexpr int NW = 8, KS = D / 16, CB = D / 32;
  using RingK = TileRing<D, 0>;
  using RingV = TileRing<D, 1>;
  constexpr int NG = 2 * (RingK::NI / NW);          // copies per wavefront and tile
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[3][TN * D];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[4][TN * D];

  const int s = blockIdx.x, g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = wave_index(), rr = l & 31, hf = l >> 5;
  const RowInfo ri = row_info(pb, g, blockIdx.y * NW + wv, l, log2iw);
  const uint16_t* kg = k + (int64_t)g * pb.kv_sh;
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;

  const int kbeg = s * kps;
  const int kend = min(pb.L, kbeg + kps);
  const int ntiles = kend > kbeg ? (kend - kbeg + TN - 1) / TN : 0;
  const uint32_t pitch = (uint32_t)pb.kv_st * 2u;
  uint32_t koff[NG / 2], voff[NG / 2];
  RingK::template plan<NW>(pitch, wv, l, koff);
  RingV::template plan<NW>(pitch, wv, l, voff);
  const uint32_t ks_base = lds_addr(&Ks[0][0]), vs_base = lds_addr(&Vs[0][0]);
  auto issue_tile = [&](int t) {
    const int kb = kbeg + min(t, ntiles - 1) * TN;   // past the end: harmless repeat into a free slot
    if (kb + TN <= pb.L) {
      const uint64_t tb = (uint64_t)kb * pitch;
      RingK::template issue_whole<NW>((const char*)kg + tb, koff, ks_base + (uint32_t)(t % 3) * (TN * D * 2), wv);
      RingV::template issue_whole<NW>((const char*)vg + tb, voff, vs_base + (uint32_t)(t & 3) * (TN * D * 2), wv);
    } else {
      RingK::template issue<NW>(kg, pitch, kb, pb.L, Ks[t % 3], wv, l);
      RingV::template issue<NW>(vg, pitch, kb, pb.L, Vs[t & 3], wv, l);
    }
  };
  if (ntiles > 0) {
    issue_tile(0);
    issue_tile(1);
  }

  bf16x8 qf[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {       // an absent row re-reads row (h, 0) and is masked: no branch around the loads
    const uint4 u = *(const uint4*)(q + (int64_t)ri.h * pb.q_sh + (int64_t)(ri.valid ? ri.i : 0) * pb.q_st + 16 * ks + 8 * hf);
    qf[ks] = as_bf16x8(ri.valid ? u : make_uint4(0, 0, 0, 0));
  }
  const int vis_last = (pb.causal && ri.valid) ? pb.P + ri.i : pb.L - 1;
  const float c2 = pb.scale * LOG2E;

  float mall = -INFINITY, mref = -INFINITY, mx = -INFINITY, lsum = 0.f;
  int nx = -1;                       // key kept out of the sums, -1: none
  f32x16 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; ++cb)
#pragma unroll
    for (int j = 0; j < 16; ++j) oacc[cb][j] = 0.f;
  bf16x8 pv[2][2];

  // lane-constant part of the transposing LDS read of the value tile: row and column of the
  // 8 bytes this lane contributes to a 16 x 16 block
  const int s16 = l & 15;
  const int vrow = 4 * hf + (s16 >> 2), vcol = 16 * ((l >> 4) & 1) + 4 * (s16 & 3);

  // P.V of one tile: O^T[c, row] += V^T P^T.  The transposing reads of the next 16-key group are
  // issued before the MFMAs of the current one, so the matrix cores do not wait one LDS round
  // trip per MFMA.
  auto accumulate = [&](const uint16_t* vt) {
    auto fetch = [&](int grp, bf16x8 (&av)[CB]) {       // grp = 2 mb + kg2
      const int r0 = 16 * grp + vrow;
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) {
        const int col = 32 * cb + vcol;
        const uint16_t* base = vt + RingV::off(r0, col >> 3) + (col & 7);   // rows r0 and r0+8 share the XOR key
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(base));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(base + 8 * D));
        union { s16x8 s; bf16x8 b; } a;
        a.s = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        av[cb] = a.b;
      }
    };
    bf16x8 av[2][CB];
    fetch(0, av[0]);
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      if (grp + 1 < 4) fetch(grp + 1, av[(grp + 1) & 1]);
#pragma unroll
      for (int cb = 0; cb < CB; ++cb) oacc[cb] = MFMA(av[grp & 1][cb], pv[grp >> 1][grp & 1], oacc[cb]);
    }
  };

  if (ntiles > 0) {
    wait_vm<NG>();           // own share of tile 0
    wg_barrier();            // B_-1
    const bool late = wv >= NW / 2;

    for (int t = 0; t < ntiles; ++t) {
      const int kb = kbeg + t * TN;
      issue_tile(t + 2);     // into the K slot of tile t-1 and the V slot of tile t-2, both last read before B_t-1
      __builtin_amdgcn_s_setprio(0);
      // ---- matrix half: P.V of the previous tile, logits S^T[key, row] = K Q^T of this one ----
      if (t > 0) accumulate(Vs[(t - 1) & 3]);
      const uint16_t* kt = Ks[t % 3];
      f32x16 sacc[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int j = 0; j < 16; ++j) sacc[mb][j] = 0.f;
      // operand reads in batches of eight ahead of their MFMAs (one LDS round trip per batch)
#pragma unroll
      for (int k0 = 0; k0 < KS; k0 += 4) {
        bf16x8 a[4][2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
            a[ks][mb] = as_bf16x8(*(const uint4*)&kt[RingK::off(32 * mb + rr, 2 * (k0 + ks) + hf)]);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
          for (int mb = 0; mb < 2; ++mb) sacc[mb] = MFMA(a[ks][mb], qf[k0 + ks], sacc[mb]);
      }
      __builtin_amdgcn_s_setprio(2);
      if (late) {            // B_t of the late wavefronts: between the halves
        wait_vm<NG>();       // own share of tile t+1 (only the copies of tile t+2 are younger)
        wg_barrier();
      }
      // ---- vector half ----
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
      // (only one wavefront of the SIMD is in its vector half: independent chains, not one long one)
      float tq[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        tq[c] = fmaxf(fmaxf(sacc[0][c], sacc[0][4 + c]), sacc[0][8 + c]);
        tq[c] = fmaxf(fmaxf(tq[c], sacc[0][12 + c]), sacc[1][c]);
        tq[c] = fmaxf(fmaxf(tq[c], sacc[1][4 + c]), sacc[1][8 + c]);
        tq[c] = fmaxf(tq[c], sacc[1][12 + c]);
      }
      float tm = xhalf_max(fmaxf(fmaxf(tq[0], tq[1]), fmaxf(tq[2], tq[3])));

      // A key is kept out of the sums only if, on arrival, it is the largest so far AND holds
      // more than half of the mass seen so far (what a key that ends with A > 1/2 always does);
      // such keys are rare after the first tile, so the expensive part of the bookkeeping (index
      // search, folding the previous kept-out key back in) almost never runs.  The weights that enter the P.V product are rounded to bf16;
      // that costs nothing where a key holds a small share of the sums, and would cost up to
      // 2^-9 of a heavy key's share.  So the reference of the exponentials is always a logit that
      // is PART of the sums (never the kept-out key's, which may be any distance above), it is
      // moved exactly onto the largest joining logit of a tile whenever that key is heavy among
      // the others (its weight is then exactly 1, which bf16 holds), and lazily otherwise.
      const bool newmax = tm > mall;
      const float pl = __builtin_amdgcn_exp2f((tm - mref) * c2);   // tile maximum in the current frame (inf on the first tile)
      mall = fmaxf(mall, tm);
      // Nothing to do unless the reference has to move or the tile maximum may be heavy: lsum is
      // this lane's share of the row's sum, so the comparison is a necessary condition for both
      // "kept out" and "heavy", which are settled below.
      if (__ballot((tm - mref) * c2 > RESCALE_TH || pl * 8.0f > lsum) != 0ull) {
        const float oth = xhalf_sum(lsum);
        bool dominant = false;
        if (newmax) {
          float total = oth;
          if (nx >= 0) total += __builtin_amdgcn_exp2f((mx - mref) * c2);
          // total = inf: the key kept out so far is the whole mass in FP32, and tm is above it
          dominant = pl > total || total == INFINITY;
        }
        float tinc = tm;                 // largest logit of the tile that joins the sums
        int cand = INT_MAX;
        if (__ballot(dominant) != 0ull) {
          if (dominant) {
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
              for (int j = 0; j < 16; ++j)
                if (sacc[mb][j] == tm) cand = min(cand, kb + 32 * mb + cidx(j, hf));
          }
          cand = xhalf_min(cand);
          // the new kept-out key leaves the tile: its weight below is exp2(-inf) = 0
          const int cz = dominant ? cand : -1;
#pragma unroll
          for (int mb = 0; mb < 2; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j)
              sacc[mb][j] = (kb + 32 * mb + cidx(j, hf)) == cz ? -INFINITY : sacc[mb][j];
          float u[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            u[c] = fmaxf(fmaxf(sacc[0][c], sacc[0][4 + c]), sacc[0][8 + c]);
            u[c] = fmaxf(fmaxf(u[c], sacc[0][12 + c]), sacc[1][c]);
            u[c] = fmaxf(fmaxf(u[c], sacc[1][4 + c]), sacc[1][8 + c]);
            u[c] = fmaxf(u[c], sacc[1][12 + c]);
          }
          tinc = xhalf_max(fmaxf(fmaxf(u[0], u[1]), fmaxf(u[2], u[3])));
        }
        // Where nothing of the tile joins (one visible key, and it is kept out) the reference
        // stays; a row without any reference yet takes the kept-out key's logit (any finite
        // value will do: its sums are empty).
        float tref = mref;
        if (tinc == -INFINITY) {
          if (mref == -INFINITY) tref = tm;
        } else {
          const float pinc = tinc == tm ? pl : __builtin_amdgcn_exp2f((tinc - mref) * c2);   // inf without a reference
          if (pinc * 8.0f > oth || (tinc - mref) * c2 > RESCALE_TH) tref = tinc;
        }
        // The key kept out so far joins the sums too (in FP32, below): the reference may not
        // stay far under it, however far it lies above the rest.
        if (dominant && nx >= 0 && (mx - tref) * c2 > RESCALE_TH) tref = mx;
        if (tref != mref) {
          const float f = __builtin_amdgcn_exp2f((mref - tref) * c2);   // first tile: 2^-inf = 0
          lsum *= f;
#pragma unroll
          for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int j = 0; j < 16; ++j) oacc[cb][j] *= f;
          mref = tref;
        }
        if (dominant) {
          if (nx >= 0) {               // the key kept out so far joins the running sums, in FP32
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
      }
      // ---- weights relative to the reference ----
      const float nm = -mref * c2;
      {
        float ls[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int b8 = 0; b8 < 16; b8 += 8) {
            float pe[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) pe[e] = fmaf(sacc[mb][b8 + e], c2, nm);
#pragma unroll
            for (int e = 0; e < 8; ++e) pe[e] = __builtin_amdgcn_exp2f(pe[e]);
#pragma unroll
            for (int e = 0; e < 8; ++e) ls[e & 3] += pe[e];
#pragma unroll
            for (int e = 0; e < 8; ++e) pv[mb][b8 >> 3][e] = (__bf16)pe[e];
          }
        lsum += (ls[0] + ls[1]) + (ls[2] + ls[3]);
      }
      if (!late) {           // B_t of the early wavefronts: after both halves
        wait_vm<NG>();
        wg_barrier();
      }
    }
    accumulate(Vs[(ntiles - 1) & 3]);   // its slot is not a target of the copies still in flight
    wait_vm<0>();            // no copy may land in LDS after the workgroup has gone
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
// Score pass: logits again, cross term u.v_n, closed form, mean over the group.
// grid (key chunks, row blocks, Hkv), 512 threads = 8 wavefronts of 32 query rows each.
//
// Per element (query row r of head h, key n), with M, l, zz the row's softmax maximum,
// denominator and z M_h z^T from the attention pass:
//   a = 2^(s c2 - M - log2(G l)) = A / G,   den = 1 - G a = 1 - A,
//   x = vv[h,n] - 2 (u.v_n - zz/2),          I/G = a sqrt(x) / den = a x rsq(x den^2)
// (1/G of the group mean and 1/l are folded into the exponent, zz/2 into the accumulator's
// start value).  Here the query rows sit on the M side of the MFMA and the keys on the N side:
// a lane owns ONE key of each 32-key block and 16 query rows, ordered so that the heads of a
// group that share a window position are consecutive registers of one lane (local row =
// position * Gp + head).  The group mean is then a few in-lane adds (plus one half swap from
// Gp = 8 on), and a store instruction writes 32 consecutive keys of a row.
//
// Schedule:
//   * K, V and vv tiles arrive through a 3-deep (vv: 4-deep) asynchronous LDS ring, two tiles
//     ahead of their use, so no wavefront waits on a global load in the steady state;
//   * every tile has a matrix half-step (48 MFMAs per wavefront) and a vector half-step
//     (closed form, group mean, stores) separated by workgroup barriers, and wavefronts 4..7
//     run ONE half-step behind wavefronts 0..3 (they pass one extra barrier before the loop,
//     the others one extra after it).  The two wavefronts of a SIMD are therefore always in
//     different half-steps: one feeds the matrix cores while the other uses the vector ALUs;
//   * a workgroup walks a long run of tiles, so the per-row setup is paid once.
// Ring safety, with barriers E_0, E_1, ... and tile t handled by the early half in
// (E_2t, E_2t+2) and by the late half in (E_2t+1, E_2t+3):  the copy of tile t+2 is issued at
// the top of a wavefront's step t, i.e. after E_2t at the earliest, into the K/V slot of tile
// t-1 (last read before E_2t) and the vv slot of tile t-2 (last read before E_2t-1); each
// wavefront waits for its own share of tile t+1 before its mid-step barrier, which for both
// halves precedes E_2t+2, the first barrier after which tile t+1 is read.
// MODE 0: the pass as described.
// MODE 1: sample pass.  The "tiles" are made of fa.ns sampled prefix keys (runs of 16 consecutive
//         keys, evenly spread); their scores go to fa.smp [Hkv*W, fa.ns] instead of `score`.
// MODE 2: fused pass (needs Gp >= 4, one row block).  Besides writing `score`, the vector
//         half-step feeds the temporal and the spatial smoothing so that nothing has to read the
//         raw score again:
//   * EMA over the window queries as a weighted sum (weights of Sec. 3.3 unrolled): partial sums
//     per wavefront meet in LDS, one wavefront writes fa.ema for the tile two steps later;
//   * per (head, query) row and lane: count and position sum of the scores above the row's
//     bracket fa.thr (registers, reduced once at the end into fa.cnt_hi / fa.sum_hi);
//   * scores inside the bracket go, with their position and row, to a compact LDS list of the
//     wavefront (places from a prefix sum over the lanes' counts); every 32 tiles, and when the
//     list would overflow, the wavefront flushes it into the slices fa.sval / fa.sidx
//     [row, key chunk = blockIdx.x, fa.caps] that only it writes (ranks by wave ballots, no
//     atomics, deterministic); the slice fill counts go to fa.scnt at the end.
struct FuseArgs {
  float* smp; int ns; int ns_tiles; double step;
  const float2* thr; uint32_t* cnt_hi; unsigned long long* sum_hi;
  uint32_t* scnt; float* sval; int* sidx; int caps;
  float* ema; float alpha;
};
constexpr int FUSE_CAPL = 512;       // candidate list entries per wavefront (a tile adds at most 512)

template <int D, int GP, int MODE>
__global__ __launch_bounds__(512) void k_score_pipe(Prob pb, const uint16_t* __restrict__ q,
                                                    const uint16_t* __restrict__ k,
                                                    const uint16_t* __restrict__ v, ScorePtrs o, int ldv,
                                                    float* __restrict__ score, int tiles_per_wg, int nwb,
                                                    FuseArgs fa) {
  constexpr int NW = 8, KS = D / 16, LG = ilog2(GP), IW = 32 / GP;
  static_assert(MODE != 2 || GP == 4 || GP == 8, "the fused pass keeps at most four rows per lane and needs LDS for its lists");
  constexpr int GV = GP < 4 ? 4 : GP;               // vv rows per ring slot (whole 1 KiB copies)
  constexpr int NVB = GV / 4;                       // 1 KiB copies per vv tile
  constexpr int ND = GP <= 4 ? GP : GP / 2;         // distinct heads among a lane's 16 registers
  using Ring = TileRing<D>;
  constexpr int NG = 2 * (Ring::NI / NW) + 1;       // copies per wavefront and tile
  __shared__ __attribute__((aligned(1024))) uint16_t Ks[3][TN * D];
  __shared__ __attribute__((aligned(1024))) uint16_t Vs[3][TN * D];
  __shared__ __attribute__((aligned(1024))) float vvs[4][GV][TN];
  __shared__ __attribute__((aligned(16))) float rowc[NW][4][32];   // per local row: accumulator start values, champion key and score
  constexpr int FL = MODE == 2 ? FUSE_CAPL : 1;
  __shared__ float fval[NW][FL];                    // MODE 2: candidate list of each wavefront, value ...
  __shared__ uint32_t fpos[NW][FL];                 // ... and position | row slot << 29 | lane half << 31
  __shared__ __attribute__((aligned(16))) uint32_t fcnt[NW][8];   // MODE 2: slice fill count of each wavefront's rows
  __shared__ __attribute__((aligned(16))) float frow[NW][3][8];   // MODE 2: per row (slot + 4 half): bracket lo, hi, EMA weight
  __shared__ float epart[2][NW][TN];                // MODE 2: EMA partial sums of two tiles

  const int g = blockIdx.z;
  const int l = threadIdx.x & 63, wv = threadIdx.x >> 6, rr = l & 31, hf = l >> 5;
  const int wvs = wave_index();                     // the same as a scalar, for the copies' addresses
  const int wb = blockIdx.y * NW + wv;              // block of IW window positions
  const uint16_t* kg = k + (int64_t)g * pb.kv_sh;
  const uint16_t* vg = v + (int64_t)g * pb.kv_sh;

  const int NT = MODE == 1 ? fa.ns_tiles : (pb.P + TN - 1) / TN;
  const int t0 = blockIdx.x * tiles_per_wg;
  const int t1 = min(NT, t0 + tiles_per_wg);
  if (t0 >= t1) return;
  // MODE 1: sample j (tile j / 64, row j % 64) is key start(j / 16) + j % 16, the starts evenly
  // spread over the prefix and multiples of 4 (a vv copy moves 4 keys)
  auto key_of = [&](int j) { return min((int)((double)(j >> 4) * fa.step) & ~3, pb.P - 16) + (j & 15); };

  // vv copy of this wavefront: block wv % NVB (duplicates write identical bytes)
  const int vb = wvs % NVB;
  const float* vv_g = o.vv + (int64_t)g * pb.G * ldv;                    // vv rows of this group
  const uint32_t vv_row = (uint32_t)min(4 * vb + (l >> 4), pb.G - 1) * (uint32_t)ldv;
  const uint32_t pitch = (uint32_t)pb.kv_st * 2u;
  uint32_t kvoff[(NG - 1) / 2];
  Ring::template plan<NW>(pitch, wvs, l, kvoff);
  const uint32_t vvoff = (vv_row + 4u * (uint32_t)(l & 15)) * 4u;
  const uint32_t ks_base = lds_addr(&Ks[0][0]), vs_base = lds_addr(&Vs[0][0]), vv_base = lds_addr(&vvs[0][0][0]);
  auto issue_tile = [&](int t) {
    const int tt = min(t, t1 - 1);                  // past the end: harmless repeat into a free slot
    const int kb = tt * TN;
    if constexpr (MODE == 1) {
      Ring::template issue_rows<NW>(kg, pitch, [&](int r) { return key_of(kb + r); }, Ks[t % 3], wv, l);
      Ring::template issue_rows<NW>(vg, pitch, [&](int r) { return key_of(kb + r); }, Vs[t % 3], wv, l);
      dma_1k(vv_g, (vv_row + (uint32_t)key_of(kb + 4 * (l & 15))) * 4u, &vvs[t & 3][4 * vb][0]);
    } else if (kb + TN <= pb.L && kb + TN <= ldv) {   // whole tile, no clamp anywhere
      const uint64_t tb = (uint64_t)kb * pitch;
      const uint32_t slot = (uint32_t)(t % 3) * (TN * D * 2);
      Ring::template issue_whole<NW>((const char*)kg + tb, kvoff, ks_base + slot, wvs);
      Ring::template issue_whole<NW>((const char*)vg + tb, kvoff, vs_base + slot, wvs);
      dma_1k_to(vv_g + kb, vvoff, vv_base + (uint32_t)((t & 3) * GV + 4 * vb) * (TN * 4));
    } else {
      Ring::template issue<NW>(kg, pitch, kb, pb.L, Ks[t % 3], wv, l);
      Ring::template issue<NW>(vg, pitch, kb, pb.L, Vs[t % 3], wv, l);
      dma_1k(vv_g, (vv_row + (uint32_t)min(kb + 4 * (l & 15), ldv - 4)) * 4u, &vvs[t & 3][4 * vb][0]);
    }
  };
  issue_tile(t0);          // ring indices run on the absolute tile number
  issue_tile(t0 + 1);

  // A operands: local row rr = position * GP + head
  const float c2 = pb.scale * LOG2E;
  // Gf: what the exponent and the leave-one-out value fold in (G for the mean over the group,
  // 1 for the maximum); Gd: the factor in 1 - A (0 for the indicators without 1 / (1 - A))
  const float Gf = pb.gmax ? 1.f : (float)pb.G, invG = 1.f / Gf;
  const float Gd = pb.ind != 0 ? 0.f : Gf;
  bf16x8 qf[KS], uhi[KS], ulo[KS];
  int nslane = -1;                                   // champion key of local row rr (for the tile test)
  {
    const int head = rr & (GP - 1), i = wb * IW + (rr >> LG);
    const bool valid = head < pb.G && i < pb.W;
    const int h = g * pb.G + (valid ? head : 0);
    const int row = h * pb.W + (valid ? i : 0);
    // operand-ordered copies left by the merge kernel: one 1 KiB run per wavefront and register
    const int64_t plane = (int64_t)pb.Hkv * nwb * (KS * 2 * 32 * 8);
    const uint16_t* ob = o.op + (((int64_t)(g * nwb + wb) * KS * 2 + hf) * 32 + rr) * 8;
    // (loaded whether the row exists or not, then masked: the buffer holds every padded row,
    // and unconditional loads are all in flight together)
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const uint16_t* pk = ob + ks * (2 * 32 * 8);
      const uint4 a = *(const uint4*)pk;
      const uint4 b = *(const uint4*)(pk + plane);
      const uint4 c = *(const uint4*)(pk + 2 * plane);
      qf[ks] = as_bf16x8(valid ? a : zero4);
      uhi[ks] = as_bf16x8(valid ? b : zero4);
      ulo[ks] = as_bf16x8(valid ? c : zero4);
    }
    // Start values of the two accumulators of this row, so that the MFMAs deliver
    //   s + (-M - log2(G l)) / c2   and   u.v_n - zz/2   directly.
    // An idle row starts at -inf (its q is zero): its exponential, hence its score, is exactly 0.
    if (valid) nslane = o.rs_nstar[row];
    if (hf == 0) {
      rowc[wv][0][rr] = valid ? (-o.rs_m[row] - log2f(Gf * o.rs_l[row])) / c2 : -INFINITY;
      rowc[wv][1][rr] = valid ? -0.5f * o.rs_zz[row] : 0.f;
      rowc[wv][2][rr] = __int_as_float(nslane);
      rowc[wv][3][rr] = valid ? o.rs_istar[row] * invG : 0.f;
    }
  }
  const float* vvlane = &vvs[0][0][0] + rr;
  // Output a of a lane (after the group mean) belongs to window position i0 + out_pos0(a):
  //   Gp <= 4: registers Gp a .. Gp a + Gp - 1, local row 8 (Gp a / 4) + 4 hf + (Gp a) % 4;
  //   Gp 8, 16: position 2 a + hf after the half swap;   Gp 32: position 0 in both halves.
  constexpr int NOUT = GP <= 4 ? 16 / GP : (GP == 8 ? 2 : 1);
  constexpr int HS = GP <= 4 ? 4 / GP : (GP == 32 ? 0 : 1);   // position step between the lane halves
  auto out_pos0 = [](int a) constexpr {
    return GP <= 4 ? (8 * ((GP * a) >> 2) + ((GP * a) & 3)) >> LG : 2 * a;
  };
  const int i0 = wb * IW + hf * HS;
  const bool rows_full = wb * IW + IW <= pb.W;       // wave-uniform: every position of the block exists
  char* sbase = (char*)(score + (int64_t)g * pb.W * pb.ld);
  const uint32_t ld4 = (uint32_t)pb.ld * 4u;
  const uint32_t voff0 = (uint32_t)i0 * ld4 + (uint32_t)rr * 4u;   // 32-bit: checked on the host
  // MODE 2: running statistics of this lane's output rows; brackets and EMA weights of the
  // wavefront's rows sit in LDS (frow)
  uint32_t hc[NOUT], hsm[NOUT];
  uint32_t wcount = 0;                               // entries in this wavefront's list (wave-uniform)
  if constexpr (MODE == 2) {
#pragma unroll
    for (int a = 0; a < NOUT; ++a) { hc[a] = 0; hsm[a] = 0; }
    if (l < 8) {                                     // row l & 3 of lane half l >> 2
      const int i = wb * IW + out_pos0(l & 3) + (l >> 2) * HS;
      const bool ok = (l & 3) < NOUT && i < pb.W;
      const float2 th = ok ? fa.thr[g * pb.W + i] : make_float2(INFINITY, INFINITY);
      frow[wv][0][l] = th.x;
      frow[wv][1][l] = th.y;
      // e_W-1 = sum_i w_i I_i with w_0 = (1-alpha)^(W-1), w_i = alpha (1-alpha)^(W-1-i)
      frow[wv][2][l] = ok ? (i == 0 ? 1.f : fa.alpha) * powf(1.f - fa.alpha, (float)(pb.W - 1 - i)) : 0.f;
      fcnt[wv][l] = 0;
    }
  }
  const unsigned long long lanes_below = (1ull << l) - 1ull;
  // MODE 2: list -> slices, 64 entries at a time; the entries of one row (tag = slot + 4 * lane
  // half in the top bits of the position word) are ranked with a ballot.  Only this wavefront
  // touches its list, its counts and its rows' slices.
  auto flush = [&]() {
    if constexpr (MODE == 2) {
      uint32_t cn[8];                          // fill counts of the wavefront's 8 rows (wave-uniform)
      {
        const uint4 c0 = *(const uint4*)&fcnt[wv][0], c1 = *(const uint4*)&fcnt[wv][4];
        cn[0] = c0.x; cn[1] = c0.y; cn[2] = c0.z; cn[3] = c0.w;
        cn[4] = c1.x; cn[5] = c1.y; cn[6] = c1.z; cn[7] = c1.w;
      }
      const int caps = fa.caps;
      float* const sval = fa.sval;
      int* const sidx = fa.sidx;
      for (uint32_t c0 = 0; c0 < wcount; c0 += 64) {
        const bool have = c0 + (uint32_t)l < wcount;
        const uint32_t pe = have ? fpos[wv][c0 + l] : 0u;
        const float ve = have ? fval[wv][c0 + l] : 0.f;
        const int tag = have ? (int)(pe >> 29) : -1;          // slot | half << 2
        uint32_t ps = 0;
#pragma unroll
        for (int r8 = 0; r8 < 8; ++r8) {
          const unsigned long long mk = __ballot(tag == r8);
          if (tag == r8) ps = cn[r8] + (uint32_t)__popcll(mk & lanes_below);
          cn[r8] += (uint32_t)__popcll(mk);
        }
        if (have && ps < (uint32_t)caps) {
          const int i = wb * IW + 2 * (tag & 3) + (tag >> 2) * HS;     // out_pos0(a) = 2 a for Gp >= 4
          const int64_t so = ((int64_t)(g * pb.W + i) * gridDim.x + blockIdx.x) * caps + ps;
          sval[so] = ve;
          sidx[so] = (int)(pe & 0x1FFFFFFFu);
        }
      }
      if (l == 0) {
        *(uint4*)&fcnt[wv][0] = make_uint4(cn[0], cn[1], cn[2], cn[3]);
        *(uint4*)&fcnt[wv][4] = make_uint4(cn[4], cn[5], cn[6], cn[7]);
      }
      wcount = 0;
    }
  };

  wait_vm<NG>();           // own share of tile t0
  wg_barrier();            // E_2t0
  const bool late = wv >= NW / 2;
  if (late) wg_barrier();

  for (int t = t0; t < t1; ++t) {
    // The wavefront in its vector half-step goes first at the issue port: it is the one with many
    // short instructions, and the half-step that bounds the tile time; the MFMAs of the other
    // wavefront of the SIMD need one issue slot in eight and find it in the gaps (measured: 1.4 %
    // against the opposite order, which is how the kernel was first written).
    __builtin_amdgcn_s_setprio(0);
    issue_tile(t + 2);
    if constexpr (MODE == 2) {
      // tile t-2: every wavefront left its partial sum before the barrier just passed
      if (wv == 0 && t - 2 >= t0) {
        const int n = (t - 2) * TN + l;
        float e = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) e += epart[t & 1][w2][l];
        if (n < pb.P) fa.ema[(int64_t)g * pb.ld + n] = e;
      }
    }
    // ---- matrix half-step ----
    const uint16_t* kt = Ks[t % 3];
    const uint16_t* vt = Vs[t % 3];
    f32x16 sacc[2], cacc[2];
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const f32x4 s0 = *(const f32x4*)&rowc[wv][0][8 * a + 4 * hf];
      const f32x4 c0 = *(const f32x4*)&rowc[wv][1][8 * a + 4 * hf];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sacc[0][4 * a + e] = s0[e]; sacc[1][4 * a + e] = s0[e];
        cacc[0][4 * a + e] = c0[e]; cacc[1][4 * a + e] = c0[e];
      }
    }
    // consecutive MFMAs never touch the same accumulator
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int of0 = Ring::off(rr, 2 * ks + hf), of1 = Ring::off(32 + rr, 2 * ks + hf);
      const bf16x8 bk0 = as_bf16x8(*(const uint4*)&kt[of0]);
      const bf16x8 bv0 = as_bf16x8(*(const uint4*)&vt[of0]);
      const bf16x8 bk1 = as_bf16x8(*(const uint4*)&kt[of1]);
      const bf16x8 bv1 = as_bf16x8(*(const uint4*)&vt[of1]);
      sacc[0] = MFMA(qf[ks], bk0, sacc[0]);
      cacc[0] = MFMA(uhi[ks], bv0, cacc[0]);
      sacc[1] = MFMA(qf[ks], bk1, sacc[1]);
      cacc[1] = MFMA(uhi[ks], bv1, cacc[1]);
      cacc[0] = MFMA(ulo[ks], bv0, cacc[0]);
      cacc[1] = MFMA(ulo[ks], bv1, cacc[1]);
    }
    wait_vm<NG>();         // own share of tile t+1 (only the copies of tile t+2 are younger)
    wg_barrier();
    __builtin_amdgcn_s_setprio(2);
    // ---- vector half-step ----
    const int kb = t * TN;
    const float* vvt = vvlane + (t & 3) * (GV * TN);
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) {
      float vvh[ND];
#pragma unroll
      for (int jd = 0; jd < ND; ++jd)
        vvh[jd] = vvt[((8 * (jd >> 2) + 4 * hf + (jd & 3)) & (GP - 1)) * TN + 32 * mb];
      // stage by stage over 8 registers: eight independent chains in flight
#pragma unroll
      for (int b8 = 0; b8 < 16; b8 += 8) {
        float a[8], x[8], den[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = sacc[mb][b8 + e] * c2;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = fmaf(-2.f, cacc[mb][b8 + e], vvh[(b8 + e) % ND]);
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = __builtin_amdgcn_exp2f(a[e]);
#pragma unroll
        for (int e = 0; e < 8; ++e) den[e] = fmaf(-Gd, a[e], 1.f);
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] *= fabsf(x[e]);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = fabsf(x[e]) * den[e];
        // the tiny addend keeps rsq finite when x is exactly 0 (the score is then 0, not NaN)
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = fmaf(x[e], den[e], 1e-37f);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __builtin_amdgcn_rsqf(x[e]);
#pragma unroll
        for (int e = 0; e < 8; ++e) sacc[mb][b8 + e] = a[e] * x[e];
      }
    }
    // key of this lane in the two 32-key blocks of the tile
    int nk[2];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb) nk[mb] = MODE == 1 ? key_of(kb + 32 * mb + rr) : kb + 32 * mb + rr;
    bool champ_here = nslane >= kb && nslane < kb + TN;
    if constexpr (MODE == 1) {             // the tile is four runs of 16 keys
      champ_here = false;
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int s0 = key_of(kb + 16 * r4);
        champ_here = champ_here || (nslane >= s0 && nslane < s0 + 16);
      }
    }
    if (__ballot(champ_here) != 0ull) {    // a champion of this wavefront is here
#pragma unroll
      for (int j = 0; j < 16; ++j) {       // register j of lane half hf is local row 8 (j/4) + 4 hf + j%4
        const int m_ = 8 * (j >> 2) + 4 * hf + (j & 3);
        const int ns = __float_as_int(rowc[wv][2][m_]);
        const float is = rowc[wv][3][m_];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
          if (nk[mb] == ns) sacc[mb][j] = is;
      }
    }
    // ---- mean (or maximum) over the group (in-lane, one half swap from GP = 8 on), store ----
    float outv[2][NOUT];
    auto group_reduce = [&](auto maxc) {
      auto comb = [](float x, float y) { return decltype(maxc)::value ? fmaxf(x, y) : x + y; };
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        if constexpr (GP <= 4) {
#pragma unroll
          for (int a = 0; a < NOUT; ++a) {
            float s = sacc[mb][GP * a];
#pragma unroll
            for (int e = 1; e < GP; ++e) s = comb(s, sacc[mb][GP * a + e]);
            outv[mb][a] = s;
          }
        } else {
          constexpr int RPG = GP / 2;                 // registers per group inside one lane half
          float s[16 / RPG];
#pragma unroll
          for (int a = 0; a < 16 / RPG; ++a) {
            s[a] = sacc[mb][RPG * a];
#pragma unroll
            for (int e = 1; e < RPG; ++e) s[a] = comb(s[a], sacc[mb][RPG * a + e]);
          }
          if constexpr (16 / RPG >= 2) {
#pragma unroll
            for (int a = 0; a < 16 / RPG; a += 2) {
              // lower half ends up with the total of position a, upper half with that of a + 1
              const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(s[a]), __float_as_uint(s[a + 1]),
                                                              false, false);
              outv[mb][a / 2] = comb(__uint_as_float(r[0]), __uint_as_float(r[1]));
            }
          } else {
            // both halves hold (and store) the same total
            outv[mb][0] = decltype(maxc)::value ? xhalf_max(s[0]) : xhalf_sum(s[0]);
          }
        }
      }
    };
    if (pb.gmax) group_reduce(std::true_type{}); else group_reduce(std::false_type{});
    if constexpr (MODE == 1) {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int a = 0; a < NOUT; ++a)
          if (i0 + out_pos0(a) < pb.W)
            fa.smp[(int64_t)(g * pb.W + i0 + out_pos0(a)) * fa.ns + kb + 32 * mb + rr] = outv[mb][a];
    } else {
    const uint32_t toff = (uint32_t)kb * 4u;
    if (rows_full && kb + TN <= pb.P) {             // wave-uniform: no lane needs a guard
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int a = 0; a < NOUT; ++a)
          *(float*)(sbase + (voff0 + toff + (uint32_t)(128 * mb) + (uint32_t)out_pos0(a) * ld4)) = outv[mb][a];
    } else {
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int a = 0; a < NOUT; ++a)
          if (i0 + out_pos0(a) < pb.W && kb + 32 * mb + rr < pb.P)
            *(float*)(sbase + (voff0 + toff + (uint32_t)(128 * mb) + (uint32_t)out_pos0(a) * ld4)) = outv[mb][a];
    }
    }
    if constexpr (MODE == 2) {
      bool cin[2][NOUT];
      float tlo[4], thi[4], wq[4];
      {
        const f32x4 x0 = *(const f32x4*)&frow[wv][0][4 * hf], x1 = *(const f32x4*)&frow[wv][1][4 * hf],
                    x2 = *(const f32x4*)&frow[wv][2][4 * hf];
#pragma unroll
        for (int a = 0; a < 4; ++a) { tlo[a] = x0[a]; thi[a] = x1[a]; wq[a] = x2[a]; }
      }
#pragma unroll
      for (int mb = 0; mb < 2; ++mb) {
        const bool inp = nk[mb] < pb.P;            // keys past the prefix count for nothing
        // temporal smoothing: this lane's rows, the other lane half's, then LDS
        float es = 0.f;
#pragma unroll
        for (int a = 0; a < NOUT; ++a) es = fmaf(wq[a], outv[mb][a], es);
        if constexpr (HS != 0) es = xhalf_sum(es);
        if (hf == 0) epart[t & 1][wv][32 * mb + rr] = inp ? es : 0.f;
        // spatial statistics against the bracket of each row
#pragma unroll
        for (int a = 0; a < NOUT; ++a) {
          const float x = outv[mb][a];
          const bool hi = inp && x > thi[a];
          hc[a] += hi ? 1u : 0u;
          hsm[a] += hi ? (uint32_t)nk[mb] : 0u;
          cin[mb][a] = inp && x > tlo[a] && !hi;   // inside the bracket
        }
      }
      // candidates of this tile: a prefix sum over the lanes' counts (rotations-free DPP shifts
      // inside the 16-lane rows, the four row totals through scalar registers) gives every lane
      // its place in the wavefront's list
      uint32_t myc = 0;
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int a = 0; a < NOUT; ++a) myc += cin[mb][a] ? 1u : 0u;
      if (__ballot(myc != 0u) != 0ull) {            // wave-uniform
        uint32_t s = myc;
#define RK_SHR(n) s += __builtin_amdgcn_update_dpp(0u, s, 0x110 + (n), 0xF, 0xF, true)
        RK_SHR(1); RK_SHR(2); RK_SHR(4); RK_SHR(8);   // inclusive sums inside each row of 16 lanes
#undef RK_SHR
        const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)s, 15), r1 = (uint32_t)__builtin_amdgcn_readlane((int)s, 31),
                       r2 = (uint32_t)__builtin_amdgcn_readlane((int)s, 47), r3 = (uint32_t)__builtin_amdgcn_readlane((int)s, 63);
        const int lr = l >> 4;
        const uint32_t before = lr == 0 ? 0u : (lr == 1 ? r0 : (lr == 2 ? r0 + r1 : r0 + r1 + r2));
        const uint32_t tot = r0 + r1 + r2 + r3;
        if (wcount + tot > (uint32_t)FUSE_CAPL) flush();   // (rare: the regular flushes below keep the list short)
        uint32_t e = wcount + before + s - myc;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int a = 0; a < NOUT; ++a)
            if (cin[mb][a]) {
              fval[wv][e] = outv[mb][a];
              fpos[wv][e] = (uint32_t)nk[mb] | ((uint32_t)a << 29) | ((uint32_t)hf << 31);
              ++e;
            }
        wcount += tot;
      }
      // every wavefront empties its list at the same tiles, so that the workgroup pays for one
      // flush, not for eight at different barriers
      if (((t - t0) & 31) == 31 && wcount) flush();
    }
    wg_barrier();
  }
  if (!late) wg_barrier();
  wait_vm<0>();            // no copy may land in LDS after the workgroup has gone
  if constexpr (MODE == 2) {
    // the last two tiles' EMA (every partial sum is in LDS after the barriers above)
    if (wv == 0) {
      for (int t = max(t0, t1 - 2); t < t1; ++t) {
        const int n = t * TN + l;
        float e = 0.f;
#pragma unroll
        for (int w2 = 0; w2 < NW; ++w2) e += epart[t & 1][w2][l];
        if (n < pb.P) fa.ema[(int64_t)g * pb.ld + n] = e;
      }
    }
    flush();
    // per row: statistics over the 32 lanes of the half (rotations inside the 16-lane rows, one
    // row swap), slice fill count
#pragma unroll
    for (int a = 0; a < NOUT; ++a) {
      uint32_t c = hc[a];
      unsigned long long s = hsm[a];                // a lane's sum fits 32 bits (checked on the host)
#pragma unroll
      for (int sh = 1; sh < 32; sh <<= 1) {
        c += (uint32_t)__shfl_xor((int)c, sh, 64);
        s += ((unsigned long long)(uint32_t)__shfl_xor((int)(s >> 32), sh, 64) << 32) |
             (unsigned long long)(uint32_t)__shfl_xor((int)(uint32_t)s, sh, 64);
      }
      const int i = i0 + out_pos0(a);
      if (rr == 0 && i < pb.W) {
        const int row = g * pb.W + i;
        if (c) { atomicAdd(&fa.cnt_hi[row], c); atomicAdd(&fa.sum_hi[row], s); }
        fa.scnt[(int64_t)row * gridDim.x + blockIdx.x] = fcnt[wv][a + 4 * hf];
      }
    }
  }
}

// compute units of the current device (queried once)
int n_cu() {
  static int n = 0;
  if (n == 0) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

// geometry of the score pass: padded group size, row blocks, tiles per workgroup, key chunks
struct ScoreGeom { int gp, gy, tpp, chunks; };
ScoreGeom score_geom(const Prob& pb) {
  ScoreGeom s;
  s.gp = 1;
  while (s.gp < pb.G) s.gp <<= 1;
  const int iw = 32 / s.gp;
  const int nwr = (pb.W + iw - 1) / iw;            // wavefronts needed to cover the window
  s.gy = (nwr + 7) / 8;                            // row blocks of 8 wavefronts
  const int NT = (pb.P + TN - 1) / TN;
  s.tpp = (int)(((int64_t)NT * s.gy * pb.Hkv + n_cu() - 1) / n_cu());
  if (s.tpp < 1) s.tpp = 1;
  s.chunks = (NT + s.tpp - 1) / s.tpp;
  return s;
}

template <int D>
int run_mfma(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
             float* score, char* ws, const ScoreWs& lay, hipStream_t st, const FusedPtrs* fp) {
  const uint16_t* qq = (const uint16_t*)q;
  const uint16_t* kk = (const uint16_t*)k;
  const uint16_t* vp = (const uint16_t*)v;
  const ScorePtrs w = score_ptrs(ws, lay);
  int gp = 1;
  while (gp < pb.G) gp <<= 1;
  const int iw = 32 / gp, log2iw = ilog2(iw);
  const int nwr = (pb.W + iw - 1) / iw;            // wavefronts needed to cover the window
  const int gy = (nwr + 7) / 8;                    // row blocks of 8 wavefronts
  // attention pass: about one workgroup per compute unit, whole tiles per split
  int S = n_cu() / (pb.Hkv * gy);
  const int max_s = (pb.L + TN - 1) / TN;
  if (S > max_s) S = max_s;
  if (S > lay.S_max) S = lay.S_max;
  if (S < 1) S = 1;
  int kps = (pb.L + S - 1) / S;
  kps = (kps + TN - 1) / TN * TN;
  const float* part_z = w.part_z;
  if (pb.ext_lse) {
    // the caller's attention output and log-sum-exp stand in for the attention pass: one "split"
    S = 1;
    const int rows = pb.Hq * pb.W;
    RK_LAUNCH(ST_ATTN, st, (k_stats_fill<0>), dim3((rows + 255) / 256), dim3(256), 0, st, rows, pb.ext_lse,
              w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l);
    part_z = pb.ext_out;
  } else {
    RK_LAUNCH(ST_ATTN, st, (k_attn_pipe<D>), dim3(S, gy, pb.Hkv), dim3(512), 0, st, pb, qq, kk, vp, S, kps,
              log2iw, w);
  }
  if (pb.ind != 0) gram = nullptr;                 // the attention-weight and value-norm indicators have no projection
  RK_LAUNCH(ST_COMBINE, st, (k_attn_combine<bf16_t, D>), combine_grid(pb), combine_block<D>(), 0, st, pb,
            (const bf16_t*)v, S, gram, w.part_m, w.part_mx, w.part_n, w.part_ref, w.part_l, part_z, w.rs_m,
            w.rs_l, w.rs_zz, w.rs_nstar, w.rs_istar, w.rs_u, (const bf16_t*)q, w.op, ilog2(gp), lay.nwb, combine_groups(pb));
  if (gram) {
    constexpr int HPW = D == 128 ? 4 : 8;
    const int NTv = (pb.P + TN - 1) / TN;
    const int hg = (pb.G + HPW - 1) / HPW;
    int tpv = (int)(((int64_t)NTv * hg * pb.Hkv + n_cu() - 1) / n_cu());
    if (tpv < 1) tpv = 1;
    RK_LAUNCH(ST_VV, st, (k_vv_pipe<D>), dim3((NTv + tpv - 1) / tpv, hg, pb.Hkv), dim3(512), 0, st, pb, vp,
              gram, w.vv, lay.ldv, tpv);
  } else {
    RK_LAUNCH(ST_VV, st, (k_vnorm2<D>), dim3((pb.P + 255) / 256, pb.Hkv), dim3(256), 0, st, pb, vp,
              w.vv, lay.ldv);
  }
  // score pass: one resident workgroup per compute unit, each walking a run of tiles
  const ScoreGeom sg = score_geom(pb);
  const int tpp = sg.tpp;
  const dim3 g2(sg.chunks, sg.gy, pb.Hkv);
  FuseArgs fa = {};
#define RK_SCORE(GPV, MODE, GRID, TPW)                                                              \
  RK_LAUNCH(ST_SCORE, st, (k_score_pipe<D, GPV, MODE>), GRID, dim3(512), 0, st, pb, qq, kk, vp, w,  \
            lay.ldv, score, TPW, lay.nwb, fa)
  if (fp) {
    // sample pass -> brackets -> fused pass
    fa.smp = fp->smp; fa.ns = fp->ns; fa.ns_tiles = fp->ns / TN;
    fa.step = (double)(pb.P - 16) / (double)(fp->ns / 16 - 1);
    fa.thr = fp->thr; fa.cnt_hi = fp->cnt_hi; fa.sum_hi = fp->sum_hi;
    fa.scnt = fp->scnt; fa.sval = fp->sval; fa.sidx = fp->sidx; fa.caps = fp->caps;
    fa.ema = fp->ema; fa.alpha = pb.alpha;
    int tps = (int)(((int64_t)fa.ns_tiles * pb.Hkv + n_cu() - 1) / n_cu());
    if (tps < 1) tps = 1;
    const dim3 gs((fa.ns_tiles + tps - 1) / tps, 1, pb.Hkv);
    switch (sg.gp) {
      case 4: RK_SCORE(4, 1, gs, tps); break;
      case 8: RK_SCORE(8, 1, gs, tps); break;
      default: return RESTKV_EUNSUPPORTED;
    }
    const int rc = launch_bracket_samples(pb, fp->smp, fp->ns, fp->thr, fp->cnt_hi, fp->sum_hi, st);
    if (rc) return rc;
    switch (sg.gp) {
      case 4: RK_SCORE(4, 2, g2, tpp); break;
      case 8: RK_SCORE(8, 2, g2, tpp); break;
      default: return RESTKV_EUNSUPPORTED;
    }
    return hip_status();
  }
  switch (sg.gp) {
    case 1: RK_SCORE(1, 0, g2, tpp); break;
    case 2: RK_SCORE(2, 0, g2, tpp); break;
    case 4: RK_SCORE(4, 0, g2, tpp); break;
    case 8: RK_SCORE(8, 0, g2, tpp); break;
    case 16: RK_SCORE(16, 0, g2, tpp); break;
    case 32: RK_SCORE(32, 0, g2, tpp); break;
    default: break;
  }
#undef RK_SCORE
  return hip_status();
}

}  // namespace

bool mfma_eligible(const Prob& pb, const void* q, const void* k, const void* v) {
  if (pb.dtype != RESTKV_BF16) return false;
  if ((((uintptr_t)q | (uintptr_t)k | (uintptr_t)v) & 15u) != 0) return false;
  if ((pb.q_sh | pb.q_st | pb.kv_sh | pb.kv_st) & 7) return false;
  if (pb.G > 32) return false;
  // 32-bit byte offsets inside one head's K/V matrix and inside one group's vv rows
  if ((uint64_t)pb.L * (uint64_t)pb.kv_st * 2u >= (1ull << 32)) return false;
  if ((uint64_t)pb.G * (uint64_t)((pb.P + 3) / 4 * 4) * 4u >= (1ull << 32)) return false;
  if ((uint64_t)(pb.W + 32) * (uint64_t)pb.ld * 4u >= (1ull << 32)) return false;   // one head's score rows
  return true;
}

int launch_score_mfma(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
                      float* score, char* ws, const ScoreWs& lay, hipStream_t st) {
  return pb.d == 64 ? run_mfma<64>(pb, q, k, v, gram, score, ws, lay, st, nullptr)
                    : run_mfma<128>(pb, q, k, v, gram, score, ws, lay, st, nullptr);
}

int launch_score_fused(const Prob& pb, const void* q, const void* k, const void* v, const float* gram,
                       float* score, char* ws, const ScoreWs& lay, const FusedPtrs& fp, hipStream_t st) {
  return pb.d == 64 ? run_mfma<64>(pb, q, k, v, gram, score, ws, lay, st, &fp)
                    : run_mfma<128>(pb, q, k, v, gram, score, ws, lay, st, &fp);
}

int score_pass_chunks(const Prob& pb) { return score_geom(pb).chunks; }

bool fused_eligible(const Prob& pb, const void* q, const void* k, const void* v) {
  if (!mfma_eligible(pb, q, k, v) || !pb.adaptive) return false;
  if (pb.ind != 0 || pb.gmax || pb.tmode != 0 || pb.pmax) return false;
  const ScoreGeom sg = score_geom(pb);
  if (sg.gy != 1 || sg.gp < 4 || sg.gp > 8) return false;
  if (pb.P < 32768 || pb.P >= (1 << 29)) return false;          // sampling pays off; 29-bit positions
  if (2ull * (uint64_t)sg.tpp * (uint64_t)pb.P >= (1ull << 32)) return false;   // a lane's position sum
  if (sg.chunks > 256) return false;                             // slice directory of the finishing kernel
  return true;
}

}  // namespace restkv
