// Block-wide exact top-k of one row of floats held in global memory (gfx950, 64-wide waves).
//
// A radix select on the order-preserving integer image of the floats finds the
// value of the k-th largest element in three histogram passes (11 + 11 + 10
// bits); an ordered pass then visits the row once more in position order so
// that, among elements equal to the threshold, the lowest positions win.  The
// visitor either sums the selected positions or writes them out in ascending
// order.  The row is re-read from L2 on every pass; nothing is written but the
// result.
#pragma once

#include "common.hpp"

namespace restkv {

constexpr int SEL_NT = 1024;             // threads per block
constexpr int SEL_NW = SEL_NT / 64;      // wavefronts per block
constexpr int SEL_BINS = 2048;

struct SelectSmem {
  uint32_t hist[SEL_BINS];
  uint32_t wsum[SEL_NW];
  uint32_t cnt_gt[SEL_NW];
  uint32_t cnt_eq[SEL_NW];
  uint32_t bin, below, take;             // results of one digit search
  unsigned long long isum[SEL_NW];
};

// inclusive scan over the block of one value per thread (thread order)
__device__ __forceinline__ uint32_t block_incl_scan(uint32_t x, uint32_t* wsum) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(x, o, 64);
    if (lane >= o) x += y;
  }
  __syncthreads();
  if (lane == 63) wsum[w] = x;
  __syncthreads();
  uint32_t base = 0;
  for (int j = 0; j < w; ++j) base += wsum[j];
  return x + base;
}

// number of set bits of `ballot` below this lane
__device__ __forceinline__ uint32_t rank_in_ballot(unsigned long long ballot) {
  const uint32_t lane = threadIdx.x & 63;
  const unsigned long long below = lane ? (ballot & (~0ull >> (64 - lane))) : 0ull;
  return (uint32_t)__popcll(below);
}

// Threshold of the k-th largest (1 <= k <= n): on return `tau` is its key, `n_gt`
// the number of keys above it and `k_eq` how many keys equal to tau belong to the
// top k (>= 1).  All threads of the block must call; all receive the result.
__device__ inline void block_kth_key(const float* __restrict__ row, int n, int k, SelectSmem& sm,
                                     uint32_t& tau, uint32_t& n_gt, uint32_t& k_eq) {
  uint32_t prefix = 0, mask = 0, krem = (uint32_t)k, above = 0;
  const int shifts[3] = {21, 10, 0};
  const int nbits[3] = {11, 11, 10};
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int sh = shifts[pass];
    const uint32_t nb = 1u << nbits[pass];
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_NT) sm.hist[b] = 0;
    __syncthreads();
    for (int x = threadIdx.x; x < n; x += SEL_NT) {
      const uint32_t key = float_key(row[x]);
      if ((key & mask) == prefix) atomicAdd(&sm.hist[(key >> sh) & (nb - 1)], 1u);
    }
    __syncthreads();
    // bins in descending order: thread t owns the reversed bins 2t, 2t+1
    const int r0 = 2 * threadIdx.x, r1 = r0 + 1;
    const uint32_t h0 = r0 < (int)nb ? sm.hist[nb - 1 - r0] : 0;
    const uint32_t h1 = r1 < (int)nb ? sm.hist[nb - 1 - r1] : 0;
    const uint32_t incl = block_incl_scan(h0 + h1, sm.wsum);
    const uint32_t before = incl - (h0 + h1);
    if (before < krem && krem <= incl) {        // exactly one thread
      if (krem <= before + h0) { sm.bin = nb - 1 - r0; sm.below = before; }
      else                     { sm.bin = nb - 1 - r1; sm.below = before + h0; }
    }
    __syncthreads();
    prefix |= sm.bin << sh;
    mask |= (nb - 1) << sh;
    above += sm.below;
    krem -= sm.below;
    __syncthreads();
  }
  tau = prefix;
  n_gt = above;
  k_eq = krem;
}

// Visits row[0..n) in position order, wave after wave; f(position, selected_rank)
// is called for every selected element, ranks ascending with position.
// Returns through `sm.cnt_*` nothing the caller needs.
template <typename F>
__device__ inline void block_visit_topk(const float* __restrict__ row, int n, uint32_t tau,
                                        uint32_t k_eq, SelectSmem& sm, F f) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int seg = (n + SEL_NW - 1) / SEL_NW;
  seg = (seg + 63) / 64 * 64;
  const int beg = min(n, w * seg), end = min(n, beg + seg);
  uint32_t cgt = 0, ceq = 0;
  for (int x0 = beg; x0 < end; x0 += 64) {
    const int x = x0 + lane;
    const uint32_t key = x < end ? float_key(row[x]) : 0u;
    const bool ok = x < end;
    cgt += __popcll(__ballot(ok && key > tau));
    ceq += __popcll(__ballot(ok && key == tau));
  }
  __syncthreads();
  if (lane == 0) { sm.cnt_gt[w] = cgt; sm.cnt_eq[w] = ceq; }
  __syncthreads();
  uint32_t eq_run = 0, out_run = 0;
  for (int j = 0; j < w; ++j) {
    out_run += sm.cnt_gt[j] + min(sm.cnt_eq[j], k_eq - min(k_eq, eq_run));
    eq_run += sm.cnt_eq[j];
  }
  for (int x0 = beg; x0 < end; x0 += 64) {
    const int x = x0 + lane;
    const bool ok = x < end;
    const uint32_t key = ok ? float_key(row[x]) : 0u;
    const bool gt = ok && key > tau, eq = ok && key == tau;
    const unsigned long long beq = __ballot(eq);
    const bool take = gt || (eq && eq_run + rank_in_ballot(beq) < k_eq);
    const unsigned long long btk = __ballot(take);
    if (take) f(x, out_run + rank_in_ballot(btk));
    eq_run += __popcll(beq);
    out_run += __popcll(btk);
  }
}

}  // namespace restkv
