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
// Any block of 64 .. SEL_NT threads whose size divides SEL_BINS.
__device__ inline void block_kth_key(const float* __restrict__ row, int n, int k, SelectSmem& sm,
                                     uint32_t& tau, uint32_t& n_gt, uint32_t& k_eq) {
  uint32_t prefix = 0, mask = 0, krem = (uint32_t)k, above = 0;
  const int shifts[3] = {21, 10, 0};
  const int nbits[3] = {11, 11, 10};
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    const int sh = shifts[pass];
    const uint32_t nb = 1u << nbits[pass];
    const int nt = (int)blockDim.x, bpt = SEL_BINS / nt;
    for (int b = threadIdx.x; b < SEL_BINS; b += nt) sm.hist[b] = 0;
    __syncthreads();
    for (int x = threadIdx.x; x < n; x += nt) {
      const uint32_t key = float_key(row[x]);
      if ((key & mask) == prefix) atomicAdd(&sm.hist[(key >> sh) & (nb - 1)], 1u);
    }
    __syncthreads();
    // bins in descending order: thread t owns the reversed bins bpt t .. bpt t + bpt - 1
    const int r0 = bpt * (int)threadIdx.x;
    uint32_t own = 0;
    for (int j = 0; j < bpt; ++j) own += r0 + j < (int)nb ? sm.hist[nb - 1 - (r0 + j)] : 0u;
    const uint32_t incl = block_incl_scan(own, sm.wsum);
    uint32_t before = incl - own;
    if (before < krem && krem <= incl) {        // exactly one thread
      for (int j = 0; j < bpt; ++j) {
        const uint32_t hj = r0 + j < (int)nb ? sm.hist[nb - 1 - (r0 + j)] : 0u;
        if (krem <= before + hj) { sm.bin = nb - 1 - (r0 + j); sm.below = before; break; }
        before += hj;
      }
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

__device__ __forceinline__ float key_float(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
}

constexpr int SEL_NS = 4096;     // samples of the bracketed search

// Block-wide counting on keys held in registers (NPT per thread; empty slots hold key 0, which
// no pivot >= 1 counts).  One barrier per call; `it` alternates the two reduction buffers.
struct CountSmem { uint32_t red[2][3][SEL_NW]; };

// counts of keys >= piv[0..NP) (NP <= 6): per-lane counts on the vector ALU, several counts per
// register through the wave reduction (three of 10 bits while a wavefront holds fewer than 1024
// keys, else two of 16 bits), one LDS word per register and wavefront.
// NWV: wavefronts that take part (0: all of the block; otherwise the first NWV, the others having left)
template <int NPT, int NP, int NWV = 0>
__device__ __forceinline__ void block_count_geN(const uint32_t (&k)[NPT], const uint32_t (&piv)[NP],
                                                CountSmem& cs, int& it, uint32_t (&cnt)[NP]) {
  static_assert(NP >= 1 && NP <= 6, "three packed registers");
  constexpr int BITS = NPT * 64 < 1024 ? 10 : 16, PER = 32 / BITS;
  constexpr int NR = (NP + PER - 1) / PER;
  constexpr uint32_t FM = (1u << BITS) - 1u;
  uint32_t c[NP];
#pragma unroll
  for (int q = 0; q < NP; ++q) c[q] = 0;
#pragma unroll
  for (int j = 0; j < NPT; ++j)
#pragma unroll
    for (int q = 0; q < NP; ++q) c[q] += k[j] >= piv[q] ? 1u : 0u;
  const int w = threadIdx.x >> 6, nw = NWV ? NWV : (int)(blockDim.x >> 6), p = it & 1;
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    uint32_t pk = 0;
#pragma unroll
    for (int u = 0; u < PER; ++u)
      if (PER * r + u < NP) pk |= c[PER * r + u] << (BITS * u);
    const uint32_t packed = wave_sum(pk);
    if ((threadIdx.x & 63) == 0) cs.red[p][r][w] = packed;
  }
  __syncthreads();
#pragma unroll
  for (int q = 0; q < NP; ++q) cnt[q] = 0;
  auto add_wave = [&](int j) {
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const uint32_t x = cs.red[p][r][j];
#pragma unroll
      for (int u = 0; u < PER; ++u)
        if (PER * r + u < NP) cnt[PER * r + u] += (x >> (BITS * u)) & FM;
    }
  };
  if constexpr (NWV != 0) {
#pragma unroll
    for (int j = 0; j < NWV; ++j) add_wave(j);
  } else {
    for (int j = 0; j < nw; ++j) add_wave(j);
  }
  ++it;
}

template <int NPT, int NWV = 0>
__device__ __forceinline__ void block_count_ge2(const uint32_t (&k)[NPT], uint32_t va, uint32_t vb,
                                                CountSmem& cs, int& it, uint32_t& ca, uint32_t& cb) {
  const uint32_t piv[2] = {va, vb};
  uint32_t cnt[2];
  block_count_geN<NPT, 2, NWV>(k, piv, cs, it, cnt);
  ca = cnt[0]; cb = cnt[1];
}

// One bisection step on `nb` (1 or 2) bits starting at `bit`: a becomes the largest of
// a | (x << (bit - nb + 1)), x in [0, 2^nb), whose count is >= kk, given the counts of x = 1..3.
__device__ __forceinline__ uint32_t bisect_pick(uint32_t a, int sh, uint32_t kk, uint32_t c1, uint32_t c2,
                                                uint32_t c3) {
  if (c3 >= kk) return a | (3u << sh);
  if (c2 >= kk) return a | (2u << sh);
  if (c1 >= kk) return a | (1u << sh);
  return a;
}

// A threshold t for the k largest keys of the block: count(key >= t) >= k, and either the count
// is exactly k (t then need not be a key: the search stops as soon as a pivot separates the k
// largest from the rest) or t is the k-th largest key itself (equal keys straddle the cut).  Bits
// above `top_bit` are known (`prefix`, e.g. the common leading bits of a bracket that holds every
// key); the others are resolved two per barrier (three pivots at a time).
template <int NPT, int NWV = 0>
__device__ inline uint32_t block_kth(const uint32_t (&k)[NPT], uint32_t kk, CountSmem& cs, int& it,
                                     int top_bit = 31, uint32_t prefix = 0u) {
  uint32_t a = prefix;
  int bit = top_bit;
  if ((bit & 1) == 0) {                 // odd number of bits: one single-bit step first
    const uint32_t piv[1] = {a | (1u << bit)};
    uint32_t c[1];
    block_count_geN<NPT, 1, NWV>(k, piv, cs, it, c);
    if (c[0] == kk) return piv[0];
    if (c[0] >= kk) a = piv[0];
    --bit;
  }
  for (; bit >= 1; bit -= 2) {
    const int sh = bit - 1;
    const uint32_t piv[3] = {a | (1u << sh), a | (2u << sh), a | (3u << sh)};
    uint32_t c[3];
    block_count_geN<NPT, 3, NWV>(k, piv, cs, it, c);
    // a pivot with exactly kk keys at or above it separates the kk largest from the rest: the
    // lower bits do not matter any more (block-uniform: every thread holds the same counts)
    if (c[0] == kk) return piv[0];
    if (c[1] == kk) return piv[1];
    if (c[2] == kk) return piv[2];
    a = bisect_pick(a, sh, kk, c[0], c[1], c[2]);
  }
  return a;
}

// Largest values ta, tb with count(key >= ta) >= ka and count(key >= tb) >= kb, i.e. the
// ka-th and kb-th largest keys of the block (0 if fewer keys than that), bit by bit (with many
// keys per thread the counting, not the barrier, is what a step costs).
// With low_bit > 0 only the bits from it up are resolved (ta, tb are then lower bounds with the
// unresolved bits zero).  Bits above `top_bit` are known (`prefix`: the leading bits that every
// key shares).
template <int NPT>
__device__ inline void block_kth2(const uint32_t (&k)[NPT], uint32_t ka, uint32_t kb, CountSmem& cs,
                                  int& it, uint32_t& ta, uint32_t& tb, int low_bit = 0, int top_bit = 31,
                                  uint32_t prefix = 0u) {
  uint32_t a = prefix, b = prefix;
  for (int bit = top_bit; bit >= low_bit; --bit) {
    const uint32_t pa = a | (1u << bit), pb = b | (1u << bit);
    uint32_t ca, cb;
    block_count_ge2<NPT>(k, pa, pb, cs, it, ca, cb);
    if (ca >= ka) a = pa;
    if (cb >= kb) b = pb;
  }
  ta = a; tb = b;
}

// Highest bit in which two keys differ (-1 if equal) and their common bits above it: every key
// between them shares that prefix.
__device__ __forceinline__ void common_prefix(uint32_t klo, uint32_t khi, int& top_bit, uint32_t& prefix) {
  const uint32_t x = klo ^ khi;
  top_bit = x ? 31 - __builtin_clz(x) : -1;
  prefix = top_bit >= 31 ? 0u : (khi & ~((2u << max(top_bit, 0)) - 1u)) | (top_bit < 0 ? khi : 0u);
}

// Smallest and largest key of the block, empty slots (key 0) aside; kmin = 0xFFFFFFFF and kmax = 0
// if there is no key.  One barrier, same buffers and turn-taking as the counting step.
template <int NPT>
__device__ inline void block_key_range(const uint32_t (&k)[NPT], CountSmem& cs, int& it, uint32_t& kmin,
                                       uint32_t& kmax) {
  uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    hi = max(hi, k[j]);
    lo = k[j] ? min(lo, k[j]) : lo;
  }
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, o, 64));
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, o, 64));
  }
  const int w = threadIdx.x >> 6, nw = (int)(blockDim.x >> 6), p = it & 1;
  if ((threadIdx.x & 63) == 0) { cs.red[p][0][w] = hi; cs.red[p][1][w] = lo; }
  __syncthreads();
  kmin = 0xFFFFFFFFu; kmax = 0u;
  for (int j = 0; j < nw; ++j) { kmax = max(kmax, cs.red[p][0][j]); kmin = min(kmin, cs.red[p][1][j]); }
  ++it;
}

// Sample ranks that bracket the k-th largest of a population of n from a sample of ns
// (1-based, descending order): five standard deviations of the hypergeometric rank plus 2.
__device__ __forceinline__ void bracket_ranks(int n, int ns, int k, int& r_hi, int& r_lo) {
  const float f = (float)ns / (float)n;
  const float kp = (float)k * f;
  const int margin = (int)(5.0f * sqrtf(fmaxf(kp * (1.0f - f), 0.f))) + 2;
  r_hi = (int)kp - margin;          // <= 0: no upper bound
  r_lo = (int)kp + 2 + margin;      // > ns: no lower bound
}

// Evenly spread sample of a row in runs of RUN consecutive floats, NPT keys per thread
// (the whole row if it has at most NPT*blockDim.x entries).  Returns the sample size.
template <int NPT, int RUN>
__device__ inline int block_sample_regs(const float* __restrict__ row, int n, uint32_t (&k)[NPT]) {
  const int cap = NPT * blockDim.x;
  if (n <= cap) {
    float f[NPT];            // unconditional loads (clamped, then masked): all in flight together
#pragma unroll
    for (int j = 0; j < NPT; ++j) f[j] = row[min((int)(threadIdx.x + j * blockDim.x), n - 1)];
#pragma unroll
    for (int j = 0; j < NPT; ++j) k[j] = (int)(threadIdx.x + j * blockDim.x) < n ? float_key(f[j]) : 0u;
    return n;
  }
  const int nch = cap / RUN;
  const double step = (double)(n - RUN) / (double)(nch - 1);     // no integer division per sample
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int x = threadIdx.x + j * blockDim.x;
    const int c = x / RUN, e = x % RUN;
    const int start = min((int)((double)c * step), n - RUN);
    k[j] = float_key(row[start + e]);
  }
  return cap;
}

// Bracket {klo, khi} (keys) of the k-th largest of row[0..n): the k-th largest key lies in
// (klo, khi] unless the sample misled us.  khi = 0xFFFFFFFF / klo = 0 mean "unbounded".
template <int NPT, int RUN>
__device__ inline void block_bracket(const float* __restrict__ row, int n, int k, CountSmem& cs, int& it,
                                     uint32_t& klo, uint32_t& khi) {
  uint32_t keys[NPT];
  const int ns = block_sample_regs<NPT, RUN>(row, n, keys);
  int r_hi, r_lo;
  bracket_ranks(n, ns, k, r_hi, r_lo);
  // a bracket only has to hold the threshold: 16 resolved bits (sign, exponent, 7 mantissa
  // bits) are plenty; the upper end is rounded up, the lower end down.  The leading bits that
  // the smallest and the largest sample share need no search.
  uint32_t kmin, kmax, prefix;
  int top_bit;
  block_key_range<NPT>(keys, cs, it, kmin, kmax);
  common_prefix(kmin, kmax, top_bit, prefix);
  uint32_t thi, tlo;
  block_kth2<NPT>(keys, (uint32_t)max(r_hi, 1), (uint32_t)min(r_lo, ns), cs, it, thi, tlo, 16, top_bit,
                  prefix & 0xFFFF0000u);
  khi = r_hi >= 1 ? (thi | 0xFFFFu) : 0xFFFFFFFFu;
  klo = r_lo <= ns ? tlo : 0u;
}

// Calls f(word index, word) for every 32-bit word of a row of ndw mask words (ndw a multiple of
// 4, the row 16-byte aligned): 16-byte loads, four of them in flight per thread (NT threads).
template <int NT, typename F>
__device__ __forceinline__ void for_each_mask_word(const uint32_t* __restrict__ mrow, int ndw, F f) {
  const int nq = ndw >> 2;
  for (int q0 = 0; q0 < nq; q0 += 4 * NT) {
    uint4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * NT + (int)threadIdx.x;
      v[u] = ((const uint4*)mrow)[min(q, nq - 1)];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int q = q0 + u * NT + (int)threadIdx.x;
      if (q < nq) { f(4 * q, v[u].x); f(4 * q + 1, v[u].y); f(4 * q + 2, v[u].z); f(4 * q + 3, v[u].w); }
    }
  }
}

// Visits row[0..n) in position order, wave after wave; f(position, selected_rank)
// is called for every selected element, ranks ascending with position.
// Returns through `sm.cnt_*` nothing the caller needs.
template <typename F>
__device__ inline void block_visit_topk(const float* __restrict__ row, int n, uint32_t tau,
                                        uint32_t k_eq, SelectSmem& sm, F f) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (int)(blockDim.x >> 6);
  int seg = (n + nw - 1) / nw;
  seg = (seg + 63) / 64 * 64;
  const int beg = min(n, w * seg), end = min(n, beg + seg);
  uint32_t cgt = 0, ceq = 0;
  for (int x0 = beg; x0 < end; x0 += 512) {
    uint32_t kk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int x = x0 + 64 * u + lane;
      kk[u] = x < end ? float_key(row[x]) : 0u;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool ok = x0 + 64 * u + lane < end;
      cgt += __popcll(__ballot(ok && kk[u] > tau));
      ceq += __popcll(__ballot(ok && kk[u] == tau));
    }
  }
  __syncthreads();
  if (lane == 0) { sm.cnt_gt[w] = cgt; sm.cnt_eq[w] = ceq; }
  __syncthreads();
  uint32_t eq_run = 0, out_run = 0;
  for (int j = 0; j < w; ++j) {
    out_run += sm.cnt_gt[j] + min(sm.cnt_eq[j], k_eq - min(k_eq, eq_run));
    eq_run += sm.cnt_eq[j];
  }
  for (int x0 = beg; x0 < end; x0 += 512) {
    uint32_t kk[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int x = x0 + 64 * u + lane;
      kk[u] = x < end ? float_key(row[x]) : 0u;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int x = x0 + 64 * u + lane;
      const bool ok = x < end;
      const bool gt = ok && kk[u] > tau, eq = ok && kk[u] == tau;
      const unsigned long long beq = __ballot(eq);
      const bool take = gt || (eq && eq_run + rank_in_ballot(beq) < k_eq);
      const unsigned long long btk = __ballot(take);
      if (take) f(x, out_run + rank_in_ballot(btk));
      eq_run += __popcll(beq);
      out_run += __popcll(btk);
    }
  }
}

}  // namespace restkv
