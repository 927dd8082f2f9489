// Spatial-temporal smoothing (Sec. 3.3): EMA over the window queries, drift statistic of
// the per-query top-B positions, adaptive window size / shift, shifted box mean.
//
// The raw score [Hkv, W, P] is read from HBM once: a sorted sample of every (head, query) row
// brackets the row's top-B threshold; the fused pass computes the EMA and, per row, counts and
// sums the positions above the bracket and collects the few entries inside it; a finishing
// kernel decides the threshold exactly among those candidates.
#include <type_traits>

#include "rowselect.hpp"

namespace restkv {

namespace {

constexpr int CAND_CAP = 4096;      // candidates kept per (head, query) row
constexpr int SMP_NS = 8192;        // samples per row that the fused score pass may leave for the bracket
constexpr int ROW_NS = 4096;        // samples per row that the bracket kernel fetches itself

// Bracket of the top-min(B,P) threshold of one (head, query) row from a sample of the row.
// thr[row] = {lo, hi}: the threshold lies in (lo, hi] unless the sample misled us (then the
// finishing kernel falls back to the exact radix search).  Also clears the row's counters.
// grid (W, Hkv), 256 threads, ROW_NS / 256 samples per thread in registers.
__global__ __launch_bounds__(256) void k_sample_bracket(Prob pb, const float* __restrict__ score,
                                                        float2* __restrict__ thr,
                                                        uint32_t* __restrict__ cnt_hi,
                                                        unsigned long long* __restrict__ sum_hi) {
  __shared__ CountSmem cs;
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const float* row = score + (int64_t)r * pb.ld;
  const int k = min(head_budget(pb, g), pb.P);
  if (threadIdx.x == 0) { cnt_hi[r] = 0; sum_hi[r] = 0ull; }
  if (k >= pb.P) {                       // every prefix position is taken: nothing to search
    if (threadIdx.x == 0) thr[r] = make_float2(INFINITY, INFINITY);
    return;
  }
  int it = 0;
  uint32_t klo, khi;
  block_bracket<ROW_NS / 256, 16>(row, pb.P, k, cs, it, klo, khi);
  if (threadIdx.x == 0)
    thr[r] = make_float2(klo ? key_float(klo) : -INFINITY, khi != 0xFFFFFFFFu ? key_float(khi) : INFINITY);
}

// The same bracket from scores of sampled keys that the score pass left contiguously:
// smp [Hkv*W, ns], ns a multiple of 256.  grid (W, Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_bracket_samples(Prob pb, const float* __restrict__ smp, int ns,
                                                         float2* __restrict__ thr,
                                                         uint32_t* __restrict__ cnt_hi,
                                                         unsigned long long* __restrict__ sum_hi) {
  constexpr int NPT = SMP_NS / 256;
  __shared__ CountSmem cs;
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const int k = min(head_budget(pb, g), pb.P);
  if (threadIdx.x == 0) { cnt_hi[r] = 0; sum_hi[r] = 0ull; }
  if (k >= pb.P) {
    if (threadIdx.x == 0) thr[r] = make_float2(INFINITY, INFINITY);
    return;
  }
  uint32_t keys[NPT];
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const int x = threadIdx.x + j * 256;
    keys[j] = x < ns ? float_key(smp[(int64_t)r * ns + x]) : 0u;
  }
  int r_hi, r_lo, it = 0;
  bracket_ranks(pb.P, ns, k, r_hi, r_lo);
  uint32_t thi, tlo;
  block_kth2<NPT>(keys, (uint32_t)max(r_hi, 1), (uint32_t)min(r_lo, ns), cs, it, thi, tlo, 16);
  const uint32_t khi = r_hi >= 1 ? (thi | 0xFFFFu) : 0xFFFFFFFFu;
  const uint32_t klo = r_lo <= ns ? tlo : 0u;
  if (threadIdx.x == 0)
    thr[r] = make_float2(klo ? key_float(klo) : -INFINITY, khi != 0xFFFFFFFFu ? key_float(khi) : INFINITY);
}

// Fused single read of the raw score: EMA over the window queries and, per (head, query) row,
// the count / position sum of the entries above the row's bracket and a bit mask of the entries
// inside it (the candidates among which the finishing kernel finds the exact threshold).
//
// A WAVEFRONT owns EW_POS consecutive prefix positions of one head for all W rows; a lane owns
// four 16-byte quads of them (quad j of lane l: positions wbase + 256 j + 4 l ..+3, so that a
// wave-load is one contiguous KiB).  There is no workgroup barrier, no LDS and no cross-wavefront
// state:
//   * EMA as the weighted sum the recursion of Sec. 3.3 unrolls to: one FMA per element with a
//     wave-uniform weight (first query (1-a)^(W-1), query i > 0: a (1-a)^(W-1-i));
//   * per element and bracket end, ONE compare and ONE add-with-carry shift the outcome into a
//     per-lane bit string (16 elements per row: bit 15 - k is element k); the count and the
//     position sum of the entries above the bracket come from population counts of masked bit
//     strings, one packed wave reduction per row, and lane (row % 64) keeps the row's totals
//     until the block of 64 rows ends (two atomics per row, wavefront and block);
//   * the entries inside the bracket leave as what they already are: the lane's 16-bit string
//     "above the lower end and not above the upper end", one 128-byte store per wavefront and
//     row into cmask [row][wavefront][lane].  The finishing kernel expands a row's masks into
//     positions and fetches those few values itself.
// EPF rows are in flight per lane, so 16 KiB per wavefront are on their way while a row is
// processed.  grid (ceil(P / (4 EW_POS)), Hkv), 256 threads.
constexpr int EW_POS = 1024;        // prefix positions per wavefront
constexpr int EW_NE = EW_POS / 64;  // elements per lane and row (16 = four quads)
constexpr int EPF = 4;              // rows in flight

// weight of window query i in the temporal smoothing (wave-uniform): the EMA recursion of
// Sec. 3.3 unrolled, or one of the alternatives of the ablation study (mean; the recursion run
// from the newest query to the oldest)
__device__ __forceinline__ float temporal_weight(const Prob& pb, int i) {
  if (pb.tmode == 1) return 1.0f / (float)pb.W;
  const bool inv = pb.tmode == 2;
  const int n = inv ? i : pb.W - 1 - i;            // queries the recursion visits after this one
  const bool first = inv ? i == pb.W - 1 : i == 0;  // the query the recursion starts from
  const float b = 1.0f - pb.alpha;
  const float decay = n == 0 ? 1.0f : exp2f((float)n * log2f(b));    // b = 0: 2^-inf = 0
  return (first ? 1.0f : pb.alpha) * decay;
}

// position of element k (bit 15 - k of a lane's string) of lane l of the wavefront that starts at wbase
__device__ __forceinline__ int scan_position(int wbase, int l, int k) { return wbase + 256 * (k >> 2) + 4 * l + (k & 3); }
__host__ __device__ inline int scan_waves(int P) { return (P + EW_POS - 1) / EW_POS; }

template <bool VEC>
__global__ __launch_bounds__(256) void k_ema_scan(Prob pb, const float* __restrict__ score,
                                                  float* __restrict__ ema, const float2* __restrict__ thr,
                                                  uint32_t* __restrict__ cnt_hi,
                                                  unsigned long long* __restrict__ sum_hi,
                                                  uint16_t* __restrict__ cmask, int rs) {
  // rs = 1, 2 or 4 wavefronts share a run of positions and split the rows of every block of 64
  // among them (short prefixes: more wavefronts, more bytes in flight); their partial weighted
  // sums meet in LDS at the end.  rs = 1: a wavefront works alone, no barrier anywhere.
  __shared__ float esum[4][EW_NE][64];
  const int g = blockIdx.y, l = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);     // (a scalar for the compiler)
  const int part = wv % rs, rpp = 64 / rs;       // this wavefront's share of a block of 64 rows
  const int wg = blockIdx.x * (4 / rs) + wv / rs;   // run of positions along the prefix
  const int wbase = wg * EW_POS;
  const bool active = wbase < pb.P;
  if (rs == 1 && !active) return;
  const int nwt = scan_waves(pb.P);
  const float* s = score + (int64_t)g * pb.W * pb.ld;
  const bool scan = pb.adaptive != 0;
  const bool tail = wbase + EW_POS > pb.P;       // some positions of this wavefront do not exist
  const int last_quad = (pb.P - 1) & ~3;

  auto load_row = [&](int i, float (&x)[EW_NE]) {
    const float* rp = s + (int64_t)i * pb.ld;
#pragma unroll
    for (int j = 0; j < EW_NE / 4; ++j) {
      const int n = wbase + 256 * j + 4 * l;
      if constexpr (VEC) {
        // past the end: the last aligned quad of the row (inside its ld floats), masked below
        const float4 v4 = *(const float4*)(rp + min(n, last_quad));
        x[4 * j] = v4.x; x[4 * j + 1] = v4.y; x[4 * j + 2] = v4.z; x[4 * j + 3] = v4.w;
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * j + e] = rp[min(n + e, pb.P - 1)];
      }
    }
  };

  float e[EW_NE];
#pragma unroll
  for (int k = 0; k < EW_NE; ++k) e[k] = 0.f;
  uint32_t acc_cnt = 0, acc_sum = 0;             // lane (row % 64): totals of that row above its bracket

  // `live` is false for the rows that pad a block to a multiple of EPF: weight 0, no bracket
  auto process = [&](int i, bool live, float (&x)[EW_NE]) {
    if (tail) {
#pragma unroll
      for (int k = 0; k < EW_NE; ++k)
        if (scan_position(wbase, l, k) >= pb.P) x[k] = -INFINITY;   // counts for nothing, never stored
    }
    const float w = live ? temporal_weight(pb, i) : 0.f;
#pragma unroll
    for (int k = 0; k < EW_NE; ++k) e[k] = fmaf(w, x[k], e[k]);
    if (!scan || !live) return;
    const float2 th = thr[g * pb.W + i];         // the threshold lies in (th.x, th.y]
    float tlo = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, th.x)));
    float thi = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, th.y)));
    settle_scalars(tlo, thi);
    uint32_t hb = 0, lb = 0;
#pragma unroll
    for (int k = 0; k < EW_NE; k += 2) shift_in_gt_2x2(hb, lb, x[k], x[k + 1], thi, tlo);
    // entries above the bracket: element k = 4 j + q of this lane sits at bit 15 - k and at
    // position wbase + 256 j + 4 l + q, so with c = popcount
    //   sum of j = 3 c - [bits 4..7, 12..15] - 2 [bits 8..15],  sum of q = 3 c - [odd bits] - 2 [bits 2,3 mod 4]
    const uint32_t c = (uint32_t)__popc(hb);
    const uint32_t sj = 3u * c - (uint32_t)__popc(hb & 0xF0F0u) - 2u * (uint32_t)__popc(hb & 0xFF00u);
    const uint32_t sq = 3u * c - (uint32_t)__popc(hb & 0xAAAAu) - 2u * (uint32_t)__popc(hb & 0xCCCCu);
    const uint32_t rel = 4u * (uint32_t)l * c + 256u * sj + sq;      // < 2^14 per lane, < 2^20 per wavefront
    const uint32_t tot = wave_sum((rel << 11) | c);                   // c <= 1024 per wavefront
    if (l == (i & 63)) { acc_cnt = tot & 0x7FFu; acc_sum = tot >> 11; }
    // entries inside the bracket
    cmask[((int64_t)(g * pb.W + i) * nwt + wg) * 64 + l] = (uint16_t)(lb & ~hb);
  };

  // end of a block of 64 rows (or of the rows): lane = row adds the wavefront's totals to the row's
  auto end_block = [&](int blk) {
    if (!scan) return;
    const int row = blk * 64 + l;
    if (row < pb.W && acc_cnt) {
      atomicAdd(&cnt_hi[g * pb.W + row], acc_cnt);
      atomicAdd(&sum_hi[g * pb.W + row],
                (unsigned long long)acc_cnt * (unsigned long long)wbase + (unsigned long long)acc_sum);
    }
    acc_cnt = 0; acc_sum = 0;
  };

  for (int blk = 0; blk * 64 < pb.W; ++blk) {
    const int r0 = blk * 64 + part * rpp, r1 = min(pb.W, r0 + rpp);
    if (!active || r0 >= r1) continue;           // wave-uniform: nothing of this block is this wavefront's
    float xs[EPF][EW_NE];
#pragma unroll
    for (int u = 0; u < EPF; ++u) load_row(min(r0 + u, r1 - 1), xs[u]);   // (past the end: the last row again)
    for (int i0 = r0; i0 < r1; i0 += EPF) {
#pragma unroll
      for (int u = 0; u < EPF; ++u) {
        // every group issues its EPF row loads whatever the row count (past the end: the last row
        // again, processed with weight 0): the number of loads in flight is then known at
        // compile time and a row only waits for its own
        const int i = i0 + u;
        process(min(i, r1 - 1), i < r1, xs[u]);
        load_row(min(i + EPF, r1 - 1), xs[u]);
      }
    }
    end_block(blk);
  }
  if (rs > 1) {                                  // workgroup-uniform
#pragma unroll
    for (int k = 0; k < EW_NE; ++k) esum[wv][k][l] = e[k];
    __syncthreads();
    if (part != 0 || !active) return;
    for (int o = 1; o < rs; ++o)
#pragma unroll
      for (int k = 0; k < EW_NE; ++k) e[k] += esum[wv + o][k][l];
  }
#pragma unroll
  for (int j = 0; j < EW_NE / 4; ++j) {
    const int n = wbase + 256 * j + 4 * l;
    float* ep = ema + (int64_t)g * pb.ld + n;
    if (VEC && n + 3 < pb.P) {
      *(float4*)ep = make_float4(e[4 * j], e[4 * j + 1], e[4 * j + 2], e[4 * j + 3]);
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (n + q < pb.P) ep[q] = e[4 * j + q];
    }
  }
}

// Exact search (radix select + ordered visit) of a row whose bracket missed or overflowed: the
// sum of the positions of its top k, for thread 0.  Every thread of the block calls.
__device__ inline unsigned long long row_exact_sum(const float* __restrict__ row, int n, int k, SelectSmem& sm) {
  uint32_t tau, n_gt, k_eq;
  block_kth_key(row, n, k, sm, tau, n_gt, k_eq);
  unsigned long long acc = 0;
  block_visit_topk(row, n, tau, k_eq, sm, [&](int x, uint32_t) { acc += (unsigned long long)x; });
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.isum[threadIdx.x >> 6] = acc;
  __syncthreads();
  unsigned long long tot = 0;
  for (int j = 0; j < (int)(blockDim.x >> 6); ++j) tot += sm.isum[j];
  return tot;
}

// Exact threshold among the candidates of one row (keys ck, positions ci, NPT per thread, 256
// threads; empty slots have key 0): `need` of them belong to the top-B, ties cut by position.
// Returns this thread's share of the position sum of the taken candidates.
template <int NPT>
__device__ inline unsigned long long finish_candidates(const uint32_t (&ck)[NPT], const uint32_t (&ci)[NPT],
                                                       uint32_t need, float2 th, CountSmem& cs) {
  int it = 0, top_bit;
  uint32_t prefix, cge, cgt;
  common_prefix(float_key(th.x), float_key(th.y), top_bit, prefix);   // every candidate lies inside the bracket
  const uint32_t t = block_kth<NPT, 4>(ck, need, cs, it, top_bit, prefix);
  block_count_ge2<NPT, 4>(ck, t, t + 1u, cs, it, cge, cgt);
  const uint32_t k_eq = need - cgt;              // ties at t to take, lowest positions first
  uint32_t pos_cut = 0xFFFFFFFFu;                // take tied entries with position <= pos_cut
  if (cge - cgt > k_eq) {
    // k_eq-th smallest position among the ties = k_eq-th largest inverted position
    uint32_t inv[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) inv[j] = ck[j] == t ? 0xFFFFFFFFu - ci[j] : 0u;
    pos_cut = 0xFFFFFFFFu - block_kth<NPT, 4>(inv, k_eq, cs, it);
  }
  // One 64-bit comparison per entry: (key, inverted position) >= (t, inverted cut).  (The form
  // "key > t || (key == t && position <= cut)" is miscompiled by hipcc 7.2 at -O3: the addend of
  // the tie case is dropped.)
  const unsigned long long cut = ((unsigned long long)t << 32) | (unsigned long long)(0xFFFFFFFFu - pos_cut);
  unsigned long long acc = 0;
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    const unsigned long long kj = ((unsigned long long)ck[j] << 32) | (unsigned long long)(0xFFFFFFFFu - ci[j]);
    acc += kj >= cut ? (unsigned long long)ci[j] : 0ull;
  }
  return acc;
}

// Sum of the positions of the top-min(B,P) entries of one (head, query) row: the entries above
// the bracket were summed by the fused pass; the entries inside it arrive as bit masks (one
// 16-bit string per lane of the scan, see k_ema_scan), are expanded into positions here and
// their values fetched from the raw score.  The threshold is found among them by bisection on
// their keys; equal values are taken in position order (a second bisection on the position,
// only when a tie straddles the cut).  A row whose bracket missed, or that has more than
// CAND_CAP candidates, is searched exactly (radix select over the whole row) on the spot.
// grid (W, Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_row_finish(Prob pb, const float* __restrict__ score,
                                                    const uint32_t* __restrict__ cnt_hi,
                                                    const unsigned long long* __restrict__ sum_hi,
                                                    const uint16_t* __restrict__ cmask,
                                                    const float2* __restrict__ thr,
                                                    unsigned long long* __restrict__ rowsum) {
  constexpr int NPT = CAND_CAP / 256;
  __shared__ CountSmem cs;
  __shared__ unsigned long long isum[4];
  __shared__ uint32_t wsum[SEL_NW];
  __shared__ int cpos[CAND_CAP];                 // positions of the row's candidates
  __shared__ SelectSmem sm;                      // (exact search only)
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const int k = min(head_budget(pb, g), pb.P);
  if (k >= pb.P) {
    if (threadIdx.x == 0) rowsum[r] = (unsigned long long)pb.P * (unsigned long long)(pb.P - 1) / 2ull;
    return;
  }
  const uint32_t ch = cnt_hi[r];
  const unsigned long long shi = sum_hi[r];          // fetched with the counters, used at the very end
  const float2 th = thr[r];
  // the row's masks, two lanes of the scan per 32-bit word (a row's masks start 128-byte aligned)
  const int nwt = scan_waves(pb.P), ndw = nwt * 32;
  const uint32_t* mrow = (const uint32_t*)(cmask + (int64_t)r * nwt * 64);
  uint32_t c = 0;
  for_each_mask_word<256>(mrow, ndw, [&](int, uint32_t m) { c += (uint32_t)__popc(m); });
  const uint32_t incl = block_incl_scan(c, wsum);
  __syncthreads();
  if (threadIdx.x == 255) wsum[0] = incl;            // (every thread has read the wave sums)
  __syncthreads();
  const uint32_t nc = wsum[0];
  const bool ok = ch < (uint32_t)k && (uint32_t)k <= ch + nc && nc <= (uint32_t)CAND_CAP;
  if (!ok) {                                         // block-uniform
    const unsigned long long tot = row_exact_sum(score + (int64_t)r * pb.ld, pb.P, k, sm);
    if (threadIdx.x == 0) rowsum[r] = tot;
    return;
  }
  uint32_t slot = incl - c;
  for_each_mask_word<256>(mrow, ndw, [&](int x, uint32_t m) {
    while (m) {
      const int b = __builtin_ctz(m);
      m &= m - 1;
      const int li = 2 * x + (b >> 4);               // lane of the scan, counted along the row (two per word)
      cpos[slot++] = scan_position((li >> 6) * EW_POS, li & 63, 15 - (b & 15));
    }
  });
  __syncthreads();
  const uint32_t need = (uint32_t)k - ch;
  const float* row = score + (int64_t)r * pb.ld;
  // All loads unconditional (an empty slot re-reads the first candidate and is then masked):
  // independent loads in flight together instead of one round trip per slot.  Only as many
  // slots per thread as the row's candidates need (block-uniform), so a short list is counted quickly.
  auto run = [&](auto nsc) {
    constexpr int NS = decltype(nsc)::value;
    uint32_t ck[NS], ci[NS];
    float fv[NS];
    int iv[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const uint32_t x = threadIdx.x + j * 256;
      iv[j] = cpos[x < nc ? x : 0u];
      fv[j] = row[iv[j]];
    }
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const bool in = (uint32_t)(threadIdx.x + j * 256) < nc;
      ck[j] = in ? float_key(fv[j]) : 0u;
      ci[j] = in ? (uint32_t)iv[j] : 0u;
    }
    return finish_candidates<NS>(ck, ci, need, th, cs);
  };
  unsigned long long acc = nc <= 1024u  ? run(std::integral_constant<int, 4>{})
                           : nc <= 2048u ? run(std::integral_constant<int, 8>{})
                           : nc <= 3072u ? run(std::integral_constant<int, 12>{})
                                         : run(std::integral_constant<int, NPT>{});
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if ((threadIdx.x & 63) == 0) isum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) rowsum[r] = isum[0] + isum[1] + isum[2] + isum[3] + shi;
}

// The finishing step when the candidates of a row sit in per-chunk slices
// (sval / sidx [row, nchunks, caps], fill counts scnt [row, nchunks]; nchunks <= 256).
// grid (W, Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_row_finish_slices(Prob pb, const float* __restrict__ score,
                                                           const uint32_t* __restrict__ cnt_hi,
                                                           const unsigned long long* __restrict__ sum_hi,
                                                           const uint32_t* __restrict__ scnt,
                                                           const float* __restrict__ sval,
                                                           const int* __restrict__ sidx, int nchunks, int caps,
                                                           const float2* __restrict__ thr,
                                                           unsigned long long* __restrict__ rowsum) {
  constexpr int NPT = CAND_CAP / 256;
  __shared__ CountSmem cs;
  __shared__ unsigned long long isum[4];
  __shared__ uint32_t pre[257];              // exclusive prefix of the slice fill counts
  __shared__ uint32_t over;
  __shared__ SelectSmem sm;                  // (exact search only)
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const int k = min(head_budget(pb, g), pb.P);
  if (k >= pb.P) {
    if (threadIdx.x == 0) rowsum[r] = (unsigned long long)pb.P * (unsigned long long)(pb.P - 1) / 2ull;
    return;
  }
  if (threadIdx.x == 0) {
    uint32_t run = 0, ov = 0;
    for (int c = 0; c < nchunks; ++c) {
      const uint32_t n = scnt[(int64_t)r * nchunks + c];
      pre[c] = run;
      run += min(n, (uint32_t)caps);
      ov |= n > (uint32_t)caps ? 1u : 0u;
    }
    pre[nchunks] = run;
    over = ov;
  }
  __syncthreads();
  const uint32_t ch = cnt_hi[r], nc = pre[nchunks];
  const bool ok = !over && ch < (uint32_t)k && (uint32_t)k <= ch + nc && nc <= (uint32_t)CAND_CAP;
  if (!ok) {
    const unsigned long long tot = row_exact_sum(score + (int64_t)r * pb.ld, pb.P, k, sm);
    if (threadIdx.x == 0) rowsum[r] = tot;
    return;
  }
  const uint32_t need = (uint32_t)k - ch;
  uint32_t ck[NPT], ci[NPT];
  {
    float fv[NPT];
    int iv[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {          // unconditional loads: see k_row_finish
      const uint32_t x0 = threadIdx.x + j * 256, x = x0 < nc ? x0 : 0u;
      int lo = 0, hi = nchunks - 1;           // last chunk whose prefix is <= x
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (pre[mid] <= x) lo = mid; else hi = mid - 1;
      }
      const int64_t o = ((int64_t)r * nchunks + lo) * caps + (x - pre[lo]);
      fv[j] = sval[o];
      iv[j] = sidx[o];
    }
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const bool in = (uint32_t)(threadIdx.x + j * 256) < nc;
      ck[j] = in ? float_key(fv[j]) : 0u;
      ci[j] = in ? (uint32_t)iv[j] : 0u;
    }
  }
  unsigned long long acc = finish_candidates<NPT>(ck, ci, need, thr[r], cs);
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if ((threadIdx.x & 63) == 0) isum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) rowsum[r] = isum[0] + isum[1] + isum[2] + isum[3] + sum_hi[r];
}

// Window size and shift from the drift statistic (device function so that every block of
// the box kernel derives the same integers without a host round trip).
// (front and rear index sums come in already added up)
__device__ inline void aws_window(const Prob& pb, unsigned long long sf, unsigned long long sr, int g,
                                  int& w_s, int& gamma, double& d_front, double& d_rear) {
  w_s = pb.base_k; gamma = 0; d_front = 0.0; d_rear = 0.0;
  if (!pb.adaptive) return;
  const int nf = pb.W / 2;
  const double bt = (double)min(head_budget(pb, g), pb.P);
  d_front = (double)sf / (bt * (double)nf);
  d_rear = (double)sr / (bt * (double)(pb.W - nf));
  const double x = d_front - d_rear;
  const double beta = (double)pb.beta;
  w_s = pb.base_k + 2 * (int)floor(fabs(x) / beta);
  const int f = (int)floor(x / beta);
  gamma = x > 0.0 ? f : f + 1;
}

// final[g,n] = (1/W_s) sum_{j=gamma-half}^{gamma+half} ema[g,n+j], zero outside [0,P).
// grid (ceil(P / (256 BOX_PT)), Hkv), 256 threads; a thread owns BOX_PT positions 256 apart (the
// loads of a window offset are independent and coalesced); every workgroup derives the head's
// window from the index sums itself.
constexpr int BOX_PT = 4;
__global__ __launch_bounds__(256) void k_box(Prob pb, const float* __restrict__ ema,
                                             const unsigned long long* __restrict__ rowsum,
                                             float* __restrict__ fin, int32_t* __restrict__ aws_info,
                                             double* __restrict__ aws_d) {
  const int g = blockIdx.y;
  __shared__ int sh_ws, sh_gamma;
  __shared__ unsigned long long sh_sum[2][4];
  __shared__ float tile[2 * 256 * BOX_PT];           // span + reach of the window (when it fits)
  // the W index sums of the head: all loads in flight at once, wavefront sums, then thread 0
  {
    unsigned long long sf = 0, sr = 0;
    if (pb.adaptive)
      for (int i = threadIdx.x; i < pb.W; i += 256) {
        const unsigned long long s = rowsum[g * pb.W + i];
        if (i < pb.W / 2) sf += s; else sr += s;
      }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { sf += __shfl_xor(sf, o, 64); sr += __shfl_xor(sr, o, 64); }
    if ((threadIdx.x & 63) == 0) { sh_sum[0][threadIdx.x >> 6] = sf; sh_sum[1][threadIdx.x >> 6] = sr; }
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int w_s0, gamma0;
    double df, dr;
    aws_window(pb, sh_sum[0][0] + sh_sum[0][1] + sh_sum[0][2] + sh_sum[0][3],
               sh_sum[1][0] + sh_sum[1][1] + sh_sum[1][2] + sh_sum[1][3], g, w_s0, gamma0, df, dr);
    sh_ws = w_s0; sh_gamma = gamma0;
    if (blockIdx.x == 0) {
      if (aws_info) { aws_info[2 * g] = w_s0; aws_info[2 * g + 1] = gamma0; }
      if (aws_d) { aws_d[2 * g] = df; aws_d[2 * g + 1] = dr; }
    }
  }
  __syncthreads();
  const int w_s = sh_ws, gamma = sh_gamma;
  const int n0 = blockIdx.x * (256 * BOX_PT) + threadIdx.x;
  const float* e = ema + (int64_t)g * pb.ld;
  const int half = w_s / 2;
  float s[BOX_PT];
#pragma unroll
  for (int j = 0; j < BOX_PT; ++j) s[j] = 0.f;
  // Window offsets in ascending order: a position's terms are added lowest index first; a term
  // outside the prefix is zero padding (it adds nothing; max pooling skips it, and a window with
  // no term inside the prefix gives 0).
  const int last = gamma + half;
  constexpr int SPAN = 256 * BOX_PT;
  if (w_s - 1 <= SPAN) {
    // the workgroup's span plus the window's reach goes through LDS: one coalesced read of the
    // smoothed scores instead of W_s reads per position
    const int t0 = blockIdx.x * SPAN + gamma - half;          // position of tile[0]
    const int tn = SPAN + 2 * half;
    const float pad = pb.pmax ? -INFINITY : 0.f;
    for (int x = threadIdx.x; x < tn; x += 256) {
      const int m = t0 + x;
      tile[x] = (m >= 0 && m < pb.P) ? e[m] : pad;
    }
    __syncthreads();
    if (pb.pmax) {
#pragma unroll
      for (int j = 0; j < BOX_PT; ++j) s[j] = -INFINITY;
      for (int u = 0; u < w_s; ++u)
#pragma unroll
        for (int j = 0; j < BOX_PT; ++j) s[j] = fmaxf(s[j], tile[threadIdx.x + 256 * j + u]);
#pragma unroll
      for (int j = 0; j < BOX_PT; ++j) s[j] = s[j] == -INFINITY ? 0.f : s[j];
    } else {
      for (int u = 0; u < w_s; ++u)
#pragma unroll
        for (int j = 0; j < BOX_PT; ++j) s[j] += tile[threadIdx.x + 256 * j + u];
    }
  } else {
    // a window wider than the span: straight from global memory, eight offsets at a time, every
    // load of the batch unconditional (clamped index) and issued before the first is used
    constexpr int OB = 8;
    auto filter = [&](auto maxc) {
      constexpr bool PMAX = decltype(maxc)::value;
      bool any[BOX_PT];
#pragma unroll
      for (int j = 0; j < BOX_PT; ++j) any[j] = false;
      for (int o0 = gamma - half; o0 <= last; o0 += OB) {
        float x[OB][BOX_PT];
#pragma unroll
        for (int u = 0; u < OB; ++u)
#pragma unroll
          for (int j = 0; j < BOX_PT; ++j) x[u][j] = e[min(max(n0 + 256 * j + o0 + u, 0), pb.P - 1)];
#pragma unroll
        for (int u = 0; u < OB; ++u)
#pragma unroll
          for (int j = 0; j < BOX_PT; ++j) {
            const int m = n0 + 256 * j + o0 + u;
            const bool in = o0 + u <= last && m >= 0 && m < pb.P;
            if constexpr (PMAX) {
              s[j] = in ? (any[j] ? fmaxf(s[j], x[u][j]) : x[u][j]) : s[j];
              any[j] = any[j] || in;
            } else {
              s[j] += in ? x[u][j] : 0.f;
            }
          }
      }
    };
    if (pb.pmax) filter(std::true_type{}); else filter(std::false_type{});
  }
#pragma unroll
  for (int j = 0; j < BOX_PT; ++j) {
    const int n = n0 + 256 * j;
    if (n < pb.P) fin[(int64_t)g * pb.ld + n] = pb.pmax ? s[j] : s[j] / (float)w_s;
  }
}

}  // namespace

int launch_smooth(const Prob& pb, const float* score, float* ema, float* fin, int32_t* aws_info,
                  double* aws_d, char* ws, const SmoothWs& lay, hipStream_t st) {
  unsigned long long* rowsum = (unsigned long long*)(ws + lay.rowsum);
  float2* thr = (float2*)(ws + lay.thr);
  uint32_t* cnt_hi = (uint32_t*)(ws + lay.cnt_hi);
  unsigned long long* sum_hi = (unsigned long long*)(ws + lay.sum_hi);
  uint16_t* cmask = (uint16_t*)(ws + lay.cmask);
  float* e = ema ? ema : (float*)(ws + lay.ema);
  const bool vec = (pb.ld & 3) == 0 && (((uintptr_t)score | (uintptr_t)e) & 15u) == 0;
  if (pb.adaptive)
    RK_LAUNCH(ST_ROWTOPK, st, k_sample_bracket, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, score, thr,
              cnt_hi, sum_hi);
  // short prefixes: 2 or 4 wavefronts per run of positions, until about a thousand wavefronts stream
  const int64_t runs = (int64_t)scan_waves(pb.P) * pb.Hkv;
  const int rs = runs >= 1024 ? 1 : (runs >= 512 ? 2 : 4);
  const int ppw = 4 / rs;
  const dim3 ge((scan_waves(pb.P) + ppw - 1) / ppw, pb.Hkv);
  if (vec)
    RK_LAUNCH(ST_EMA, st, k_ema_scan<true>, ge, dim3(256), 0, st, pb, score, e, thr, cnt_hi, sum_hi, cmask, rs);
  else
    RK_LAUNCH(ST_EMA, st, k_ema_scan<false>, ge, dim3(256), 0, st, pb, score, e, thr, cnt_hi, sum_hi, cmask, rs);
  if (pb.adaptive) {
    RK_LAUNCH(ST_ROWTOPK, st, k_row_finish, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, score, cnt_hi, sum_hi,
              cmask, thr, rowsum);
  }
  RK_LAUNCH(ST_BOX, st, k_box, dim3((pb.P + 256 * BOX_PT - 1) / (256 * BOX_PT), pb.Hkv), dim3(256), 0, st, pb, e, rowsum, fin,
            aws_info, aws_d);
  return hip_status();
}

int launch_bracket_samples(const Prob& pb, const float* smp, int ns, float2* thr, uint32_t* cnt_hi,
                           unsigned long long* sum_hi, hipStream_t st) {
  if (ns > SMP_NS) return RESTKV_EINVAL;
  RK_LAUNCH(ST_ROWTOPK, st, k_bracket_samples, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, smp, ns, thr,
            cnt_hi, sum_hi);
  return hip_status();
}

int launch_smooth_fused_tail(const Prob& pb, const float* score, const float* ema, float* fin,
                             int32_t* aws_info, double* aws_d, char* ws, const SmoothWs& lay,
                             const FusedPtrs& fp, int nchunks, hipStream_t st) {
  unsigned long long* rowsum = (unsigned long long*)(ws + lay.rowsum);
  RK_LAUNCH(ST_ROWTOPK, st, k_row_finish_slices, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, score, fp.cnt_hi,
            fp.sum_hi, fp.scnt, fp.sval, fp.sidx, nchunks, fp.caps, fp.thr, rowsum);
  RK_LAUNCH(ST_BOX, st, k_box, dim3((pb.P + 256 * BOX_PT - 1) / (256 * BOX_PT), pb.Hkv), dim3(256), 0, st, pb, ema, rowsum, fin,
            aws_info, aws_d);
  return hip_status();
}

}  // namespace restkv
