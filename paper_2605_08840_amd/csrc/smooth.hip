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
constexpr int SMP_NS = 8192;        // samples per row for the bracket
constexpr int RG = 4;               // rows in flight per thread of the fused pass (multiple of 4)
constexpr int NPB = 1024;           // prefix positions per workgroup of the fused pass

// Bracket of the top-min(B,P) threshold of one (head, query) row from a sample of the row.
// thr[row] = {lo, hi}: the threshold lies in (lo, hi] unless the sample misled us (then the
// finishing kernel falls back to the exact radix search).  Also clears the row's counters.
// grid (W, Hkv), 256 threads, SMP_NS / 256 samples per thread in registers.
__global__ __launch_bounds__(256) void k_sample_bracket(Prob pb, const float* __restrict__ score,
                                                        float2* __restrict__ thr,
                                                        uint32_t* __restrict__ cnt_hi,
                                                        unsigned long long* __restrict__ sum_hi,
                                                        uint32_t* __restrict__ ncand) {
  __shared__ CountSmem cs;
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const float* row = score + (int64_t)r * pb.ld;
  const int k = min(head_budget(pb, g), pb.P);
  if (threadIdx.x == 0) { cnt_hi[r] = 0; sum_hi[r] = 0ull; ncand[r] = 0; }
  if (k >= pb.P) {                       // every prefix position is taken: nothing to search
    if (threadIdx.x == 0) thr[r] = make_float2(INFINITY, INFINITY);
    return;
  }
  int it = 0;
  uint32_t klo, khi;
  block_bracket<SMP_NS / 256, 16>(row, pb.P, k, cs, it, klo, khi);
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

// Fused single read of the raw score: EMA over the window queries (the recursion of Sec. 3.3:
// first query as is, every later one enters with weight alpha) and, per (head, query) row,
// the count / position sum of the entries above the bracket and the list of entries inside it.
// A workgroup owns NPB prefix positions of one head for all W queries; a thread owns 4 of them.
// While streaming, a thread works alone (no cross-lane work, no scalar-ALU ballots): per group
// of RG rows it packs two LDS words (per row: 3-bit count and 3-bit element-offset sum of its
// entries above the bracket; 4-bit mask of its entries inside it) and keeps the values of the
// latter in a private LDS list.  After every ROWS_BLK rows the workgroup turns around:
//   * thread j = (row, quarter of the workgroup's threads) walks the 64 packed words of its
//     quarter: it adds up the statistics and leaves every thread's running candidate offset;
//     the four quarters of a row meet through lane shuffles and one thread per row issues the
//     row's global atomics (statistics, space in the row's candidate list);
//   * every thread then writes its own candidates to their final places.  A wavefront whose
//     private lists did not suffice (a dense cluster of candidates) re-reads its rows instead.
// grid (ceil(P/NPB), Hkv), 256 threads.
constexpr int ROWS_BLK = 32;        // rows per turn-around of the fused pass
constexpr int CAPT = 12;            // private candidate values per thread between turn-arounds

__global__ __launch_bounds__(256) void k_ema_scan(Prob pb, const float* __restrict__ score,
                                                  float* __restrict__ ema, const float2* __restrict__ thr,
                                                  uint32_t* __restrict__ cnt_hi,
                                                  unsigned long long* __restrict__ sum_hi,
                                                  uint32_t* __restrict__ ncand,
                                                  float* __restrict__ cand_val, int* __restrict__ cand_idx,
                                                  int vec) {
  constexpr int PG = 4;                          // rows per packed LDS word
  constexpr int NGRP = ROWS_BLK / PG;
  __shared__ __attribute__((aligned(16))) uint32_t pk0[NGRP][256];            // per thread and row group: RG x (count:3 | offset sum:3)
  __shared__ __attribute__((aligned(16))) uint32_t pk1[NGRP][256];            // RG x 4-bit masks of the entries inside the bracket
  __shared__ __attribute__((aligned(16))) uint8_t pk2[NGRP][PG][256];   // candidates of the row in earlier threads of the quarter
  __shared__ float pval[CAPT][256];              // private lists of candidates, in stream order: value ...
  __shared__ uint8_t pmeta[CAPT][256];           // ... and (row in block) * 4 + element
  __shared__ uint32_t rbase[ROWS_BLK][4];        // first list position of each (row, quarter)
  const int g = blockIdx.y, tid = threadIdx.x, lane = tid & 63;
  const int nb0 = blockIdx.x * NPB, n0 = nb0 + tid * 4;
  const float* s = score + (int64_t)g * pb.W * pb.ld;
  const float a = pb.alpha, b = 1.0f - pb.alpha;
  const bool scan = pb.adaptive != 0;
  int kp = 0;                        // candidates of this thread since the last turn-around

  // rows [rb0, rb0 + nrows) of the head have been streamed
  auto turn_around = [&](int rb0, int nrows) {
    __syncthreads();
    {
      const int rl = tid >> 2, qd = tid & 3;
      const int itr = rl / PG, rr = rl % PG, sh0 = 6 * rr, sh1 = 4 * rr;
      uint32_t cnt = 0, els = 0, wsum = 0, nc = 0;
      if (rl < nrows) {
        // Four threads' words per step (16-byte LDS reads; the four offset bytes leave as one
        // word).  Lanes with the same row group and quarter read the same address; the 16
        // (row group, quarter) pairs of a wavefront start their walk 16 bytes apart, so that no
        // two of them meet in an LDS bank.
        const int rot = ((lane >> 4) << 2) | (lane & 3);
#pragma unroll 4
        for (int tt = 0; tt < 16; ++tt) {
          const int t4 = (tt + rot) & 15, src = 64 * qd + 4 * t4;
          const uint4 a4 = *(const uint4*)&pk0[itr][src];
          const uint4 m4 = *(const uint4*)&pk1[itr][src];
          const uint32_t aw[4] = {a4.x, a4.y, a4.z, a4.w}, mw[4] = {m4.x, m4.y, m4.z, m4.w};
          uint32_t offs = 0;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t a0 = (aw[e] >> sh0) & 63u;
            const uint32_t c = a0 & 7u;
            cnt += c;
            els += a0 >> 3;
            wsum += c * (uint32_t)(4 * t4 + e);
            offs |= (nc & 255u) << (8 * e);       // at most 252: a quarter holds 256 positions
            nc += (uint32_t)__popc((mw[e] >> sh1) & 15u);
          }
          *(uint32_t*)&pk2[itr][rr][src] = offs;
        }
      }
      // positions above the bracket seen by this quarter: thread t of it owns nb0 + 4 (64 qd + t) + el
      const unsigned long long hs_own = (unsigned long long)cnt * (unsigned long long)(nb0 + 256 * qd) +
                                        4ull * wsum + (unsigned long long)els;
      unsigned long long hs = hs_own;
      uint32_t cnt_tot = cnt, nc_tot = nc, nc_below = 0;
      // the four quarters of a row sit in four adjacent lanes
#pragma unroll
      for (int d = 1; d < 4; ++d) {
        const int src = (lane & ~3) | ((lane + d) & 3);
        const uint32_t onc = (uint32_t)__shfl((int)nc, src, 64);
        cnt_tot += (uint32_t)__shfl((int)cnt, src, 64);
        hs += ((unsigned long long)(uint32_t)__shfl((int)(hs_own >> 32), src, 64) << 32) |
              (unsigned long long)(uint32_t)__shfl((int)(uint32_t)hs_own, src, 64);
        nc_tot += onc;
        if (((lane + d) & 3) < qd) nc_below += onc;
      }
      uint32_t base = 0;
      if (qd == 0 && rl < nrows) {
        const int row = g * pb.W + rb0 + rl;
        if (cnt_tot) { atomicAdd(&cnt_hi[row], cnt_tot); atomicAdd(&sum_hi[row], hs); }
        if (nc_tot) base = atomicAdd(&ncand[row], nc_tot);
      }
      base = (uint32_t)__shfl((int)base, lane & ~3, 64);
      if (rl < nrows) rbase[rl][qd] = base + nc_below;
    }
    __syncthreads();
    // every thread places its own candidates (the walk above visited this thread's quarter
    // starting at the walker's rotation, which only permutes the order inside the list)
    const int qd = tid >> 6;
    if (__ballot(kp > CAPT) == 0ull) {
      // Every private list of the wavefront is complete.  All LDS reads are issued up front
      // (clamped, not branched around), only the stores are predicated: three LDS round trips
      // and at most 2 CAPT store instructions per wavefront.
      int mt[CAPT];
      float pv[CAPT];
#pragma unroll
      for (int k = 0; k < CAPT; ++k) { mt[k] = pmeta[k][tid]; pv[k] = pval[k][tid]; }
      uint32_t pos[CAPT];
#pragma unroll
      for (int k = 0; k < CAPT; ++k) {
        const int rl = k < kp ? mt[k] >> 2 : 0;
        pos[k] = rbase[rl][qd] + pk2[rl / PG][rl % PG][tid];
      }
      int prev = -1;
      uint32_t run = 0;
#pragma unroll
      for (int k = 0; k < CAPT; ++k) {
        const int rl = mt[k] >> 2;
        run = rl == prev ? run + 1u : 0u;          // this thread's earlier candidates of the same row
        prev = rl;
        const uint32_t ps = pos[k] + run;
        if (k < kp && ps < (uint32_t)CAND_CAP) {
          const int64_t o = (int64_t)(g * pb.W + rb0 + rl) * CAND_CAP + ps;
          cand_val[o] = pv[k];
          cand_idx[o] = n0 + (mt[k] & 3);
        }
      }
    } else {
      // a dense cluster: the wavefront re-reads its rows (coalesced, two row groups = 8 rows per
      // round trip) and walks its masks
      for (int it0 = 0; it0 * PG < nrows; it0 += 2) {
        float x4[2 * PG][4];
#pragma unroll
        for (int q = 0; q < 2 * PG; ++q) {
          const int rl = min(it0 * PG + q, nrows - 1);
          const float* rp = s + (int64_t)(rb0 + rl) * pb.ld + n0;
#pragma unroll
          for (int el = 0; el < 4; ++el) x4[q][el] = n0 + el < pb.P ? rp[el] : 0.f;
        }
#pragma unroll
        for (int q = 0; q < 2 * PG; ++q) {
          const int itr = it0 + q / PG, rr = q % PG, rl = it0 * PG + q;
          if (rl >= nrows) break;
          const uint32_t mk = (pk1[itr][tid] >> (4 * rr)) & 15u;
          const int row = g * pb.W + rb0 + rl;
          uint32_t ps = rbase[rl][qd] + pk2[itr][rr][tid];
#pragma unroll
          for (int el = 0; el < 4; ++el) {
            if ((mk >> el) & 1u) {
              if (ps < (uint32_t)CAND_CAP) {
                cand_val[(int64_t)row * CAND_CAP + ps] = x4[q][el];
                cand_idx[(int64_t)row * CAND_CAP + ps] = n0 + el;
              }
              ++ps;
            }
          }
        }
      }
    }
    kp = 0;
    __syncthreads();
  };

  float e[4] = {0.f, 0.f, 0.f, 0.f};
  // the rows of the next group are fetched while the current group is scanned
  float xs[RG][4];
  float2 ths[RG];
  auto fetch = [&](int i0) {
#pragma unroll
    for (int r = 0; r < RG; ++r) {
      const int i = i0 + r;
      if (i < pb.W) {
        if (vec) {
          // one 16-byte load per thread, no branch at the tail: threads past the end re-read the
          // last aligned quad of the row (inside its ld floats) and discard it
          const float4 v4 = *(const float4*)(s + (int64_t)i * pb.ld + min(n0, (pb.P - 1) & ~3));
          xs[r][0] = n0 + 0 < pb.P ? v4.x : -INFINITY;
          xs[r][1] = n0 + 1 < pb.P ? v4.y : -INFINITY;
          xs[r][2] = n0 + 2 < pb.P ? v4.z : -INFINITY;
          xs[r][3] = n0 + 3 < pb.P ? v4.w : -INFINITY;
        } else {
          const float* rp = s + (int64_t)i * pb.ld + n0;
#pragma unroll
          for (int el = 0; el < 4; ++el) xs[r][el] = n0 + el < pb.P ? rp[el] : -INFINITY;
        }
        ths[r] = scan ? thr[g * pb.W + i] : make_float2(INFINITY, INFINITY);
      }
    }
  };
  fetch(0);
  int rb0 = 0;                       // first row since the last turn-around
  for (int i0 = 0; i0 < pb.W; i0 += RG) {
    float xc[RG][4];
    float2 thc[RG];
#pragma unroll
    for (int r = 0; r < RG; ++r) {
      thc[r] = ths[r];
#pragma unroll
      for (int el = 0; el < 4; ++el) xc[r][el] = xs[r][el];
    }
    if (i0 + RG < pb.W) fetch(i0 + RG);
    uint32_t w0[RG / PG], w1[RG / PG];
#pragma unroll
    for (int q = 0; q < RG / PG; ++q) { w0[q] = 0; w1[q] = 0; }
#pragma unroll
    for (int r = 0; r < RG; ++r) {
      const int i = i0 + r;
      if (i >= pb.W) break;
      const float* x = xc[r];
      const float2 th = thc[r];
      uint32_t cnt = 0, els = 0, cm = 0;
#pragma unroll
      for (int el = 0; el < 4; ++el) {
        e[el] = i == 0 ? x[el] : a * x[el] + b * e[el];
        const bool hi = x[el] > th.y;              // th.y = +inf: the bracket has no upper bound
        cnt += hi ? 1u : 0u;
        els += hi ? (uint32_t)el : 0u;
        if (x[el] > th.x && !hi) {                 // inside the bracket: rare
          if (kp < CAPT) { pval[kp][tid] = x[el]; pmeta[kp][tid] = (uint8_t)((i - rb0) * 4 + el); }
          ++kp;
          cm |= 1u << el;
        }
      }
      w0[r / PG] |= (cnt | (els << 3)) << (6 * (r % PG));
      w1[r / PG] |= cm << (4 * (r % PG));
    }
    if (scan) {
#pragma unroll
      for (int q = 0; q < RG / PG; ++q) {
        pk0[(i0 - rb0) / PG + q][tid] = w0[q];
        pk1[(i0 - rb0) / PG + q][tid] = w1[q];
      }
      if (i0 + RG - rb0 >= ROWS_BLK || i0 + RG >= pb.W) {      // block-uniform
        turn_around(rb0, min(i0 + RG, pb.W) - rb0);
        rb0 = i0 + RG;
      }
    }
  }
#pragma unroll
  for (int el = 0; el < 4; ++el)
    if (n0 + el < pb.P) ema[(int64_t)g * pb.ld + n0 + el] = e[el];
}

constexpr unsigned long long ROW_PENDING = ~0ull;   // rowsum marker: the bracket missed this row

// Exact threshold among the candidates of one row (keys ck, positions ci, NPT per thread, 256
// threads; empty slots have key 0): `need` of them belong to the top-B, ties cut by position.
// Returns this thread's share of the position sum of the taken candidates.
template <int NPT>
__device__ inline unsigned long long finish_candidates(const uint32_t (&ck)[NPT], const uint32_t (&ci)[NPT],
                                                       uint32_t need, float2 th, CountSmem& cs) {
  int it = 0, top_bit;
  uint32_t prefix, cge, cgt;
  common_prefix(float_key(th.x), float_key(th.y), top_bit, prefix);   // every candidate lies inside the bracket
  const uint32_t t = block_kth<NPT>(ck, need, cs, it, top_bit, prefix);
  block_count_ge2<NPT>(ck, t, t + 1u, cs, it, cge, cgt);
  const uint32_t k_eq = need - cgt;              // ties at t to take, lowest positions first
  uint32_t pos_cut = 0xFFFFFFFFu;                // take tied entries with position <= pos_cut
  if (cge - cgt > k_eq) {
    // k_eq-th smallest position among the ties = k_eq-th largest inverted position
    uint32_t inv[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) inv[j] = ck[j] == t ? 0xFFFFFFFFu - ci[j] : 0u;
    pos_cut = 0xFFFFFFFFu - block_kth<NPT>(inv, k_eq, cs, it);
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
// the bracket were summed by the fused pass; the threshold is found among the candidates by
// bisection on their keys, equal values are taken in position order (a second bisection on the
// position, only when a tie straddles the cut).  A row whose bracket missed is marked pending
// and searched exactly by k_row_fallback.  grid (W, Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_row_finish(Prob pb, const uint32_t* __restrict__ cnt_hi,
                                                    const unsigned long long* __restrict__ sum_hi,
                                                    const uint32_t* __restrict__ ncand,
                                                    const float* __restrict__ cand_val,
                                                    const int* __restrict__ cand_idx,
                                                    const float2* __restrict__ thr,
                                                    unsigned long long* __restrict__ rowsum) {
  constexpr int NPT = CAND_CAP / 256;
  __shared__ CountSmem cs;
  __shared__ unsigned long long isum[4];
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  const int k = min(head_budget(pb, g), pb.P);
  if (k >= pb.P) {
    if (threadIdx.x == 0) rowsum[r] = (unsigned long long)pb.P * (unsigned long long)(pb.P - 1) / 2ull;
    return;
  }
  const uint32_t ch = cnt_hi[r], nc = ncand[r];
  const unsigned long long shi = sum_hi[r];          // fetched with the counters, used at the very end
  const bool ok = ch < (uint32_t)k && (uint32_t)k <= ch + nc && nc <= (uint32_t)CAND_CAP;
  if (!ok) {
    if (threadIdx.x == 0) rowsum[r] = ROW_PENDING;
    return;
  }
  const uint32_t need = (uint32_t)k - ch;
  // All loads unconditional (an empty slot re-reads entry 0 and is then masked): independent
  // loads in flight together instead of one round trip per slot.  Only as many slots per thread
  // as the row's candidates need (block-uniform), so a short list is counted quickly.
  const float2 th = thr[r];
  auto run = [&](auto nsc) {
    constexpr int NS = decltype(nsc)::value;
    uint32_t ck[NS], ci[NS];
    float fv[NS];
    int iv[NS];
#pragma unroll
    for (int j = 0; j < NS; ++j) {
      const uint32_t x = threadIdx.x + j * 256;
      const int64_t o = (int64_t)r * CAND_CAP + (x < nc ? x : 0u);
      fv[j] = cand_val[o];
      iv[j] = cand_idx[o];
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
__global__ __launch_bounds__(256) void k_row_finish_slices(Prob pb, const uint32_t* __restrict__ cnt_hi,
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
    if (threadIdx.x == 0) rowsum[r] = ROW_PENDING;
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

// Exact search (radix select + ordered visit) of the rows k_row_finish marked pending.
// grid (W, Hkv), SEL_NT threads; a workgroup whose row is done exits at once.
__global__ __launch_bounds__(SEL_NT) void k_row_fallback(Prob pb, const float* __restrict__ score,
                                                         unsigned long long* __restrict__ rowsum) {
  __shared__ SelectSmem sm;
  const int i = blockIdx.x, g = blockIdx.y, r = g * pb.W + i;
  if (rowsum[r] != ROW_PENDING) return;
  const float* row = score + (int64_t)r * pb.ld;
  const int k = min(head_budget(pb, g), pb.P);
  uint32_t tau, n_gt, k_eq;
  block_kth_key(row, pb.P, k, sm, tau, n_gt, k_eq);
  unsigned long long acc = 0;
  block_visit_topk(row, pb.P, tau, k_eq, sm, [&](int x, uint32_t) { acc += (unsigned long long)x; });
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) acc += __shfl_xor(acc, o, 64);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sm.isum[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long tot = 0;
    for (int j = 0; j < SEL_NW; ++j) tot += sm.isum[j];
    rowsum[r] = tot;
  }
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
// grid (ceil(P/256), Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_box(Prob pb, const float* __restrict__ ema,
                                             const unsigned long long* __restrict__ rowsum,
                                             float* __restrict__ fin, int32_t* __restrict__ aws_info,
                                             double* __restrict__ aws_d) {
  const int g = blockIdx.y;
  __shared__ int sh_ws, sh_gamma;
  __shared__ unsigned long long sh_sum[2][4];
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
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= pb.P) return;
  const float* e = ema + (int64_t)g * pb.ld;
  const int half = w_s / 2;
  const int lo = max(0, n + gamma - half), hi = min(pb.P - 1, n + gamma + half);
  float s = 0.f;
  for (int m = lo; m <= hi; ++m) s += e[m];
  fin[(int64_t)g * pb.ld + n] = s / (float)w_s;
}

}  // namespace

int launch_smooth(const Prob& pb, const float* score, float* ema, float* fin, int32_t* aws_info,
                  double* aws_d, char* ws, const SmoothWs& lay, hipStream_t st) {
  unsigned long long* rowsum = (unsigned long long*)(ws + lay.rowsum);
  float2* thr = (float2*)(ws + lay.thr);
  uint32_t* cnt_hi = (uint32_t*)(ws + lay.cnt_hi);
  unsigned long long* sum_hi = (unsigned long long*)(ws + lay.sum_hi);
  uint32_t* ncand = (uint32_t*)(ws + lay.ncand);
  float* cand_val = (float*)(ws + lay.cand_val);
  int* cand_idx = (int*)(ws + lay.cand_idx);
  float* e = ema ? ema : (float*)(ws + lay.ema);
  const int vec = ((pb.ld & 3) == 0 && ((uintptr_t)score & 15u) == 0) ? 1 : 0;
  if (pb.adaptive)
    RK_LAUNCH(ST_ROWTOPK, st, k_sample_bracket, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, score, thr,
              cnt_hi, sum_hi, ncand);
  RK_LAUNCH(ST_EMA, st, k_ema_scan, dim3((pb.P + NPB - 1) / NPB, pb.Hkv), dim3(256), 0, st, pb, score, e,
            thr, cnt_hi, sum_hi, ncand, cand_val, cand_idx, vec);
  if (pb.adaptive) {
    RK_LAUNCH(ST_ROWTOPK, st, k_row_finish, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, cnt_hi, sum_hi,
              ncand, cand_val, cand_idx, thr, rowsum);
    RK_LAUNCH(ST_ROWTOPK, st, k_row_fallback, dim3(pb.W, pb.Hkv), dim3(SEL_NT), 0, st, pb, score, rowsum);
  }
  RK_LAUNCH(ST_BOX, st, k_box, dim3((pb.P + 255) / 256, pb.Hkv), dim3(256), 0, st, pb, e, rowsum, fin,
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
  RK_LAUNCH(ST_ROWTOPK, st, k_row_finish_slices, dim3(pb.W, pb.Hkv), dim3(256), 0, st, pb, fp.cnt_hi,
            fp.sum_hi, fp.scnt, fp.sval, fp.sidx, nchunks, fp.caps, fp.thr, rowsum);
  RK_LAUNCH(ST_ROWTOPK, st, k_row_fallback, dim3(pb.W, pb.Hkv), dim3(SEL_NT), 0, st, pb, score, rowsum);
  RK_LAUNCH(ST_BOX, st, k_box, dim3((pb.P + 255) / 256, pb.Hkv), dim3(256), 0, st, pb, ema, rowsum, fin,
            aws_info, aws_d);
  return hip_status();
}

}  // namespace restkv
