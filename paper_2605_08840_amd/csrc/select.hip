// Per-head selection (Sec. 3.3, Eq. topk): top-(B-W) prefix positions in ascending order,
// window positions appended.
//
// The row of final scores of a head is cut into chunks that many workgroups scan in parallel:
//   scan    : per chunk: a sample of the row brackets the threshold of the top-(B-W) (every
//             workgroup of the head repeats this search); count the entries above the bracket;
//             those inside it leave as bit masks
//   finish  : per head, exact threshold among the candidates (bisection on keys; ties by
//             position), or the exact radix search of the whole row if the bracket missed;
//             number of selected entries before every chunk
//   emit    : per chunk, ordered write at that offset
#include <mutex>

#include "rowselect.hpp"

namespace restkv {

namespace {

// Scratch of restkv_select_static: one array per GPU, held until the process ends.  Host code
// never passes the array's name to a kernel: its device address is looked up once per device.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
char* g_scratch_ptr[MAX_DEVICES];    // device address of `scratch` on each GPU, nullptr until asked for

// Device address of the current GPU's copy of `scratch` (RESTKV_EHIP if the runtime refuses).
int static_scratch(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return RESTKV_EHIP;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return RESTKV_EHIP;
    g_scratch_ptr[dev] = (char*)ptr;
  }
  *out = g_scratch_ptr[dev];
  return RESTKV_OK;
}

constexpr int SCH = 4096;            // positions per chunk = workgroup of the scan (16 per thread)
constexpr int SCAP = 4096;           // candidates the finishing step can take
constexpr int LHIST = 8192;          // chunk counters kept in LDS by the finishing step

struct SelPtrs {
  float2* thr;            // [Hkv] bracket of the head's threshold
  uint32_t* above;        // [Hkv, nchunks] entries above the bracket
  uint16_t* cmask;        // [Hkv, nchunks * 256] entries inside the bracket: 16 bits per thread of the scan
  uint32_t* cut;          // [Hkv, 4] threshold key, position cut for ties
  uint32_t* offs;         // [Hkv, nchunks] selected entries in the chunks before
};

SelPtrs sel_ptrs(const Prob& pb, char* ws, size_t* bytes) {
  const size_t nch = (size_t)(pb.P + SCH - 1) / SCH;
  size_t off = 0;
  auto take = [&](size_t b) { char* p = ws ? ws + off : nullptr; off = align_up(off + b); return p; };
  SelPtrs w;
  w.thr = (float2*)take((size_t)pb.Hkv * 8);
  w.above = (uint32_t*)take((size_t)pb.Hkv * nch * 4);
  w.cmask = (uint16_t*)take((size_t)pb.Hkv * nch * 512);
  w.cut = (uint32_t*)take((size_t)pb.Hkv * 16);
  w.offs = (uint32_t*)take((size_t)pb.Hkv * nch * 4);
  if (bytes) *bytes = off;
  return w;
}

__device__ __forceinline__ bool sel_pred(float x, int n, uint32_t tau, uint32_t pos_cut) {
  const uint32_t key = float_key(x);
  // one 64-bit comparison of (key, inverted position) against (tau, inverted cut); the form
  // "key > tau || (key == tau && n <= pos_cut)" has been seen miscompiled by hipcc 7.2 at -O3
  const unsigned long long a = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)n);
  const unsigned long long b = ((unsigned long long)tau << 32) | (unsigned long long)(0xFFFFFFFFu - pos_cut);
  return a >= b;
}

// Bracket and scan of one chunk of a head's final scores.  Every workgroup of a head first
// brackets the head's top-(B-W) threshold from the same sample of the row (same arithmetic, same
// result: thirty-two workgroups repeating a search that would otherwise leave all but eight
// compute units idle behind a launch of its own), with the loads of its own chunk already in
// flight.  Thread t then owns positions chunk * 4096 + 16 t .. + 15: the entries above the bracket
// are counted (one count per chunk), the entries inside it leave as a 16-bit mask per thread
// (element e at bit 15 - e).  grid (chunks, Hkv), 256 threads.
__global__ __launch_bounds__(256) void k_sel_scan(Prob pb, const float* __restrict__ fin, SelPtrs w,
                                                  int nchunks, int vec) {
  __shared__ CountSmem cs;
  __shared__ uint32_t red[4];
  const int g = blockIdx.y, ch = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float* row = fin + (int64_t)g * pb.ld;
  const int n0 = ch * SCH + 16 * tid;
  float x[16];
  if (vec && n0 + 15 < pb.P) {
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const float4 v4 = *(const float4*)(row + n0 + 4 * q4);
      x[4 * q4] = v4.x; x[4 * q4 + 1] = v4.y; x[4 * q4 + 2] = v4.z; x[4 * q4 + 3] = v4.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = row[min(n0 + e, pb.P - 1)];     // unconditional, masked below
#pragma unroll
    for (int e = 0; e < 16; ++e) x[e] = n0 + e < pb.P ? x[e] : -INFINITY;
  }
  const int k = head_budget(pb, g) - pb.W;
  float2 th = make_float2(INFINITY, INFINITY);          // everything is kept: nothing above, nothing inside
  if (k < pb.P) {                                       // block-uniform
    int it = 0;
    uint32_t klo, khi;
    block_bracket<SEL_NS / 256, 1>(row, pb.P, k, cs, it, klo, khi);   // smoothed rows: single, spread samples
    th = make_float2(klo ? key_float(klo) : -INFINITY, khi != 0xFFFFFFFFu ? key_float(khi) : INFINITY);
  }
  if (ch == 0 && tid == 0) w.thr[g] = th;
  float tlo = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, th.x)));
  float thi = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, th.y)));
  settle_scalars(tlo, thi);
  uint32_t hb = 0, lb = 0;
#pragma unroll
  for (int e = 0; e < 16; e += 2) shift_in_gt_2x2(hb, lb, x[e], x[e + 1], thi, tlo);
  w.cmask[((int64_t)g * nchunks + ch) * 256 + tid] = (uint16_t)(lb & ~hb);
  const uint32_t c = wave_sum((uint32_t)__popc(hb));
  if (lane == 0) red[wv] = c;
  __syncthreads();
  if (tid == 0) w.above[g * nchunks + ch] = red[0] + red[1] + red[2] + red[3];
}

// Exact threshold of a head and the chunks' output offsets.  One workgroup per head
//   * adds up the chunks' counts, expands the head's masks into candidate positions and fetches
//     their values (at most SCAP);
//   * finds the threshold among them by bisection on the keys (from below the bracket's common
//     leading bits), cuts a run of equal values by position; this chain of barriers is run by
//     four wavefronts, the other twelve leave before it;
//   * or, if the bracket missed or holds too many candidates, searches the row exactly (radix
//     select and ordered visit, all sixteen wavefronts);
//   * leaves the cut and, per chunk, the number of selected entries in the chunks before it.
// grid (Hkv), SEL_NT = 1024 threads.
__global__ __launch_bounds__(SEL_NT) void k_sel_finish(Prob pb, const float* __restrict__ fin, SelPtrs w,
                                                       int nchunks) {
  __shared__ SelectSmem sm;
  __shared__ CountSmem cs;
  __shared__ uint32_t red[SEL_NW];
  __shared__ uint32_t flag, maxpos;
  __shared__ int cpos[SCAP];
  __shared__ uint32_t lhist[LHIST];
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float* row = fin + (int64_t)g * pb.ld;
  const int k = head_budget(pb, g) - pb.W;
  const float2 th = w.thr[g];
  uint32_t* cut = w.cut + 4 * g;
  uint32_t* offs = w.offs + (int64_t)g * nchunks;
  const uint32_t* above = w.above + (int64_t)g * nchunks;
  if (k >= pb.P) {                               // everything is kept
    if (tid == 0) { cut[0] = 0u; cut[1] = 0xFFFFFFFFu; }
    for (int c = tid; c < nchunks; c += SEL_NT) offs[c] = (uint32_t)c * (uint32_t)SCH;
    return;
  }
  const bool lds_hist = nchunks <= LHIST;
  if (lds_hist) for (int c = tid; c < nchunks; c += SEL_NT) lhist[c] = 0;
  else for (int c = tid; c < nchunks; c += SEL_NT) offs[c] = 0;      // (global counters: offs itself)
  // counts above the bracket and number of candidates
  const int ndw = nchunks * 128;                 // two threads of the scan per 32-bit word
  const uint32_t* mrow = (const uint32_t*)(w.cmask + (int64_t)g * nchunks * 256);
  uint32_t c_mine = 0, a_mine = 0;
  for_each_mask_word<SEL_NT>(mrow, ndw, [&](int, uint32_t m) { c_mine += (uint32_t)__popc(m); });
  for (int c = tid; c < nchunks; c += SEL_NT) a_mine += above[c];
  const uint32_t incl = block_incl_scan(c_mine, sm.wsum);
  __syncthreads();
  a_mine = wave_sum(a_mine);
  if (lane == 0) red[wv] = a_mine;
  if (tid == SEL_NT - 1) flag = incl;
  __syncthreads();
  const uint32_t nc = flag;
  uint32_t n_above = 0;
  for (int j = 0; j < SEL_NW; ++j) n_above += red[j];
  const bool ok = n_above < (uint32_t)k && (uint32_t)k <= n_above + nc && nc <= (uint32_t)SCAP;
  uint32_t tau, pos_cut;
  int nthr = SEL_NT;                             // threads that go on
  if (ok) {                                      // block-uniform
    uint32_t slot = incl - c_mine;
    for_each_mask_word<SEL_NT>(mrow, ndw, [&](int x, uint32_t m) {
      while (m) {
        const int b = __builtin_ctz(m);
        m &= m - 1;
        cpos[slot++] = 16 * (2 * x + (b >> 4)) + 15 - (b & 15);  // half word = thread of the scan, bit 15 - e = element e
      }
    });
    __syncthreads();
    // The bisection is a chain of barriers: four wavefronts go through it much faster than
    // sixteen, so the other twelve leave here (whole wavefronts; a barrier only counts the
    // wavefronts that are still there).
    constexpr int FW = 4, FT = FW * 64, FPT = SCAP / FT;
    if (tid >= FT) return;
    nthr = FT;
    const uint32_t need = (uint32_t)k - n_above;
    uint32_t ck[FPT], ci[FPT];
    {
      float fv[FPT];
      int iv[FPT];
#pragma unroll
      for (int j = 0; j < FPT; ++j) {            // unconditional loads, masked afterwards: all in flight at once
        const uint32_t x = tid + j * FT;
        iv[j] = cpos[x < nc ? x : 0u];
        fv[j] = row[iv[j]];
      }
#pragma unroll
      for (int j = 0; j < FPT; ++j) {
        const bool in = (uint32_t)(tid + j * FT) < nc;
        ck[j] = in ? float_key(fv[j]) : 0u;
        ci[j] = in ? (uint32_t)iv[j] : 0u;
      }
    }
    int it = 0, top_bit;
    uint32_t prefix;
    common_prefix(float_key(th.x), float_key(th.y), top_bit, prefix);   // every candidate lies inside the bracket
    tau = block_kth<FPT, FW>(ck, need, cs, it, top_bit, prefix);
    uint32_t cge, cgt;
    block_count_ge2<FPT, FW>(ck, tau, tau + 1u, cs, it, cge, cgt);
    const uint32_t k_eq = need - cgt;
    pos_cut = 0xFFFFFFFFu;
    if (cge - cgt > k_eq) {                      // a run of equal values straddles the cut: lowest positions win
      uint32_t inv[FPT];
#pragma unroll
      for (int j = 0; j < FPT; ++j) inv[j] = ck[j] == tau ? 0xFFFFFFFFu - ci[j] : 0u;
      pos_cut = 0xFFFFFFFFu - block_kth<FPT, FW>(inv, k_eq, cs, it);
    }
    // selected candidates per chunk
    const unsigned long long cutw = ((unsigned long long)tau << 32) | (unsigned long long)(0xFFFFFFFFu - pos_cut);
#pragma unroll
    for (int j = 0; j < FPT; ++j) {
      const unsigned long long kj = ((unsigned long long)ck[j] << 32) | (unsigned long long)(0xFFFFFFFFu - ci[j]);
      if ((uint32_t)(tid + j * FT) < nc && kj >= cutw) atomicAdd(lds_hist ? &lhist[ci[j] / SCH] : &offs[ci[j] / SCH], 1u);
    }
  } else {
    // exact search of the whole row: threshold, then an ordered visit that counts the selected
    // entries of every chunk and finds the last tie that is taken
    uint32_t n_gt, k_eq;
    block_kth_key(row, pb.P, k, sm, tau, n_gt, k_eq);
    if (tid == 0) maxpos = 0;
    __syncthreads();
    block_visit_topk(row, pb.P, tau, k_eq, sm, [&](int x, uint32_t) {
      if (float_key(row[x]) == tau) atomicMax(&maxpos, (uint32_t)x);
      atomicAdd(lds_hist ? &lhist[x / SCH] : &offs[x / SCH], 1u);
    });
    __syncthreads();
    pos_cut = maxpos;
  }
  __syncthreads();
  if (!lds_hist) __threadfence();              // (the global counters were atomics of this workgroup)
  if (tid == 0) { cut[0] = tau; cut[1] = pos_cut; }
  // selected entries before each chunk: running sum over the chunks, nthr at a time
  uint32_t run = 0;
  for (int c0 = 0; c0 < nchunks; c0 += nthr) {
    const int c = c0 + tid;
    uint32_t v = 0;
    if (c < nchunks) {
      v = lds_hist ? lhist[c] : __hip_atomic_load(&offs[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (ok) v += above[c];
    }
    const uint32_t inc = block_incl_scan(v, sm.wsum);
    if (c < nchunks) offs[c] = run + inc - v;
    __syncthreads();
    if (tid == nthr - 1) flag = inc;
    __syncthreads();
    run += flag;
    __syncthreads();
  }
}

// Ordered emission: the selected entries of a chunk go to idx at the offset the scan left; the
// window tokens and the unused tail of a smaller per-head budget are written by chunk 0.
// grid (chunks, Hkv), 256 threads; thread t owns the 16 consecutive positions 16 t .. 16 t + 15
__global__ __launch_bounds__(256) void k_sel_emit(Prob pb, const float* __restrict__ fin, SelPtrs w,
                                                  int nchunks, int32_t* __restrict__ idx) {
  __shared__ uint32_t wsum[4];
  const int g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float* row = fin + (int64_t)g * pb.ld;
  const uint32_t tau = w.cut[4 * g], pos_cut = w.cut[4 * g + 1];
  const int bg = head_budget(pb, g), bp = bg - pb.W;
  int32_t* out = idx + (int64_t)g * pb.B;
  const uint32_t off = w.offs[(int64_t)g * nchunks + blockIdx.x];
  const int n0 = blockIdx.x * SCH + tid * 16;
  uint32_t mask = 0;
#pragma unroll
  for (int q4 = 0; q4 < 4; ++q4) {
    float x[4];
    if (n0 + 4 * q4 + 3 < pb.P && (pb.ld & 3) == 0 && (((uintptr_t)fin) & 15u) == 0) {
      const float4 v4 = *(const float4*)(row + n0 + 4 * q4);
      x[0] = v4.x; x[1] = v4.y; x[2] = v4.z; x[3] = v4.w;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = n0 + 4 * q4 + e < pb.P ? row[n0 + 4 * q4 + e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = n0 + 4 * q4 + e;
      if (n < pb.P && sel_pred(x[e], n, tau, pos_cut)) mask |= 1u << (4 * q4 + e);
    }
  }
  // exclusive prefix of the per-thread counts over the block
  const uint32_t c = (uint32_t)__popc(mask);
  uint32_t incl = c;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t y = __shfl_up(incl, o, 64);
    if (lane >= o) incl += y;
  }
  if (lane == 63) wsum[wv] = incl;
  __syncthreads();
  uint32_t pos = off + incl - c;
  for (int j = 0; j < wv; ++j) pos += wsum[j];
  for (uint32_t m = mask; m; m &= m - 1) {
    const int e = __ffs(m) - 1;
    if (pos < (uint32_t)bp) out[pos] = n0 + e;
    ++pos;
  }
  if (blockIdx.x == 0) {
    for (int j = tid; j < pb.W; j += 256) out[bp + j] = pb.P + j;
    for (int j = bg + tid; j < pb.B; j += 256) out[j] = -1;     // a smaller per-head budget: unused tail
  }
}

}  // namespace

size_t select_ws_bytes(const Prob& pb) {
  size_t n = 0;
  sel_ptrs(pb, nullptr, &n);
  return n;
}

int launch_select(const Prob& pb, const float* fin, int32_t* idx, char* ws, hipStream_t st) {
  const int nch = (pb.P + SCH - 1) / SCH;
  const SelPtrs w = sel_ptrs(pb, ws, nullptr);
  const int vec = ((pb.ld & 3) == 0 && ((uintptr_t)fin & 15u) == 0) ? 1 : 0;
  RK_LAUNCH(ST_SELECT, st, k_sel_scan, dim3(nch, pb.Hkv), dim3(256), 0, st, pb, fin, w, nch, vec);
  RK_LAUNCH(ST_SELECT, st, k_sel_finish, dim3(pb.Hkv), dim3(SEL_NT), 0, st, pb, fin, w, nch);
  RK_LAUNCH(ST_SELECT, st, k_sel_emit, dim3(nch, pb.Hkv), dim3(256), 0, st, pb, fin, w, nch, idx);
  return hip_status();
}

size_t select_static_capacity() { return STATIC_SCRATCH_BYTES; }

int launch_select_static(const Prob& pb, const float* fin, int32_t* idx, hipStream_t st) {
  if (select_ws_bytes(pb) > STATIC_SCRATCH_BYTES) return RESTKV_EWORKSPACE;
  char* ws = nullptr;
  const int rc = static_scratch(&ws);
  if (rc) return rc;
  return launch_select(pb, fin, idx, ws, st);
}

}  // namespace restkv
