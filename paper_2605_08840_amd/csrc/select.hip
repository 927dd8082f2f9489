// Per-head selection (Sec. 3.3, Eq. topk): top-(B-W) prefix positions in ascending order,
// window positions appended.
//
// The row of final scores of a head is cut into chunks that many workgroups scan in parallel:
//   bracket : a sample of the row brackets the threshold of the top-(B-W)
//   scan    : per chunk, count the entries above the bracket, collect those inside it
//   finish  : exact threshold among the candidates (bisection on keys; ties by position)
//   fallback: a head whose bracket missed is searched with the exact radix select
//   count   : per chunk, number of selected entries
//   emit    : per chunk, ordered write at the offset given by the counts of the earlier chunks
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

constexpr int SCH = 4096;            // positions per chunk
constexpr int SCAP = 4096;           // candidates kept per head
constexpr uint32_t PENDING = 0xFFFFFFFFu;

struct SelPtrs {
  float2* thr; uint32_t* cnt_hi; uint32_t* ncand; float* cand_val; int* cand_idx;
  uint32_t* cut;          // [Hkv,4]: threshold key, position cut for ties, state, unused
  uint32_t* counts;       // [Hkv, nchunks]
};

// grid (Hkv), 256 threads
__global__ __launch_bounds__(256) void k_sel_bracket(Prob pb, const float* __restrict__ fin, SelPtrs w) {
  __shared__ CountSmem cs;
  const int g = blockIdx.x;
  const float* row = fin + (int64_t)g * pb.ld;
  const int k = head_budget(pb, g) - pb.W;
  if (threadIdx.x == 0) { w.cnt_hi[g] = 0; w.ncand[g] = 0; }
  if (k >= pb.P) {
    if (threadIdx.x == 0) w.thr[g] = make_float2(INFINITY, INFINITY);
    return;
  }
  int it = 0;
  uint32_t klo, khi;
  block_bracket<SEL_NS / 256, 1>(row, pb.P, k, cs, it, klo, khi);   // smoothed rows: single, spread samples
  if (threadIdx.x == 0)
    w.thr[g] = make_float2(klo ? key_float(klo) : -INFINITY, khi != 0xFFFFFFFFu ? key_float(khi) : INFINITY);
}

// grid (chunks, Hkv), 256 threads, 16 positions per thread
__global__ __launch_bounds__(256) void k_sel_scan(Prob pb, const float* __restrict__ fin, SelPtrs w) {
  __shared__ uint32_t list[SCH];
  __shared__ uint32_t lcnt, hcnt, base;
  const int g = blockIdx.y, tid = threadIdx.x;
  const int n00 = blockIdx.x * SCH;
  const float* row = fin + (int64_t)g * pb.ld;
  const float2 th = w.thr[g];
  if (tid == 0) { lcnt = 0; hcnt = 0; }
  __syncthreads();
  uint32_t nh = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int nl = (j * 256 + tid) * 4;            // coalesced float4 per thread
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int n = n00 + nl + e;
      const float x = n < pb.P ? row[n] : -INFINITY;
      if (x > th.y) ++nh;
      else if (x > th.x) list[atomicAdd(&lcnt, 1u)] = (uint32_t)(nl + e);
    }
  }
  nh = wave_sum(nh);
  if ((tid & 63) == 0 && nh) atomicAdd(&hcnt, nh);
  __syncthreads();
  const uint32_t E = lcnt;
  if (tid == 0) {
    if (E) base = atomicAdd(&w.ncand[g], E);
    if (hcnt) atomicAdd(&w.cnt_hi[g], hcnt);
  }
  __syncthreads();
  for (uint32_t x = tid; x < E; x += 256) {
    const uint32_t pos = base + x;
    if (pos < (uint32_t)SCAP) {
      const int n = n00 + (int)list[x];
      w.cand_val[(int64_t)g * SCAP + pos] = row[n];
      w.cand_idx[(int64_t)g * SCAP + pos] = n;
    }
  }
}

// grid (Hkv), 256 threads
__global__ __launch_bounds__(256) void k_sel_finish(Prob pb, SelPtrs w) {
  constexpr int NPT = SCAP / 256;
  __shared__ CountSmem cs;
  const int g = blockIdx.x;
  const int k = head_budget(pb, g) - pb.W;
  uint32_t* cut = w.cut + 4 * g;
  if (k >= pb.P) {                      // everything is kept
    if (threadIdx.x == 0) { cut[0] = 0u; cut[1] = 0xFFFFFFFFu; cut[2] = 1u; }
    return;
  }
  const uint32_t ch = w.cnt_hi[g], nc = w.ncand[g];
  const bool ok = ch < (uint32_t)k && (uint32_t)k <= ch + nc && nc <= (uint32_t)SCAP;
  if (!ok) {
    if (threadIdx.x == 0) cut[2] = PENDING;
    return;
  }
  const uint32_t need = (uint32_t)k - ch;
  // unconditional loads (an empty slot re-reads entry 0 and is then masked): all in flight at once
  uint32_t ck[NPT], ci[NPT];
  {
    float fv[NPT];
    int iv[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const uint32_t x = threadIdx.x + j * 256;
      const int64_t o = (int64_t)g * SCAP + (x < nc ? x : 0u);
      fv[j] = w.cand_val[o];
      iv[j] = w.cand_idx[o];
    }
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const bool in = (uint32_t)(threadIdx.x + j * 256) < nc;
      ck[j] = in ? float_key(fv[j]) : 0u;
      ci[j] = in ? (uint32_t)iv[j] : 0u;
    }
  }
  int it = 0, top_bit;
  uint32_t prefix;
  {                                     // every candidate lies inside the bracket: its leading bits are known
    const float2 th = w.thr[g];
    common_prefix(float_key(th.x), float_key(th.y), top_bit, prefix);
  }
  const uint32_t t = block_kth<NPT>(ck, need, cs, it, top_bit, prefix);
  uint32_t cge, cgt;
  block_count_ge2<NPT>(ck, t, t + 1u, cs, it, cge, cgt);
  const uint32_t k_eq = need - cgt;
  uint32_t pos_cut = 0xFFFFFFFFu;
  if (cge - cgt > k_eq) {               // a run of equal values straddles the cut: lowest positions win
    uint32_t inv[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) inv[j] = ck[j] == t ? 0xFFFFFFFFu - ci[j] : 0u;
    pos_cut = 0xFFFFFFFFu - block_kth<NPT>(inv, k_eq, cs, it);
  }
  if (threadIdx.x == 0) { cut[0] = t; cut[1] = pos_cut; cut[2] = 1u; }
}

// grid (Hkv), SEL_NT threads; exits unless the head is pending
__global__ __launch_bounds__(SEL_NT) void k_sel_fallback(Prob pb, const float* __restrict__ fin, SelPtrs w) {
  __shared__ SelectSmem sm;
  __shared__ uint32_t maxpos;
  const int g = blockIdx.x;
  uint32_t* cut = w.cut + 4 * g;
  if (cut[2] != PENDING) return;
  const float* row = fin + (int64_t)g * pb.ld;
  uint32_t tau, n_gt, k_eq;
  block_kth_key(row, pb.P, head_budget(pb, g) - pb.W, sm, tau, n_gt, k_eq);
  if (threadIdx.x == 0) maxpos = 0;
  __syncthreads();
  // position of the last tie that is taken
  block_visit_topk(row, pb.P, tau, k_eq, sm, [&](int x, uint32_t) {
    if (float_key(row[x]) == tau) atomicMax(&maxpos, (uint32_t)x);
  });
  __syncthreads();
  if (threadIdx.x == 0) { cut[0] = tau; cut[1] = maxpos; cut[2] = 1u; }
}

__device__ __forceinline__ bool sel_pred(float x, int n, uint32_t tau, uint32_t pos_cut) {
  const uint32_t key = float_key(x);
  // one 64-bit comparison of (key, inverted position) against (tau, inverted cut); the form
  // "key > tau || (key == tau && n <= pos_cut)" has been seen miscompiled by hipcc 7.2 at -O3
  const unsigned long long a = ((unsigned long long)key << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)n);
  const unsigned long long b = ((unsigned long long)tau << 32) | (unsigned long long)(0xFFFFFFFFu - pos_cut);
  return a >= b;
}

// grid (chunks, Hkv), 256 threads; thread t owns the 16 consecutive positions 16 t .. 16 t + 15
__global__ __launch_bounds__(256) void k_sel_count(Prob pb, const float* __restrict__ fin, SelPtrs w,
                                                   int nchunks) {
  __shared__ uint32_t tot;
  const int g = blockIdx.y, tid = threadIdx.x;
  const float* row = fin + (int64_t)g * pb.ld;
  const uint32_t tau = w.cut[4 * g], pos_cut = w.cut[4 * g + 1];
  if (tid == 0) tot = 0;
  __syncthreads();
  uint32_t c = 0;
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    const int n = blockIdx.x * SCH + j * 256 + tid;          // order is irrelevant for a count
    if (n < pb.P && sel_pred(row[n], n, tau, pos_cut)) ++c;
  }
  c = wave_sum(c);
  if ((tid & 63) == 0 && c) atomicAdd(&tot, c);
  __syncthreads();
  if (tid == 0) w.counts[g * nchunks + blockIdx.x] = tot;
}

__global__ __launch_bounds__(256) void k_sel_emit(Prob pb, const float* __restrict__ fin, SelPtrs w,
                                                  int nchunks, int32_t* __restrict__ idx) {
  __shared__ uint32_t wsum[4];
  const int g = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const float* row = fin + (int64_t)g * pb.ld;
  const uint32_t tau = w.cut[4 * g], pos_cut = w.cut[4 * g + 1];
  const int bg = head_budget(pb, g), bp = bg - pb.W;
  int32_t* out = idx + (int64_t)g * pb.B;
  // selected entries in the chunks before this one: loads spread over the threads, then summed
  __shared__ uint32_t offs[4];
  uint32_t off = 0;
  for (int c = tid; c < (int)blockIdx.x; c += 256) off += w.counts[g * nchunks + c];
  off = wave_sum(off);
  if (lane == 0) offs[wv] = off;
  __syncthreads();
  off = offs[0] + offs[1] + offs[2] + offs[3];
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
  const int nch = (pb.P + SCH - 1) / SCH;
  size_t off = 0;
  auto take = [&](size_t b) { off = align_up(off + b); };
  take((size_t)pb.Hkv * 8); take((size_t)pb.Hkv * 4); take((size_t)pb.Hkv * 4);
  take((size_t)pb.Hkv * SCAP * 4); take((size_t)pb.Hkv * SCAP * 4);
  take((size_t)pb.Hkv * 16); take((size_t)pb.Hkv * nch * 4);
  return off;
}

int launch_select(const Prob& pb, const float* fin, int32_t* idx, char* ws, hipStream_t st) {
  const int nch = (pb.P + SCH - 1) / SCH;
  SelPtrs w;
  size_t off = 0;
  auto take = [&](size_t b) { char* p = ws + off; off = align_up(off + b); return p; };
  w.thr = (float2*)take((size_t)pb.Hkv * 8);
  w.cnt_hi = (uint32_t*)take((size_t)pb.Hkv * 4);
  w.ncand = (uint32_t*)take((size_t)pb.Hkv * 4);
  w.cand_val = (float*)take((size_t)pb.Hkv * SCAP * 4);
  w.cand_idx = (int*)take((size_t)pb.Hkv * SCAP * 4);
  w.cut = (uint32_t*)take((size_t)pb.Hkv * 16);
  w.counts = (uint32_t*)take((size_t)pb.Hkv * nch * 4);
  RK_LAUNCH(ST_SELECT, st, k_sel_bracket, dim3(pb.Hkv), dim3(256), 0, st, pb, fin, w);
  RK_LAUNCH(ST_SELECT, st, k_sel_scan, dim3(nch, pb.Hkv), dim3(256), 0, st, pb, fin, w);
  RK_LAUNCH(ST_SELECT, st, k_sel_finish, dim3(pb.Hkv), dim3(256), 0, st, pb, w);
  RK_LAUNCH(ST_SELECT, st, k_sel_fallback, dim3(pb.Hkv), dim3(SEL_NT), 0, st, pb, fin, w);
  RK_LAUNCH(ST_SELECT, st, k_sel_count, dim3(nch, pb.Hkv), dim3(256), 0, st, pb, fin, w, nch);
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
