// C ABI of the ReST-KV eviction library: argument validation, scratch layout, dispatch.
// Everything behind these entry points is a hand-written HIP kernel for gfx950.
#include <math.h>

#include "common.hpp"

namespace restkv {

int resolve(const restkv_params* p, Prob* o) {
  if (!p || !o) return RESTKV_EINVAL;
  if (p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->n_q_heads % p->n_kv_heads) return RESTKV_EINVAL;
  if (p->seq_len < 2 || p->window < 1 || p->window >= p->seq_len) return RESTKV_EINVAL;
  if (p->budget <= p->window || p->budget > p->seq_len) return RESTKV_EINVAL;
  if (p->base_window < 1 || !(p->base_window & 1)) return RESTKV_EINVAL;
  if (p->variant & ~0x77) return RESTKV_EINVAL;
  if ((p->variant & 3) == 3 || ((p->variant >> 4) & 3) == 3) return RESTKV_EINVAL;
  if (!(p->ema_alpha >= 0.f && p->ema_alpha <= 1.f)) return RESTKV_EINVAL;
  if (p->adaptive && !(p->beta > 0.f)) return RESTKV_EINVAL;
  // |D_front - D_rear| < L, so floor(|x| / beta) stays a 32-bit integer with room to spare
  if (p->adaptive && (double)p->seq_len / (double)p->beta >= 1073741824.0) return RESTKV_EINVAL;
  if (!(p->scale >= 0.f) || isinf(p->scale)) return RESTKV_EINVAL;
  if (p->head_dim != 64 && p->head_dim != 128) return RESTKV_EUNSUPPORTED;
  if (p->dtype != RESTKV_F32 && p->dtype != RESTKV_BF16) return RESTKV_EUNSUPPORTED;
  o->Hq = p->n_q_heads; o->Hkv = p->n_kv_heads; o->G = o->Hq / o->Hkv;
  o->d = p->head_dim; o->L = p->seq_len; o->W = p->window; o->P = o->L - o->W;
  o->B = p->budget; o->R = o->G * o->W; o->hb = nullptr; o->ext_out = nullptr; o->ext_lse = nullptr;
  if ((int64_t)o->G * o->W > 4096) return RESTKV_EUNSUPPORTED;
  o->dtype = p->dtype; o->causal = p->causal ? 1 : 0; o->base_k = p->base_window;
  o->ind = p->variant & 3; o->gmax = (p->variant >> 2) & 1; o->tmode = (p->variant >> 4) & 3;
  o->pmax = (p->variant >> 6) & 1;
  o->adaptive = (p->adaptive && o->W >= 2) ? 1 : 0;
  o->scale = p->scale > 0.f ? p->scale : 1.0f / sqrtf((float)o->d);
  o->alpha = p->ema_alpha; o->beta = p->beta;
  o->q_st = p->q_stride_t ? p->q_stride_t : o->d;
  o->q_sh = p->q_stride_h ? p->q_stride_h : (int64_t)o->W * o->d;
  o->kv_st = p->kv_stride_t ? p->kv_stride_t : o->d;
  o->kv_sh = p->kv_stride_h ? p->kv_stride_h : (int64_t)o->L * o->d;
  o->ld = p->ld_score ? p->ld_score : o->P;
  if (o->q_st < o->d || o->kv_st < o->d || o->q_sh < 0 || o->kv_sh < 0 || o->ld < o->P) return RESTKV_EINVAL;
  return RESTKV_OK;
}

ScoreWs score_ws(const Prob& pb) {
  ScoreWs w;
  // enough key splits to give every CU work, each at least one 64-key tile
  int S = (pb.L + 1023) / 1024;
  if (S < 1) S = 1;
  if (S > 64) S = 64;
  w.S_simple = S;
  w.S_max = 64;
  S = w.S_max;
  w.ldv = (pb.P + 3) / 4 * 4;
  const size_t rows = (size_t)pb.Hq * pb.W;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  w.part_m = take(rows * S * 4);
  w.part_mx = take(rows * S * 4);
  w.part_n = take(rows * S * 4);
  w.part_ref = take(rows * S * 4);
  w.part_l = take(rows * S * 4);
  w.part_z = take(rows * S * (size_t)pb.d * 4);
  w.rs_m = take(rows * 4);
  w.rs_l = take(rows * 4);
  w.rs_zz = take(rows * 4);
  w.rs_nstar = take(rows * 4);
  w.rs_istar = take(rows * 4);
  w.rs_u = take(rows * (size_t)pb.d * 4);
  w.vv = take((size_t)pb.Hq * w.ldv * 4);
  // operand-ordered copies for the matrix-core path: 32-row blocks hold Gp (power of two >= G)
  // heads of 32/Gp window positions
  w.nwb = 0;
  if (pb.G <= 32) {
    int gp = 1;
    while (gp < pb.G) gp <<= 1;
    const int iw = 32 / gp;
    w.nwb = (pb.W + iw - 1) / iw;
  }
  w.op = take((size_t)3 * pb.Hkv * w.nwb * 32 * pb.d * 2);
  w.bytes = off;
  return w;
}

SmoothWs smooth_ws(const Prob& pb) {
  SmoothWs w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  w.rowsum = take((size_t)pb.Hkv * pb.W * 8);
  w.ema = take((size_t)pb.Hkv * pb.ld * 4);
  const size_t rows = (size_t)pb.Hkv * pb.W;
  w.thr = take(rows * 8);
  w.cnt_hi = take(rows * 4);
  w.sum_hi = take(rows * 8);
  w.cmask = take(rows * (size_t)((pb.P + 1023) / 1024) * 64 * 2);
  w.bytes = off;
  return w;
}

FuseWs fuse_ws(const Prob& pb) {
  FuseWs w;
  w.ns = 8192;
  w.nchunks = pb.G <= 32 ? score_pass_chunks(pb) : 1;
  // a row's candidates (at most 4096 are usable) cluster in a few chunks: room for half of them
  // in every chunk, for all of them when there are only a few chunks
  const int caps = w.nchunks < 8 ? 4096 : 2048;
  w.caps = caps;
  const size_t rows = (size_t)pb.Hkv * pb.W;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  w.smp = take(rows * w.ns * 4);
  w.scnt = take(rows * w.nchunks * 4);
  w.sval = take(rows * w.nchunks * w.caps * 4);
  w.sidx = take(rows * w.nchunks * w.caps * 4);
  w.bytes = off;
  return w;
}

static bool g_force_fp32 = false;   // see restkv_debug_force_fp32

static int check_ws(const void* ws, size_t have, size_t need) {
  if (!ws || ((uintptr_t)ws & 255u) || have < need) return RESTKV_EWORKSPACE;
  return RESTKV_OK;
}

}  // namespace restkv

using namespace restkv;

extern "C" {

size_t restkv_workspace_bytes(const restkv_params* p) {
  Prob pb;
  if (resolve(p, &pb) != RESTKV_OK) return 0;
  size_t n = score_ws(pb).bytes;
  if (smooth_ws(pb).bytes > n) n = smooth_ws(pb).bytes;
  if (select_ws_bytes(pb) > n) n = select_ws_bytes(pb);
  // the fused call keeps the score scratch, the smoothing scratch and its own side by side
  const size_t f = align_up(score_ws(pb).bytes) + align_up(smooth_ws(pb).bytes) + fuse_ws(pb).bytes;
  if (f > n) n = f;
  return n;
}

int restkv_prepare_wo(const restkv_params* p, const float* w_o, int64_t d_model, float* gram,
                      restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!w_o || !gram || d_model < 1) return RESTKV_EINVAL;
  return launch_gram(pb, w_o, d_model, gram, (hipStream_t)stream);
}

int restkv_score(const restkv_params* p, const void* q, const void* k, const void* v,
                 const float* gram, float* score, void* workspace, size_t workspace_bytes,
                 restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!q || !k || !v || !score) return RESTKV_EINVAL;
  const ScoreWs lay = score_ws(pb);
  rc = check_ws(workspace, workspace_bytes, lay.bytes);
  if (rc) return rc;
  if (mfma_eligible(pb, q, k, v) && !g_force_fp32)
    return launch_score_mfma(pb, q, k, v, gram, score, (char*)workspace, lay, (hipStream_t)stream);
  return launch_score_simple(pb, q, k, v, gram, score, (char*)workspace, lay, (hipStream_t)stream);
}

int restkv_score_from_attention(const restkv_params* p, const void* q, const void* k, const void* v,
                                const float* gram, const float* attn_out, const float* lse, float* score,
                                void* workspace, size_t workspace_bytes, restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!q || !k || !v || !score || !attn_out || !lse) return RESTKV_EINVAL;
  pb.ext_out = attn_out;
  pb.ext_lse = lse;
  const ScoreWs lay = score_ws(pb);
  rc = check_ws(workspace, workspace_bytes, lay.bytes);
  if (rc) return rc;
  if (mfma_eligible(pb, q, k, v) && !g_force_fp32)
    return launch_score_mfma(pb, q, k, v, gram, score, (char*)workspace, lay, (hipStream_t)stream);
  return launch_score_simple(pb, q, k, v, gram, score, (char*)workspace, lay, (hipStream_t)stream);
}

static int smooth_impl(const restkv_params* p, const float* score, const int32_t* head_budget, float* ema,
                       float* final_score, int32_t* aws_info, double* aws_d, void* workspace,
                       size_t workspace_bytes, restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!score || !final_score) return RESTKV_EINVAL;
  pb.hb = head_budget;
  const SmoothWs lay = smooth_ws(pb);
  rc = check_ws(workspace, workspace_bytes, lay.bytes);
  if (rc) return rc;
  return launch_smooth(pb, score, ema, final_score, aws_info, aws_d, (char*)workspace, lay,
                       (hipStream_t)stream);
}

int restkv_smooth(const restkv_params* p, const float* score, float* ema, float* final_score,
                  int32_t* aws_info, double* aws_d, void* workspace, size_t workspace_bytes,
                  restkv_stream_t stream) {
  return smooth_impl(p, score, nullptr, ema, final_score, aws_info, aws_d, workspace, workspace_bytes, stream);
}

int restkv_smooth_b(const restkv_params* p, const float* score, const int32_t* head_budget, float* ema,
                    float* final_score, int32_t* aws_info, double* aws_d, void* workspace,
                    size_t workspace_bytes, restkv_stream_t stream) {
  if (!head_budget) return RESTKV_EINVAL;
  return smooth_impl(p, score, head_budget, ema, final_score, aws_info, aws_d, workspace, workspace_bytes, stream);
}

int restkv_score_smooth(const restkv_params* p, const void* q, const void* k, const void* v,
                        const float* gram, float* score, float* ema, float* final_score,
                        int32_t* aws_info, double* aws_d, void* workspace, size_t workspace_bytes,
                        restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!q || !k || !v || !score || !final_score) return RESTKV_EINVAL;
  const ScoreWs ls = score_ws(pb);
  const SmoothWs lm = smooth_ws(pb);
  hipStream_t st = (hipStream_t)stream;
  if (g_force_fp32 || p->variant != 0 || !fused_eligible(pb, q, k, v)) {
    // same result from the two separate calls (they use the workspace one after the other);
    // both sizes are checked first so that nothing is enqueued when the second call would fail
    rc = check_ws(workspace, workspace_bytes, ls.bytes > lm.bytes ? ls.bytes : lm.bytes);
    if (rc) return rc;
    rc = restkv_score(p, q, k, v, gram, score, workspace, workspace_bytes, stream);
    if (rc) return rc;
    return restkv_smooth(p, score, ema, final_score, aws_info, aws_d, workspace, workspace_bytes, stream);
  }
  const FuseWs lf = fuse_ws(pb);
  const size_t o_sm = align_up(ls.bytes), o_fu = o_sm + align_up(lm.bytes);
  rc = check_ws(workspace, workspace_bytes, o_fu + lf.bytes);
  if (rc) return rc;
  char* ws = (char*)workspace;
  char* wm = ws + o_sm;
  char* wf = ws + o_fu;
  FusedPtrs fp;
  fp.smp = (float*)(wf + lf.smp); fp.ns = lf.ns;
  fp.thr = (float2*)(wm + lm.thr); fp.cnt_hi = (uint32_t*)(wm + lm.cnt_hi);
  fp.sum_hi = (unsigned long long*)(wm + lm.sum_hi);
  fp.scnt = (uint32_t*)(wf + lf.scnt); fp.sval = (float*)(wf + lf.sval); fp.sidx = (int*)(wf + lf.sidx);
  fp.caps = lf.caps;
  fp.ema = ema ? ema : (float*)(wm + lm.ema);
  rc = launch_score_fused(pb, q, k, v, gram, score, ws, ls, fp, st);
  if (rc) return rc;
  return launch_smooth_fused_tail(pb, score, fp.ema, final_score, aws_info, aws_d, wm, lm, fp, lf.nchunks, st);
}

static int select_impl(const restkv_params* p, const float* final_score, const int32_t* head_budget,
                       int32_t* idx, void* workspace, size_t workspace_bytes, restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!final_score || !idx) return RESTKV_EINVAL;
  pb.hb = head_budget;
  rc = check_ws(workspace, workspace_bytes, select_ws_bytes(pb));
  if (rc) return rc;
  return launch_select(pb, final_score, idx, (char*)workspace, (hipStream_t)stream);
}

int restkv_select(const restkv_params* p, const float* final_score, int32_t* idx, void* workspace,
                  size_t workspace_bytes, restkv_stream_t stream) {
  return select_impl(p, final_score, nullptr, idx, workspace, workspace_bytes, stream);
}

int restkv_select_b(const restkv_params* p, const float* final_score, const int32_t* head_budget,
                    int32_t* idx, void* workspace, size_t workspace_bytes, restkv_stream_t stream) {
  if (!head_budget) return RESTKV_EINVAL;
  return select_impl(p, final_score, head_budget, idx, workspace, workspace_bytes, stream);
}

int restkv_select_static(const restkv_params* p, const float* final_score, int32_t* idx,
                         restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!final_score || !idx) return RESTKV_EINVAL;
  return launch_select_static(pb, final_score, idx, (hipStream_t)stream);
}

size_t restkv_select_static_capacity(void) { return select_static_capacity(); }

int restkv_compact(const restkv_params* p, const void* k, const void* v, const int32_t* idx,
                   void* k_out, void* v_out, restkv_stream_t stream) {
  Prob pb;
  int rc = resolve(p, &pb);
  if (rc) return rc;
  if (!k || !v || !idx || !k_out || !v_out) return RESTKV_EINVAL;
  return launch_compact(pb, k, v, idx, k_out, v_out, (hipStream_t)stream);
}

const char* restkv_strerror(int code) {
  switch (code) {
    case RESTKV_OK: return "ok";
    case RESTKV_EINVAL: return "invalid argument (null pointer, inconsistent shape or budget outside (W, L])";
    case RESTKV_EUNSUPPORTED: return "unsupported configuration (head_dim must be 64 or 128; dtype f32 or bf16)";
    case RESTKV_EWORKSPACE: return "workspace missing, not 256-byte aligned or smaller than restkv_workspace_bytes() (restkv_select_static: the problem needs more than the library's static scratch)";
    case RESTKV_EHIP: return "HIP runtime error at kernel launch";
    default: return "unknown error code";
  }
}

int restkv_version(void) { return 100; }

int restkv_debug_force_fp32(int on) {
  g_force_fp32 = on != 0;
  return RESTKV_OK;
}

}  // extern "C"
