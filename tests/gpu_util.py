"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding,
run the oracle, and the tolerance model of the indicator."""
from __future__ import annotations

import numpy as np
import torch

import workloads

RTOL = 1e-3          # relative tolerance of the indicator named by the benchmark spec
KAPPA_F32 = 2e-6     # relative accuracy of zz - 2 u.v + vv with every product in FP32
KAPPA_BF16 = 2e-6    # ... with bf16 MFMA operands (u split in two bf16 terms, FP32 accumulation)


def params_for(rk, w: workloads.Workload, **over):
    kw = dict(n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads, head_dim=w.head_dim, seq_len=w.seq_len,
              window=w.window, budget=w.budget, dtype=w.dtype, ema_alpha=w.alpha,
              base_window=w.base_window, beta=w.beta)
    kw.update(over)
    return rk.make_params(**kw)


def run_gpu_layer(rk, w, q, k, v, wo, dev="cuda", **over):
    """Whole path on the GPU; returns numpy copies of every output."""
    p = params_for(rk, w, **over)
    qd, kd, vd = (t.to(dev) for t in (q, k, v))
    gram = None
    if wo is not None:
        gram = torch.empty((w.n_q_heads, w.head_dim, w.head_dim), dtype=torch.float32, device=dev)
        rk.restkv_prepare_wo(p, wo.to(dev), gram)
    buf = rk.alloc_layer_buffers(p, qd.dtype, dev)
    rk.evict_layer(p, qd, kd, vd, gram, buf)
    torch.cuda.synchronize()
    P = w.seq_len - w.window
    out = dict(score=buf.score[..., :P].cpu().numpy(), ema=buf.ema[..., :P].cpu().numpy(),
               final=buf.final[..., :P].cpu().numpy(), aws_info=buf.aws_info.cpu().numpy(),
               aws_d=buf.aws_d.cpu().numpy(), idx=buf.idx.cpu().numpy(),
               k_out=buf.k_out.float().cpu().numpy(), v_out=buf.v_out.float().cpu().numpy(),
               gram=None if gram is None else gram.cpu().numpy())
    return out


def oracle_score(oracle, w, q, k, v, wo, heads=None, rows=None, causal=True, scale=None, group="mean",
                 dominant_exact=True, with_amax=False):
    """Oracle indicator with the per-element tolerance. Returns {g: (Ig [nq,P], tol [nq,P])}.
    group='max': the largest indicator of the group, with the largest of the heads' tolerances."""
    qn, kn, vn = (t.float().numpy() for t in (q, k, v))
    G, d, W = w.group, w.head_dim, w.window
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    fac = None if wo is None else oracle.gram_factor(wo.double().numpy().reshape(w.n_q_heads, d, -1))
    kappa = KAPPA_F32 if w.dtype == "f32" else KAPPA_BF16
    res = {}
    for g in (range(w.n_kv_heads) if heads is None else heads):
        fg = None if fac is None else fac[g * G:(g + 1) * G]
        Ig, I, A, ub = oracle.score_head(qn[g * G:(g + 1) * G], kn[g], vn[g], fg, W, scale, causal,
                                         rows=rows, aux=True, group=group)
        with np.errstate(divide="ignore", invalid="ignore"):
            second = np.minimum(np.where(I > 0, kappa * ub * ub / (2 * I), np.inf), np.sqrt(kappa) * ub)
        if dominant_exact:
            second = np.where(A > 0.5, 0.0, second)    # dominant token: leave-one-out form, no cancellation
        # FP32 flushes subnormals: a head's weight A/G below 2^-126 comes out of the exponential as
        # 0, and with it a contribution of up to 2^-126 sqrt(x)/(1-A) <= 2^-126 ub/A to the group's sum
        with np.errstate(divide="ignore", invalid="ignore"):
            flush = 2.0 ** -126 * np.where(A > 0, ub / A, 0.0)
        tol = ((RTOL * I + second).mean(axis=0) + flush.sum(axis=0) if group == "mean"
               else (RTOL * I + second + flush).max(axis=0))
        res[g] = (Ig, tol, A.max(axis=0)) if with_amax else (Ig, tol)
    return res


def attention_statistics(q, k, v, W, scale=None, causal=True):
    """What a fused attention kernel hands back for the window queries: output [Hq,W,d] and
    log-sum-exp [Hq,W] (natural log), FP32, computed in FP64 with the library softmax.  Input
    of restkv_score_from_attention in the tests."""
    Hq, _, d = q.shape
    Hkv, L, _ = k.shape
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    out = torch.empty((Hq, W, d), dtype=torch.float32)
    lse = torch.empty((Hq, W), dtype=torch.float32)
    for h in range(Hq):
        s = (q[h].double() @ k[h // G].double().T) * scale
        if causal:
            pos = torch.arange(L, device=s.device)[None, :] > (L - W + torch.arange(W, device=s.device))[:, None]
            s = s.masked_fill(pos, float("-inf"))
        lse[h] = torch.logsumexp(s, dim=-1).float()
        out[h] = (torch.softmax(s, dim=-1) @ v[h // G].double()).float()
    return out, lse


def assert_score_close(got, ref, tol, what=""):
    # The score array is FP32 and the kernels flush subnormal results to zero: a value below the
    # smallest normal FP32 number (2^-126) may come back as 0.
    bad = np.abs(got - ref) > tol + 2.0 ** -126
    if bad.any():
        j = np.argmax(np.where(bad, np.abs(got - ref) / (tol + 2.0 ** -126), 0.0))
        g_, r_, t_ = got.flat[j], ref.flat[j], tol.flat[j]
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements out of tolerance; worst at flat "
                             f"index {j}: got {g_!r} ref {r_!r} tol {t_!r}")


def check_selection(idx_gpu, ref_final, W, B, margin):
    """GPU index set against the oracle's final scores: the two top-(B-W) sets may differ only
    in elements whose oracle score lies within `margin` (relative) of the oracle threshold."""
    P = ref_final.shape[0]
    Bp = B - W
    assert np.array_equal(idx_gpu[Bp:], np.arange(P, P + W)), "window tokens must close the list"
    pre = idx_gpu[:Bp]
    assert np.all(np.diff(pre) > 0) and pre.min() >= 0 and pre.max() < P, "prefix indices ascending, in range"
    order = np.argsort(-ref_final, kind="stable")
    ref_set = set(order[:Bp].tolist())
    tau = ref_final[order[Bp - 1]]
    diff = ref_set.symmetric_difference(pre.tolist())
    for n in diff:
        assert abs(ref_final[n] - tau) <= margin * abs(tau) + 1e-300, \
            f"index {n}: oracle score {ref_final[n]} is not within {margin} of the threshold {tau}"
    return len(diff)


def topb_sum_bounds(ref_row, tol_row, bt):
    """Range of the index sum of the top-`bt` entries of a row whose every entry is only known
    to lie within ref +- tol.  An entry is surely selected when its lower bound lies above the
    (bt+1)-th largest upper bound, surely not when its upper bound lies below the bt-th largest
    lower bound; the rest of the selection may be any subset of the remaining entries.
    Returns (lowest possible sum, highest possible sum, number of undecided entries)."""
    P = ref_row.shape[0]
    if bt >= P:
        s = P * (P - 1) // 2
        return s, s, 0
    lo, hi = ref_row - tol_row, ref_row + tol_row
    tau_lo = np.partition(lo, P - bt)[P - bt]              # bt-th largest lower bound
    tau_hi = np.partition(hi, P - bt - 1)[P - bt - 1]      # (bt+1)-th largest upper bound
    sure = lo > tau_hi
    amb = np.nonzero((hi >= tau_lo) & ~sure)[0]            # ascending positions
    need = bt - int(sure.sum())
    assert 0 <= need <= amb.size, (need, amb.size)
    base = int(np.nonzero(sure)[0].sum())
    return base + int(amb[:need].sum()), base + int(amb[amb.size - need:].sum()), int(amb.size)


def drift_bounds(Ig, tol, budget, W):
    """Intervals that D_front and D_rear of a head must fall in when its raw scores are only
    known to +- tol (Sec. 3.3: mean index of the per-query top-B over each half of the window).
    Returns ((front lo, front hi), (rear lo, rear hi))."""
    P = Ig.shape[1]
    bt = min(budget, P)
    nf = W // 2
    fl = fh = rl = rh = 0
    for i in range(W):
        a, b, _ = topb_sum_bounds(Ig[i], tol[i], bt)
        if i < nf:
            fl, fh = fl + a, fh + b
        else:
            rl, rh = rl + a, rh + b
    den_f, den_r = float(bt) * max(nf, 1), float(bt) * (W - nf)
    return (fl / den_f, fh / den_f), (rl / den_r, rh / den_r)
