"""CPU oracle of the ReST-KV eviction path (test infrastructure, not the product).

Thin ctypes/numpy front end of ``restkv_oracle.c`` (plain C, double precision).
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the HIP library never does, and nothing here imports the HIP
binding.

Passages followed (paper sections / equations) are cited on each C function.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "restkv_oracle.c")
# RESTKV_ORACLE_SANITIZE=1: the oracle is built with clang under AddressSanitizer + UBSan into a
# library of its own (the process that loads it must preload the sanitizer runtime)
_SAN = os.environ.get("RESTKV_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "librestkv_oracle_san.so" if _SAN else "librestkv_oracle.so")
_CLANG = "/opt/rocm/lib/llvm/bin/clang"
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc, OpenMP); returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        if _SAN:
            cmd = [_CLANG, "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                   "-shared-libsan", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        else:
            cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
    return _lib


def num_threads() -> int:
    return int(_load().rk_oracle_num_threads())


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def attention(q, k, v, scale: float, causal: bool = True):
    """A [Hq,W,L], z [Hq,W,d] of the window queries (Eq. softmax)."""
    q, k, v = _f32(q), _f32(k), _f32(v)
    Hq, W, d = q.shape
    Hkv, L, _ = k.shape
    A = np.empty((Hq, W, L), np.float64)
    z = np.empty((Hq, W, d), np.float64)
    rc = _load().rk_oracle_attention(_p(q), _p(k), _p(v), Hq, Hkv, d, ctypes.c_int64(L),
                                     ctypes.c_int64(W), ctypes.c_double(scale), int(causal),
                                     _p(A), _p(z))
    _check(rc, "attention")
    return A, z


def _head_args(q, qpos, k, v, fac):
    q, k, v = _f32(q), _f32(k), _f32(v)
    G, nq, d = q.shape
    L = k.shape[0]
    assert k.shape == (L, d) and v.shape == (L, d)
    qp = None if qpos is None else np.ascontiguousarray(qpos, dtype=np.int64)
    if qp is not None:
        assert qp.shape == (nq,)
    if fac is None:
        f, r = None, d
    else:
        f = _f64(fac)
        assert f.shape[0] == G and f.shape[1] == d
        r = f.shape[2]
    return q, qp, k, v, f, r, G, nq, d, L


def indicator_loo(q, qpos, k, v, fac, P: int, scale: float) -> np.ndarray:
    """Eq. (ori) by brute force for one KV head: I [G,nq,P]."""
    q, qp, k, v, f, r, G, nq, d, L = _head_args(q, qpos, k, v, fac)
    I = np.empty((G, nq, P), np.float64)
    rc = _load().rk_oracle_indicator_loo(_p(q), _p(qp), _p(k), _p(v), _p(f), r, G, nq, d,
                                         ctypes.c_int64(L), ctypes.c_int64(P),
                                         ctypes.c_double(scale), _p(I))
    _check(rc, "indicator_loo")
    return I


def indicator_closed(q, qpos, k, v, fac, P: int, scale: float, aux: bool = False):
    """Eq. (rec_ei) for one KV head: I [G,nq,P] (and, with aux, A and the
    triangle bound A/(1-A)(||zW||+||v_nW||) per element)."""
    q, qp, k, v, f, r, G, nq, d, L = _head_args(q, qpos, k, v, fac)
    I = np.empty((G, nq, P), np.float64)
    aA = np.empty((G, nq, P), np.float64) if aux else None
    aU = np.empty((G, nq, P), np.float64) if aux else None
    rc = _load().rk_oracle_indicator_closed(_p(q), _p(qp), _p(k), _p(v), _p(f), r, G, nq, d,
                                            ctypes.c_int64(L), ctypes.c_int64(P),
                                            ctypes.c_double(scale), _p(I), _p(aA), _p(aU))
    _check(rc, "indicator_closed")
    return (I, aA, aU) if aux else I


def gram_factor(wo_heads) -> np.ndarray:
    """Per-head [d,d] factor F with F F^T = W_O^h W_O^hT, so ||x W_O^h|| = ||x F||.

    wo_heads [n,d,D] (z W_O orientation).  Gram product in float64, then the
    library Cholesky; a semi-definite Gram falls back to its eigen-decomposition.
    """
    w = _f64(wo_heads)
    out = np.empty((w.shape[0], w.shape[1], w.shape[1]), np.float64)
    for h in range(w.shape[0]):
        m = w[h] @ w[h].T
        try:
            out[h] = np.linalg.cholesky(m)
        except np.linalg.LinAlgError:
            ev, U = np.linalg.eigh(m)
            out[h] = U * np.sqrt(np.clip(ev, 0.0, None))
    return out


def group_mean(I) -> np.ndarray:
    I = _f64(I)
    G, nq, P = I.shape
    out = np.empty((nq, P), np.float64)
    _check(_load().rk_oracle_group_mean(_p(I), G, nq, ctypes.c_int64(P), _p(out)), "group_mean")
    return out


def ema(Ig, alpha: float) -> np.ndarray:
    Ig = _f64(Ig)
    W, P = Ig.shape
    out = np.empty((P,), np.float64)
    _check(_load().rk_oracle_ema(_p(Ig), W, ctypes.c_int64(P), ctypes.c_double(alpha), _p(out)), "ema")
    return out


def aws_stats(Ig, B: int):
    """(D_front, D_rear, index-sum front, index-sum rear) of one KV head."""
    Ig = _f64(Ig)
    W, P = Ig.shape
    df, dr = ctypes.c_double(), ctypes.c_double()
    sf, sr = ctypes.c_int64(), ctypes.c_int64()
    rc = _load().rk_oracle_aws_stats(_p(Ig), W, ctypes.c_int64(P), ctypes.c_int64(B),
                                     ctypes.byref(df), ctypes.byref(dr), ctypes.byref(sf),
                                     ctypes.byref(sr))
    _check(rc, "aws_stats")
    return df.value, dr.value, sf.value, sr.value


def aws_window(d_front: float, d_rear: float, beta: float, base_k: int, adaptive: bool = True):
    ws, gm = ctypes.c_int64(), ctypes.c_int64()
    rc = _load().rk_oracle_aws_window(ctypes.c_double(d_front), ctypes.c_double(d_rear),
                                      ctypes.c_double(beta), int(base_k), int(adaptive),
                                      ctypes.byref(ws), ctypes.byref(gm))
    _check(rc, "aws_window")
    return ws.value, gm.value


def box(ema_row, w_s: int, gamma: int) -> np.ndarray:
    e = _f64(ema_row)
    out = np.empty_like(e)
    rc = _load().rk_oracle_box(_p(e), ctypes.c_int64(e.shape[0]), ctypes.c_int64(w_s),
                               ctypes.c_int64(gamma), _p(out))
    _check(rc, "box")
    return out


def select(score, W: int, B: int) -> np.ndarray:
    s = _f64(score)
    idx = np.empty((B,), np.int64)
    rc = _load().rk_oracle_select(_p(s), ctypes.c_int64(s.shape[0]), ctypes.c_int64(W),
                                  ctypes.c_int64(B), _p(idx))
    _check(rc, "select")
    return idx


def gather(src, idx) -> np.ndarray:
    s = _f32(src)
    ix = np.ascontiguousarray(idx, dtype=np.int64)
    out = np.empty((ix.shape[0], s.shape[1]), np.float32)
    rc = _load().rk_oracle_gather(_p(s), _p(ix), ctypes.c_int64(ix.shape[0]), s.shape[1], _p(out))
    _check(rc, "gather")
    return out


def indicator_attention(q, qpos, k, v, P: int, scale: float, value_norm: bool = False) -> np.ndarray:
    """Ablation indicators (App., indicator table): A[n], or A[n] * ||v_n||_2; I [G,nq,P]."""
    q, qp, k, v, _, _, G, nq, d, L = _head_args(q, qpos, k, v, None)
    I = np.empty((G, nq, P), np.float64)
    rc = _load().rk_oracle_indicator_attention(_p(q), _p(qp), _p(k), _p(v), G, nq, d, ctypes.c_int64(L),
                                               ctypes.c_int64(P), ctypes.c_double(scale), int(value_norm), _p(I))
    _check(rc, "indicator_attention")
    return I


def group_max(I) -> np.ndarray:
    I = _f64(I)
    G, nq, P = I.shape
    out = np.empty((nq, P), np.float64)
    _check(_load().rk_oracle_group_max(_p(I), G, nq, ctypes.c_int64(P), _p(out)), "group_max")
    return out


TEMPORAL = {"ema": 0, "mean": 1, "inv_ema": 2}


def temporal(Ig, mode: str, alpha: float) -> np.ndarray:
    """Temporal smoothing over the window queries: 'ema' (Sec. 3.3), 'mean', 'inv_ema' (App.)."""
    Ig = _f64(Ig)
    W, P = Ig.shape
    out = np.empty((P,), np.float64)
    _check(_load().rk_oracle_temporal(_p(Ig), W, ctypes.c_int64(P), TEMPORAL[mode], ctypes.c_double(alpha),
                                      _p(out)), "temporal")
    return out


def pool_max(ema_row, w_s: int, gamma: int) -> np.ndarray:
    e = _f64(ema_row)
    out = np.empty_like(e)
    rc = _load().rk_oracle_pool_max(_p(e), ctypes.c_int64(e.shape[0]), ctypes.c_int64(w_s),
                                    ctypes.c_int64(gamma), _p(out))
    _check(rc, "pool_max")
    return out


def score_head(q_g, k_g, v_g, fac_g, W: int, scale: float, causal: bool = True,
               rows: Optional[Sequence[int]] = None, aux: bool = False,
               indicator: str = "reconstruction", group: str = "mean"):
    """Group-reduced indicator of one KV head: Ig [nq,P] for the window queries
    ``rows`` (default all W).  q_g [G,W,d]; k_g,v_g [L,d]; fac_g [G,d,r] or None.
    indicator: 'reconstruction' (Eq. rec_ei), 'attention', 'value_norm'; group: 'mean' or 'max'."""
    q_g = _f32(q_g)
    L = k_g.shape[0]
    P = L - W
    rows = list(range(W)) if rows is None else list(rows)
    qsel = q_g[:, rows, :]
    qpos = np.array([P + i if causal else -1 for i in rows], np.int64)
    reduce = group_mean if group == "mean" else group_max
    if indicator != "reconstruction":
        assert not aux
        return reduce(indicator_attention(qsel, qpos, k_g, v_g, P, scale, indicator == "value_norm"))
    res = indicator_closed(qsel, qpos, k_g, v_g, fac_g, P, scale, aux=aux)
    if aux:
        I, aA, aU = res
        return reduce(I), I, aA, aU
    return reduce(res)


def smooth_head(Ig, alpha: float, beta: float, base_k: int, adaptive: bool, B: int,
                temporal_mode: str = "ema", pool: str = "avg"):
    """Temporal smoothing + (adaptive) window for one KV head.
    Returns dict(ema, final, w_s, gamma, d_front, d_rear)."""
    Ig = _f64(Ig)
    W = Ig.shape[0]
    e = temporal(Ig, temporal_mode, alpha)
    if adaptive and W >= 2:
        df, dr, sf, sr = aws_stats(Ig, B)
        ws, gm = aws_window(df, dr, beta, base_k, True)
    else:
        df = dr = 0.0
        sf = sr = 0
        ws, gm = aws_window(0.0, 0.0, 1.0, base_k, False)
    fin = box(e, ws, gm) if pool == "avg" else pool_max(e, ws, gm)
    return dict(ema=e, final=fin, w_s=ws, gamma=gm, d_front=df, d_rear=dr, sum_front=sf, sum_rear=sr)


def run_layer(q, k, v, wo, *, window: int, budget: int, alpha: float, beta: float,
              base_k: int, adaptive: bool = True, scale: Optional[float] = None,
              causal: bool = True, indicator: str = "reconstruction", group: str = "mean",
              temporal_mode: str = "ema", pool: str = "avg"):
    """The whole path for one layer.  q [Hq,W,d], k,v [Hkv,L,d], wo [Hq*d,D] or None.

    Returns dict with score [Hkv,W,P], ema/final [Hkv,P], w_s/gamma [Hkv],
    d_front/d_rear [Hkv], idx [Hkv,B], k_out/v_out [Hkv,B,d].
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    Hq, W, d = q.shape
    Hkv, L, _ = k.shape
    assert W == window and Hq % Hkv == 0
    G = Hq // Hkv
    P = L - W
    scale = (1.0 / np.sqrt(d)) if scale is None else scale
    fac = None
    if wo is not None:
        fac = gram_factor(_f64(wo).reshape(Hq, d, -1))
    out = dict(score=np.empty((Hkv, W, P)), ema=np.empty((Hkv, P)), final=np.empty((Hkv, P)),
               w_s=np.empty(Hkv, np.int64), gamma=np.empty(Hkv, np.int64),
               d_front=np.empty(Hkv), d_rear=np.empty(Hkv),
               idx=np.empty((Hkv, budget), np.int64),
               k_out=np.empty((Hkv, budget, d), np.float32),
               v_out=np.empty((Hkv, budget, d), np.float32))
    for g in range(Hkv):
        fg = None if fac is None else fac[g * G:(g + 1) * G]
        Ig = score_head(q[g * G:(g + 1) * G], k[g], v[g], fg, W, scale, causal, indicator=indicator, group=group)
        sm = smooth_head(Ig, alpha, beta, base_k, adaptive, budget, temporal_mode, pool)
        idx = select(sm["final"], W, budget)
        out["score"][g] = Ig
        out["ema"][g] = sm["ema"]
        out["final"][g] = sm["final"]
        out["w_s"][g], out["gamma"][g] = sm["w_s"], sm["gamma"]
        out["d_front"][g], out["d_rear"][g] = sm["d_front"], sm["d_rear"]
        out["idx"][g] = idx
        out["k_out"][g] = gather(k[g], idx)
        out["v_out"][g] = gather(v[g], idx)
    return out
