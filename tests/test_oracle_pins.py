"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself or with the HIP path: brute
force against closed form (App. A identity), closed forms worked out in numpy
for degenerate inputs, invariants, library routines for the steps that reduce
to one, and hand-computed cases of the adaptive-window integers.
"""
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def rand_head(seed, G=2, nq=3, d=8, L=24, D=12, peaked=False):
    r = rng(seed)
    q = r.standard_normal((G, nq, d)).astype(np.float32)
    k = r.standard_normal((L, d)).astype(np.float32)
    v = r.standard_normal((L, d)).astype(np.float32)
    wo = (r.standard_normal((G, d, D)) / np.sqrt(D)).astype(np.float32)
    if peaked:
        k[3] *= 12.0
        q[:, :, :] = np.sign(k[3])[None, None, :] * np.abs(q)   # align queries with key 3
    return q, k, v, wo


# ---------------------------------------------------------------- attention
def test_attention_matches_library_softmax(oracle_mod):
    r = rng(0)
    Hq, Hkv, d, L, W = 4, 2, 16, 40, 5
    q = r.standard_normal((Hq, W, d)).astype(np.float32)
    k = r.standard_normal((Hkv, L, d)).astype(np.float32)
    v = r.standard_normal((Hkv, L, d)).astype(np.float32)
    scale = 1 / np.sqrt(d)
    for causal in (True, False):
        A, z = oracle_mod.attention(q, k, v, scale, causal)
        assert np.allclose(A.sum(-1), 1.0, atol=1e-13)
        for h in range(Hq):
            g = h // (Hq // Hkv)
            s = torch.tensor(q[h], dtype=torch.float64) @ torch.tensor(k[g], dtype=torch.float64).T * scale
            if causal:
                pos = torch.arange(L)[None, :] > (L - W + torch.arange(W))[:, None]
                s = s.masked_fill(pos, float("-inf"))
            Aref = torch.softmax(s, dim=-1)
            assert np.allclose(A[h], Aref.numpy(), atol=1e-13)
            assert np.allclose(z[h], (Aref @ torch.tensor(v[g], dtype=torch.float64)).numpy(), atol=1e-12)
        if causal:   # masked keys carry exactly zero weight
            for i in range(W):
                assert np.all(A[:, i, L - W + i + 1:] == 0.0)


# ---------------------------------------------------------------- indicator
@pytest.mark.parametrize("peaked", [False, True])
@pytest.mark.parametrize("causal", [False, True])
def test_closed_form_equals_leave_one_out(oracle_mod, peaked, causal):
    """App. A: Eq. (ori) and Eq. (rec_ei) are the same number."""
    q, k, v, wo = rand_head(1 + peaked, peaked=peaked)
    L, P = k.shape[0], k.shape[0] - 3
    qpos = np.array([P, P + 1, P + 2]) if causal else None
    scale = 1 / np.sqrt(q.shape[-1])
    I0 = oracle_mod.indicator_loo(q, qpos, k, v, wo, P, scale)
    I1, A, _ = oracle_mod.indicator_closed(q, qpos, k, v, wo, P, scale, aux=True)
    assert I0.shape == I1.shape == (2, 3, P)
    assert np.all(I1 >= 0)
    np.testing.assert_allclose(I1, I0, rtol=1e-9, atol=1e-14)
    if peaked:
        assert A.max() > 0.9          # exercises the dominant-token branch
    # ranks agree as well (the weaker statement, the one a user cares about).  The brute-force
    # value is a difference of two nearly equal outputs: for tokens whose weight is ~1e-13 of the
    # row's largest it is rounding noise, so ranks are compared above 1e-6 of each row's maximum.
    for r0, r1 in zip(I0.reshape(-1, P), I1.reshape(-1, P)):
        big = np.nonzero(r1 > 1e-6 * r1.max())[0]
        assert len(big) >= 1
        assert np.array_equal(big[np.argsort(-r0[big], kind="stable")],
                              big[np.argsort(-r1[big], kind="stable")])


def test_leave_one_out_is_independent_numpy_brute_force(oracle_mod):
    """Drop each token, renormalise, recompute the projected output - in numpy."""
    q, k, v, wo = rand_head(5, G=1, nq=2, d=6, L=10, D=7)
    scale = 0.37
    P = 10
    I0 = oracle_mod.indicator_loo(q, None, k, v, wo, P, scale)
    for i in range(2):
        s = (q[0, i].astype(np.float64) @ k.astype(np.float64).T) * scale
        full = (np.exp(s - s.max()) / np.exp(s - s.max()).sum()) @ v.astype(np.float64) @ wo[0].astype(np.float64)
        for n in range(P):
            keep = [m for m in range(10) if m != n]
            e = np.exp(s[keep] - s[keep].max())
            part = (e / e.sum()) @ v[keep].astype(np.float64) @ wo[0].astype(np.float64)
            assert abs(I0[0, i, n] - np.linalg.norm(full - part)) < 1e-12


def test_two_token_closed_form(oracle_mod):
    """L = 2: I[0] = A0 ||(v1 - v0) W_O||, I[1] = A1 ||(v0 - v1) W_O||."""
    r = rng(7)
    d, D = 5, 9
    q = r.standard_normal((1, 1, d)).astype(np.float32)
    k = r.standard_normal((2, d)).astype(np.float32)
    v = r.standard_normal((2, d)).astype(np.float32)
    wo = r.standard_normal((1, d, D)).astype(np.float32)
    scale = 0.8
    s = (q[0, 0].astype(np.float64) @ k.astype(np.float64).T) * scale
    A = np.exp(s) / np.exp(s).sum()
    dist = np.linalg.norm((v[1].astype(np.float64) - v[0]) @ wo[0].astype(np.float64))
    I = oracle_mod.indicator_closed(q, None, k, v, wo, 2, scale)
    np.testing.assert_allclose(I[0, 0], [A[0] * dist, A[1] * dist], rtol=1e-12)


def test_uniform_attention_closed_form(oracle_mod):
    """q = 0: A = 1/L, so I[n] = ||(mean(v) - v_n) W_O|| / (L - 1)."""
    r = rng(8)
    d, D, L = 6, 4, 17
    q = np.zeros((1, 2, d), np.float32)
    k = r.standard_normal((L, d)).astype(np.float32)
    v = r.standard_normal((L, d)).astype(np.float32)
    wo = r.standard_normal((1, d, D)).astype(np.float32)
    I = oracle_mod.indicator_closed(q, None, k, v, wo, L, 1.0)
    v64 = v.astype(np.float64)
    ref = np.linalg.norm((v64.mean(0)[None] - v64) @ wo[0].astype(np.float64), axis=1) / (L - 1)
    np.testing.assert_allclose(I[0, 0], ref, rtol=1e-12)
    np.testing.assert_allclose(I[0, 1], ref, rtol=1e-12)


def test_degenerate_inputs_and_homogeneity(oracle_mod):
    q, k, v, wo = rand_head(9)
    P, scale = k.shape[0], 0.5
    base = oracle_mod.indicator_closed(q, None, k, v, wo, P, scale)
    # all values equal: removing any token changes nothing
    vc = np.repeat(v[:1], v.shape[0], axis=0)
    assert np.abs(oracle_mod.indicator_closed(q, None, k, vc, wo, P, scale)).max() < 1e-12
    # zero projection
    assert np.all(oracle_mod.indicator_closed(q, None, k, v, wo * 0, P, scale) == 0)
    # degree-1 homogeneity in V and in W_O (exact powers of two keep float inputs exact)
    np.testing.assert_allclose(oracle_mod.indicator_closed(q, None, k, v * -4, wo, P, scale), 4 * base, rtol=1e-12)
    np.testing.assert_allclose(oracle_mod.indicator_closed(q, None, k, v, wo * 0.5, P, scale), 0.5 * base, rtol=1e-12)


def test_orthonormal_projection_equals_identity(oracle_mod):
    q, k, v, _ = rand_head(10, d=8, D=12)
    Q, _ = np.linalg.qr(rng(11).standard_normal((12, 8)))     # [12,8], orthonormal columns
    wo = np.stack([Q.T, Q.T]).astype(np.float64)               # [G,d,D] with W W^T = I
    P = k.shape[0]
    a = oracle_mod.indicator_closed(q, None, k, v, wo, P, 0.4)
    b = oracle_mod.indicator_closed(q, None, k, v, None, P, 0.4)
    np.testing.assert_allclose(a, b, rtol=1e-10)


def test_gram_factor_preserves_norms(oracle_mod):
    """||x W_O|| only depends on W_O W_O^T: the Cholesky factor gives the same indicator."""
    q, k, v, wo = rand_head(12, d=8, D=20)
    P = k.shape[0] - 3
    qpos = np.array([P, P + 1, P + 2])
    fac = oracle_mod.gram_factor(wo)
    for h in range(wo.shape[0]):
        np.testing.assert_allclose(fac[h] @ fac[h].T, wo[h].astype(np.float64) @ wo[h].T, atol=1e-12)
    a = oracle_mod.indicator_closed(q, qpos, k, v, wo, P, 0.3)
    b = oracle_mod.indicator_closed(q, qpos, k, v, fac, P, 0.3)
    np.testing.assert_allclose(a, b, rtol=1e-9)


def test_masked_key_scores_zero_and_far_key_scores_nearly_zero(oracle_mod):
    q, k, v, wo = rand_head(13)
    L = k.shape[0]
    qpos = np.array([L - 6, L - 5, L - 4])
    I = oracle_mod.indicator_closed(q, qpos, k, v, wo, L, 0.35)
    for i, p in enumerate(qpos):
        assert np.all(I[:, i, p + 1:] == 0.0)       # not yet visible -> weight 0 -> score 0
        assert np.all(I[:, i, :p + 1] > 0.0)
    # a key whose logit is ~ -1e3 has weight exp(-1e3) = 0
    k2 = k.copy()
    k2[2] = -1e3 * q[0, 0] / np.dot(q[0, 0], q[0, 0])
    I2 = oracle_mod.indicator_closed(q[:1, :1], None, k2, v, wo[:1], L, 1.0)
    assert I2[0, 0, 2] == 0.0


def test_indicator_vectorised_numpy_large_random(oracle_mod):
    """Second implementation (numpy, vectorised) of Eq. (rec_ei) on a random case with a
    non-square projection: guards operand order / transposition in the C loops."""
    q, k, v, wo = rand_head(14, G=2, nq=4, d=16, L=200, D=24)
    P, scale = 190, 0.25
    qpos = np.arange(P + 2, P + 6)
    I = oracle_mod.indicator_closed(q, qpos, k, v, wo, P, scale)
    k64, v64 = k.astype(np.float64), v.astype(np.float64)
    for h in range(2):
        for i, p in enumerate(qpos):
            s = (q[h, i].astype(np.float64) @ k64[:p + 1].T) * scale
            A = np.exp(s - s.max())
            A /= A.sum()
            mha = (A @ v64[:p + 1]) @ wo[h].astype(np.float64)
            ref = A[:P] / (1 - A[:P]) * np.linalg.norm(mha[None] - v64[:P] @ wo[h].astype(np.float64), axis=1)
            np.testing.assert_allclose(I[h, i], ref, rtol=1e-9)


def test_group_mean(oracle_mod):
    I = rng(15).random((3, 4, 11))
    np.testing.assert_allclose(oracle_mod.group_mean(I), I.mean(0), rtol=1e-15)


# ---------------------------------------------------------------- EMA
def test_ema_limits_and_closed_form_weights(oracle_mod):
    r = rng(20)
    W, P = 7, 13
    Ig = r.random((W, P))
    np.testing.assert_array_equal(oracle_mod.ema(Ig, 1.0), Ig[-1])    # decay 0 -> last query
    np.testing.assert_array_equal(oracle_mod.ema(Ig, 0.0), Ig[0])     # alpha 0 -> first query
    for alpha in (0.1, 0.3, 0.9):
        w = np.array([(1 - alpha) ** (W - 1)] + [alpha * (1 - alpha) ** (W - 1 - i) for i in range(1, W)])
        assert abs(w.sum() - 1) < 1e-14
        np.testing.assert_allclose(oracle_mod.ema(Ig, alpha), w @ Ig, rtol=1e-13)
        const = np.full((W, P), 2.5)
        np.testing.assert_allclose(oracle_mod.ema(const, alpha), 2.5, rtol=1e-14)
    np.testing.assert_array_equal(oracle_mod.ema(Ig[:1], 0.3), Ig[0])  # single query


# ---------------------------------------------------------------- adaptive window
def test_aws_stats_planted_spikes(oracle_mod):
    """Front queries spike at positions F, rear queries at positions R: D is their mean."""
    W, P, B = 6, 500, 4
    F = np.array([10, 20, 30, 40])
    R = np.array([310, 320, 330, 348])
    Ig = rng(21).random((W, P)) * 0.01
    Ig[:3, F] = 5.0 + np.arange(4)
    Ig[3:, R] = 9.0
    df, dr, sf, sr = oracle_mod.aws_stats(Ig, B)
    assert df == F.mean() and dr == R.mean()
    assert sf == 3 * F.sum() and sr == 3 * R.sum()
    # paper's normalisation 2 / (B * S_w) for even windows
    assert df == 2.0 / (B * W) * sf


def test_aws_stats_odd_window_ties_and_short_prefix(oracle_mod):
    # odd W: front = first floor(W/2) queries
    Ig = np.zeros((5, 50))
    Ig[:2, 7] = 1.0
    Ig[2:, 40] = 1.0
    df, dr, _, _ = oracle_mod.aws_stats(Ig, 1)
    assert (df, dr) == (7.0, 40.0)
    # all-equal scores: ties resolve to the lowest indices 0..B-1
    df, dr, _, _ = oracle_mod.aws_stats(np.ones((4, 30)), 6)
    assert df == dr == 2.5
    # budget larger than the prefix: every index is taken
    df, dr, _, _ = oracle_mod.aws_stats(rng(22).random((4, 9)), 100)
    assert df == dr == 4.0


def test_aws_window_hand_computed_cases(oracle_mod):
    n = 0
    with open(os.path.join(GOLDEN, "aws_window_cases.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            df, dr, beta, k, ws, gm = line.split()
            got = oracle_mod.aws_window(float(df), float(dr), float(beta), int(k), True)
            assert got == (int(ws), int(gm)), line
            n += 1
    assert n >= 10
    assert oracle_mod.aws_window(1000.0, 9000.0, 2000.0, 5, False) == (5, 0)


def test_box_identity_library_pool_shift_and_edges(oracle_mod):
    r = rng(23)
    e = r.random(64)
    np.testing.assert_array_equal(oracle_mod.box(e, 1, 0), e)                    # window 1 = identity
    for ws in (3, 5, 21):
        ref = torch.nn.functional.avg_pool1d(torch.tensor(e)[None, None], ws, 1, ws // 2,
                                             count_include_pad=True)[0, 0].numpy()
        np.testing.assert_allclose(oracle_mod.box(e, ws, 0), ref, rtol=1e-13)
        for gm in (-3, -1, 1, 2, 7):
            got = oracle_mod.box(e, ws, gm)
            pad = np.concatenate([np.zeros(40), e, np.zeros(40)])
            want = np.array([pad[40 + n + gm - ws // 2: 40 + n + gm + ws // 2 + 1].sum() / ws for n in range(64)])
            np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    c = oracle_mod.box(np.full(20, 3.0), 5, 0)
    np.testing.assert_allclose(c[2:-2], 3.0)
    np.testing.assert_allclose(c[[0, 1, -2, -1]], [3 * 3 / 5, 3 * 4 / 5, 3 * 4 / 5, 3 * 3 / 5])


# ---------------------------------------------------------------- select / gather
def test_select_is_stable_argsort_with_window_appended(oracle_mod):
    r = rng(24)
    P, W, B = 200, 8, 40
    s = r.integers(0, 12, P).astype(np.float64)          # many ties
    idx = oracle_mod.select(s, W, B)
    want = np.sort(np.argsort(-s, kind="stable")[:B - W])
    np.testing.assert_array_equal(idx[:B - W], want)
    np.testing.assert_array_equal(idx[B - W:], np.arange(P, P + W))
    assert len(set(idx.tolist())) == B
    # budget equal to the whole cache keeps everything
    np.testing.assert_array_equal(oracle_mod.select(s, W, P + W), np.arange(P + W))


def test_gather_is_fancy_indexing(oracle_mod):
    src = rng(25).standard_normal((30, 6)).astype(np.float32)
    idx = np.array([29, 0, 3, 3, 17])
    np.testing.assert_array_equal(oracle_mod.gather(src, idx), src[idx])


# ---------------------------------------------------------------- whole layer
def test_run_layer_invariants_tiny(oracle_mod):
    import workloads
    w = workloads.small_case(Hq=4, Hkv=2, d=16, L=160, W=6, B=24, D=20, k=1)
    q, k, v = workloads.make_qkv(w)
    wo = workloads.make_wo(w)
    out = oracle_mod.run_layer(q.numpy(), k.numpy(), v.numpy(), wo.numpy(), window=6, budget=24,
                               alpha=1.0, beta=2000.0, base_k=1, adaptive=False)
    P = 160 - 6
    assert out["score"].shape == (2, 6, P) and np.all(out["score"] >= 0)
    np.testing.assert_array_equal(out["ema"], out["score"][:, -1, :])        # decay 0
    np.testing.assert_array_equal(out["final"], out["ema"])                  # window 1
    for g in range(2):
        idx = out["idx"][g]
        assert np.all(np.diff(idx) > 0) and np.array_equal(idx[-6:], np.arange(P, 160))
        np.testing.assert_array_equal(out["k_out"][g], k.numpy()[g][idx])
        np.testing.assert_array_equal(out["v_out"][g], v.numpy()[g][idx])


def test_smooth_head_planted_drift_hand_derived_window(oracle_mod):
    """The composition EMA -> D_front/D_rear -> W_s, gamma -> Eq. (final_ei) on a planted drift.
    Front queries (0, 1) have their top-3 at positions 10, 20, 30 (D_front = 20), rear queries
    (2, 3) at 110, 120, 130 (D_rear = 120): x = -100.  With beta = 40: floor(2.5) = 2, so
    W_s = k + 4 = 7 for k = 3, and gamma = floor(-2.5) + 1 = -2 (Sec. 3.3).  The final score is
    then the mean of the EMA over positions n - 5 .. n + 1, written out here directly."""
    W, P, B, alpha = 4, 200, 3, 0.3
    Ig = rng(31).random((W, P)) * 0.01
    Ig[:2, [10, 20, 30]] = [[3.0, 2.0, 1.0], [1.0, 2.0, 3.0]]
    Ig[2:, [110, 120, 130]] = [[5.0, 5.0, 5.0], [4.0, 6.0, 5.0]]
    sm = oracle_mod.smooth_head(Ig, alpha, 40.0, 3, True, B)
    assert (sm["d_front"], sm["d_rear"]) == (20.0, 120.0)
    assert (sm["w_s"], sm["gamma"]) == (7, -2)
    wts = np.array([(1 - alpha) ** 3, alpha * (1 - alpha) ** 2, alpha * (1 - alpha), alpha])
    e = wts @ Ig
    np.testing.assert_allclose(sm["ema"], e, rtol=1e-13)
    pad = np.concatenate([np.zeros(8), e, np.zeros(8)])
    want = np.array([pad[8 + n - 5: 8 + n + 2].sum() / 7.0 for n in range(P)])
    np.testing.assert_allclose(sm["final"], want, rtol=1e-12, atol=1e-16)
    # without the adaptive window: kernel k, no shift
    sm0 = oracle_mod.smooth_head(Ig, alpha, 40.0, 3, False, B)
    assert (sm0["w_s"], sm0["gamma"]) == (3, 0)
    want0 = np.array([pad[8 + n - 1: 8 + n + 2].sum() / 3.0 for n in range(P)])
    np.testing.assert_allclose(sm0["final"], want0, rtol=1e-12, atol=1e-16)


def test_run_layer_adaptive_composition(oracle_mod):
    """run_layer with the adaptive window on: every stage's output is what the next stage's
    definition gives when applied to it with independent numpy code."""
    import workloads
    w = workloads.small_case(Hq=4, Hkv=2, d=16, L=400, W=8, B=40, D=20, k=3, beta=7.0, alpha=0.3)
    q, k, v = workloads.make_qkv(w)
    wo = workloads.make_wo(w)
    out = oracle_mod.run_layer(q.numpy(), k.numpy(), v.numpy(), wo.numpy(), window=8, budget=40,
                               alpha=0.3, beta=7.0, base_k=3, adaptive=True)
    P, W, B = 392, 8, 40
    wts = np.array([0.7 ** 7] + [0.3 * 0.7 ** (7 - i) for i in range(1, 8)])
    seen = set()
    for g in range(2):
        s = out["score"][g]
        np.testing.assert_allclose(out["ema"][g], wts @ s, rtol=1e-12)
        top = np.argsort(-s, axis=1, kind="stable")[:, :B]
        df, dr = top[:4].mean(), top[4:].mean()
        assert abs(out["d_front"][g] - df) < 1e-9 and abs(out["d_rear"][g] - dr) < 1e-9
        x = df - dr
        ws = 3 + 2 * int(np.floor(abs(x) / 7.0))
        gm = int(np.floor(x / 7.0)) + (0 if x > 0 else 1)
        assert (out["w_s"][g], out["gamma"][g]) == (ws, gm)
        seen.add((ws, gm))
        e = out["ema"][g]
        pad = np.concatenate([np.zeros(P), e, np.zeros(P)])
        want = np.array([pad[P + n + gm - ws // 2: P + n + gm + ws // 2 + 1].sum() / ws for n in range(P)])
        np.testing.assert_allclose(out["final"][g], want, rtol=1e-12, atol=1e-18)
        keep = np.sort(np.argsort(-out["final"][g], kind="stable")[:B - W])
        np.testing.assert_array_equal(out["idx"][g], np.concatenate([keep, np.arange(P, P + W)]))
        np.testing.assert_array_equal(out["k_out"][g], k.numpy()[g][out["idx"][g]])
    assert any(ws > 3 or gm != 0 for ws, gm in seen), seen       # the window did adapt


# ---------------------------------------------------------------- ablation variants
def test_attention_and_value_norm_indicators(oracle_mod):
    """App. (indicator table): A[n] and A[n] * ||v_n||_2, against the library softmax."""
    q, k, v, _ = rand_head(40, G=3, nq=4, d=12, L=60)
    P, scale = 50, 0.31
    qpos = np.array([P + 1, P + 3, P + 6, -1])
    Ia = oracle_mod.indicator_attention(q, qpos, k, v, P, scale)
    Iv = oracle_mod.indicator_attention(q, qpos, k, v, P, scale, value_norm=True)
    vn = np.linalg.norm(v.astype(np.float64), axis=1)
    for h in range(3):
        for i, p in enumerate(qpos):
            nvis = 60 if p < 0 else p + 1
            s = torch.tensor(q[h, i], dtype=torch.float64) @ torch.tensor(k[:nvis], dtype=torch.float64).T * scale
            A = torch.softmax(s, dim=-1).numpy()
            np.testing.assert_allclose(Ia[h, i], A[:P], rtol=1e-12)
            np.testing.assert_allclose(Iv[h, i], A[:P] * vn[:P], rtol=1e-12)
    # a query that sees fewer keys than the prefix gives zero weight to the rest
    I2 = oracle_mod.indicator_attention(q[:, :1], np.array([20]), k, v, P, scale)
    assert np.all(I2[:, 0, 21:] == 0) and abs(I2[0, 0, :21].sum() - 1) < 1e-12


def test_group_max_and_score_head_variants(oracle_mod):
    I = rng(41).random((4, 3, 17))
    np.testing.assert_array_equal(oracle_mod.group_max(I), I.max(0))
    q, k, v, wo = rand_head(42, G=2, nq=5, d=8, L=40)
    W, scale = 5, 0.4
    P = 35
    a = oracle_mod.score_head(q, k, v, None, W, scale, indicator="attention", group="max")
    Aall = oracle_mod.indicator_attention(q, np.arange(P, P + W), k, v, P, scale)
    np.testing.assert_array_equal(a, Aall.max(0))
    b = oracle_mod.score_head(q, k, v, wo, W, scale, group="max")
    Ic = oracle_mod.indicator_closed(q, np.arange(P, P + W), k, v, wo, P, scale)
    np.testing.assert_array_equal(b, Ic.max(0))


def test_temporal_mean_and_inverse_ema(oracle_mod):
    r = rng(43)
    W, P = 6, 11
    Ig = r.random((W, P))
    np.testing.assert_array_equal(oracle_mod.temporal(Ig, "ema", 0.3), oracle_mod.ema(Ig, 0.3))
    np.testing.assert_allclose(oracle_mod.temporal(Ig, "mean", 0.3), Ig.mean(0), rtol=1e-14)
    for alpha in (0.1, 0.3, 0.8):
        # closed-form weights of the recursion run newest -> oldest: the newest query keeps
        # (1-alpha)^(W-1), query i < W-1 gets alpha (1-alpha)^i
        w = np.array([alpha * (1 - alpha) ** i for i in range(W - 1)] + [(1 - alpha) ** (W - 1)])
        assert abs(w.sum() - 1) < 1e-14
        np.testing.assert_allclose(oracle_mod.temporal(Ig, "inv_ema", alpha), w @ Ig, rtol=1e-13)
    np.testing.assert_array_equal(oracle_mod.temporal(Ig, "inv_ema", 1.0), Ig[0])     # all weight on the oldest
    np.testing.assert_array_equal(oracle_mod.temporal(Ig, "inv_ema", 0.0), Ig[-1])
    np.testing.assert_array_equal(oracle_mod.temporal(Ig[:1], "mean", 0.3), Ig[0])


def test_pool_max_against_library_pool_and_shifts(oracle_mod):
    r = rng(44)
    e = r.random(50)
    np.testing.assert_array_equal(oracle_mod.pool_max(e, 1, 0), e)
    for ws in (3, 5, 21):
        ref = torch.nn.functional.max_pool1d(torch.tensor(e)[None, None], ws, 1, ws // 2)[0, 0].numpy()
        np.testing.assert_array_equal(oracle_mod.pool_max(e, ws, 0), ref)
    got = oracle_mod.pool_max(e, 3, 4)                 # window n+3 .. n+5
    want = np.array([e[n + 3:n + 6].max() if n + 3 < 50 else 0.0 for n in range(50)])
    np.testing.assert_array_equal(got, want)
    got = oracle_mod.pool_max(e, 5, -60)               # entirely outside the prefix
    assert np.all(got == 0.0)


def test_run_layer_variant_composition(oracle_mod):
    import workloads
    w = workloads.small_case(Hq=4, Hkv=2, d=16, L=200, W=6, B=30, D=20, k=3)
    q, k, v = workloads.make_qkv(w)
    out = oracle_mod.run_layer(q.numpy(), k.numpy(), v.numpy(), None, window=6, budget=30, alpha=0.3, beta=2000.0,
                               base_k=3, adaptive=False, indicator="value_norm", group="max",
                               temporal_mode="mean", pool="max")
    P = 194
    vn = np.linalg.norm(v.numpy().astype(np.float64), axis=2)
    for g in range(2):
        A, _ = oracle_mod.attention(q.numpy()[2 * g:2 * g + 2], k.numpy()[g:g + 1], v.numpy()[g:g + 1], 0.25, True)
        want = (A[:, :, :P] * vn[g][None, None, :P]).max(0)
        np.testing.assert_allclose(out["score"][g], want, rtol=1e-12)
        np.testing.assert_allclose(out["ema"][g], want.mean(0), rtol=1e-12)
        e = out["ema"][g]
        pad = np.concatenate([[0.0], e, [0.0]])
        np.testing.assert_array_equal(out["final"][g], np.maximum(np.maximum(pad[:-2], pad[1:-1]), pad[2:]))
