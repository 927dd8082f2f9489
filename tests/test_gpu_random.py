"""Seeded random sweeps of the GPU path against the oracle: cases drawn from generators rather
than chosen by hand (planted keys far above the rest, wide groups and long windows, many KV
heads, the smoothing / selection stage with per-head budgets and variants).  Every case is a pure
function of its seed."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import assert_score_close, oracle_score, params_for, run_gpu_layer
from test_gpu_parity import _score_against_oracle_then_every_stage_exactly, _smooth_select_inputs
from test_gpu_parity import rk  # noqa: F401  (the module-scoped fixture that loads the library)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", range(16))
def test_random_planted_spikes(rk, oracle_mod, seed):
    """One to four keys 15 ... 500 nats above the rest at random places (spread over the prefix or
    packed into a few tiles, so that they supersede one another inside a key split)."""
    r = np.random.default_rng(50000 + seed)
    G = int(r.choice([1, 2, 4]))
    Hkv = int(r.choice([1, 2, 8]))
    d = int(r.choice([64, 128]))
    W = int(r.choice([4, 16, 64]))
    L = W + int(r.integers(100, 9000))
    B = W + int(r.integers(1, min(L - W, 500) + 1))
    w = workloads.small_case(Hq=G * Hkv, Hkv=Hkv, d=d, L=L, W=W, B=B, dtype=str(r.choice(["bf16", "bf16", "f32"])),
                             D=d, seed=51000 + seed)
    P = L - W
    spikes = [(int(r.integers(0, P)), float(r.choice([15.0, 40.0, 70.0, 100.0, 150.0, 300.0, 500.0])))
              for _ in range(int(r.integers(1, 5)))]
    if r.random() < 0.5:
        base = int(r.integers(0, max(1, P - 200)))
        spikes = [(min(P - 1, base + int(r.integers(0, 200))), g) for _, g in spikes]
    q, k, v = workloads.make_qkv(w)
    wo = workloads.make_wo(w)
    e = torch.zeros(d)
    e[3] = 1.0
    q = (q.float() + 8.0 * e).to(q.dtype)
    k = k.float().clone()
    for n, gap in spikes:
        k[:, n, :] = (gap * d ** 0.5 / 8.0) * e
    k = k.to(q.dtype)
    got = run_gpu_layer(rk, w, q, k, v, wo)
    assert np.all(np.isfinite(got["score"])) and np.all(got["score"] >= 0)
    for g, (Ig, tol) in oracle_score(oracle_mod, w, q, k, v, wo).items():
        assert_score_close(got["score"][g], Ig, tol, f"spikes {spikes} {w} head {g}")


@pytest.mark.parametrize("seed", range(12))
def test_random_wide_groups_long_windows(rk, oracle_mod, seed):
    """Groups up to 32 query heads, windows up to 128, extreme EMA factors, adaptive windows many
    positions wide (beta down to 0.5), kernel sizes up to 63; the same again through a token-major
    cache (bit-identical) and through the no-allocation selection."""
    r = np.random.default_rng(60000 + seed)
    G = int(r.choice([1, 4, 7, 16, 24, 32]))
    Hkv = 1 if G > 8 else int(r.integers(1, 3))
    d = int(r.choice([64, 128]))
    W = min(int(r.choice([2, 9, 33, 64, 100, 128])), 4096 // G)
    L = W + int(r.integers(1, 3000))
    B = W + int(r.integers(1, L - W + 1))
    w = workloads.small_case(Hq=G * Hkv, Hkv=Hkv, d=d, L=L, W=W, B=B, dtype=str(r.choice(["bf16", "bf16", "f32"])),
                             D=d, alpha=float(r.choice([0.001, 0.3, 0.999])), k=int(r.choice([1, 5, 63])),
                             beta=float(r.choice([0.5, 1.0, 3.0, 100.0])),
                             structure=str(r.choice(["plain", "sinks", "drift", "lowrank"])), seed=61000 + seed)
    _score_against_oracle_then_every_stage_exactly(rk, oracle_mod, w, f"wide case {seed} {w}")
    q, k, v = workloads.make_qkv(w)
    wo = workloads.make_wo(w)
    base = run_gpu_layer(rk, w, q, k, v, wo)
    Hq = w.n_q_heads
    qt, kt, vt = (t.permute(1, 0, 2).contiguous().cuda() for t in (q, k, v))
    p = params_for(rk, w, q_stride_h=d, q_stride_t=Hq * d, kv_stride_h=d, kv_stride_t=Hkv * d)
    gram = torch.empty((Hq, d, d), dtype=torch.float32, device="cuda")
    rk.restkv_prepare_wo(p, wo.cuda(), gram)
    buf = rk.alloc_layer_buffers(p, qt.dtype, "cuda")
    rk.evict_layer(p, qt, kt, vt, gram, buf)
    torch.cuda.synchronize()
    assert np.array_equal(buf.score[..., :w.prefix].cpu().numpy(), base["score"])
    assert np.array_equal(buf.idx.cpu().numpy(), base["idx"])
    idx2 = torch.empty_like(buf.idx)
    rk.restkv_select_static(p, buf.final, idx2)
    torch.cuda.synchronize()
    assert torch.equal(idx2, buf.idx)


@pytest.mark.parametrize("seed", range(4))
def test_random_many_kv_heads(rk, oracle_mod, seed):
    """16 to 300 KV heads (layers folded into the head dimension): one key split per head."""
    r = np.random.default_rng(70000 + seed)
    Hkv = int(r.choice([16, 40, 100, 256, 300]))
    G = int(r.choice([1, 2, 4]))
    d = int(r.choice([64, 128]))
    W = int(r.choice([4, 16, 64]))
    L = W + int(r.integers(1, 2200))
    B = W + int(r.integers(1, L - W + 1))
    w = workloads.small_case(Hq=G * Hkv, Hkv=Hkv, d=d, L=L, W=W, B=B, dtype=str(r.choice(["bf16", "bf16", "f32"])),
                             D=d, structure=str(r.choice(["plain", "sinks", "drift", "lowrank"])), seed=71000 + seed,
                             beta=float(r.choice([20.0, 2000.0])))
    _score_against_oracle_then_every_stage_exactly(rk, oracle_mod, w, f"many heads {seed} {w}")


@pytest.mark.parametrize("seed", range(32))
def test_random_smoothing_and_selection_stage(rk, oracle_mod, seed):
    """Same FP32 scores into both sides (log-normal, ties, constant, drifting mass), prefix lengths
    around the tile, chunk and sampling thresholds up to 140k, per-head budgets from one prefix
    token to everything, the temporal and spatial variants: index sums, window, EMA, final score
    and selection of every head, exactly where the stage is integer work."""
    r = np.random.default_rng(20000 + seed)
    Hkv = int(r.integers(1, 5))
    W = int(r.choice([1, 2, 3, 7, 16, 31, 64, 65, 100]))
    P = int(r.choice([1, 5, 63, 64, 65, 1000, 4095, 4096, 4097, 8191, 20000, 33000, 70000, 140001])) + int(r.integers(0, 3))
    kind = str(r.choice(["lognormal", "ties", "constant", "drifting"]))
    k = int(r.choice([1, 3, 5, 21, 63]))
    beta = float(r.choice([1.0, 8.0, 100.0, 2000.0]))
    alpha = float(np.float32(r.choice([0.01, 0.3, 0.9, 1.0])))
    L = P + W
    budgets = [W + int(r.integers(1, min(P, 5000) + 1)) for _ in range(Hkv)]
    if r.random() < 0.15:
        budgets[0] = L
    if r.random() < 0.15:
        budgets[-1] = W + 1
    tmode = str(r.choice(["ema", "mean", "inv_ema"]))
    pool = str(r.choice(["avg", "avg", "max"]))
    adaptive = bool(r.integers(0, 2)) and pool == "avg"
    var = {"ema": 0, "mean": rk.RESTKV_TEMPORAL_MEAN, "inv_ema": rk.RESTKV_TEMPORAL_INV_EMA}[tmode]
    var |= rk.RESTKV_POOL_MAX if pool == "max" else 0
    tag = f"case {seed}: Hkv {Hkv} W {W} P {P} {kind} k {k} beta {beta} alpha {alpha} budgets {budgets} {tmode} {pool} adaptive {adaptive}"
    s = _smooth_select_inputs(seed, Hkv, W, P, kind)
    p = rk.make_params(n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=64, seq_len=L, window=W, budget=max(budgets), dtype="bf16",
                       ema_alpha=alpha, base_window=k, beta=beta, adaptive=adaptive, variant=var)
    buf = rk.alloc_layer_buffers(p, torch.bfloat16, "cuda")
    buf.score[..., :P].copy_(torch.from_numpy(s))
    hb = torch.tensor(budgets, dtype=torch.int32, device="cuda")
    rk.restkv_smooth_b(p, buf.score, hb, buf.ema, buf.final, buf.aws_info, buf.aws_d, buf.workspace)
    rk.restkv_select_b(p, buf.final, hb, buf.idx, buf.workspace)
    torch.cuda.synchronize()
    ema, fin = buf.ema.cpu().numpy()[..., :P], buf.final.cpu().numpy()[..., :P]
    info, dd, idx = buf.aws_info.cpu().numpy(), buf.aws_d.cpu().numpy(), buf.idx.cpu().numpy()
    for g in range(Hkv):
        Bg = budgets[g]
        sm = oracle_mod.smooth_head(s[g], alpha, beta, k, adaptive, Bg, tmode, pool)
        if adaptive and W >= 2:
            assert dd[g, 0] == sm["d_front"] and dd[g, 1] == sm["d_rear"], tag
        assert tuple(info[g]) == (sm["w_s"], sm["gamma"]), tag
        np.testing.assert_allclose(ema[g], sm["ema"], rtol=1e-5, atol=1e-30, err_msg=tag)
        want = oracle_mod.box(ema[g].astype(np.float64), sm["w_s"], sm["gamma"]) if pool == "avg" else sm["final"]
        np.testing.assert_allclose(fin[g], want, rtol=2e-5, atol=1e-30, err_msg=tag)
        np.testing.assert_array_equal(idx[g, :Bg], oracle_mod.select(fin[g].astype(np.float64), W, Bg), err_msg=tag)
        assert np.all(idx[g, Bg:] == -1), tag


GUARD = 4096          # bytes of sentinel on either side of every output buffer


def _carved_buffers(rk, p, dtype):
    """The layer's output buffers and workspace as views into ONE byte pool, each between two
    guard zones filled with a sentinel; returns (LayerBuffers, pool, list of guard slices)."""
    Hkv, W, B, d = p.n_kv_heads, p.window, p.budget, p.head_dim
    ld = p.ld_score if p.ld_score else p.seq_len - p.window
    esz = 2 if dtype == torch.bfloat16 else 4
    specs = [("score", torch.float32, (Hkv, W, ld)), ("ema", torch.float32, (Hkv, ld)), ("final", torch.float32, (Hkv, ld)),
             ("aws_info", torch.int32, (Hkv, 2)), ("aws_d", torch.float64, (Hkv, 2)), ("idx", torch.int32, (Hkv, B)),
             ("k_out", dtype, (Hkv, B, d)), ("v_out", dtype, (Hkv, B, d)),
             ("workspace", torch.uint8, (max(int(rk.restkv_workspace_bytes(p)), 256),))]
    sizes = {torch.float32: 4, torch.int32: 4, torch.float64: 8, torch.uint8: 1, dtype: esz}
    off, place = GUARD, []
    for name, dt, shape in specs:
        nbytes = int(np.prod(shape)) * sizes[dt]
        place.append((name, dt, shape, off, nbytes))
        off = (off + nbytes + GUARD + 255) // 256 * 256
    pool = torch.full((off + GUARD,), 0xA5, dtype=torch.uint8, device="cuda")
    views, guards, prev_end = {}, [], 0
    for name, dt, shape, o, nbytes in place:
        views[name] = pool[o:o + nbytes].view(dt).view(shape)
        guards.append((prev_end, o))
        prev_end = o + nbytes
    guards.append((prev_end, pool.numel()))
    return rk.LayerBuffers(**views), pool, guards


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes_write_nothing_outside_their_buffers(rk, seed):
    """Every output buffer and the workspace sit between guard zones in one pool: after the whole
    path (every third case through the fused call, with a long enough prefix) no guard byte has
    changed."""
    r = np.random.default_rng(80000 + seed)
    fused = seed % 3 == 0
    G = int(r.choice([4, 8])) if fused else int(r.choice([1, 2, 3, 4, 8, 16]))
    Hkv = int(r.integers(1, 4)) if G <= 4 else 1
    d = int(r.choice([64, 128]))
    W = int(r.choice([1, 5, 16, 32, 64])) if not fused else int(r.choice([8, 32]))
    L = W + (int(r.integers(32768, 50000)) if fused else int(r.integers(1, 9000)))
    B = W + int(r.integers(1, min(L - W, 3000) + 1))
    dtype = "bf16" if fused else str(r.choice(["bf16", "f32"]))
    w = workloads.small_case(Hq=G * Hkv, Hkv=Hkv, d=d, L=L, W=W, B=B, dtype=dtype, D=d, beta=float(r.choice([8.0, 2000.0])),
                             k=int(r.choice([1, 5, 21])), structure=str(r.choice(["plain", "sinks", "drift", "lowrank"])),
                             seed=81000 + seed)
    q, k, v = workloads.make_qkv(w, 0, "cuda")
    wo = workloads.make_wo(w, 0, "cuda")
    p = params_for(rk, w)
    gram = torch.empty((w.n_q_heads, d, d), dtype=torch.float32, device="cuda")
    rk.restkv_prepare_wo(p, wo, gram)
    buf, pool, guards = _carved_buffers(rk, p, q.dtype)
    rk.evict_layer(p, q, k, v, gram, buf, fused=fused)
    torch.cuda.synchronize()
    for a, b in guards:
        assert bool((pool[a:b] == 0xA5).all()), f"guard bytes [{a}, {b}) changed: {w} fused={fused}"
    assert int(buf.idx.min()) >= 0 and int(buf.idx.max()) < L
