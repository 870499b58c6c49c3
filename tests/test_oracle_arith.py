"""Pins for the oracle's arithmetic (CPU only).

The paper prints no worked numeric example of an aggregation, so the oracle is
pinned by what mathematics fixes: closed forms of the momentum recurrence in
exact rationals on dyadic inputs (bit-exact), hand-derived IEEE-754 rounding
cases that separate the prescribed evaluation order from its plausible
variants, the library routine torch.optim.SGD as the W=1 special case, a
binary64 error bound, and the independence of blocks (paper, Section 2.2,
"Tensor-Based Model Structure").
"""
from fractions import Fraction as Fr

import numpy as np
import pytest
import torch

F = np.float32


def f32_exact(x: Fr) -> np.float32:
    y = np.float32(float(x))
    assert Fr(float(y)) == x, f"{x} is not a binary32 value"
    return y


def run_rounds(orc, p0, v0, grads_per_round, lr, mu, wd):
    p = np.array(p0, dtype=F).copy()
    v = np.array(v0, dtype=F).copy()
    hist = []
    for gs in grads_per_round:
        n2 = orc.aggregate_block([np.array(g, dtype=F) for g in gs], p, v, lr, mu, wd)
        hist.append((p.copy(), v.copy(), n2))
    return hist


# --- closed form 1: constant gradient, no decay -----------------------------
def test_constant_gradient_geometric_momentum(orc):
    """wd=0, one worker, constant g: v_k = g (1-mu^k)/(1-mu) and
    p_k = p_0 - lr * sum_{i<=k} v_i (textbook heavy-ball).  Dyadic values keep
    every intermediate exact, so binary32 must reproduce the rationals."""
    lr, mu = Fr(1, 2), Fr(1, 2)
    cases = [(Fr(5, 4), Fr(3, 16)), (Fr(-7, 8), Fr(-5, 16)), (Fr(0), Fr(1, 16))]
    K = 8
    p0 = [c[0] for c in cases]
    g = [c[1] for c in cases]
    hist = run_rounds(orc, [float(x) for x in p0], [0.0] * 3,
                      [[[float(x) for x in g]]] * K, float(lr), float(mu), 0.0)
    for k in range(1, K + 1):
        pk, vk, _ = hist[k - 1]
        for i in range(3):
            v_closed = g[i] * (1 - mu ** k) / (1 - mu)
            p_closed = p0[i] - lr * sum(g[i] * (1 - mu ** j) / (1 - mu) for j in range(1, k + 1))
            assert vk[i] == f32_exact(v_closed)
            assert pk[i] == f32_exact(p_closed)


# --- closed form 2: pure weight decay ---------------------------------------
def test_pure_weight_decay_is_geometric(orc):
    """g=0, mu=0: p_k = p_0 (1 - lr wd)^k; with lr=1/2, wd=1/4 the factor is 7/8."""
    lr, wd = Fr(1, 2), Fr(1, 4)
    p0 = [Fr(1), Fr(-3, 2), Fr(1, 64)]
    hist = run_rounds(orc, [float(x) for x in p0], [0.0] * 3, [[[0.0, 0.0, 0.0]]] * 7,
                      float(lr), 0.0, float(wd))
    for k in range(1, 8):
        pk, vk, n2 = hist[k - 1]
        assert n2 == 0.0
        for i in range(3):
            assert pk[i] == f32_exact(p0[i] * (1 - lr * wd) ** k)
            assert vk[i] == f32_exact(wd * p0[i] * (1 - lr * wd) ** (k - 1))


# --- closed form 3: zero gradient, momentum coasting -------------------------
def test_zero_gradient_momentum_coasts(orc):
    """wd=0.  With v=0 and g=0 the parameter is a fixed point.  After one
    non-zero round seeds v, zero gradients move p by lr*mu^k*v each round."""
    hist = run_rounds(orc, [0.75], [0.0], [[[0.0]]] * 3, 0.5, 0.5, 0.0)
    assert all(h[0][0] == F(0.75) and h[1][0] == 0.0 for h in hist)
    lr, mu, g = Fr(1, 4), Fr(1, 2), Fr(3, 8)
    hist = run_rounds(orc, [2.0], [0.0], [[[float(g)]]] + [[[0.0]]] * 6, float(lr), float(mu), 0.0)
    p = Fr(2) - lr * g
    assert hist[0][0][0] == f32_exact(p)
    for k in range(1, 7):
        p -= lr * mu ** k * g
        assert hist[k][0][0] == f32_exact(p)
        assert hist[k][1][0] == f32_exact(mu ** k * g)


# --- closed form 4: the full linear recurrence as a matrix power -------------
def test_full_recurrence_matrix_power(orc):
    """With constant g the state x=(p,v) obeys x' = A x + b with
    A = [[1 - lr wd, -lr mu], [wd, mu]], b = (-lr g, g):
    x_k = A^k x_0 + (I + A + ... + A^{k-1}) b.  Evaluated in exact rationals."""
    lr, mu, wd = Fr(1, 2), Fr(1, 2), Fr(1, 4)
    A = [[1 - lr * wd, -lr * mu], [wd, mu]]

    def matmul(X, Y):
        return [[sum(X[i][k] * Y[k][j] for k in range(2)) for j in range(2)] for i in range(2)]

    for p0, v0, g in [(Fr(3, 4), Fr(0), Fr(5, 16)), (Fr(-9, 16), Fr(0), Fr(7, 16))]:
        # two workers pushing g/2 each: their sum is exact
        hist = run_rounds(orc, [float(p0)], [float(v0)], [[[float(g / 2)], [float(g / 2)]]] * 3,
                          float(lr), float(mu), float(wd))
        Ak = [[Fr(1), Fr(0)], [Fr(0), Fr(1)]]
        S = [[Fr(0), Fr(0)], [Fr(0), Fr(0)]]
        b = [-lr * g, g]
        for k in range(1, 4):
            S = [[S[i][j] + Ak[i][j] for j in range(2)] for i in range(2)]
            Ak = matmul(Ak, A)
            pk = Ak[0][0] * p0 + Ak[0][1] * v0 + S[0][0] * b[0] + S[0][1] * b[1]
            vk = Ak[1][0] * p0 + Ak[1][1] * v0 + S[1][0] * b[0] + S[1][1] * b[1]
            assert hist[k - 1][0][0] == f32_exact(pk)
            assert hist[k - 1][1][0] == f32_exact(vk)
            assert hist[k - 1][2] == float(g * g)


# --- the aggregate is a sum, not a mean --------------------------------------
@pytest.mark.parametrize("W", [2, 3, 4, 8, 16, 32])
def test_identical_workers_give_W_times_g(orc, W):
    rng = np.random.default_rng(W)
    g = (rng.integers(-1023, 1024, size=257) * 2.0 ** -10).astype(F)  # 11 bits: W*g exact
    assert np.array_equal(orc.sum_block([g] * W), (W * g.astype(np.float64)).astype(F))
    # and through the update: W identical pushes == one push of W*g
    p = (rng.integers(-512, 512, size=257) * 2.0 ** -8).astype(F)
    pa, va = p.copy(), np.zeros_like(p)
    pb, vb = p.copy(), np.zeros_like(p)
    for _ in range(3):
        na = orc.aggregate_block([g] * W, pa, va, 0.1, 0.9, 1e-4)
        nb = orc.aggregate_block([(W * g.astype(np.float64)).astype(F)], pb, vb, 0.1, 0.9, 1e-4)
        assert na == nb
    assert np.array_equal(pa, pb) and np.array_equal(va, vb)


# --- summation order: strictly left to right over worker index ---------------
def test_sum_order_is_sequential_in_worker_index(orc):
    """binary32: 1 + 2^-24 ties to 1, so ((1 + e) + e) - 1 = 0 while
    ((-1 + e) + e) + 1 = 2^-23 and the pairwise (1+e) + (e-1) = 2^-24."""
    e = F(2.0 ** -24)
    fwd = [F(1), e, e, F(-1)]
    S = orc.sum_block([np.array([x], dtype=F) for x in fwd])
    assert S[0] == 0.0
    S = orc.sum_block([np.array([x], dtype=F) for x in fwd[::-1]])
    assert S[0] == F(2.0 ** -23)
    # the same through the fused update: lr=1, mu=0, wd=0, p=v=0  =>  v' = S, p' = -S
    for order, want in ((fwd, 0.0), (fwd[::-1], 2.0 ** -23)):
        p, v = np.zeros(1, F), np.zeros(1, F)
        n2 = orc.aggregate_block([np.array([x], dtype=F) for x in order], p, v, 1.0, 0.0, 0.0)
        assert v[0] == F(want) and p[0] == F(-want) and n2 == want * want


def test_sum_starts_from_worker_zero_value(orc):
    """Starting from g_0 (not from +0) keeps the sign of an all-negative-zero sum."""
    z = np.array([-0.0], dtype=F)
    assert np.signbit(orc.sum_block([z, z, z])[0])
    assert np.signbit(orc.sum_block([z])[0])


def test_sum_matches_independent_sequential_loop(orc):
    rng = np.random.default_rng(7)
    for W in (1, 2, 5, 8, 16):
        gs = [rng.normal(0, 1e-3, 1000).astype(F) for _ in range(W)]
        acc = gs[0].copy()
        for w in range(1, W):
            acc = (acc + gs[w]).astype(F)      # numpy: one rounded binary32 add per step
        assert np.array_equal(orc.sum_block(gs), acc)


# --- every operation separately rounded: three fused-multiply-add sites -------
def test_no_fused_multiply_add_anywhere(orc):
    """a = 1 + 2^-12: a*a = 1 + 2^-11 + 2^-24 ties to 1 + 2^-11 in binary32.
    A fused a*a - (1 + 2^-11) would give 2^-24; separate rounding gives 0."""
    a = F(1 + 2.0 ** -12)
    b = F(1 + 2.0 ** -11)
    # site 1: d = S + wd*p        (mu=0, lr=1)  -> v' = d
    p, v = np.array([a]), np.zeros(1, F)
    orc.aggregate_block([np.array([-b])], p, v, 1.0, 0.0, float(a))
    assert v[0] == 0.0 and p[0] == a
    # site 2: v' = mu*v + d       (wd=0, lr=1)
    p, v = np.zeros(1, F), np.array([a])
    orc.aggregate_block([np.array([-b])], p, v, 1.0, float(a), 0.0)
    assert v[0] == 0.0 and p[0] == 0.0
    # site 3: p' = p - lr*v'      (wd=0, mu=0, S = a)
    p, v = np.array([b]), np.zeros(1, F)
    orc.aggregate_block([np.array([a])], p, v, float(a), 0.0, 0.0)
    assert v[0] == a and p[0] == 0.0


# --- weight decay multiplies the parameter before the step -------------------
def test_weight_decay_uses_pre_update_parameter(orc):
    # lr=1, mu=0, g=0: v' = wd*p, p' = p - wd*p = p(1-wd); one round, exact
    p, v = np.array([8.0], dtype=F), np.zeros(1, F)
    orc.aggregate_block([np.zeros(1, F)], p, v, 1.0, 0.0, 0.25)
    assert v[0] == 2.0 and p[0] == 6.0


# --- library routine as the special case -------------------------------------
@pytest.mark.parametrize("W", [1, 4])
def test_against_torch_sgd(orc, W):
    rng = np.random.default_rng(11 + W)
    n, lr, mu, wd = 4096, 0.1, 0.9, 1e-4
    p0 = rng.normal(0, 0.05, n).astype(F)
    p, v = p0.copy(), np.zeros(n, F)
    tp = torch.nn.Parameter(torch.from_numpy(p0.copy()))
    opt = torch.optim.SGD([tp], lr=lr, momentum=mu, weight_decay=wd, dampening=0, nesterov=False)
    for _ in range(4):
        gs = [rng.normal(0, 1e-2, n).astype(F) for _ in range(W)]
        orc.aggregate_block(gs, p, v, lr, mu, wd)
        tp.grad = torch.from_numpy(np.sum(np.stack(gs).astype(np.float64), axis=0).astype(F))
        opt.step()
    tv = opt.state[tp]["momentum_buffer"].numpy()
    # the library may contract or reorder: allow a few units in the last place
    # of the largest magnitude involved (cancellation makes small outputs coarse)
    ulps = 8 * 2.0 ** -24
    np.testing.assert_allclose(p, tp.detach().numpy(), rtol=ulps, atol=ulps * np.abs(p).max())
    np.testing.assert_allclose(v, tv, rtol=ulps, atol=ulps * np.abs(v).max())


# --- binary64 error bound -----------------------------------------------------
def test_within_rounding_bound_of_exact(orc):
    rng = np.random.default_rng(3)
    n, W, lr, mu, wd = 2048, 8, 0.01, 0.9, 5e-4
    gs = [rng.normal(0, 1e-3, n).astype(F) for _ in range(W)]
    p0 = rng.normal(0, 0.05, n).astype(F)
    v0 = rng.normal(0, 0.01, n).astype(F)
    p, v = p0.copy(), v0.copy()
    n2 = orc.aggregate_block(gs, p, v, lr, mu, wd)
    G = np.stack(gs).astype(np.float64)
    lr_, mu_, wd_ = float(F(lr)), float(F(mu)), float(F(wd))
    S = G.sum(0)
    vx = mu_ * v0 + S + wd_ * p0
    px = p0 - lr_ * vx
    u = 2.0 ** -24
    mag_v = np.abs(G).sum(0) + abs(wd_) * np.abs(p0) + abs(mu_) * np.abs(v0)
    assert np.all(np.abs(v - vx) <= (W + 3) * u * mag_v)
    assert np.all(np.abs(p - px) <= 2 * u * (np.abs(p0) + lr_ * mag_v) + lr_ * (W + 3) * u * mag_v)
    S32 = orc.sum_block(gs).astype(np.float64)
    assert n2 == pytest.approx(float((S32 * S32).sum()), rel=1e-12)


# --- blocks are independent ---------------------------------------------------
def test_block_independence(orc):
    """Any block cap, any order of blocks inside a wave, any split of a wave
    leaves every parameter and momentum bit unchanged."""
    rng = np.random.default_rng(5)
    layers = (1000, 37, 4099, 64)
    W = 3
    grads = [[[rng.normal(0, 1e-2, n).astype(F) for n in layers] for _ in range(W)]
             for _ in range(3)]
    p0 = [rng.normal(0, 0.05, n).astype(F) for n in layers]

    def run(cap, shuffle_seed):
        job = orc.OracleJob(layers, W, 0.1, 0.9, 1e-4, cap_elems=cap)
        for l in range(len(layers)):
            job.p[l][:] = p0[l]
        for r in range(3):
            order = job.arrival()
            if shuffle_seed is not None:
                np.random.default_rng(shuffle_seed + r).shuffle(order)
            for b in order:
                layer, off, n = job.blocks[b]
                job.aggregate(b, [grads[r][w][layer][off:off + n] for w in range(W)])
        return job

    base = run(1 << 20, None)
    for cap, sh in [(1 << 20, 1), (1024, None), (1000, 2), (7, 3)]:
        other = run(cap, sh)
        for l in range(len(layers)):
            assert np.array_equal(base.p[l], other.p[l])
            assert np.array_equal(base.v[l], other.v[l])
        # telemetry of a tensor is the sum over its blocks
        for l in range(len(layers)):
            tot = sum(other.norm2[b] for b, blk in enumerate(other.blocks) if blk[0] == l)
            ref = sum(base.norm2[b] for b, blk in enumerate(base.blocks) if blk[0] == l)
            assert tot == pytest.approx(ref, rel=1e-12)


# --- brute force on the small configuration ----------------------------------
def test_small_config_three_rounds_vs_numpy(orc):
    """784-512-10 perceptron, W=2, three rounds with fresh gradients; numpy's
    float32 ufuncs round every elementwise op separately, as the oracle must."""
    import workloads as wl
    spec = wl.job_config("mlp")
    job = orc.OracleJob(spec.layer_numel, spec.W, spec.lr, spec.momentum, spec.wd)
    assert len(job.blocks) == 4
    lr, mu, wd = F(spec.lr), F(spec.momentum), F(spec.wd)
    ref_p, ref_v = [], []
    for l, n in enumerate(spec.layer_numel):
        t = torch.empty(n)
        wl.fill_normal_like(t, wl.stream_key(0, "param", 0, l), spec.param_std)
        job.p[l][:] = t.numpy()
        ref_p.append(t.numpy().copy())
        ref_v.append(np.zeros(n, F))
    for r in range(3):
        for b in job.arrival():
            layer, off, n = job.blocks[b]
            gs = []
            for w in range(spec.W):
                t = torch.empty(n)
                wl.fill_normal_like(t, wl.stream_key(0, "grad", 0, w, r, layer), spec.grad_std, start=off)
                gs.append(t.numpy())
            job.aggregate(b, gs)
            S = gs[0] + gs[1]
            d = S + wd * ref_p[layer]
            ref_v[layer] = mu * ref_v[layer] + d
            ref_p[layer] = ref_p[layer] - lr * ref_v[layer]
            assert ref_p[layer].dtype == F and ref_v[layer].dtype == F
    for l in range(4):
        assert np.array_equal(job.p[l], ref_p[l]) and np.array_equal(job.v[l], ref_v[l])
    assert job.round == [3, 3, 3, 3]
