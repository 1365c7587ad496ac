"""Pins for the CPU oracle: closed forms, library routines, hand-computed cases and
the schedule constants the paper prints.  None of these re-types the oracle's own
expression sequence; each is a different route to the same number."""
import os

import numpy as np
import pytest
import torch

from oracle import pier_oracle as O

HP = dict(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def f32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def tol(ref):
    """The parity bar: 1e-6 * max(1, |x|)."""
    return 1e-6 * np.maximum(1.0, np.abs(ref))


# ---------------------------------------------------------------- exact symmetries
#
# IEEE arithmetic rounds symmetrically in sign and is exact under scaling by a power of two
# (away from overflow and subnormals), so some symmetries of the update rules must hold bit for
# bit, whatever the operation order: a wrong sign, a term that does not scale, a constant added
# where a product belongs breaks them.

def test_adamw_is_odd_in_theta_m_g_bit_for_bit():
    rng = np.random.default_rng(21)
    n = 4096
    p0, m0 = f32(rng.normal(0, 0.02, n)), f32(rng.normal(0, 1e-3, n))
    v0, g0 = f32(rng.uniform(0, 1e-6, n)), f32(rng.normal(0, 1e-3, n))
    a = [p0.copy(), m0.copy(), v0.copy()]
    b = [-p0, -m0, v0.copy()]
    for step in (1, 2, 7):
        O.adamw(*a, g0, step=step, **HP)
        O.adamw(*b, f32(-g0), step=step, **HP)
        assert np.array_equal(a[0], -b[0]) and np.array_equal(a[1], -b[1]) and np.array_equal(a[2], b[2])
    assert not np.array_equal(a[0], p0)


def test_outer_is_odd_and_scales_by_powers_of_two_bit_for_bit():
    rng = np.random.default_rng(22)
    n, G = 2048, 4
    a0, M0 = f32(rng.normal(0, 0.02, n)), f32(rng.normal(0, 1e-3, n))
    th0 = [f32(a0 + rng.normal(0, 1e-3, n)) for _ in range(G)]
    for phase in (1, 0):
        ref = [t.copy() for t in th0], a0.copy(), M0.copy()
        O.outer(*ref, mu=0.95, lr=1.1, phase=phase)
        for scale in (-1.0, 4.0, -0.125):
            sc = [f32(scale * t) for t in th0], f32(scale * a0), f32(scale * M0)
            O.outer(*sc, mu=0.95, lr=1.1, phase=phase)
            assert np.array_equal(sc[1], f32(scale * ref[1])) and np.array_equal(sc[2], f32(scale * ref[2]))
            for g in range(G):
                assert np.array_equal(sc[0][g], f32(scale * ref[0][g]))
    # and the order of the groups matters only through rounding: a permutation stays within tolerance
    ref = [t.copy() for t in th0], a0.copy(), M0.copy()
    O.outer(*ref, mu=0.95, lr=1.1, phase=1)
    perm = [th0[2].copy(), th0[0].copy(), th0[3].copy(), th0[1].copy()], a0.copy(), M0.copy()
    O.outer(*perm, mu=0.95, lr=1.1, phase=1)
    assert np.all(np.abs(perm[1] - ref[1]) <= tol(ref[1]))


def test_clip_coefficient_scales_inversely_with_the_gradient():
    rng = np.random.default_rng(23)
    g = f32(rng.normal(0, 1e-2, 10_000))
    s1, s4 = O.sumsq(g), O.sumsq(f32(4.0 * g))
    assert s4 == 16.0 * s1                                   # exact: every term scales by 2^4
    c1, c4 = O.clip_coef(s1, 0.5), O.clip_coef(s4, 0.5)
    assert c1 < 1.0 and abs(c4 * 4.0 / c1 - 1.0) < 2e-6      # the 1e-6 in the denominator is not scaled
    assert O.clip_coef(s1, 1e3) == 1.0


# ---------------------------------------------------------------- inner AdamW

def test_adamw_first_step_closed_form_hand_case():
    # m0 = v0 = 0  =>  mhat = g, vhat = g^2  =>  theta1 = theta0 - lr (g/(|g|+eps) + wd theta0)
    th0 = np.array([0.5, -0.25, 0.0, 2.0])
    g = np.array([1e-3, -2e-3, 4e-4, 0.0])
    lr, eps, wd = HP["lr"], HP["eps"], HP["weight_decay"]
    want = th0 - lr * (g / (np.abs(g) + eps) + wd * th0)
    # by hand: 0.5 - 3e-4*(~1 + 0.05), -0.25 - 3e-4*(~-1 - 0.025), -3e-4*~1, 2 - 3e-4*0.2
    np.testing.assert_allclose(want, [0.4996850030, -0.2496925015, -2.999925e-4, 1.99994],
                               rtol=0, atol=1e-9)
    p, m, v = f32(th0), f32(np.zeros(4)), f32(np.zeros(4))
    O.adamw(p, m, v, f32(g), step=1, **HP)
    np.testing.assert_allclose(p, want, rtol=0, atol=2e-7)
    # the moments after one step from zero: (1-b1) g and (1-b2) g^2
    np.testing.assert_allclose(m, 0.1 * g, rtol=1e-6, atol=0)
    np.testing.assert_allclose(v, 0.05 * g * g, rtol=1e-6, atol=0)


@pytest.mark.parametrize("steps", [1, 2, 10, 60])
def test_adamw_constant_gradient_closed_form(steps):
    # g constant => mhat_t = g and vhat_t = g^2 for every t, hence
    # theta_t = (1 - lr wd)^t theta0 - lr s sum_{k<t} (1 - lr wd)^k,  s = g / (|g| + eps)
    rng = np.random.default_rng(1)
    th0 = rng.normal(0, 0.02, 64)
    g = rng.normal(0, 1e-3, 64)
    lr, eps, wd = HP["lr"], HP["eps"], HP["weight_decay"]
    q = 1.0 - lr * wd
    s = g / (np.abs(g) + eps)
    want = q ** steps * th0 - lr * s * sum(q ** k for k in range(steps))
    p, m, v = f32(th0), f32(np.zeros(64)), f32(np.zeros(64))
    for t in range(1, steps + 1):
        O.adamw(p, m, v, f32(g), step=t, **HP)
    # fp32 state: each step rounds theta (|theta| ~ 0.02..0.06) and the update once
    np.testing.assert_allclose(p, want, rtol=0, atol=steps * 1.5e-8)
    # bias-corrected moments recover g and g^2
    np.testing.assert_allclose(m / (1 - 0.9 ** steps), f32(g), rtol=2e-6)
    np.testing.assert_allclose(v / (1 - 0.95 ** steps), f32(g).astype(np.float64) ** 2, rtol=4e-6)


@pytest.mark.parametrize("hp", [HP, dict(lr=1.5e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1)])
def test_adamw_matches_torch_library(hp):
    # independent library routine: torch.optim.AdamW, CPU, fp32, per-tensor loop
    rng = np.random.default_rng(2)
    n, steps = 100_000, 100
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    p, m, v = th0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    opt = torch.optim.AdamW([tp], lr=hp["lr"], betas=(hp["beta1"], hp["beta2"]), eps=hp["eps"],
                            weight_decay=hp["weight_decay"], foreach=False, fused=False)
    for t in range(1, steps + 1):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        O.adamw(p, m, v, g, step=t, **hp)
        tp.grad = torch.from_numpy(g.copy())
        opt.step()
    ref = tp.detach().numpy()
    assert np.all(np.abs(p - ref) <= tol(ref))
    # torch multiplies theta by the fp32-rounded factor (1 - lr wd) each step, a systematic
    # ~3e-8 relative offset per step; the float64 recurrence below is the tight pin
    assert np.max(np.abs(p - ref)) < 5e-7
    st = opt.state[tp]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-5, atol=1e-9)   # torch lerps: differs near m = 0
    # float(0.999) is 0.99900001, so 1 - beta2 formed from the fp32 value sits 1.3e-5 below torch's double 0.001
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=3e-5, atol=1e-14)
    assert np.max(np.abs(p - th0)) > 1e-3         # and the 100 steps did move the model


def test_adamw_matches_float64_recurrence():
    # the same rule evaluated in float64 throughout: fp32 rounding stays within the bar
    rng = np.random.default_rng(3)
    n, steps = 4096, 200
    th = rng.normal(0, 0.02, n)
    m64, v64 = np.zeros(n), np.zeros(n)
    p, m, v = f32(th), f32(m64), f32(v64)
    b1, b2, lr, eps, wd = (float(np.float32(HP[k])) for k in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    th = p.astype(np.float64)
    for t in range(1, steps + 1):
        g = rng.normal(0, 1e-3, n).astype(np.float32)
        O.adamw(p, m, v, g, step=t, **HP)
        g64 = g.astype(np.float64)
        m64 = b1 * m64 + (1 - b1) * g64
        v64 = b2 * v64 + (1 - b2) * g64 * g64
        th = th - lr * (m64 / (1 - b1 ** t) / (np.sqrt(v64 / (1 - b2 ** t)) + eps) + wd * th)
    assert np.all(np.abs(p - th) <= tol(th))
    np.testing.assert_allclose(m, m64, rtol=2e-6, atol=2e-10)   # m ~ 3e-4, its fp32 ulp ~ 3e-11
    np.testing.assert_allclose(v, v64, rtol=5e-6, atol=1e-16)


@pytest.mark.parametrize("case", range(12))
def test_rounds_with_random_scalars_stay_near_the_float64_evaluation(case):
    """Random hyper-parameters, group counts and phase sequences: the fp32 oracle stays within the
    parity bar of the same rules carried in float64 (numpy, whole arrays at once).  A breadth check on
    top of the pins above: nothing in the oracle is tuned to one set of scalars."""
    rng = np.random.default_rng(500 + case)
    n = 2000
    G = int(rng.choice([1, 2, 3, 5, 8]))
    hp = dict(lr=float(rng.choice([1e-4, 3e-4, 1e-3])), beta1=float(rng.choice([0.8, 0.9])),
              beta2=float(rng.choice([0.95, 0.99, 0.999])), eps=float(rng.choice([1e-8, 1e-6])),
              weight_decay=float(rng.choice([0.0, 0.01, 0.1])), grad_scale=float(rng.choice([1.0, 0.25, 0.6]))
              )
    c = {k: float(np.float32(v)) for k, v in hp.items()}
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    P = [th0.copy() for _ in range(G)]
    M1 = [np.zeros(n, np.float32) for _ in range(G)]
    V = [np.zeros(n, np.float32) for _ in range(G)]
    a, Mo = th0.copy(), np.zeros(n, np.float32)
    P64 = [th0.astype(np.float64) for _ in range(G)]
    M64 = [np.zeros(n) for _ in range(G)]
    V64 = [np.zeros(n) for _ in range(G)]
    a64, Mo64 = th0.astype(np.float64), np.zeros(n)
    t = 0
    for rnd in range(4):
        lazy = rnd < int(rng.integers(0, 3))
        for _ in range(int(rng.integers(1, 6))):
            t += 1
            shared = rng.normal(0, 1e-3, n).astype(np.float32)
            for g in range(G):
                gr = shared if lazy else rng.normal(0, 1e-3, n).astype(np.float32)
                O.adamw(P[g], M1[g], V[g], gr, step=t, **hp)
                g64 = gr.astype(np.float64) * c["grad_scale"]
                M64[g] = c["beta1"] * M64[g] + (1 - c["beta1"]) * g64
                V64[g] = c["beta2"] * V64[g] + (1 - c["beta2"]) * g64 * g64
                P64[g] = P64[g] - c["lr"] * (M64[g] / (1 - c["beta1"] ** t) / (np.sqrt(V64[g] / (1 - c["beta2"] ** t)) + c["eps"])
                                             + c["weight_decay"] * P64[g])
        mu, lr_o = float(np.float32(rng.choice([0.9, 0.95, 0.99]))), float(np.float32(rng.choice([0.3, 0.7, 1.1])))
        O.outer(P, a, Mo, mu=mu, lr=lr_o, phase=O.WARMUP if lazy else O.PIER)
        if lazy:
            Mo64 = mu * Mo64 + (P64[0] - a64)
            a64 = P64[0].copy()
        else:
            d = np.mean(np.stack(P64), axis=0) - a64
            Mo64 = mu * Mo64 + d
            a64 = a64 + lr_o * (mu * Mo64 + d)
            P64 = [a64.copy() for _ in range(G)]
        assert np.all(np.abs(a - a64) <= tol(a64)), (case, rnd)
        np.testing.assert_allclose(Mo, Mo64, rtol=1e-4, atol=2e-8)      # a difference of models: a few ulp of theta
        for g in range(G):
            assert np.all(np.abs(P[g] - P64[g]) <= tol(P64[g])), (case, rnd, g)
            np.testing.assert_allclose(M1[g], M64[g], rtol=1e-5, atol=1e-10)
            np.testing.assert_allclose(V[g], V64[g], rtol=1e-5, atol=1e-16)


def test_adamw_bf16_gradients_widen_exactly():
    from pier_inputs import generator as gen
    rng = np.random.default_rng(4)
    n = 1000
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    gb = gen.to_bf16_bits(g)
    gw = gen.bf16_bits_to_f32(gb)
    assert np.max(np.abs(gw - g)) <= np.max(np.abs(g)) * 2 ** -8
    # torch's own bf16 rounding is the independent check of the bit patterns
    tb = torch.from_numpy(g).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(tb, gb)
    a = [rng.normal(0, 0.02, n).astype(np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32)]
    b = [x.copy() for x in a]
    for t in (1, 2, 3):
        O.adamw(*a, gb, step=t, **HP)
        O.adamw(*b, gw, step=t, **HP)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_adamw_grad_scale_is_a_gradient_multiplier():
    rng = np.random.default_rng(5)
    n = 512
    g = rng.normal(0, 1e-3, n).astype(np.float32)
    a = [rng.normal(0, 0.02, n).astype(np.float32), np.zeros(n, np.float32), np.zeros(n, np.float32)]
    b = [x.copy() for x in a]
    O.adamw(*a, g, step=1, grad_scale=0.25, **HP)          # power of two: scaling is exact
    O.adamw(*b, (g * np.float32(0.25)).astype(np.float32), step=1, **HP)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ---------------------------------------------------------------- gradient clipping

def test_clip_hand_case_and_closed_form():
    # |(3, 4)| = 5: coefficient 1 / (5 + 1e-6); no clipping below the threshold
    ss = O.sumsq(f32([3.0, 4.0]))
    assert ss == 25.0
    assert O.clip_coef(ss, 1.0) == np.float32(1.0 / (5.0 + 1e-6))
    assert O.clip_coef(ss, 1.0) != np.float32(0.2)             # the 1e-6 is there
    assert O.clip_coef(ss, 10.0) == 1.0 and O.clip_coef(0.0, 1.0) == 1.0
    # constant gradient: norm = |c| sqrt(n); chained over a tensor list
    c, n = 1e-3, 1 << 20
    g = np.full(n, c, np.float32)
    ss = O.sumsq(g[:1000], 0.0)
    ss = O.sumsq(g[1000:], ss)
    assert abs(np.sqrt(ss) - abs(float(np.float32(c))) * np.sqrt(n)) < 1e-9      # 2^20 double additions
    assert abs(O.clip_coef(ss, 1.0) - 1.0 / (float(np.float32(c)) * 1024.0 + 1e-6)) < 1e-7
    # bf16 gradients are widened exactly
    from pier_inputs import generator as gen
    h = gen.to_bf16_bits(np.array([3.0, 4.0, -12.0], np.float32))
    assert O.sumsq(h) == 169.0


def test_clip_matches_torch_clip_grad_norm():
    # library routine: torch.nn.utils.clip_grad_norm_ over a list of tensors
    rng = np.random.default_rng(12)
    sizes = [1000, 33, 70_000, 5]
    gs = [rng.normal(0, 1e-3, k).astype(np.float32) for k in sizes]
    ss = 0.0
    for g in gs:
        ss = O.sumsq(g, ss)
    ps = [torch.nn.Parameter(torch.zeros(k)) for k in sizes]
    for p, g in zip(ps, gs):
        p.grad = torch.from_numpy(g.copy())
    for max_norm in (0.05, 1.0):
        for p, g in zip(ps, gs):
            p.grad = torch.from_numpy(g.copy())
        total = torch.nn.utils.clip_grad_norm_(ps, max_norm, foreach=False)
        assert abs(float(total) - np.sqrt(ss)) < 2e-7 * np.sqrt(ss)   # the library sums in fp32
        coef = O.clip_coef(ss, max_norm)
        if np.sqrt(ss) <= max_norm:
            assert coef == 1.0
        else:
            assert coef < 1.0
        for p, g in zip(ps, gs):
            np.testing.assert_allclose(p.grad.numpy(), g * coef, rtol=3e-7, atol=0)
    # feeding the coefficient as grad_scale equals stepping on the clipped gradient
    coef = O.clip_coef(ss, 0.05)
    a = [rng.normal(0, 0.02, 1000).astype(np.float32), np.zeros(1000, np.float32), np.zeros(1000, np.float32)]
    b = [x.copy() for x in a]
    O.adamw(*a, gs[0], step=1, grad_scale=coef, **HP)
    O.adamw(*b, (gs[0] * np.float32(coef)).astype(np.float32), step=1, **HP)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ---------------------------------------------------------------- bf16 working weights

def test_bf16_rounding_matches_the_library_and_the_definition():
    rng = np.random.default_rng(13)
    x = np.concatenate([
        rng.normal(0, 0.02, 100_000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, np.inf, -np.inf, 1e-40, -1e-40, 3.3895314e38, 65504.0], np.float32),
        # exact ties: 1 + 2^-8 (even below -> down), 1 + 3*2^-8 (odd below -> up)
        np.array([1.00390625, 1.01171875, -1.00390625, -1.01171875], np.float32),
    ])
    got = O.to_bf16(np.ascontiguousarray(x))
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got, lib)
    # definition: nearest representable value, never further than half a bf16 ulp
    back = (got.astype(np.uint32) << 16).view(np.float32)
    fin = np.isfinite(x) & (np.abs(x) < 3e38) & (np.abs(x) > 1e-30)
    assert np.all(np.abs(back[fin] - x[fin]) <= np.abs(x[fin]) * 2.0 ** -8)
    ties = O.to_bf16(np.array([1.00390625, 1.01171875], np.float32))
    assert list(ties) == [0x3F80, 0x3F82]                       # ties go to the even mantissa
    assert O.to_bf16(np.array([np.nan], np.float32))[0] == 0x7FC0
    # NaNs whose payload would carry into the exponent or sign if they were rounded like numbers
    nans = np.array([0x7FFFFFFF, 0xFFFFFFFF, 0x7F800001, 0xFF800001], np.uint32).view(np.float32)
    assert list(O.to_bf16(nans)) == [0x7FC0] * 4
    lib = torch.from_numpy(nans.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert all((v & 0x7F80) == 0x7F80 and (v & 0x007F) != 0 for v in lib)      # the library keeps them NaN too


# ---------------------------------------------------------------- outer step

def test_outer_single_group_unit_rate_returns_the_model():
    # G = 1, M = 0, mu = 0, lr = 1: plain AdamW plus the anchor copy
    rng = np.random.default_rng(6)
    n = 1000
    a0 = rng.normal(0, 0.02, n).astype(np.float32)
    th = (a0 + rng.normal(0, 1e-3, n)).astype(np.float32)
    for ph in (O.WARMUP, O.PIER):
        a, M, t = a0.copy(), np.zeros(n, np.float32), th.copy()
        O.outer([t], a, M, mu=0.0, lr=1.0, phase=ph)
        if ph == O.WARMUP:
            assert np.array_equal(a, th) and np.array_equal(t, th)
        else:
            assert np.max(np.abs(a - th)) <= 2 ** -29      # a + (theta - a): within an ulp of 0.06
            assert np.array_equal(t, a)
        np.testing.assert_allclose(M, th.astype(np.float64) - a0, rtol=0, atol=1e-9)


def test_outer_unit_rate_no_momentum_is_the_replica_mean():
    rng = np.random.default_rng(7)
    n, G = 777, 4
    a0 = rng.normal(0, 0.02, n).astype(np.float32)
    ths = [(a0 + rng.normal(0, 1e-3, n)).astype(np.float32) for _ in range(G)]
    mean = np.mean(np.stack(ths).astype(np.float64), axis=0)
    a, M = a0.copy(), (rng.normal(0, 1e-3, n)).astype(np.float32)   # mu = 0 must ignore old M
    t = [x.copy() for x in ths]
    O.outer(t, a, M, mu=0.0, lr=1.0, phase=O.PIER)
    np.testing.assert_allclose(a, mean, rtol=0, atol=4e-9)
    for x in t:
        assert np.array_equal(x, a)                        # every group re-synchronised
    np.testing.assert_allclose(M, mean - a0, rtol=0, atol=1e-9)


@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 8, 16, 64])
def test_lazy_start_sync_returns_the_model_bit_for_bit(G):
    """Algorithm 1 works on one model: after a synchronisation the stored theta_{t-r} IS theta_t,
    whatever the number of (identical) copies a caller keeps, and M <- mu M + (theta_t - theta_{t-r}).
    One fp32 subtraction is the exactly rounded difference, and with mu a power of two mu M is
    exact, so double arithmetic rounded once gives the fp32 result bit for bit."""
    rng = np.random.default_rng(60 + G)
    n = 4096
    a0 = f32(rng.normal(0, 0.02, n))
    th = f32(a0 + rng.normal(0, 1e-3, n))
    th[:7] = [0.0, -0.0, 1e-30, -3.0, 1e3, a0[5], -a0[6]]
    M0 = f32(rng.normal(0, 1e-3, n))
    reps = [th.copy() for _ in range(G)]
    # first synchronisation, M = 0
    a, M = a0.copy(), np.zeros(n, np.float32)
    O.outer(reps, a, M, mu=0.9, lr=55.0, phase=O.WARMUP)
    assert np.array_equal(a.view(np.uint32), th.view(np.uint32))           # signed zeros included
    assert all(np.array_equal(r.view(np.uint32), th.view(np.uint32)) for r in reps)
    exact = (th.astype(np.float64) - a0.astype(np.float64)).astype(np.float32)
    assert np.array_equal(M, exact)
    # mu = 1/2: mu M is exact, the sum of two floats is exact in double
    a, M = a0.copy(), M0.copy()
    O.outer(reps, a, M, mu=0.5, lr=0.0, phase=O.WARMUP)
    want = (0.5 * M0.astype(np.float64) + exact.astype(np.float64)).astype(np.float32)
    assert np.array_equal(M, want) and np.array_equal(a, th)
    # the number of copies does not enter the result
    a1, M1 = a0.copy(), M0.copy()
    O.outer([th.copy()], a1, M1, mu=0.9, lr=0.0, phase=O.WARMUP)
    aG, MG = a0.copy(), M0.copy()
    O.outer(reps, aG, MG, mu=0.9, lr=0.0, phase=O.WARMUP)
    assert np.array_equal(a1, aG) and np.array_equal(M1, MG)
    ref = 0.9 * M0.astype(np.float64) + (th.astype(np.float64) - a0)
    np.testing.assert_allclose(MG, ref, rtol=2e-7, atol=2e-10)


def test_outer_nesterov_two_rounds_by_hand():
    # a = 0, M = 0, lr = 0.7, mu = 0.9, one group, exactly representable deltas.
    # first step:  delta1 = 0.5          M1 = 0.5      theta1 = 0.7 (0.9*0.5 + 0.5) = 0.665
    # second step: model moved by 0.25   M2 = 0.9*0.5 + 0.25 = 0.7
    #          theta2 = 0.665 + 0.7 (0.9*0.7 + 0.25) = 0.665 + 0.616 = 1.281
    a, M = f32([0.0]), f32([0.0])
    th = f32([0.5])
    O.outer([th], a, M, mu=0.9, lr=0.7, phase=O.PIER)
    assert abs(M[0] - 0.5) < 1e-7 and abs(a[0] - 0.665) < 1e-7 and th[0] == a[0]
    th[0] = np.float32(th[0] + np.float32(0.25))
    O.outer([th], a, M, mu=0.9, lr=0.7, phase=O.PIER)
    assert abs(M[0] - 0.7) < 1e-7
    assert abs(a[0] - 1.281) < 2e-7 and th[0] == a[0]


def test_outer_matches_torch_sgd_nesterov():
    # library routine: SGD(momentum, nesterov=True) fed the gradient a - mean(theta);
    # its buffer is -M and its parameter is the anchor
    rng = np.random.default_rng(8)
    n, G = 5000, 8
    a0 = rng.normal(0, 0.02, n).astype(np.float32)
    a, M = a0.copy(), np.zeros(n, np.float32)
    tp = torch.nn.Parameter(torch.from_numpy(a0.copy()))
    sched = [(0.99, 0.3), (0.95, 0.8), (0.9, 1.1), (0.9, 0.9)]
    for k, (mu, lr) in enumerate(sched):
        ths = [(a + rng.normal(0, 2e-3, n)).astype(np.float32) for _ in range(G)]
        mean = torch.from_numpy(np.mean(np.stack(ths).astype(np.float64), axis=0).astype(np.float32))
        opt = torch.optim.SGD([tp], lr=lr, momentum=mu, nesterov=True)
        if k:
            opt.state[tp]["momentum_buffer"] = buf
        tp.grad = tp.detach() - mean
        opt.step()
        buf = opt.state[tp]["momentum_buffer"]
        O.outer(ths, a, M, mu=mu, lr=lr, phase=O.PIER)
        ref = tp.detach().numpy()
        assert np.all(np.abs(a - ref) <= tol(ref)), k
        assert np.max(np.abs(a - ref)) < 2e-8
        np.testing.assert_allclose(M, -buf.numpy(), rtol=1e-5, atol=1e-8)  # the library rounds the mean to fp32 first
        for x in ths:
            assert np.array_equal(x, a)


@pytest.mark.parametrize("G", [2, 3, 8])
def test_warmup_accumulates_without_touching_the_model(G):
    rng = np.random.default_rng(9)
    n, K = 300, 5
    th = rng.normal(0, 0.02, n).astype(np.float32)
    a, M, M1 = th.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    a1 = th.copy()
    th0 = th.copy()
    deltas = []
    for _ in range(K):
        new = (th + rng.normal(0, 1e-3, n)).astype(np.float32)
        deltas.append(new.astype(np.float64) - th)
        th = new
        reps = [th.copy() for _ in range(G)]
        O.outer(reps, a, M, mu=0.9, lr=123.0, phase=O.WARMUP)    # lr must be ignored
        for r in reps:
            assert np.array_equal(r, th)                           # model not updated
        assert np.array_equal(a, th)                               # anchor follows the model
        O.outer([th.copy()], a1, M1, mu=1.0, lr=0.0, phase=O.WARMUP)
    want = sum(0.9 ** (K - 1 - j) * d for j, d in enumerate(deltas))   # M = sum mu^(k-j) delta_j
    np.testing.assert_allclose(M, want, rtol=0, atol=5e-9)
    np.testing.assert_allclose(M1, th.astype(np.float64) - th0, rtol=0, atol=5e-9)  # mu = 1 telescopes


def test_difference_then_mean_equals_mean_then_difference():
    # the all-reduce may average differences or difference the average: same number
    rng = np.random.default_rng(10)
    n, G = 2048, 8
    a0 = rng.normal(0, 0.02, n).astype(np.float32)
    ths = [(a0 + rng.normal(0, 1e-3, n)).astype(np.float32) for _ in range(G)]
    a, M = a0.copy(), np.zeros(n, np.float32)
    O.outer([t.copy() for t in ths], a, M, mu=0.9, lr=0.7, phase=O.PIER)
    d = np.mean(np.stack(ths).astype(np.float64), axis=0) - a0
    want = a0 + 0.7 * 1.9 * d
    assert np.all(np.abs(a - want) <= tol(want))
    assert np.max(np.abs(a - want)) < 1e-8


# ---------------------------------------------------------------- whole rounds

def test_rounds_against_torch_optimizers():
    """H inner steps per group then an outer step, three rounds: AdamW moments and
    the step count carry across outer steps; checked against torch's two optimizers."""
    rng = np.random.default_rng(11)
    n, G, H = 3000, 2, 5
    th0 = rng.normal(0, 0.02, n).astype(np.float32)
    P = [th0.copy() for _ in range(G)]
    Mo = [np.zeros(n, np.float32) for _ in range(G)]
    V = [np.zeros(n, np.float32) for _ in range(G)]
    a, M = th0.copy(), np.zeros(n, np.float32)
    tps = [torch.nn.Parameter(torch.from_numpy(th0.copy())) for _ in range(G)]
    inner = [torch.optim.AdamW([tp], lr=HP["lr"], betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1,
                               foreach=False) for tp in tps]
    anchor = torch.nn.Parameter(torch.from_numpy(th0.copy()))
    outer = torch.optim.SGD([anchor], lr=0.7, momentum=0.9, nesterov=True)
    t = 0
    for _ in range(3):
        for _ in range(H):
            t += 1
            for g in range(G):
                gr = rng.normal(0, 1e-3, n).astype(np.float32)
                O.adamw(P[g], Mo[g], V[g], gr, step=t, **HP)
                tps[g].grad = torch.from_numpy(gr.copy())
                inner[g].step()
        O.outer(P, a, M, mu=0.9, lr=0.7, phase=O.PIER)
        with torch.no_grad():
            anchor.grad = anchor.detach() - torch.stack([tp.detach() for tp in tps]).mean(0)
            outer.step()
            for tp in tps:
                tp.copy_(anchor)
        ref = anchor.detach().numpy()
        assert np.all(np.abs(a - ref) <= tol(ref))
        assert np.max(np.abs(a - ref)) < 2e-7        # torch's rounded decay factor, see above
        assert all(np.array_equal(p, a) for p in P)


# ---------------------------------------------------------------- schedules

def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "schedules.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                t, T, ph, mu, lr = line.split()
                rows.append((int(t), int(T), int(ph), float(mu), float(lr)))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_schedules_match_the_printed_constants(row):
    t, T, ph, mu, lr = row
    assert O.phase(t, T) == ph
    assert O.mu(t, T) == np.float32(mu)
    assert abs(O.outer_lr(t, T) - lr) <= 1e-7
    p2, mu2, lr2 = O.outer_scalars(t, T)
    assert p2 == ph
    if ph == 0:
        assert mu2 == np.float32(0.9) and lr2 == 0.0       # Algorithm 1's default mu
    else:
        assert mu2 == np.float32(mu) and abs(lr2 - lr) <= 1e-7


def test_inner_lr_schedule_endpoints_and_library_cosine():
    # Table I: GPT-2 small 4e-4 -> 4e-5, medium 3e-4 -> 3e-5, XL 1.5e-4 -> 1.5e-5; T = 100000; 2% warmup
    T = 100_000
    for lr_max, lr_min in ((4e-4, 4e-5), (3e-4, 3e-5), (1.5e-4, 1.5e-5)):
        assert O.inner_lr(2000, T, lr_max, lr_min) == np.float32(lr_max)         # end of warmup
        assert O.inner_lr(1000, T, lr_max, lr_min) == np.float32(np.float32(lr_max) / 2.0)
        assert O.inner_lr(T, T, lr_max, lr_min) == np.float32(lr_min)
        assert O.inner_lr(T + 5, T, lr_max, lr_min) == np.float32(lr_min)
        mid = O.inner_lr(51_000, T, lr_max, lr_min)                              # half way down the cosine
        assert abs(mid - (np.float32(lr_max) + np.float32(lr_min)) / 2) < 1e-10
        lrs = [O.inner_lr(t, T, lr_max, lr_min) for t in range(1, T + 1, 97)]
        k = lrs.index(max(lrs))
        assert all(a <= b for a, b in zip(lrs[:k], lrs[1:k + 1])) and all(a >= b for a, b in zip(lrs[k:], lrs[k + 1:]))
    # the cosine leg against torch's CosineAnnealingLR (library routine), T_max = T - W steps
    W, lr_max, lr_min = 2000, 3e-4, 3e-5
    p = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([p], lr=lr_max)
    sched = torch.optim.lr_scheduler.CosineAnnealingLR(opt, T_max=T - W, eta_min=lr_min)
    for k in range(1, 3001):
        opt.step()
        sched.step()
        if k % 500 == 0:
            assert abs(sched.get_last_lr()[0] - O.inner_lr(W + k, T, lr_max, lr_min)) < 3e-11
    # no warmup at all
    assert O.inner_lr(1, 100, 1.0, 0.1, 0.0) < 1.0 and O.inner_lr(1, 100, 1.0, 0.1, 0.0) > 0.99


def test_schedule_is_monotone_where_the_paper_says_so():
    T = 1000
    mus = [O.mu(t, T) for t in range(100, T + 1)]
    assert all(x >= y for x, y in zip(mus, mus[1:]))          # 0.99 -> 0.95 -> 0.9
    lrs = [O.outer_lr(t, T) for t in range(100, 200)]
    assert all(x < y for x, y in zip(lrs, lrs[1:])) and lrs[0] == 0.0 and lrs[-1] < 1.0
