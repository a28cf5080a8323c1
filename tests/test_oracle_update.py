"""Pins for the oracle's arithmetic: closed forms, textbook special cases and
library routines it must reduce to."""
import math

import numpy as np
import pytest
import torch

import oracle as orc
from parity import check_moments_and_params, ulp_distance_f32

HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, grad_scale=0.25, max_norm=0.0,
          adamw=True)
f32 = np.float32


def _rand(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


# ---- fold ---------------------------------------------------------------------
def test_fold_is_a_left_fold_in_the_given_order():
    # one element, values chosen so the association order is visible in the result
    big, one = f32(2.0 ** 24), f32(1.0)
    a = [np.array([v], np.float32) for v in (big, one, one, -big)]
    assert orc.fold(a, 4)[0] == 0.0                     # ((big+1)+1)-big : the ones are absorbed
    assert orc.fold([a[1], a[2], a[0], a[3]], 4)[0] == 2.0
    # two groups of two: (big + 1) + (1 + -big) = big + (1-big) -> 0 ; partials are formed first
    assert orc.fold([a[0], a[1], a[2], a[3]], 2)[0] == f32(big + (one - big))
    assert orc.fold([a[1], a[2], a[0], a[3]], 2)[0] == 2.0
    # -0 survives (no add with a zero start value)
    nz = [np.array([-0.0], np.float32)]
    assert np.signbit(orc.fold(nz, 1)[0])
    assert np.signbit(orc.fold(nz * 4, 2)[0])


def test_fold_bf16_equals_fold_of_upconverted_values():
    rng = np.random.default_rng(1)
    P, n = 6, 1000
    bits = [rng.integers(0, 1 << 16, n).astype(np.uint16) for _ in range(P)]
    for b in bits:                                      # keep finite values only
        b[(b & 0x7F80) == 0x7F80] = 0x3F80
    up = [orc.bf16_bits_to_f32(b) for b in bits]
    for gl in (1, 2, 3, 6):
        assert orc.fold(bits, gl).tobytes() == orc.fold(up, gl).tobytes()
    # the up-conversion itself, against torch's
    t = torch.from_numpy(bits[0].view(np.int16)).view(torch.bfloat16).float().numpy()
    assert t.tobytes() == up[0].tobytes()


def test_fold_matches_python_float32_loop():
    rng = np.random.default_rng(2)
    P, n = 8, 50
    x = [(rng.standard_normal(n) * 10.0 ** rng.integers(-4, 4, n)).astype(np.float32) for _ in range(P)]
    for gl in (8, 4, 2, 1):
        want = np.empty(n, np.float32)
        for e in range(n):
            parts = []
            for k0 in range(0, P, gl):
                a = x[k0][e]
                for l in range(1, gl):
                    a = f32(a + x[k0 + l][e])
                parts.append(a)
            acc = parts[0]
            for a in parts[1:]:
                acc = f32(acc + a)
            want[e] = acc
        assert orc.fold(x, gl).tobytes() == want.tobytes()


# ---- sum of squares and the clip coefficient -------------------------------------
def test_sumsq_against_exact_sum():
    g = _rand(200_001, 3, 1e-3)
    exact = math.fsum(float(x) * float(x) for x in g)
    assert abs(orc.sumsq(g) - exact) <= 1e-13 * exact
    assert orc.sumsq(np.zeros(0, np.float32)) == 0.0
    c = np.full(4096, 0.5, np.float32)
    assert orc.sumsq(c) == 1024.0


def test_clip_coef_closed_forms():
    # constant gradient x over n elements: norm = grad_scale * |x| * sqrt(n)
    n, x, gs = 10_000, 0.3, 0.25
    tot = orc.sumsq(np.full(n, x, np.float32))
    norm = gs * float(f32(x)) * math.sqrt(n)
    assert orc.clip_coef(tot, gs, 1.0) == pytest.approx(1.0 / (norm + 1e-6), rel=1e-12)
    assert orc.clip_coef(tot, gs, 100.0) == 1.0          # norm below the threshold: no scaling
    assert orc.clip_coef(tot, gs, 0.0) == 1.0            # clipping disabled
    assert orc.clip_coef(tot, gs, -1.0) == 1.0
    assert orc.clip_coef(0.0, gs, 1.0) == 1.0


def test_clip_matches_torch_clip_grad_norm():
    rng = np.random.default_rng(5)
    for max_norm in (0.5, 1.0, 50.0):
        # fp32-representable gradients, held in fp64 by torch, so both sides see the same numbers
        gs = [(rng.standard_normal(s) * 0.7).astype(np.float32) for s in (5, 1000, 37)]
        params = [torch.nn.Parameter(torch.zeros(x.shape[0], dtype=torch.float64)) for x in gs]
        for p, x in zip(params, gs):
            p.grad = torch.from_numpy(x.astype(np.float64))
        torch.nn.utils.clip_grad_norm_(params, max_norm)
        flat = np.concatenate(gs)
        coef = orc.clip_coef(orc.sumsq(flat), 1.0, max_norm)
        got = np.concatenate([p.grad.numpy() for p in params])
        assert np.allclose(got, flat.astype(np.float64) * coef, rtol=1e-12, atol=0)
        assert (coef < 1.0) == (max_norm < 10)


# ---- Adam -------------------------------------------------------------------------
def _state(n, seed):
    return _rand(n, seed, 0.02), np.zeros(n, np.float32), np.zeros(n, np.float32)


@pytest.mark.parametrize("literal32", [False, True])
def test_adam_first_step_closed_form(literal32):
    # from m = v = 0 the bias corrections cancel: m1 = (1-b1) gh, v1 = (1-b2) gh^2,
    # p1 = p0 (1 - lr wd) - lr * gh / (|gh| + eps)
    n = 4096
    g = _rand(n, 11, 1e-3)
    p, m, v = _state(n, 12)
    p0 = p.astype(np.float64)
    sc = 0.25 * 0.8
    orc.adam(g, p, m, v, sc=sc, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8),
             weight_decay=f32(0.01), step=1, literal32=literal32)
    b1, b2, lr, eps, wd = (float(f32(x)) for x in (0.9, 0.999, 1e-4, 1e-8, 0.01))
    gh = (float(f32(sc)) if literal32 else sc) * g.astype(np.float64)
    tol = 4e-7 if literal32 else 1e-7
    assert np.allclose(m, (1 - b1) * gh, rtol=tol, atol=0)
    assert np.allclose(v, (1 - b2) * gh * gh, rtol=tol, atol=0)
    want = p0 * (1 - lr * wd) - lr * gh / (np.abs(gh) + eps)
    assert (np.abs(p - want) <= tol * (np.abs(p0) + lr)).all()      # p may cancel against the step
    # the update has the sign of the gradient and size ~ lr
    moved = p0 * (1 - lr * wd) - p
    assert (np.sign(moved[g != 0]) == np.sign(g[g != 0])).all()
    assert np.allclose(np.abs(moved[np.abs(gh) > 1e-6]), lr, rtol=2e-2)


@pytest.mark.parametrize("adamw", [True, False])
def test_adam_matches_torch_optimizer_in_fp64(adamw):
    n, steps = 513, 5
    p, m, v = _state(n, 21)
    tp = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
    b1, b2, lr, eps, wd = (float(f32(x)) for x in (0.9, 0.999, 1e-4, 1e-8, 0.01))
    cls = torch.optim.AdamW if adamw else torch.optim.Adam
    opt = cls([tp], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    err = 0.0
    eb_m = np.zeros(n)
    eb_v = np.zeros(n)
    for t in range(1, steps + 1):
        g = _rand(n, 30 + t, 1e-3)
        sc = 0.125
        tp.grad = torch.from_numpy(g.astype(np.float64) * sc)
        opt.step()
        orc.adam(g, p, m, v, sc=sc, lr=f32(lr), beta1=f32(b1), beta2=f32(b2), eps=f32(eps),
                 weight_decay=f32(wd), step=t, adamw=adamw)
        ref, ref_m, ref_v = (x.detach().numpy() for x in (tp, opt.state[tp]["exp_avg"],
                                                            opt.state[tp]["exp_avg_sq"]))
        # the oracle keeps fp32 state (one rounding of half an ulp per step, carried on by the
        # moving average); torch keeps fp64
        eb_m = b1 * eb_m + 6.0e-8 * np.abs(ref_m) + 1e-30
        eb_v = b2 * eb_v + 6.0e-8 * np.abs(ref_v) + 1e-30
        if not adamw:
            # L2 mode feeds wd * p into the moments, so p's own rounding error enters them
            dp = wd * t * 1.2e-7 * (np.abs(ref) + lr)
            gh = np.abs(g.astype(np.float64) * sc) + wd * np.abs(ref)
            eb_m += (1 - b1) * dp
            eb_v += (1 - b2) * 2 * gh * dp
        assert (np.abs(m - ref_m) <= 1.01 * eb_m).all(), t
        assert (np.abs(v - ref_v) <= 1.01 * eb_v).all(), t
        assert (np.abs(p - ref) <= t * 1.2e-7 * (np.abs(ref) + lr)).all(), t
        err = max(err, np.max(np.abs(p - ref)))
    assert err > 0          # and the comparison is not vacuous (fp32 rounding is visible)


def test_adam_fp32_literal_stays_within_the_parity_tolerance_of_the_reference():
    n = 100_000
    g = _rand(n, 41, 1e-3)
    pa, ma, va = _state(n, 42)
    ma[:] = _rand(n, 43, 1e-4)
    va[:] = np.abs(_rand(n, 44, 1e-7))
    pb, mb, vb = pa.copy(), ma.copy(), va.copy()
    kw = dict(sc=0.0625 * 0.37, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8),
              weight_decay=f32(0.01), step=7)
    m_old, p_old = ma.copy(), pa.copy()
    orc.adam(g, pa, ma, va, literal32=False, **kw)
    orc.adam(g, pb, mb, vb, literal32=True, **kw)
    gh = float(f32(kw["sc"])) * g.astype(np.float64)
    check_moments_and_params(pb, mb, vb, pa, ma, va, p_old=p_old, m_old=m_old, g_hat=gh)
    assert ulp_distance_f32(vb, va) <= 8          # v has no cancellation: a few ulp at most


def test_adam_without_decay_and_zero_gradient_keeps_parameters():
    n = 100
    p, m, v = _state(n, 51)
    p0 = p.copy()
    orc.adam(np.zeros(n, np.float32), p, m, v, sc=1.0, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999),
             eps=f32(1e-8), weight_decay=f32(0.0), step=1)
    assert (p == p0).all() and (m == 0).all() and (v == 0).all()
    # padding (all-zero state and gradient) stays zero even with decay
    z = [np.zeros(8, np.float32) for _ in range(4)]
    orc.adam(*z, sc=1.0, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8),
             weight_decay=f32(0.01), step=3)
    assert all((a == 0).all() for a in z)


def test_adam_moments_are_exponential_moving_averages():
    # constant gradient: m_t = (1 - b1^t) gh, v_t = (1 - b2^t) gh^2  (geometric series)
    n = 64
    g = np.full(n, 0.002, np.float32)
    p, m, v = _state(n, 61)
    b1, b2 = float(f32(0.9)), float(f32(0.999))
    for t in range(1, 21):
        orc.adam(g, p, m, v, sc=1.0, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8),
                 weight_decay=f32(0.0), step=t)
        gh = float(g[0])
        assert np.allclose(m, (1 - b1 ** t) * gh, rtol=t * 1e-7)
        assert np.allclose(v, (1 - b2 ** t) * gh * gh, rtol=t * 1e-7)


# ---- bf16 pack ---------------------------------------------------------------------
def test_bf16_rne_matches_torch_cast_on_a_dense_sweep():
    # every upper half x a set of lower halves that covers below / at / above the tie
    rng = np.random.default_rng(9)
    lows = np.concatenate([np.array([0, 1, 0x7FFF, 0x8000, 0x8001, 0xFFFF], np.uint32),
                           rng.integers(0, 1 << 16, 26).astype(np.uint32)])
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for lo in lows:
        bits = hi | lo
        x = bits.view(np.float32)
        got = orc.bf16_rne(x)
        want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        nan = np.isnan(x)
        assert (got[~nan] == want[~nan]).all()
        # NaN in, NaN out, sign kept
        assert ((got[nan] & 0x7F80) == 0x7F80).all() and ((got[nan] & 0x007F) != 0).all()
        assert ((got[nan] >> 15) == (bits[nan] >> 31)).all()


def test_bf16_rne_ties_and_specials():
    def r(u):
        return int(orc.bf16_rne(np.array([u], np.uint32).view(np.float32))[0])
    assert r(0x3F808000) == 0x3F80          # tie, kept half even: down
    assert r(0x3F818000) == 0x3F82          # tie, kept half odd: up
    assert r(0x3F808001) == 0x3F81
    assert r(0x3F807FFF) == 0x3F80
    assert r(0x7F7FFFFF) == 0x7F80          # largest finite rounds to +inf
    assert r(0x7F800000) == 0x7F80 and r(0xFF800000) == 0xFF80
    assert r(0x80000000) == 0x8000 and r(0x00000000) == 0x0000
    assert r(0x00008000) == 0x0000 and r(0x00018000) == 0x0002     # denormal ties


# ---- the whole path on tiny inputs, against brute force -------------------------------
@pytest.mark.parametrize("strategy", ["IIG", "GGG", "III", "NNN", "NIG", "NNI"])
def test_reduce_shard_equals_direct_sum_and_shards_tile_the_model(strategy):
    P, G = 4, 2
    sizes = [37, 1, 200, 0, 19]
    lay = orc.layout(P, G, sizes)
    rng = np.random.default_rng(17)
    grads = [[rng.integers(-8, 9, s).astype(np.float32) for s in sizes] for _ in range(P)]
    flat_sum = np.zeros(P * lay.L)
    for q in range(P):
        flat_sum[:lay.total] += np.concatenate(grads[q])
    seen = np.zeros(P * lay.L, np.int32)
    tot = 0.0
    for r in range(P):
        g, ss = orc.reduce_shard(lay, strategy, orc.HORING, r, grads, "tensors")
        b, n = orc.state_range(lay, r, strategy[2])
        assert (g == flat_sum[b:b + n]).all()            # small integers: exact
        seen[b:b + n] += 1
        tot += ss
    reps = {"G": 1, "I": P // G, "N": P}[strategy[2]]
    assert (seen == reps).all()
    assert tot == float(np.sum(flat_sum ** 2))           # every element counted once in the norm


# ---- fp16 inputs and fp16 pack ---------------------------------------------------------
def test_f16_pack_matches_torch_cast():
    rng = np.random.default_rng(10)
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    for lo in [0, 1, 0x0FFF, 0x1000, 0x1001, 0x1FFF, 0x2000, 0xFFFF] + [int(x) for x in rng.integers(0, 1 << 16, 8)]:
        x = (hi | np.uint32(lo)).view(np.float32)
        got = orc.f16_rne(x)
        want = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
        with np.errstate(over="ignore", under="ignore"):
            want_np = x.astype(np.float16).view(np.uint16)             # a second, unrelated implementation
        nan = np.isnan(x)
        assert (got[~nan] == want[~nan]).all() and (got[~nan] == want_np[~nan]).all()
        assert ((got[nan] & 0x7C00) == 0x7C00).all() and ((got[nan] & 0x03FF) != 0).all()
        assert ((got[nan] >> 15) == (x[nan].view(np.uint32) >> 31)).all()
    f = lambda v: int(orc.f16_rne(np.array([v], np.float32))[0])       # noqa: E731
    assert f(65504.0) == 0x7BFF and f(65520.0) == 0x7C00 and f(65519.9) == 0x7BFF    # overflow threshold
    assert f(2.0 ** -24) == 0x0001 and f(2.0 ** -25) == 0x0000 and f(1.5 * 2.0 ** -25) == 0x0001
    # every binary16 value converts back to itself, and the midpoint between neighbours goes to the even one
    h = np.arange(0x7C00, dtype=np.uint16)
    vals = h.view(np.float16).astype(np.float32)
    assert (orc.f16_rne(vals) == h).all() and (orc.f16_rne(-vals) == (h | 0x8000)).all()
    mid = ((vals[:-1].astype(np.float64) + vals[1:].astype(np.float64)) / 2).astype(np.float32)   # exact in fp32
    even = np.where(h[:-1] & 1, h[1:], h[:-1])
    assert (orc.f16_rne(mid) == even).all()
    above = np.nextafter(mid, np.float32(np.inf))
    below = np.nextafter(mid, np.float32(-np.inf))
    assert (orc.f16_rne(above) == h[1:]).all() and (orc.f16_rne(below[1:]) == h[1:-1]).all()


def test_fold_of_f16_inputs_is_the_fold_of_their_exact_values():
    rng = np.random.default_rng(12)
    bits = [rng.integers(0, 1 << 16, 500).astype(np.uint16) for _ in range(4)]
    for b in bits:
        b[(b & 0x7C00) == 0x7C00] = 0x3C00
    halves = [b.view(np.float16) for b in bits]
    exact = [torch.from_numpy(b.view(np.int16)).view(torch.float16).float().numpy() for b in bits]
    assert orc.fold(halves, 2).tobytes() == orc.fold(exact, 2).tobytes()


def test_skipped_step_changes_nothing():
    lay = orc.layout(2, 1, [64])
    g = _rand(lay.L, 1)
    p, m, v = _state(lay.L, 2)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    hp = dict(HP, skip_nonfinite=True)
    for tot in (float("inf"), float("nan")):
        coef = orc.adam_shard(lay, "GGG", 0, g, p, m, v, total_sumsq=tot, hp=hp, step=1)
        assert math.isnan(coef) and p.tobytes() == p0.tobytes() and m.tobytes() == m0.tobytes() and v.tobytes() == v0.tobytes()
    orc.adam_shard(lay, "GGG", 0, g, p, m, v, total_sumsq=1.0, hp=hp, step=1)
    assert p.tobytes() != p0.tobytes()
