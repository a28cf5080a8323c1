"""More pins for the oracle, each against something that is not the oracle: the
per-tensor weight-decay mask and the chunk-layout reduce against brute force, Adam
against the textbook algorithm written in numpy, the all-fp32 evaluation against
numpy's own float32 arithmetic, and the tolerance checker against planted errors."""
import numpy as np
import pytest

import oracle as orc
from parity import check_bf16_within_one_ulp, check_moments_and_params

f32 = np.float32
HP = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, grad_scale=0.25, max_norm=0.0)


def _rand(n, seed, scale=1.0):
    return (np.random.default_rng(seed).standard_normal(n) * scale).astype(np.float32)


# ---- Adam, Kingma & Ba Algorithm 1, written as the textbook writes it -----------------------
def _textbook_adam(g, p, m, v, *, lr, b1, b2, eps, wd, t, adamw):
    """fp64 numpy.  Bias-corrected moments m_hat, v_hat formed explicitly; decoupled decay as a
    separate step before the update (Loshchilov & Hutter), classic L2 as wd * p joined to the
    gradient."""
    g, p, m, v = (a.astype(np.float64) for a in (g, p, m, v))
    if not adamw:
        g = g + wd * p
    m = b1 * m + (1 - b1) * g
    v = b2 * v + (1 - b2) * g * g
    m_hat = m / (1 - b1 ** t)
    v_hat = v / (1 - b2 ** t)
    if adamw:
        p = p - lr * wd * p
    p = p - lr * m_hat / (np.sqrt(v_hat) + eps)
    return p, m, v


@pytest.mark.parametrize("adamw", [True, False])
@pytest.mark.parametrize("literal32", [False, True])
def test_adam_against_textbook_algorithm_in_numpy(adamw, literal32):
    """Four steps with fresh gradients; the oracle carries fp32 state, the textbook fp64 state
    restarted from the oracle's fp32 state at every step, so each step is compared on its own."""
    n = 3000
    p, m, v = _rand(n, 1, 0.02), _rand(n, 2, 1e-4), np.abs(_rand(n, 3, 1e-7))
    b1, b2, lr, eps, wd = (float(f32(HP[k])) for k in ("beta1", "beta2", "lr", "eps", "weight_decay"))
    for t in range(1, 5):
        g = _rand(n, 10 + t, 1e-3)
        sc = 0.25 * 0.7
        gh = (float(f32(sc)) if literal32 else sc) * g.astype(np.float64)
        want_p, want_m, want_v = _textbook_adam(gh, p, m, v, lr=lr, b1=b1, b2=b2, eps=eps, wd=wd, t=t, adamw=adamw)
        p_old = p.astype(np.float64)
        orc.adam(g, p, m, v, sc=sc, lr=f32(lr), beta1=f32(b1), beta2=f32(b2), eps=f32(eps), weight_decay=f32(wd),
                 step=t, adamw=adamw, literal32=literal32)
        tol = 2e-6 if literal32 else 1.5e-7               # half an ulp of fp32 is 6e-8 relative
        gin = np.abs(gh) + (0 if adamw else wd * np.abs(p_old))
        assert (np.abs(v - want_v) <= tol * np.maximum(np.abs(want_v), (1 - b2) * gin * gin)).all(), t
        assert (np.abs(m - want_m) <= tol * np.maximum(np.abs(want_m), (1 - b1) * gin)).all(), t
        # p: relative to the terms of the difference; L2's gradient sum may cancel, which the step sees
        slack = tol * (np.abs(p_old) + np.abs(want_p - p_old)) + (0 if adamw else 4 * tol * lr)
        assert (np.abs(p - want_p) <= slack).all(), t
    assert np.abs(p.astype(np.float64) - want_p).max() > 0


def _numpy_f32_adam(g, p, m, v, *, sc, lr, b1, b2, eps, wd, t, adamw):
    """The all-fp32 evaluation with numpy float32 arrays: every numpy operation on float32
    operands is one correctly rounded IEEE operation (sqrt and division included), so this is the
    stated operation sequence without any compiler in between.  Scalars that do not depend on
    the element are formed in Python floats (fp64) from the fp32 hyper-parameters, rounded once."""
    sc = f32(sc)
    b1, b2, lr, eps, wd = f32(b1), f32(b2), f32(lr), f32(eps), f32(wd)
    omb1, omb2 = f32(1.0 - float(b1)), f32(1.0 - float(b2))
    bc1, bc2 = f32(1.0 - float(b1) ** t), f32(1.0 - float(b2) ** t)
    step_size = f32(float(lr) / float(bc1))
    sqrt_bc2 = f32(np.sqrt(float(bc2)))
    decay = f32(1.0 - float(lr) * float(wd))
    gh = sc * g
    if not adamw:
        gh = gh + wd * p
    m = b1 * m + omb1 * gh
    v = b2 * v + omb2 * (gh * gh)
    den = np.sqrt(v) / sqrt_bc2 + eps
    upd = step_size * (m / den)
    p = (p * decay if adamw else p) - upd
    for a in (gh, m, v, den, upd, p):
        assert a.dtype == np.float32
    return p, m, v


@pytest.mark.parametrize("adamw", [True, False])
def test_adam32_is_the_stated_sequence_of_fp32_operations(adamw):
    """orc_adam32 (C, gcc) against numpy float32: bit for bit, over several steps."""
    n = 50_000
    p, m, v = _rand(n, 4, 0.02), _rand(n, 5, 1e-4), np.abs(_rand(n, 6, 1e-7))
    for t in (1, 2, 7, 1000):
        g = _rand(n, 20 + t, 1e-3)
        want = _numpy_f32_adam(g, p.copy(), m.copy(), v.copy(), sc=0.0625 * 0.91, lr=HP["lr"], b1=HP["beta1"],
                               b2=HP["beta2"], eps=HP["eps"], wd=HP["weight_decay"], t=t, adamw=adamw)
        orc.adam(g, p, m, v, sc=0.0625 * 0.91, lr=f32(HP["lr"]), beta1=f32(HP["beta1"]), beta2=f32(HP["beta2"]),
                 eps=f32(HP["eps"]), weight_decay=f32(HP["weight_decay"]), step=t, adamw=adamw, literal32=True)
        for got, w, name in zip((p, m, v), want, "pmv"):
            assert got.tobytes() == w.tobytes(), (name, t)


# ---- the per-tensor weight-decay mask ---------------------------------------------------------
@pytest.mark.parametrize("strategy", ["IIG", "III", "NNN", "GGG"])
@pytest.mark.parametrize("adamw", [True, False])
def test_adam_shard_decay_mask_brute_force(strategy, adamw):
    """adam_shard(no_decay=...) against one call of the element-wise routine per element, each
    with the decay of the tensor that a brute-force element -> tensor map names.  The list has
    empty tensors (masked and not), one-element tensors, a masked tensor that straddles a chunk
    edge, a masked last tensor followed by padding (padding decays like any element: with zero
    state it stays zero; the classic-L2 variant gives it non-zero state so that the decay shows)."""
    P, G = 4, 2
    sizes = [5, 0, 3, 1, 0, 40, 1, 9, 0, 30]
    no_decay = [0, 1, 1, 0, 0, 1, 1, 0, 1, 1]
    lay = orc.layout(P, G, sizes)
    assert lay.L == 24 and lay.total == 89 and P * lay.L > lay.total
    owner = np.repeat(np.arange(len(sizes)), sizes)              # flat element -> tensor, by brute force
    assert owner[lay.L - 1] == owner[lay.L] == 5 and no_decay[5]  # the masked tensor crosses the first chunk edge
    exempt = np.zeros(P * lay.L, bool)
    exempt[:lay.total] = np.array(no_decay, bool)[owner]         # padding: not exempt
    hp = dict(HP, adamw=adamw, max_norm=0.05)
    f = np.float32
    for rank in range(P):
        ob, ol = orc.state_range(lay, rank, strategy[2])
        g = _rand(ol, 100 + rank, 1e-2)
        p0, m0, v0 = _rand(ol, 200 + rank, 0.5), _rand(ol, 300 + rank, 1e-3), np.abs(_rand(ol, 400 + rank, 1e-5))
        g[max(0, lay.total - ob):] = 0
        if adamw:       # padding as the path keeps it: all zero.  (The other variant leaves the state of the
            for a in (p0, m0, v0):      # padding non-zero, so that "padding decays" can be seen at all.)
                a[max(0, lay.total - ob):] = 0
        total = 3.0
        for literal32 in (False, True):
            p, m, v = p0.copy(), m0.copy(), v0.copy()
            coef = orc.adam_shard(lay, strategy, rank, g, p, m, v, total_sumsq=total, hp=hp, step=3, no_decay=no_decay,
                                  literal32=literal32)
            assert coef == orc.clip_coef(total, f(hp["grad_scale"]), f(hp["max_norm"])) and coef < 1
            sc = float(f(hp["grad_scale"])) * coef
            for e in range(ol):
                one = [a[e:e + 1].copy() for a in (g, p0, m0, v0)]
                wd = f(0.0) if exempt[ob + e] else f(hp["weight_decay"])
                orc.adam(*one, sc=sc, lr=f(hp["lr"]), beta1=f(hp["beta1"]), beta2=f(hp["beta2"]), eps=f(hp["eps"]),
                         weight_decay=wd, step=3, adamw=adamw, literal32=literal32)
                assert (p[e], m[e], v[e]) == (one[1][0], one[2][0], one[3][0]), (rank, e, literal32)
            # and the mask is visible: decayed and exempt elements moved differently
            if not literal32:
                want, _, _ = _textbook_adam(sc * g.astype(np.float64), p0, m0, v0, lr=float(f(hp["lr"])),
                                            b1=float(f(0.9)), b2=float(f(0.999)), eps=float(f(1e-8)),
                                            wd=np.where(exempt[ob:ob + ol], 0.0, float(f(hp["weight_decay"]))), t=3,
                                            adamw=adamw)
                assert np.allclose(p, want, rtol=0, atol=1e-6 * (np.abs(p0) + 1e-3))
                wrong, _, _ = _textbook_adam(sc * g.astype(np.float64), p0, m0, v0, lr=float(f(hp["lr"])),
                                             b1=float(f(0.9)), b2=float(f(0.999)), eps=float(f(1e-8)),
                                             wd=float(f(hp["weight_decay"])), t=3, adamw=adamw)
                ex = exempt[ob:ob + ol] & (np.abs(p0) > 0.05)
                if ex.any():
                    assert (np.abs(p[ex] - wrong[ex]) > 1e-6 * np.abs(p0[ex])).all()
            pad = slice(max(0, lay.total - ob), ol)
            if adamw:
                assert not p[pad].any() and not m[pad].any() and not v[pad].any()


# ---- the chunk-layout branch of reduce_shard ----------------------------------------------------
@pytest.mark.parametrize("P,G,strategy", [(4, 2, "IIG"), (4, 2, "III"), (6, 3, "NNN"), (6, 2, "GGG"), (8, 4, "NIG")])
def test_reduce_shard_chunk_layout_brute_force(P, G, strategy):
    """Chunk layout (contributions are arrays over the update range): small integers against the
    direct sum over ranks; random values against a Python loop that adds, element by element in
    numpy float32, in the order the literal message-passing simulation of the reduce-scatter
    delivers them; the sum of squares covers the rank's own chunk only; and the tensor layout on
    the same data gives the same bits."""
    sizes = [41, 0, 7, 130, 1]
    lay = orc.layout(P, G, sizes)
    L, n = lay.L, P * lay.L
    rng = np.random.default_rng(P * 10 + G)
    sched = orc.default_sched(P, G)
    ints = [np.zeros(n, np.float32) for _ in range(P)]
    vals = [np.zeros(n, np.float32) for _ in range(P)]
    for q in range(P):
        ints[q][:lay.total] = rng.integers(-8, 9, lay.total)
        vals[q][:lay.total] = (rng.standard_normal(lay.total) * 10.0 ** rng.integers(-3, 3, lay.total))
    direct = np.sum([a.astype(np.float64) for a in ints], axis=0)
    sim = [a.copy() for a in vals]
    orc.simulate(lay, sched, orc.RS, sim)                  # literal message passing: rank r ends with its chunk reduced
    seen = np.zeros(n, int)
    norm_total = 0.0
    for r in range(P):
        ob, ol = orc.state_range(lay, r, strategy[2])
        g, ss = orc.reduce_shard(lay, strategy, sched, r, [a[ob:ob + ol] for a in ints], "chunk")
        assert (g == direct[ob:ob + ol]).all()
        own = orc.chunk_of_rank(r, P, G) * L
        assert ss == float(np.sum(direct[own:own + L] ** 2))
        norm_total += ss
        seen[ob:ob + ol] += 1
        g, ss = orc.reduce_shard(lay, strategy, sched, r, [a[ob:ob + ol] for a in vals], "chunk")
        for c in range(ob // L, (ob + ol) // L):                   # each chunk as its owner's ring delivers it
            o = orc.owner_of_chunk(c, P, G)
            assert g[c * L - ob:(c + 1) * L - ob].tobytes() == sim[o][c * L:(c + 1) * L].tobytes(), (r, c)
        as_tensors = [[a[off:off + s] for off, s in zip(np.cumsum([0] + sizes[:-1]), sizes)] for a in vals]
        gt, sst = orc.reduce_shard(lay, strategy, sched, r, as_tensors, "tensors")
        assert gt.tobytes() == g.tobytes() and sst == ss
    assert (seen == {"G": 1, "I": P // G, "N": P}[strategy[2]]).all()
    assert norm_total == float(np.sum(direct ** 2))


def test_range_sumsq_is_the_exact_sum_over_the_update_range():
    """The norm the fused step forms on one rank: all of the rank's update range, against math.fsum;
    equal to reduce_shard's own-chunk value exactly where the range is one chunk."""
    import math
    P, G = 6, 3
    lay = orc.layout(P, G, [1000, 37, 4000])
    rng = np.random.default_rng(3)
    for strategy in ("GGG", "IIG", "III", "NNI", "NNN"):
        for rank in (0, 4):
            ob, ol = orc.state_range(lay, rank, strategy[2])
            contribs = [(rng.standard_normal(ol) * 1e-2).astype(np.float32) for _ in range(P)]
            g, own = orc.reduce_shard(lay, strategy, orc.default_sched(P, G), rank, contribs, "chunk")
            tot = orc.range_sumsq(lay, strategy, rank, g)
            exact = math.fsum(float(x) * float(x) for x in g)
            assert abs(tot - exact) <= 1e-14 * exact
            if strategy[2] == "G":
                assert tot == own
            else:
                assert tot > own * 1.5


# ---- the tolerance checker itself: planted errors must be caught ------------------------------------
def _one_step(n=20_000, seed=7):
    g = _rand(n, seed, 1e-3)
    p, m, v = _rand(n, seed + 1, 0.02), _rand(n, seed + 2, 1e-4), np.abs(_rand(n, seed + 3, 1e-7))
    p_old, m_old = p.copy(), m.copy()
    sc = 0.0625
    orc.adam(g, p, m, v, sc=sc, lr=f32(1e-4), beta1=f32(0.9), beta2=f32(0.999), eps=f32(1e-8), weight_decay=f32(0.01),
             step=5)
    return dict(p=p, m=m, v=v, p_old=p_old, m_old=m_old, g_hat=sc * g.astype(np.float64))


def _check(r, **over):
    a = dict(r, **over)
    return check_moments_and_params(a["p"], a["m"], a["v"], r["p"], r["m"], r["v"], p_old=r["p_old"], m_old=r["m_old"],
                                    g_hat=r["g_hat"])


@pytest.mark.parametrize("which", ["p", "m", "v"])
def test_tolerance_checker_rejects_3e6_relative_on_ordinary_elements(which):
    """An error of 3e-6 relative on elements where nothing cancels (|result| is of the size of its
    terms) must fail, one element at a time; 0.3e-6 must pass."""
    r = _one_step()
    _check(r)                                              # the reference against itself
    ref = r[which].astype(np.float64)
    if which == "p":        # ordinary: the parameter is far larger than the step it took
        ordinary = np.abs(ref) > 100 * np.abs(ref - r["p_old"])
    elif which == "m":      # ordinary: both terms of the moving average have the result's sign
        ordinary = np.sign(r["m_old"]) == np.sign(r["g_hat"])
    else:
        ordinary = ref > 0
    idx = np.flatnonzero(ordinary)
    assert idx.size > r[which].size // 4
    for k in idx[:: max(1, idx.size // 50)]:
        for sign in (1.0, -1.0):
            bad = r[which].copy()
            bad[k] = f32(ref[k] * (1.0 + sign * 3e-6))
            with pytest.raises(AssertionError):
                _check(r, **{which: bad})
            ok = r[which].copy()
            ok[k] = f32(ref[k] * (1.0 + sign * 0.3e-6))
            _check(r, **{which: ok})
    everywhere = (ref * (1.0 + 3e-6)).astype(np.float32)
    with pytest.raises(AssertionError):
        _check(r, **{which: everywhere})


def test_tolerance_checker_rejects_3_ulp_of_the_packed_value():
    r = _one_step()
    tol_p = _check(r)
    q = orc.bf16_rne(r["p"])
    check_bf16_within_one_ulp(q, q, ref_p=r["p"], tol_p=tol_p)
    ordinary = np.flatnonzero(np.abs(r["p"].astype(np.float64)) > 100 * np.abs(r["p"].astype(np.float64) - r["p_old"]))
    assert ordinary.size > 1000
    for k in ordinary[::200]:
        for d in (3, -3, 2, -2):
            bad = q.copy()
            bad[k] = np.uint16(int(q[k]) + d)
            with pytest.raises(AssertionError):
                check_bf16_within_one_ulp(bad, q, ref_p=r["p"], tol_p=tol_p)
        near = q.copy()
        near[k] = np.uint16(int(q[k]) + 1)
        check_bf16_within_one_ulp(near, q, ref_p=r["p"], tol_p=tol_p)
    # the fp16 format too
    h = orc.f16_rne(r["p"])
    bad = h.copy()
    bad[ordinary[0]] = np.uint16(int(h[ordinary[0]]) + 3)
    with pytest.raises(AssertionError):
        check_bf16_within_one_ulp(bad, h, ref_p=r["p"], tol_p=tol_p, fmt="f16")
