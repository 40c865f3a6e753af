"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

Each test checks oracle/comp_ams_oracle.c against something that is not the oracle:
hand-derived worked examples (tests/golden), brute force on tiny inputs, closed forms,
invariants, and the special case k = d that reduces to vanilla distributed AMSGrad.
"""
import ctypes
import json
import math
import os

import numpy as np
import pytest

from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")
f32 = np.float32


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def brute_topk(x, k):
    """Definition of Top-k with the lower-index tie rule, by Python sorting."""
    mag = [abs(float(v)) for v in x]          # fp32 -> python float is exact, |+-0| = 0
    order = sorted(range(len(x)), key=lambda j: (-mag[j], j))
    return sorted(order[:k])


# ----------------------------------------------------------------------------- Top-k

@pytest.mark.parametrize("seed", range(40))
def test_topk_matches_bruteforce_tiny(seed):
    rng = np.random.default_rng(seed)
    d = int(rng.integers(1, 65))
    k = int(rng.integers(1, d + 1))
    pool = np.array([0.0, -0.0, 1.0, -1.0, 0.5, 2.0, -2.0, 3.5, 1e-40, -1e-40, 1e-45, 7.25, -7.25],
                    dtype=np.float32)
    if seed % 2:
        x = pool[rng.integers(0, pool.size, d)]           # many ties, +-0, denormals
    else:
        x = rng.standard_normal(d).astype(np.float32)
    c, sel = O.topk(x, k)
    want = brute_topk(x, k)
    assert sel.tolist() == want
    mask = np.zeros(d, bool)
    mask[want] = True
    assert np.array_equal(bits(c)[mask], bits(x)[mask])     # kept values are x itself
    assert np.all(bits(c)[~mask] == 0)                      # the rest is +0.0


def test_topk_degenerate_inputs():
    # all equal -> the k lowest indices
    c, sel = O.topk(np.full(17, -3.0, f32), 5)
    assert sel.tolist() == [0, 1, 2, 3, 4]
    # all zero (mixed signs) -> still the k lowest indices, kept value is the signed zero
    x = np.array([0.0, -0.0, 0.0, -0.0], f32)
    c, sel = O.topk(x, 2)
    assert sel.tolist() == [0, 1] and np.array_equal(bits(c), bits([0.0, -0.0, 0.0, 0.0]))
    # k = 1 picks the largest magnitude whatever its sign
    c, sel = O.topk(np.array([1.0, -9.0, 8.0], f32), 1)
    assert sel.tolist() == [1] and c.tolist() == [0.0, -9.0, 0.0]
    # k = d is the identity
    x = np.array([0.5, -0.0, 3.0, 1e-42], f32)
    c, sel = O.topk(x, 4)
    assert sel.tolist() == [0, 1, 2, 3] and np.array_equal(bits(c), bits(x))
    # denormals order correctly and are not flushed
    x = np.array([1, 3, 2, 0], np.uint32).view(f32)        # 1, 3 and 2 denormal ulps
    c, sel = O.topk(x, 2)
    assert sel.tolist() == [1, 2]
    # a tie exactly at rank k: lower index wins
    x = np.array([5.0, 2.0, -2.0, 2.0, 7.0], f32)
    c, sel = O.topk(x, 3)
    assert sel.tolist() == [0, 1, 4]
    # Inf sorts above every finite value
    c, sel = O.topk(np.array([1e38, -np.inf, 3.0], f32), 1)
    assert sel.tolist() == [1]


@pytest.mark.parametrize("seed", range(5))
def test_topk_contraction_and_norm_bound(seed):
    """||C(x)-x||^2 <= (1-k/d)||x||^2 (Appendix A, squared form as for Rand-k) and
    ||C(x)|| <= (1+sqrt(pi))||x|| (Lemma 1's first bound)."""
    rng = np.random.default_rng(100 + seed)
    d = 1000
    k = int(rng.integers(1, d))
    x = (rng.standard_normal(d) * np.exp(rng.uniform(-5, 2, d))).astype(f32)
    c, _ = O.topk(x, k)
    xd, cd = x.astype(np.float64), c.astype(np.float64)
    pi = 1.0 - k / d
    assert np.sum((cd - xd) ** 2) <= pi * np.sum(xd ** 2) * (1 + 1e-12)
    assert np.linalg.norm(cd) <= (1 + math.sqrt(pi)) * np.linalg.norm(xd)


# ----------------------------------------------------------------------------- scaled sign

def test_scaled_sign_golden_example_b():
    g = json.load(open(os.path.join(GOLD, "example_b_scaled_sign.json")))
    x = np.array(g["x"], f32)
    c, s = O.blocksign(x, [0, x.size])
    assert s.tolist() == [g["scale"]]
    assert c.tolist() == g["c"]
    e = x - c
    assert e.tolist() == g["error"]
    assert float(np.abs(c).sum()) == g["l1_c"] == g["l1_x"]
    assert float((e.astype(np.float64) ** 2).sum()) == g["err_sq"]
    assert g["err_sq"] == g["x_sq"] - g["l1_x"] ** 2 / x.size        # the appendix identity


@pytest.mark.parametrize("seed", range(6))
def test_scaled_sign_whole_vector_formula_and_identities(seed):
    rng = np.random.default_rng(200 + seed)
    d = int(rng.integers(2, 3000))
    x = rng.laplace(0, 1, d).astype(f32) * np.exp(rng.uniform(-6, 0, d)).astype(f32)
    c, s = O.blocksign(x, [0, d])
    xd = x.astype(np.float64)
    l1 = np.abs(xd).sum()
    # literal definition ||x||_1 sign(x) / d
    want = l1 * np.sign(xd) / d
    assert np.allclose(c.astype(np.float64), want, rtol=2 ** -23, atol=0)
    # every entry has magnitude s  =>  ||C(x)||_1 = d*s = ||x||_1
    assert np.all(np.abs(c) == s[0])
    assert abs(d * float(s[0]) - l1) <= 1e-6 * l1
    # ||C(x)-x||^2 = ||x||^2 - ||x||_1^2/d = (1 - ||x||_1^2/(d||x||^2)) ||x||^2
    err = np.sum((c.astype(np.float64) - xd) ** 2)
    closed = np.sum(xd ** 2) - l1 ** 2 / d
    assert abs(err - closed) <= 1e-5 * np.sum(xd ** 2)
    pi = 1 - l1 ** 2 / (d * np.sum(xd ** 2))
    assert np.linalg.norm(c.astype(np.float64)) <= (1 + math.sqrt(pi)) * np.linalg.norm(xd) * (1 + 1e-6)


def test_scaled_sign_blocks_partial_tail_and_zero_sign():
    x = np.array([1, -3, 2, 2, -0.0, 0.0, 8], f32)
    # blocks [0,2) [2,4) [4,6) [6,7): every block uses its own length as divisor
    c, s = O.blocksign(x, [0, 2, 4, 6, 7])
    assert s.tolist() == [2.0, 2.0, 0.0, 8.0]
    assert np.array_equal(bits(c), bits([2, -2, 2, 2, -0.0, 0.0, 8]))   # sign = IEEE sign bit
    # per-block L1 norm is preserved
    for lo, hi in [(0, 2), (2, 4), (4, 6), (6, 7)]:
        assert np.abs(c[lo:hi]).sum() == np.abs(x[lo:hi]).sum()
    # an all-(-0) block with a non-zero neighbour: -0 takes -s
    c, s = O.blocksign(np.array([-0.0, 4.0], f32), [0, 2])
    assert c.tolist() == [-2.0, 2.0] and math.copysign(1, c[0]) == -1


def test_uniform_blocks_of_create_clip_and_partial_last():
    d, n = 10, 1
    x = np.arange(1, 11, dtype=f32)[None, :]
    o = O.Oracle(d, n, O.BLOCKSIGN, 4, 0.9, 0.999, 1e-8, 1e-3)
    o.step(x)
    assert o.n_blocks == 3
    assert o.scales[0].tolist() == [2.5, 6.5, 9.5]          # (1+2+3+4)/4, (5..8)/4, (9+10)/2
    o.close()
    o = O.Oracle(d, n, O.BLOCKSIGN, 64, 0.9, 0.999, 1e-8, 1e-3)     # block longer than d
    o.step(x)
    assert o.n_blocks == 1 and o.scales[0].tolist() == [5.5]
    o.close()


# ----------------------------------------------------------------------------- AMSGrad

def test_amsgrad_constant_gradient_closed_form():
    """With gbar = c at every step the recursions have closed forms:
    m_t = c(1-beta1^t), v_t = c^2(1-beta2^t) (increasing, so vhat_t = v_t)."""
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    cvals = np.array([0.3, -2.0, 1e-3, 0.0], np.float64)
    d = cvals.size
    th, m, v, vh = (np.zeros(d, f32) for _ in range(4))
    th[:] = 1.0
    want_th = np.ones(d)
    for t in range(1, 201):
        th, m, v, vh = O.amsgrad(th, m, v, vh, cvals.astype(f32), b1, b2, eps, lr, 0)
        mt = cvals * (1 - b1 ** t)
        vt = cvals ** 2 * (1 - b2 ** t)
        want_th = want_th - lr * mt / (np.sqrt(vt) + eps)
        if t in (1, 2, 10, 200):
            assert np.allclose(m, mt, rtol=2e-5, atol=0)
            assert np.allclose(v, vt, rtol=2e-5, atol=0)
            assert np.array_equal(vh, v)
            assert np.allclose(th, want_th, rtol=2e-5, atol=0)
    # sign: a positive gradient moves theta down, a negative one up, zero leaves it alone
    assert th[0] < 1 and th[1] > 1 and th[3] == 1.0


def test_amsgrad_vhat_keeps_the_running_max():
    b1, b2 = 0.5, 0.5
    th, m, v, vh = (np.zeros(1, f32) for _ in range(4))
    seq = [4.0, 0.0, 0.0, 1.0]
    vs, vhs = [], []
    for g in seq:
        th, m, v, vh = O.amsgrad(th, m, v, vh, np.array([g], f32), b1, b2, 0.25, 1.0, 0)
        vs.append(float(v[0]))
        vhs.append(float(vh[0]))
    assert vs == [8.0, 4.0, 2.0, 1.5]                 # v decays
    assert vhs == [8.0, 8.0, 8.0, 8.0]                # vhat does not


def test_amsgrad_eps_placement_modes():
    """mode 0: m/(sqrt(vhat)+eps); mode 1 (the paper's Vhat = diag(vhat+nu)): m/sqrt(vhat+eps).
    Checked against fp64 where vhat ~ eps, where the two differ by a large factor."""
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    g = np.array([1e-3, 1e-5, 3e-2, -1e-4], f32)
    z = np.zeros(4, f32)
    gd = g.astype(np.float64)
    md, vd = (1 - b1) * gd, (1 - b2) * gd ** 2
    th0, *_ = O.amsgrad(z, z, z, z, g, b1, b2, eps, lr, 0)
    th1, *_ = O.amsgrad(z, z, z, z, g, b1, b2, eps, lr, 1)
    assert np.allclose(th0, -lr * md / (np.sqrt(vd) + eps), rtol=1e-5, atol=0)
    assert np.allclose(th1, -lr * md / np.sqrt(vd + eps), rtol=1e-5, atol=0)
    assert abs(th0[1] / th1[1]) > 100            # materially different where vhat << eps


# ----------------------------------------------------------------------------- whole step

def test_golden_example_a_two_steps():
    gold = json.load(open(os.path.join(GOLD, "example_a_topk_ef_amsgrad.json")))
    g = np.array(gold["grads_every_step"], f32)
    for mode in (0, 1):
        o = O.Oracle(gold["d"], gold["n"], O.TOPK, gold["k"], gold["beta1"], gold["beta2"], gold["eps"],
                     gold["lr"])
        o.set_theta(np.array(gold["theta0"], f32))
        o.set_eps_mode(mode)
        for t, want in enumerate(gold["steps"]):
            o.step(g)
            assert o.selected.tolist() == want["selected"]
            assert np.array_equal(bits(o.error), bits(want["error"]))     # incl. +0.0 where selected
            assert o.gbar.tolist() == want["gbar"]
            assert o.m.tolist() == want["m"]
            assert o.v.tolist() == want["v"]
            assert o.vhat.tolist() == want["vhat"]
            key = f"theta_mode{mode}"
            if key in want:
                assert np.allclose(o.theta, want[key], rtol=3e-7, atol=0)
        o.close()


def vanilla_amsgrad_numpy(theta0, grads_by_step, b1, b2, eps, lr):
    """Independent vanilla distributed AMSGrad (Section 3): gbar = (1/n) sum_i g_i with
    fp32 adds in worker order, then the recursion, one fp32 rounding per operation."""
    b1, b2, eps, lr = f32(b1), f32(b2), f32(eps), f32(lr)
    omb1, omb2 = f32(1) - b1, f32(1) - b2
    th = theta0.astype(f32).copy()
    m = np.zeros_like(th)
    v = np.zeros_like(th)
    vh = np.zeros_like(th)
    for g in grads_by_step:
        acc = np.zeros_like(th)
        for i in range(g.shape[0]):
            acc = acc + g[i]
        gb = acc / f32(g.shape[0])
        m = b1 * m + omb1 * gb
        v = b2 * v + omb2 * (gb * gb)
        vh = np.maximum(vh, v)
        th = th - (lr * m) / (np.sqrt(vh) + eps)
    return th, m, v, vh


def test_topk_with_k_equal_d_is_vanilla_amsgrad_bit_for_bit():
    rng = np.random.default_rng(7)
    n, d, T = 5, 777, 12
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gs = [(rng.standard_normal((n, d)) * np.exp(rng.uniform(-6, 0, d))).astype(f32) for _ in range(T)]
    o = O.Oracle(d, n, O.TOPK, d, b1, b2, eps, lr)
    o.set_theta(theta0)
    for g in gs:
        o.step(g)
        assert not o.error.any()                       # pi = 0: nothing is left behind
    th, m, v, vh = vanilla_amsgrad_numpy(theta0, gs, b1, b2, eps, lr)
    assert np.array_equal(bits(o.theta), bits(th))
    assert np.array_equal(bits(o.m), bits(m))
    assert np.array_equal(bits(o.v), bits(v))
    assert np.array_equal(bits(o.vhat), bits(vh))
    o.close()


def test_average_order_and_divisor():
    # ascending-worker fp32 accumulation: ((1e8 + 1) - 1e8) = 0 in fp32, any other order gives 1
    g = np.array([[1e8], [1.0], [-1e8]], f32)
    o = O.Oracle(1, 3, O.TOPK, 1, 0.9, 0.999, 1e-8, 1e-3)
    o.step(g)
    assert o.gbar.tolist() == [0.0]
    o.close()
    # the divisor is n even where a single worker contributed
    g = np.array([[8.0, 1.0], [1.0, 2.0], [1.0, 1.0], [1.0, 1.0]], f32)
    o = O.Oracle(2, 4, O.TOPK, 1, 0.9, 0.999, 1e-8, 1e-3)
    o.step(g)
    assert o.selected.tolist() == [[0], [1], [0], [0]]
    assert o.gbar.tolist() == [(8.0 + 1.0 + 1.0) / 4, 2.0 / 4]
    o.close()


@pytest.mark.parametrize("comp", [O.TOPK, O.BLOCKSIGN])
def test_error_feedback_bookkeeping_monotone_vhat_and_telescoping(comp):
    rng = np.random.default_rng(11 + comp)
    n, d, T = 3, 500, 8
    kb = 7 if comp == O.TOPK else 64
    o = O.Oracle(d, n, comp, kb, 0.9, 0.999, 1e-8, 1e-3)
    e_prev = np.zeros((n, d), f32)
    vhat_prev = np.zeros(d, f32)
    sum_g = np.zeros((n, d))
    sum_c = np.zeros((n, d))
    for t in range(T):
        g = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-4, 0, d))).astype(f32)
        o.step(g)
        x = g + e_prev                                   # one fp32 add
        c, e = o.compressed.copy(), o.error.copy()
        if comp == O.TOPK:
            # e_new + C(x) == x exactly: one of the two is always zero
            assert np.array_equal(e + c, x)
            assert np.all((c != 0).sum(axis=1) <= kb)
            for i in range(n):
                assert o.selected[i].tolist() == brute_topk(x[i], kb)
        else:
            assert np.array_equal(bits(e), bits(x - c))   # delta = fl(x - C(x))
            ulp = np.spacing(np.maximum(np.abs(x), np.abs(c)))
            assert np.all(np.abs((e + c) - x) <= ulp)
            # per-block L1 norm preserved (up to the one rounding of the scale)
            nb = o.n_blocks
            for i in range(n):
                for b in range(nb):
                    lo, hi = b * kb, min((b + 1) * kb, d)
                    l1 = np.abs(x[i, lo:hi].astype(np.float64)).sum()
                    assert abs(np.abs(c[i, lo:hi].astype(np.float64)).sum() - l1) <= 1e-6 * l1
        # average: fp32, ascending workers, divided by n
        acc = np.zeros(d, f32)
        for i in range(n):
            acc = acc + c[i]
        assert np.array_equal(bits(o.gbar), bits(acc / f32(n)))
        # vhat is monotone and dominates v
        assert np.all(o.vhat >= vhat_prev) and np.all(o.vhat >= o.v)
        vhat_prev = o.vhat.copy()
        e_prev = e
        sum_g += g
        sum_c += c
    # telescoping of delta_t = g_t + delta_{t-1} - ghat_t :  sum_t ghat_t + delta_T = sum_t g_t
    assert np.allclose(sum_c + e_prev, sum_g, rtol=0, atol=1e-5 * np.abs(sum_g).max())
    o.close()


def test_result_does_not_depend_on_thread_count():
    gomp = ctypes.CDLL("libgomp.so.1")
    rng = np.random.default_rng(3)
    n, d = 6, 3000
    g = [rng.standard_normal((n, d)).astype(f32) for _ in range(3)]
    outs = []
    for threads in (1, 5):
        gomp.omp_set_num_threads(threads)
        o = O.Oracle(d, n, O.TOPK, 30, 0.9, 0.999, 1e-8, 1e-3)
        for gi in g:
            o.step(gi)
        outs.append((o.theta.copy(), o.error.copy(), o.selected.copy()))
        o.close()
    gomp.omp_set_num_threads(os.cpu_count() or 1)
    for a, b in zip(*outs):
        assert np.array_equal(bits(a) if a.dtype == f32 else a, bits(b) if b.dtype == f32 else b)


# ----------------------------------------------------------------------------- per-layer tables, step-size schedule

def scaled_sign_by_definition(x, offsets):
    """Appendix A's scaled sign on each block with the block's own length as divisor, written out
    with Python floats (exact sums of fp32 values via math.fsum, one rounding to fp32)."""
    c = np.empty_like(x)
    s = np.empty(len(offsets) - 1, f32)
    for b in range(len(offsets) - 1):
        lo, hi = int(offsets[b]), int(offsets[b + 1])
        s[b] = f32(math.fsum(abs(float(v)) for v in x[lo:hi]) / (hi - lo))
        c[lo:hi] = np.copysign(s[b], x[lo:hi])
    return c, s


def test_layer_table_hand_example_in_the_stateful_optimiser():
    """oracle_set_blocks: the table replaces the uniform blocks of create.  Hand example (tests/golden/example_e...:
    Appendix A's scaled sign per block; under error feedback the second step compresses g + e with the same table)."""
    ex = json.load(open(os.path.join(GOLD, "example_e_layer_table_scaled_sign.json")))
    g = np.array([ex["g_every_step"]], f32)
    o = O.Oracle(ex["d"], ex["n"], O.BLOCKSIGN, 3, 0.9, 0.999, 1e-8, 1e-3)       # create says blocks of 3 ...
    o.set_blocks(ex["offsets"])                                                    # ... the table says otherwise
    assert o.n_blocks == len(ex["offsets"]) - 1
    for t, want in enumerate(ex["steps"]):
        o.step(g)
        assert o.scales[0].tolist() == want["scales"], t
        assert np.array_equal(bits(o.compressed[0]), bits(want["compressed"])), t
        assert np.array_equal(bits(o.error[0]), bits(want["error"])), t          # x - C(x)
    o.close()


@pytest.mark.parametrize("method", [O.EF, O.CD, O.NAIVE])
def test_layer_table_in_every_method_matches_the_definition_per_worker_and_step(method):
    """The stateful optimiser with a per-layer table (blocks of 1 to a few hundred coordinates, not
    aligned to anything) against the definition written out in Python for every worker and step: the
    compressed vector and scales are those of the block-wise scaled sign of g + e (error feedback),
    g - ghat_i and ghat - gtilde (Algorithm 1) or g (naive); the memory follows Section 4 / Algorithm 1;
    a table changed between steps applies from the next step on and leaves the memory as it is."""
    rng = np.random.default_rng(23 + method)
    n, d, T = 3, 613, 6
    tables = [np.array([0, 1, 2, 66, 67, 300, 301, 555, 613]), np.array([0, 200, 613])]
    o = O.Oracle(d, n, O.BLOCKSIGN, 64, 0.9, 0.999, 1e-8, 1e-3, method=method)
    o.set_blocks(tables[0])
    mem = np.zeros((n, d), f32)                 # e_i, or ghat_i for Algorithm 1
    ghat_s = np.zeros(d, f32)
    gtil = np.zeros(d, f32)
    for t in range(T):
        off = tables[0] if t < 4 else tables[1]
        if t == 4:
            o.set_blocks(off)
        g = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-5, 0, d))).astype(f32)
        g[0, 66] = 0.0
        o.step(g)
        assert o.n_blocks == off.size - 1
        x = g + mem if method == O.EF else g - mem if method == O.CD else g
        acc = np.zeros(d, f32)
        for i in range(n):
            c, s = scaled_sign_by_definition(x[i], off)
            assert np.array_equal(bits(o.compressed[i]), bits(c)), (t, i)
            assert np.array_equal(bits(o.scales[i]), bits(s)), (t, i)
            # per-block L1 norm is preserved with the block's own length as divisor
            for b in range(off.size - 1):
                l1 = np.abs(x[i, off[b]:off[b + 1]].astype(np.float64)).sum()
                assert abs(float(s[b]) * (off[b + 1] - off[b]) - l1) <= 1e-6 * l1
            if method == O.EF:
                mem[i] = x[i] - c
                assert np.array_equal(bits(o.error[i]), bits(mem[i])), (t, i)
            elif method == O.CD:
                mem[i] = mem[i] + c
                assert np.array_equal(bits(o.ghat_workers[i]), bits(mem[i])), (t, i)
            acc = acc + c
        gbar = acc / f32(n)
        assert np.array_equal(bits(o.gbar), bits(gbar))
        if method == O.CD:
            ghat_s = ghat_s + gbar
            cs, ss = scaled_sign_by_definition(ghat_s - gtil, off)
            gtil = gtil + cs
            assert np.array_equal(bits(o.server_scales), bits(ss)), t
            assert np.array_equal(bits(o.server_compressed), bits(cs)), t
            assert np.array_equal(bits(o.ghat_server), bits(ghat_s)), t
            assert np.array_equal(bits(o.gtilde), bits(gtil)), t
    o.close()


def test_step_size_schedule_matches_independent_amsgrad():
    """oracle_set_lr: Algorithm 1 takes a non-increasing sequence alpha_t.  With no compression the
    optimiser is vanilla distributed AMSGrad (Section 3); changing the step size between steps must
    give, bit for bit, an independent numpy recursion that uses alpha_t at step t - and m, v, vhat
    must not depend on the schedule at all."""
    rng = np.random.default_rng(29)
    n, d, T = 4, 400, 12
    b1, b2, eps = f32(0.9), f32(0.999), f32(1e-8)
    omb1, omb2 = f32(1) - b1, f32(1) - b2
    sched = [f32(1e-2 / math.sqrt(t + 1)) for t in range(T)]          # non-increasing
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gs = [(rng.standard_normal((n, d)) * np.exp(rng.uniform(-6, 0, d))).astype(f32) for _ in range(T)]
    th, m, v, vh = theta0.copy(), np.zeros(d, f32), np.zeros(d, f32), np.zeros(d, f32)
    o = O.Oracle(d, n, O.TOPK, d, float(b1), float(b2), float(eps), 123.0, method=O.NONE)   # lr of create is never used
    o.set_theta(theta0)
    fixed = O.Oracle(d, n, O.TOPK, d, float(b1), float(b2), float(eps), float(sched[0]), method=O.NONE)
    fixed.set_theta(theta0)
    for t, g in enumerate(gs):
        o.set_lr(float(sched[t]))
        o.step(g)
        fixed.step(g)
        acc = np.zeros(d, f32)
        for i in range(n):
            acc = acc + g[i]
        gb = acc / f32(n)
        m = b1 * m + omb1 * gb
        v = b2 * v + omb2 * (gb * gb)
        vh = np.maximum(vh, v)
        th = th - (sched[t] * m) / (np.sqrt(vh) + eps)
        assert np.array_equal(bits(o.theta), bits(th)), t
        assert np.array_equal(bits(o.m), bits(m)) and np.array_equal(bits(o.v), bits(v))
        assert np.array_equal(bits(o.vhat), bits(vh))
        assert np.array_equal(bits(fixed.m), bits(m)) and np.array_equal(bits(fixed.vhat), bits(vh))
        if t == 0:
            assert np.array_equal(bits(fixed.theta), bits(th))        # same alpha_1 ...
        else:
            assert not np.array_equal(bits(fixed.theta), bits(th))    # ... a constant step size differs later
    o.close()
    fixed.close()


def test_step_size_schedule_under_error_feedback_leaves_compression_alone():
    """alpha_t enters the last line of the update only: under error feedback the kept sets, the error
    memory, m, v and vhat are those of a constant step size; theta moves by alpha_t * m / denominator."""
    rng = np.random.default_rng(31)
    n, d, T = 3, 257, 6
    gs = [rng.standard_normal((n, d)).astype(f32) for _ in range(T)]
    a = O.Oracle(d, n, O.TOPK, 9, 0.9, 0.999, 1e-8, 1e-3)
    b = O.Oracle(d, n, O.TOPK, 9, 0.9, 0.999, 1e-8, 1e-3)
    for t, g in enumerate(gs):
        th_before = b.theta.copy()
        b.set_lr(1e-3 / (t + 1))
        a.step(g)
        b.step(g)
        assert np.array_equal(a.selected, b.selected) and np.array_equal(bits(a.error), bits(b.error))
        assert np.array_equal(bits(a.m), bits(b.m)) and np.array_equal(bits(a.vhat), bits(b.vhat))
        want = th_before - (f32(1e-3 / (t + 1)) * b.m) / (np.sqrt(b.vhat) + f32(1e-8))
        assert np.array_equal(bits(b.theta), bits(want)), t
    a.close()
    b.close()


# ----------------------------------------------------------------------------- CD-Adam (Algorithm 1)

def test_cd_adam_golden_example_c_topk():
    ex = json.load(open(os.path.join(GOLD, "example_c_cd_adam_topk.json")))
    g = np.array(ex["g"], f32)
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    o = O.Oracle(ex["d"], ex["n"], O.TOPK, ex["k"], b1, b2, eps, lr, method=O.CD)
    o.set_eps_mode(1)
    th, m, v, vh = (np.zeros(ex["d"], f32) for _ in range(4))
    for t, want in enumerate(ex["steps"]):
        o.step(g)
        assert np.array_equal(bits(o.compressed), bits(np.array(want["c_workers"], f32))), t
        assert np.array_equal(bits(o.ghat_workers), bits(np.array(want["ghat_workers"], f32))), t
        assert np.array_equal(bits(o.ghat_server), bits(np.array(want["ghat_server"], f32))), t
        assert o.server_selected.tolist() == want["server_selected"], t
        assert np.array_equal(bits(o.server_compressed), bits(np.array(want["c_server"], f32))), t
        assert np.array_equal(bits(o.gtilde), bits(np.array(want["gtilde"], f32))), t
        # the model update is AMSGrad (pinned on its own above) fed with gtilde
        th, m, v, vh = O.amsgrad(th, m, v, vh, np.array(want["gtilde"], f32), b1, b2, eps, lr, eps_mode=1)
        assert np.array_equal(bits(o.theta), bits(th)) and np.array_equal(bits(o.vhat), bits(vh))
    o.close()


def test_cd_adam_golden_example_d_scaled_sign():
    ex = json.load(open(os.path.join(GOLD, "example_d_cd_adam_scaled_sign.json")))
    g = np.array(ex["g"], f32)
    o = O.Oracle(ex["d"], ex["n"], O.BLOCKSIGN, ex["d"], 0.9, 0.999, 1e-8, 1e-3, method=O.CD)
    for t, want in enumerate(ex["steps"]):
        o.step(g)
        assert o.scales[:, 0].tolist() == want["scales_workers"], t
        assert np.array_equal(bits(o.ghat_workers), bits(np.array(want["ghat_workers"], f32))), t
        assert np.array_equal(bits(o.ghat_server), bits(np.array(want["ghat_server"], f32))), t
        assert o.server_scales.tolist() == [want["scale_server"]], t
        assert np.array_equal(bits(o.gtilde), bits(np.array(want["gtilde"], f32))), t
    o.close()


def test_cd_adam_with_k_equal_d_is_vanilla_amsgrad_bit_for_bit():
    """pi = 0: C is the identity, so ghat_i = g_i, ghat = gtilde = mean g (Algorithm 1 reduces to the
    vanilla distributed AMSGrad of Section 3).  Integer gradients and n = 4 keep every sum and
    difference exact, so the identity holds bit for bit against an independent numpy AMSGrad."""
    rng = np.random.default_rng(17)
    n, d, T = 4, 300, 10
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gs = [rng.integers(-50, 51, (n, d)).astype(f32) for _ in range(T)]
    o = O.Oracle(d, n, O.TOPK, d, b1, b2, eps, lr, method=O.CD)
    o.set_theta(theta0)
    for g in gs:
        o.step(g)
        assert np.array_equal(bits(o.ghat_workers), bits(g))
        assert np.array_equal(bits(o.gtilde), bits(g.sum(axis=0, dtype=np.float64).astype(f32) / f32(n)))
    th, m, v, vh = vanilla_amsgrad_numpy(theta0, gs, b1, b2, eps, lr)
    assert np.array_equal(bits(o.theta), bits(th))
    assert np.array_equal(bits(o.vhat), bits(vh))
    o.close()


def test_cd_adam_constant_gradients_are_recovered_in_finitely_many_steps():
    """Markov compression of a constant sequence with Top-k: every step makes k more coordinates of
    ghat_i exact (0 + (g - 0) = g) and they stay exact, so after ceil(d/k) steps ghat_i = g_i and the
    workers send zeros; the server's gtilde then reaches mean_i g_i the same way."""
    rng = np.random.default_rng(23)
    n, d, k = 4, 40, 7
    g = rng.integers(-64, 65, (n, d)).astype(f32)
    g[g == 0] = 1.0
    o = O.Oracle(d, n, O.TOPK, k, 0.9, 0.999, 1e-8, 1e-3, method=O.CD)
    need = math.ceil(d / k)
    for t in range(need):
        o.step(g)
        # exactly k*(t+1) coordinates are exact so far (none of g is 0, so exact means != 0 here)
        assert np.count_nonzero(o.ghat_workers, axis=1).tolist() == [min(d, k * (t + 1))] * n
    assert np.array_equal(bits(o.ghat_workers), bits(g))
    mean = g.sum(axis=0) / f32(n)                               # exact: integers, n = 4
    assert np.array_equal(bits(o.ghat_server), bits(mean))
    for t in range(need):
        o.step(g)
        assert not o.compressed.any()                           # workers have nothing left to send
    assert np.array_equal(bits(o.gtilde), bits(mean))
    o.close()


@pytest.mark.parametrize("comp", [O.TOPK, O.BLOCKSIGN])
def test_cd_adam_markov_bookkeeping_and_contraction(comp):
    """Per step and worker (Algorithm 1 lines 5-6, Assumption 1 with the compressor's own pi):
    ghat_i(t) - ghat_i(t-1) = c_i(t);  ||ghat_i(t) - g_i(t)||^2 <= pi ||g_i(t) - ghat_i(t-1)||^2 with
    pi = 1 - k/d (Top-k), and = ||u||^2 - ||u||_1^2 / |b| per block for the scaled sign (its error
    identity, Appendix A).  Server (lines 8-10): ghat(t) = mean_i ghat_i(t) up to rounding; gtilde moves
    by the server's message; vhat never decreases."""
    rng = np.random.default_rng(29 + comp)
    n, d, T = 3, 600, 8
    kb = 9 if comp == O.TOPK else 64
    o = O.Oracle(d, n, comp, kb, 0.9, 0.999, 1e-8, 1e-3, method=O.CD)
    off = np.array(list(range(0, d, 64)) + [d])
    prev_w = np.zeros((n, d), f32)
    prev_t = np.zeros(d, f32)
    prev_vh = np.zeros(d, f32)
    for t in range(T):
        g = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-4, 0, d)) + 0.3).astype(f32)
        o.step(g)
        gw, c = o.ghat_workers.copy(), o.compressed.copy()
        assert np.array_equal(bits(gw), bits(prev_w + c))
        u = g.astype(np.float64) - prev_w
        left = ((gw.astype(np.float64) - g) ** 2)
        if comp == O.TOPK:
            assert np.count_nonzero(c, axis=1).max() <= kb
            assert (left.sum(axis=1) <= (1 - kb / d) * (u ** 2).sum(axis=1) * (1 + 1e-6)).all()
        else:
            for b in range(off.size - 1):
                ub = u[:, off[b]:off[b + 1]]
                want = (ub ** 2).sum(axis=1) - np.abs(ub).sum(axis=1) ** 2 / ub.shape[1]
                got = left[:, off[b]:off[b + 1]].sum(axis=1)
                assert np.allclose(got, want, rtol=1e-4, atol=1e-9)
        assert np.allclose(o.ghat_server, gw.astype(np.float64).mean(axis=0), rtol=1e-5, atol=1e-6)
        assert np.array_equal(bits(o.gtilde), bits(prev_t + o.server_compressed))
        assert (o.vhat >= prev_vh).all()
        prev_w, prev_t, prev_vh = gw, o.gtilde.copy(), o.vhat.copy()
    o.close()


# ----------------------------------------------------------------------------- comparison arms (Section 3, Section 4)

def test_uncompressed_method_is_vanilla_distributed_amsgrad_bit_for_bit():
    rng = np.random.default_rng(31)
    n, d, T = 5, 400, 9
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gs = [(rng.standard_normal((n, d)) * np.exp(rng.uniform(-5, 0, d))).astype(f32) for _ in range(T)]
    for comp, kb in ((O.TOPK, 3), (O.BLOCKSIGN, 50)):          # the compressor must not matter
        o = O.Oracle(d, n, comp, kb, b1, b2, eps, lr, method=O.NONE)
        o.set_theta(theta0)
        for g in gs:
            o.step(g)
        th, m, v, vh = vanilla_amsgrad_numpy(theta0, gs, b1, b2, eps, lr)
        assert np.array_equal(bits(o.theta), bits(th)) and np.array_equal(bits(o.m), bits(m))
        assert np.array_equal(bits(o.v), bits(v)) and np.array_equal(bits(o.vhat), bits(vh))
        o.close()


@pytest.mark.parametrize("comp", [O.TOPK, O.BLOCKSIGN])
def test_naive_compression_has_no_memory(comp):
    """Section 4, "Naive compression": ghat_i = C(g_i) every step, whatever came before.  The averaged
    message of step t therefore equals what the (separately pinned) compressor gives on g_t alone,
    averaged in ascending worker order, and the model follows AMSGrad (pinned above) on it; it also
    equals the first step of error feedback, whose memory is still empty."""
    rng = np.random.default_rng(37 + comp)
    n, d, T = 3, 300, 6
    kb = 11 if comp == O.TOPK else 64
    b1, b2, eps, lr = 0.9, 0.999, 1e-8, 1e-3
    off = np.array(list(range(0, d, 64)) + [d])
    o = O.Oracle(d, n, comp, kb, b1, b2, eps, lr, method=O.NAIVE)
    th, m, v, vh = (np.zeros(d, f32) for _ in range(4))
    for t in range(T):
        g = (rng.standard_normal((n, d)) * np.exp(rng.uniform(-4, 0, d))).astype(f32)
        o.step(g)
        c = np.stack([O.topk(g[i], kb)[0] if comp == O.TOPK else O.blocksign(g[i], off)[0] for i in range(n)])
        acc = np.zeros(d, f32)
        for i in range(n):
            acc = acc + c[i]
        gbar = acc / f32(n)
        assert np.array_equal(bits(o.compressed), bits(c)), t
        assert np.array_equal(bits(o.gbar), bits(gbar)), t
        assert not o.error.any()
        th, m, v, vh = O.amsgrad(th, m, v, vh, gbar, b1, b2, eps, lr)
        assert np.array_equal(bits(o.theta), bits(th)) and np.array_equal(bits(o.vhat), bits(vh))
        ef = O.Oracle(d, n, comp, kb, b1, b2, eps, lr)          # first step of error feedback: same message
        ef.step(g)
        assert np.array_equal(bits(ef.gbar), bits(gbar))
        ef.close()
    o.close()


def test_case_study_ordering_of_the_four_strategies():
    """Section 6.1 (nonconvex logistic regression, scaled sign): after the same number of iterations
    CD-Adam's gradient norm is far below error feedback's, which is far below naive compression's,
    and uncompressed AMSGrad is the reference at the bottom.  Synthetic data of the LibSVM sets'
    shape; block-wise scaled sign (16 coordinates per block), nu = 1e-3, step size 0.003."""
    import workloads as W
    a, y = W.logreg_problem()
    n, _, d = a.shape
    norm = {}
    for name, method in (("none", O.NONE), ("cd", O.CD), ("ef", O.EF), ("naive", O.NAIVE)):
        o = O.Oracle(d, n, O.BLOCKSIGN, 16, 0.9, 0.999, 1e-3, 0.003, method=method)
        o.set_eps_mode(1)
        for _ in range(1500):
            o.step(W.logreg_grads(a, y, o.theta))
        norm[name] = float(np.linalg.norm(W.logreg_grads(a, y, o.theta).astype(np.float64).mean(axis=0)))
        o.close()
    assert norm["none"] < 1e-6
    assert norm["cd"] < 1e-2 * norm["ef"], norm
    assert norm["ef"] < 1e-1 * norm["naive"], norm


# ---- Rand-k (Appendix A, "Rand-k") ------------------------------------------------------------
# The paper fixes: S has exactly k elements, C(x) = x on S and 0 elsewhere, S is drawn at random
# (so it cannot depend on x), and E||C(x) - x||^2 = (1 - k/d) ||x||^2 - which holds iff every
# coordinate is in S with probability k/d.  How S is drawn is this build's reading; the generator
# is pinned by an independent transcription of its published building block plus statistics.

def py_mix32(h):
    h &= 0xFFFFFFFF
    h ^= h >> 16
    h = (h * 0x85EBCA6B) & 0xFFFFFFFF
    h ^= h >> 13
    h = (h * 0xC2B2AE35) & 0xFFFFFFFF
    h ^= h >> 16
    return h


def py_unmix32(h):
    """Inverse of the finaliser: undo each xor-shift, multiply by the inverse constants mod 2^32."""
    def unshift(v, s):
        out = v
        for _ in range(32 // s + 1):
            out = v ^ (out >> s)
        return out
    h = unshift(h, 16)
    h = (h * pow(0xC2B2AE35, -1, 1 << 32)) & 0xFFFFFFFF
    h = unshift(h, 13)
    h = (h * pow(0x85EBCA6B, -1, 1 << 32)) & 0xFFFFFFFF
    return unshift(h, 16)


def py_score(seed, draw, who, j):
    M = 0xFFFFFFFF
    per_step = py_mix32(((seed & M) + draw * 0x9E3779B9) & M)
    a = py_mix32(per_step ^ (seed >> 32) ^ ((who * 0x85EBCA6B) & M))
    b = py_mix32((a + 0xC2B2AE35) & M)
    return py_mix32(py_mix32((j + a) & M) ^ b) >> 1


def test_randk_generator_is_the_stated_one_and_a_bijection():
    rng = np.random.default_rng(0)
    words = [0, 1, 2, 0xFFFFFFFF, 0x80000000] + [int(w) for w in rng.integers(0, 1 << 32, 200)]
    for w in words:
        assert O.mix32(w) == py_mix32(w)
        assert py_unmix32(O.mix32(w)) == w               # invertible: distinct words stay distinct
    assert O.mix32(0) == 0 and O.mix32(1) == 0x514E28B7   # the finaliser's fixed point and a known value
    for seed, draw, who, j in [(0, 0, 0, 0), (1, 2, 3, 4), (0xDEADBEEF12345678, 1000, 16, 11_173_961),
                               (2 ** 64 - 1, 2 ** 32 - 1, 2 ** 32 - 1, 2 ** 32 - 1)]:
        assert O.randk_score(seed, draw, who, j) == py_score(seed, draw, who, j)
    # for a fixed draw the scores of all coordinates are distinct before the final shift: at most
    # two coordinates share a 31-bit score
    s = np.array([O.randk_score(5, 9, 2, j) for j in range(20_000)])
    _, counts = np.unique(s, return_counts=True)
    assert counts.max() <= 2


@pytest.mark.parametrize("d,k", [(1, 1), (10, 1), (10, 10), (257, 31), (5000, 50)])
def test_randk_keeps_exactly_k_values_unchanged_and_ignores_the_vector(d, k):
    rng = np.random.default_rng(d + k)
    x = rng.standard_normal(d).astype(f32)
    x[x == 0] = 1.0
    c, sel = O.randk(x, k, 42, 3, 1)
    assert sel.size == k and np.all(np.diff(sel.astype(np.int64)) > 0) and sel.max() < d
    mask = np.zeros(d, bool)
    mask[sel] = True
    assert np.array_equal(bits(c[mask]), bits(x[mask]))
    assert np.array_equal(bits(c[~mask]), np.zeros(d - k, np.uint32))        # +0.0
    # S is the k coordinates of largest score, lower index first among equals (brute force)
    score = [py_score(42, 3, 1, j) for j in range(d)]
    want = sorted(sorted(range(d), key=lambda j: (-score[j], j))[:k])
    assert sel.tolist() == want
    # S does not depend on x: another vector, the same draw
    y = rng.standard_normal(d).astype(f32) * 1e3
    assert np.array_equal(O.randk(y, k, 42, 3, 1)[1], sel)
    # ... and depends on each of seed, draw, who (with d choose k > 1)
    if 1 < k < d and d > 100:
        for other in ((43, 3, 1), (42, 4, 1), (42, 3, 2), (42 + (1 << 32), 3, 1)):
            assert not np.array_equal(O.randk(x, k, *other)[1], sel)


def test_randk_inclusion_is_uniform_and_the_expected_error_is_the_papers():
    """Appendix A, "Rand-k": E||C(x) - x||^2 = (1 - k/d) ||x||^2; every coordinate is kept with
    probability k/d and pairs as in sampling without replacement."""
    d, k, T = 120, 30, 6000
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(d) * np.exp(rng.uniform(-3, 0, d))).astype(f32)
    hits = np.zeros(d)
    pair = 0
    err = 0.0
    for t in range(T):
        c, sel = O.randk(x, k, 2024, t, t % 7)
        hits[sel] += 1
        pair += int(0 in sel and 1 in sel)
        err += float(((c.astype(np.float64) - x) ** 2).sum())
    p = k / d
    # each count is Binomial(T, p): six standard deviations
    assert np.all(np.abs(hits - T * p) <= 6 * math.sqrt(T * p * (1 - p)))
    # chi-square over coordinates: mean d, standard deviation about sqrt(2 d) (slightly less: the counts sum to T k)
    chi = ((hits - T * p) ** 2 / (T * p * (1 - p))).sum()
    assert chi < d + 6 * math.sqrt(2 * d)
    pp = k * (k - 1) / (d * (d - 1))
    assert abs(pair - T * pp) <= 6 * math.sqrt(T * pp * (1 - pp))
    want = (1 - p) * float((x.astype(np.float64) ** 2).sum())
    assert abs(err / T - want) <= 0.02 * want


def test_topk_error_never_exceeds_randk_error():
    """Appendix A: ||C_top(x) - x|| <= ||C_rand(x) - x|| for every draw of S."""
    rng = np.random.default_rng(2)
    for t in range(50):
        d = int(rng.integers(2, 400))
        k = int(rng.integers(1, d + 1))
        x = rng.standard_normal(d).astype(f32)
        ct, _ = O.topk(x, k)
        cr, _ = O.randk(x, k, 9, t, 0)
        assert np.linalg.norm(ct.astype(np.float64) - x) <= np.linalg.norm(cr.astype(np.float64) - x)


@pytest.mark.parametrize("method", [O.EF, O.NAIVE, O.CD])
def test_randk_inside_the_methods_draws_per_step_and_worker(method):
    """The optimiser uses draw = number of steps taken and who = worker index (n for the server of
    Algorithm 1); the bookkeeping identities of each method hold with the random selection."""
    rng = np.random.default_rng(5 + method)
    n, d, k, T = 3, 400, 40, 6
    o = O.Oracle(d, n, O.RANDK, k, 0.9, 0.999, 1e-8, 1e-3, method=method)
    o.set_rand(77, 0)
    e_prev = np.zeros((n, d), f32)
    gh_prev = np.zeros((n, d), f32)
    ghs_prev = np.zeros(d, f32)
    gt_prev = np.zeros(d, f32)
    for t in range(T):
        g = rng.standard_normal((n, d)).astype(f32)
        o.step(g)
        for i in range(n):
            x = {O.EF: g[i] + e_prev[i], O.NAIVE: g[i], O.CD: g[i] - gh_prev[i]}[method]
            c, sel = O.randk(x, k, 77, t, i)
            assert np.array_equal(o.selected[i], sel), (t, i)
            assert np.array_equal(bits(o.compressed[i]), bits(c))
            if method == O.EF:
                assert np.array_equal(o.error[i] + c, x)              # one of the two is always zero
            elif method == O.NAIVE:
                assert not o.error[i].any()
            else:
                assert np.array_equal(bits(o.ghat_workers[i]), bits(gh_prev[i] + c))
        if method == O.CD:
            w = o.ghat_server - gt_prev
            acc = np.zeros(d, f32)
            for i in range(n):
                acc = acc + o.compressed[i]
            assert np.array_equal(bits(o.ghat_server), bits(ghs_prev + acc / f32(n)))
            cs, sels = O.randk(w, k, 77, t, n)
            assert np.array_equal(o.server_selected, sels)
            assert np.array_equal(bits(o.gtilde), bits(gt_prev + cs))
            gh_prev = o.ghat_workers.copy()
            ghs_prev = o.ghat_server.copy()
            gt_prev = o.gtilde.copy()
        e_prev = o.error.copy()
    o.close()


def test_randk_resumes_from_a_given_draw_and_k_equal_d_is_vanilla():
    rng = np.random.default_rng(8)
    n, d, k = 2, 300, 30
    gs = [rng.standard_normal((n, d)).astype(f32) for _ in range(5)]
    a = O.Oracle(d, n, O.RANDK, k, 0.9, 0.999, 1e-8, 1e-3)
    a.set_rand(5, 0)
    for g in gs:
        a.step(g)
    b = O.Oracle(d, n, O.RANDK, k, 0.9, 0.999, 1e-8, 1e-3)
    b.set_rand(5, 4)                       # only the last step, with the draw it had in the full run
    b.step(gs[4])
    # same kept sets at that draw, whatever the vectors were
    assert np.array_equal(a.selected, b.selected)
    a.close(); b.close()
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    o = O.Oracle(d, n, O.RANDK, d, 0.9, 0.999, 1e-8, 1e-3)
    o.set_rand(1, 0)
    o.set_theta(theta0)
    for g in gs:
        o.step(g)
        assert not o.error.any()
    th, m, v, vh = vanilla_amsgrad_numpy(theta0, gs, 0.9, 0.999, 1e-8, 1e-3)
    assert np.array_equal(bits(o.theta), bits(th)) and np.array_equal(bits(o.vhat), bits(vh))
    o.close()
