"""GPU parity of CD-Adam (Section 5, Algorithm 1) with the block-wise scaled sign: the HIP library
through the C ABI against the CPU oracle, element by element, on the same seeded inputs.

Bars: the workers' and the server's block scales within 1e-5 relative (the GPU adds the fp64 piece
sums in a different order than the oracle's index order; a difference needs a sum that sits on an
fp32 rounding boundary).  Where all scales of a run so far are bit-identical - the expected case -
ghat_i, ghat and gtilde must be bit-exact; theta, m, v, vhat within 1e-6 relative per coordinate.
"""
import json
import os

import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import SCALE_RTOL, STATE_RTOL, bits, rel_close

pytestmark = pytest.mark.gpu
f32 = np.float32
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def torch_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def announce(msg):
    print(f"[case] {msg}", flush=True)


def make_cd_pair(d, n, block, theta0=None, offsets=None, eps_mode=1, lr=W.LR):
    gpu = P.CompAms(d, n, P.BLOCKSIGN, block, W.BETA1, W.BETA2, W.EPS, lr)
    ora = O.Oracle(d, n, O.BLOCKSIGN, block, W.BETA1, W.BETA2, W.EPS, lr, method=O.CD)
    gpu.set_method(P.METHOD_CD)
    if offsets is not None:
        gpu.set_blocks(offsets)
        ora.set_blocks(offsets)
    if theta0 is not None:
        gpu.set_theta(np.ascontiguousarray(theta0, dtype=f32))
        ora.set_theta(theta0)
    gpu.set_eps_mode(eps_mode)
    ora.set_eps_mode(eps_mode)
    return gpu, ora


def compare_cd(gpu, ora, tag, exact):
    """exact: every scale so far was bit-identical.  Returns whether that still holds."""
    sw, ss = gpu.get_scales(), gpu.get_server_scales()
    assert rel_close(sw, ora.scales, SCALE_RTOL).all(), f"{tag}: worker scales beyond {SCALE_RTOL}"
    assert rel_close(ss, ora.server_scales, SCALE_RTOL).all(), f"{tag}: server scales beyond {SCALE_RTOL}"
    exact = exact and np.array_equal(bits(sw), bits(ora.scales)) and np.array_equal(bits(ss), bits(ora.server_scales))
    pairs = [(f"ghat_{i}", gpu.get_ghat_worker(i), ora.ghat_workers[i]) for i in range(gpu.n)]
    pairs += [("ghat", gpu.get_ghat_server(), ora.ghat_server), ("gtilde", gpu.get_gtilde(), ora.gtilde)]
    for name, got, want in pairs:
        if exact:
            assert np.array_equal(bits(got), bits(want)), f"{tag} {name}: not bit-identical " \
                f"({np.count_nonzero(bits(got) != bits(want))} coordinates)"
        else:
            assert np.allclose(got, want, rtol=1e-5, atol=1e-5 * float(np.abs(want).max() + 1e-30)), f"{tag} {name}"
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                            ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
        if exact:
            ok = rel_close(got, want, STATE_RTOL)
            assert ok.all(), f"{tag} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL} relative"
        else:
            assert np.allclose(got, want, rtol=1e-4, atol=1e-7), f"{tag} {name}"
    return exact


def run_cd(gpu, ora, grads_fn, steps, tag):
    exact = True
    for t in range(steps):
        g = grads_fn(t)
        gpu.step(torch_dev(g))
        ora.step(g)
        exact = compare_cd(gpu, ora, f"{tag} step {t}", exact)
    return exact


def test_cd_golden_example_d_on_gpu():
    announce("CD-Adam golden example D")
    ex = json.load(open(os.path.join(GOLD, "example_d_cd_adam_scaled_sign.json")))
    g = np.array(ex["g"], f32)
    h = P.CompAms(ex["d"], ex["n"], P.BLOCKSIGN, ex["d"])
    h.set_method(P.METHOD_CD)
    gd = torch_dev(g)
    for t, want in enumerate(ex["steps"]):
        h.step(gd)
        assert h.get_scales()[:, 0].tolist() == want["scales_workers"], t
        for i in range(ex["n"]):
            assert np.array_equal(bits(h.get_ghat_worker(i)), bits(np.array(want["ghat_workers"][i], f32))), (t, i)
        assert np.array_equal(bits(h.get_ghat_server()), bits(np.array(want["ghat_server"], f32))), t
        assert h.get_server_scales().tolist() == [want["scale_server"]], t
        assert np.array_equal(bits(h.get_gtilde()), bits(np.array(want["gtilde"], f32))), t
    h.destroy()


@pytest.mark.parametrize("d,n,B", [(1, 1, 1), (7, 2, 3), (64, 2, 64), (1000, 3, 4096), (4096, 2, 4096),
                                   (4097, 2, 4096), (10_007, 5, 100), (3 * 4096 + 5, 4, 8192), (5_001, 3, 1),
                                   (30_000, 2, 1 << 20)])
def test_cd_uniform_blocks_small_shapes(d, n, B):
    announce(f"CD-Adam uniform blocks d={d} n={n} B={B}")
    rng = np.random.default_rng(d * 13 + n)
    scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    gpu, ora = make_cd_pair(d, n, B, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run_cd(gpu, ora, lambda t: (np.random.default_rng([d, n, t]).standard_normal((n, d)) * scale + 0.1 * scale).astype(f32),
           steps=5, tag=f"d={d}")
    gpu.destroy()


@pytest.mark.parametrize("eps_mode", [0, 1])
def test_cd_layer_blocks_degenerate_values_and_eps_modes(eps_mode):
    announce(f"CD-Adam layer blocks, eps mode {eps_mode}")
    d, n = 70_003, 3
    offsets = [0, 1, 2, 300, 4096, 4097, 9000, 30_000, 30_001, 65_536, d]      # one-element blocks, tile straddlers
    rng = np.random.default_rng(77)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    gpu, ora = make_cd_pair(d, n, d, theta0=(0.01 * rng.standard_normal(d)).astype(f32), offsets=offsets,
                            eps_mode=eps_mode)

    def grads(t):
        g = (np.random.default_rng([77, t]).standard_normal((n, d)) * scale).astype(f32)
        g[:, 300:4096] = 0.0 if t % 2 == 0 else g[:, 300:4096]      # an all-zero block every other step
        g[0, 5000:5100] = -0.0
        return g

    run_cd(gpu, ora, grads, steps=6, tag="layers")
    gpu.destroy()


@pytest.mark.parametrize("idx,d,n", [(1, 150_001, 16), (3, 400_001, 8)])
def test_cd_on_the_block_sign_workloads_scaled(idx, d, n):
    w = W.get(idx).scaled(d, n=n)
    announce(f"CD-Adam on {w.name}")
    s = w.scales()
    off = w.block_offsets() if w.layer_blocks else None
    gpu, ora = make_cd_pair(w.d, w.n, w.block if w.block else w.d, theta0=w.theta0(), offsets=off)
    run_cd(gpu, ora, lambda t: w.grads(t, scales=s), steps=5, tag=w.name)
    gpu.destroy()


def test_cd_many_workers():
    announce("CD-Adam n=70")
    n, d = 70, 20_001
    rng = np.random.default_rng(70)
    gpu, ora = make_cd_pair(d, n, 4096)
    run_cd(gpu, ora, lambda t: np.random.default_rng([70, t]).standard_normal((n, d)).astype(f32), steps=3, tag="n=70")
    gpu.destroy()


def test_cd_resume_determinism_device_getters_and_status_codes():
    import torch
    announce("CD-Adam resume / status codes")
    d, n, B = 25_003, 3, 1000
    grads = [np.random.default_rng([5, t]).standard_normal((n, d)).astype(f32) for t in range(6)]

    def fresh():
        h = P.CompAms(d, n, P.BLOCKSIGN, B)
        h.set_method(P.METHOD_CD)
        return h

    def state(h):
        return [h.get_theta(), h.get_m(), h.get_v(), h.get_vhat(), h.get_ghat_server(), h.get_gtilde()] + \
               [h.get_ghat_worker(i) for i in range(n)]

    a = fresh()
    for g in grads:
        a.step(torch_dev(g))
    b = fresh()
    for g in grads[:3]:
        b.step(torch_dev(g))
    saved = state(b)
    b.destroy()
    c = fresh()
    c.set_theta(saved[0])
    c.set_state(m=saved[1], v=saved[2], vhat=saved[3])
    c.set_markov_state(ghat_workers=np.stack(saved[6:]), ghat_server=saved[4], gtilde=saved[5])
    for g in grads[3:]:
        c.step(torch_dev(g))
    for x, y in zip(state(a), state(c)):
        assert np.array_equal(bits(x), bits(y))
    out = torch.empty(d, dtype=torch.float32, device="cuda")
    a.get_ghat_worker(1, out)
    assert np.array_equal(bits(out.cpu().numpy()), bits(a.get_ghat_worker(1)))
    # status codes
    with pytest.raises(P.CompAmsError) as ei:
        a.set_method(P.METHOD_EF)                     # after the first step
    assert ei.value.code == P.ESTATE
    with pytest.raises(P.CompAmsError) as ei:
        a.get_error(0)
    assert ei.value.code == P.ESTATE
    with pytest.raises(P.CompAmsError) as ei:
        a.set_state(e=np.zeros((n, d), f32))
    assert ei.value.code == P.ESTATE
    with pytest.raises(P.CompAmsError) as ei:
        a.get_ghat_worker(n)
    assert ei.value.code == P.EINVAL
    e = P.CompAms(100, 2, P.BLOCKSIGN, 10)
    for call in (lambda: e.get_gtilde(), lambda: e.get_ghat_worker(0), lambda: e.get_server_scales(),
                 lambda: e.set_markov_state(gtilde=np.zeros(100, f32))):
        with pytest.raises(P.CompAmsError) as ei:
            call()
        assert ei.value.code == P.ESTATE
    with pytest.raises(P.CompAmsError) as ei:
        e.set_method(7)
    assert ei.value.code == P.EINVAL
    a.destroy(); c.destroy(); e.destroy()


def test_cd_block_table_change_between_steps():
    """set_blocks while a c_i is still owed to the stored rows: the rows are brought up to date with
    the old table first."""
    announce("CD-Adam set_blocks between steps")
    d, n = 20_000, 2
    gpu, ora = make_cd_pair(d, n, 4096)
    gf = lambda t: np.random.default_rng([8, t]).standard_normal((n, d)).astype(f32)
    exact = run_cd(gpu, ora, gf, steps=2, tag="before")
    off = [0, 5000, 5001, 12_000, d]
    gpu.set_blocks(off)
    ora.set_blocks(off)
    for t in range(2, 4):
        g = gf(t)
        gpu.step(torch_dev(g))
        ora.step(g)
        exact = compare_cd(gpu, ora, f"after step {t}", exact)
    gpu.destroy()


# ------------------------------------------------------------------------------- CD-Adam with Top-k
# Bars: kept index sets and kept values of the workers and of the server, ghat_i, ghat and gtilde
# bit-exact; theta, m, v, vhat within 1e-6 relative per coordinate.

def make_cd_topk_pair(d, n, k, theta0=None, eps_mode=1):
    gpu = P.CompAms(d, n, P.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, O.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR, method=O.CD)
    gpu.set_method(P.METHOD_CD)
    if theta0 is not None:
        gpu.set_theta(np.ascontiguousarray(theta0, dtype=f32))
        ora.set_theta(theta0)
    gpu.set_eps_mode(eps_mode)
    ora.set_eps_mode(eps_mode)
    return gpu, ora


def run_cd_topk(gpu, ora, grads_fn, steps, tag):
    for t in range(steps):
        g = grads_fn(t)
        u = g - ora.ghat_workers                       # what the workers compress in this step
        w_prev = ora.gtilde.copy()
        gpu.step(torch_dev(g))
        ora.step(g)
        for i in range(gpu.n):
            idx, val = gpu.get_selected(i)
            assert np.array_equal(idx, ora.selected[i]), f"{tag} step {t} worker {i}: kept index set differs"
            assert np.array_equal(bits(val), bits(u[i][idx])), f"{tag} step {t} worker {i}: kept values differ"
            assert np.array_equal(bits(gpu.get_ghat_worker(i)), bits(ora.ghat_workers[i])), f"{tag} step {t} ghat_{i}"
        assert np.array_equal(bits(gpu.get_ghat_server()), bits(ora.ghat_server)), f"{tag} step {t} ghat"
        idx, val = gpu.get_server_selected()
        assert np.array_equal(idx, ora.server_selected), f"{tag} step {t}: server's kept index set differs"
        assert np.array_equal(bits(val), bits((ora.ghat_server - w_prev)[idx])), f"{tag} step {t}: server's kept values"
        assert np.array_equal(bits(gpu.get_gtilde()), bits(ora.gtilde)), f"{tag} step {t} gtilde"
        for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                                ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
            ok = rel_close(got, want, STATE_RTOL)
            assert ok.all(), f"{tag} step {t} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL}"


def test_cd_topk_golden_example_c_on_gpu():
    announce("CD-Adam golden example C (Top-k)")
    ex = json.load(open(os.path.join(GOLD, "example_c_cd_adam_topk.json")))
    g = np.array(ex["g"], f32)
    h = P.CompAms(ex["d"], ex["n"], P.TOPK, ex["k"])
    h.set_method(P.METHOD_CD)
    gd = torch_dev(g)
    for t, want in enumerate(ex["steps"]):
        h.step(gd)
        for i in range(ex["n"]):
            assert np.array_equal(bits(h.get_ghat_worker(i)), bits(np.array(want["ghat_workers"][i], f32))), (t, i)
        assert np.array_equal(bits(h.get_ghat_server()), bits(np.array(want["ghat_server"], f32))), t
        assert h.get_server_selected()[0].tolist() == want["server_selected"], t
        assert np.array_equal(bits(h.get_gtilde()), bits(np.array(want["gtilde"], f32))), t
    h.destroy()


@pytest.mark.parametrize("d,n,k", [(1, 1, 1), (5, 3, 5), (63, 2, 7), (4097, 2, 41), (10_007, 5, 100),
                                   (3 * 4096, 4, 123), (20_000, 3, 20_000), (300_003, 4, 3000)])
def test_cd_topk_small_shapes(d, n, k):
    announce(f"CD-Adam Top-k d={d} n={n} k={k}")
    rng = np.random.default_rng(d * 17 + n)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    gpu, ora = make_cd_topk_pair(d, n, k, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run_cd_topk(gpu, ora, lambda t: (np.random.default_rng([d, 3, t]).standard_normal((n, d)) * scale + 0.2 * scale).astype(f32),
                steps=5, tag=f"d={d}")
    gpu.destroy()


def test_cd_topk_scale_jumps_ties_and_many_workers():
    announce("CD-Adam Top-k jumps / ties / n=70")
    n, d, k = 4, 150_001, 1500
    rng = np.random.default_rng(41)
    base_scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    factors = [1.0, 1.0, 300.0, 1e-4, 1e-4, 1.0, 1.003, 20.0, 1.0]
    gpu, ora = make_cd_topk_pair(d, n, k)
    run_cd_topk(gpu, ora, lambda t: (np.random.default_rng([41, t]).standard_normal((n, d)).astype(f32) * base_scale
                                     * f32(factors[t])).astype(f32), steps=len(factors), tag="jumps")
    gpu.destroy()
    vals = np.array([0.125, 0.25, -0.25, 0.5, -0.5, 1.0], f32)
    n, d, k = 3, 100_003, 25_000
    gpu, ora = make_cd_topk_pair(d, n, k, eps_mode=0)
    run_cd_topk(gpu, ora, lambda t: vals[np.random.default_rng([42, t]).integers(0, vals.size, (n, d))], steps=3, tag="ties")
    gpu.destroy()
    n, d, k = 70, 9000, 17
    gpu, ora = make_cd_topk_pair(d, n, k)
    run_cd_topk(gpu, ora, lambda t: np.random.default_rng([43, t]).standard_normal((n, d)).astype(f32), steps=3, tag="n=70")
    gpu.destroy()


def test_cd_topk_on_the_resnet_sized_workload_scaled():
    w = W.get(2).scaled(300_003, n=16)
    announce(f"CD-Adam Top-k on {w.name}")
    s = w.scales()
    gpu, ora = make_cd_topk_pair(w.d, w.n, w.k, theta0=w.theta0())
    run_cd_topk(gpu, ora, lambda t: w.grads(t, scales=s), steps=5, tag=w.name)
    gpu.destroy()


def test_cd_topk_resume_and_status_codes():
    announce("CD-Adam Top-k resume")
    d, n, k = 25_003, 3, 250
    grads = [np.random.default_rng([6, t]).standard_normal((n, d)).astype(f32) for t in range(6)]

    def fresh():
        h = P.CompAms(d, n, P.TOPK, k)
        h.set_method(P.METHOD_CD)
        return h

    def state(h):
        return [h.get_theta(), h.get_m(), h.get_v(), h.get_vhat(), h.get_ghat_server(), h.get_gtilde()] + \
               [h.get_ghat_worker(i) for i in range(n)]

    a = fresh()
    for g in grads:
        a.step(torch_dev(g))
    b = fresh()
    for g in grads[:3]:
        b.step(torch_dev(g))
    saved = state(b)
    b.destroy()
    c = fresh()
    c.set_theta(saved[0])
    c.set_state(m=saved[1], v=saved[2], vhat=saved[3])
    c.set_markov_state(ghat_workers=np.stack(saved[6:]), ghat_server=saved[4], gtilde=saved[5])
    for g in grads[3:]:
        c.step(torch_dev(g))
    for x, y in zip(state(a), state(c)):
        assert np.array_equal(bits(x), bits(y))
    with pytest.raises(P.CompAmsError) as ei:
        a.get_server_scales()
    assert ei.value.code == P.ESTATE
    ef = P.CompAms(d, n, P.TOPK, k)
    with pytest.raises(P.CompAmsError) as ei:
        ef.get_server_selected()
    assert ei.value.code == P.ESTATE
    a.destroy(); c.destroy(); ef.destroy()


def test_cd_topk_long_run_with_a_wandering_gradient_scale():
    announce("CD-Adam Top-k long run")
    n, d, k, steps = 4, 200_003, 2000, 30
    rng = np.random.default_rng(2025)
    base_scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    walk = np.cumprod(1.0 + rng.uniform(-0.08, 0.08, steps))
    walk[[9, 21]] *= 0.5
    gpu, ora = make_cd_topk_pair(d, n, k, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run_cd_topk(gpu, ora, lambda t: (np.random.default_rng([2025, t]).standard_normal((n, d)).astype(f32) * base_scale
                                     * f32(walk[t])).astype(f32), steps=steps, tag="long run")
    gpu.destroy()
