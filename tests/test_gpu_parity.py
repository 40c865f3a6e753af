"""GPU parity: the HIP library (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Bars are stated in tests/parity_util.py."""
import json
import os

import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import bits, compare, make_pair, pair_for, run_steps

pytestmark = pytest.mark.gpu
f32 = np.float32
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def torch_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def announce(msg):
    print(f"[case] {msg}", flush=True)


# ------------------------------------------------------------------------------- worked example

def test_golden_example_a_on_gpu():
    gold = json.load(open(os.path.join(GOLD, "example_a_topk_ef_amsgrad.json")))
    g = np.array(gold["grads_every_step"], f32)
    for mode in (0, 1):
        announce(f"golden example A, eps mode {mode}")
        h = P.CompAms(gold["d"], gold["n"], P.TOPK, gold["k"], gold["beta1"], gold["beta2"], gold["eps"], gold["lr"])
        h.set_eps_mode(mode)
        gd = torch_dev(g)
        for want in gold["steps"]:
            h.step(gd)
            for i in range(gold["n"]):
                idx, _ = h.get_selected(i)
                assert idx.tolist() == want["selected"][i]
                assert np.array_equal(bits(h.get_error(i)), bits(want["error"][i]))
            assert h.get_m().tolist() == want["m"]
            assert h.get_v().tolist() == want["v"]
            assert h.get_vhat().tolist() == want["vhat"]
            key = f"theta_mode{mode}"
            if key in want:
                assert np.allclose(h.get_theta(), want[key], rtol=3e-7, atol=0)
        h.destroy()


# ------------------------------------------------------------------------------- Top-k, small

@pytest.mark.parametrize("d,n,k", [(1, 1, 1), (3, 2, 1), (5, 3, 5), (63, 2, 7), (257, 3, 100), (4097, 2, 41),
                                   (10007, 5, 100), (3 * 4096, 4, 123), (20000, 3, 20000)])
def test_topk_small_shapes(d, n, k):
    announce(f"topk small d={d} n={n} k={k}")
    rng = np.random.default_rng(d * 31 + n)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gpu, ora = make_pair(d, n, P.TOPK, k, theta0=theta0)
    run_steps(gpu, ora, lambda t: (np.random.default_rng([d, t]).standard_normal((n, d)) * scale).astype(f32),
              steps=4, tag=f"d={d}")
    gpu.destroy()


@pytest.mark.parametrize("case", ["all_equal", "all_zero", "signed_zero_mix", "denormals", "ties_at_rank_k",
                                  "few_nonzero", "huge_and_inf"])
def test_topk_degenerate_inputs(case):
    announce(f"topk degenerate {case}")
    d, n, k = 9001, 3, 500
    rng = np.random.default_rng(5)
    if case == "all_equal":
        g = np.full((n, d), -2.5, f32)
    elif case == "all_zero":
        g = np.zeros((n, d), f32)
    elif case == "signed_zero_mix":
        g = np.where(rng.random((n, d)) < 0.5, f32(0.0), f32(-0.0)).astype(f32)
        g[:, ::97] = 1.0
    elif case == "denormals":
        g = rng.integers(0, 50, (n, d)).astype(np.uint32).view(f32).copy()      # 0 .. 49 denormal ulps
        g[:, ::2] *= -1
    elif case == "ties_at_rank_k":
        g = rng.choice(np.array([0.25, -0.25, 0.5, -0.5, 1.0, 3.0], f32), (n, d))
    elif case == "few_nonzero":
        g = np.zeros((n, d), f32)
        g[:, 10:20] = rng.standard_normal((n, 10)).astype(f32)
    else:
        g = rng.standard_normal((n, d)).astype(f32) * f32(1e30)
        g[0, 17] = np.inf
        g[1, 4000] = -np.inf
    gpu, ora = make_pair(d, n, P.TOPK, k)
    # theta would become NaN with Inf gradients on both sides; the comparison below treats NaN == NaN
    steps = 3
    import torch
    for t in range(steps):
        gd = torch_dev(g)
        gpu.step(gd)
        e_prev = ora.error.copy()
        ora.step(g)
        for i in range(n):
            idx, val = gpu.get_selected(i)
            assert np.array_equal(idx, ora.selected[i]), f"{case} step {t} worker {i}"
            assert np.array_equal(bits(val), bits((g + e_prev)[i][idx]))
            assert np.array_equal(bits(gpu.get_error(i)), bits(ora.error[i]))
        if case != "huge_and_inf":
            compare(gpu, ora, tag=f"{case} step {t}")
        else:
            assert np.array_equal(bits(gpu.get_m()), bits(ora.m))
            assert np.array_equal(bits(gpu.get_vhat()), bits(ora.vhat))
    gpu.destroy()


def test_topk_k_equal_d_is_vanilla_amsgrad_on_gpu():
    announce("topk k=d")
    n, d = 4, 6000
    rng = np.random.default_rng(9)
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gpu, ora = make_pair(d, n, P.TOPK, d, theta0=theta0)
    stats = run_steps(gpu, ora, lambda t: np.random.default_rng([9, t]).standard_normal((n, d)).astype(f32), 5)
    for i in range(n):
        assert not gpu.get_error(i).any()
    assert all(s["theta_bit_identical"] for s in stats)
    gpu.destroy()


def test_gradient_base_pointer_alignment_classes():
    """Rows of a dense [n][d] array start 16-, 8- or 4-byte aligned depending on d and on the base."""
    import torch
    for d, shift in [(1001, 0), (1002, 0), (1002, 1), (1004, 2), (1003, 3), (8191, 1)]:
        for comp, kb in [(P.TOPK, 37), (P.BLOCKSIGN, 200)]:
            announce(f"alignment d={d} shift={shift} comp={comp}")
            n = 4
            g = np.random.default_rng([d, shift]).standard_normal((n, d)).astype(f32)
            buf = torch.zeros(n * d + 8, dtype=torch.float32, device="cuda")
            view = buf[shift:shift + n * d]
            view.copy_(torch.from_numpy(g).reshape(-1))
            gpu, ora = make_pair(d, n, comp, kb)
            for t in range(2):
                gpu.step_ptr(view.data_ptr(), torch.cuda.current_stream().cuda_stream)
                ora.step(g)
                compare(gpu, ora, tag=f"d={d} shift={shift} comp={comp} step {t}")
            gpu.destroy()


# ------------------------------------------------------------------------------- block sign, small

@pytest.mark.parametrize("d,n,B", [(1, 1, 1), (7, 2, 3), (64, 2, 64), (1000, 3, 4096), (4096, 2, 4096),
                                   (4097, 2, 4096), (10007, 5, 1000), (50001, 4, 4096), (30000, 3, 7)])
def test_blocksign_uniform_small_shapes(d, n, B):
    announce(f"blocksign small d={d} n={n} B={B}")
    rng = np.random.default_rng(d + B)
    scale = np.exp(rng.uniform(-7, -1, d)).astype(f32)
    theta0 = (0.01 * rng.standard_normal(d)).astype(f32)
    gpu, ora = make_pair(d, n, P.BLOCKSIGN, B, theta0=theta0)
    off = np.minimum(np.arange(0, d + B, B), d)
    off = off[: (d + B - 1) // B + 1]
    stats = run_steps(gpu, ora, lambda t: (np.random.default_rng([d, B, t]).laplace(0, 1, (n, d)) * scale).astype(f32),
                      steps=4, tag=f"d={d} B={B}", offsets=off)
    assert gpu.n_blocks() == ora.n_blocks == off.size - 1
    assert sum(s["scales_not_bit_identical"] for s in stats) == 0
    gpu.destroy()


def test_blocksign_layer_blocks_and_degenerate_values():
    announce("blocksign layer table")
    d, n = 70001, 3
    off = np.array([0, 1, 3, 64, 5000, 5001, 20000, 69999, 70001], np.int64)
    gpu, ora = make_pair(d, n, P.BLOCKSIGN, d, offsets=off)
    rng = np.random.default_rng(77)

    def grads(t):
        g = rng.standard_normal((n, d)).astype(f32)
        g[:, 3:64] = 0.0                       # an all-zero block: scale 0, C(x) = +-0
        g[0, 5:30] = -0.0
        g[:, 5000] = 1e-41                      # one-element block holding a denormal
        return g

    run_steps(gpu, ora, grads, steps=3, tag="layers", offsets=off)
    gpu.destroy()


# ------------------------------------------------------------------------------- API behaviour on the GPU

def test_determinism_resume_lr_and_error_codes():
    import torch
    announce("determinism / resume / set_lr / status codes")
    w = W.get(0).scaled(30_011, n=3)
    s = w.scales()
    grads = [w.grads(t, scales=s) for t in range(6)]

    def run(h, ts):
        for t in ts:
            if t == 3:
                h.set_lr(5e-4)
            h.step(torch_dev(grads[t]))

    def state(h):
        return [h.get_theta(), h.get_m(), h.get_v(), h.get_vhat()] + [h.get_error(i) for i in range(w.n)]

    a = P.CompAms(w.d, w.n, P.TOPK, w.k)
    a.set_theta(w.theta0())
    run(a, range(6))
    b = P.CompAms(w.d, w.n, P.TOPK, w.k)
    b.set_theta(w.theta0())
    run(b, range(3))
    saved = state(b)
    b.destroy()
    c = P.CompAms(w.d, w.n, P.TOPK, w.k)                    # resume from the saved state
    c.set_theta(saved[0])
    c.set_state(m=saved[1], v=saved[2], vhat=saved[3], e=np.stack(saved[4:]))
    run(c, range(3, 6))
    for x, y in zip(state(a), state(c)):
        assert np.array_equal(bits(x), bits(y))
    # the oracle agrees with the lr change too
    o = O.Oracle(w.d, w.n, O.TOPK, w.k, w.beta1, w.beta2, w.eps, w.lr)
    o.set_theta(w.theta0())
    for t in range(6):
        if t == 3:
            o.set_lr(5e-4)
        o.step(grads[t])
    compare(a, o, tag="lr schedule")
    # status codes
    with pytest.raises(P.CompAmsError) as ei:
        a.get_scales()
    assert ei.value.code == P.ESTATE
    with pytest.raises(P.CompAmsError) as ei:
        a.get_error(w.n)
    assert ei.value.code == P.EINVAL
    with pytest.raises(P.CompAmsError) as ei:
        a.set_blocks([0, w.d])
    assert ei.value.code == P.ESTATE
    fresh = P.CompAms(100, 2, P.BLOCKSIGN, 10)
    with pytest.raises(P.CompAmsError) as ei:
        fresh.get_scales()
    assert ei.value.code == P.ESTATE
    for bad in ([0, 50], [1, 100], [0, 60, 40, 100], [0, 50, 50, 100]):
        with pytest.raises(P.CompAmsError) as ei:
            fresh.set_blocks(bad)
        assert ei.value.code == P.EINVAL
    # device-side getters
    out = torch.empty(w.d, dtype=torch.float32, device="cuda")
    a.get_theta(out)
    assert np.array_equal(bits(out.cpu().numpy()), bits(a.get_theta()))
    a.destroy(); c.destroy(); fresh.destroy()


def test_eps_mode_one_matches_the_papers_placement():
    announce("eps mode 1")
    w = W.get(1).scaled(20_003, n=4)
    gpu, ora = make_pair(w.d, w.n, P.BLOCKSIGN, 4096, theta0=w.theta0(), eps_mode=1)
    s = w.scales()
    run_steps(gpu, ora, lambda t: w.grads(t, scales=s), steps=3, tag="eps1", offsets=w.block_offsets())
    gpu.destroy()


# ------------------------------------------------------------------------------- the five workloads

def test_cfg0_full_all_steps():
    w = W.get(0)
    announce(w.name)
    gpu, ora = pair_for(w)
    s = w.scales()
    run_steps(gpu, ora, lambda t: w.grads(t, scales=s), steps=w.steps, tag=w.name)
    gpu.destroy()


def test_cfg1_full_all_steps():
    w = W.get(1)
    announce(w.name)
    gpu, ora = pair_for(w)
    s = w.scales()
    stats = run_steps(gpu, ora, lambda t: w.grads(t, scales=s), steps=w.steps, tag=w.name, check_every=1,
                      offsets=w.block_offsets())
    print("cfg1 stats", stats[-1], flush=True)
    gpu.destroy()


@pytest.mark.parametrize("idx,d,n", [(2, 300_003, 16), (3, 400_001, 8), (4, 500_002, 8)])
def test_cfg2_3_4_scaled(idx, d, n):
    w = W.get(idx).scaled(d, n=n, steps=5)
    announce(w.name)
    gpu, ora = pair_for(w)
    s = w.scales()
    run_steps(gpu, ora, lambda t: w.grads(t, scales=s), steps=w.steps, tag=w.name, offsets=w.block_offsets())
    gpu.destroy()


# ------------------------------------------------------------------------------- rarely taken Top-k paths

def test_topk_threshold_jumps_and_drops_between_steps():
    """The candidate guess is carried from step to step; a gradient scale that jumps up (threshold far
    above the guess: coarse-bin path) or collapses (threshold below the guess: candidates are listed
    again) must not change the result."""
    announce("topk threshold jumps")
    n, d, k = 4, 150_001, 1500
    rng = np.random.default_rng(123)
    base_scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    factors = [1.0, 1.0, 300.0, 300.0, 1e-4, 1e-4, 1.0, 1.003, 0.997, 20.0, 1.0, 1.0]
    gpu, ora = make_pair(d, n, P.TOPK, k, theta0=(0.01 * rng.standard_normal(d)).astype(f32))

    def grads(t):
        g = np.random.default_rng([123, t]).standard_normal((n, d)).astype(f32) * base_scale
        return (g * f32(factors[t])).astype(f32)

    run_steps(gpu, ora, grads, steps=len(factors), tag="jumps")
    gpu.destroy()


@pytest.mark.parametrize("n,d,k", [(40, 30_011, 300), (70, 9_000, 17), (2, 1_300_003, 13_000), (1, 2_500_000, 999),
                                   (2, 600_000, 300_000)])
def test_topk_many_workers_and_many_lists(n, d, k):
    """n > 64 walks two worker groups in tk_final; long models fill all 64 candidate regions of a
    worker with several tiles each; a large k cuts each region into several pieces for the candidate
    histogram and the compaction, and gives wavefronts more than 64 candidates per tile."""
    announce(f"topk n={n} d={d} k={k}")
    rng = np.random.default_rng(n * 7 + 1)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    gpu, ora = make_pair(d, n, P.TOPK, k, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run_steps(gpu, ora, lambda t: (np.random.default_rng([n, d, t]).standard_normal((n, d)) * scale).astype(f32),
              steps=4, tag=f"n={n}")
    gpu.destroy()


def test_topk_selection_info_reports_the_path_taken():
    """The carried guess must actually be used: with a steady gradient scale the threshold is found
    among the listed candidates (no second listing) from the second step on, a collapse of the scale
    forces a second listing in that step only, and the reported threshold bin is the fine bin of the
    k-th largest magnitude of g + e (taken from the oracle's kept set)."""
    announce("topk selection info")
    import torch
    n, d, k = 3, 90_001, 900
    rng = np.random.default_rng(321)
    base_scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    factors = [1.0, 1.0, 1.0, 1.0, 1e-3, 1e-3, 1.0, 1.0]
    gpu, ora = make_pair(d, n, P.TOPK, k)
    relisted = []
    guess = [1 << 17] * n                            # before the first step nothing can be listed
    for t, f in enumerate(factors):
        g = (np.random.default_rng([321, t]).standard_normal((n, d)).astype(f32) * base_scale * f32(f)).astype(f32)
        x = g + ora.error
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
        row = []
        for i in range(n):
            info = gpu.get_selection_info(i)
            listed = int(np.count_nonzero(((bits(x[i]) & 0x7FFFFFFF) >> 14) >= guess[i]))
            assert info["relisted"] == (1 if listed < k else 0), f"step {t} worker {i}: {listed} listed"
            guess[i] = info["next_guess"]
            kth = np.abs(x[i][ora.selected[i]]).min()
            assert info["threshold_fine_bin"] == int(bits(np.array([kth], f32))[0] >> 14), f"step {t} worker {i}"
            assert 8 <= info["slack"] <= 512
            assert info["next_guess"] == max(info["threshold_fine_bin"] - info["slack"], 0)
            row.append(info["relisted"])
        relisted.append(row)
        compare(gpu, ora, x_for_values=x, tag=f"info step {t}")
    assert relisted[0] == [1] * n                    # nothing is listed before the first threshold exists
    assert relisted[1:4] == [[0] * n] * 3            # steady: the guess holds
    assert relisted[6] == [0] * n                    # a rising threshold needs no second listing
    gpu.destroy()


def test_topk_heavy_ties_need_deep_digits_and_big_tiles():
    """Few distinct magnitudes: the threshold magnitude is shared by thousands of coordinates, so the
    index digits of the radix select decide, and a tile holds more candidates than one staging chunk."""
    announce("topk heavy ties")
    n, d, k = 3, 200_003, 50_000
    rng = np.random.default_rng(99)
    vals = np.array([0.125, 0.25, -0.25, 0.5, -0.5, 1.0], f32)
    gpu, ora = make_pair(d, n, P.TOPK, k)
    run_steps(gpu, ora, lambda t: vals[np.random.default_rng([99, t]).integers(0, vals.size, (n, d))],
              steps=3, tag="ties")
    gpu.destroy()


def test_blocksign_many_workers():
    announce("blocksign n=70")
    n, d = 70, 20_001
    rng = np.random.default_rng(70)
    scale = np.exp(rng.uniform(-6, -1, d)).astype(f32)
    for B, offsets in ((4096, None), (8192, None), (d, np.array([0, 5, 4096, 4100, 12_288, d], np.int64))):
        gpu, ora = make_pair(d, n, P.BLOCKSIGN, B, offsets=offsets)
        off = offsets if offsets is not None else np.minimum(np.arange(0, d + B, B), d)[: (d + B - 1) // B + 1]
        run_steps(gpu, ora, lambda t: (np.random.default_rng([70, t]).laplace(0, 1, (n, d)) * scale).astype(f32),
                  steps=3, tag=f"n=70 B={B}", offsets=off)
        gpu.destroy()


def test_topk_long_run_with_a_wandering_gradient_scale():
    """The guess and its slack are carried from step to step; over many steps with a gradient scale that
    wanders (±8 % per step, with occasional drops) the threshold moves up and down, through the slack
    and back.  Every step must still agree with the oracle, whichever path found the threshold."""
    announce("topk long run")
    import torch
    n, d, k, steps = 4, 200_003, 2000, 40
    rng = np.random.default_rng(2024)
    base_scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    walk = np.cumprod(1.0 + rng.uniform(-0.08, 0.08, steps))
    walk[[11, 23, 31]] *= 0.5
    gpu, ora = make_pair(d, n, P.TOPK, k, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    second_listings = 0
    for t in range(steps):
        g = (np.random.default_rng([2024, t]).standard_normal((n, d)).astype(f32) * base_scale * f32(walk[t])).astype(f32)
        x = g + ora.error
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
        compare(gpu, ora, x_for_values=x, tag=f"long run step {t}")
        second_listings += sum(gpu.get_selection_info(i)["relisted"] for i in range(n))
    assert n <= second_listings < n * steps // 2      # the first step always; later ones only now and then
    gpu.destroy()


@pytest.mark.parametrize("d,n,k,density", [(300_007, 3, 3000, 0.004), (300_007, 3, 3000, 0.02), (50_000, 2, 50_000, 0.3),
                                           (9_000, 2, 4500, 0.0), (1_300_003, 2, 13_000, 0.005)])
def test_topk_with_fewer_nonzeros_than_k(d, n, k, density):
    """Sparse vectors: when fewer than k coordinates are non-zero the k-th largest is a zero, and zeros are
    selected by lower index.  Gradients with a fixed sparse support (plus signed zeros) keep the error memory
    sparse too, so the regime persists over the steps; density 0.02 crosses in and out of it."""
    announce(f"sparse top-k d={d} k={k} density={density}")
    rng = np.random.default_rng(d + k)
    support = rng.random(d) < density
    gpu, ora = make_pair(d, n, P.TOPK, k)

    def grads(t):
        r = np.random.default_rng([d, k, t])
        g = r.standard_normal((n, d)).astype(f32) * support
        g[:, ~support] = np.where(r.random((n, int((~support).sum()))) < 0.5, f32(0.0), f32(-0.0))
        if t == 2:
            g[0] = 0.0                                    # an all-zero gradient for one worker
        return g

    run_steps(gpu, ora, grads, steps=5, tag=f"sparse d={d}")
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("block", [1, 3, 16, 64, 1000, 2048, 5000])
def test_blocksign_with_blocks_shorter_and_longer_than_a_tile(block):
    """Uniform blocks that cut every tile into several pieces (summed by teams of 16 lanes, scales written by
    the pass itself) or span several tiles with a ragged cut."""
    announce(f"blocksign block={block}")
    d, n = 40_011, 3
    gpu, ora = make_pair(d, n, P.BLOCKSIGN, block)
    scale = np.exp(np.random.default_rng(block).uniform(-5, 0, d)).astype(f32)
    run_steps(gpu, ora, lambda t: (np.random.default_rng([block, t]).standard_normal((n, d)) * scale).astype(f32),
              steps=4, tag=f"block {block}", offsets=ora_offsets(d, block))
    gpu.destroy()
    ora.close()


def ora_offsets(d, block):
    return np.minimum(np.arange((d + block - 1) // block + 1, dtype=np.int64) * block, d)


def test_probe_update_adds_in_place_in_both_launch_shapes():
    """comp_ams_probe_update (a measurement aid): x += g, exactly, for a small problem (plain launch shape) and
    for one beyond a GiB (three workgroups per compute unit, XCD-aware piece order), ragged row lengths included."""
    import torch
    announce("probe_update")
    for rows, d in ((3, 4 * 1237), (5, 4 * 13_500_001)):
        g = torch.randn(rows, d, device="cuda")
        x = torch.randn(rows, d, device="cuda")
        want = x + g
        P.probe_update(x, g)
        torch.cuda.synchronize()
        assert torch.equal(x, want)
        del g, x, want
    with pytest.raises(P.CompAmsError) as ei:
        P.probe_update(torch.zeros(2, 6, device="cuda"), torch.zeros(2, 6, device="cuda"))      # d not a multiple of 4
    assert ei.value.code == P.EINVAL


@pytest.mark.parametrize("n,d,block", [(3000, 8200, 4096), (1100, 20_000, 8192), (65_531, 4100, 4096)])
def test_block_sign_with_uniform_tile_blocks_and_many_workers(n, d, block):
    """The one-launch path of block sign (the pass kernel carries the previous step's update): more workers than
    the 1024 whose scales the update stages at a time, blocks of one and of two tiles, a partial last block, and
    the largest worker count the path takes; steps back to back, then compared, then one more step."""
    import torch
    announce(f"block sign, uniform tile blocks, n={n} d={d} B={block}")
    gpu, ora = make_pair(d, n, P.BLOCKSIGN, block)
    off = np.minimum(np.arange((d + block - 1) // block + 1, dtype=np.int64) * block, d)
    rng = np.random.default_rng(n)
    for t in range(4):
        g = rng.standard_normal((n, d)).astype(f32)
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
        if t == 2:
            compare(gpu, ora, tag=f"n={n} step {t}", check_error=(n <= 4000), offsets=off)
    compare(gpu, ora, tag=f"n={n} after the last step", check_error=(n <= 4000), offsets=off)
    gpu.destroy()
    ora.close()
