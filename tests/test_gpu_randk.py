"""Rand-k (Appendix A, "Rand-k") through the Top-k kernels with pseudo-random keys: parity with the
oracle.  Kept sets, error memory and Markov sequences bit-exact; theta, m, v, vhat within 1e-6
relative."""
import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import STATE_RTOL, bits, rel_close

pytestmark = pytest.mark.gpu
f32 = np.float32


def announce(msg):
    print(f"[case] {msg}", flush=True)


def check_state(gpu, ora, tag):
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                            ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
        ok = rel_close(got, want, STATE_RTOL)
        assert ok.all(), f"{tag} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL}"


def pair(d, n, k, method, seed, draw=0):
    gpu = P.CompAms(d, n, P.RANDK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, O.RANDK, k, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    gpu.set_rand(seed, draw)
    ora.set_rand(seed, draw)
    return gpu, ora


def compare(gpu, ora, method, n, tag):
    check_state(gpu, ora, tag)
    for i in range(n):
        idx, val = gpu.get_selected(i)
        assert np.array_equal(idx, ora.selected[i]), (tag, i)
        assert np.array_equal(bits(val), bits(ora.compressed[i][ora.selected[i]])), (tag, i)
        if method == P.METHOD_EF:
            assert np.array_equal(bits(gpu.get_error(i)), bits(ora.error[i])), (tag, i)
        if method == P.METHOD_CD:
            assert np.array_equal(bits(gpu.get_ghat_worker(i)), bits(ora.ghat_workers[i])), (tag, i)
    if method == P.METHOD_CD:
        assert np.array_equal(bits(gpu.get_ghat_server()), bits(ora.ghat_server)), tag
        assert np.array_equal(bits(gpu.get_gtilde()), bits(ora.gtilde)), tag
        assert np.array_equal(gpu.get_server_selected()[0], ora.server_selected), tag


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_NAIVE, P.METHOD_CD])
@pytest.mark.parametrize("d,n,k", [(1, 1, 1), (7, 2, 3), (4096, 3, 41), (30_011, 5, 300), (70_001, 2, 70_001),
                                   (200_003, 3, 150)])
def test_randk_matches_the_oracle(method, d, n, k):
    announce(f"randk method={method} d={d} n={n} k={k}")
    gpu, ora = pair(d, n, k, method, seed=0xABCDEF0123456789 + d)
    scale = np.exp(np.random.default_rng(d).uniform(-5, 0, d)).astype(f32)
    for t in range(5):
        g = (np.random.default_rng([d, method, t]).standard_normal((n, d)) * scale).astype(f32)
        gpu.step(__import__("torch").from_numpy(g).cuda())
        ora.step(g)
        compare(gpu, ora, method, n, f"step {t}")
    gpu.destroy()
    ora.close()


def test_randk_many_steps_the_guess_follows_the_score_threshold():
    """The threshold of the scores moves a little from draw to draw; over many steps the carried guess
    must sometimes miss and be recovered, with the same kept sets throughout."""
    import torch
    announce("randk long run")
    d, n, k = 120_000, 4, 1200
    gpu, ora = pair(d, n, k, P.METHOD_EF, seed=99)
    relists = 0
    for t in range(40):
        g = np.random.default_rng([5, t]).standard_normal((n, d)).astype(f32)
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
        for i in range(n):
            assert np.array_equal(gpu.get_selected(i)[0], ora.selected[i]), (t, i)
            relists += int(gpu.get_selection_info(i)["relisted"]) if t > 0 else 0
    compare(gpu, ora, P.METHOD_EF, n, "end")
    print(f"relisted after the first step: {relists} of {39 * n}", flush=True)
    assert relists < 39 * n // 2
    gpu.destroy()
    ora.close()


def test_randk_resumes_at_a_given_draw_and_half_precision_gradients():
    import torch
    announce("randk resume + bf16")
    d, n, k = 50_001, 3, 500
    gs = [np.random.default_rng([6, t]).standard_normal((n, d)).astype(f32) for t in range(4)]
    gpu, ora = pair(d, n, k, P.METHOD_NAIVE, seed=7, draw=1000)
    for g in gs:
        t16 = torch.from_numpy(g).to(torch.bfloat16)
        gpu.step_bf16(t16.cuda())
        ora.step(t16.float().numpy())
    compare(gpu, ora, P.METHOD_NAIVE, n, "bf16 from draw 1000")
    gpu.destroy()
    ora.close()


def test_randk_argument_checks():
    import torch
    announce("randk checks")
    a = P.CompAms(100, 2, P.TOPK, 10)
    with pytest.raises(P.CompAmsError) as ei:
        a.set_rand(1, 0)
    assert ei.value.code == P.ESTATE
    a.destroy()
    b = P.CompAms(100, 2, P.RANDK, 10)
    b.set_rand(1, 5)
    b.step(torch.zeros(2, 100, device="cuda"))
    with pytest.raises(P.CompAmsError) as ei:
        b.set_rand(1, 0)
    assert ei.value.code == P.ESTATE
    b.destroy()
    with pytest.raises(P.CompAmsError):
        P.CompAms(100, 2, P.RANDK, 101)
