"""Gradients handed over as bfloat16 (comp_ams_step_bf16): the step must compute exactly what the
fp32 entry point and the oracle compute on the widened values.  Bars as everywhere: error memory,
Markov sequences and kept sets bit-exact; theta, m, v, vhat within 1e-6 relative; scales 1e-5."""
import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import SCALE_RTOL, STATE_RTOL, bits, rel_close

pytestmark = pytest.mark.gpu
f32 = np.float32


def announce(msg):
    print(f"[case] {msg}", flush=True)


def to_bf16(g):
    """(device bfloat16 tensor, the same values widened to float32 on the host)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(g, dtype=f32)).to(torch.bfloat16)
    return t.cuda(), t.float().numpy()


def check_state(gpu, ora, tag):
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                            ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
        ok = rel_close(got, want, STATE_RTOL)
        assert ok.all(), f"{tag} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL}"


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD, P.METHOD_NAIVE, P.METHOD_NONE])
@pytest.mark.parametrize("comp,d,n,kb", [(P.TOPK, 30_011, 5, 300), (P.BLOCKSIGN, 30_011, 5, 4096),
                                         (P.TOPK, 7, 2, 3), (P.BLOCKSIGN, 4097, 3, 100)])
def test_bf16_gradients_match_the_oracle_on_the_widened_values(method, comp, d, n, kb):
    announce(f"bf16 method={method} comp={comp} d={d}")
    rng = np.random.default_rng(d + 10 * method + comp)
    scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    gpu = P.CompAms(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    for t in range(4):
        g = (np.random.default_rng([d, method, t]).standard_normal((n, d)) * scale).astype(f32)
        g16, gw = to_bf16(g)
        gpu.step_bf16(g16)
        ora.step(gw)
        check_state(gpu, ora, f"step {t}")
        if method == P.METHOD_EF:
            for i in range(n):
                assert np.array_equal(bits(gpu.get_error(i)), bits(ora.error[i])), (t, i)
        if method == P.METHOD_CD:
            for i in range(n):
                assert np.array_equal(bits(gpu.get_ghat_worker(i)), bits(ora.ghat_workers[i])), (t, i)
            assert np.array_equal(bits(gpu.get_gtilde()), bits(ora.gtilde)), t
        if method != P.METHOD_NONE and comp == P.TOPK:
            for i in range(n):
                assert np.array_equal(gpu.get_selected(i)[0], ora.selected[i]), (t, i)
        if method != P.METHOD_NONE and comp == P.BLOCKSIGN:
            assert rel_close(gpu.get_scales(), ora.scales, SCALE_RTOL).all()
    gpu.destroy()


def test_bf16_rows_at_every_alignment_and_same_result_as_fp32_entry():
    """Odd d puts the rows at all four 2-byte alignment classes; a shifted base pointer moves them all.
    The fp32 entry point on the widened values must give bit-identical state."""
    import torch
    announce("bf16 alignment classes")
    d, n = 10_001, 4
    a = P.CompAms(d, n, P.BLOCKSIGN, 1000)
    b = P.CompAms(d, n, P.BLOCKSIGN, 1000)
    for t in range(4):
        g = np.random.default_rng([91, t]).standard_normal((n, d)).astype(f32)
        g16, gw = to_bf16(g)
        buf = torch.empty(n * d + 4, dtype=torch.bfloat16, device="cuda")
        view = buf[t: t + n * d]
        view.copy_(g16.reshape(-1))
        a.step_bf16_ptr(view.data_ptr(), torch.cuda.current_stream().cuda_stream)
        b.step(torch.from_numpy(gw).cuda())
        for x, y in ((a.get_theta(), b.get_theta()), (a.get_vhat(), b.get_vhat()), (a.get_error(1), b.get_error(1))):
            assert np.array_equal(bits(x), bits(y)), t
    with pytest.raises(P.CompAmsError) as ei:
        a.step_bf16_ptr(buf.data_ptr() + 1)           # not 2-byte aligned
    assert ei.value.code == P.EINVAL
    a.destroy(); b.destroy()


def test_bf16_on_the_large_model_workload_scaled():
    """cfg4's gradients are bfloat16-representable by construction: both entry points see the same numbers."""
    import torch
    w = W.get(4).scaled(500_002, n=8)
    announce(f"bf16 on {w.name}")
    s = w.scales()
    gpu = P.CompAms(w.d, w.n, P.TOPK, w.k, w.beta1, w.beta2, w.eps, w.lr)
    ora = O.Oracle(w.d, w.n, O.TOPK, w.k, w.beta1, w.beta2, w.eps, w.lr)
    gpu.set_theta(w.theta0()); ora.set_theta(w.theta0())
    for t in range(3):
        g = w.grads(t, scales=s)
        g16, gw = to_bf16(g)
        assert np.array_equal(bits(gw), bits(g))          # nothing is lost: the recipe rounds to bfloat16 itself
        gpu.step_bf16(g16)
        ora.step(g)
        check_state(gpu, ora, f"step {t}")
        for i in range(w.n):
            assert np.array_equal(gpu.get_selected(i)[0], ora.selected[i])
            assert np.array_equal(bits(gpu.get_error(i)), bits(ora.error[i]))
    gpu.destroy()
