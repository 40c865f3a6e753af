"""Gradients handed over as IEEE half precision (comp_ams_step_f16): every finite half value is an
fp32 value, so the step must compute exactly what the oracle computes on the widened numbers.
Bars as everywhere: error memory, Markov sequences and kept sets bit-exact; theta, m, v, vhat within
1e-6 relative; scales 1e-5."""
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


def to_f16(g):
    """(device float16 tensor, the same values widened to float32 on the host by numpy)."""
    import torch
    h = np.ascontiguousarray(g, dtype=f32).astype(np.float16)
    return torch.from_numpy(h).cuda(), h.astype(f32)


def check_state(gpu, ora, tag):
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                            ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
        ok = rel_close(got, want, STATE_RTOL)
        assert ok.all(), f"{tag} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL}"


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD, P.METHOD_NAIVE, P.METHOD_NONE])
@pytest.mark.parametrize("comp,d,n,kb", [(P.TOPK, 30_011, 5, 300), (P.BLOCKSIGN, 30_011, 5, 4096),
                                         (P.TOPK, 7, 2, 3)])
def test_f16_gradients_match_the_oracle_on_the_widened_values(method, comp, d, n, kb):
    announce(f"f16 method={method} comp={comp} d={d}")
    rng = np.random.default_rng(d + 10 * method + comp)
    # scales down to 2^-20: a good share of the values are half-precision subnormals or round to zero
    scale = np.exp(rng.uniform(-14, 0, d)).astype(f32)
    gpu = P.CompAms(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    for t in range(4):
        g = (np.random.default_rng([d, method, t, 16]).standard_normal((n, d)) * scale).astype(f32)
        g16, gw = to_f16(g)
        if t == 0 and d > 100:
            sub = np.count_nonzero((np.abs(gw) < 2.0 ** -14) & (gw != 0))
            assert sub > d // 100, "the input is meant to hold subnormal half values"
        gpu.step_f16(g16)
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


def test_every_finite_half_value_is_widened_exactly():
    """All 63488 finite bit patterns (normals, subnormals, both zeros) as one gradient row, with no
    compression and one worker: m after the first step is (1 - beta1) * g, which numpy's own widening
    of the same patterns must reproduce within the state bar, and zero exactly where g is zero."""
    import torch
    announce("f16 all finite patterns")
    pat = np.arange(1 << 16, dtype=np.uint16)
    pat = pat[(pat & 0x7C00) != 0x7C00]
    want = pat.view(np.float16).astype(f32)
    d = pat.size
    gpu = P.CompAms(d, 1, P.TOPK, 1, W.BETA1, W.BETA2, W.EPS, W.LR)
    gpu.set_method(P.METHOD_NONE)
    gpu.step_f16(torch.from_numpy(pat.view(np.float16).copy()).cuda())
    m = gpu.get_m()
    ref = (f32(1.0) - f32(W.BETA1)) * want
    assert rel_close(m, ref.astype(np.float64), STATE_RTOL).all()
    assert np.array_equal(m == 0, want == 0)
    v = gpu.get_v()
    ref_v = (1.0 - np.float64(f32(W.BETA2))) * want.astype(np.float64) ** 2
    big = ref_v > 1e-37          # below that fp32 itself leaves the normal range
    assert rel_close(v[big], ref_v[big], STATE_RTOL).all()
    gpu.destroy()


def test_f16_rows_at_every_alignment_and_same_result_as_fp32_entry():
    """Odd d puts the rows at all four 2-byte alignment classes; a shifted base pointer moves them all.
    The fp32 entry point on the widened values must give bit-identical state."""
    import torch
    announce("f16 alignment classes")
    d, n = 10_001, 4
    for comp, kb in ((P.BLOCKSIGN, 1000), (P.TOPK, 100)):
        a = P.CompAms(d, n, comp, kb)
        b = P.CompAms(d, n, comp, kb)
        for t in range(4):
            g = np.random.default_rng([92, t]).standard_normal((n, d)).astype(f32)
            g16, gw = to_f16(g)
            buf = torch.empty(n * d + 4, dtype=torch.float16, device="cuda")
            view = buf[t: t + n * d]
            view.copy_(g16.reshape(-1))
            a.step_f16_ptr(view.data_ptr(), torch.cuda.current_stream().cuda_stream)
            b.step(torch.from_numpy(gw).cuda())
            torch.cuda.synchronize()
        for name in ("theta", "m", "v", "vhat"):
            assert np.array_equal(bits(getattr(a, "get_" + name)()), bits(getattr(b, "get_" + name)())), name
        for i in range(n):
            assert np.array_equal(bits(a.get_error(i)), bits(b.get_error(i)))
        a.destroy()
        b.destroy()


def test_misaligned_f16_pointer_is_rejected():
    import torch
    announce("f16 odd pointer")
    gpu = P.CompAms(64, 2, P.BLOCKSIGN, 16)
    buf = torch.zeros(2 * 64 + 2, dtype=torch.float16, device="cuda")
    with pytest.raises(P.CompAmsError):
        gpu.step_f16_ptr(buf.data_ptr() + 1, 0)
    gpu.destroy()
