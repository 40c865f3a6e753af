"""The candidate lists of the Top-k selection are bounded (a vector's regions hold about 8 k entries or d / 32,
whichever is more), and inputs exist whose candidates cannot fit: the library must detect that and select
another way, with the same result bit for bit.  These cases force both fallbacks - the second listing with the
exact coarse bin after a region filled up in the listing pass, and the selection without lists when even that
does not fit (all-equal magnitudes: nothing narrower than the whole composite key separates the elements) - under
error feedback, naive compression and CD-Adam, and check the state after every step against the oracle."""
import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import bits, rel_close, STATE_RTOL

pytestmark = pytest.mark.gpu
f32 = np.float32


def check(gpu, ora, method, tag):
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m), ("v", gpu.get_v(), ora.v),
                            ("vhat", gpu.get_vhat(), ora.vhat)):
        assert rel_close(got, want, STATE_RTOL).all(), f"{tag}: {name} differs"
    for i in range(gpu.n):
        idx, val = gpu.get_selected(i)
        assert np.array_equal(idx, ora.selected[i]), f"{tag}: kept set of worker {i} differs"
        assert np.array_equal(bits(val), bits(ora.compressed[i][idx])), f"{tag}: kept values of worker {i} differ"
        if method == P.METHOD_EF:
            assert np.array_equal(bits(gpu.get_error(i)), bits(ora.error[i])), f"{tag}: error memory of worker {i} differs"
        elif method == P.METHOD_CD:
            assert np.array_equal(bits(gpu.get_ghat_worker(i)), bits(ora.ghat_workers[i])), f"{tag}: ghat_{i} differs"
    if method == P.METHOD_CD:
        assert np.array_equal(gpu.get_server_selected()[0], ora.server_selected), f"{tag}: server's kept set differs"
        assert np.array_equal(bits(gpu.get_gtilde()), bits(ora.gtilde)), f"{tag}: gtilde differs"


def gradient_sequence(d, n, seed):
    """Steps that do not fit bounded lists, between steps that do."""
    rng = np.random.default_rng(seed)
    scale = np.exp(rng.uniform(-4, 0, d)).astype(f32)
    ordinary = lambda: (rng.standard_normal((n, d)).astype(f32) * scale)
    sign = np.where(rng.random((n, d)) < 0.5, f32(-1), f32(1))
    two = np.where(rng.random((n, d)) < 0.3, f32(2.5), f32(0.25)) * sign
    return [
        ("all equal at the start", np.full((n, d), 0.5, f32)),
        ("ordinary", ordinary()),
        ("all equal", np.full((n, d), 0.75, f32)),
        ("all equal, mixed signs", (f32(3.0) * sign).astype(f32)),
        ("ordinary after", ordinary()),
        ("two magnitudes", two.astype(f32)),
        ("thousand times larger", (ordinary() * f32(1000.0)).astype(f32)),
        ("all equal again", np.full((n, d), -1e-3, f32)),
        ("ordinary at the end", ordinary()),
        ("all zero", np.zeros((n, d), f32)),
        ("ordinary after zeros", ordinary()),
    ]


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_NAIVE, P.METHOD_CD])
@pytest.mark.parametrize("d,n,k", [(300_007, 3, 3_000), (70_001, 2, 9)])
def test_inputs_that_overflow_the_candidate_lists(method, d, n, k):
    import torch
    print(f"[case] bounded lists method={method} d={d} n={n} k={k}", flush=True)
    gpu = P.CompAms(d, n, P.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, O.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    for t, (what, g) in enumerate(gradient_sequence(d, n, 100 + method)):
        g = np.ascontiguousarray(g, dtype=f32)
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
        check(gpu, ora, method, f"step {t} ({what})")
        # the records say which way the threshold was found (3 = without lists).  Only where the vector that is
        # compressed is itself all-equal: the gradient under naive compression, the first step's otherwise
        if what.startswith("all equal") and (method == P.METHOD_NAIVE or t == 0):
            assert gpu.get_selection_info(0)["whole_bin"] == 3, f"step {t} ({what}): expected the selection without lists"
        if what == "thousand times larger":
            assert gpu.get_selection_info(0)["relisted"] == 1, f"step {t} ({what}): expected a second listing"
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("method", [P.METHOD_NAIVE, P.METHOD_CD])
def test_selection_without_lists_reforms_the_vector_from_16_bit_gradients(method, dtype):
    """Naive compression and the workers of CD-Adam compress a vector that is not stored (g, g - ghat_i): the
    selection without lists re-forms it from the gradients, which may be bfloat16 or half."""
    import torch
    print(f"[case] bounded lists, 16-bit gradients method={method} {dtype}", flush=True)
    d, n, k = 120_001, 2, 1_200
    tt = torch.bfloat16 if dtype == "bf16" else torch.float16
    gpu = P.CompAms(d, n, P.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, O.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    rng = np.random.default_rng(9)
    seq = [np.full((n, d), 0.25, f32), rng.standard_normal((n, d)).astype(f32), np.full((n, d), -3.0, f32),
           rng.standard_normal((n, d)).astype(f32)]
    for t, g in enumerate(seq):
        g16 = torch.from_numpy(g).to(tt)
        (gpu.step_bf16 if dtype == "bf16" else gpu.step_f16)(g16.cuda())
        ora.step(g16.float().numpy())
        check(gpu, ora, method, f"step {t}")
        if t == 0 or (method == P.METHOD_NAIVE and t == 2):
            assert gpu.get_selection_info(0)["whole_bin"] == 3, f"step {t}: expected the selection without lists"
    gpu.destroy()
    ora.close()


def test_all_equal_input_over_many_steps_without_reading_state_in_between():
    """The deferred update and the fallbacks together: ten steps in a row with nothing read back, every second
    one all-equal, compared at the end."""
    import torch
    print("[case] bounded lists, steps back to back", flush=True)
    d, n, k = 200_003, 4, 2_000
    rng = np.random.default_rng(5)
    gpu = P.CompAms(d, n, P.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, O.TOPK, k, W.BETA1, W.BETA2, W.EPS, W.LR)
    for t in range(10):
        g = np.full((n, d), 0.5, f32) if t % 2 else rng.standard_normal((n, d)).astype(f32)
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
    check(gpu, ora, P.METHOD_EF, "after ten steps")
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("d,n,k", [(8_000_000, 8, 8_000), (110_000_000, 8, 110_000)])
def test_handle_memory_is_bounded(d, n, k):
    """What the handle allocates besides state and error memory stays a fraction of the error memory: the lists are
    sized for a multiple of the steady-state candidate count, not for every coordinate.  The second case is the
    largest of the five workloads: 3.52 GB of error memory, 1.76 GB of state, and the whole handle under 6.5 GB."""
    import torch
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    gpu = P.CompAms(d, n, P.TOPK, k)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    used = free0 - free1
    rows = 4 * n * d
    state = 4 * 4 * d
    print(f"[case] handle memory: {used / 1e6:.0f} MB for rows {rows / 1e6:.0f} MB + state {state / 1e6:.0f} MB", flush=True)
    assert used < rows + state + rows // 4 + (64 << 20)
    if d == 110_000_000:
        assert used < 6.5e9
    gpu.destroy()
