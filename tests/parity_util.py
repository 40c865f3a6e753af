"""Shared helpers of the GPU parity tests: run the HIP library and the CPU oracle side by side
on the same seeded inputs and compare element by element.

Acceptance bars (written out here, used by every parity test):
  * kept index sets, kept values and the error memory e_i: bit-exact
    (block sign: bit-exact whenever the GPU's block scales are bit-identical to the oracle's, which
    is the expected case; a scale that differs - only possible when the fp64 block sum sits on an
    fp32 rounding boundary - must agree to 1e-5 relative, and e is then checked against the
    GPU's own scale);
  * theta, m, v, vhat: |a-b| <= 1e-6 * max(|a|,|b|) per coordinate (both zero passes);
  * block-sign scales: 1e-5 relative.
"""
from __future__ import annotations

import numpy as np

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O

STATE_RTOL = 1e-6
SCALE_RTOL = 1e-5


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def rel_close(a, b, rtol):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return np.abs(a - b) <= rtol * np.maximum(np.abs(a), np.abs(b))


def make_pair(d, n, compressor, k_or_block, beta1=W.BETA1, beta2=W.BETA2, eps=W.EPS, lr=W.LR, theta0=None,
              offsets=None, eps_mode=0):
    gpu = P.CompAms(d, n, compressor, k_or_block, beta1, beta2, eps, lr)
    ora = O.Oracle(d, n, compressor, k_or_block, beta1, beta2, eps, lr)
    if offsets is not None:
        gpu.set_blocks(offsets)
        ora.set_blocks(offsets)
    if theta0 is not None:
        gpu.set_theta(np.ascontiguousarray(theta0, dtype=np.float32))
        ora.set_theta(theta0)
    if eps_mode:
        gpu.set_eps_mode(eps_mode)
        ora.set_eps_mode(eps_mode)
    return gpu, ora


def pair_for(w: W.Workload):
    kb = w.k if w.compressor == W.TOPK else (w.block if w.block else w.d)
    off = w.block_offsets() if (w.compressor == W.BLOCKSIGN and w.layer_blocks) else None
    return make_pair(w.d, w.n, w.compressor, kb, w.beta1, w.beta2, w.eps, w.lr, theta0=w.theta0(), offsets=off)


def compare(gpu: P.CompAms, ora: O.Oracle, x_for_values=None, check_error=True, tag="", offsets=None):
    """Element-by-element comparison of the whole optimiser state after a step."""
    stats = {}
    for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                            ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
        ok = rel_close(got, want, STATE_RTOL)
        assert ok.all(), f"{tag} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL} relative, " \
                         f"first at {int(np.argmin(ok))}: gpu={got[np.argmin(ok)]!r} oracle={want[np.argmin(ok)]!r}"
        stats[name + "_bit_identical"] = bool(np.array_equal(bits(got), bits(want)))
    if gpu.compressor != P.BLOCKSIGN:
        for i in range(gpu.n):
            idx, val = gpu.get_selected(i)
            assert np.array_equal(idx, ora.selected[i]), f"{tag} worker {i}: kept index set differs"
            if x_for_values is not None:
                assert np.array_equal(bits(val), bits(x_for_values[i][idx])), f"{tag} worker {i}: kept values differ"
            if check_error:
                e = gpu.get_error(i)
                assert np.array_equal(bits(e), bits(ora.error[i])), f"{tag} worker {i}: error memory differs"
    else:
        s_gpu, s_ora = gpu.get_scales(), ora.scales
        assert rel_close(s_gpu, s_ora, SCALE_RTOL).all(), f"{tag} block scales beyond {SCALE_RTOL} relative"
        same = bits(s_gpu) == bits(s_ora)
        stats["scales_not_bit_identical"] = int(np.count_nonzero(~same))
        if check_error:
            for i in range(gpu.n):
                e = gpu.get_error(i)
                if same[i].all():
                    assert np.array_equal(bits(e), bits(ora.error[i])), f"{tag} worker {i}: error memory differs"
                else:
                    assert x_for_values is not None and offsets is not None, \
                        f"{tag}: a block scale differs in its last bit; rerun with x and offsets to check e"
                    off = np.asarray(offsets)
                    for b in range(off.size - 1):
                        lo, hi = off[b], off[b + 1]
                        x = x_for_values[i][lo:hi]
                        want = x - np.copysign(s_gpu[i, b], x).astype(np.float32)
                        assert np.array_equal(bits(e[lo:hi]), bits(want)), f"{tag} worker {i} block {b}"
    return stats


def run_steps(gpu, ora, grads_fn, steps, device="cuda", check_every=1, check_error=True, tag="", offsets=None):
    """grads_fn(step) -> float32 [n, d].  Feeds identical bytes to both sides."""
    import torch
    all_stats = []
    for t in range(steps):
        g = grads_fn(t)
        gd = torch.from_numpy(g).to(device)
        gpu.step(gd)
        ora_e_prev = ora.error.copy() if (check_every and gpu.d * gpu.n <= 50_000_000) else None
        ora.step(g)
        if check_every and ((t + 1) % check_every == 0 or t == steps - 1):
            x = (g + ora_e_prev) if ora_e_prev is not None else None
            all_stats.append(compare(gpu, ora, x_for_values=x, check_error=check_error, tag=f"{tag} step {t}",
                                     offsets=offsets))
        gpu.sync()
        del gd
    return all_stats
