"""Randomly drawn (seeded) shapes, compressors, methods and gradient streams: the HIP library through the C ABI
against the CPU oracle, compared after every step.  The draws mix what the fixed cases hold one at a time -
odd dimensions, one worker or dozens, k from 1 to d, blocks from 1 to beyond d, steps whose scale jumps by a
thousand either way, all-zero steps, sparse supports, quantised values with many ties, a cluster of large
entries - so that the paths which only inputs can choose (candidate lists that overflow, guesses that miss,
thresholds among zeros, short and long vectors, the pass that carries the previous update) meet each other.

Bars as everywhere: kept sets, kept values and error memory bit-exact; theta, m, v, vhat within 1e-6 relative;
block scales within 1e-5 relative.
"""
import os

import numpy as np
import pytest

import paper_2111_00705_amd as P
from oracle import oracle as O
from parity_util import compare, make_pair, run_steps
from test_gpu_cd_adam import make_cd_pair, make_cd_topk_pair, run_cd, run_cd_topk
from test_gpu_methods import make as make_method_pair, run as run_method

pytestmark = pytest.mark.gpu
f32 = np.float32
# other draws than the committed ones: COMP_AMS_SEED_BASE=1000 python -m pytest tests/test_gpu_random_shapes.py
BASE = int(os.environ.get("COMP_AMS_SEED_BASE", "0"))
# larger shapes (the oracle then takes seconds per step): COMP_AMS_SHAPE_SCALE=16
SCALE = int(os.environ.get("COMP_AMS_SHAPE_SCALE", "1"))


def announce(msg):
    print(f"[case] {msg}", flush=True)


def draw_shape(rng, budget):
    """n and d with n * d <= budget; d log-uniform so that short vectors (one tile, a few tiles) are as likely as
    long ones."""
    n = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 33]))
    d_max = max(2, budget * SCALE // n)
    d = int(np.exp(rng.uniform(np.log(1.0) if rng.random() < 0.25 else np.log(min(3000.0, d_max)), np.log(d_max))))
    d = max(1, min(d, d_max))
    if rng.random() < 0.3:                          # a tile boundary, one short of it or one beyond
        d = max(1, (max(d, 4096) // 4096) * 4096 + int(rng.integers(-1, 2)))
    return n, d


def draw_k(rng, d):
    kind = rng.integers(0, 5)
    if kind == 0:
        return 1
    if kind == 1:
        return d
    if kind == 2:
        return max(1, d // 100)
    if kind == 3:
        return max(1, d // 2)
    return int(rng.integers(1, d + 1))


def draw_block(rng, d):
    kind = rng.integers(0, 6)
    if kind == 0:
        return 1
    if kind == 1:
        return 4096
    if kind == 2:
        return 8192
    if kind == 3:
        return d + int(rng.integers(0, 3))          # whole-vector sign
    if kind == 4:
        return int(rng.choice([3, 64, 100, 255, 1000, 5000]))
    return int(rng.integers(1, max(2, d)))


def gradient_stream(seed, n, d):
    """grads(t) -> float32 [n, d]; every step draws its own scale, support and value grid."""
    base = np.random.default_rng([seed, 1])
    seg = max(1, d // int(base.integers(1, 9)))
    layer_scale = np.exp(base.normal(0.0, 1.5, size=(d + seg - 1) // seg)).repeat(seg)[:d].astype(f32)

    def grads(t):
        rng = np.random.default_rng([seed, 2, t])
        g = rng.standard_normal((n, d)).astype(f32) * layer_scale
        what = rng.integers(0, 10)
        if what == 0:
            g[:] = 0.0                                               # nothing arrives
        elif what == 1:
            g *= f32(1e3)                                            # the scale jumps up
        elif what == 2:
            g *= f32(1e-3)                                           # and down
        elif what == 3:
            g *= (rng.random((n, d)) < 10.0 ** rng.uniform(-3, -0.3)).astype(f32)   # sparse support
        elif what == 4:
            g = (np.round(g * 2.0) / 2.0).astype(f32)                # few distinct magnitudes: ties everywhere
        elif what == 5:
            lo = int(rng.integers(0, d))
            g[:, lo:lo + max(1, d // 50)] *= f32(300.0)              # a cluster that holds most of the top
        elif what == 6:
            g[int(rng.integers(0, n))] = 0.0                         # one silent worker
        return np.ascontiguousarray(g, dtype=f32)

    return grads


@pytest.mark.parametrize("seed", range(72))
def test_error_feedback_random_case(seed):
    seed += BASE
    rng = np.random.default_rng([seed, 0])
    n, d = draw_shape(rng, 5_000_000)
    comp = [P.TOPK, P.BLOCKSIGN, P.RANDK][int(rng.integers(0, 3))]
    kb = draw_block(rng, d) if comp == P.BLOCKSIGN else draw_k(rng, d)
    announce(f"error feedback, seed {seed}: compressor {comp}, n={n}, d={d}, k or block={kb}")
    gpu, ora = make_pair(d, n, comp, kb, theta0=rng.standard_normal(d).astype(f32))
    if comp == P.RANDK:
        gpu.set_rand(1234 + seed, 0)
        ora.set_rand(1234 + seed, 0)
    offsets = None
    if comp == P.BLOCKSIGN:
        offsets = np.minimum(np.arange((d + kb - 1) // kb + 1, dtype=np.int64) * kb, d)
    run_steps(gpu, ora, gradient_stream(seed, n, d), steps=6, tag=f"seed {seed}", offsets=offsets)
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("seed", range(100, 130))
def test_cd_adam_random_case(seed):
    seed += BASE
    rng = np.random.default_rng([seed, 0])
    n, d = draw_shape(rng, 3_000_000)
    grads = gradient_stream(seed, n, d)
    if rng.random() < 0.5:
        k = draw_k(rng, d)
        announce(f"CD-Adam, seed {seed}: Top-k, n={n}, d={d}, k={k}")
        gpu, ora = make_cd_topk_pair(d, n, k, theta0=rng.standard_normal(d).astype(f32))
        run_cd_topk(gpu, ora, grads, 5, f"seed {seed}")
    else:
        block = draw_block(rng, d)
        announce(f"CD-Adam, seed {seed}: block sign, n={n}, d={d}, block={block}")
        gpu, ora = make_cd_pair(d, n, block, theta0=rng.standard_normal(d).astype(f32))
        run_cd(gpu, ora, grads, 5, f"seed {seed}")
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("seed", range(200, 224))
def test_naive_compression_random_case(seed):
    seed += BASE
    rng = np.random.default_rng([seed, 0])
    n, d = draw_shape(rng, 3_000_000)
    comp = [P.TOPK, P.BLOCKSIGN][int(rng.integers(0, 2))]
    kb = draw_block(rng, d) if comp == P.BLOCKSIGN else draw_k(rng, d)
    announce(f"naive compression, seed {seed}: compressor {comp}, n={n}, d={d}, k or block={kb}")
    gpu, ora = make_method_pair(d, n, comp, kb, O.NAIVE, theta0=rng.standard_normal(d).astype(f32))
    run_method(gpu, ora, gradient_stream(seed, n, d), 5, f"seed {seed}")
    gpu.destroy()
    ora.close()


@pytest.mark.parametrize("seed", range(300, 330))
def test_error_feedback_random_case_with_16_bit_gradients(seed):
    """The same draws with the gradients handed over as bfloat16 or half precision: the step must equal the step on
    the widened values (which is what the oracle gets)."""
    import torch
    seed += BASE
    rng = np.random.default_rng([seed, 0])
    n, d = draw_shape(rng, 3_000_000)
    comp = [P.TOPK, P.BLOCKSIGN, P.RANDK][int(rng.integers(0, 3))]
    kb = draw_block(rng, d) if comp == P.BLOCKSIGN else draw_k(rng, d)
    narrow = [torch.bfloat16, torch.float16][int(rng.integers(0, 2))]
    announce(f"error feedback, {narrow}, seed {seed}: compressor {comp}, n={n}, d={d}, k or block={kb}")
    gpu, ora = make_pair(d, n, comp, kb, theta0=rng.standard_normal(d).astype(f32))
    if comp == P.RANDK:
        gpu.set_rand(99 + seed, 0)
        ora.set_rand(99 + seed, 0)
    offsets = None
    if comp == P.BLOCKSIGN:
        offsets = np.minimum(np.arange((d + kb - 1) // kb + 1, dtype=np.int64) * kb, d)
    grads = gradient_stream(seed, n, d)
    for t in range(5):
        g16 = torch.from_numpy(np.clip(grads(t), -6e4, 6e4)).to(narrow).cuda()        # half precision ends at 65504
        wide = g16.float().cpu().numpy()
        e_prev = ora.error.copy()
        (gpu.step_bf16 if narrow == torch.bfloat16 else gpu.step_f16)(g16)
        ora.step(wide)
        compare(gpu, ora, x_for_values=wide + e_prev, tag=f"seed {seed} step {t}", offsets=offsets)
    gpu.destroy()
    ora.close()
