"""The C ABI used from C: tests/c/abi_roundtrip.c (built by paper_2111_00705_amd/build.py with gcc, device memory
from the HIP runtime, no Python or torch in the process) runs a seeded problem, and what it writes is compared
with the CPU oracle - the same bars as everywhere: error memory and Markov sequences bit-exact, theta, m, v, vhat
within 1e-6 relative."""
import os
import subprocess

import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import STATE_RTOL, bits, rel_close

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
EXE = os.path.join(ROOT, "tests", "c", "abi_roundtrip.bin")


@pytest.mark.parametrize("comp,kb,method", [(P.TOPK, 700, P.METHOD_EF), (P.BLOCKSIGN, 4096, P.METHOD_EF),
                                            (P.BLOCKSIGN, 1000, P.METHOD_CD), (P.TOPK, 700, P.METHOD_NAIVE)])
def test_a_c_program_gets_the_oracles_result(tmp_path, comp, kb, method):
    print(f"[case] C caller comp={comp} method={method}", flush=True)
    if not os.path.exists(EXE):                  # normally built with the library (paper_2111_00705_amd/build.py)
        from paper_2111_00705_amd import build as B
        B.build_c_caller()
    d, n, steps = 70_003, 3, 4
    rng = np.random.default_rng([comp, method])
    theta0 = (0.01 * rng.standard_normal(d)).astype(np.float32)
    scale = np.exp(rng.uniform(-4, 0, d)).astype(np.float32)
    grads = [(rng.standard_normal((n, d)).astype(np.float32) * scale) for _ in range(steps)]
    problem, result = tmp_path / "problem.bin", tmp_path / "result.bin"
    with open(problem, "wb") as f:
        np.array([d, n, comp, kb, method, steps], np.int64).tofile(f)
        theta0.tofile(f)
        for g in grads:
            np.ascontiguousarray(g).tofile(f)
    r = subprocess.run([EXE, str(problem), str(result)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True,
                       timeout=100)
    assert r.returncode == 0, r.stdout
    ora = O.Oracle(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    ora.set_theta(theta0)
    for g in grads:
        ora.step(g)
    got = np.fromfile(result, np.float32)
    rows = n if method in (P.METHOD_EF, P.METHOD_CD) else 0
    assert got.size == (4 + rows) * d
    got = got.reshape(4 + rows, d)
    for q, name in enumerate(("theta", "m", "v", "vhat")):
        assert rel_close(got[q], getattr(ora, name), STATE_RTOL).all(), name
    mem = ora.error if method == P.METHOD_EF else ora.ghat_workers if method == P.METHOD_CD else None
    for i in range(rows):
        assert np.array_equal(bits(got[4 + i]), bits(mem[i])), f"memory of worker {i}"
    ora.close()
