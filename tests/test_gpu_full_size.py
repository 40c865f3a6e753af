"""GPU parity at the full sizes of the three large workloads, in the launch configuration that
bench.py times (same create arguments, same kernels), against the CPU oracle run in full on the
same gradient bytes.  Fewer steps than the workloads name (the oracle's full sorts take tens of
seconds per step at d = 110 M), but more than one, so that the error memory, the carried
threshold guess and the deferred error form are all exercised at scale.  The whole state is
compared element by element; bars are those of tests/parity_util.py."""
import numpy as np
import pytest

import workloads as W
from parity_util import make_pair, pair_for, run_steps

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("idx,steps", [(2, 3), (3, 2), (4, 2)])
def test_full_size_workload_matches_oracle(idx, steps):
    w = W.get(idx)
    print(f"[case] full size {w.name}, {steps} steps", flush=True)
    gpu, ora = pair_for(w)
    s = w.scales()

    def grads(t):
        print(f"[case] {w.name}: generating step {t}", flush=True)
        return w.grads(t, scales=s, threads=16)

    stats = run_steps(gpu, ora, grads, steps=steps, tag=w.name, check_every=1, offsets=w.block_offsets())
    print(f"[case] {w.name}: {stats[-1]}", flush=True)
    gpu.destroy()
    ora.close()


def test_full_size_randk_matches_oracle():
    """Rand-k (Appendix A) at the size and launch configuration of the 11 M-coordinate workload: the
    score threshold, the carried guess and the deferred error memory at scale, three steps."""
    import paper_2111_00705_amd as P
    w = W.get(2)
    print(f"[case] full size Rand-k on {w.name}", flush=True)
    gpu, ora = make_pair(w.d, w.n, P.RANDK, w.k, w.beta1, w.beta2, w.eps, w.lr, theta0=w.theta0())
    gpu.set_rand(0x1234567887654321, 0)
    ora.set_rand(0x1234567887654321, 0)
    s = w.scales()
    stats = run_steps(gpu, ora, lambda t: w.grads(t, scales=s, threads=16), steps=3, tag="randk " + w.name)
    print(f"[case] randk {w.name}: {stats[-1]}", flush=True)
    gpu.destroy()
    ora.close()
