"""GPU parity of the paper's comparison arms - naive compression (Section 4) and no compression
(vanilla distributed AMSGrad, Section 3) - against the CPU oracle, element by element.
Bars as in tests/parity_util.py: kept index sets and kept values bit-exact, block scales within
1e-5 relative, theta, m, v, vhat within 1e-6 relative per coordinate."""
import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W
from oracle import oracle as O
from parity_util import SCALE_RTOL, STATE_RTOL, bits, rel_close

pytestmark = pytest.mark.gpu
f32 = np.float32


def torch_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def announce(msg):
    print(f"[case] {msg}", flush=True)


def make(d, n, comp, kb, method, theta0=None, offsets=None):
    gpu = P.CompAms(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    if offsets is not None:
        gpu.set_blocks(offsets)
        ora.set_blocks(offsets)
    if theta0 is not None:
        gpu.set_theta(np.ascontiguousarray(theta0, dtype=f32))
        ora.set_theta(theta0)
    return gpu, ora


def run(gpu, ora, grads_fn, steps, tag):
    for t in range(steps):
        g = grads_fn(t)
        gpu.step(torch_dev(g))
        ora.step(g)
        if ora.method == O.NAIVE and gpu.compressor == P.TOPK:
            for i in range(gpu.n):
                idx, val = gpu.get_selected(i)
                assert np.array_equal(idx, ora.selected[i]), f"{tag} step {t} worker {i}: kept index set differs"
                assert np.array_equal(bits(val), bits(g[i][idx])), f"{tag} step {t} worker {i}: kept values differ"
        if ora.method == O.NAIVE and gpu.compressor == P.BLOCKSIGN:
            assert rel_close(gpu.get_scales(), ora.scales, SCALE_RTOL).all(), f"{tag} step {t}: scales"
        for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("m", gpu.get_m(), ora.m),
                                ("v", gpu.get_v(), ora.v), ("vhat", gpu.get_vhat(), ora.vhat)):
            ok = rel_close(got, want, STATE_RTOL)
            assert ok.all(), f"{tag} step {t} {name}: {np.count_nonzero(~ok)} coordinates beyond {STATE_RTOL}"


def noise(seed, n, d, scale):
    return lambda t: (np.random.default_rng([seed, t]).standard_normal((n, d)) * scale).astype(f32)


@pytest.mark.parametrize("d,n", [(1, 1), (5, 3), (4097, 2), (10_007, 5), (3 * 4096, 4), (150_001, 16), (9000, 70)])
def test_uncompressed_amsgrad(d, n):
    announce(f"no compression d={d} n={n}")
    rng = np.random.default_rng(d + n)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    gpu, ora = make(d, n, P.TOPK, 1, P.METHOD_NONE, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run(gpu, ora, noise(d, n, d, scale), steps=4, tag=f"none d={d}")
    for call in (lambda: gpu.get_selected(0), lambda: gpu.get_error(0)):
        with pytest.raises(P.CompAmsError) as ei:
            call()
        assert ei.value.code == P.ESTATE
    gpu.destroy()


def test_uncompressed_amsgrad_any_gradient_alignment():
    import torch
    announce("no compression, unaligned gradient rows")
    d, n = 10_001, 3                      # odd d: rows start at every 4-byte alignment class
    gpu, ora = make(d, n, P.BLOCKSIGN, 64, P.METHOD_NONE)
    for t in range(3):
        g = np.random.default_rng([77, t]).standard_normal((n, d)).astype(f32)
        buf = torch.empty(n * d + 3, dtype=torch.float32, device="cuda")
        view = buf[1 + t % 3: 1 + t % 3 + n * d]
        view.copy_(torch.from_numpy(g).reshape(-1))
        gpu.step_ptr(view.data_ptr(), torch.cuda.current_stream().cuda_stream)
        ora.step(g)
        assert rel_close(gpu.get_theta(), ora.theta, STATE_RTOL).all()
        assert np.array_equal(bits(gpu.get_vhat()), bits(ora.vhat))
    gpu.destroy()


@pytest.mark.parametrize("d,n,k", [(1, 1, 1), (63, 2, 7), (4097, 2, 41), (10_007, 5, 100), (20_000, 3, 20_000),
                                   (300_003, 8, 3000)])
def test_naive_topk(d, n, k):
    announce(f"naive Top-k d={d} n={n} k={k}")
    rng = np.random.default_rng(d * 3 + n)
    scale = np.exp(rng.uniform(-6, 0, d)).astype(f32)
    gpu, ora = make(d, n, P.TOPK, k, P.METHOD_NAIVE, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    factors = [1.0, 1.0, 50.0, 1e-3, 1.0]           # the carried guess must survive scale changes here too
    run(gpu, ora, lambda t: noise(d, n, d, scale)(t) * f32(factors[t]), steps=5, tag=f"naive topk d={d}")
    gpu.destroy()


@pytest.mark.parametrize("d,n,B", [(7, 2, 3), (4096, 2, 4096), (10_007, 5, 100), (3 * 4096 + 5, 4, 8192), (150_001, 16, 4096)])
def test_naive_blocksign(d, n, B):
    announce(f"naive block sign d={d} n={n} B={B}")
    rng = np.random.default_rng(d * 5 + n)
    scale = np.exp(rng.uniform(-5, 0, d)).astype(f32)
    gpu, ora = make(d, n, P.BLOCKSIGN, B, P.METHOD_NAIVE, theta0=(0.01 * rng.standard_normal(d)).astype(f32))
    run(gpu, ora, noise(d + 1, n, d, scale), steps=4, tag=f"naive sign d={d}")
    gpu.destroy()


def test_naive_blocksign_layer_blocks():
    announce("naive block sign, layer blocks")
    d, n = 70_003, 3
    offsets = [0, 1, 2, 300, 4096, 4097, 9000, 30_000, 30_001, 65_536, d]
    gpu, ora = make(d, n, P.BLOCKSIGN, d, P.METHOD_NAIVE, offsets=offsets)
    run(gpu, ora, noise(9, n, d, f32(1.0)), steps=3, tag="naive layers")
    gpu.destroy()


def test_case_study_ordering_of_the_four_strategies_on_gpu():
    """Section 6.1 on the GPU library: same problem, same settings and same assertion as the oracle's
    test of that name; the models must also agree with the oracle's at the end."""
    announce("logistic regression case study")
    a, y = W.logreg_problem()
    n, _, d = a.shape
    norm = {}
    for name, method in (("none", P.METHOD_NONE), ("cd", P.METHOD_CD), ("ef", P.METHOD_EF), ("naive", P.METHOD_NAIVE)):
        gpu = P.CompAms(d, n, P.BLOCKSIGN, 16, 0.9, 0.999, 1e-3, 0.003)
        ora = O.Oracle(d, n, O.BLOCKSIGN, 16, 0.9, 0.999, 1e-3, 0.003, method=method)
        gpu.set_method(method)
        gpu.set_eps_mode(1)
        ora.set_eps_mode(1)
        theta = np.zeros(d, f32)
        for _ in range(1500):
            g = W.logreg_grads(a, y, theta)
            gpu.step(torch_dev(g))
            theta = gpu.get_theta()
        for _ in range(1500):
            ora.step(W.logreg_grads(a, y, ora.theta))
        norm[name] = float(np.linalg.norm(W.logreg_grads(a, y, theta).astype(np.float64).mean(axis=0)))
        assert np.allclose(theta, ora.theta, rtol=1e-3, atol=1e-5), name
        gpu.destroy()
        ora.close()
    assert norm["none"] < 1e-6
    assert norm["cd"] < 1e-2 * norm["ef"], norm
    assert norm["ef"] < 1e-1 * norm["naive"], norm


def test_message_bits_follow_the_papers_accounting():
    """The table "Average runtime and total bits": uncompressed 32 d per direction, CD-Adam with the
    whole-vector scaled sign (32 + d) per direction, Top-k about 64 k per message."""
    announce("message bits")
    d, n, k = 10_000, 4, 160
    h = P.CompAms(d, n, P.BLOCKSIGN, d)
    assert h.message_bits() == (32 + d, 32 * d)                   # error feedback: only the upload is compressed
    h.set_method(P.METHOD_CD)
    assert h.message_bits() == (32 + d, 32 + d)
    h.destroy()
    h = P.CompAms(d, n, P.BLOCKSIGN, 4096)
    h.set_method(P.METHOD_CD)
    assert h.message_bits() == (d + 32 * 3, d + 32 * 3)           # three blocks, three scales
    h.set_blocks([0, 10, 20, 30, d])
    assert h.message_bits() == (d + 32 * 4, d + 32 * 4)
    h.destroy()
    h = P.CompAms(d, n, P.TOPK, k)
    assert h.message_bits() == (64 * k, 32 * d)
    h.set_method(P.METHOD_NAIVE)
    assert h.message_bits() == (64 * k, 32 * d)
    h.set_method(P.METHOD_CD)
    assert h.message_bits() == (64 * k, 64 * k)
    h.set_method(P.METHOD_NONE)
    assert h.message_bits() == (32 * d, 32 * d)
    h.destroy()


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_NAIVE, P.METHOD_CD])
def test_scaled_sign_message_rebuilt_from_bits_and_scales(method):
    """What goes over the wire - one bit per coordinate and one scale per block - must rebuild the
    oracle's compressed vectors C(.) of every worker (and of the server for CD-Adam) exactly."""
    announce(f"sign message, method {method}")
    d, n = 70_003, 3
    offsets = np.array([0, 1, 2, 300, 4096, 4097, 9000, 30_000, 30_001, 65_536, d])
    gpu, ora = make(d, n, P.BLOCKSIGN, d, method, offsets=offsets)
    block_of = np.repeat(np.arange(offsets.size - 1), np.diff(offsets))

    def rebuild(bits_packed, scales):
        neg = np.unpackbits(bits_packed, bitorder="little")[:d].astype(bool)
        return np.where(neg, -scales[block_of], scales[block_of]).astype(f32)

    for t in range(3):
        g = np.random.default_rng([55, t]).standard_normal((n, d)).astype(f32)
        g[1, 100:200] = -0.0
        gpu.step(torch_dev(g))
        ora.step(g)
        s = gpu.get_scales()
        assert np.array_equal(bits(s), bits(ora.scales)), "scales are expected bit-identical on this input"
        for i in range(n):
            assert np.array_equal(bits(rebuild(gpu.get_signs(i), s[i])), bits(ora.compressed[i])), (t, i)
        if method == P.METHOD_CD:
            msg = rebuild(gpu.get_signs(n), gpu.get_server_scales())
            assert np.array_equal(bits(msg), bits(ora.server_compressed)), t
    with pytest.raises(P.CompAmsError) as ei:
        gpu.get_signs(n if method != P.METHOD_CD else n + 1)
    assert ei.value.code == P.EINVAL
    gpu.destroy()


@pytest.mark.parametrize("comp,kb,method", [(P.TOPK, 300, P.METHOD_EF), (P.BLOCKSIGN, 4096, P.METHOD_EF),
                                            (P.TOPK, 300, P.METHOD_CD), (P.BLOCKSIGN, 1000, P.METHOD_CD),
                                            (P.RANDK, 300, P.METHOD_EF), (P.RANDK, 300, P.METHOD_CD)])
def test_a_step_can_be_captured_in_a_graph_and_replayed(comp, kb, method):
    """comp_ams_step allocates nothing and clears its counters in kernels, so a caller may capture it.
    The captured step is replayed several times, with fresh gradients copied into the captured buffer
    by ordinary eager work in between, and every replay is checked against the oracle.
    Rand-k: a replayed step repeats the draw it was recorded with, so the oracle's draw is held at
    that number; under error feedback the deferred error memory of each replay must then be read with
    the draw of its predecessor - the same draw from the second replay on."""
    import torch
    announce(f"graph capture comp={comp} method={method}")
    d, n = 30_011, 4
    gpu = P.CompAms(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR)
    ora = O.Oracle(d, n, comp, kb, W.BETA1, W.BETA2, W.EPS, W.LR, method=method)
    gpu.set_method(method)
    seed = 0xfeedface12345678
    if comp == P.RANDK:
        gpu.set_rand(seed, 0)
        ora.set_rand(seed, 0)
    grads = [np.random.default_rng([13, t]).standard_normal((n, d)).astype(f32) for t in range(7)]
    side = torch.cuda.Stream()
    gbuf = torch.empty((n, d), dtype=torch.float32, device="cuda")
    with torch.cuda.stream(side):
        for t in range(2):                                 # eager steps on the stream that will capture
            gbuf.copy_(torch.from_numpy(grads[t]))
            gpu.step(gbuf)
            ora.step(grads[t])
    side.synchronize()
    gpu.sync()                                             # nothing of the eager steps may be pending at capture
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.step(gbuf)                                     # recorded, not run
    for t in range(2, 7):
        with torch.cuda.stream(side):
            gbuf.copy_(torch.from_numpy(grads[t]))
        side.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        if comp == P.RANDK:
            ora.set_rand(seed, 2)                          # the recorded step was the third: draw number 2
        ora.step(grads[t])
        for name, got, want in (("theta", gpu.get_theta(), ora.theta), ("vhat", gpu.get_vhat(), ora.vhat)):
            ok = rel_close(got, want, STATE_RTOL)
            assert ok.all(), f"replay {t} {name}: {np.count_nonzero(~ok)} coordinates differ"
        if method == P.METHOD_EF:
            assert np.array_equal(bits(gpu.get_error(1)), bits(ora.error[1])), t
        else:
            assert np.array_equal(bits(gpu.get_ghat_worker(1)), bits(ora.ghat_workers[1])), t
        if comp != P.BLOCKSIGN:
            assert np.array_equal(gpu.get_selected(2)[0], ora.selected[2]), t
    gpu.destroy()


@pytest.mark.parametrize("comp,kb", [(P.TOPK, 300), (P.BLOCKSIGN, 1000)])
@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD])
def test_the_cache_policy_does_not_change_results(comp, kb, method):
    """comp_ams_set_streaming only picks load / store flavours: every combination, also switched between
    steps, must leave bit-identical state."""
    import torch
    announce(f"cache policy comp={comp} method={method}")
    d, n = 30_011, 3
    gs = [np.random.default_rng([77, t]).standard_normal((n, d)).astype(f32) for t in range(4)]
    ref = None
    for rows, state in ((-1, -1), (0, 0), (1, 1), (0, 1), (1, 0)):
        h = P.CompAms(d, n, comp, kb)
        h.set_method(method)
        h.set_streaming(rows, state)
        for t, g in enumerate(gs):
            if t == 2:
                h.set_streaming(state, rows)          # swapped, between steps
            h.step(torch.from_numpy(g).cuda())
        out = [bits(h.get_theta()), bits(h.get_m()), bits(h.get_v()), bits(h.get_vhat())]
        out += [bits(h.get_error(i) if method == P.METHOD_EF else h.get_ghat_worker(i)) for i in range(n)]
        h.destroy()
        if ref is None:
            ref = out
        else:
            assert all(np.array_equal(a, b) for a, b in zip(ref, out)), (rows, state)
    h = P.CompAms(64, 1, comp, 8)
    with pytest.raises(P.CompAmsError):
        h.set_streaming(2, 0)
    h.destroy()


def test_the_tile_order_does_not_change_the_uncompressed_update():
    """The update without compression takes its tiles in the order comp_ams_set_tile_order names as well: any
    chunk, and a change between steps, must leave bit-identical state (74 tiles, the last one ragged)."""
    import torch
    announce("tile order, no compression")
    d, n = 300_007, 5
    gs = [np.random.default_rng([79, t]).standard_normal((n, d)).astype(f32) for t in range(3)]
    ref = None
    for chunk in (0, 1, 3, 16, 37, 100, -1):
        h = P.CompAms(d, n, P.TOPK, 10)
        h.set_method(P.METHOD_NONE)
        h.set_tile_order(chunk)
        for t, g in enumerate(gs):
            if t == 2:
                h.set_tile_order(7 if chunk else 4)
            h.step(torch.from_numpy(g).cuda())
        out = [bits(h.get_theta()), bits(h.get_m()), bits(h.get_v()), bits(h.get_vhat())]
        h.destroy()
        if ref is None:
            ref = out
        else:
            assert all(np.array_equal(a, b) for a, b in zip(ref, out)), chunk


@pytest.mark.parametrize("comp,kb", [(P.TOPK, 3000), (P.RANDK, 3000), (P.BLOCKSIGN, 1000), (P.BLOCKSIGN, 4096)])
@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD, P.METHOD_NAIVE])
def test_the_tile_order_does_not_change_results(comp, kb, method):
    """comp_ams_set_tile_order only permutes which workgroup takes which tile, comp_ams_set_pass_lds only
    how many workgroups share a compute unit: chunks that divide the tile count, that do not, that exceed
    it, several LDS amounts and a switch between steps must leave bit-identical state.
    d = 300 007 is 74 tiles, the last one ragged."""
    import torch
    announce(f"tile order comp={comp} kb={kb} method={method}")
    d, n = 300_007, 3
    gs = [np.random.default_rng([78, t]).standard_normal((n, d)).astype(f32) for t in range(3)]
    ref = None
    for chunk in (0, 1, 2, 3, 5, 16, 37, 100, -1):
        h = P.CompAms(d, n, comp, kb)
        h.set_method(method)
        h.set_tile_order(chunk)
        h.set_pass_lds({0: -1, 1: 0, 2: 8192, 3: 30000, 5: 61440}.get(chunk, -1))
        for t, g in enumerate(gs):
            if t == 2:
                h.set_tile_order(7 if chunk else 4)          # changed between steps
            h.step(torch.from_numpy(g).cuda())
        out = [bits(h.get_theta()), bits(h.get_m()), bits(h.get_v()), bits(h.get_vhat())]
        if method == P.METHOD_EF:
            out += [bits(h.get_error(i)) for i in range(n)]
        elif method == P.METHOD_CD:
            out += [bits(h.get_ghat_worker(i)) for i in range(n)]
        if comp != P.BLOCKSIGN:
            out += [np.sort(h.get_selected(i)[0]) for i in range(n)]
        else:
            out += [bits(h.get_scales())]
        h.destroy()
        if ref is None:
            ref = out
        else:
            assert all(np.array_equal(a, b) for a, b in zip(ref, out)), chunk
    h = P.CompAms(64, 1, comp, 8)
    with pytest.raises(P.CompAmsError):
        h.set_tile_order(-2)
    with pytest.raises(P.CompAmsError):
        h.set_tile_order(65537)
    with pytest.raises(P.CompAmsError):
        h.set_pass_lds(-2)
    with pytest.raises(P.CompAmsError):
        h.set_pass_lds(61441)
    h.destroy()


@pytest.mark.parametrize("count", [4, 1020, 4096, 4100, 1 << 20, (1 << 20) + 12, 64 << 20, (80 << 20) + 4100 + 12])
def test_probe_copy_copies_exactly_what_it_is_given(count):
    """The plain copy that calibrates the HBM counters: dst == src, nothing written past the end.  From 256 MB
    on it runs in another launch shape (chunked piece order, padded grid): the last two sizes, one a whole
    number of chunk groups and one ragged."""
    import torch
    announce(f"probe_copy count={count}")
    src = torch.randn(count, device="cuda")
    dst = torch.full((count + 8,), -7.0, device="cuda")
    P.probe_copy(dst[:count], src)
    torch.cuda.synchronize()
    assert torch.equal(dst[:count], src)
    assert bool((dst[count:] == -7.0).all())


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD, P.METHOD_NAIVE])
@pytest.mark.parametrize("comp,d,kb", [(P.BLOCKSIGN, 30_011, 1000), (P.BLOCKSIGN, 4096 * 3, 4096), (P.BLOCKSIGN, 37, 100),
                                       (P.TOPK, 30_011, 300), (P.RANDK, 5_003, 77)])
def test_packed_messages_decode_to_the_oracles_compressed_vectors(method, comp, d, kb):
    """comp_ams_pack_message: the wire form of every worker's (and, for CD-Adam, the server's) message,
    decoded on the host, is C(.) of the oracle bit for bit; its size is the paper's bit count rounded up
    to whole 32-bit words."""
    import torch
    announce(f"pack method={method} comp={comp} d={d}")
    n = 3
    gpu = P.CompAms(d, n, comp, kb)
    ora = O.Oracle(d, n, comp, kb, 0.9, 0.999, 1e-8, 1e-3, method=method)
    gpu.set_method(method)
    for t in range(3):
        g = np.random.default_rng([d, comp, method, t]).standard_normal((n, d)).astype(f32)
        gpu.step(torch.from_numpy(g).cuda())
        ora.step(g)
    nbytes = gpu.message_bytes()
    up, down = gpu.message_bits()
    assert up <= 8 * nbytes < up + 32
    buf = torch.zeros(nbytes + 8, dtype=torch.uint8, device="cuda")
    with pytest.raises(P.CompAmsError):
        gpu.pack_message(0, buf[: nbytes - 8])
    vectors = [(i, ora.compressed[i]) for i in range(n)]
    if method == P.METHOD_CD:
        vectors.append((n, ora.server_compressed))
    for who, want in vectors:
        buf.fill_(0xAB)
        assert gpu.pack_message(who, buf) == nbytes
        raw = buf.cpu().numpy()
        assert (raw[nbytes:] == 0xAB).all(), "written past the message"
        got = np.zeros(d, f32)
        if comp == P.BLOCKSIGN:
            nb = gpu.n_blocks()
            scales = raw[: 4 * nb].view(f32)
            words = raw[4 * nb: nbytes].view(np.uint32)
            neg = ((words[np.arange(d) // 32] >> (np.arange(d) % 32).astype(np.uint32)) & 1).astype(bool)
            assert not (int(words[-1]) >> ((d - 1) % 32 + 1)) if d % 32 else True
            blk = np.minimum(np.arange(d) // kb, nb - 1)
            got = np.where(neg, -scales[blk], scales[blk]).astype(f32)
        else:
            pairs = raw[:nbytes].view(np.uint32).reshape(-1, 2)
            assert len(set(pairs[:, 0].tolist())) == kb and pairs[:, 0].max() < d
            got[pairs[:, 0]] = pairs[:, 1].copy().view(f32)
        assert np.array_equal(bits(got), bits(want)), f"vector {who}"
    gpu.destroy()
    ora.close()
