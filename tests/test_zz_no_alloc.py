"""comp_ams_pack_message_noalloc (the entry point for callers that cannot allocate: its gather works
in a fixed array of device memory inside the library) against comp_ams_pack_message, through the C
ABI: the same bytes, on two calls in a row of which the second is smaller (the array keeps the first
call's contents), for every vector of a handle, both kinds of message, and the size limit."""
import ctypes as C

import numpy as np
import pytest

import paper_2111_00705_amd as P
import workloads as W

pytestmark = pytest.mark.gpu
f32 = np.float32


def run_steps(h, d, n, steps, seed):
    import torch
    for t in range(steps):
        g = np.random.default_rng([seed, t]).standard_normal((n, d)).astype(f32)
        g[:, ::97] = 0.0
        h.step(torch.from_numpy(g).cuda())
    h.sync()


def both_messages(h, who):
    """(bytes of comp_ams_pack_message, bytes of comp_ams_pack_message_noalloc) as uint8 arrays, raw ABI calls."""
    import torch
    L = P.lib()
    need = h.message_bytes()
    outs = []
    for fn in (L.comp_ams_pack_message, L.comp_ams_pack_message_noalloc):
        buf = torch.full((need + 64,), 0xAB, dtype=torch.uint8, device="cuda")
        got = C.c_uint64(0)
        rc = fn(h._h, who, buf.data_ptr(), buf.numel(), C.byref(got))
        assert rc == P.OK, L.comp_ams_last_error(h._h)
        assert got.value == need
        assert L.comp_ams_sync(h._h) == P.OK
        host = buf.cpu().numpy()
        assert (host[need:] == 0xAB).all(), "wrote past the message"
        outs.append(host[:need].copy())
    return outs


def sorted_pairs(raw):
    pairs = raw.view(np.uint32).reshape(-1, 2)
    return pairs[np.argsort(pairs[:, 0], kind="stable")]


@pytest.mark.parametrize("comp", [P.TOPK, P.RANDK])
@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD])
def test_sparse_message_equals_the_allocating_entry_point_on_two_calls_in_a_row(comp, method):
    print(f"[case] no-alloc sparse comp={comp} method={method}", flush=True)
    handles = []
    for d, n, k, seed in ((200_003, 3, 2_000, 5), (5_001, 2, 50, 6)):       # the second call is the smaller one
        h = P.CompAms(d, n, comp, k, W.BETA1, W.BETA2, W.EPS, W.LR)
        h.set_method(method)
        run_steps(h, d, n, 3, seed)
        handles.append((h, n, k))
    for rounds in range(2):                      # large, small, large, small: stale contents either way
        for h, n, k in handles:
            for who in range(n + (1 if method == P.METHOD_CD else 0)):
                ref, got = both_messages(h, who)
                a, b = sorted_pairs(ref), sorted_pairs(got)
                assert a.shape == (k, 2) and np.array_equal(a, b), (who, rounds)
                assert np.unique(a[:, 0]).size == k
                if who < n:
                    idx, val = h.get_selected(who)
                    assert np.array_equal(a[:, 0], idx) and np.array_equal(a[:, 1], val.view(np.uint32))
    for h, _, _ in handles:
        h.destroy()


def test_fewer_nonzeros_than_k_takes_the_zero_tail_through_the_scratch_array():
    """Error feedback with Top-k keeps zeros by lower index when fewer than k coordinates are non-zero: those
    come from the stored row, appended after the listed candidates."""
    import torch
    print("[case] no-alloc zero tail", flush=True)
    d, n, k = 50_000, 2, 500
    h = P.CompAms(d, n, P.TOPK, k)
    g = np.zeros((n, d), f32)
    g[:, 1000:1200] = np.random.default_rng(3).standard_normal((n, 200)).astype(f32)
    h.step(torch.from_numpy(g).cuda())
    for who in range(n):
        ref, got = both_messages(h, who)
        assert np.array_equal(sorted_pairs(ref), sorted_pairs(got))
        assert np.count_nonzero(sorted_pairs(got)[:, 1]) <= 200
    h.destroy()


@pytest.mark.parametrize("method", [P.METHOD_EF, P.METHOD_CD])
def test_sign_message_equals_the_allocating_entry_point(method):
    print(f"[case] no-alloc sign method={method}", flush=True)
    for d, n, block in ((70_001, 3, 1000), (4_097, 2, 64)):
        h = P.CompAms(d, n, P.BLOCKSIGN, block)
        h.set_method(method)
        run_steps(h, d, n, 2, 9)
        for who in range(n + (1 if method == P.METHOD_CD else 0)):
            ref, got = both_messages(h, who)
            assert np.array_equal(ref, got), who
        h.destroy()


def test_size_limit_and_argument_errors():
    import torch
    print("[case] no-alloc limits", flush=True)
    L = P.lib()
    d, n, k = 1_200_000, 1, (1 << 20) + 1
    h = P.CompAms(d, n, P.TOPK, k)
    buf = torch.zeros(8 * k, dtype=torch.uint8, device="cuda")
    got = C.c_uint64(0)
    assert L.comp_ams_pack_message_noalloc(h._h, 0, buf.data_ptr(), buf.numel(), C.byref(got)) == P.ESTATE   # no step yet
    h.step(torch.randn(n, d, device="cuda"))
    assert L.comp_ams_pack_message_noalloc(h._h, 0, buf.data_ptr(), buf.numel(), C.byref(got)) == P.EINVAL   # k too large
    assert b"exceeds" in L.comp_ams_last_error(h._h)
    assert got.value == 8 * k
    assert L.comp_ams_pack_message(h._h, 0, buf.data_ptr(), buf.numel(), C.byref(got)) == P.OK           # the other one still serves
    h.destroy()
    h = P.CompAms(10_000, 2, P.TOPK, 1 << 10)
    h.step(torch.randn(2, 10_000, device="cuda"))
    assert L.comp_ams_pack_message_noalloc(h._h, 2, buf.data_ptr(), buf.numel(), C.byref(got)) == P.EINVAL   # no such vector
    assert L.comp_ams_pack_message_noalloc(h._h, 0, None, 0, C.byref(got)) == P.EINVAL
    assert L.comp_ams_pack_message_noalloc(h._h, 0, buf.data_ptr() + 4, 1 << 20, C.byref(got)) == P.EINVAL   # alignment
    assert L.comp_ams_pack_message_noalloc(h._h, 0, buf.data_ptr(), 8, C.byref(got)) == P.EINVAL             # too small
    assert got.value == 8 * (1 << 10)
    assert L.comp_ams_pack_message_noalloc(None, 0, buf.data_ptr(), buf.numel(), C.byref(got)) == P.EINVAL
    h.destroy()
