"""Thin ctypes binding of include/comp_ams.h.

Argument marshalling only: every step of the method runs in the HIP kernels of
libcomp_ams.so.  Tensors are torch CUDA(HIP) tensors used as device memory; the
current torch stream is passed through as the HIP stream.  If the library has
not been built the import of the library raises: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

TOPK = 0
BLOCKSIGN = 1
RANDK = 2
METHOD_EF = 0     # error feedback (Section 4)
METHOD_CD = 1     # CD-Adam (Section 5, Algorithm 1)
METHOD_NAIVE = 2  # naive compression (Section 4), no memory
METHOD_NONE = 3   # no compression (vanilla distributed AMSGrad, Section 3)

OK, EINVAL, ENOMEM, EDEVICE, ESTATE = 0, -1, -2, -3, -4

EXPORTS = [
    "comp_ams_create", "comp_ams_destroy", "comp_ams_set_blocks", "comp_ams_set_theta", "comp_ams_set_lr",
    "comp_ams_set_eps_mode", "comp_ams_step", "comp_ams_get_theta", "comp_ams_get_m", "comp_ams_get_v",
    "comp_ams_get_vhat", "comp_ams_get_error", "comp_ams_get_selected", "comp_ams_get_scales",
    "comp_ams_n_blocks", "comp_ams_set_state", "comp_ams_sync", "comp_ams_last_error", "comp_ams_profile",
    "comp_ams_profile_read", "comp_ams_probe_copy", "comp_ams_get_selection_info",
    "comp_ams_set_method", "comp_ams_get_ghat_worker", "comp_ams_get_ghat_server", "comp_ams_get_gtilde",
    "comp_ams_get_server_scales", "comp_ams_set_markov_state", "comp_ams_get_server_selected",
    "comp_ams_message_bits", "comp_ams_get_signs", "comp_ams_step_bf16", "comp_ams_step_f16", "comp_ams_set_rand", "comp_ams_set_streaming", "comp_ams_set_tile_order", "comp_ams_set_pass_lds", "comp_ams_message_bytes", "comp_ams_pack_message",
    "comp_ams_pack_message_noalloc", "comp_ams_probe_update",
]


class CompAmsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"comp_ams status {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Loads the in-tree HIP library (building it only if no build exists)."""
    global _lib
    if _lib is None:
        # torch ships its own HIP runtime; importing it first makes this library bind to that same
        # copy (matched by soname) instead of bringing a second runtime into the process
        import torch  # noqa: F401
        if not os.path.exists(_build.LIB):
            _build.build(force=True)
        L = C.CDLL(_build.LIB)
        vp, fp, i64p, u32p = C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), C.POINTER(C.c_uint32)
        L.comp_ams_create.argtypes = [C.POINTER(vp), C.c_int64, C.c_int32, C.c_int32, C.c_int64, C.c_float,
                                      C.c_float, C.c_float, C.c_float]
        L.comp_ams_destroy.argtypes = [vp]
        L.comp_ams_destroy.restype = None
        L.comp_ams_set_blocks.argtypes = [vp, i64p, C.c_int32]
        L.comp_ams_set_theta.argtypes = [vp, fp, C.c_int]
        L.comp_ams_set_lr.argtypes = [vp, C.c_float]
        L.comp_ams_set_eps_mode.argtypes = [vp, C.c_int32]
        L.comp_ams_set_rand.argtypes = [vp, C.c_uint64, C.c_uint32]
        L.comp_ams_set_streaming.argtypes = [vp, C.c_int32, C.c_int32]
        L.comp_ams_set_tile_order.argtypes = [vp, C.c_int32]
        L.comp_ams_set_pass_lds.argtypes = [vp, C.c_int32]
        L.comp_ams_message_bytes.argtypes = [vp, C.POINTER(C.c_uint64)]
        L.comp_ams_pack_message.argtypes = [vp, C.c_int32, vp, C.c_uint64, C.POINTER(C.c_uint64)]
        L.comp_ams_pack_message_noalloc.argtypes = [vp, C.c_int32, vp, C.c_uint64, C.POINTER(C.c_uint64)]
        L.comp_ams_step.argtypes = [vp, fp, vp]
        L.comp_ams_step_bf16.argtypes = [vp, fp, vp]
        L.comp_ams_step_f16.argtypes = [vp, vp, vp]
        for name in ("theta", "m", "v", "vhat"):
            getattr(L, "comp_ams_get_" + name).argtypes = [vp, fp, C.c_int]
        L.comp_ams_get_error.argtypes = [vp, C.c_int32, fp, C.c_int]
        L.comp_ams_get_selected.argtypes = [vp, C.c_int32, u32p, fp]
        L.comp_ams_get_scales.argtypes = [vp, fp]
        L.comp_ams_n_blocks.argtypes = [vp]
        L.comp_ams_n_blocks.restype = C.c_int32
        L.comp_ams_set_state.argtypes = [vp, fp, fp, fp, fp, C.c_int]
        L.comp_ams_sync.argtypes = [vp]
        L.comp_ams_profile.argtypes = [vp, C.c_int]
        L.comp_ams_profile_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                            C.POINTER(C.c_int64)]
        L.comp_ams_probe_copy.argtypes = [fp, fp, C.c_int64, vp]
        L.comp_ams_probe_update.argtypes = [fp, fp, C.c_int64, C.c_int64, vp]
        L.comp_ams_get_selection_info.argtypes = [vp, C.c_int32, u32p]
        L.comp_ams_set_method.argtypes = [vp, C.c_int32]
        L.comp_ams_get_ghat_worker.argtypes = [vp, C.c_int32, fp, C.c_int]
        L.comp_ams_get_ghat_server.argtypes = [vp, fp, C.c_int]
        L.comp_ams_get_gtilde.argtypes = [vp, fp, C.c_int]
        L.comp_ams_get_server_scales.argtypes = [vp, fp]
        L.comp_ams_set_markov_state.argtypes = [vp, fp, fp, fp, C.c_int]
        L.comp_ams_get_server_selected.argtypes = [vp, u32p, fp]
        L.comp_ams_get_signs.argtypes = [vp, C.c_int32, C.c_void_p]
        L.comp_ams_message_bits.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.comp_ams_last_error.argtypes = [vp]
        L.comp_ams_last_error.restype = C.c_char_p
        _lib = L
    return _lib


def _ptr(a):
    """(pointer, on_device) of a torch tensor or a numpy float32 array."""
    if a is None:
        return None, 0
    if isinstance(a, np.ndarray):
        assert a.dtype == np.float32 and a.flags.c_contiguous
        return a.ctypes.data, 0
    assert a.dtype.is_floating_point and a.element_size() == 4 and a.is_contiguous()
    return a.data_ptr(), 1 if a.is_cuda else 0


def probe_update(x, g, stream=None):
    """x += g in place (torch float32 CUDA tensors [rows, d], d a multiple of 4): the passes' access pattern alone."""
    import torch
    assert x.is_cuda and g.is_cuda and x.shape == g.shape and x.dim() == 2 and x.is_contiguous() and g.is_contiguous()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    rc = lib().comp_ams_probe_update(x.data_ptr(), g.data_ptr(), x.shape[0], x.shape[1], stream)
    if rc != OK:
        raise CompAmsError(rc, lib().comp_ams_last_error(None).decode())


def probe_copy(dst, src, stream=None):
    """Plain device copy dst <- src (torch float32 CUDA tensors of equal size, multiple of 4)."""
    import torch
    assert dst.is_cuda and src.is_cuda and dst.numel() == src.numel()
    if stream is None:
        stream = torch.cuda.current_stream(dst.device).cuda_stream
    rc = lib().comp_ams_probe_copy(dst.data_ptr(), src.data_ptr(), dst.numel(), stream)
    if rc != OK:
        raise CompAmsError(rc, lib().comp_ams_last_error(None).decode())


class CompAms:
    """comp_ams_create / comp_ams_step / getters, same names as the C ABI."""

    def __init__(self, d, n, compressor, k_or_block, beta1=0.9, beta2=0.999, eps=1e-8, lr=1e-3):
        self._h = C.c_void_p()
        self.d, self.n, self.compressor = int(d), int(n), int(compressor)
        self.k = int(k_or_block) if compressor != BLOCKSIGN else 0
        rc = lib().comp_ams_create(C.byref(self._h), d, n, compressor, k_or_block, beta1, beta2, eps, lr)
        if rc != OK:
            self._h = C.c_void_p()
            raise CompAmsError(rc, lib().comp_ams_last_error(None).decode())

    def _check(self, rc):
        if rc != OK:
            raise CompAmsError(rc, lib().comp_ams_last_error(self._h).decode())

    def destroy(self):
        if self._h:
            lib().comp_ams_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def set_blocks(self, offsets):
        off = np.ascontiguousarray(offsets, dtype=np.int64)
        self._check(lib().comp_ams_set_blocks(self._h, off.ctypes.data_as(C.POINTER(C.c_int64)), off.size - 1))

    def set_theta(self, theta):
        p, dev = _ptr(theta)
        self._check(lib().comp_ams_set_theta(self._h, p, dev))

    def set_lr(self, lr):
        self._check(lib().comp_ams_set_lr(self._h, lr))

    def message_bytes(self):
        out = C.c_uint64(0)
        self._check(lib().comp_ams_message_bytes(self._h, C.byref(out)))
        return out.value

    def pack_message(self, who, buf):
        """Writes the wire form of vector `who`'s last message into buf (torch uint8 CUDA tensor); returns its size."""
        assert buf.is_cuda and buf.is_contiguous()
        out = C.c_uint64(0)
        self._check(lib().comp_ams_pack_message(self._h, who, buf.data_ptr(), buf.numel() * buf.element_size(),
                                                C.byref(out)))
        return out.value

    def pack_message_noalloc(self, who, buf):
        """pack_message through the library's fixed scratch array: allocates nothing and does not wait
        (call sync() before reading buf)."""
        assert buf.is_cuda and buf.is_contiguous()
        out = C.c_uint64(0)
        self._check(lib().comp_ams_pack_message_noalloc(self._h, who, buf.data_ptr(),
                                                        buf.numel() * buf.element_size(), C.byref(out)))
        return out.value

    def set_streaming(self, rows=-1, state=-1):
        """Cache policy of the stored rows and of theta, m, v, vhat: 1 streamed, 0 cached, -1 automatic."""
        self._check(lib().comp_ams_set_streaming(self._h, rows, state))

    def set_tile_order(self, chunk=-1):
        """Tiles per XCD and group in the streaming pass: 0 plain order, -1 automatic."""
        self._check(lib().comp_ams_set_tile_order(self._h, chunk))

    def set_pass_lds(self, nbytes=-1):
        """LDS bytes per workgroup of the block-sign pass (sets workgroups per compute unit): -1 automatic."""
        self._check(lib().comp_ams_set_pass_lds(self._h, nbytes))

    def set_rand(self, seed, draw=0):
        """Rand-k: seed of the draws and number of the next draw (before the first step)."""
        self._check(lib().comp_ams_set_rand(self._h, seed, draw))

    def set_eps_mode(self, mode):
        self._check(lib().comp_ams_set_eps_mode(self._h, mode))

    def set_method(self, method):
        self._check(lib().comp_ams_set_method(self._h, method))

    def get_ghat_worker(self, worker, out=None):
        if out is None:
            out = np.empty(self.d, dtype=np.float32)
        p, dev = _ptr(out)
        self._check(lib().comp_ams_get_ghat_worker(self._h, worker, p, dev))
        return out

    def get_ghat_server(self, out=None):
        return self._get_vec(lib().comp_ams_get_ghat_server, out)

    def get_gtilde(self, out=None):
        return self._get_vec(lib().comp_ams_get_gtilde, out)

    def get_server_selected(self):
        idx = np.empty(self.k, dtype=np.uint32)
        val = np.empty(self.k, dtype=np.float32)
        self._check(lib().comp_ams_get_server_selected(self._h, idx.ctypes.data_as(C.POINTER(C.c_uint32)),
                                                       val.ctypes.data))
        return idx, val

    def get_signs(self, worker):
        """Packed sign bits (numpy uint8, (d + 7) // 8 bytes, coordinate order) of a worker's last message;
        worker = n on a CD handle: the server's."""
        out = np.zeros((self.d + 7) // 8, dtype=np.uint8)
        self._check(lib().comp_ams_get_signs(self._h, worker, out.ctypes.data))
        return out

    def message_bits(self):
        """(bits one worker sends, bits the server sends back to each worker) per step."""
        up, down = C.c_uint64(), C.c_uint64()
        self._check(lib().comp_ams_message_bits(self._h, C.byref(up), C.byref(down)))
        return up.value, down.value

    def get_server_scales(self):
        out = np.empty(self.n_blocks(), dtype=np.float32)
        self._check(lib().comp_ams_get_server_scales(self._h, out.ctypes.data))
        return out

    def set_markov_state(self, ghat_workers=None, ghat_server=None, gtilde=None):
        ptrs, devs = [], set()
        for a in (ghat_workers, ghat_server, gtilde):
            p, dev = _ptr(a)
            ptrs.append(p)
            if a is not None:
                devs.add(dev)
        assert len(devs) <= 1, "all arrays must live on the same side (host or device)"
        self._check(lib().comp_ams_set_markov_state(self._h, *ptrs, devs.pop() if devs else 0))

    def step(self, grads, stream=None):
        """grads: torch float32 tensor [n, d] on the GPU.  stream: raw hipStream_t value
        (int) or None for torch's current stream."""
        import torch
        assert grads.is_cuda and grads.dtype == torch.float32 and grads.is_contiguous()
        assert grads.numel() == self.n * self.d
        if stream is None:
            stream = torch.cuda.current_stream(grads.device).cuda_stream
        self._check(lib().comp_ams_step(self._h, grads.data_ptr(), stream))

    def step_ptr(self, grads_ptr, stream=0):
        self._check(lib().comp_ams_step(self._h, grads_ptr, stream))

    def step_bf16(self, grads, stream=None):
        """grads: torch bfloat16 tensor [n, d] on the GPU."""
        import torch
        assert grads.is_cuda and grads.dtype == torch.bfloat16 and grads.is_contiguous()
        assert grads.numel() == self.n * self.d
        if stream is None:
            stream = torch.cuda.current_stream(grads.device).cuda_stream
        self._check(lib().comp_ams_step_bf16(self._h, grads.data_ptr(), stream))

    def step_bf16_ptr(self, grads_ptr, stream=0):
        self._check(lib().comp_ams_step_bf16(self._h, grads_ptr, stream))

    def step_f16(self, grads, stream=None):
        """grads: torch float16 tensor [n, d] on the GPU."""
        import torch
        assert grads.is_cuda and grads.dtype == torch.float16 and grads.is_contiguous()
        assert grads.numel() == self.n * self.d
        if stream is None:
            stream = torch.cuda.current_stream(grads.device).cuda_stream
        self._check(lib().comp_ams_step_f16(self._h, grads.data_ptr(), stream))

    def step_f16_ptr(self, grads_ptr, stream=0):
        self._check(lib().comp_ams_step_f16(self._h, grads_ptr, stream))

    def _get_vec(self, fn, out):
        if out is None:
            out = np.empty(self.d, dtype=np.float32)
        p, dev = _ptr(out)
        self._check(fn(self._h, p, dev))
        return out

    def get_theta(self, out=None):
        return self._get_vec(lib().comp_ams_get_theta, out)

    def get_m(self, out=None):
        return self._get_vec(lib().comp_ams_get_m, out)

    def get_v(self, out=None):
        return self._get_vec(lib().comp_ams_get_v, out)

    def get_vhat(self, out=None):
        return self._get_vec(lib().comp_ams_get_vhat, out)

    def get_error(self, worker, out=None):
        if out is None:
            out = np.empty(self.d, dtype=np.float32)
        p, dev = _ptr(out)
        self._check(lib().comp_ams_get_error(self._h, worker, p, dev))
        return out

    def get_selected(self, worker):
        idx = np.empty(self.k, dtype=np.uint32)
        val = np.empty(self.k, dtype=np.float32)
        self._check(lib().comp_ams_get_selected(self._h, worker, idx.ctypes.data_as(C.POINTER(C.c_uint32)),
                                                val.ctypes.data))
        return idx, val

    def get_selection_info(self, worker):
        out = np.zeros(8, dtype=np.uint32)
        self._check(lib().comp_ams_get_selection_info(self._h, worker, out.ctypes.data_as(C.POINTER(C.c_uint32))))
        keys = ("next_guess", "slack", "relisted", "open_bits", "prefix", "rank", "whole_bin", "threshold_fine_bin")
        return dict(zip(keys, (int(v) for v in out)))

    def n_blocks(self):
        return lib().comp_ams_n_blocks(self._h)

    def get_scales(self):
        out = np.empty((self.n, self.n_blocks()), dtype=np.float32)
        self._check(lib().comp_ams_get_scales(self._h, out.ctypes.data))
        return out

    def set_state(self, m=None, v=None, vhat=None, e=None):
        ptrs = [_ptr(a) for a in (m, v, vhat, e)]
        devs = {dev for p, dev in ptrs if p is not None}
        assert len(devs) <= 1, "all arrays must live on the same side"
        self._check(lib().comp_ams_set_state(self._h, *[p for p, _ in ptrs], devs.pop() if devs else 0))

    def profile(self, enable):
        self._check(lib().comp_ams_profile(self._h, 1 if enable else 0))

    def profile_read(self):
        """{kernel name: (total_ms, launches)} of the launches recorded since profile(True)."""
        out = {}
        slot = 0
        while True:
            name, ms, cnt = C.c_char_p(), C.c_double(), C.c_int64()
            rc = lib().comp_ams_profile_read(self._h, slot, C.byref(name), C.byref(ms), C.byref(cnt))
            if rc == 1:
                return out
            self._check(rc)
            if cnt.value:
                out[name.value.decode()] = (ms.value, cnt.value)
            slot += 1

    def sync(self):
        self._check(lib().comp_ams_sync(self._h))
