"""Python binding of the spdnn C-ABI library (include/spdnn.h).

Argument marshalling only: every step of the inference runs in the HIP kernels
of csrc/.  torch is used to allocate device memory and to provide the stream.
There is no CPU fallback: if csrc/libspdnn.so is missing or cannot be loaded the
import of the library raises.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

_lib = None

SPDNN_OK = 0
SPDNN_EINVAL = -1
SPDNN_EBIAS = -2
SPDNN_EHIP = -3
SPDNN_ESIZE = -4
SPDNN_HOST = 0
SPDNN_DEVICE = 1
SPDNN_KERNEL_SINGLE = 0
SPDNN_KERNEL_STAGED = 1
SPDNN_KERNEL_WIDE = 2
SPDNN_KERNEL_PAIR = 3
SPDNN_KERNEL_WIDE_PAIR = 4
SPDNN_KERNEL_WIDE_PAIR4 = 5
SPDNN_KERNEL_ROW2 = 6

EXPORTS = ("spdnn_weights_bytes", "spdnn_work_bytes", "spdnn_create", "spdnn_infer", "spdnn_destroy",
           "spdnn_last_error", "spdnn_set_profiling", "spdnn_get_profile", "spdnn_infer_static",
           "spdnn_host_work_bytes", "spdnn_infer_host",
           "spdnn_weights_bytes_for_window", "spdnn_scan_windows", "spdnn_layer_kernel",
           "spdnn_csr_passes", "spdnn_create_csr", "spdnn_layer_passes", "spdnn_ooc_bytes", "spdnn_create_ooc",
           "spdnn_one_launch")
KERNEL_NAMES = {0: "fused_layer_kernel<false>", 1: "fused_layer_kernel<true>", 2: "fused_wide_kernel",
                3: "fused_pair_kernel", 4: "fused_wide_pair_kernel", 5: "fused_wide_pair4_kernel", 6: "fused_row2_kernel"}


class SpdnnError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("spdnn error %d: %s" % (code, msg))
        self.code = code


def lib():
    """Load csrc/libspdnn.so (build it first with build.build() or __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            raise RuntimeError("%s is missing: build the HIP library first (python -m "
                               "paper_2007_14152_amd.build); there is no fallback path" % _build.LIB)
        L = ctypes.CDLL(_build.LIB)
        vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
        L.spdnn_weights_bytes.argtypes = [i32, i32, ctypes.POINTER(sz)]
        L.spdnn_work_bytes.argtypes = [i32, i32, ctypes.POINTER(sz)]
        L.spdnn_create.argtypes = [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                   i32, vp, sz, vp]
        L.spdnn_infer.argtypes = [vp, vp, i32, vp, sz, ctypes.POINTER(i32), vp, vp]
        L.spdnn_destroy.argtypes = [vp]
        L.spdnn_last_error.argtypes = []
        L.spdnn_last_error.restype = ctypes.c_char_p
        L.spdnn_set_profiling.argtypes = [vp, i32]
        L.spdnn_get_profile.argtypes = [vp, i32, ctypes.POINTER(i32), vp, vp]
        L.spdnn_infer_static.argtypes = [vp, vp, i32, ctypes.POINTER(i32), vp, vp]
        L.spdnn_host_work_bytes.argtypes = [i32, i32, ctypes.POINTER(sz)]
        L.spdnn_infer_host.argtypes = [vp, vp, i32, i32, vp, sz, ctypes.POINTER(i32), vp, vp]
        L.spdnn_weights_bytes_for_window.argtypes = [i32, i32, i32, ctypes.POINTER(sz)]
        L.spdnn_scan_windows.argtypes = [i32, i32, ctypes.POINTER(vp), i32, vp, sz, vp, ctypes.POINTER(i32)]
        L.spdnn_layer_kernel.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.spdnn_layer_passes.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.spdnn_one_launch.argtypes = [vp, i32, ctypes.POINTER(i32)]
        L.spdnn_ooc_bytes.argtypes = [i32, i32, i32, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.spdnn_create_ooc.argtypes = [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp,
                                       i32, vp, sz, vp, sz, vp]
        L.spdnn_csr_passes.argtypes = [i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, sz, vp, vp,
                                       ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.spdnn_create_csr.argtypes = [ctypes.POINTER(vp), i32, i32, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                       ctypes.POINTER(vp), vp, vp, sz, vp]
        for n in EXPORTS:
            if n != "spdnn_last_error":
                getattr(L, n).restype = ctypes.c_int
        _lib = L
    return _lib


def spdnn_last_error() -> str:
    return lib().spdnn_last_error().decode()


def _check(rc):
    if rc != SPDNN_OK:
        raise SpdnnError(rc, spdnn_last_error())


def spdnn_weights_bytes(N: int, L: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().spdnn_weights_bytes(N, L, ctypes.byref(out)))
    return out.value


def spdnn_weights_bytes_for_window(N: int, L: int, widest_window: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().spdnn_weights_bytes_for_window(N, L, widest_window, ctypes.byref(out)))
    return out.value


def spdnn_scan_windows(N, L, idx_ptrs, where, scratch_ptr, scratch_bytes, stream=0) -> int:
    ip = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in idx_ptrs])
    w = ctypes.c_int32(0)
    _check(lib().spdnn_scan_windows(N, L, ip, where, ctypes.c_void_p(int(scratch_ptr)), scratch_bytes,
                                    ctypes.c_void_p(int(stream)), ctypes.byref(w)))
    return w.value


def spdnn_work_bytes(N: int, max_batch: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().spdnn_work_bytes(N, max_batch, ctypes.byref(out)))
    return out.value


def spdnn_create(N, L, idx_ptrs, val_ptrs, bias_ptr, where, arena_ptr, arena_bytes, stream=0):
    """idx_ptrs / val_ptrs: sequences of L raw addresses (host or device as `where`
    says); returns the opaque handle (an integer address)."""
    ip = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in idx_ptrs])
    vp = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in val_ptrs])
    h = ctypes.c_void_p(0)
    _check(lib().spdnn_create(ctypes.byref(h), N, L, ip, vp, ctypes.c_void_p(int(bias_ptr)), where,
                              ctypes.c_void_p(int(arena_ptr)), arena_bytes, ctypes.c_void_p(int(stream))))
    return h.value


def spdnn_ooc_bytes(N: int, L: int, widest_window: int):
    """Returns (device_bytes, host_bytes) of the out-of-core arenas."""
    d, h = ctypes.c_size_t(0), ctypes.c_size_t(0)
    _check(lib().spdnn_ooc_bytes(N, L, widest_window, ctypes.byref(d), ctypes.byref(h)))
    return d.value, h.value


def spdnn_create_ooc(N, L, idx_ptrs, val_ptrs, bias_ptr, where, dev_ptr, dev_bytes, host_ptr, host_bytes, stream=0):
    """Out-of-core weights: as spdnn_create, with a small device arena and a host arena."""
    ip = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in idx_ptrs])
    vp = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in val_ptrs])
    h = ctypes.c_void_p(0)
    _check(lib().spdnn_create_ooc(ctypes.byref(h), N, L, ip, vp, ctypes.c_void_p(int(bias_ptr)), where,
                                  ctypes.c_void_p(int(dev_ptr)), dev_bytes, ctypes.c_void_p(int(host_ptr)), host_bytes,
                                  ctypes.c_void_p(int(stream))))
    return h.value


def spdnn_csr_passes(N, L, ptr_ptrs, scratch_ptr, scratch_bytes, stream=0, idx_ptrs=None):
    """ptr_ptrs (idx_ptrs): L device addresses of int32[N+1] (of the column arrays).  Returns
    (passes per layer, their sum), and with idx_ptrs also the widest column window."""
    import numpy as np
    pp = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in ptr_ptrs])
    ip = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in idx_ptrs]) if idx_ptrs is not None else None
    passes = np.zeros(max(L, 1), dtype=np.int32)
    total = ctypes.c_int32(0)
    widest = ctypes.c_int32(0)
    _check(lib().spdnn_csr_passes(N, L, pp, ip, ctypes.c_void_p(int(scratch_ptr)), scratch_bytes,
                                  ctypes.c_void_p(int(stream)), passes.ctypes.data, ctypes.byref(total),
                                  ctypes.byref(widest) if idx_ptrs is not None else None))
    if idx_ptrs is not None:
        return passes[:L], total.value, widest.value
    return passes[:L], total.value


def spdnn_create_csr(N, L, ptr_ptrs, idx_ptrs, val_ptrs, bias_ptr, arena_ptr, arena_bytes, stream=0):
    """General layers; every address is device memory.  Returns the opaque handle."""
    pp = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in ptr_ptrs])
    ip = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in idx_ptrs])
    vp = (ctypes.c_void_p * max(L, 1))(*[int(p) for p in val_ptrs])
    h = ctypes.c_void_p(0)
    _check(lib().spdnn_create_csr(ctypes.byref(h), N, L, pp, ip, vp, ctypes.c_void_p(int(bias_ptr)),
                                  ctypes.c_void_p(int(arena_ptr)), arena_bytes, ctypes.c_void_p(int(stream))))
    return h.value


def spdnn_infer(h, y0_ptr, batch, work_ptr, work_bytes, active_rows_ptr, y_final_ptr) -> int:
    """Returns n_active."""
    n = ctypes.c_int32(-1)
    _check(lib().spdnn_infer(ctypes.c_void_p(h), ctypes.c_void_p(int(y0_ptr)), batch,
                             ctypes.c_void_p(int(work_ptr)), work_bytes, ctypes.byref(n),
                             ctypes.c_void_p(int(active_rows_ptr)),
                             ctypes.c_void_p(int(y_final_ptr)) if y_final_ptr else None))
    return n.value


def spdnn_destroy(h) -> None:
    _check(lib().spdnn_destroy(ctypes.c_void_p(h) if h else None))


def spdnn_set_profiling(h, on: bool) -> None:
    _check(lib().spdnn_set_profiling(ctypes.c_void_p(h), 1 if on else 0))


def spdnn_get_profile(h, cap: int):
    """Returns (layers_run, rows_in[:n], fused_ms[:n]) of the last profiled spdnn_infer."""
    import numpy as np
    rows = np.zeros(max(cap, 1), dtype=np.int32)
    ms = np.zeros(max(cap, 1), dtype=np.float32)
    run = ctypes.c_int32(0)
    _check(lib().spdnn_get_profile(ctypes.c_void_p(h), cap, ctypes.byref(run), rows.ctypes.data, ms.ctypes.data))
    n = min(cap, run.value)
    return run.value, rows[:n], ms[:n]


def spdnn_layer_kernel(h, l: int) -> int:
    """Kernel kind (SPDNN_KERNEL_*: 0 single, 1 staged, 2 wide, 3 pair, 4 wide pair, 5 wide pair of 3-4 stages) of layer l."""
    k = ctypes.c_int32(-1)
    _check(lib().spdnn_layer_kernel(ctypes.c_void_p(h), l, ctypes.byref(k)))
    return k.value


def spdnn_layer_passes(h, l: int) -> int:
    """Fused-kernel passes of layer l (1 unless some neuron has more than 32 connections)."""
    k = ctypes.c_int32(-1)
    _check(lib().spdnn_layer_passes(ctypes.c_void_p(h), l, ctypes.byref(k)))
    return k.value


def spdnn_one_launch(h, batch: int) -> bool:
    """Does spdnn_infer run all layers of the model in one launch on `batch` rows?"""
    k = ctypes.c_int32(-1)
    _check(lib().spdnn_one_launch(ctypes.c_void_p(h), batch, ctypes.byref(k)))
    return bool(k.value)


SPDNN_STATIC_SCRATCH_BYTES = 64 << 20


def spdnn_infer_static(h, y0_ptr, batch, active_rows_ptr, y_final_ptr) -> int:
    """spdnn_infer with the library's static scratch array as work memory.  Returns n_active."""
    n = ctypes.c_int32(-1)
    _check(lib().spdnn_infer_static(ctypes.c_void_p(h), ctypes.c_void_p(int(y0_ptr)), batch, ctypes.byref(n),
                                    ctypes.c_void_p(int(active_rows_ptr)),
                                    ctypes.c_void_p(int(y_final_ptr)) if y_final_ptr else None))
    return n.value


def spdnn_host_work_bytes(N: int, rows_per_batch: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().spdnn_host_work_bytes(N, rows_per_batch, ctypes.byref(out)))
    return out.value


def spdnn_infer_host(h, y0_host_ptr, batch, rows_per_batch, work_ptr, work_bytes, active_rows_ptr, y_final_ptr) -> int:
    """Inputs in host memory, inferred in serial batches of rows_per_batch rows.  Returns n_active."""
    n = ctypes.c_int32(-1)
    _check(lib().spdnn_infer_host(ctypes.c_void_p(h), ctypes.c_void_p(int(y0_host_ptr)), batch, rows_per_batch,
                                  ctypes.c_void_p(int(work_ptr)), work_bytes, ctypes.byref(n),
                                  ctypes.c_void_p(int(active_rows_ptr)),
                                  ctypes.c_void_p(int(y_final_ptr)) if y_final_ptr else None))
    return n.value


class Model:
    """Convenience owner of a handle and its arenas (torch tensors on the GPU).

    idx / val: lists of L arrays [N, 32] -- numpy arrays or CPU torch tensors
    (copied through the host path) or CUDA torch tensors (device path); bias: [N].
    """

    def __init__(self, idx, val, bias, device="cuda:0", stream=None, window_hint=None, ptr=None, out_of_core=False):
        import numpy as np
        import torch
        self.torch = torch
        self.device = torch.device(device)
        L = len(idx)
        N = int(bias.shape[0])
        self.N, self.L = N, L
        if ptr is not None:
            self._init_general(ptr, idx, val, bias, stream)
            return
        on_dev = hasattr(idx[0], "is_cuda") and idx[0].is_cuda
        keep = []
        if on_dev:
            idx = [a.to(torch.int32).contiguous() for a in idx]
            val = [a.to(torch.float32).contiguous() for a in val]
            b = bias.to(self.device, torch.float32).contiguous()
            ip = [a.data_ptr() for a in idx]
            vp = [a.data_ptr() for a in val]
            bp = b.data_ptr()
            where = SPDNN_DEVICE
        else:
            idx = [np.ascontiguousarray(np.asarray(a), dtype=np.int32) for a in idx]
            val = [np.ascontiguousarray(np.asarray(a), dtype=np.float32) for a in val]
            b = np.ascontiguousarray(np.asarray(bias), dtype=np.float32)
            ip = [a.ctypes.data for a in idx]
            vp = [a.ctypes.data for a in val]
            bp = b.ctypes.data
            where = SPDNN_HOST
        for a, v in zip(idx, val):
            assert tuple(a.shape) == (N, 32) and tuple(v.shape) == (N, 32)
        keep += [idx, val, b]
        with torch.cuda.device(self.device):
            s = stream if stream is not None else torch.cuda.current_stream(self.device)
            self.stream = s
            # size the arena for the patterns' widest column window instead of the worst case
            scratch = torch.empty(N * 32 * 4 + 2 * N // 128 + 4096, dtype=torch.uint8, device=self.device)
            self.widest_window = spdnn_scan_windows(N, L, ip, where, scratch.data_ptr(), scratch.numel(),
                                                    s.cuda_stream)
            del scratch
            if out_of_core:   # weights in pinned host memory, two layer buffers on the device
                dbytes, hbytes = spdnn_ooc_bytes(N, L, window_hint or self.widest_window)
                self.arena = torch.empty(dbytes, dtype=torch.uint8, device=self.device)
                self.host_arena = torch.empty(hbytes, dtype=torch.uint8, pin_memory=True)
                self.h = spdnn_create_ooc(N, L, ip, vp, bp, where, self.arena.data_ptr(), dbytes,
                                          self.host_arena.data_ptr(), hbytes, s.cuda_stream)
            else:
                nbytes = spdnn_weights_bytes_for_window(N, L, window_hint or self.widest_window)
                self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
                self.h = spdnn_create(N, L, ip, vp, bp, where, self.arena.data_ptr(), nbytes, s.cuda_stream)
        self.work = None
        del keep

    @classmethod
    def from_csr(cls, ptr, idx, val, bias, device="cuda:0", stream=None):
        """General layers: ptr[l] int32 [N+1], idx[l] / val[l] flat arrays of ptr[l][N] entries
        (numpy arrays or torch tensors; copied to the device with torch)."""
        return cls(idx, val, bias, device=device, stream=stream, ptr=ptr)

    def _init_general(self, ptr, idx, val, bias, stream):
        torch = self.torch
        N, L = self.N, self.L
        dev = self.device

        def to(a, dt):   # a layer without connections still needs a non-null address
            t = torch.as_tensor(a).to(dev, dt).contiguous()
            return t if t.numel() else torch.zeros(1, dtype=dt, device=dev)

        ptr = [to(a, torch.int32) for a in ptr]
        idx = [to(a, torch.int32) for a in idx]
        val = [to(a, torch.float32) for a in val]
        b = to(bias, torch.float32)
        for q, a, v in zip(ptr, idx, val):
            assert q.numel() == N + 1 and a.numel() == v.numel()
        with torch.cuda.device(dev):
            s = stream if stream is not None else torch.cuda.current_stream(dev)
            self.stream = s
            scratch = torch.empty(8 * L + 8 * ((N + 1023) // 1024) + 256, dtype=torch.uint8, device=dev)
            self.passes, total, self.widest_window = spdnn_csr_passes(
                N, L, [q.data_ptr() for q in ptr], scratch.data_ptr(), scratch.numel(), s.cuda_stream,
                idx_ptrs=[a.data_ptr() for a in idx])
            del scratch
            # size the arena for the patterns' widest column window instead of the worst case
            nbytes = spdnn_weights_bytes_for_window(N, total, self.widest_window)
            self.arena = torch.empty(nbytes, dtype=torch.uint8, device=dev)
            self.h = spdnn_create_csr(N, L, [q.data_ptr() for q in ptr], [a.data_ptr() for a in idx],
                                      [v.data_ptr() for v in val], b.data_ptr(), self.arena.data_ptr(), nbytes,
                                      s.cuda_stream)
        self.work = None

    def infer(self, Y0, want_Y=True):
        """Y0: CUDA float32 [batch, N].  Returns (n_active, active_rows[int32 n], Y[n, N] or None)."""
        torch = self.torch
        assert Y0.is_cuda and Y0.dtype == torch.float32 and Y0.is_contiguous()
        batch = int(Y0.shape[0])
        assert Y0.shape[1] == self.N
        with torch.cuda.device(self.device):
            need = spdnn_work_bytes(self.N, batch)
            if self.work is None or self.work.numel() < need:
                self.work = None
                self.work = torch.empty(need, dtype=torch.uint8, device=self.device)
            rows = torch.empty(max(batch, 1), dtype=torch.int32, device=self.device)
            Yf = torch.empty((max(batch, 1), self.N), dtype=torch.float32, device=self.device) if want_Y else None
            n = spdnn_infer(self.h, Y0.data_ptr(), batch, self.work.data_ptr(), self.work.numel(),
                            rows.data_ptr(), Yf.data_ptr() if want_Y else 0)
        return n, rows[:n], (Yf[:n] if want_Y else None)

    def infer_static(self, Y0, want_Y=True):
        """infer() through spdnn_infer_static: the library's fixed scratch array is the work memory."""
        torch = self.torch
        assert Y0.is_cuda and Y0.dtype == torch.float32 and Y0.is_contiguous() and Y0.shape[1] == self.N
        batch = int(Y0.shape[0])
        with torch.cuda.device(self.device):
            rows = torch.empty(max(batch, 1), dtype=torch.int32, device=self.device)
            Yf = torch.empty((max(batch, 1), self.N), dtype=torch.float32, device=self.device) if want_Y else None
            n = spdnn_infer_static(self.h, Y0.data_ptr(), batch, rows.data_ptr(), Yf.data_ptr() if want_Y else 0)
        return n, rows[:n], (Yf[:n] if want_Y else None)

    def infer_batched(self, Y0_host, rows_per_batch, want_Y=True):
        """Inputs that stay in host memory, processed in serial batches (Section III-B-2) by
        spdnn_infer_host: Y0_host is a CPU float32 tensor [batch, N] (pinned memory lets the copies
        overlap the kernels).  Returns what infer() returns for the whole input."""
        torch = self.torch
        assert not Y0_host.is_cuda and Y0_host.dtype == torch.float32 and Y0_host.is_contiguous()
        batch = int(Y0_host.shape[0])
        assert Y0_host.shape[1] == self.N
        step = max(1, min(int(rows_per_batch), max(batch, 1)))
        with torch.cuda.device(self.device):
            need = spdnn_host_work_bytes(self.N, step)
            work = torch.empty(need, dtype=torch.uint8, device=self.device)
            rows = torch.empty(max(batch, 1), dtype=torch.int32, device=self.device)
            Yf = torch.empty((max(batch, 1), self.N), dtype=torch.float32, device=self.device) if want_Y else None
            n = spdnn_infer_host(self.h, Y0_host.data_ptr(), batch, step, work.data_ptr(), need, rows.data_ptr(),
                                 Yf.data_ptr() if want_Y else 0)
        return n, rows[:n], (Yf[:n] if want_Y else None)

    def set_profiling(self, on=True):
        spdnn_set_profiling(self.h, on)

    def profile(self):
        return spdnn_get_profile(self.h, self.L)

    def layer_kernel(self, l):
        return spdnn_layer_kernel(self.h, l)

    def layer_passes(self, l):
        return spdnn_layer_passes(self.h, l)

    def one_launch(self, batch):
        return spdnn_one_launch(self.h, batch)

    def close(self):
        if getattr(self, "h", None):
            spdnn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
