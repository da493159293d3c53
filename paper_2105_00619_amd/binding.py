"""ctypes binding of liboptorch_seq.so -- argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used here
to allocate the two device arenas and to supply the HIP stream.  There is no CPU
fallback: if the shared library is missing the import of the library fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboptorch_seq.so")

OK, E_INVALID, E_BUDGET, E_HIP, E_ORDER = 0, -1, -2, -3, -4

SYMBOLS = (
    "optorch_seq_create", "optorch_seq_query", "optorch_seq_bind", "optorch_seq_set_params",
    "optorch_seq_get_params", "optorch_seq_step", "optorch_seq_schedule_info", "optorch_seq_last_error",
    "optorch_seq_destroy", "optorch_seq_predict", "optorch_seq_running_stats", "optorch_seq_profile_enable", "optorch_seq_profile_select", "optorch_seq_profile_read", "optorch_seq_profile_read_entries",
    "optorch_seq_step_encoded", "optorch_seq_predict_encoded", "optorch_seq_plan_info", "optorch_seq_step_static", "optorch_seq_debug_unit_output",
    "optorch_encoded_words", "optorch_encode", "optorch_decode", "optorch_decode_normalized", "optorch_encode_lossless",
    "optorch_decode_lossless", "optorch_dataflow_last_error",
)

KERNEL_CLASSES = ("cast_in", "conv_fwd", "conv_dgrad", "conv_wgrad", "bn_stats", "bn_apply", "bn_bwd", "pool", "head",
                  "relu_bias_bwd", "optimizer", "conv1x1_fwd", "conv1x1_dgrad", "conv1x1_wgrad")


class optorch_unit_t(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("kind", "cin", "cout", "ksize", "stride", "pad", "has_bn", "has_relu", "has_bias", "reserved")]


class optorch_seq_config_t(C.Structure):
    _fields_ = [
        ("k_segments", C.c_int32), ("boundaries", C.POINTER(C.c_int32)), ("plan_mode", C.c_int32),
        ("precision", C.c_int32), ("batch", C.c_int32), ("height", C.c_int32), ("width", C.c_int32),
        ("channels", C.c_int32), ("num_classes", C.c_int32), ("activation_budget_bytes", C.c_uint64),
        ("momentum", C.c_float), ("bn_eps", C.c_float), ("bn_momentum", C.c_float),
        ("loss_scale_init", C.c_float), ("scale_growth", C.c_float), ("scale_backoff", C.c_float),
        ("growth_interval", C.c_int32), ("storage_mode", C.c_int32),
    ]


_lib = None


def load_library() -> C.CDLL:
    """Loads the HIP library built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s not found: build it with `python -m paper_2105_00619_amd.build` "
                          "(there is no CPU fallback)" % LIB_PATH)
    lib = C.CDLL(LIB_PATH)
    H = C.c_void_p
    lib.optorch_seq_create.argtypes = [C.POINTER(optorch_unit_t), C.c_int32, C.POINTER(optorch_seq_config_t), C.POINTER(H)]
    lib.optorch_seq_create.restype = C.c_int
    lib.optorch_seq_query.argtypes = [H, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                      C.POINTER(C.c_uint64), C.POINTER(C.c_int32)]
    lib.optorch_seq_query.restype = C.c_int
    lib.optorch_seq_bind.argtypes = [H, C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p]
    lib.optorch_seq_bind.restype = C.c_int
    lib.optorch_seq_set_params.argtypes = [H, C.c_void_p, C.c_uint64, C.c_int32]
    lib.optorch_seq_set_params.restype = C.c_int
    lib.optorch_seq_get_params.argtypes = [H, C.c_void_p, C.c_uint64, C.c_int32]
    lib.optorch_seq_get_params.restype = C.c_int
    lib.optorch_seq_step.argtypes = [H, C.c_void_p, C.c_void_p, C.c_float, C.POINTER(C.c_float), C.c_void_p,
                                     C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_float),
                                     C.POINTER(C.c_int32)]
    lib.optorch_seq_step.restype = C.c_int
    lib.optorch_seq_step_static.argtypes = lib.optorch_seq_step.argtypes
    lib.optorch_seq_step_static.restype = C.c_int
    lib.optorch_seq_debug_unit_output.argtypes = [H, C.c_void_p, C.c_int32, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64),
                                                  C.POINTER(C.c_int32)]
    lib.optorch_seq_debug_unit_output.restype = C.c_int
    lib.optorch_seq_step_encoded.argtypes = [H, C.c_void_p, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p,
                                             C.c_float, C.POINTER(C.c_float), C.c_void_p, C.POINTER(C.c_uint64),
                                             C.POINTER(C.c_uint64), C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.optorch_seq_step_encoded.restype = C.c_int
    lib.optorch_seq_predict_encoded.argtypes = [H, C.c_void_p, C.c_int32, C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_void_p]
    lib.optorch_seq_predict_encoded.restype = C.c_int
    lib.optorch_encoded_words.argtypes = [C.c_int32, C.c_int32]
    lib.optorch_encoded_words.restype = C.c_int32
    lib.optorch_encode.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.optorch_encode.restype = C.c_int
    lib.optorch_decode.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.optorch_decode.restype = C.c_int
    lib.optorch_decode_normalized.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.POINTER(C.c_float),
                                              C.POINTER(C.c_float), C.c_int32, C.c_void_p, C.c_void_p]
    lib.optorch_decode_normalized.restype = C.c_int
    lib.optorch_encode_lossless.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.optorch_encode_lossless.restype = C.c_int
    lib.optorch_decode_lossless.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
    lib.optorch_decode_lossless.restype = C.c_int
    lib.optorch_dataflow_last_error.argtypes = []
    lib.optorch_dataflow_last_error.restype = C.c_char_p
    lib.optorch_seq_predict.argtypes = [H, C.c_void_p, C.c_void_p]
    lib.optorch_seq_predict.restype = C.c_int
    lib.optorch_seq_running_stats.argtypes = [H, C.c_void_p, C.c_uint64, C.POINTER(C.c_uint64), C.c_int32]
    lib.optorch_seq_running_stats.restype = C.c_int
    lib.optorch_seq_plan_info.argtypes = [H, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.optorch_seq_plan_info.restype = C.c_int
    lib.optorch_seq_schedule_info.argtypes = [H, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    lib.optorch_seq_schedule_info.restype = C.c_int
    lib.optorch_seq_profile_enable.argtypes = [H, C.c_int32]
    lib.optorch_seq_profile_enable.restype = C.c_int
    lib.optorch_seq_profile_select.argtypes = [H, C.c_uint32]
    lib.optorch_seq_profile_select.restype = C.c_int
    lib.optorch_seq_profile_read.argtypes = [H, C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                                             C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.optorch_seq_profile_read.restype = C.c_int
    lib.optorch_seq_profile_read_entries.argtypes = [H, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                                     C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_double),
                                                     C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.optorch_seq_profile_read_entries.restype = C.c_int
    lib.optorch_seq_last_error.argtypes = [H]
    lib.optorch_seq_last_error.restype = C.c_char_p
    lib.optorch_seq_destroy.argtypes = [H]
    lib.optorch_seq_destroy.restype = None
    _lib = lib
    return lib


class OptorchError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("optorch_seq error %d: %s" % (code, message))
        self.code = code


class SeqPlan:
    """optorch_seq_create + optorch_seq_query: host-side plan, no device needed."""

    def __init__(self, units: Sequence, *, k_segments: int, precision: int, batch: int, height: int, width: int,
                 channels: int, num_classes: int, boundaries: Optional[Sequence[int]] = None, plan_mode: int = 0,
                 activation_budget_bytes: int = 0, momentum: float = 0.0, bn_eps: float = 0.0, bn_momentum: float = 0.0,
                 loss_scale_init: float = 0.0, scale_growth: float = 0.0, scale_backoff: float = 0.0,
                 growth_interval: int = 0, storage_mode: int = 0):
        self.lib = load_library()
        self.handle = C.c_void_p()
        arr = (optorch_unit_t * len(units))()
        for i, u in enumerate(units):
            arr[i] = optorch_unit_t(u.kind, u.cin, u.cout, u.ksize, u.stride, u.pad, u.has_bn, u.has_relu, u.has_bias, 0)
        cfg = optorch_seq_config_t()
        cfg.k_segments = k_segments
        barr = None
        if boundaries is not None:
            barr = (C.c_int32 * max(1, len(boundaries)))(*boundaries)
            cfg.boundaries = C.cast(barr, C.POINTER(C.c_int32))
        cfg.plan_mode, cfg.precision = plan_mode, precision
        cfg.batch, cfg.height, cfg.width, cfg.channels, cfg.num_classes = batch, height, width, channels, num_classes
        cfg.activation_budget_bytes = activation_budget_bytes
        cfg.momentum, cfg.bn_eps, cfg.bn_momentum = momentum, bn_eps, bn_momentum
        cfg.loss_scale_init, cfg.scale_growth, cfg.scale_backoff = loss_scale_init, scale_growth, scale_backoff
        cfg.growth_interval = growth_interval
        cfg.storage_mode = storage_mode
        rc = self.lib.optorch_seq_create(arr, len(units), C.byref(cfg), C.byref(self.handle))
        if rc != OK:
            msg = self.lib.optorch_seq_last_error(None).decode()
            self.handle = C.c_void_p()
            raise OptorchError(rc, msg)
        kk, sm = C.c_int32(), C.c_int32()
        self._check(self.lib.optorch_seq_plan_info(self.handle, C.byref(kk), C.byref(sm)))
        k_segments = kk.value  # the plan's choice when 0 was asked for
        self.k_segments, self.storage_mode = k_segments, sm.value
        self.batch, self.height, self.width, self.channels = batch, height, width, channels
        self.num_classes = num_classes
        pc, pb, ab, ps = C.c_uint64(), C.c_uint64(), C.c_uint64(), C.c_uint64()
        bo = (C.c_int32 * max(1, k_segments - 1))()
        self._check(self.lib.optorch_seq_query(self.handle, C.byref(pc), C.byref(pb), C.byref(ab), C.byref(ps), bo))
        self.param_count, self.param_arena_bytes = pc.value, pb.value
        self.act_arena_bytes, self.planned_peak_saved_bytes = ab.value, ps.value
        self.boundaries = [bo[i] for i in range(k_segments - 1)]
        nl, nr = C.c_int32(), C.c_int32()
        self._check(self.lib.optorch_seq_schedule_info(self.handle, C.byref(nl), C.byref(nr)))
        self.n_launches, self.n_replay_launches = nl.value, nr.value

    @classmethod
    def from_workload(cls, w, **override):
        kw = dict(k_segments=w.k_segments, precision=w.precision, batch=w.batch, height=w.height, width=w.width,
                  channels=w.channels, num_classes=w.classes, plan_mode=w.plan_mode,
                  activation_budget_bytes=w.budget_bytes, momentum=w.momentum, loss_scale_init=w.loss_scale_init)
        kw.update(override)
        return cls(w.units, **kw)

    def _check(self, rc: int):
        if rc != OK:
            raise OptorchError(rc, self.lib.optorch_seq_last_error(self.handle).decode())

    def close(self):
        if getattr(self, "handle", None) and self.handle.value:
            self.lib.optorch_seq_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class SeqTrainer(SeqPlan):
    """A bound plan: device arenas allocated through torch, steps run on torch's current stream."""

    GUARD_BYTE = 0xA5

    def __init__(self, units, *, device="cuda:0", guard_bytes: int = 0, **kw):
        """guard_bytes > 0: each arena is allocated with that many bytes of a fixed pattern in front of and behind the
        bytes lent to the library, and `guards_intact()` checks that no kernel wrote outside them."""
        import torch
        super().__init__(units, **kw)
        self.torch = torch
        self.device = torch.device(device)
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the training step only runs on the HIP path")
        self.guard_bytes = g = (int(guard_bytes) + 255) // 256 * 256
        self._arenas = []
        ptrs = []
        for nbytes in (self.param_arena_bytes, self.act_arena_bytes):
            buf = torch.empty(nbytes + 2 * g + 256, dtype=torch.uint8, device=self.device)
            start = (buf.data_ptr() + 255) // 256 * 256 - buf.data_ptr() + g  # offset of the lent bytes inside buf
            if g:
                buf[:start].fill_(self.GUARD_BYTE)
                buf[start + nbytes:].fill_(self.GUARD_BYTE)
            self._arenas.append((buf, start, nbytes))
            ptrs.append(buf.data_ptr() + start)
        self.param_arena, self.act_arena = self._arenas[0][0], self._arenas[1][0]
        self.stream = torch.cuda.current_stream(self.device)
        self._check(self.lib.optorch_seq_bind(self.handle, ptrs[0], self.param_arena_bytes, ptrs[1], self.act_arena_bytes,
                                              self.stream.cuda_stream))

    def guards_intact(self) -> bool:
        """True if every guard byte around both arenas still holds the pattern (needs guard_bytes > 0)."""
        assert self.guard_bytes > 0, "the trainer was created without guard bands"
        self.torch.cuda.synchronize(self.device)
        for buf, start, nbytes in self._arenas:
            if not bool((buf[:start] == self.GUARD_BYTE).all()) or not bool((buf[start + nbytes:] == self.GUARD_BYTE).all()):
                return False
        return True

    @classmethod
    def from_workload(cls, w, device="cuda:0", **override):
        kw = dict(k_segments=w.k_segments, precision=w.precision, batch=w.batch, height=w.height, width=w.width,
                  channels=w.channels, num_classes=w.classes, plan_mode=w.plan_mode,
                  activation_budget_bytes=w.budget_bytes, momentum=w.momentum, loss_scale_init=w.loss_scale_init)
        kw.update(override)
        return cls(w.units, device=device, **kw)

    def set_params(self, params):
        torch = self.torch
        if isinstance(params, np.ndarray):
            p = np.ascontiguousarray(params, dtype=np.float32)
            self._check(self.lib.optorch_seq_set_params(self.handle, p.ctypes.data, p.size, 0))
        else:
            p = params.to(device=self.device, dtype=torch.float32).contiguous()
            self._check(self.lib.optorch_seq_set_params(self.handle, p.data_ptr(), p.numel(), 1))

    def get_params(self) -> np.ndarray:
        out = np.empty(self.param_count, dtype=np.float32)
        self._check(self.lib.optorch_seq_get_params(self.handle, out.ctypes.data, out.size, 0))
        return out

    def step(self, x, y, lr: float, grads=None, static_arena: bool = False) -> dict:
        """x: cuda float32 NHWC tensor, y: cuda int32 tensor, grads: optional cuda float32 tensor (param_count).
        static_arena: run optorch_seq_step_static (the library's static activation arena; allocates nothing)."""
        torch = self.torch
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
        assert tuple(x.shape) == (self.batch, self.height, self.width, self.channels)
        assert y.is_cuda and y.dtype == torch.int32 and y.numel() == self.batch
        if grads is not None:
            assert grads.is_cuda and grads.dtype == torch.float32 and grads.numel() == self.param_count
        loss, scale, skipped = C.c_float(), C.c_float(), C.c_int32()
        ps, pa = C.c_uint64(), C.c_uint64()
        fn = self.lib.optorch_seq_step_static if static_arena else self.lib.optorch_seq_step
        self._check(fn(self.handle, x.data_ptr(), y.data_ptr(), lr, C.byref(loss),
                                              grads.data_ptr() if grads is not None else None, C.byref(ps), C.byref(pa),
                                              C.byref(scale), C.byref(skipped)))
        return {"loss": loss.value, "peak_saved_bytes": ps.value, "peak_arena_bytes": pa.value,
                "loss_scale": scale.value, "skipped": bool(skipped.value)}

    def step_encoded(self, a, z: int, scale, shift, y, lr: float, grads=None) -> dict:
        """`step` on a batch in encoded form: a = `encode(pixels, z)` of the batch's 8-bit pixels; the decode layer maps
        every pixel to pixel * scale[c] + shift[c] (`channels` floats each)."""
        torch = self.torch
        words = encoded_words(z)
        groups = -(-self.batch // z)
        assert a.is_cuda and a.dtype == torch.int64 and a.is_contiguous()
        assert a.numel() == groups * self.height * self.width * self.channels * words
        assert y.is_cuda and y.dtype == torch.int32 and y.numel() == self.batch
        if grads is not None:
            assert grads.is_cuda and grads.dtype == torch.float32 and grads.numel() == self.param_count
        sc, sh = _float_array(scale, self.channels), _float_array(shift, self.channels)
        loss, lscale, skipped = C.c_float(), C.c_float(), C.c_int32()
        ps, pa = C.c_uint64(), C.c_uint64()
        self._check(self.lib.optorch_seq_step_encoded(self.handle, a.data_ptr(), z, sc, sh, y.data_ptr(), lr, C.byref(loss),
                                                      grads.data_ptr() if grads is not None else None, C.byref(ps),
                                                      C.byref(pa), C.byref(lscale), C.byref(skipped)))
        return {"loss": loss.value, "peak_saved_bytes": ps.value, "peak_arena_bytes": pa.value,
                "loss_scale": lscale.value, "skipped": bool(skipped.value)}

    def predict(self, x):
        """Inference-mode logits (running BatchNorm statistics): cuda float32 tensor batch x num_classes."""
        torch = self.torch
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
        assert tuple(x.shape) == (self.batch, self.height, self.width, self.channels)
        out = torch.empty((self.batch, self.num_classes), dtype=torch.float32, device=self.device)
        self._check(self.lib.optorch_seq_predict(self.handle, x.data_ptr(), out.data_ptr()))
        return out

    def predict_encoded(self, a, z: int, scale, shift):
        """`predict` on a batch in encoded form (see `step_encoded`)."""
        torch = self.torch
        groups = -(-self.batch // z)
        assert a.is_cuda and a.dtype == torch.int64 and a.is_contiguous()
        assert a.numel() == groups * self.height * self.width * self.channels * encoded_words(z)
        out = torch.empty((self.batch, self.num_classes), dtype=torch.float32, device=self.device)
        self._check(self.lib.optorch_seq_predict_encoded(self.handle, a.data_ptr(), z, _float_array(scale, self.channels),
                                                         _float_array(shift, self.channels), out.data_ptr()))
        return out

    def unit_output(self, x, unit: int):
        """The output activation of body unit `unit` in a training-mode forward pass on x: cuda float32 NHWC tensor
        (optorch_seq_debug_unit_output)."""
        torch = self.torch
        assert x.is_cuda and x.dtype == torch.float32 and x.is_contiguous()
        n, shape = C.c_uint64(), (C.c_int32 * 4)()
        self._check(self.lib.optorch_seq_debug_unit_output(self.handle, None, unit, None, 0, C.byref(n), shape))
        out = torch.empty(tuple(shape), dtype=torch.float32, device=self.device)
        self._check(self.lib.optorch_seq_debug_unit_output(self.handle, x.data_ptr(), unit, out.data_ptr(), n.value,
                                                           C.byref(n), shape))
        return out

    def running_stats(self) -> np.ndarray:
        """Per BatchNorm in parameter order: C running means, then C running variances."""
        n = C.c_uint64()
        self._check(self.lib.optorch_seq_running_stats(self.handle, None, 0, C.byref(n), 0))
        out = np.empty(n.value, dtype=np.float32)
        if n.value:
            self._check(self.lib.optorch_seq_running_stats(self.handle, out.ctypes.data, out.size, C.byref(n), 0))
        return out

    def profile_enable(self, enable: bool = True):
        self._check(self.lib.optorch_seq_profile_enable(self.handle, 1 if enable else 0))

    def profile_select(self, classes=None):
        """Restrict event timing to the named kernel classes (None: all)."""
        mask = 0xFFFFFFFF if classes is None else sum(1 << KERNEL_CLASSES.index(c) for c in classes)
        self._check(self.lib.optorch_seq_profile_select(self.handle, mask))

    def profile_read(self) -> dict:
        """Per kernel class: launches, schedule entries, GPU ms, algorithmic FLOPs and bytes, summed over the
        profiled steps; plus "steps"."""
        n = len(KERNEL_CLASSES)
        steps = C.c_int32()
        la, en = (C.c_uint64 * n)(), (C.c_uint64 * n)()
        ms, fl, by = (C.c_double * n)(), (C.c_double * n)(), (C.c_double * n)()
        self._check(self.lib.optorch_seq_profile_read(self.handle, C.byref(steps), la, en, ms, fl, by))
        out = {"steps": steps.value, "classes": {}}
        for i, name in enumerate(KERNEL_CLASSES):
            out["classes"][name] = {"launches": la[i], "entries": en[i], "gpu_ms": ms[i], "flops": fl[i], "bytes": by[i]}
        return out

    def profile_read_entries(self) -> list:
        """Per schedule entry, in launch order: kernel class, unit, phase, GPU ms, algorithmic FLOPs and bytes."""
        cap = 8192
        n = C.c_int32()
        kind, unit, phase = (C.c_int32 * cap)(), (C.c_int32 * cap)(), (C.c_int32 * cap)()
        ms, fl, by = (C.c_double * cap)(), (C.c_double * cap)(), (C.c_double * cap)()
        self._check(self.lib.optorch_seq_profile_read_entries(self.handle, cap, C.byref(n), kind, unit, phase, ms, fl, by))
        return [{"kind": KERNEL_CLASSES[kind[i]], "unit": unit[i], "phase": phase[i], "gpu_ms": ms[i], "flops": fl[i],
                 "bytes": by[i]} for i in range(min(n.value, cap))]


# ---- image data-flow (optorch_dataflow.h): tensors allocated through torch, kernels on torch's current stream ----------
# Encoded words are unsigned 64-bit; torch carries them as int64 tensors of the same bits.

def _float_array(values, n: int):
    v = [float(t) for t in values]
    if len(v) != n:
        raise ValueError("expected %d values, got %d" % (n, len(v)))
    return (C.c_float * n)(*v)


def _df_check(rc: int):
    if rc != OK:
        raise OptorchError(rc, (load_library().optorch_dataflow_last_error() or b"").decode())


def _stream(torch):
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def encoded_words(z: int, lossless: bool = False) -> int:
    """64-bit words per position for groups of z images; raises for z outside the form's range."""
    n = load_library().optorch_encoded_words(z, 1 if lossless else 0)
    if n == 0:
        raise OptorchError(E_INVALID, "images per group must be 1..%d, got %d" % (32 if lossless else 16, z))
    return n


def _batch_shape(x):
    batch = x.shape[0]
    n_pos = 1
    for d in x.shape[1:]:
        n_pos *= d
    return batch, n_pos


def encode(x, z: int, out=None):
    """Algorithm "Encode": x cuda uint8 [batch, ...] -> cuda int64 [ceil(batch / z), n_pos, words]."""
    import torch
    assert x.is_cuda and x.dtype == torch.uint8 and x.is_contiguous()
    batch, n_pos = _batch_shape(x)
    words = encoded_words(z)
    if out is None:
        out = torch.empty((-(-batch // z), n_pos, words), dtype=torch.int64, device=x.device)
    assert out.is_cuda and out.dtype == torch.int64 and out.is_contiguous() and out.numel() == -(-batch // z) * n_pos * words
    _df_check(load_library().optorch_encode(x.data_ptr(), batch, n_pos, z, out.data_ptr(), _stream(torch)))
    return out


def decode(a, batch: int, n_pos: int, z: int, out=None):
    """Algorithm "Decode": the inverse of `encode`; returns cuda uint8 [batch, n_pos]."""
    import torch
    words = encoded_words(z)
    assert a.is_cuda and a.dtype == torch.int64 and a.is_contiguous() and a.numel() == -(-batch // z) * n_pos * words
    if out is None:
        out = torch.empty((batch, n_pos), dtype=torch.uint8, device=a.device)
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous() and out.numel() == batch * n_pos
    _df_check(load_library().optorch_decode(a.data_ptr(), batch, n_pos, z, out.data_ptr(), _stream(torch)))
    return out


def decode_normalized(a, batch: int, n_pos: int, z: int, channels: int, scale, shift, precision: int, out=None):
    """Decode fused with pixel * scale[c] + shift[c] and the cast: cuda [batch, n_pos] in fp32 / bf16 / fp16."""
    import torch
    words = encoded_words(z)
    assert a.is_cuda and a.dtype == torch.int64 and a.is_contiguous() and a.numel() == -(-batch // z) * n_pos * words
    dtype = {0: torch.float32, 1: torch.bfloat16, 2: torch.float16}[precision]
    if out is None:
        out = torch.empty((batch, n_pos), dtype=dtype, device=a.device)
    assert out.is_cuda and out.dtype == dtype and out.is_contiguous() and out.numel() == batch * n_pos
    _df_check(load_library().optorch_decode_normalized(a.data_ptr(), batch, n_pos, z, channels, _float_array(scale, channels),
                                                       _float_array(shift, channels), precision, out.data_ptr(),
                                                       _stream(torch)))
    return out


def encode_lossless(x, z: int):
    """Algorithm "Loss-less Forced Encoding": x cuda uint8 [batch, ...] -> (cuda int64 [G, n_pos, words], cuda int32 [G, n_pos])."""
    import torch
    assert x.is_cuda and x.dtype == torch.uint8 and x.is_contiguous()
    batch, n_pos = _batch_shape(x)
    words = encoded_words(z, True)
    groups = -(-batch // z)
    a = torch.empty((groups, n_pos, words), dtype=torch.int64, device=x.device)
    o = torch.empty((groups, n_pos), dtype=torch.int32, device=x.device)
    _df_check(load_library().optorch_encode_lossless(x.data_ptr(), batch, n_pos, z, a.data_ptr(), o.data_ptr(), _stream(torch)))
    return a, o


def decode_lossless(a, o, batch: int, n_pos: int, z: int):
    """The inverse of `encode_lossless`; returns cuda uint8 [batch, n_pos]."""
    import torch
    words = encoded_words(z, True)
    groups = -(-batch // z)
    assert a.is_cuda and a.dtype == torch.int64 and a.is_contiguous() and a.numel() == groups * n_pos * words
    assert o.is_cuda and o.dtype == torch.int32 and o.is_contiguous() and o.numel() == groups * n_pos
    out = torch.empty((batch, n_pos), dtype=torch.uint8, device=a.device)
    _df_check(load_library().optorch_decode_lossless(a.data_ptr(), o.data_ptr(), batch, n_pos, z, out.data_ptr(), _stream(torch)))
    return out
