"""ctypes binding with the same names as include/bpd.h.  Argument marshalling only.

PyTorch is used for device memory (the workspace and result tensors) and for the stream
handle; nothing here computes anything.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libbpd.so")

BPD_F32, BPD_BF16 = 0, 1
PHASE_NONE, PHASE_LAYERS, PHASE_HEAD_HIDDEN, PHASE_HEAD_OUT, PHASE_VOCAB, PHASE_ACCEPT, PHASE_STEP, PHASE_EMPTY = range(8)
ERRORS = {-1: "BPD_E_ARG", -2: "BPD_E_STATE", -3: "BPD_E_CAPACITY", -4: "BPD_E_WEIGHTS", -5: "BPD_E_HIP"}


class BpdError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{ERRORS.get(code, code)}: {msg}")
        self.code = code


class bpd_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_enc_layers", "n_dec_layers", "d_model", "n_heads", "d_ff", "vocab", "k_max",
        "max_batch", "max_src_len", "max_out_len", "dtype", "eos_id", "pad_id")] + [("ln_eps", C.c_float)]


class bpd_tensor(C.Structure):
    _fields_ = [("name", C.c_char_p), ("data", C.c_void_p), ("dtype", C.c_int32), ("ndim", C.c_int32),
                ("shape", C.c_int64 * 4), ("on_device", C.c_int32)]


class bpd_stats(C.Structure):
    _fields_ = [("steps", C.c_int64), ("invocations", C.c_int64), ("seq_steps", C.c_int64),
                ("accepted_total", C.c_int64), ("hist", C.c_int64 * 17), ("finished", C.c_int32)]


EXPORTS = ["bpd_workspace_bytes", "bpd_create", "bpd_destroy", "bpd_load_weights", "bpd_encode", "bpd_step", "bpd_step_static",
           "bpd_set_acceptance", "bpd_set_top_n", "bpd_set_two_phase", "bpd_set_local_attention", "bpd_decode", "bpd_get_state", "bpd_get_output", "bpd_get_stats",
           "bpd_set_proposals", "bpd_debug_step_logits", "bpd_profile_enable", "bpd_profile_read",
           "bpd_profile_samples", "bpd_measure_hbm_read", "bpd_measure_mfma_bf16", "bpd_last_error"]

_lib = None


def lib() -> C.CDLL:
    """Load libbpd.so.  There is no fallback: without the HIP library nothing runs."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_1811_03115_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        vp, i32p = C.c_void_p, C.c_void_p
        L.bpd_workspace_bytes.restype = C.c_size_t
        L.bpd_workspace_bytes.argtypes = [C.POINTER(bpd_config)]
        L.bpd_create.argtypes = [C.POINTER(bpd_config), vp, C.c_size_t, vp, C.POINTER(vp)]
        L.bpd_destroy.argtypes = [vp]
        L.bpd_load_weights.argtypes = [vp, C.POINTER(bpd_tensor), C.c_int]
        L.bpd_encode.argtypes = [vp, i32p, i32p, i32p, C.c_int, C.c_int]
        L.bpd_step.argtypes = [vp, C.c_int, i32p, i32p]
        L.bpd_step_static.argtypes = [vp, C.c_int, i32p, i32p]
        L.bpd_set_acceptance.argtypes = [vp, C.c_int, C.c_int]
        L.bpd_set_top_n.argtypes = [vp, C.c_int]
        L.bpd_set_two_phase.argtypes = [vp, C.c_int]
        L.bpd_set_local_attention.argtypes = [vp, C.c_int, C.c_int]
        L.bpd_decode.argtypes = [vp, C.c_int, i32p, C.c_int, i32p, i32p, C.POINTER(bpd_stats)]
        L.bpd_get_state.argtypes = [vp, i32p, i32p, i32p, i32p]
        L.bpd_get_output.argtypes = [vp, i32p, i32p]
        L.bpd_get_stats.argtypes = [vp, C.POINTER(bpd_stats)]
        L.bpd_set_proposals.argtypes = [vp, i32p]
        L.bpd_debug_step_logits.argtypes = [vp, C.c_int, vp]
        L.bpd_profile_enable.argtypes = [vp, C.c_int]
        L.bpd_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.bpd_profile_samples.argtypes = [vp, vp, C.c_int64, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.bpd_measure_hbm_read.argtypes = [vp, C.c_size_t, vp, C.c_int, C.POINTER(C.c_double)]
        L.bpd_measure_mfma_bf16.argtypes = [vp, vp, C.c_int, C.POINTER(C.c_double)]
        L.bpd_last_error.restype = C.c_char_p
        L.bpd_last_error.argtypes = [vp]
        _lib = L
    return _lib


def make_config(**kw) -> bpd_config:
    c = bpd_config()
    for k, v in kw.items():
        setattr(c, k, v)
    return c


def config_from_workload(w, max_batch: Optional[int] = None) -> bpd_config:
    """bpd_config for a workloads.Config."""
    return make_config(n_enc_layers=w.n_enc, n_dec_layers=w.n_dec, d_model=w.d_model, n_heads=w.n_heads,
                       d_ff=w.d_ff, vocab=w.vocab, k_max=w.k, max_batch=max_batch or w.batch,
                       max_src_len=w.max_src, max_out_len=w.max_out,
                       dtype=BPD_BF16 if w.dtype == "bf16" else BPD_F32, eos_id=w.eos_id, pad_id=w.pad_id,
                       ln_eps=w.ln_eps)


def _ptr(a) -> Optional[int]:
    """Raw address of a numpy array (host) or torch tensor (host or device), or None."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        assert a.flags["C_CONTIGUOUS"]
        return a.ctypes.data
    assert a.is_contiguous()
    return a.data_ptr()


def _i32(a):
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return np.ascontiguousarray(a, dtype=np.int32)
    import torch
    assert a.dtype == torch.int32
    return a.contiguous()


class Context:
    """Owns the workspace tensor and the opaque bpd_ctx*.  Methods mirror the C entry points."""

    def __init__(self, cfg: bpd_config, device: str = "cuda:0", stream=None):
        import torch
        self.torch = torch
        self.L = lib()
        self.cfg = cfg
        self.device = torch.device(device)
        nbytes = self.L.bpd_workspace_bytes(C.byref(cfg))
        if nbytes == 0:
            raise BpdError(-1, "invalid configuration")
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        aligned = (base + 255) // 256 * 256
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        handle = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = self.L.bpd_create(C.byref(cfg), aligned, nbytes, self.stream.cuda_stream, C.byref(handle))
        if rc != 0:
            raise BpdError(rc, "bpd_create failed")
        self.h = handle
        self.B = 0

    # -- helpers
    def _check(self, rc: int):
        if rc != 0:
            raise BpdError(rc, self.L.bpd_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.L.bpd_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- C ABI mirrors
    def bpd_load_weights(self, weights: Dict[str, object]):
        """weights: name -> numpy float32 array (host) or torch float32/bfloat16 tensor (host or device)."""
        torch = self.torch
        arr = (bpd_tensor * len(weights))()
        keep = []
        for i, (name, a) in enumerate(weights.items()):
            if isinstance(a, np.ndarray):
                a = np.ascontiguousarray(a, dtype=np.float32)
                dtype, on_dev, shape = BPD_F32, 0, a.shape
            else:
                a = a.contiguous()
                dtype = BPD_BF16 if a.dtype == torch.bfloat16 else BPD_F32
                assert a.dtype in (torch.bfloat16, torch.float32)
                on_dev, shape = int(a.is_cuda), tuple(a.shape)
            keep.append(a)
            t = arr[i]
            t.name = name.encode()
            t.data = _ptr(a)
            t.dtype = dtype
            t.ndim = len(shape)
            for d_, s in enumerate(shape):
                t.shape[d_] = s
            t.on_device = on_dev
        self._check(self.L.bpd_load_weights(self.h, arr, len(weights)))

    def bpd_encode(self, src_ids, src_len, max_len=None):
        src_ids, src_len, max_len = _i32(src_ids), _i32(src_len), _i32(max_len)
        B, S = src_ids.shape
        self._check(self.L.bpd_encode(self.h, _ptr(src_ids), _ptr(src_len), _ptr(max_len), B, S))
        self.B = B

    def bpd_step(self, k: int, imposed_accept=None, accepted_len=None):
        imposed_accept = _i32(imposed_accept)
        self._check(self.L.bpd_step(self.h, k, _ptr(imposed_accept), _ptr(accepted_len)))

    def bpd_step_static(self, k: int, imposed_accept=None, accepted_len=None):
        imposed_accept = _i32(imposed_accept)
        self._check(self.L.bpd_step_static(self.h, k, _ptr(imposed_accept), _ptr(accepted_len)))

    def bpd_set_acceptance(self, distance_eps: int = 0, min_block: int = 1):
        self._check(self.L.bpd_set_acceptance(self.h, distance_eps, min_block))

    def bpd_set_top_n(self, n: int = 1):
        self._check(self.L.bpd_set_top_n(self.h, n))

    def bpd_set_two_phase(self, on: bool = True):
        self._check(self.L.bpd_set_two_phase(self.h, int(on)))

    def bpd_set_local_attention(self, query_block: int, memory_len: int):
        self._check(self.L.bpd_set_local_attention(self.h, int(query_block), int(memory_len)))

    def bpd_decode(self, k: int, schedule=None, max_steps: Optional[int] = None):
        """Returns (out_ids [B,max_out] int32 numpy, out_len [B], stats)."""
        schedule = _i32(schedule)
        if max_steps is None:
            max_steps = self.cfg.max_out_len if schedule is None else schedule.shape[0]
        out_ids = np.empty((self.B, self.cfg.max_out_len), dtype=np.int32)
        out_len = np.empty(self.B, dtype=np.int32)
        st = bpd_stats()
        self._check(self.L.bpd_decode(self.h, k, _ptr(schedule), max_steps, _ptr(out_ids), _ptr(out_len), C.byref(st)))
        return out_ids, out_len, st

    def bpd_get_state(self):
        k = self.cfg.k_max
        P = np.empty((self.B, k), dtype=np.int32)
        A = np.empty((self.B, k, k), dtype=np.int32)
        j = np.empty(self.B, dtype=np.int32)
        fin = np.empty(self.B, dtype=np.int32)
        self._check(self.L.bpd_get_state(self.h, _ptr(P), _ptr(A), _ptr(j), _ptr(fin)))
        return P, A, j, fin

    def bpd_get_output(self):
        out_ids = np.empty((self.B, self.cfg.max_out_len), dtype=np.int32)
        out_len = np.empty(self.B, dtype=np.int32)
        self._check(self.L.bpd_get_output(self.h, _ptr(out_ids), _ptr(out_len)))
        return out_ids, out_len

    def bpd_get_stats(self) -> bpd_stats:
        st = bpd_stats()
        self._check(self.L.bpd_get_stats(self.h, C.byref(st)))
        return st

    def bpd_set_proposals(self, P):
        P = _i32(P)
        assert tuple(P.shape) == (self.B, self.cfg.k_max)
        self._check(self.L.bpd_set_proposals(self.h, _ptr(P)))

    def bpd_debug_step_logits(self, k: int):
        """Returns a device float32 tensor [B, k, k, vocab]."""
        torch = self.torch
        out = torch.empty((self.B, k, k, self.cfg.vocab), dtype=torch.float32, device=self.device)
        self._check(self.L.bpd_debug_step_logits(self.h, k, out.data_ptr()))
        return out

    def bpd_profile_enable(self, phase: int):
        self._check(self.L.bpd_profile_enable(self.h, phase))

    def bpd_profile_read(self):
        ms, n = C.c_double(), C.c_int64()
        self._check(self.L.bpd_profile_read(self.h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def bpd_profile_samples(self, capacity: int):
        """Returns (per-launch milliseconds [<= capacity] float32 numpy, total ms, launches)."""
        out = np.zeros(capacity, dtype=np.float32)
        ms, n = C.c_double(), C.c_int64()
        self._check(self.L.bpd_profile_samples(self.h, _ptr(out), capacity, C.byref(ms), C.byref(n)))
        return out[:min(capacity, n.value)], ms.value, n.value

    @staticmethod
    def bpd_measure_hbm_read(nbytes: int = 1 << 30, iters: int = 4) -> float:
        """GB/s of a streaming read over a fresh `nbytes` device buffer on torch's current stream."""
        import torch
        buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        gbps = C.c_double()
        rc = lib().bpd_measure_hbm_read(buf.data_ptr(), nbytes, torch.cuda.current_stream().cuda_stream, iters, C.byref(gbps))
        if rc:
            raise BpdError(rc, "bpd_measure_hbm_read")
        return gbps.value

    @staticmethod
    def bpd_measure_mfma_bf16(iters: int = 20000) -> float:
        """TFLOP/s of back-to-back bf16 MFMAs on torch's current stream."""
        import torch
        buf = torch.zeros(64, dtype=torch.float32, device="cuda")
        tf = C.c_double()
        rc = lib().bpd_measure_mfma_bf16(buf.data_ptr(), torch.cuda.current_stream().cuda_stream, iters, C.byref(tf))
        if rc:
            raise BpdError(rc, "bpd_measure_mfma_bf16")
        return tf.value
