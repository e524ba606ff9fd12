"""Thin ctypes binding of libpt.so (see include/pt.h): argument marshalling only.

PyTorch is used for device memory (the four arenas, inputs, labels) and for the
HIP stream handle; every step of the training path runs in the library's
kernels.  There is no fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpt.so")

PT_OK, PT_EINVAL, PT_ESTATE, PT_ENOMEM, PT_EDEVICE, PT_ECACHE_MISS = range(6)
PT_VIT_PRELN, PT_BERT_POSTLN = 0, 1
PT_F32, PT_BF16 = 0, 1
PT_SGDM, PT_ADAMW = 0, 1
PT_HEAD_DEFAULT, PT_HEAD_CLS = 0, 1
KIND_PARAM, KIND_GRAD, KIND_MOMENT1, KIND_MOMENT2, KIND_SHADOW = range(5)
ACT_HK, ACT_HL, ACT_LOGITS, ACT_DHK = range(4)
PROF_CATEGORIES = ("gemm_generic", "gemm_nn", "gemm_nt", "gemm_tn", "attn_fwd", "attn_bwd", "ln_fwd", "ln_bwd",
                   "colsum", "opt", "norms", "cache", "wgrad_block", "splitk_reduce")
_STATUS = {0: "PT_OK", 1: "PT_EINVAL", 2: "PT_ESTATE", 3: "PT_ENOMEM", 4: "PT_EDEVICE", 5: "PT_ECACHE_MISS"}


class PtConfig(C.Structure):
    _fields_ = [("arch", C.c_int32), ("dtype", C.c_int32), ("L", C.c_int32), ("D", C.c_int32), ("H", C.c_int32),
                ("F", C.c_int32), ("S", C.c_int32), ("B", C.c_int32), ("n_out", C.c_int32), ("img", C.c_int32),
                ("patch", C.c_int32), ("chans", C.c_int32), ("vocab", C.c_int32), ("max_pos", C.c_int32),
                ("ln_eps", C.c_float), ("optimizer", C.c_int32), ("head", C.c_int32), ("grad_accum", C.c_int32),
                ("k_min", C.c_int32), ("cache_slots", C.c_int64), ("host_slots", C.c_int64), ("window_slots", C.c_int64)]


class PtOptHparams(C.Structure):
    _fields_ = [("lr", C.c_float), ("momentum", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("weight_decay", C.c_float)]


class PtError(RuntimeError):
    def __init__(self, status, msg=""):
        super().__init__(f"{_STATUS.get(status, status)}: {msg}")
        self.status = status


_lib = None


def load_library():
    """Loads libpt.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2102_03161_amd.build`")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    P = C.POINTER
    sig = {
        "pt_query_arena_bytes": [P(PtConfig), P(sz), P(sz), P(sz), P(sz)],
        "pt_create": [P(PtConfig), vp, vp, vp, vp, vp, P(vp)],
        "pt_destroy": [vp],
        "pt_set_freeze_boundary": [vp, i32],
        "pt_get_freeze_boundary": [vp, P(i32)],
        "pt_frozen_forward": [vp, vp, i32, P(i64), P(vp)],
        "pt_active_fwd_bwd": [vp, vp, vp, P(C.c_float)],
        "pt_last_loss": [vp, P(C.c_float)],
        "pt_layer_grad_norms": [vp, P(C.c_float)],
        "pt_layer_grad_norms_begin": [vp],
        "pt_layer_grad_norms_end": [vp, P(C.c_float)],
        "pt_layer_grad_norms_static": [vp, P(C.c_float)],
        "pt_optimizer_step": [vp, P(PtOptHparams)],
        "pt_accumulate_grads": [vp, i32],
        "pt_finish_accumulation": [vp, P(C.c_float)],
        "pt_next_boundary": [P(C.c_float), i32, i32, C.c_double, P(i32)],
        "pt_num_tensors": [vp, P(i32)],
        "pt_tensor_info": [vp, i32, C.c_char_p, sz, P(i64), P(i32), P(i32), P(i32), P(i32)],
        "pt_write_tensor": [vp, i32, i32, P(C.c_float)],
        "pt_read_tensor": [vp, i32, i32, P(C.c_float)],
        "pt_get_step_count": [vp, P(i64)],
        "pt_set_step_count": [vp, i64],
        "pt_read_activation": [vp, i32, P(C.c_float), sz],
        "pt_cache_row": [vp, i64, vp, sz, P(i32)],
        "pt_cache_stats": [vp, P(i64), P(i64), P(i64), P(i64)],
        "pt_time_frozen_forward": [vp, vp, i32, P(i64), i32, P(C.c_float), P(C.c_float)],
        "pt_attach_host_tier": [vp, vp, sz],
        "pt_cache_prefetch": [vp, P(i64), i32, P(i32)],
        "pt_host_tier_stats": [vp, P(i64), P(i64), P(i64), P(i64)],
        "pt_profile_enable": [vp, i32],
        "pt_profile_reset": [vp],
        "pt_profile_read": [vp, i32, P(C.c_double), P(i64), P(C.c_double)],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.pt_last_error.argtypes = [vp]
    lib.pt_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def make_config(w: dict, B: int | None = None, cache_slots: int = 0, grad_accum: bool = False,
                host_slots: int = 0, window_slots: int = 0, k_min: int = 0) -> PtConfig:
    """pt_config from a workload dict (see synth.WORKLOADS)."""
    return PtConfig(
        arch=PT_VIT_PRELN if w["arch"] == "vit" else PT_BERT_POSTLN,
        dtype=PT_BF16 if w["dtype"] == "bf16" else PT_F32,
        L=w["L"], D=w["D"], H=w["H"], F=w["F"], S=w["S"], B=w["B"] if B is None else B, n_out=w["n_out"],
        img=w["img"], patch=w["patch"], chans=w["chans"], vocab=w["vocab"], max_pos=w["max_pos"],
        ln_eps=w["ln_eps"], optimizer=PT_ADAMW if w["optimizer"] == "adamw" else PT_SGDM,
        head=PT_HEAD_CLS if w.get("head", "default") == "cls" else PT_HEAD_DEFAULT, grad_accum=1 if grad_accum else 0,
        k_min=k_min, cache_slots=cache_slots, host_slots=host_slots, window_slots=window_slots)


def query_arena_bytes(cfg: PtConfig):
    lib = load_library()
    a, b, c, d = C.c_size_t(), C.c_size_t(), C.c_size_t(), C.c_size_t()
    st = lib.pt_query_arena_bytes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c), C.byref(d))
    if st != PT_OK:
        raise PtError(st, "pt_query_arena_bytes")
    return a.value, b.value, c.value, d.value


def next_boundary(norms, L: int, k_prev: int, alpha: float) -> int:
    lib = load_library()
    arr = np.ascontiguousarray(norms, dtype=np.float32)
    out = C.c_int32()
    st = lib.pt_next_boundary(arr.ctypes.data_as(C.POINTER(C.c_float)), L, k_prev, alpha, C.byref(out))
    if st != PT_OK:
        raise PtError(st, "pt_next_boundary")
    return out.value


class Context:
    """Owns the device arenas (torch tensors) and a pt_ctx."""

    def __init__(self, cfg: PtConfig, device="cuda:0", stream=None):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        sizes = query_arena_bytes(cfg)
        with torch.cuda.device(self.device):
            self.arenas = [torch.empty(max(n, 256), dtype=torch.uint8, device=self.device) for n in sizes]
            self.stream = torch.cuda.current_stream(self.device) if stream is None else stream
            h = C.c_void_p()
            st = self.lib.pt_create(C.byref(cfg), *[C.c_void_p(a.data_ptr()) for a in self.arenas[:3]],
                                    C.c_void_p(self.arenas[3].data_ptr()) if cfg.cache_slots + cfg.window_slots > 0 else None,
                                    C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if st != PT_OK:
            raise PtError(st, "pt_create")
        self.h = h
        self.esz = 2 if cfg.dtype == PT_BF16 else 4
        self._names = None
        self.host_tier = None
        if cfg.host_slots > 0:
            # the lower cache tier: pinned host memory owned here, attached once
            nbytes = cfg.host_slots * cfg.S * cfg.D * self.esz
            self.host_tier = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
            self._chk(self.lib.pt_attach_host_tier(self.h, C.c_void_p(self.host_tier.data_ptr()), nbytes))

    def close(self):
        if self.h:
            self.lib.pt_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _chk(self, st, allow=()):
        if st != PT_OK and st not in allow:
            raise PtError(st, (self.lib.pt_last_error(self.h) or b"").decode())
        return st

    # ---- the five calls ------------------------------------------------------
    def set_freeze_boundary(self, k: int):
        self._chk(self.lib.pt_set_freeze_boundary(self.h, k))

    def get_freeze_boundary(self) -> int:
        k = C.c_int32()
        self._chk(self.lib.pt_get_freeze_boundary(self.h, C.byref(k)))
        return k.value

    def frozen_forward(self, d_input, sample_ids=None) -> int:
        """d_input: torch tensor on the device.  Returns the device pointer of h_k."""
        nb = int(d_input.shape[0])
        ids = None
        if sample_ids is not None:
            arr = np.ascontiguousarray(sample_ids, dtype=np.int64)
            assert arr.shape == (nb,)
            ids = arr.ctypes.data_as(C.POINTER(C.c_int64))
        out = C.c_void_p()
        self._chk(self.lib.pt_frozen_forward(self.h, C.c_void_p(d_input.data_ptr()), nb, ids, C.byref(out)))
        return out.value

    def active_fwd_bwd(self, d_hk: int, d_labels, want_loss=True):
        loss = C.c_float()
        self._chk(self.lib.pt_active_fwd_bwd(self.h, C.c_void_p(d_hk), C.c_void_p(d_labels.data_ptr()),
                                             C.byref(loss) if want_loss else None))
        return loss.value if want_loss else None

    def last_loss(self) -> float:
        loss = C.c_float()
        self._chk(self.lib.pt_last_loss(self.h, C.byref(loss)))
        return loss.value

    def layer_grad_norms(self) -> np.ndarray:
        out = np.zeros(self.cfg.L + 2, dtype=np.float32)
        self._chk(self.lib.pt_layer_grad_norms(self.h, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def layer_grad_norms_static(self) -> np.ndarray:
        out = np.zeros(self.cfg.L + 2, dtype=np.float32)
        self._chk(self.lib.pt_layer_grad_norms_static(self.h, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def layer_grad_norms_begin(self):
        self._chk(self.lib.pt_layer_grad_norms_begin(self.h))

    def layer_grad_norms_end(self) -> np.ndarray:
        out = np.zeros(self.cfg.L + 2, dtype=np.float32)
        self._chk(self.lib.pt_layer_grad_norms_end(self.h, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def accumulate_grads(self, first: bool):
        self._chk(self.lib.pt_accumulate_grads(self.h, 1 if first else 0))

    def finish_accumulation(self, want_loss: bool = True):
        out = C.c_float()
        self._chk(self.lib.pt_finish_accumulation(self.h, C.byref(out) if want_loss else None))
        return out.value if want_loss else None

    def optimizer_step(self, lr, momentum=0.9, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
        hp = PtOptHparams(lr, momentum, beta1, beta2, eps, weight_decay)
        self._chk(self.lib.pt_optimizer_step(self.h, C.byref(hp)))

    # ---- tensor table --------------------------------------------------------
    def tensors(self):
        """[(id, name, shape, group, decayed)] in arena order."""
        if self._names is None:
            n = C.c_int32()
            self._chk(self.lib.pt_num_tensors(self.h, C.byref(n)))
            out = []
            for i in range(n.value):
                buf = C.create_string_buffer(64)
                numel, rows, cols, grp, dec = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32()
                self._chk(self.lib.pt_tensor_info(self.h, i, buf, 64, C.byref(numel), C.byref(rows), C.byref(cols),
                                                  C.byref(grp), C.byref(dec)))
                shape = (cols.value,) if rows.value == 1 else (rows.value, cols.value)
                out.append((i, buf.value.decode(), shape, grp.value, bool(dec.value)))
            self._names = out
        return self._names

    def write_tensor(self, tid: int, kind: int, arr):
        a = np.ascontiguousarray(arr, dtype=np.float32)
        self._chk(self.lib.pt_write_tensor(self.h, tid, kind, a.ctypes.data_as(C.POINTER(C.c_float))))

    def read_tensor(self, tid: int, kind: int) -> np.ndarray:
        _, _, shape, _, _ = self.tensors()[tid]
        out = np.empty(shape, dtype=np.float32)
        self._chk(self.lib.pt_read_tensor(self.h, tid, kind, out.ctypes.data_as(C.POINTER(C.c_float))))
        return out

    def get_step_count(self) -> int:
        t = C.c_int64()
        self._chk(self.lib.pt_get_step_count(self.h, C.byref(t)))
        return t.value

    def set_step_count(self, t: int):
        self._chk(self.lib.pt_set_step_count(self.h, t))

    def read_activation(self, which: int, shape) -> np.ndarray:
        out = np.empty(shape, dtype=np.float32)
        self._chk(self.lib.pt_read_activation(self.h, which, out.ctypes.data_as(C.POINTER(C.c_float)), out.size))
        return out

    # ---- cache ---------------------------------------------------------------
    def cache_row(self, sample_id: int):
        """(raw row bytes as uint8 array, k the row was written at) or None on a miss."""
        n = self.cfg.S * self.cfg.D * self.esz
        out = np.empty(n, dtype=np.uint8)
        k = C.c_int32()
        st = self._chk(self.lib.pt_cache_row(self.h, sample_id, C.c_void_p(out.ctypes.data), n, C.byref(k)),
                       allow=(PT_ECACHE_MISS,))
        return None if st == PT_ECACHE_MISS else (out, k.value)

    def cache_stats(self):
        a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        self._chk(self.lib.pt_cache_stats(self.h, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return {"hits": a.value, "advances": b.value, "misses": c.value, "block_runs": d.value}

    def time_frozen_forward(self, d_input, sample_ids, reps: int = 3):
        """(ms per call recomputing the prefix, ms per call served from the cache) for this batch."""
        ids = np.ascontiguousarray(sample_ids, dtype=np.int64)
        a, b = C.c_float(), C.c_float()
        self._chk(self.lib.pt_time_frozen_forward(self.h, C.c_void_p(d_input.data_ptr()), len(ids),
                                                  ids.ctypes.data_as(C.POINTER(C.c_int64)), reps, C.byref(a), C.byref(b)))
        return a.value, b.value

    def cache_prefetch(self, sample_ids) -> int:
        ids = np.ascontiguousarray(sample_ids, dtype=np.int64)
        n = C.c_int32()
        self._chk(self.lib.pt_cache_prefetch(self.h, ids.ctypes.data_as(C.POINTER(C.c_int64)), len(ids), C.byref(n)))
        return n.value

    def host_tier_stats(self):
        a, b, c, d = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int64()
        self._chk(self.lib.pt_host_tier_stats(self.h, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return {"rows_to_device": a.value, "rows_to_host": b.value, "prefetched": c.value, "prefetched_used": d.value}

    # ---- kernel timing ---------------------------------------------------------
    def profile_enable(self, on: bool):
        self._chk(self.lib.pt_profile_enable(self.h, 1 if on else 0))

    def profile_reset(self):
        self._chk(self.lib.pt_profile_reset(self.h))

    def profile_read(self) -> dict:
        """{category: (total_ms, launches, work)}"""
        out = {}
        for i, name in enumerate(PROF_CATEGORIES):
            ms, n, wk = C.c_double(), C.c_int64(), C.c_double()
            self._chk(self.lib.pt_profile_read(self.h, i, C.byref(ms), C.byref(n), C.byref(wk)))
            out[name] = (ms.value, n.value, wk.value)
        return out
