"""ctypes binding of libadwin_opd: argument marshalling only.

Every step of the path runs inside the library's HIP kernels; torch is used for device
memory (`torch.empty(..., device="cuda")`, `.data_ptr()`) and for the current stream
handle.  There is no CPU fallback: if the shared library is missing the import of this
module fails, and the compute entry points fail with a status if no GPU is present.
The function names are those of include/adwin_opd.h.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# ADWIN_OPD_LIB: load another build of the same library (A/B timing of kernel variants)
LIB_PATH = os.environ.get("ADWIN_OPD_LIB") or os.path.join(_HERE, "libadwin_opd.so")

ADWIN_OK = 0
ADWIN_E_NULL, ADWIN_E_SHAPE, ADWIN_E_OFFSETS, ADWIN_E_WINDOW = -1, -2, -3, -4
ADWIN_E_ALIGN, ADWIN_E_WORKSPACE, ADWIN_E_MODE, ADWIN_E_HIP = -5, -6, -7, -8
ADWIN_PREFIX_ONLY, ADWIN_PREFIX_AND_FULL = 0, 1
ADWIN_RED_SEQ_MEAN, ADWIN_RED_SUM, ADWIN_RED_TOKEN_MEAN = 0, 1, 2
ADWIN_DT_BF16, ADWIN_DT_F32 = 0, 1
ADWIN_DEV_BAD_ID, ADWIN_DEV_NONFINITE = 1, 2
ADWIN_MAX_CANDIDATES = 16
ADWIN_STATIC_SCRATCH_BYTES = 1 << 20
ADWIN_EST_EXPECTED, ADWIN_EST_SAMPLED = 0, 1
ADWIN_SCHEME_AUTO, ADWIN_SCHEME_SINGLE, ADWIN_SCHEME_TWO_SWEEP, ADWIN_SCHEME_TWO_SWEEP_REG = 0, 1, 2, 3
ADWIN_LOGITS_AUTO, ADWIN_LOGITS_RESIDENT, ADWIN_LOGITS_STREAMING = 0, 1, 2


class adwin_opd_problem(C.Structure):
    _fields_ = [
        ("struct_bytes", C.c_size_t), ("T", C.c_int64),
        ("B", C.c_int32), ("V", C.c_int32), ("H_s", C.c_int32), ("H_t", C.c_int32),
        ("offsets", C.c_void_p), ("window", C.c_void_p),
        ("h_s", C.c_void_p), ("h_t", C.c_void_p), ("W_s", C.c_void_p), ("W_t", C.c_void_p),
        ("ids", C.c_void_p),
        ("mode", C.c_int32), ("reduction", C.c_int32), ("grad_scale", C.c_float),
        ("dh_dtype", C.c_int32),
        ("kl", C.c_void_p), ("c", C.c_void_p), ("dh_prefix", C.c_void_p), ("dh_full", C.c_void_p),
        ("loss_prefix", C.c_void_p), ("loss_full", C.c_void_p),
        ("rho_pooled", C.c_void_p), ("rho_field", C.c_void_p), ("batch", C.c_void_p),
        ("n_out", C.c_void_p), ("n_adm_out", C.c_void_p), ("status_dev", C.c_void_p),
        ("candidates", C.c_void_p), ("n_candidates", C.c_int32),
        ("cand_rho_pooled", C.c_void_p), ("cand_rho_field", C.c_void_p), ("cand_batch", C.c_void_p),
        ("t_logp", C.c_void_p), ("t_entropy", C.c_void_p), ("t_rank", C.c_void_p),
        ("estimator", C.c_int32),
        ("dW_prefix", C.c_void_p), ("dW_full", C.c_void_p),
        ("topk", C.c_int32), ("t_first_reject", C.c_void_p), ("t_logp_mean", C.c_void_p),
        ("cand_loss_share", C.c_void_p),
        ("scheme", C.c_int32),
    ]


class adwin_opd_logits_problem(C.Structure):
    _fields_ = [
        ("struct_bytes", C.c_size_t), ("T", C.c_int64), ("B", C.c_int32), ("V", C.c_int32),
        ("offsets", C.c_void_p), ("window", C.c_void_p),
        ("z_s", C.c_void_p), ("z_t", C.c_void_p), ("ids", C.c_void_p),
        ("reduction", C.c_int32), ("grad_scale", C.c_float),
        ("kl", C.c_void_p), ("c", C.c_void_p), ("dz", C.c_void_p),
        ("loss_prefix", C.c_void_p), ("batch", C.c_void_p),
        ("n_out", C.c_void_p), ("n_adm_out", C.c_void_p), ("status_dev", C.c_void_p),
        ("t_logp", C.c_void_p), ("t_entropy", C.c_void_p), ("t_rank", C.c_void_p),
        ("estimator", C.c_int32),
        ("topk", C.c_int32), ("t_first_reject", C.c_void_p), ("t_logp_mean", C.c_void_p),
        ("scheme", C.c_int32),
    ]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; "
            "g.build()').  There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    lib.adwin_opd_version.restype = C.c_int
    lib.adwin_opd_strerror.restype = C.c_char_p
    lib.adwin_opd_strerror.argtypes = [C.c_int]
    lib.adwin_opd_plan_host.restype = C.c_int
    lib.adwin_opd_plan_host.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.c_void_p, C.c_void_p, C.c_void_p]
    lib.adwin_opd_snr.restype = C.c_int
    lib.adwin_opd_snr.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    lib.adwin_opd_next_window.restype = C.c_int
    lib.adwin_opd_next_window.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_float, C.c_void_p]
    lib.adwin_opd_probe_staleness.restype = C.c_int
    lib.adwin_opd_probe_staleness.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p,
                                              C.c_void_p]
    lib.adwin_opd_workspace_bytes.restype = C.c_int
    lib.adwin_opd_workspace_bytes.argtypes = [C.POINTER(adwin_opd_problem), C.POINTER(C.c_size_t)]
    lib.adwin_opd_fused_launch_info.restype = C.c_int
    lib.adwin_opd_fused_launch_info.argtypes = [C.POINTER(adwin_opd_problem), C.POINTER(C.c_int64)]
    lib.adwin_opd_fused.restype = C.c_int
    lib.adwin_opd_fused.argtypes = [C.POINTER(adwin_opd_problem), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.adwin_opd_logits_workspace_bytes.restype = C.c_int
    lib.adwin_opd_logits_workspace_bytes.argtypes = [C.POINTER(adwin_opd_logits_problem),
                                                     C.POINTER(C.c_size_t)]
    lib.adwin_opd_from_logits.restype = C.c_int
    lib.adwin_opd_from_logits.argtypes = [C.POINTER(adwin_opd_logits_problem), C.c_void_p,
                                          C.c_size_t, C.c_void_p]
    lib.adwin_opd_from_logits_static.restype = C.c_int
    lib.adwin_opd_from_logits_static.argtypes = [C.POINTER(adwin_opd_logits_problem), C.c_void_p]
    lib.adwin_opd_fused_profile.restype = C.c_int
    lib.adwin_opd_fused_profile.argtypes = [C.POINTER(adwin_opd_problem), C.c_void_p, C.c_size_t,
                                            C.c_void_p, C.POINTER(C.c_float)]
    lib.adwin_opd_from_logits_profile.restype = C.c_int
    lib.adwin_opd_from_logits_profile.argtypes = [C.POINTER(adwin_opd_logits_problem), C.c_void_p,
                                                  C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
    lib.adwin_opd_init.restype = C.c_int
    lib.adwin_opd_init.argtypes = []
    lib.adwin_opd_ceiling_copy.restype = C.c_int
    lib.adwin_opd_ceiling_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_void_p,
                                           C.POINTER(C.c_float)]
    lib.adwin_opd_ceiling_mfma.restype = C.c_int
    lib.adwin_opd_ceiling_mfma.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.POINTER(C.c_float)]
    lib.adwin_opd_ceiling_mfma_random.restype = C.c_int
    lib.adwin_opd_ceiling_mfma_random.argtypes = [C.c_void_p, C.c_int, C.c_void_p, C.POINTER(C.c_float)]
    return lib


lib = _load()

ADWIN_N_PHASES = 6
PHASE_NAMES = ("setup", "stats", "merge", "dz", "grad", "reduce")


class AdwinError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"libadwin_opd status {status}: {adwin_opd_strerror(status)}")


def _check(status: int) -> None:
    if status != ADWIN_OK:
        raise AdwinError(status)


def adwin_opd_version() -> int:
    return int(lib.adwin_opd_version())


def adwin_opd_strerror(status: int) -> str:
    return lib.adwin_opd_strerror(int(status)).decode()


def _host_i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def adwin_opd_plan_host(offsets, window, T=None, want_rows: bool = True) -> dict:
    """Host integer bookkeeping; returns n[B], n_adm and (optionally) the admitted-row list."""
    off, win = _host_i64(offsets), _host_i32(window)
    B = int(win.shape[0])
    T = int(off[-1]) if T is None else int(T)
    n = np.zeros(B, np.int32)
    n_adm = C.c_int64(0)
    st = lib.adwin_opd_plan_host(T, B, off.ctypes.data, win.ctypes.data, n.ctypes.data, None, None,
                                 C.addressof(n_adm))
    _check(st)
    out = {"n": n, "n_adm": int(n_adm.value)}
    if want_rows:
        rows = np.zeros(max(1, out["n_adm"]), np.int64)
        seq = np.zeros(max(1, out["n_adm"]), np.int32)
        _check(lib.adwin_opd_plan_host(T, B, off.ctypes.data, win.ctypes.data, n.ctypes.data,
                                       rows.ctypes.data, seq.ctypes.data, C.addressof(n_adm)))
        out["rows"], out["row_seq"] = rows[:out["n_adm"]], seq[:out["n_adm"]]
    return out


def adwin_opd_snr(rho) -> np.ndarray:
    r = np.ascontiguousarray(np.asarray(rho, dtype=np.float32))
    out = np.zeros_like(r)
    _check(lib.adwin_opd_snr(r.ctypes.data, int(r.shape[0]), out.ctypes.data))
    return out


def adwin_opd_next_window(rho, candidates, rho_star: float = 0.0) -> int:
    r = np.ascontiguousarray(np.asarray(rho, dtype=np.float32))
    c = _host_i32(candidates)
    nxt = C.c_int32(0)
    _check(lib.adwin_opd_next_window(r.ctypes.data, c.ctypes.data, int(c.shape[0]), float(rho_star),
                                     C.addressof(nxt)))
    return int(nxt.value)


def adwin_opd_probe_staleness(age, pending, limit: int = 5):
    """Advances `age` (int32 array, in place); returns (force[n] uint8, n_forced)."""
    assert age.dtype == np.int32 and age.flags.c_contiguous
    pend = np.ascontiguousarray(np.asarray(pending, dtype=np.uint8))
    force = np.zeros(age.shape[0], np.uint8)
    cnt = C.c_int32(0)
    _check(lib.adwin_opd_probe_staleness(age.ctypes.data, pend.ctypes.data, int(age.shape[0]), int(limit),
                                         force.ctypes.data, C.addressof(cnt)))
    return force, int(cnt.value)


def _ptr(t) -> int | None:
    return None if t is None else int(t.data_ptr())


def _stream_handle(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None


class FusedCall:
    """A marshalled adwin_opd_fused call: problem struct, output tensors and workspace,
    all allocated once; `run()` only enqueues."""

    DEFAULT_OUTPUTS = ("kl", "c", "dh_prefix", "dh_full", "loss_prefix", "loss_full", "rho_pooled",
                       "rho_field", "batch", "n_out", "n_adm_out", "status_dev")

    def __init__(self, h_s, h_t, W_s, W_t, ids, offsets, window, mode=ADWIN_PREFIX_ONLY,
                 reduction=ADWIN_RED_SEQ_MEAN, grad_scale=1.0, dh_dtype=ADWIN_DT_F32,
                 want=DEFAULT_OUTPUTS, topk=0, device=None, allocate=True, candidates=None, estimator=ADWIN_EST_EXPECTED,
                 cand_outputs=True, scheme=ADWIN_SCHEME_AUTO):
        self.offsets, self.window = _host_i64(offsets), _host_i32(window)
        self.candidates = None if candidates is None else _host_i32(candidates)
        self.inputs = (h_s, h_t, W_s, W_t, ids)
        B = int(self.window.shape[0])
        T = int(h_s.shape[0]) if h_s is not None else int(self.offsets[-1])
        V, H_s = int(W_s.shape[0]), int(W_s.shape[1])
        H_t = int(W_t.shape[1])
        dev = device if device is not None else (h_s.device if h_s is not None else "cuda")
        self.device = dev
        p = adwin_opd_problem()
        p.struct_bytes = C.sizeof(adwin_opd_problem)
        p.T, p.B, p.V, p.H_s, p.H_t = T, B, V, H_s, H_t
        p.offsets, p.window = self.offsets.ctypes.data, self.window.ctypes.data
        p.h_s, p.h_t, p.W_s, p.W_t, p.ids = _ptr(h_s), _ptr(h_t), _ptr(W_s), _ptr(W_t), _ptr(ids)
        p.mode, p.reduction, p.grad_scale, p.dh_dtype = mode, reduction, float(grad_scale), dh_dtype
        p.estimator = estimator
        p.scheme = scheme
        p.topk = int(topk)
        K = 0 if self.candidates is None else int(self.candidates.shape[0])
        if K:
            p.candidates, p.n_candidates = self.candidates.ctypes.data, K
        self.p = p
        self.out = {}
        self.workspace = None
        self.workspace_bytes = 0
        if allocate:
            dh_t = torch.bfloat16 if dh_dtype == ADWIN_DT_BF16 else torch.float32
            shapes = {
                "kl": ((T,), torch.float32), "c": ((T,), torch.float32),
                "dh_prefix": ((T, H_s), dh_t), "dh_full": ((T, H_s), dh_t),
                "loss_prefix": ((B,), torch.float32), "loss_full": ((B,), torch.float32),
                "rho_pooled": ((B,), torch.float32), "rho_field": ((B,), torch.float32),
                "batch": ((8,), torch.float32), "n_out": ((B,), torch.int32),
                "n_adm_out": ((1,), torch.int64), "status_dev": ((1,), torch.int32),
                "t_logp": ((T,), torch.float32), "t_entropy": ((T,), torch.float32),
                "t_rank": ((T,), torch.int32),
                "dW_prefix": ((V, H_s), torch.float32), "dW_full": ((V, H_s), torch.float32),
                "t_first_reject": ((B,), torch.int32), "t_logp_mean": ((B + 1, 2), torch.float32),
                "cand_loss_share": ((K,), torch.float32),
            }
            for k in want:
                if k in ("dh_full", "dW_full") and mode != ADWIN_PREFIX_AND_FULL:
                    continue
                shp, dt = shapes[k]
                self.out[k] = torch.empty(shp, dtype=dt, device=dev)
                setattr(p, k, _ptr(self.out[k]))
            if K and cand_outputs:     # the audit's alignment outputs; cand_loss_share goes through `want`
                for k, shp in (("cand_rho_pooled", (K, B)), ("cand_rho_field", (K, B)),
                               ("cand_batch", (K, 4))):
                    self.out[k] = torch.empty(shp, dtype=torch.float32, device=dev)
                    setattr(p, k, _ptr(self.out[k]))
            self.workspace_bytes = adwin_opd_workspace_bytes(p)
            self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=dev)

    def _ws_ptr(self) -> int:
        return (int(self.workspace.data_ptr()) + 255) // 256 * 256

    def run(self, stream=None) -> int:
        return int(lib.adwin_opd_fused(C.byref(self.p), self._ws_ptr(), self.workspace_bytes,
                                       _stream_handle(stream)))


def adwin_opd_fused_profile(call: "FusedCall", stream=None) -> dict:
    """Runs the call with per-phase HIP-event timing; returns {phase name: ms}."""
    ms = (C.c_float * ADWIN_N_PHASES)()
    _check(lib.adwin_opd_fused_profile(C.byref(call.p), call._ws_ptr(), call.workspace_bytes,
                                       _stream_handle(stream), ms))
    return dict(zip(PHASE_NAMES, [float(x) for x in ms]))


def adwin_opd_from_logits_profile(call: "LogitsCall", stream=None) -> dict:
    ms = (C.c_float * ADWIN_N_PHASES)()
    _check(lib.adwin_opd_from_logits_profile(C.byref(call.p), call._ws_ptr(), call.workspace_bytes,
                                             _stream_handle(stream), ms))
    return dict(zip(PHASE_NAMES, [float(x) for x in ms]))


def adwin_opd_workspace_bytes(p: adwin_opd_problem) -> int:
    n = C.c_size_t(0)
    _check(lib.adwin_opd_workspace_bytes(C.byref(p), C.byref(n)))
    return int(n.value)


def adwin_opd_fused_launch_info(p: adwin_opd_problem) -> dict:
    info = (C.c_int64 * 4)()
    _check(lib.adwin_opd_fused_launch_info(C.byref(p), info))
    return {"rows": int(info[0]), "padded_rows": int(info[1]), "slab_rows": int(info[2]),
            "slabs": int(info[3])}


def adwin_opd_fused(h_s, h_t, W_s, W_t, ids, offsets, window, stream=None, **kw) -> dict:
    """One fused call; returns the output tensors (device)."""
    call = FusedCall(h_s, h_t, W_s, W_t, ids, offsets, window, **kw)
    _check(call.run(stream))
    return call.out


class LogitsCall:
    """A marshalled adwin_opd_from_logits call (see FusedCall)."""

    def __init__(self, z_s, z_t, ids, offsets, window, reduction=ADWIN_RED_SEQ_MEAN, grad_scale=1.0,
                 want=("kl", "c", "dz", "loss_prefix", "batch", "n_out", "n_adm_out", "status_dev"),
                 allocate=True, estimator=ADWIN_EST_EXPECTED, topk=0, scheme=ADWIN_LOGITS_AUTO,
                 workspace=True):
        self.offsets, self.window = _host_i64(offsets), _host_i32(window)
        self.inputs = (z_s, z_t, ids)
        B = int(self.window.shape[0])
        T, V = int(z_s.shape[0]), int(z_s.shape[1])
        dev = z_s.device
        p = adwin_opd_logits_problem()
        p.struct_bytes = C.sizeof(adwin_opd_logits_problem)
        p.T, p.B, p.V = T, B, V
        p.offsets, p.window = self.offsets.ctypes.data, self.window.ctypes.data
        p.z_s, p.z_t, p.ids = _ptr(z_s), _ptr(z_t), _ptr(ids)
        p.reduction, p.grad_scale = reduction, float(grad_scale)
        p.estimator = estimator
        p.scheme = scheme
        p.topk = int(topk)
        self.p = p
        self.out = {}
        self.workspace = None
        self.workspace_bytes = 0
        if allocate:
            shapes = {
                "t_first_reject": ((B,), torch.int32), "t_logp_mean": ((B + 1, 2), torch.float32),
                "kl": ((T,), torch.float32), "c": ((T,), torch.float32),
                "dz": ((T, V), torch.bfloat16), "loss_prefix": ((B,), torch.float32),
                "batch": ((8,), torch.float32), "n_out": ((B,), torch.int32),
                "n_adm_out": ((1,), torch.int64), "status_dev": ((1,), torch.int32),
                "t_logp": ((T,), torch.float32), "t_entropy": ((T,), torch.float32),
                "t_rank": ((T,), torch.int32),
            }
            for k in want:
                shp, dt = shapes[k]
                self.out[k] = torch.empty(shp, dtype=dt, device=dev)
                setattr(p, k, _ptr(self.out[k]))
            self.workspace_bytes = adwin_opd_logits_workspace_bytes(p)
            if workspace:       # run_static() needs none
                self.workspace = torch.empty(self.workspace_bytes + 256, dtype=torch.uint8, device=dev)

    def _ws_ptr(self) -> int:
        return (int(self.workspace.data_ptr()) + 255) // 256 * 256

    def run(self, stream=None) -> int:
        return int(lib.adwin_opd_from_logits(C.byref(self.p), self._ws_ptr(), self.workspace_bytes,
                                             _stream_handle(stream)))

    def run_static(self, stream=None) -> int:
        """The same call through the entry point that takes no workspace and allocates nothing."""
        return int(lib.adwin_opd_from_logits_static(C.byref(self.p), _stream_handle(stream)))


def adwin_opd_logits_workspace_bytes(p: adwin_opd_logits_problem) -> int:
    n = C.c_size_t(0)
    _check(lib.adwin_opd_logits_workspace_bytes(C.byref(p), C.byref(n)))
    return int(n.value)


def adwin_opd_from_logits(z_s, z_t, ids, offsets, window, stream=None, **kw) -> dict:
    call = LogitsCall(z_s, z_t, ids, offsets, window, **kw)
    _check(call.run(stream))
    return call.out


def adwin_opd_from_logits_static(z_s, z_t, ids, offsets, window, stream=None, **kw) -> dict:
    """adwin_opd_from_logits with the library's own static scratch (outputs are still allocated
    here, by torch; the library call itself allocates nothing)."""
    call = LogitsCall(z_s, z_t, ids, offsets, window, workspace=False, **kw)
    _check(call.run_static(stream))
    return call.out


def adwin_opd_init() -> None:
    """Sets the kernel attributes on the current device (optional; see the header)."""
    _check(lib.adwin_opd_init())


def adwin_opd_ceiling_copy(nbytes: int = 1 << 30, reps: int = 10, stream=None) -> float:
    """Measured streaming-copy rate in GB/s (read + write bytes)."""
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").zero_()
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    ms = C.c_float(0)
    _check(lib.adwin_opd_ceiling_copy(_ptr(src), _ptr(dst), nbytes, reps, _stream_handle(stream),
                                      C.byref(ms)))
    return 2.0 * nbytes / (ms.value * 1e-3) / 1e9


def adwin_opd_ceiling_mfma(iters: int = 20000, stream=None) -> float:
    """Measured register-resident bf16 MFMA rate in TFLOP/s."""
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    tf = C.c_float(0)
    _check(lib.adwin_opd_ceiling_mfma(_ptr(scratch), iters, _stream_handle(stream), C.byref(tf)))
    return float(tf.value)


def adwin_opd_ceiling_mfma_random(iters: int = 20000, stream=None) -> float:
    """Measured bf16 MFMA rate in TFLOP/s with pseudo-random operands."""
    scratch = torch.zeros(16, dtype=torch.float32, device="cuda")
    tf = C.c_float(0)
    _check(lib.adwin_opd_ceiling_mfma_random(_ptr(scratch), iters, _stream_handle(stream), C.byref(tf)))
    return float(tf.value)
