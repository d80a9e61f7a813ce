"""ctypes binding of libfastclip.so: the same names as include/fastclip.h, argument marshalling only.

PyTorch is used for nothing but device memory (`tensor.data_ptr()`) and the current
stream handle; every step of the path runs in the library's HIP kernels.  There is no
CPU or PyTorch fallback: if the library cannot be loaded, calls raise.
"""
from __future__ import annotations

import ctypes as C
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libfastclip.so")

OK, ERR_NULL, ERR_SHAPE, ERR_VALUE, ERR_WORKSPACE, ERR_UNSUPPORTED, ERR_LAUNCH, ERR_INDEX = range(8)
V0, V1, V2, V3 = 0, 1, 2, 3
GATHERED_STATE = 1
FINE_TILES = 2
SINGLE_PASS = 4
TILES_128 = 8
TILES_256 = 16
F32, BF16 = 0, 1
N_PHASES = 8


class fastclip_plan(C.Structure):
    _fields_ = [("tile", C.c_int32), ("single_pass", C.c_int32), ("gathered", C.c_int32), ("fused_state", C.c_int32),
                ("nsplit", C.c_int32), ("nparts", C.c_int32)]


class fastclip_config(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("version", C.c_int32), ("emb_dtype", C.c_int32),
                ("flags", C.c_int32),
                ("B", C.c_int64), ("b", C.c_int64), ("off", C.c_int64), ("d", C.c_int64),
                ("ld_img", C.c_int64), ("ld_txt", C.c_int64), ("N", C.c_int64), ("state_stride", C.c_int64),
                ("gamma", C.c_float), ("eps", C.c_float), ("rho", C.c_float), ("tau_grad_scale", C.c_float)]


_BUF_FIELDS = ["img_glob", "txt_glob", "idx", "u_img", "u_txt", "tau", "tau_img", "tau_txt", "d_img", "d_txt",
               "loss", "d_tau", "d_tau_img", "d_tau_txt", "g_img", "g_txt", "u_new_img", "u_new_txt",
               "u_glob_img", "u_glob_txt", "tau_glob_img", "tau_glob_txt", "norm_img", "norm_txt"]


class fastclip_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _BUF_FIELDS]


TAU_SGDM, TAU_LAMB, TAU_LION, TAU_ADAMW = 1, 2, 3, 4


class fastclip_tau_update(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("optimizer", C.c_int32), ("step", C.c_int64),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("tau_min", C.c_float), ("lr_drop_below", C.c_float), ("lr_drop_factor", C.c_float),
                ("state_stride", C.c_int32)]


_TAU_STATE_FIELDS = ["tau", "m", "v", "tau_img", "tau_txt", "m_img", "v_img", "m_txt", "v_txt"]


class fastclip_tau_state(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _TAU_STATE_FIELDS]


_lib = None


def load(build_if_missing: bool = True):
    """Load libfastclip.so (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise RuntimeError("libfastclip.so is not built: run __graft_entry__.build()")
        from .build import build
        build()
    # torch ships its own HIP runtime; it has to be in the process before the library is, so that the library's
    # kernels and torch's device pointers and streams belong to one and the same runtime
    import torch  # noqa: F401
    lib = C.CDLL(LIB_PATH)
    cfgp, bufp = C.POINTER(fastclip_config), C.POINTER(fastclip_buffers)
    lib.fastclip_workspace_bytes.restype = C.c_size_t
    lib.fastclip_workspace_bytes.argtypes = [cfgp]
    lib.fastclip_describe.restype = C.c_int
    lib.fastclip_describe.argtypes = [cfgp, C.POINTER(fastclip_plan)]
    lib.fastclip_validate.restype = C.c_int
    lib.fastclip_validate.argtypes = [cfgp, bufp]
    lib.fastclip_step.restype = C.c_int
    lib.fastclip_step.argtypes = [cfgp, bufp, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fastclip_step_static.restype = C.c_int
    lib.fastclip_step_static.argtypes = [cfgp, bufp, C.c_void_p]
    lib.fastclip_step_timed.restype = C.c_int
    lib.fastclip_step_timed.argtypes = [cfgp, bufp, C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_float)]
    lib.fastclip_phase_name.restype = C.c_char_p
    lib.fastclip_phase_name.argtypes = [C.c_int]
    lib.fastclip_state_update.restype = C.c_int
    lib.fastclip_state_update.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_float, C.c_float] + [C.c_void_p] * 7
    lib.fastclip_state_update_strided.restype = C.c_int
    lib.fastclip_state_update_strided.argtypes = ([C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_float, C.c_float] +
                                                  [C.c_void_p] * 7)
    lib.fastclip_check_indices_workspace_bytes.restype = C.c_size_t
    lib.fastclip_check_indices_workspace_bytes.argtypes = [C.c_int64]
    lib.fastclip_check_indices.restype = C.c_int
    lib.fastclip_check_indices.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fastclip_gamma_cosine.restype = C.c_float
    lib.fastclip_gamma_cosine.argtypes = [C.c_int64, C.c_int64, C.c_int64, C.c_float]
    lib.fastclip_status_string.restype = C.c_char_p
    lib.fastclip_status_string.argtypes = [C.c_int]
    updp, tstp = C.POINTER(fastclip_tau_update), C.POINTER(fastclip_tau_state)
    lib.fastclip_temperature_update.restype = C.c_int
    lib.fastclip_temperature_update.argtypes = [C.c_int32, updp, tstp, C.c_void_p, C.c_int64, C.c_int64, C.c_void_p,
                                                C.c_void_p, C.c_void_p, C.c_void_p]
    lib.fastclip_step_update_tau.restype = C.c_int
    lib.fastclip_step_update_tau.argtypes = [cfgp, bufp, updp, tstp, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fastclip_state_phase_workspace_bytes.restype = C.c_size_t
    lib.fastclip_state_phase_workspace_bytes.argtypes = [C.c_int64]
    lib.fastclip_state_phase.restype = C.c_int
    lib.fastclip_state_phase.argtypes = [cfgp, bufp, updp, tstp, C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.fastclip_measure_mfma_ceiling.restype = C.c_int
    lib.fastclip_measure_mfma_ceiling.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_size_t, C.c_void_p,
                                                  C.POINTER(C.c_float), C.POINTER(C.c_double)]
    lib.fastclip_measure_record_rmw.restype = C.c_int
    lib.fastclip_measure_record_rmw.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_void_p, C.c_int64, C.c_void_p]
    lib.fastclip_normalize_rows.restype = C.c_int
    lib.fastclip_normalize_rows.argtypes = [C.c_void_p, C.c_int32, C.c_int64, C.c_int64, C.c_int64, C.c_void_p, C.c_int32,
                                            C.c_int64, C.c_void_p, C.c_void_p]
    lib.fastclip_measure_strips.restype = C.c_int
    lib.fastclip_measure_strips.argtypes = [cfgp, bufp, C.c_void_p, C.c_size_t, C.c_void_p, C.c_int32, C.c_int32,
                                            C.POINTER(C.c_float), C.POINTER(C.c_double)]
    lib.fastclip_last_hip_error.restype = C.c_char_p
    lib.fastclip_last_hip_error.argtypes = []
    _lib = lib
    return lib


class FastclipError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        detail = ""
        if status == ERR_LAUNCH:
            detail = ": " + fastclip_last_hip_error()
        super().__init__("fastclip: %s (status %d)%s" % (fastclip_status_string(status), status, detail))


def make_config(*, version, emb_dtype, B, b, off, d, N, gamma, eps, rho=0.0, tau_grad_scale=1.0,
                ld_img=None, ld_txt=None, flags=0, state_stride=1) -> fastclip_config:
    return fastclip_config(C.sizeof(fastclip_config), int(version), int(emb_dtype), int(flags), int(B), int(b), int(off),
                           int(d), int(d if ld_img is None else ld_img), int(d if ld_txt is None else ld_txt),
                           int(N), int(state_stride), float(gamma), float(eps), float(rho), float(tau_grad_scale))


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise TypeError("fastclip buffers must be device tensors")
    return t.data_ptr()


def make_buffers(**tensors) -> fastclip_buffers:
    """Field name -> CUDA tensor (or raw device address, or None).  The struct holds plain addresses; the returned
    object also keeps the tensors referenced, so that a tensor passed as a temporary lives as long as the struct."""
    unknown = set(tensors) - set(_BUF_FIELDS)
    if unknown:
        raise TypeError("unknown buffer(s): %s" % sorted(unknown))
    out = fastclip_buffers(*[_ptr(tensors.get(n)) for n in _BUF_FIELDS])
    out._keepalive = tuple(tensors.values())
    return out


def make_tau_update(*, optimizer, step, lr, beta1, beta2, eps=1e-8, tau_min=0.0, lr_drop_below=0.0,
                    lr_drop_factor=1.0, state_stride=0) -> fastclip_tau_update:
    return fastclip_tau_update(C.sizeof(fastclip_tau_update), int(optimizer), int(step), float(lr), float(beta1),
                               float(beta2), float(eps), float(tau_min), float(lr_drop_below), float(lr_drop_factor),
                               int(state_stride))


def make_tau_state(**tensors) -> fastclip_tau_state:
    """Field name -> CUDA tensor (or raw device address, or None); keeps the tensors referenced like make_buffers."""
    unknown = set(tensors) - set(_TAU_STATE_FIELDS)
    if unknown:
        raise TypeError("unknown temperature state field(s): %s" % sorted(unknown))
    out = fastclip_tau_state(*[_ptr(tensors.get(n)) for n in _TAU_STATE_FIELDS])
    out._keepalive = tuple(tensors.values())
    return out


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def fastclip_workspace_bytes(cfg: fastclip_config) -> int:
    return int(load().fastclip_workspace_bytes(C.byref(cfg)))


def fastclip_describe(cfg: fastclip_config) -> dict:
    """The header's fastclip_plan as a dict; raises on an invalid configuration."""
    plan = fastclip_plan()
    st = int(load().fastclip_describe(C.byref(cfg), C.byref(plan)))
    if st != OK:
        raise RuntimeError("fastclip_describe: status %d" % st)
    return {n: int(getattr(plan, n)) for n, _ in fastclip_plan._fields_}


def fastclip_validate(cfg, bufs=None) -> int:
    return int(load().fastclip_validate(C.byref(cfg) if cfg is not None else None,
                                        C.byref(bufs) if bufs is not None else None))


def fastclip_step(cfg, bufs, workspace, workspace_bytes=None, stream=None, check=True) -> int:
    """workspace: CUDA uint8 tensor (or raw address with workspace_bytes given)."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    st = int(load().fastclip_step(C.byref(cfg), C.byref(bufs), _ptr(workspace), nbytes, _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


STATIC_SCRATCH_BYTES = 64 << 20


def fastclip_step_static(cfg, bufs, stream=None, check=True) -> int:
    """The step with its workspace in the library's static device array (no workspace argument, no allocation)."""
    st = int(load().fastclip_step_static(C.byref(cfg), C.byref(bufs), _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_measure_mfma_ceiling(workgroups, iters, workspace, stream=None) -> dict:
    """Returns {ms, flop, tflops, cycles_per_wave, ghz, cycles_per_mfma}."""
    ms = C.c_float(0.0)
    stats = (C.c_double * 4)()
    st = int(load().fastclip_measure_mfma_ceiling(int(workgroups), int(iters), _ptr(workspace),
                                                  workspace.numel() * workspace.element_size(), _stream(stream),
                                                  C.byref(ms), stats))
    if st != OK:
        raise FastclipError(st)
    return dict(ms=ms.value, flop=stats[0], tflops=stats[0] / (ms.value * 1e-3) / 1e12, cycles_per_wave=stats[1],
                ghz=stats[2], cycles_per_mfma=stats[3])


MEASURE_STRIPS_EXTRA_BYTES = 16 << 10


def fastclip_measure_strips(cfg, bufs, workspace, ablation, reps=10, stream=None) -> dict:
    """workspace: fastclip_workspace_bytes(cfg) + MEASURE_STRIPS_EXTRA_BYTES.  Returns the header's ms and stats by name."""
    ms = C.c_float(0.0)
    stats = (C.c_double * 6)()
    st = int(load().fastclip_measure_strips(C.byref(cfg), C.byref(bufs), _ptr(workspace),
                                            workspace.numel() * workspace.element_size(), _stream(stream), int(ablation),
                                            int(reps), C.byref(ms), stats))
    if st != OK:
        raise FastclipError(st)
    return dict(ms=ms.value, cycles_older_wave=stats[0], cycles_younger_wave=stats[1], cycles_between_tiles=stats[2],
                stages_per_workgroup=stats[3], ghz=stats[4], workgroups=int(stats[5]))


def fastclip_measure_record_rmw(idx, n, N, records, record_floats, stream=None, check=True) -> int:
    st = int(load().fastclip_measure_record_rmw(_ptr(idx), int(n), int(N), _ptr(records), int(record_floats), _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_normalize_rows(raw, raw_dtype, ld_raw, b, d, unit, unit_dtype, ld_unit, norm, stream=None, check=True) -> int:
    """raw / unit: device tensors or raw device addresses (an address lets `unit` be a slice of the global batch)."""
    st = int(load().fastclip_normalize_rows(_ptr(raw), int(raw_dtype), int(ld_raw), int(b), int(d), _ptr(unit),
                                            int(unit_dtype), int(ld_unit), _ptr(norm), _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_state_phase_workspace_bytes(b) -> int:
    return int(load().fastclip_state_phase_workspace_bytes(int(b)))


def fastclip_state_phase(cfg, bufs, upd, state, sums, coef, workspace, stream=None, check=True) -> int:
    """sums [4, b], coef [3, b] float32 device tensors; upd / state both None for no temperature update."""
    nbytes = workspace.numel() * workspace.element_size()
    st = int(load().fastclip_state_phase(C.byref(cfg), C.byref(bufs), C.byref(upd) if upd is not None else None,
                                         C.byref(state) if state is not None else None, _ptr(sums), _ptr(coef),
                                         _ptr(workspace), nbytes, _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_step_update_tau(cfg, bufs, upd, state, workspace, workspace_bytes=None, stream=None, check=True) -> int:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    st = int(load().fastclip_step_update_tau(C.byref(cfg), C.byref(bufs), C.byref(upd) if upd is not None else None,
                                             C.byref(state) if state is not None else None, _ptr(workspace), nbytes,
                                             _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_temperature_update(version, upd, state, idx, b, N, d_tau, d_tau_img, d_tau_txt, stream=None,
                                check=True) -> int:
    st = int(load().fastclip_temperature_update(int(version), C.byref(upd) if upd is not None else None,
                                                C.byref(state) if state is not None else None, _ptr(idx), int(b),
                                                int(N), _ptr(d_tau), _ptr(d_tau_img), _ptr(d_tau_txt),
                                                _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_step_timed(cfg, bufs, workspace, workspace_bytes=None, stream=None):
    """Returns {phase name: milliseconds}.  Synchronises."""
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    ms = (C.c_float * N_PHASES)()
    st = int(load().fastclip_step_timed(C.byref(cfg), C.byref(bufs), _ptr(workspace), nbytes, _stream(stream), ms))
    if st != OK:
        raise FastclipError(st)
    return {fastclip_phase_name(i): float(ms[i]) for i in range(N_PHASES) if fastclip_phase_name(i) != "unused"}


def fastclip_phase_name(phase: int) -> str:
    return load().fastclip_phase_name(phase).decode()


def fastclip_state_update(idx, n, N, gamma, M, sum_img, sum_txt, u_img, u_txt, u_new_img, u_new_txt,
                          stream=None, check=True) -> int:
    st = int(load().fastclip_state_update(_ptr(idx), int(n), int(N), float(gamma), float(M), _ptr(sum_img),
                                          _ptr(sum_txt), _ptr(u_img), _ptr(u_txt), _ptr(u_new_img),
                                          _ptr(u_new_txt), _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_state_update_strided(idx, n, N, state_stride, gamma, M, sum_img, sum_txt, u_img, u_txt, u_new_img,
                                  u_new_txt, stream=None, check=True) -> int:
    st = int(load().fastclip_state_update_strided(_ptr(idx), int(n), int(N), int(state_stride), float(gamma), float(M),
                                                  _ptr(sum_img), _ptr(sum_txt), _ptr(u_img), _ptr(u_txt),
                                                  _ptr(u_new_img), _ptr(u_new_txt), _stream(stream)))
    if check and st != OK:
        raise FastclipError(st)
    return st


def fastclip_check_indices_workspace_bytes(b: int) -> int:
    return int(load().fastclip_check_indices_workspace_bytes(int(b)))


def fastclip_check_indices(idx, b, N, workspace, workspace_bytes=None, stream=None) -> int:
    nbytes = workspace.numel() * workspace.element_size() if workspace_bytes is None else workspace_bytes
    return int(load().fastclip_check_indices(_ptr(idx), int(b), int(N), _ptr(workspace), nbytes, _stream(stream)))


def fastclip_gamma_cosine(t, iters_per_epoch, decay_epochs, gamma_min) -> float:
    return float(load().fastclip_gamma_cosine(int(t), int(iters_per_epoch), int(decay_epochs), float(gamma_min)))


def fastclip_last_hip_error() -> str:
    return load().fastclip_last_hip_error().decode()


def fastclip_status_string(status: int) -> str:
    return load().fastclip_status_string(int(status)).decode()
