"""ctypes binding of include/lshbeam.h.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liblshbeam.so")

LSH_F32, LSH_BF16 = 0, 1
NUM_KERNELS = 5

# every symbol include/lshbeam.h declares
EXPORTED_SYMBOLS = (
    "lsh_build_tables", "lsh_free_tables", "lsh_step_workspace_bytes", "lsh_decode_step",
    "lsh_debug_codes", "lsh_debug_embedding_codes", "lsh_debug_bucket", "lsh_debug_csr",
    "lsh_debug_cuckoo_shape", "lsh_debug_candidates", "lsh_debug_logprobs", "lsh_profiler_create",
    "lsh_profiler_destroy", "lsh_profiler_read", "lsh_decode_step_timed", "lsh_kernel_name",
    "lsh_status_string", "lsh_step_is_fused", "lsh_debug_build_info", "lsh_beam_advance",
    "lsh_beam_backtrace", "lsh_set_option", "lsh_get_option", "lsh_decode_step_static",
    "lsh_static_scratch_bytes", "lsh_debug_counts",
)

OPTION_AUTO = -1
OPTION_NAMES = ("fused", "fused_grid", "logits_grid", "logits_waves", "logits_hlds", "logits_estage",
                "hlds_rem", "logits_planes", "hlds_rows", "part_rows", "stage_rows", "one_launch", "fused_tile",
                "estage_union")


class LshBeamError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {_status_string(status)} (status {status})")


class BuildParams(ctypes.Structure):
    _fields_ = [("V", ctypes.c_int32), ("d", ctypes.c_int32), ("ld_e", ctypes.c_int64),
                ("e_dtype", ctypes.c_int32), ("K", ctypes.c_int32), ("P", ctypes.c_int32),
                ("bands", ctypes.c_int32), ("seed", ctypes.c_uint64)]


class BeamParams(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("B", ctypes.c_int32), ("n_states", ctypes.c_int32),
                ("state_dim", ctypes.c_int32), ("eos", ctypes.c_int32), ("max_len", ctypes.c_int32)]


class StepParams(ctypes.Structure):
    _fields_ = [("S", ctypes.c_int32), ("B", ctypes.c_int32), ("T", ctypes.c_int32),
                ("threshold", ctypes.c_int32), ("full_vocab", ctypes.c_int32)]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load liblshbeam.so (built in-tree by `python -m paper_1806_00588_amd.build`).  Raises if
    it is missing: there is no fallback implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} not found: build it with `python -m paper_1806_00588_amd.build`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.lsh_build_tables.argtypes = [vp, vp, ctypes.POINTER(BuildParams), vp, ctypes.POINTER(vp)]
    lib.lsh_free_tables.argtypes = [vp]
    lib.lsh_free_tables.restype = None
    lib.lsh_step_workspace_bytes.argtypes = [vp, ctypes.POINTER(StepParams)]
    lib.lsh_step_workspace_bytes.restype = sz
    lib.lsh_decode_step.argtypes = [vp, vp, vp, vp, ctypes.POINTER(StepParams), vp, sz, vp, vp, vp, vp]
    lib.lsh_debug_codes.argtypes = [vp, vp, i32, i32p]
    lib.lsh_debug_embedding_codes.argtypes = [vp, i32, i32, i32p]
    lib.lsh_debug_bucket.argtypes = [vp, i32, i32, i32p, i32, i32p]
    lib.lsh_debug_csr.argtypes = [vp, i32, i32p, i32p, i32p, i32, i32p]
    lib.lsh_debug_cuckoo_shape.argtypes = [vp, i32, i32p, i32p]
    lib.lsh_debug_build_info.argtypes = [vp, i32p, i32p]
    lib.lsh_beam_advance.argtypes = [ctypes.POINTER(BeamParams), i32, vp, vp, vp, ctypes.POINTER(vp),
                                     ctypes.POINTER(vp), vp, vp, vp, vp, vp]
    lib.lsh_beam_advance.restype = i32
    lib.lsh_beam_backtrace.argtypes = [ctypes.POINTER(BeamParams), i32, vp, vp, vp, vp, vp, vp, vp]
    lib.lsh_beam_backtrace.restype = i32
    lib.lsh_debug_build_info.restype = i32
    lib.lsh_debug_candidates.argtypes = [vp, vp, ctypes.POINTER(StepParams), i32, i32p, i32, i32p]
    lib.lsh_debug_counts.argtypes = [vp, vp, ctypes.POINTER(StepParams), i32p]
    lib.lsh_debug_logprobs.argtypes = [vp, vp, ctypes.POINTER(StepParams), i32,
                                       ctypes.POINTER(ctypes.c_float), i32, i32p]
    lib.lsh_decode_step_timed.argtypes = lib.lsh_decode_step.argtypes + [vp]
    lib.lsh_decode_step_static.argtypes = [vp, vp, vp, vp, ctypes.POINTER(StepParams), vp, vp, vp, vp]
    lib.lsh_static_scratch_bytes.argtypes = []
    lib.lsh_static_scratch_bytes.restype = sz
    lib.lsh_profiler_create.argtypes = [i32, ctypes.POINTER(vp)]
    lib.lsh_profiler_destroy.argtypes = [vp]
    lib.lsh_profiler_destroy.restype = None
    lib.lsh_profiler_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), i32p]
    lib.lsh_set_option.argtypes = [vp, ctypes.c_char_p, i32]
    lib.lsh_get_option.argtypes = [vp, ctypes.c_char_p, i32p]
    lib.lsh_step_is_fused.argtypes = [vp, ctypes.POINTER(StepParams)]
    lib.lsh_kernel_name.argtypes = [i32]
    lib.lsh_kernel_name.restype = ctypes.c_char_p
    lib.lsh_status_string.argtypes = [ctypes.c_int]
    lib.lsh_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _status_string(status: int) -> str:
    try:
        return load_library().lsh_status_string(status).decode()
    except Exception:
        return "?"


def _check(status: int, what: str):
    if status != 0:
        raise LshBeamError(status, what)


def kernel_names():
    lib = load_library()
    return [lib.lsh_kernel_name(i).decode() for i in range(NUM_KERNELS)]


def _i32p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _stream_ptr(stream) -> int:
    import torch
    if isinstance(stream, int):  # a raw hipStream_t
        return stream
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _require_cuda(x, name, dtypes):
    if not x.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if x.dtype not in dtypes:
        raise ValueError(f"{name}: dtype {x.dtype} not in {dtypes}")
    if not x.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


class Tables:
    """Owns an lsh_tables handle and keeps the borrowed embedding tensor alive."""

    def __init__(self, handle: int, E, K: int, P: int, W: int, e_dtype: int):
        self._h = handle
        self.E = E
        self.V, self.d = int(E.shape[0]), int(E.shape[1])
        self.K, self.P, self.W, self.e_dtype = K, P, W, e_dtype
        self._prof = None          # lsh_profiler* while profile_begin .. profile_end is open

    @property
    def handle(self) -> int:
        if not self._h:
            raise ValueError("tables already freed")
        return self._h

    def close(self):
        if self._prof:
            load_library().lsh_profiler_destroy(self._prof)
            self._prof = None
        if self._h:
            load_library().lsh_free_tables(self._h)
            self._h = None

    # ---- launch-plan options ------------------------------------------------------------------
    def set_option(self, name: str, value: int = OPTION_AUTO):
        """lsh_set_option: force a launch-plan rule (value >= 0) or restore it (OPTION_AUTO)."""
        _check(load_library().lsh_set_option(self.handle, name.encode(), int(value)),
               f"lsh_set_option({name})")

    def get_option(self, name: str) -> int:
        v = ctypes.c_int32(0)
        _check(load_library().lsh_get_option(self.handle, name.encode(), ctypes.byref(v)),
               f"lsh_get_option({name})")
        return v.value

    def set_options(self, **kw):
        for k, v in kw.items():
            self.set_option(k, v)

    def reset_options(self):
        for k in OPTION_NAMES:
            self.set_option(k, OPTION_AUTO)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- inspection -------------------------------------------------------------------------
    def debug_codes(self, H) -> np.ndarray:
        import torch
        _require_cuda(H, "H", (torch.float32,))
        R = int(H.shape[0])
        out = np.empty((R, self.W), dtype=np.int32)
        _check(load_library().lsh_debug_codes(self.handle, H.data_ptr(), R, _i32p(out)),
               "lsh_debug_codes")
        return out

    def debug_embedding_codes(self, row0: int = 0, n: Optional[int] = None) -> np.ndarray:
        n = self.V - row0 if n is None else n
        out = np.empty((n, self.W), dtype=np.int32)
        _check(load_library().lsh_debug_embedding_codes(self.handle, row0, n, _i32p(out)),
               "lsh_debug_embedding_codes")
        return out

    def debug_bucket(self, band: int, code: int):
        out = np.empty(self.V, dtype=np.int32)
        n = ctypes.c_int32(0)
        _check(load_library().lsh_debug_bucket(self.handle, band, int(code), _i32p(out), self.V,
                                               ctypes.byref(n)), "lsh_debug_bucket")
        return None if n.value < 0 else out[: n.value].copy()

    def debug_csr(self, band: int):
        nk = ctypes.c_int32(0)
        lib = load_library()
        _check(lib.lsh_debug_csr(self.handle, band, ctypes.byref(nk), None, None, 0, None),
               "lsh_debug_csr")
        keys = np.empty(nk.value, dtype=np.int32)
        offs = np.empty(nk.value + 1, dtype=np.int32)
        words = np.empty(self.V, dtype=np.int32)
        _check(lib.lsh_debug_csr(self.handle, band, ctypes.byref(nk), _i32p(keys), _i32p(offs),
                                 nk.value, _i32p(words)), "lsh_debug_csr")
        return keys, offs, words

    def debug_build_info(self):
        """(built on the device?, insertion rounds the device made)"""
        dev, att = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(load_library().lsh_debug_build_info(self.handle, ctypes.byref(dev), ctypes.byref(att)),
               "lsh_debug_build_info")
        return bool(dev.value), att.value

    def debug_cuckoo_shape(self, band: int):
        cap, nk = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(load_library().lsh_debug_cuckoo_shape(self.handle, band, ctypes.byref(cap),
                                                     ctypes.byref(nk)), "lsh_debug_cuckoo_shape")
        return cap.value, nk.value

    def debug_candidates(self, workspace, sp: StepParams, s: int) -> np.ndarray:
        out = np.empty(self.V, dtype=np.int32)
        n = ctypes.c_int32(0)
        _check(load_library().lsh_debug_candidates(self.handle, workspace.data_ptr(),
                                                   ctypes.byref(sp), s, _i32p(out), self.V,
                                                   ctypes.byref(n)), "lsh_debug_candidates")
        return out[: n.value].copy()

    def debug_counts(self, workspace, sp: StepParams) -> np.ndarray:
        """Candidate counts of all sentences of the last step on this workspace."""
        out = np.empty(sp.S, dtype=np.int32)
        _check(load_library().lsh_debug_counts(self.handle, workspace.data_ptr(), ctypes.byref(sp),
                                               _i32p(out)), "lsh_debug_counts")
        return out

    def debug_logprobs(self, workspace, sp: StepParams, s: int, cap: Optional[int] = None):
        cap = self.V if cap is None else cap
        out = np.empty((sp.B, cap), dtype=np.float32)
        n = ctypes.c_int32(0)
        _check(load_library().lsh_debug_logprobs(
            self.handle, workspace.data_ptr(), ctypes.byref(sp), s,
            out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), cap, ctypes.byref(n)),
            "lsh_debug_logprobs")
        return out[:, : min(n.value, cap)].copy()

    # ---- per-kernel timing ------------------------------------------------------------------
    def profile_begin(self, max_steps: int):
        """Steps made through this object (decode_step, make_step_caller) from now on are timed
        per kernel (lsh_decode_step_timed with a profiler this object owns), up to max_steps."""
        lib = load_library()
        if self._prof:
            lib.lsh_profiler_destroy(self._prof)
            self._prof = None
        out = ctypes.c_void_p(0)
        _check(lib.lsh_profiler_create(max_steps, ctypes.byref(out)), "lsh_profiler_create")
        self._prof = out.value

    def profile_end(self):
        """{kernel name: (mean ms per launch, launches)}; ends the timing."""
        lib = load_library()
        if not self._prof:
            raise ValueError("profile_end without profile_begin")
        ms = (ctypes.c_double * NUM_KERNELS)()
        n = (ctypes.c_int32 * NUM_KERNELS)()
        rc = lib.lsh_profiler_read(self._prof, ms, n)
        lib.lsh_profiler_destroy(self._prof)
        self._prof = None
        _check(rc, "lsh_profiler_read")
        return {name: (ms[i], n[i]) for i, name in enumerate(kernel_names())}


def build_tables(E, perms, K: int, bands: int, seed: int = 0, stream=None) -> Tables:
    """lsh_build_tables.  E: device tensor [V, d], float32, or bfloat16 / int16 / uint16 holding
    bf16 bit patterns; perms: device int32 [P, K]."""
    import torch
    lib = load_library()
    if E.dtype == torch.float32:
        dt = LSH_F32
    elif E.dtype in (torch.bfloat16, torch.int16, torch.uint16):
        dt = LSH_BF16
    else:
        raise ValueError(f"E: unsupported dtype {E.dtype}")
    _require_cuda(perms, "perms", (torch.int32,))
    if E.dim() != 2 or perms.dim() != 2 or int(perms.shape[1]) != K:
        raise ValueError("E must be [V, d] and perms [P, K]")
    # rows may be pitched (a [:, a:b] view of a wider matrix): unit stride inside a row only
    if not E.is_cuda or int(E.stride(1)) != 1 or int(E.stride(0)) < int(E.shape[1]):
        raise ValueError("E must be a device tensor with contiguous rows (row pitch >= d)")
    bp = BuildParams(int(E.shape[0]), int(E.shape[1]), int(E.stride(0)), dt, K,
                     int(perms.shape[0]), bands, seed)
    out = ctypes.c_void_p(0)
    _check(lib.lsh_build_tables(E.data_ptr(), perms.data_ptr(), ctypes.byref(bp),
                                _stream_ptr(stream), ctypes.byref(out)), "lsh_build_tables")
    return Tables(out.value, E, K, int(perms.shape[0]), bands, dt)


def step_params(S: int, B: int, T: int, threshold: int = 1, full_vocab: bool = False) -> StepParams:
    return StepParams(S, B, T, threshold, 1 if full_vocab else 0)


def step_is_fused(tables: Tables, sp: StepParams) -> bool:
    return bool(load_library().lsh_step_is_fused(tables.handle, ctypes.byref(sp)))


def step_workspace_bytes(tables: Tables, sp: StepParams) -> int:
    return int(load_library().lsh_step_workspace_bytes(tables.handle, ctypes.byref(sp)))


def decode_step(tables: Tables, H, beam_scores, topfreq, sp: StepParams, workspace, out_beam,
                out_word, out_score, stream=None):
    """lsh_decode_step: asynchronous on `stream` (default: torch's current stream)."""
    import torch
    _require_cuda(H, "H", (torch.float32,))
    _require_cuda(beam_scores, "beam_scores", (torch.float32,))
    _require_cuda(out_beam, "out_beam", (torch.int32,))
    _require_cuda(out_word, "out_word", (torch.int32,))
    _require_cuda(out_score, "out_score", (torch.float32,))
    R = sp.S * sp.B
    if H.numel() != R * tables.d or beam_scores.numel() != R:
        raise ValueError("H must be [S*B, d] and beam_scores [S*B]")
    if min(out_beam.numel(), out_word.numel(), out_score.numel()) < R:
        raise ValueError("outputs must hold S*B elements")
    tf_ptr = 0
    if topfreq is not None:
        _require_cuda(topfreq, "topfreq", (torch.int32,))
        if topfreq.numel() < sp.T:
            raise ValueError("topfreq shorter than T")
        tf_ptr = topfreq.data_ptr()
    args = (tables.handle, H.data_ptr(), beam_scores.data_ptr(), tf_ptr, ctypes.byref(sp),
            workspace.data_ptr(), workspace.numel() * workspace.element_size(), out_beam.data_ptr(),
            out_word.data_ptr(), out_score.data_ptr(), _stream_ptr(stream))
    if tables._prof:
        _check(load_library().lsh_decode_step_timed(*args, tables._prof), "lsh_decode_step_timed")
    else:
        _check(load_library().lsh_decode_step(*args), "lsh_decode_step")


def static_scratch_bytes() -> int:
    return int(load_library().lsh_static_scratch_bytes())


def decode_step_static(tables: Tables, H, beam_scores, topfreq, sp: StepParams, out_beam, out_word,
                       out_score, stream=None):
    """lsh_decode_step_static: the step in the library's built-in scratch buffer (no workspace)."""
    import torch
    for x, name, dt in ((H, "H", torch.float32), (beam_scores, "beam_scores", torch.float32),
                        (out_beam, "out_beam", torch.int32), (out_word, "out_word", torch.int32),
                        (out_score, "out_score", torch.float32)):
        _require_cuda(x, name, (dt,))
    R = sp.S * sp.B
    if H.numel() != R * tables.d or beam_scores.numel() != R:
        raise ValueError("H must be [S*B, d] and beam_scores [S*B]")
    if min(out_beam.numel(), out_word.numel(), out_score.numel()) < R:
        raise ValueError("outputs must hold S*B elements")
    tf_ptr = 0
    if topfreq is not None:
        _require_cuda(topfreq, "topfreq", (torch.int32,))
        if topfreq.numel() < sp.T:
            raise ValueError("topfreq shorter than T")
        tf_ptr = topfreq.data_ptr()
    _check(load_library().lsh_decode_step_static(
        tables.handle, H.data_ptr(), beam_scores.data_ptr(), tf_ptr, ctypes.byref(sp),
        out_beam.data_ptr(), out_word.data_ptr(), out_score.data_ptr(), _stream_ptr(stream)),
        "lsh_decode_step_static")


def make_step_caller(tables: Tables, sp: StepParams, workspace, topfreq):
    """Pre-marshalled lsh_decode_step for tight loops: returns
    f(H_ptr, beam_scores_ptr, out_beam_ptr, out_word_ptr, out_score_ptr, stream_ptr) -> None,
    all arguments raw device addresses (ints).  Same entry point, same kernels; only the Python
    argument checking is hoisted out of the loop."""
    lib = load_library()
    fn, fn_timed = lib.lsh_decode_step, lib.lsh_decode_step_timed
    h = ctypes.c_void_p(tables.handle)
    spp = ctypes.pointer(sp)
    ws = ctypes.c_void_p(workspace.data_ptr())
    wsn = ctypes.c_size_t(workspace.numel() * workspace.element_size())
    tf = ctypes.c_void_p(topfreq.data_ptr() if topfreq is not None else 0)
    keep = (tables, sp, workspace, topfreq)

    def call(H_ptr, bs_ptr, ob_ptr, ow_ptr, osc_ptr, stream_ptr, _keep=keep):
        if tables._prof:
            rc = fn_timed(h, H_ptr, bs_ptr, tf, spp, ws, wsn, ob_ptr, ow_ptr, osc_ptr, stream_ptr,
                          tables._prof)
        else:
            rc = fn(h, H_ptr, bs_ptr, tf, spp, ws, wsn, ob_ptr, ow_ptr, osc_ptr, stream_ptr)
        if rc:
            raise LshBeamError(rc, "lsh_decode_step")

    return call


class BeamHistory:
    """Caller-owned device arrays of the beam bookkeeping calls (torch is only the allocator)."""

    def __init__(self, S: int, B: int, max_len: int, n_states: int = 0, state_dim: int = 0, eos: int = -1):
        import torch
        self.bp = BeamParams(S, B, n_states, state_dim, eos, max_len)
        self.backptr = torch.empty((max_len, S, B), dtype=torch.int32, device="cuda")
        self.words = torch.empty((max_len, S, B), dtype=torch.int32, device="cuda")
        self.scores = torch.empty((max_len, S, B), dtype=torch.float32, device="cuda")


def beam_advance(hist: BeamHistory, step: int, out_beam, out_word, out_score, states_in, states_out,
                 next_scores, stream=None) -> None:
    """lsh_beam_advance; states_in / states_out are sequences of device tensors [S*B, state_dim]."""
    n = hist.bp.n_states
    assert len(states_in) == n and len(states_out) == n
    pin = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in states_in])
    pout = (ctypes.c_void_p * max(n, 1))(*[t.data_ptr() for t in states_out])
    _check(load_library().lsh_beam_advance(ctypes.byref(hist.bp), step, out_beam.data_ptr(),
                                           out_word.data_ptr(), out_score.data_ptr(), pin, pout,
                                           hist.backptr.data_ptr(), hist.words.data_ptr(),
                                           hist.scores.data_ptr(), next_scores.data_ptr(),
                                           _stream_ptr(stream)), "lsh_beam_advance")


def beam_backtrace(hist: BeamHistory, n_steps: int, stream=None):
    """lsh_beam_backtrace -> (tokens [S, max_len] int32, length [S] int32, score [S] fp32), device."""
    import torch
    S, L = hist.bp.S, hist.bp.max_len
    tokens = torch.full((S, L), -1, dtype=torch.int32, device="cuda")
    length = torch.empty(S, dtype=torch.int32, device="cuda")
    score = torch.empty(S, dtype=torch.float32, device="cuda")
    _check(load_library().lsh_beam_backtrace(ctypes.byref(hist.bp), n_steps, hist.backptr.data_ptr(),
                                             hist.words.data_ptr(), hist.scores.data_ptr(),
                                             tokens.data_ptr(), length.data_ptr(), score.data_ptr(),
                                             _stream_ptr(stream)), "lsh_beam_backtrace")
    return tokens, length, score
