"""ctypes front end of the CPU oracle (oracle/lsh_oracle.cpp).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's cpu_baseline leg may import
this; the product package never does.  Nothing here touches the GPU or the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lsh_oracle.cpp")
_LIB = os.path.join(_HERE, "liblsh_oracle.so")

_c_i32p = ctypes.POINTER(ctypes.c_int32)
_c_f32p = ctypes.POINTER(ctypes.c_float)
_c_f64p = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the oracle with g++ -O2 (no fast-math).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-o", tmp,
                               _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized(out_dir: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (g++ -O1 -g), built
    into out_dir.  A process that loads it needs libasan first in its library list (LD_PRELOAD)
    and names it in the environment variable LSH_ORACLE_LIB; tests/test_oracle_sanitized.py does
    both."""
    out = os.path.join(out_dir, "liblsh_oracle_asan.so")
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
        tmp = out + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-Wall",
                               "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                               "-o", tmp, _SRC])
        os.replace(tmp, out)
    return out


_lib = None


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(os.environ.get("LSH_ORACLE_LIB") or build())
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        lib.orc_wta_codes.argtypes = [vp, i64, i32, i64, i32, _c_i32p, i32, i32, _c_i32p]
        lib.orc_band_codes.argtypes = [_c_i32p, i64, i32, i32, i32, _c_i32p]
        lib.orc_build.argtypes = [vp, i32, i32, i64, i32, _c_i32p, i32, i32, i32]
        lib.orc_build.restype = vp
        lib.orc_free.argtypes = [vp]
        lib.orc_free.restype = None
        lib.orc_num_buckets.argtypes = [vp, i32]
        lib.orc_bucket_keys.argtypes = [vp, i32, _c_i32p, i32]
        lib.orc_bucket.argtypes = [vp, i32, ctypes.c_int32, _c_i32p, i32]
        lib.orc_hidden_band_codes.argtypes = [vp, _c_f32p, i32, _c_i32p]
        lib.orc_hit_counts.argtypes = [vp, _c_f32p, i32, _c_i32p]
        lib.orc_candidates.argtypes = [vp, _c_f32p, i32, _c_i32p, i32, i32, _c_i32p, i32]
        lib.orc_logprobs.argtypes = [vp, _c_f32p, i32, _c_i32p, i32, _c_f64p, _c_f64p]
        lib.orc_topb.argtypes = [_c_f64p, _c_f64p, i32, _c_i32p, i32, i32, _c_i32p, _c_i32p,
                                 _c_f64p]
        lib.orc_decode_step.argtypes = [vp, _c_f32p, _c_f32p, _c_i32p, i32, i32, i32, i32, i32,
                                        _c_i32p, _c_i32p, _c_f64p, _c_i32p]
        _lib = lib
    return _lib


def _i32(a):
    return a.ctypes.data_as(_c_i32p)


def _f32(a):
    return a.ctypes.data_as(_c_f32p)


def _f64(a):
    return a.ctypes.data_as(_c_f64p)


def _matrix(X):
    """Accept fp32 (dtype 0) or uint16 bf16 bit patterns (dtype 1), C-contiguous 2-D."""
    if X.dtype == np.uint16:
        dt = 1
    elif X.dtype == np.float32:
        dt = 0
    else:
        raise TypeError("matrix must be float32 or uint16 (bf16 bits)")
    X = np.ascontiguousarray(X)
    return X, dt


def wta_codes(X, perms) -> np.ndarray:
    """Eq. 4-5: raw winner-take-all codes, int32 [n, P], 0-based."""
    X, dt = _matrix(X)
    perms = np.ascontiguousarray(perms, dtype=np.int32)
    n, d = X.shape
    P, K = perms.shape
    out = np.empty((n, P), dtype=np.int32)
    rc = _L().orc_wta_codes(X.ctypes.data, n, d, d, dt, _i32(perms), P, K, _i32(out))
    if rc:
        raise ValueError("orc_wta_codes: invalid arguments")
    return out


def band_codes(codes, W: int, K: int) -> np.ndarray:
    """Eq. 6-8: pack u = P/W consecutive codes per band, first code most significant."""
    codes = np.ascontiguousarray(codes, dtype=np.int32)
    n, P = codes.shape
    out = np.empty((n, W), dtype=np.int32)
    rc = _L().orc_band_codes(_i32(codes), n, P, W, K, _i32(out))
    if rc:
        raise ValueError("orc_band_codes: invalid arguments")
    return out


class Index:
    """T_w = {band code: [word ids]} for every band, built over the rows of E."""

    def __init__(self, E, perms, W: int):
        self.E, self.dtype = _matrix(E)
        self.perms = np.ascontiguousarray(perms, dtype=np.int32)
        self.V, self.d = self.E.shape
        self.P, self.K = self.perms.shape
        self.W = W
        self._h = _L().orc_build(self.E.ctypes.data, self.V, self.d, self.d, self.dtype,
                                 _i32(self.perms), self.P, self.K, W)
        if not self._h:
            raise ValueError("orc_build: invalid arguments")

    def close(self):
        if self._h:
            _L().orc_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def num_buckets(self, band: int) -> int:
        return _L().orc_num_buckets(self._h, band)

    def bucket_keys(self, band: int) -> np.ndarray:
        n = self.num_buckets(band)
        out = np.empty(n, dtype=np.int32)
        _L().orc_bucket_keys(self._h, band, _i32(out), n)
        return out

    def bucket(self, band: int, code: int):
        """Word ids filed under `code` in table `band` (insertion = ascending id), or None."""
        out = np.empty(self.V, dtype=np.int32)
        n = _L().orc_bucket(self._h, band, int(code), _i32(out), self.V)
        return None if n < 0 else out[:n].copy()

    def _H(self, H):
        H = np.ascontiguousarray(H, dtype=np.float32)
        assert H.ndim == 2 and H.shape[1] == self.d
        return H

    def hidden_band_codes(self, H) -> np.ndarray:
        H = self._H(H)
        out = np.empty((H.shape[0], self.W), dtype=np.int32)
        _L().orc_hidden_band_codes(self._h, _f32(H), H.shape[0], _i32(out))
        return out

    def hit_counts(self, H) -> np.ndarray:
        """Eq. 9 via Algorithm 1: L int32 [B, V]."""
        H = self._H(H)
        L = np.empty((H.shape[0], self.V), dtype=np.int32)
        _L().orc_hit_counts(self._h, _f32(H), H.shape[0], _i32(L))
        return L

    def candidates(self, H, topfreq, t: int = 1) -> np.ndarray:
        """Eq. 10 + Eq. 3 for one sentence (rows of H): ascending int32 word ids."""
        H = self._H(H)
        topfreq = np.ascontiguousarray(topfreq, dtype=np.int32)
        out = np.empty(self.V, dtype=np.int32)
        n = _L().orc_candidates(self._h, _f32(H), H.shape[0], _i32(topfreq), topfreq.size, t,
                                _i32(out), self.V)
        return out[:n].copy()

    def logprobs(self, H, cand=None, want_logits: bool = False):
        """Eq. 2 on the candidate columns + Eq. 1 normalised over them; fp64 [B, C]."""
        H = self._H(H)
        B = H.shape[0]
        if cand is None:
            C, cp = self.V, None
        else:
            cand = np.ascontiguousarray(cand, dtype=np.int32)
            C, cp = cand.size, _i32(cand)
        lp = np.empty((B, C), dtype=np.float64)
        lg = np.empty((B, C), dtype=np.float64) if want_logits else None
        _L().orc_logprobs(self._h, _f32(H), B, cp, C, _f64(lg) if want_logits else None, _f64(lp))
        return (lp, lg) if want_logits else lp

    def decode_step(self, H, beam_scores, topfreq, S: int, B: int, t: int = 1,
                    full_vocab: bool = False):
        """Whole step for S sentences: (beam [S,B], word [S,B], score fp64 [S,B], counts [S])."""
        H = self._H(H)
        assert H.shape[0] == S * B
        bs = np.ascontiguousarray(beam_scores, dtype=np.float32).reshape(-1)
        topfreq = np.ascontiguousarray(topfreq, dtype=np.int32)
        ob = np.empty((S, B), dtype=np.int32)
        ow = np.empty((S, B), dtype=np.int32)
        osc = np.empty((S, B), dtype=np.float64)
        cnt = np.empty(S, dtype=np.int32)
        _L().orc_decode_step(self._h, _f32(H), _f32(bs), _i32(topfreq), topfreq.size, t,
                             1 if full_vocab else 0, S, B, _i32(ob), _i32(ow), _f64(osc), _i32(cnt))
        return ob, ow, osc, cnt


def topb(beam_scores, lp, cand, nsel: int):
    """Heap beam expansion over lp [B, C]; returns (beam, word, score) arrays of length nsel."""
    lp = np.ascontiguousarray(lp, dtype=np.float64)
    B, C = lp.shape
    bs = np.ascontiguousarray(beam_scores, dtype=np.float64)
    cp = None
    if cand is not None:
        cand = np.ascontiguousarray(cand, dtype=np.int32)
        cp = _i32(cand)
    ob = np.empty(nsel, dtype=np.int32)
    ow = np.empty(nsel, dtype=np.int32)
    osc = np.empty(nsel, dtype=np.float64)
    _L().orc_topb(_f64(bs), _f64(lp), B, cp, C, nsel, _i32(ob), _i32(ow), _f64(osc))
    return ob, ow, osc
