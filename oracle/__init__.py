"""CPU oracle for the KeyDiff block step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``keydiff_oracle.c`` (plain C, fp64).  Only ``tests/``,
``__graft_entry__.smoke()`` and the benchmark's ``cpu_baseline`` leg may import
this package; the product path never does and has no CPU fallback.

Every function cites the passage of the paper it states; see the C file's header
for the readings taken where the paper is silent.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "keydiff_oracle.c")
_LIB = os.path.join(_HERE, "libkeydiff_oracle.so")

_u16p = C.POINTER(C.c_uint16)
_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)
_f64p = C.POINTER(C.c_double)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over heads x query rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fvisibility=hidden", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.kdo_attention.argtypes = [_u16p, _u16p, _u16p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.c_int, C.c_double, _f32p]
        L.kdo_attention.restype = None
        L.kdo_anchor.argtypes = [_u16p, C.c_int, C.c_int, C.c_int, _f64p]
        L.kdo_anchor.restype = None
        L.kdo_scores.argtypes = [_u16p, C.c_int, C.c_int, _f64p, C.c_double, _f64p, _f32p]
        L.kdo_scores.restype = None
        L.kdo_select.argtypes = [_f32p, _i32p, C.c_int, C.c_int, C.c_int, _i32p]
        L.kdo_select.restype = None
        L.kdo_new.argtypes = [C.c_int] * 7 + [C.c_double, C.c_double]
        L.kdo_new.restype = C.c_void_p
        L.kdo_free.argtypes = [C.c_void_p]
        L.kdo_free.restype = None
        L.kdo_len.argtypes = [C.c_void_p]
        L.kdo_len.restype = C.c_int
        for name, rt in (("kdo_K", _u16p), ("kdo_V", _u16p), ("kdo_pos", _i32p)):
            getattr(L, name).argtypes = [C.c_void_p]
            getattr(L, name).restype = rt
        L.kdo_load.argtypes = [C.c_void_p, _u16p, _u16p, _i32p, C.c_int]
        L.kdo_load.restype = C.c_int
        L.kdo_prefill_block.argtypes = [C.c_void_p, _u16p, _u16p, _u16p, C.c_int, C.c_int64, _f32p, _f32p]
        L.kdo_prefill_block.restype = C.c_int
        L.kdo_scores_of_cache.argtypes = [C.c_void_p, _f32p]
        L.kdo_scores_of_cache.restype = None
        L.kdo_pairwise_rowsum.argtypes = [_u16p, C.c_int, C.c_int, _f64p]
        L.kdo_pairwise_rowsum.restype = None
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(_u16p)


def _ptr(a, t):
    return a.ctypes.data_as(t)


# ----------------------------------------------------------------- free functions
def attention(q, K, V, length: int, Bt: int, scale: float | None = None) -> np.ndarray:
    """Eq. 1-2.  q [hq][Bt][d], K/V [hkv][cap][d] bf16 bits with the block already
    at rows [length, length + Bt).  Returns float32 [hq][Bt][d]."""
    q, qp = _u16(q)
    K, Kp = _u16(K)
    V, Vp = _u16(V)
    hq, _, d = q.shape
    hkv, cap, _ = K.shape
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    out = np.empty((hq, Bt, d), dtype=np.float32)
    lib().kdo_attention(qp, Kp, Vp, hq, hkv, d, cap, length, Bt, float(scale), _ptr(out, _f32p))
    return out


def anchor(Kh, mode: int = 0) -> np.ndarray:
    """Anchor vector of one KV head's rows Kh [n][d] (Method, "Efficient Variant")."""
    Kh, Kp = _u16(Kh)
    n, d = Kh.shape
    mu = np.empty(d, dtype=np.float64)
    lib().kdo_anchor(Kp, n, d, mode, _ptr(mu, _f64p))
    return mu


def scores(Kh, mu=None, mode: int = 0, eps: float = 1e-8):
    """Cosine-to-anchor scores of rows Kh [n][d] (appendix "FLOP count of KeyDiff").
    Returns (float64 scores, float32 scores = the deciding value)."""
    Kh, Kp = _u16(Kh)
    n, d = Kh.shape
    if mu is None:
        mu = anchor(Kh, mode)
    mu = np.ascontiguousarray(mu, dtype=np.float64)
    s64 = np.empty(n, dtype=np.float64)
    s32 = np.empty(n, dtype=np.float32)
    lib().kdo_scores(Kp, n, d, _ptr(mu, _f64p), float(eps), _ptr(s64, _f64p), _ptr(s32, _f32p))
    return s64, s32


def select(s32, pos, keep: int, window_W: int = 0) -> np.ndarray:
    """Rows kept (Eq. 6/7, lowest similarity), ordered by ascending position."""
    s32 = np.ascontiguousarray(s32, dtype=np.float32)
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    n = s32.shape[0]
    kept = np.empty(min(keep, n), dtype=np.int32)
    lib().kdo_select(_ptr(s32, _f32p), _ptr(pos, _i32p), n, keep, window_W, _ptr(kept, _i32p))
    return kept


def pairwise_rowsum(Kh) -> np.ndarray:
    """Row sums of the pairwise cosine-similarity matrix (Eq. 6), O(n^2)."""
    Kh, Kp = _u16(Kh)
    n, d = Kh.shape
    out = np.empty(n, dtype=np.float64)
    lib().kdo_pairwise_rowsum(Kp, n, d, _ptr(out, _f64p))
    return out


# ------------------------------------------------------------------------- state
class OracleCache:
    """Block prompt processing (Eq. 5) over `batch` independent sequences."""

    def __init__(self, batch, n_q_heads, n_kv_heads, head_dim, budget_N, block_B,
                 anchor_mode=0, window_W=0, eps=0.0, softmax_scale=0.0):
        self.batch, self.hq, self.hkv, self.d = batch, n_q_heads, n_kv_heads, head_dim
        self.N, self.B = budget_N, block_B
        self.cap = budget_N + block_B
        self._L = lib()
        self._s = [self._L.kdo_new(n_q_heads, n_kv_heads, head_dim, budget_N, block_B, anchor_mode,
                                   window_W, float(eps), float(softmax_scale)) for _ in range(batch)]

    def __del__(self):
        for s in getattr(self, "_s", []):
            self._L.kdo_free(s)
        self._s = []

    @property
    def len(self) -> int:
        return self._L.kdo_len(self._s[0])

    def prefill_block(self, q, k_new, v_new, pos0: int, want_scores: bool = False):
        """q [batch][hq][Bt][d] or None (skip attention); k_new, v_new [batch][hkv][Bt][d].
        Returns (out float32 [batch][hq][Bt][d] or None, scores or None, evicted per head)."""
        k_new, _ = _u16(k_new)
        v_new, _ = _u16(v_new)
        Bt = k_new.shape[2]
        n = self.len + Bt
        out = None
        if q is not None:
            q, _ = _u16(q)
            out = np.empty((self.batch, self.hq, Bt, self.d), dtype=np.float32)
        sc = np.zeros((self.batch, self.hkv, n), dtype=np.float32) if want_scores else None
        ev = 0
        for b in range(self.batch):
            ev = self._L.kdo_prefill_block(
                self._s[b],
                _ptr(q[b], _u16p) if q is not None else None,
                _ptr(k_new[b], _u16p), _ptr(v_new[b], _u16p), Bt, int(pos0),
                _ptr(out[b], _f32p) if out is not None else None,
                _ptr(sc[b], _f32p) if sc is not None else None)
            if ev < 0:
                raise ValueError("oracle: bad block size")
        return out, sc, ev

    def decode_step(self, q, k_new, v_new, pos: int):
        """B = 1 is the generation phase (Background, block prompt processing)."""
        return self.prefill_block(q, k_new, v_new, pos)

    def load(self, K, V, pos):
        """Teacher forcing: K, V [batch][hkv][len][d] bits, pos [batch][hkv][len]."""
        K, _ = _u16(K)
        V, _ = _u16(V)
        pos = np.ascontiguousarray(pos, dtype=np.int32)
        ln = K.shape[2]
        for b in range(self.batch):
            rc = self._L.kdo_load(self._s[b], _ptr(K[b], _u16p), _ptr(V[b], _u16p), _ptr(pos[b], _i32p), ln)
            if rc:
                raise ValueError("oracle: bad load length")

    def _view(self, getter, shape, dtype):
        outs = []
        for s in self._s:
            p = getter(s)
            outs.append(np.ctypeslib.as_array(p, shape=shape).astype(dtype, copy=True))
        return np.stack(outs)

    def keys(self) -> np.ndarray:
        """[batch][hkv][len][d] bf16 bits, ascending position."""
        return self._view(self._L.kdo_K, (self.hkv, self.cap, self.d), np.uint16)[:, :, :self.len]

    def values(self) -> np.ndarray:
        return self._view(self._L.kdo_V, (self.hkv, self.cap, self.d), np.uint16)[:, :, :self.len]

    def positions(self) -> np.ndarray:
        """[batch][hkv][len] int32, ascending."""
        return self._view(self._L.kdo_pos, (self.hkv, self.cap), np.int32)[:, :, :self.len]

    def scores(self) -> np.ndarray:
        """Scores of the cached rows, no mutation: float32 [batch][hkv][len]."""
        out = np.empty((self.batch, self.hkv, self.len), dtype=np.float32)
        for b in range(self.batch):
            self._L.kdo_scores_of_cache(self._s[b], _ptr(out[b], _f32p))
        return out
