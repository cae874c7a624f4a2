"""ctypes binding of include/keydiff.h -- argument marshalling only.

Every step of the path runs in the library's HIP kernels.  PyTorch appears only
as the owner of device memory and streams.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkeydiff.so")

OK, EINVAL, ESHAPE, ESTATE, EHIP = 0, -1, -2, -3, -4
ANCHOR_MEAN_KEY, ANCHOR_MEAN_UNIT_KEY = 0, 1
LAYOUT_ORDERED, LAYOUT_FILL = 0, 1
KERNEL_NAMES = ("step_main", "step_score", "step_post", "compact_ordered", "aux", "event_pair", "select_alone")

EXPORTS = (
    "keydiff_workspace_bytes", "keydiff_init_cache", "keydiff_prefill_block", "keydiff_prefill_block_static",
    "keydiff_prefill_block_deferred",
    "keydiff_prefill_block_layers", "keydiff_prefill_block_rope", "keydiff_prefill_block_layers_rope", "keydiff_finish", "keydiff_decode_step",
    "keydiff_scores", "keydiff_cache_len", "keydiff_cache_plan", "keydiff_cache_positions", "keydiff_cache_load",
    "keydiff_cache_status", "keydiff_profile_enable", "keydiff_profile_read", "keydiff_destroy_cache",
    "keydiff_last_error", "keydiff_version",
)


class KeyDiffError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"keydiff error {code}: {message}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "n_q_heads", "n_kv_heads", "head_dim", "budget_N", "block_B",
                                         "anchor_mode", "window_W", "layout")] + \
               [("eps", C.c_float), ("softmax_scale", C.c_float)]


@dataclass
class KeyDiffConfig:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    budget_N: int
    block_B: int
    anchor_mode: int = ANCHOR_MEAN_KEY
    window_W: int = 0
    layout: int = LAYOUT_ORDERED
    eps: float = 0.0
    softmax_scale: float = 0.0

    def _c(self) -> _Config:
        return _Config(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.budget_N, self.block_B,
                       self.anchor_mode, self.window_W, self.layout, self.eps, self.softmax_scale)


_lib = None


def load_library() -> C.CDLL:
    """Load libkeydiff.so; there is no fallback if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("KEYDIFF_LIBRARY", LIB_PATH)   # override: another build of the same ABI
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: build it with `python -m paper_2504_15364_amd.build`")
    L = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    szp = C.POINTER(C.c_size_t)
    L.keydiff_workspace_bytes.argtypes = [C.POINTER(_Config), szp, szp, szp, szp]
    L.keydiff_init_cache.argtypes = [C.POINTER(_Config), vp, vp, vp, vp, vp, C.POINTER(vp)]
    L.keydiff_prefill_block.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp]
    L.keydiff_prefill_block_static.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp]
    L.keydiff_prefill_block_deferred.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, vp]
    pp = C.POINTER(vp)
    L.keydiff_prefill_block_layers.argtypes = [pp, i32, pp, pp, pp, i32, i64, pp, vp]
    L.keydiff_prefill_block_rope.argtypes = [vp, vp, vp, vp, i32, i64, vp, vp, i64, vp, vp, vp]
    L.keydiff_prefill_block_layers_rope.argtypes = [pp, i32, pp, pp, pp, i32, i64, vp, vp, i64, pp, vp]
    L.keydiff_finish.argtypes = [vp, vp]
    L.keydiff_decode_step.argtypes = [vp, vp, vp, vp, i64, vp, vp]
    L.keydiff_scores.argtypes = [vp, vp, vp]
    L.keydiff_cache_len.argtypes = [vp, C.POINTER(i32)]
    L.keydiff_cache_plan.argtypes = [vp, C.POINTER(i32)]
    L.keydiff_cache_positions.argtypes = [vp, vp, vp]
    L.keydiff_cache_load.argtypes = [vp, vp, vp, vp, i32, vp]
    L.keydiff_cache_status.argtypes = [vp, C.POINTER(i32), vp]
    L.keydiff_profile_enable.argtypes = [vp, i32]
    L.keydiff_profile_read.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(i32)]
    L.keydiff_destroy_cache.argtypes = [vp]
    L.keydiff_destroy_cache.restype = None
    L.keydiff_last_error.argtypes = []
    L.keydiff_last_error.restype = C.c_char_p
    L.keydiff_version.argtypes = []
    for name in EXPORTS:
        if name not in ("keydiff_destroy_cache", "keydiff_last_error"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(rc: int):
    if rc != OK:
        raise KeyDiffError(rc, load_library().keydiff_last_error().decode())


def workspace_bytes(cfg: KeyDiffConfig):
    k, v, m, s = (C.c_size_t() for _ in range(4))
    c = cfg._c()
    _check(load_library().keydiff_workspace_bytes(C.byref(c), C.byref(k), C.byref(v), C.byref(m), C.byref(s)))
    return k.value, v.value, m.value, s.value


def _stream_ptr(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return getattr(stream, "cuda_stream", stream)


def check_block_shapes(cfg, q, k_new, v_new, out=None, Bt=None):
    """The tensors of one block against the cache's configuration: q (and out) [batch][Hq][Bt][d],
    k_new / v_new [batch][Hkv][Bt][d].  The C ABI takes bare pointers and cannot know how much memory
    lies behind them: a tensor smaller than the configuration says would be read past its end by the
    kernels, so the wrapper refuses it here, before anything is enqueued.  Returns Bt."""
    if Bt is None:
        Bt = int(k_new.shape[-2])
    want_q = (cfg.batch, cfg.n_q_heads, Bt, cfg.head_dim)
    want_kv = (cfg.batch, cfg.n_kv_heads, Bt, cfg.head_dim)
    for name, t, want in (("q", q, want_q), ("k_new", k_new, want_kv), ("v_new", v_new, want_kv), ("out", out, want_q)):
        if t is None:
            continue
        if tuple(t.shape) != want:
            raise ValueError(f"{name} has shape {tuple(t.shape)}, the cache's configuration needs {want}")
    return Bt


def check_load_shapes(cfg, cap, k, v, pos):
    """Tensors handed to keydiff_cache_load: k, v [batch][Hkv][len][d] bf16, pos [batch][Hkv][len] int32."""
    import torch
    if k.dim() != 4:
        raise ValueError(f"k has shape {tuple(k.shape)}, expected [batch][Hkv][len][d]")
    ln = int(k.shape[2])
    want = (cfg.batch, cfg.n_kv_heads, ln, cfg.head_dim)
    if ln > cap:
        raise ValueError(f"{ln} rows do not fit a cache of {cap} rows per head")
    for name, t in (("k", k), ("v", v)):
        if tuple(t.shape) != want or t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous bf16 tensor of shape {want}, got {tuple(t.shape)} {t.dtype}")
    if tuple(pos.shape) != want[:3] or pos.dtype != torch.int32 or not pos.is_contiguous():
        raise ValueError(f"pos must be a contiguous int32 tensor of shape {want[:3]}, got {tuple(pos.shape)} {pos.dtype}")
    return ln


def check_rope_tables(cfg, cos, sin):
    import torch
    for name, t in (("cos", cos), ("sin", sin)):
        if t.dtype != torch.float32 or not t.is_contiguous() or t.dim() != 2 or t.shape[1] != cfg.head_dim // 2:
            raise ValueError(f"{name} must be a contiguous float32 table [positions][{cfg.head_dim // 2}], got {tuple(t.shape)} {t.dtype}")
    if cos.shape != sin.shape:
        raise ValueError("cos and sin tables differ in shape")


def prefill_block_layers(caches, q, k_new, v_new, pos0: int, out=None, stream=None, rope=None):
    """One block through the layers of a model: `caches`, `q`, `k_new`, `v_new` (and `out`) are
    sequences with one entry per layer; every layer's eviction rides in the next layer's launch.
    rope = (cos, sin): float32 device tables [positions][head_dim / 2]; q and k_new are then rotated
    inside the call (keydiff_prefill_block_layers_rope)."""
    import torch
    n = len(caches)
    assert n >= 1 and len(q) == len(k_new) == len(v_new) == n
    Bt = k_new[0].shape[-2]
    for c, tq, tk, tv in zip(caches, q, k_new, v_new):
        for t in (tq, tk, tv):
            assert t.is_contiguous() and t.dtype == torch.bfloat16 and t.device == c.device
        check_block_shapes(c.cfg, tq, tk, tv, Bt=Bt)
    if out is None:
        out = [torch.empty_like(t) for t in q]
    assert len(out) == n
    for c, to in zip(caches, out):
        assert to.is_contiguous() and to.dtype == torch.bfloat16 and to.device == c.device
        check_block_shapes(c.cfg, None, None, None, out=to, Bt=Bt)
    arr = lambda ptrs: (C.c_void_p * n)(*ptrs)
    L = caches[0]._L
    if rope is not None:
        cos, sin = rope
        check_rope_tables(caches[0].cfg, cos, sin)
        _check(L.keydiff_prefill_block_layers_rope(arr([c._h.value for c in caches]), n,
                                                   arr([t.data_ptr() for t in q]), arr([t.data_ptr() for t in k_new]),
                                                   arr([t.data_ptr() for t in v_new]), Bt, int(pos0), cos.data_ptr(),
                                                   sin.data_ptr(), cos.shape[0], arr([t.data_ptr() for t in out]),
                                                   _stream_ptr(stream)))
        return out
    _check(L.keydiff_prefill_block_layers(arr([c._h.value for c in caches]), n,
                                          arr([t.data_ptr() for t in q]), arr([t.data_ptr() for t in k_new]),
                                          arr([t.data_ptr() for t in v_new]), Bt, int(pos0),
                                          arr([t.data_ptr() for t in out]), _stream_ptr(stream)))
    return out


class KeyDiffCache:
    """keydiff_cache_t over torch-owned device buffers.  Method names follow the C ABI."""

    def __init__(self, cfg: KeyDiffConfig, device="cuda:0", stream=None):
        import torch
        self._L = load_library()
        self.cfg = cfg
        self.device = torch.device(device)
        kb, vb, mb, sb = workspace_bytes(cfg)
        # the library never allocates device memory: torch owns these four buffers
        self._k = torch.empty(kb, dtype=torch.uint8, device=self.device)
        self._v = torch.empty(vb, dtype=torch.uint8, device=self.device)
        self._meta = torch.empty(mb, dtype=torch.uint8, device=self.device)
        self._scratch = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        c = cfg._c()
        with torch.cuda.device(self.device):
            _check(self._L.keydiff_init_cache(C.byref(c), self._k.data_ptr(), self._v.data_ptr(),
                                              self._meta.data_ptr(), self._scratch.data_ptr(),
                                              _stream_ptr(stream), C.byref(self._h)))
        self.cap = (cfg.budget_N + cfg.block_B + 3) & ~3   # rows per head of the cache buffers (see keydiff.h)

    def close(self):
        if getattr(self, "_h", None):
            self._L.keydiff_destroy_cache(self._h)
            self._h = None

    __del__ = close

    def _block_args(self, q, k_new, v_new, out, scores_out, allocate=True):
        """Checks the tensors of one block (dtype, device, layout, shape) and returns (Bt, out)."""
        import torch
        for t in (q, k_new, v_new) + ((out,) if out is not None else ()):
            if not (t.is_contiguous() and t.dtype == torch.bfloat16 and t.device == self.device):
                raise ValueError("block tensors must be contiguous bf16 tensors on the cache's device")
        Bt = check_block_shapes(self.cfg, q, k_new, v_new, out)
        if out is None:
            if not allocate:
                raise ValueError("this call needs the caller's `out`")
            out = torch.empty_like(q)
        if scores_out is not None:
            need = self.cfg.batch * self.cfg.n_kv_heads * (self.len + Bt)
            if not (scores_out.is_contiguous() and scores_out.dtype == torch.float32 and scores_out.device == self.device
                    and scores_out.numel() >= need):
                raise ValueError(f"scores_out must be a contiguous float32 device tensor of at least {need} elements")
        return Bt, out

    # -- the calls of the C ABI ------------------------------------------------
    def prefill_block(self, q, k_new, v_new, pos0: int, out=None, scores_out=None, stream=None):
        """q [batch][Hq][Bt][d], k_new/v_new [batch][Hkv][Bt][d] bf16 device tensors."""
        Bt, out = self._block_args(q, k_new, v_new, out, scores_out)
        _check(self._L.keydiff_prefill_block(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), Bt,
                                             int(pos0), out.data_ptr(),
                                             scores_out.data_ptr() if scores_out is not None else None,
                                             _stream_ptr(stream)))
        return out

    def prefill_block_rope(self, q, k_new, v_new, pos0: int, cos, sin, out=None, scores_out=None, stream=None):
        """prefill_block on a block whose q and k_new are not rotated yet: cos, sin float32 device
        tables [positions][head_dim / 2]."""
        Bt, out = self._block_args(q, k_new, v_new, out, scores_out)
        check_rope_tables(self.cfg, cos, sin)
        _check(self._L.keydiff_prefill_block_rope(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), Bt,
                                                  int(pos0), cos.data_ptr(), sin.data_ptr(), cos.shape[0], out.data_ptr(),
                                                  scores_out.data_ptr() if scores_out is not None else None,
                                                  _stream_ptr(stream)))
        return out

    def prefill_block_static(self, q, k_new, v_new, pos0: int, out, scores_out=None, stream=None):
        """prefill_block with the step's temporaries in the library's static device array; `out` is
        the caller's (this wrapper allocates nothing either)."""
        Bt, out = self._block_args(q, k_new, v_new, out, scores_out, allocate=False)
        _check(self._L.keydiff_prefill_block_static(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), Bt,
                                                    int(pos0), out.data_ptr(),
                                                    scores_out.data_ptr() if scores_out is not None else None,
                                                    _stream_ptr(stream)))
        return out

    def prefill_block_deferred(self, q, k_new, v_new, pos0: int, out=None, carry=None, stream=None):
        """The block step with its eviction left pending; `carry` is another KeyDiffCache whose
        pending eviction this call takes along."""
        Bt, out = self._block_args(q, k_new, v_new, out, None)
        _check(self._L.keydiff_prefill_block_deferred(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), Bt,
                                                      int(pos0), out.data_ptr(),
                                                      carry._h if carry is not None else None, _stream_ptr(stream)))
        return out

    def finish(self, stream=None):
        _check(self._L.keydiff_finish(self._h, _stream_ptr(stream)))

    def decode_step(self, q, k_new, v_new, pos: int, out=None, stream=None):
        Bt, out = self._block_args(q, k_new, v_new, out, None)
        if Bt != 1:
            raise ValueError("decode_step takes one token per sequence")
        _check(self._L.keydiff_decode_step(self._h, q.data_ptr(), k_new.data_ptr(), v_new.data_ptr(), int(pos),
                                           out.data_ptr(), _stream_ptr(stream)))
        return out

    def scores(self, stream=None):
        import torch
        out = torch.empty((self.cfg.batch, self.cfg.n_kv_heads, self.len), dtype=torch.float32, device=self.device)
        _check(self._L.keydiff_scores(self._h, out.data_ptr(), _stream_ptr(stream)))
        return out

    @property
    def len(self) -> int:
        n = C.c_int32()
        _check(self._L.keydiff_cache_len(self._h, C.byref(n)))
        return n.value

    def plan(self):
        """(key ranges, row tiles per head, key tiles, passengers: bit 0 a selection, bit 1 a row shift) of the last block step."""
        out = (C.c_int32 * 4)()
        _check(self._L.keydiff_cache_plan(self._h, out))
        return tuple(out)

    def positions(self, stream=None):
        import torch
        out = torch.empty((self.cfg.batch, self.cfg.n_kv_heads, self.len), dtype=torch.int32, device=self.device)
        if self.len:
            _check(self._L.keydiff_cache_positions(self._h, out.data_ptr(), _stream_ptr(stream)))
        return out

    def load(self, k, v, pos, stream=None):
        ln = check_load_shapes(self.cfg, self.cap, k, v, pos)
        if not (k.device == v.device == pos.device == self.device):
            raise ValueError("k, v and pos must live on the cache's device")
        _check(self._L.keydiff_cache_load(self._h, k.data_ptr(), v.data_ptr(), pos.data_ptr(), ln,
                                          _stream_ptr(stream)))

    def status(self, stream=None) -> int:
        s = C.c_int32()
        _check(self._L.keydiff_cache_status(self._h, C.byref(s), _stream_ptr(stream)))
        return s.value

    def profile_enable(self, on: bool):
        _check(self._L.keydiff_profile_enable(self._h, int(on)))

    def profile_read(self):
        ms = (C.c_float * len(KERNEL_NAMES))()
        cnt = (C.c_int32 * len(KERNEL_NAMES))()
        _check(self._L.keydiff_profile_read(self._h, ms, cnt))
        return {n: (ms[i], cnt[i]) for i, n in enumerate(KERNEL_NAMES)}

    # -- views of the caller-owned buffers (tests, not the hot path) -------------
    def key_rows(self):
        """Cache keys as a [batch][Hkv][cap][d] bf16 view (rows >= len are stale)."""
        import torch
        c = self.cfg
        n = c.batch * c.n_kv_heads * self.cap * c.head_dim
        return self._k[:n * 2].view(torch.bfloat16).view(c.batch, c.n_kv_heads, self.cap, c.head_dim)

    def value_rows(self):
        import torch
        c = self.cfg
        n = c.batch * c.n_kv_heads * self.cap * c.head_dim
        return self._v[:n * 2].view(torch.bfloat16).view(c.batch, c.n_kv_heads, self.cap, c.head_dim)
