"""ctypes binding of include/zipvl.h.  Tensors are torch CUDA(HIP) tensors used
purely as device memory; the stream is torch's current stream."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libzipvl.so"

OUT_FULL, OUT_COMPACT, KV_ALREADY_COMPACT, T_PER_BATCH = 0, 1, 2, 4
SCORE_PER_QHEAD = 1
SELECT_NEGATIVE, SELECT_NONFINITE, SELECT_OVERFLOW = 1, 2, 4
OP_SCORE, OP_SELECT, OP_SPARSE_PREFILL, OP_DECODE, OP_QUANTIZE_KV, OP_DECODE_Q, OP_SCORE_ALL_ROWS, OP_DECODE_STEP = 1, 2, 3, 4, 5, 6, 7, 8

EXPORTS = ("zipvl_version", "zipvl_last_error", "zipvl_workspace_bytes", "zipvl_score", "zipvl_select",
           "zipvl_score_all_rows", "zipvl_share_scores", "zipvl_quantize_kv", "zipvl_decode_attn_q", "zipvl_sparse_prefill", "zipvl_compact_kv", "zipvl_kv_append", "zipvl_decode_attn", "zipvl_decode_attn_static", "zipvl_decode_step",
           "zipvl_timing_enable", "zipvl_timing_read", "zipvl_probe_mfma", "zipvl_probe_stream_read")


class ZipvlError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"zipvl error {code}: {text}")
        self.code = code


class Dims(C.Structure):
    _fields_ = [("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("n", C.c_int32), ("d", C.c_int32),
                ("dtype", C.c_int32), ("q_strides", C.c_int64 * 3), ("k_strides", C.c_int64 * 3),
                ("v_strides", C.c_int64 * 3)]


class QTensor(C.Structure):
    """zipvl_qtensor: one tensor (K or V) of the mixed-precision cache."""
    _fields_ = [("hi_codes", C.c_void_p), ("hi_params", C.c_void_p), ("lo_codes", C.c_void_p), ("lo_params", C.c_void_p)]


_lib = None


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load libzipvl.so from the package directory; raise if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ZipvlError(-100, f"{path} is missing: build it with `python -m paper_2410_08584_amd.build` "
                               "(there is no CPU fallback)")
    lib = C.CDLL(path)
    vp, i32p, f32p = C.c_void_p, C.c_void_p, C.c_void_p
    lib.zipvl_version.restype = C.c_int
    lib.zipvl_last_error.restype = C.c_char_p
    lib.zipvl_workspace_bytes.restype = C.c_size_t
    lib.zipvl_workspace_bytes.argtypes = [C.c_int, C.POINTER(Dims), C.c_int]
    lib.zipvl_score.argtypes = [vp, vp, C.POINTER(Dims), C.POINTER(C.c_int32), C.c_int, C.c_float, C.c_int,
                                f32p, f32p, vp, C.c_size_t, vp]
    lib.zipvl_select.argtypes = [f32p, f32p, C.c_int, C.c_int, C.c_double, i32p, i32p, i32p, vp, C.c_size_t, vp]
    lib.zipvl_sparse_prefill.argtypes = [vp, vp, vp, C.POINTER(Dims), i32p, i32p, C.c_float, C.c_int,
                                         vp, vp, C.c_size_t, vp]
    lib.zipvl_compact_kv.argtypes = [vp, vp, C.POINTER(Dims), i32p, i32p, vp, vp, C.c_int32, i32p, C.c_int, vp]
    lib.zipvl_quantize_kv.argtypes = [vp, vp, C.POINTER(Dims), i32p, i32p, C.POINTER(QTensor), C.POINTER(QTensor),
                                      C.c_int32, C.c_int32, i32p, i32p, C.c_int, vp, C.c_size_t, vp]
    lib.zipvl_decode_attn_q.argtypes = [vp, C.POINTER(QTensor), C.POINTER(QTensor), i32p, i32p, C.c_int32, C.c_int32,
                                        vp, vp, i32p, C.c_int32, C.POINTER(Dims), C.c_float, vp, vp, C.c_size_t, vp]
    lib.zipvl_score_all_rows.argtypes = [vp, vp, C.POINTER(Dims), C.c_float, f32p, f32p, vp, C.c_size_t, vp]
    lib.zipvl_probe_mfma.argtypes = [C.c_int, C.c_int, f32p, vp]
    lib.zipvl_probe_stream_read.argtypes = [vp, C.c_size_t, C.c_int, vp, vp]
    lib.zipvl_probe_mfma.restype = C.c_int
    lib.zipvl_probe_stream_read.restype = C.c_int
    lib.zipvl_share_scores.argtypes = [f32p, f32p, C.c_int, C.c_int, C.c_int, f32p, f32p, vp]
    lib.zipvl_kv_append.argtypes = [vp, vp, i32p, C.c_int32, vp, vp, C.POINTER(Dims), vp]
    lib.zipvl_decode_attn.argtypes = [vp, vp, vp, i32p, C.c_int32, C.POINTER(Dims), C.c_float, vp, vp,
                                      C.c_size_t, vp]
    lib.zipvl_decode_attn_static.argtypes = [vp, vp, vp, i32p, C.c_int32, C.POINTER(Dims), C.c_float, vp, vp]
    lib.zipvl_decode_attn_static.restype = C.c_int
    lib.zipvl_decode_step.argtypes = [vp, vp, vp, i32p, C.c_int32, vp, vp, C.POINTER(Dims), C.c_float, vp, vp,
                                      C.c_size_t, vp]
    lib.zipvl_timing_enable.argtypes = [C.c_int]
    lib.zipvl_timing_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int)]
    lib.zipvl_timing_enable.restype = C.c_int
    lib.zipvl_timing_read.restype = C.c_int
    for name in ("zipvl_score", "zipvl_score_all_rows", "zipvl_select", "zipvl_share_scores", "zipvl_quantize_kv",
                 "zipvl_decode_attn_q", "zipvl_sparse_prefill", "zipvl_compact_kv", "zipvl_kv_append", "zipvl_decode_attn",
                 "zipvl_decode_step"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def zipvl_version() -> int:
    return int(load_library().zipvl_version())


def zipvl_last_error() -> str:
    return load_library().zipvl_last_error().decode()


def _check(rc: int):
    if rc != 0:
        raise ZipvlError(rc, zipvl_last_error())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.bfloat16:
        return 1
    raise ZipvlError(-5, f"unsupported tensor dtype {t.dtype}")


def _strides3(t: Optional[torch.Tensor]) -> Tuple[int, int, int]:
    if t is None:
        return (0, 0, 0)
    if t.dim() != 4 or t.stride(3) != 1:
        raise ZipvlError(-1, "expected a [B,H,n,d] view with a contiguous last dimension")
    return (t.stride(0), t.stride(1), t.stride(2))


def dims_of(Q: Optional[torch.Tensor], K: Optional[torch.Tensor], V: Optional[torch.Tensor] = None, *,
            B=None, Hq=None, Hkv=None, n=None, d=None, dtype=None) -> Dims:
    """Fill a zipvl_dims from [B,H,n,d] tensors (any memory order with d contiguous)."""
    ref = Q if Q is not None else K
    dm = Dims()
    dm.B = B if B is not None else ref.shape[0]
    dm.Hq = Hq if Hq is not None else (Q.shape[1] if Q is not None else K.shape[1])
    dm.Hkv = Hkv if Hkv is not None else (K.shape[1] if K is not None else dm.Hq)
    dm.n = n if n is not None else ref.shape[2]
    dm.d = d if d is not None else ref.shape[3]
    dm.dtype = dtype if dtype is not None else _dtype_code(ref)
    dm.q_strides = (C.c_int64 * 3)(*_strides3(Q))
    dm.k_strides = (C.c_int64 * 3)(*_strides3(K))
    dm.v_strides = (C.c_int64 * 3)(*_strides3(V))
    return dm


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _dense(*tensors):
    """The library addresses these arrays as contiguous rows: refuse views with other strides."""
    for t in tensors:
        if t is not None and not t.is_contiguous():
            raise ZipvlError(-1, f"expected a contiguous tensor, got strides {tuple(t.stride())} for shape {tuple(t.shape)}")


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def workspace_bytes(op: int, dims: Dims, m: int = 0) -> int:
    return int(load_library().zipvl_workspace_bytes(op, C.byref(dims), m))


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def zipvl_score(Q: torch.Tensor, K: torch.Tensor, probe_pos: Sequence[int], softmax_scale: float, *,
                mass: Optional[torch.Tensor] = None, rank: Optional[torch.Tensor] = None,
                want_rank: bool = True, ws: Optional[torch.Tensor] = None, flags: int = 0):
    """(mass, rank) fp32 [B*Hkv, n] from the probe rows of Q against K ([B*Hq, n] with flags=SCORE_PER_QHEAD)."""
    lib = load_library()
    dm = dims_of(Q, K)
    units = dm.B * (dm.Hq if flags & SCORE_PER_QHEAD else dm.Hkv)
    pp = [int(p) for p in probe_pos]
    arr = (C.c_int32 * max(len(pp), 1))(*pp)
    if mass is None:
        mass = torch.empty((units, dm.n), dtype=torch.float32, device=Q.device)
    if rank is None and want_rank:
        rank = torch.empty((units, dm.n), dtype=torch.float32, device=Q.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SCORE, dm, len(pp)), Q.device)
    _dense(mass, rank)
    _check(lib.zipvl_score(_ptr(Q), _ptr(K), C.byref(dm), arr, len(pp), float(softmax_scale), int(flags),
                           _ptr(mass), _ptr(rank), _ptr(ws), ws.numel(), _stream()))
    return mass, rank


def select_workspace(units: int, device) -> torch.Tensor:
    """A zero-filled workspace for the two-kernel form of zipvl_select (kept between calls: every call leaves it zero)."""
    dm = dims_of(None, None, None, B=units, Hq=1, Hkv=1, n=64, d=64, dtype=0)
    return torch.zeros(max(256, workspace_bytes(OP_SELECT, dm)), dtype=torch.uint8, device=device)


def zipvl_select(mass: torch.Tensor, rank: Optional[torch.Tensor], tau: float, *,
                 idx: Optional[torch.Tensor] = None, k: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None,
                 status: Optional[torch.Tensor] = None):
    """(idx [units,n] int32 with the first k entries valid and ascending, k [units] int32).  ws: select_workspace(units)
    for the two-kernel form, None for the one-kernel form.  status: int32 [units] tensor that receives the SELECT_* bits."""
    lib = load_library()
    _dense(mass, rank, idx, k)
    units, n = mass.shape
    if idx is None:
        idx = torch.empty((units, n), dtype=torch.int32, device=mass.device)
    if k is None:
        k = torch.empty((units,), dtype=torch.int32, device=mass.device)
    _check(lib.zipvl_select(_ptr(mass), _ptr(rank), units, n, float(tau), _ptr(idx), _ptr(k), _ptr(status), _ptr(ws),
                            0 if ws is None else ws.numel(), _stream()))
    return idx, k


def zipvl_score_all_rows(Q: torch.Tensor, K: torch.Tensor, softmax_scale: float, *,
                         mass: Optional[torch.Tensor] = None, rank: Optional[torch.Tensor] = None,
                         ws: Optional[torch.Tensor] = None, want_rank: bool = True):
    """(mass, rank) [B*Hkv, n] fp32 from every row of the attention matrix (exact Eq. (6) / Eq. (8))."""
    lib = load_library()
    dm = dims_of(Q, K)
    units = dm.B * dm.Hkv
    if mass is None:
        mass = torch.empty((units, dm.n), dtype=torch.float32, device=Q.device)
    if rank is None and want_rank:
        rank = torch.empty((units, dm.n), dtype=torch.float32, device=Q.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SCORE_ALL_ROWS, dm), Q.device)
    _check(lib.zipvl_score_all_rows(_ptr(Q), _ptr(K), C.byref(dm), float(softmax_scale), _ptr(mass), _ptr(rank),
                                    _ptr(ws), ws.numel(), _stream()))
    return mass, rank


def zipvl_share_scores(mass: torch.Tensor, rank: Optional[torch.Tensor], B: int, *,
                       mass_b: Optional[torch.Tensor] = None, rank_b: Optional[torch.Tensor] = None):
    """(mass_b, rank_b [B, n]): the per-unit scores [B*Hkv, n] averaged over the units of each batch element."""
    lib = load_library()
    _dense(mass, rank, mass_b, rank_b)
    units, n = mass.shape
    Hkv = units // B
    if mass_b is None:
        mass_b = torch.empty((B, n), dtype=torch.float32, device=mass.device)
    if rank is not None and rank_b is None:
        rank_b = torch.empty((B, n), dtype=torch.float32, device=mass.device)
    _check(lib.zipvl_share_scores(_ptr(mass), _ptr(rank), int(B), int(Hkv), int(n), _ptr(mass_b), _ptr(rank_b), _stream()))
    return mass_b, rank_b


def zipvl_sparse_prefill(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, idx: Optional[torch.Tensor],
                         k: Optional[torch.Tensor], softmax_scale: float, flags: int = OUT_FULL, *,
                         O: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """O [B,Hq,n,d]: causal attention over the kept tokens (idx=k=None: all tokens)."""
    lib = load_library()
    dm = dims_of(Q, K, V)
    if O is None:
        O = torch.empty((dm.B, dm.Hq, dm.n, dm.d), dtype=Q.dtype, device=Q.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_SPARSE_PREFILL, dm), Q.device)
    _check(lib.zipvl_sparse_prefill(_ptr(Q), _ptr(K), _ptr(V), C.byref(dm), _ptr(idx), _ptr(k),
                                    float(softmax_scale), int(flags), _ptr(O), _ptr(ws), ws.numel(), _stream()))
    return O


def zipvl_compact_kv(K: torch.Tensor, V: torch.Tensor, idx: Optional[torch.Tensor], k: Optional[torch.Tensor],
                     cap: int, flags: int = 0, *, Kc: Optional[torch.Tensor] = None, Vc: Optional[torch.Tensor] = None,
                     length: Optional[torch.Tensor] = None):
    """(Kc, Vc [B*Hkv, cap, d], len [B*Hkv] int32): the evicted cache (flags: 0 or T_PER_BATCH)."""
    lib = load_library()
    dm = dims_of(None, K, V, Hq=K.shape[1])
    units = dm.B * dm.Hkv
    if Kc is None:
        Kc = torch.empty((units, cap, dm.d), dtype=K.dtype, device=K.device)
    if Vc is None:
        Vc = torch.empty((units, cap, dm.d), dtype=K.dtype, device=K.device)
    if length is None:
        length = torch.empty((units,), dtype=torch.int32, device=K.device)
    _check(lib.zipvl_compact_kv(_ptr(K), _ptr(V), C.byref(dm), _ptr(idx), _ptr(k), _ptr(Kc), _ptr(Vc),
                                int(cap), _ptr(length), int(flags), _stream()))
    return Kc, Vc, length


def zipvl_kv_append(Kc: torch.Tensor, Vc: torch.Tensor, length: torch.Tensor, k_new: torch.Tensor,
                    v_new: torch.Tensor, *, B: int, Hkv: int):
    lib = load_library()
    units, cap, d = Kc.shape
    dm = dims_of(None, None, None, B=B, Hq=Hkv, Hkv=Hkv, n=cap, d=d, dtype=_dtype_code(Kc))
    _check(lib.zipvl_kv_append(_ptr(Kc), _ptr(Vc), _ptr(length), int(cap), _ptr(k_new), _ptr(v_new),
                               C.byref(dm), _stream()))
    return length


def zipvl_decode_attn(q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, length: torch.Tensor,
                      softmax_scale: float, *, B: int, Hq: int, Hkv: int,
                      o: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """o [B*Hq, d]: one query per head against the first len[u] cached rows."""
    lib = load_library()
    units, cap, d = Kc.shape
    dm = dims_of(None, None, None, B=B, Hq=Hq, Hkv=Hkv, n=cap, d=d, dtype=_dtype_code(Kc))
    if o is None:
        o = torch.empty((B * Hq, d), dtype=q.dtype, device=q.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_DECODE, dm), q.device)
    _check(lib.zipvl_decode_attn(_ptr(q), _ptr(Kc), _ptr(Vc), _ptr(length), int(cap), C.byref(dm),
                                 float(softmax_scale), _ptr(o), _ptr(ws), ws.numel(), _stream()))
    return o


def zipvl_decode_attn_static(q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, length: torch.Tensor,
                             softmax_scale: float, *, B: int, Hq: int, Hkv: int, o: torch.Tensor):
    """zipvl_decode_attn without a workspace (the library's built-in scratch array); `o` is the caller's."""
    lib = load_library()
    units, cap, d = Kc.shape
    dm = dims_of(None, None, None, B=B, Hq=Hq, Hkv=Hkv, n=cap, d=d, dtype=_dtype_code(Kc))
    _check(lib.zipvl_decode_attn_static(_ptr(q), _ptr(Kc), _ptr(Vc), _ptr(length), int(cap), C.byref(dm),
                                        float(softmax_scale), _ptr(o), _stream()))
    return o


def decode_step_workspace(B: int, Hq: int, Hkv: int, cap: int, d: int, dtype_like: torch.Tensor) -> torch.Tensor:
    """A zero-filled workspace for zipvl_decode_step (its arrival counters must start at zero)."""
    dm = dims_of(None, None, None, B=B, Hq=Hq, Hkv=Hkv, n=cap, d=d, dtype=_dtype_code(dtype_like))
    return torch.zeros(max(256, workspace_bytes(OP_DECODE_STEP, dm)), dtype=torch.uint8, device=dtype_like.device)


def zipvl_decode_step(q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, length: torch.Tensor,
                      k_new: torch.Tensor, v_new: torch.Tensor, softmax_scale: float, *, B: int, Hq: int, Hkv: int,
                      ws: torch.Tensor, o: Optional[torch.Tensor] = None):
    """Append k_new / v_new and attend, one launch; ws from decode_step_workspace (kept between steps)."""
    lib = load_library()
    units, cap, d = Kc.shape
    dm = dims_of(None, None, None, B=B, Hq=Hq, Hkv=Hkv, n=cap, d=d, dtype=_dtype_code(Kc))
    if o is None:
        o = torch.empty((B * Hq, d), dtype=q.dtype, device=q.device)
    _check(lib.zipvl_decode_step(_ptr(q), _ptr(Kc), _ptr(Vc), _ptr(length), int(cap), _ptr(k_new), _ptr(v_new),
                                 C.byref(dm), float(softmax_scale), _ptr(o), _ptr(ws), ws.numel(), _stream()))
    return o


class QCache:
    """Device arrays of the mixed-precision cache built by zipvl_quantize_kv."""

    def __init__(self, units: int, cap_hi: int, cap_lo: int, d: int, device):
        def tensor():
            return dict(hi_codes=torch.empty((units, cap_hi, d // 2), dtype=torch.uint8, device=device),
                        hi_params=torch.empty((units, cap_hi, 2), dtype=torch.float16, device=device),
                        lo_codes=torch.empty((units, cap_lo, d // 4), dtype=torch.uint8, device=device),
                        lo_params=torch.empty((units, cap_lo, 2), dtype=torch.float16, device=device))
        self.K, self.V = tensor(), tensor()
        self.len_hi = torch.empty((units,), dtype=torch.int32, device=device)
        self.len_lo = torch.empty((units,), dtype=torch.int32, device=device)
        self.units, self.cap_hi, self.cap_lo, self.d = units, cap_hi, cap_lo, d

    @staticmethod
    def _struct(t) -> QTensor:
        return QTensor(t["hi_codes"].data_ptr(), t["hi_params"].data_ptr(), t["lo_codes"].data_ptr(), t["lo_params"].data_ptr())

    def structs(self):
        return self._struct(self.K), self._struct(self.V)

    def nbytes(self) -> int:
        return sum(x.numel() * x.element_size() for t in (self.K, self.V) for x in t.values())


def zipvl_quantize_kv(K: torch.Tensor, V: torch.Tensor, idx: Optional[torch.Tensor], k: Optional[torch.Tensor],
                      cap_hi: int, cap_lo: int, flags: int = 0, *, cache: Optional[QCache] = None,
                      ws: Optional[torch.Tensor] = None) -> QCache:
    """Mixed-precision cache: tokens of T at 4 bits, the others at 2 bits (flags: 0 or T_PER_BATCH)."""
    lib = load_library()
    dm = dims_of(None, K, V, Hq=K.shape[1])
    units = dm.B * dm.Hkv
    if cache is None:
        cache = QCache(units, cap_hi, cap_lo, dm.d, K.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_QUANTIZE_KV, dm), K.device)
    kq, vq = cache.structs()
    _check(lib.zipvl_quantize_kv(_ptr(K), _ptr(V), C.byref(dm), _ptr(idx), _ptr(k), C.byref(kq), C.byref(vq),
                                 int(cap_hi), int(cap_lo), _ptr(cache.len_hi), _ptr(cache.len_lo), int(flags),
                                 _ptr(ws), ws.numel(), _stream()))
    return cache


def zipvl_decode_attn_q(q: torch.Tensor, cache: QCache, softmax_scale: float, *, B: int, Hq: int, Hkv: int,
                        K_tail: Optional[torch.Tensor] = None, V_tail: Optional[torch.Tensor] = None,
                        len_tail: Optional[torch.Tensor] = None,
                        o: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """o [B*Hq, d]: one query per head against the dequantised cache followed by the appended rows."""
    lib = load_library()
    cap_tail = 0 if K_tail is None else K_tail.shape[1]
    dm = dims_of(None, None, None, B=B, Hq=Hq, Hkv=Hkv, n=cache.cap_hi + cache.cap_lo + cap_tail, d=cache.d,
                 dtype=_dtype_code(q))
    if o is None:
        o = torch.empty((B * Hq, cache.d), dtype=q.dtype, device=q.device)
    if ws is None:
        ws = _workspace(workspace_bytes(OP_DECODE_Q, dm), q.device)
    kq, vq = cache.structs()
    _check(lib.zipvl_decode_attn_q(_ptr(q), C.byref(kq), C.byref(vq), _ptr(cache.len_hi), _ptr(cache.len_lo),
                                   int(cache.cap_hi), int(cache.cap_lo), _ptr(K_tail), _ptr(V_tail), _ptr(len_tail),
                                   int(cap_tail), C.byref(dm), float(softmax_scale), _ptr(o), _ptr(ws), ws.numel(),
                                   _stream()))
    return o


KERNELS = ("score_rowstats", "score_colsum", "select", "compact_kv", "kv_append", "zero_fill",
           "pack_kv", "flash_kept", "decode_partial", "decode_combine", "score_rowfinal", "share_scores",
           "token_slots", "quantize_rows", "decode_q_partial", "allrows_lse", "allrows_colsum", "probe_mfma", "probe_read",
           "decode_step", "select_hist")


def zipvl_probe_peaks(device="cuda:0", iters: int = 4096, read_mib: int = 4096):
    """(sustained bf16 MFMA TFLOP/s, sustained read GB/s) of this GPU, from the library's two probe kernels."""
    lib = load_library()
    wgs = 2048                                               # 8 workgroups per CU queue up; 2 are resident (256 CUs)
    out = torch.empty((wgs * 256,), dtype=torch.float32, device=device)
    src = torch.empty((read_mib << 20,), dtype=torch.uint8, device=device).fill_(3)
    outr = torch.empty((4096 * 256,), dtype=torch.int32, device=device)
    res = []
    for kid, call in ((KERNELS.index("probe_mfma"), lambda: lib.zipvl_probe_mfma(iters, wgs, _ptr(out), _stream())),
                      (KERNELS.index("probe_read"), lambda: lib.zipvl_probe_stream_read(_ptr(src), src.numel(), 4096, _ptr(outr), _stream()))):
        for _ in range(3):
            _check(call())
        torch.cuda.synchronize()
        zipvl_timing_enable(True)
        for _ in range(5):
            _check(call())
        torch.cuda.synchronize()
        ms, cnt = zipvl_timing_read(kid)
        zipvl_timing_enable(False)
        res.append(ms / cnt)
    tflops = wgs * 4 * iters * 8 * 32768.0 / (res[0] * 1e-3) / 1e12
    gbps = src.numel() / (res[1] * 1e-3) / 1e9
    return tflops, gbps


def zipvl_timing_enable(on: bool) -> None:
    _check(load_library().zipvl_timing_enable(1 if on else 0))


def zipvl_timing_read(kernel: int):
    """(total milliseconds, launches) of one kernel since timing was enabled."""
    ms, cnt = C.c_double(0.0), C.c_int(0)
    _check(load_library().zipvl_timing_read(int(kernel), C.byref(ms), C.byref(cnt)))
    return ms.value, cnt.value
