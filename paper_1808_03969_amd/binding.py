"""ctypes binding of ``include/rii.h``.  Argument marshalling only.

Host-side entry points take numpy arrays; device-side entry points take torch tensors that
live on the GPU and launch on torch's current stream.  There is no fallback: if the compiled
library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
import re

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librii_hip.so")
_INCLUDE = os.path.join(os.path.dirname(_HERE), "include")
_HEADERS = [os.path.join(_INCLUDE, "rii.h"), os.path.join(_INCLUDE, "rii_bench.h")]
_lib = None

RII_MEM_HOST, RII_MEM_DEVICE = 0, 1
RII_MAX_TOPK, RII_MAX_SORT = 1024, 16384
RII_OPT_GATHER_COPY = 2
RII_SCAN_COUNTERS = 8


class RiiError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        msg = load_library().rii_status_string(status).decode()
        super().__init__(f"{what}: {msg} (status {status})")


def library_path() -> str:
    return _LIB_PATH


def declared_symbols() -> list[str]:
    """Names of the functions the headers under ``include/`` declare."""
    names = set()
    for h in _HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names.update(re.findall(r"\b(rii_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def load_library():
    """Load ``librii_hip.so``; raises when it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_1808_03969_amd.build` "
                "(there is no fallback path)")
        lib = ctypes.CDLL(_LIB_PATH)
        lib.rii_status_string.restype = ctypes.c_char_p
        lib.rii_status_string.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise RiiError(rc, what)


def _np(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _hp(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dp(t, dtype=None):
    """Device pointer of a contiguous CUDA/HIP tensor (None passes NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device entry points need contiguous GPU tensors")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


i64 = ctypes.c_int64


# ------------------------------------------------------------------ host, offline
def rii_train_codebooks(x: np.ndarray, M: int, Ks: int = 256, iters: int = 20, seed: int = 0) -> np.ndarray:
    x = _np(x, np.float32)
    n, D = x.shape
    if M <= 0 or D % M:
        raise RiiError(-2, "rii_train_codebooks")
    out = np.empty((M, Ks, D // M), dtype=np.float32)
    _check(load_library().rii_train_codebooks(_hp(x), i64(n), D, M, Ks, iters, ctypes.c_uint64(seed), _hp(out)),
           "rii_train_codebooks")
    return out


def rii_encode(codebooks: np.ndarray, x: np.ndarray) -> np.ndarray:
    cb, x = _np(codebooks, np.float32), _np(x, np.float32)
    M, Ks, Ds = cb.shape
    n, D = x.shape
    if D != M * Ds:
        raise RiiError(-2, "rii_encode")
    out = np.empty((n, M), dtype=np.uint8)
    _check(load_library().rii_encode(_hp(cb), D, M, Ks, _hp(x), i64(n), _hp(out)), "rii_encode")
    return out


# ------------------------------------------------------------------ index handle
class Index:
    """Owner of an ``rii_index_t*``.  Methods mirror the ``rii_index_*`` functions."""

    def __init__(self, codebooks: np.ndarray):
        cb = _np(codebooks, np.float32)
        if cb.ndim != 3:
            raise ValueError("codebooks must be [M][Ks][D/M]")
        self.M, self.Ks, self.Ds = cb.shape
        self.D = self.M * self.Ds
        self._h = ctypes.c_void_p()
        self._lib = load_library()
        _check(self._lib.rii_index_create(_hp(cb), self.D, self.M, self.Ks, ctypes.byref(self._h)), "rii_index_create")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            self._lib.rii_index_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def handle(self):
        return self._h

    def add(self, codes):
        """PushBack n codes ([n][M] uint8; numpy array on the host or torch tensor on the GPU)."""
        if isinstance(codes, torch.Tensor) and codes.is_cuda:
            if codes.dtype != torch.uint8 or codes.dim() != 2 or codes.shape[1] != self.M:
                raise ValueError("codes must be uint8 [n][M]")
            _check(self._lib.rii_index_add(self._h, _dp(codes.contiguous()), i64(codes.shape[0]), RII_MEM_DEVICE),
                   "rii_index_add")
        else:
            c = _np(codes, np.uint8)
            if c.ndim != 2 or c.shape[1] != self.M:
                raise ValueError("codes must be uint8 [n][M]")
            _check(self._lib.rii_index_add(self._h, _hp(c), i64(c.shape[0]), RII_MEM_HOST), "rii_index_add")

    def set_lists(self, coarse, list_offsets, list_ids):
        c, o, l = _np(coarse, np.uint8), _np(list_offsets, np.int64), _np(list_ids, np.int32)
        _check(self._lib.rii_index_set_lists(self._h, _hp(c), c.shape[0], _hp(o), _hp(l), RII_MEM_HOST),
               "rii_index_set_lists")

    def build_lists(self, coarse):
        c = _np(coarse, np.uint8)
        _check(self._lib.rii_index_build_lists(self._h, _hp(c), c.shape[0]), "rii_index_build_lists")

    def reconfigure(self, K: int, iters: int = 20, seed: int = 0):
        _check(self._lib.rii_index_reconfigure(self._h, K, iters, ctypes.c_uint64(seed)), "rii_index_reconfigure")

    def set_option(self, option: int, value: int):
        _check(self._lib.rii_index_set_option(self._h, option, i64(value)), "rii_index_set_option")

    def reserve_workspace(self, Q: int, topk: int, max_targets: int = 0, nprobe: int = 0):
        _check(self._lib.rii_index_reserve_workspace(self._h, Q, topk, i64(max_targets), nprobe),
               "rii_index_reserve_workspace")

    def set_threshold(self, theta: int):
        _check(self._lib.rii_index_set_threshold(self._h, i64(theta)), "rii_index_set_threshold")

    def calibrate_threshold(self, L: int, topk: int = 100, nq: int = 64, max_targets: int = 0, seed: int = 0) -> int:
        """Measure the linear-scan / inverted-index crossover and store it as theta."""
        theta = ctypes.c_int64(0)
        _check(self._lib.rii_index_calibrate_threshold(self._h, i64(L), topk, nq, i64(max_targets),
                                                       ctypes.c_uint64(seed), ctypes.byref(theta)),
               "rii_index_calibrate_threshold")
        return int(theta.value)

    def info(self) -> dict:
        out = np.zeros(8, dtype=np.int64)
        _check(self._lib.rii_index_info(self._h, _hp(out)), "rii_index_info")
        keys = ("N", "D", "M", "Ks", "K", "theta", "paper_bytes", "device_bytes")
        return dict(zip(keys, (int(v) for v in out)))

    def get_lists(self):
        """(coarse [K][M], list_offsets [K+1], list_ids [N], assign [N]) as numpy arrays."""
        inf = self.info()
        coarse = np.empty((inf["K"], self.M), dtype=np.uint8)
        off = np.empty(inf["K"] + 1, dtype=np.int64)
        ids = np.empty(inf["N"], dtype=np.int32)
        a = np.empty(inf["N"], dtype=np.int32)
        _check(self._lib.rii_index_get_lists(self._h, _hp(coarse), _hp(off), _hp(ids), _hp(a), RII_MEM_HOST),
               "rii_index_get_lists")
        return coarse, off, ids, a

    def get_codes(self, first: int = 0, n: int | None = None) -> np.ndarray:
        if n is None:
            n = self.info()["N"] - first
        out = np.empty((n, self.M), dtype=np.uint8)
        _check(self._lib.rii_index_get_codes(self._h, i64(first), i64(n), _hp(out), RII_MEM_HOST), "rii_index_get_codes")
        return out


# ------------------------------------------------------------------ device, online
def _out(Q, k, device):
    return (torch.empty((Q, k), dtype=torch.int32, device=device), torch.empty((Q, k), dtype=torch.float32, device=device))


def rii_build_lut(index: Index, q: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    Q = q.shape[0]
    if q.dim() != 2 or q.shape[1] != index.D:
        raise ValueError("q must be [Q][D]")
    lut = out if out is not None else torch.empty((Q, index.M, index.Ks), dtype=torch.float32, device=q.device)
    _check(load_library().rii_build_lut(index.handle, _dp(q, torch.float32), Q, _dp(lut, torch.float32), _stream()),
           "rii_build_lut")
    return lut


def rii_coarse_assign(index: Index, lut: torch.Tensor, nprobe: int, want_d0: bool = True):
    Q = lut.shape[0]
    n = max(nprobe, 1)
    ids = torch.empty((Q, n), dtype=torch.int32, device=lut.device)
    d0 = torch.empty((Q, n), dtype=torch.float32, device=lut.device) if want_d0 else None
    _check(load_library().rii_coarse_assign(index.handle, _dp(lut, torch.float32), Q, nprobe, _dp(ids), _dp(d0), _stream()),
           "rii_coarse_assign")
    return ids, d0


def rii_adc_scan_linear(index: Index, lut: torch.Tensor, topk: int, out=None):
    Q = lut.shape[0]
    ids, dist = out if out is not None else _out(Q, max(topk, 1), lut.device)
    _check(load_library().rii_adc_scan_linear(index.handle, _dp(lut, torch.float32), Q, topk, _dp(ids, torch.int32),
                                              _dp(dist, torch.float32), _stream()), "rii_adc_scan_linear")
    return ids, dist


def rii_check_target_ids(index: Index, target_ids: torch.Tensor | None, target_offsets: torch.Tensor) -> int:
    """Status of the precondition check (0, RII_ERR_UNSORTED_IDS or RII_ERR_INVALID_ARG); does not raise."""
    Q = target_offsets.numel() - 1
    tid = _dp(target_ids, torch.int32) if target_ids is not None and target_ids.numel() else None
    return int(load_library().rii_check_target_ids(index.handle, tid, _dp(target_offsets, torch.int64), Q, _stream()))


def rii_adc_scan_subset(index: Index, lut: torch.Tensor, target_ids: torch.Tensor, target_offsets: torch.Tensor,
                        max_targets: int, topk: int, out=None):
    Q = lut.shape[0]
    ids, dist = out if out is not None else _out(Q, max(topk, 1), lut.device)
    tid = _dp(target_ids, torch.int32) if target_ids is not None and target_ids.numel() else None
    _check(load_library().rii_adc_scan_subset(index.handle, _dp(lut, torch.float32), Q, tid,
                                              _dp(target_offsets, torch.int64), i64(max_targets), topk,
                                              _dp(ids, torch.int32), _dp(dist, torch.float32), _stream()),
           "rii_adc_scan_subset")
    return ids, dist


def rii_adc_scan_ivf(index: Index, lut: torch.Tensor, probe_lists: torch.Tensor, topk: int,
                     target_ids: torch.Tensor | None = None, target_offsets: torch.Tensor | None = None,
                     L: int = 0, out=None):
    Q = lut.shape[0]
    ids, dist = out if out is not None else _out(Q, max(topk, 1), lut.device)
    _check(load_library().rii_adc_scan_ivf(index.handle, _dp(lut, torch.float32), Q, _dp(probe_lists, torch.int32),
                                           probe_lists.shape[1], _dp(target_ids, torch.int32),
                                           _dp(target_offsets, torch.int64), i64(L), topk, _dp(ids, torch.int32),
                                           _dp(dist, torch.float32), _stream()), "rii_adc_scan_ivf")
    return ids, dist


def rii_topk(cand_dist: torch.Tensor, cand_ids: torch.Tensor | None, cand_offsets: torch.Tensor, topk: int,
             max_segment: int = 0):
    Q = cand_offsets.numel() - 1
    ids, dist = _out(Q, max(topk, 1), cand_dist.device)
    _check(load_library().rii_topk(_dp(cand_dist, torch.float32), _dp(cand_ids, torch.int32),
                                   _dp(cand_offsets, torch.int64), Q, i64(max_segment), topk, _dp(ids), _dp(dist),
                                   _stream()), "rii_topk")
    return ids, dist


def rii_query(index: Index, q: torch.Tensor, topk: int, target_ids: torch.Tensor | None = None,
              target_offsets: torch.Tensor | None = None, max_targets: int = 0, L: int = 1, out=None):
    Q = q.shape[0]
    if q.dim() != 2 or q.shape[1] != index.D:
        raise ValueError("q must be [Q][D]")
    ids, dist = out if out is not None else _out(Q, max(topk, 1), q.device)
    tid = target_ids
    if tid is not None and tid.numel() == 0:  # every target set empty: a valid 1-element dummy keeps it non-NULL
        tid = torch.zeros(1, dtype=torch.int32, device=q.device)
    _check(load_library().rii_query(index.handle, _dp(q, torch.float32), Q, topk, _dp(tid, torch.int32),
                                    _dp(target_offsets, torch.int64), i64(max_targets), i64(L), _dp(ids, torch.int32),
                                    _dp(dist, torch.float32), _stream()), "rii_query")
    return ids, dist


def rii_query_noalloc(index: Index, q: torch.Tensor, topk: int, target_ids: torch.Tensor | None = None,
                      target_offsets: torch.Tensor | None = None, max_targets: int = 0, L: int = 1, out=None):
    """rii_query on the library's static scratch array; `out` = (ids, dist) must be given when the
    caller may not allocate (otherwise torch allocates the two result tensors)."""
    Q = q.shape[0]
    if q.dim() != 2 or q.shape[1] != index.D:
        raise ValueError("q must be [Q][D]")
    ids, dist = out if out is not None else _out(Q, max(topk, 1), q.device)
    _check(load_library().rii_query_noalloc(index.handle, _dp(q, torch.float32), Q, topk, _dp(target_ids, torch.int32),
                                            _dp(target_offsets, torch.int64), i64(max_targets), i64(L),
                                            _dp(ids, torch.int32), _dp(dist, torch.float32), _stream()),
           "rii_query_noalloc")
    return ids, dist


# ------------------------------------------------------------------ device, offline
def rii_encode_device(index: Index, x: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    n = x.shape[0]
    codes = out if out is not None else torch.empty((n, index.M), dtype=torch.uint8, device=x.device)
    _check(load_library().rii_encode_device(index.handle, _dp(x, torch.float32), i64(n), _dp(codes, torch.uint8), _stream()),
           "rii_encode_device")
    return codes


def rii_rotate(R: torch.Tensor, x: torch.Tensor) -> torch.Tensor:
    """y = R x per row (the rotation of the OPQ variant, Sec. 4.5)."""
    n, D = x.shape
    if R.shape != (D, D):
        raise ValueError("rotation must be D x D")
    y = torch.empty_like(x)
    _check(load_library().rii_rotate(_dp(R, torch.float32), D, _dp(x, torch.float32), i64(n), _dp(y, torch.float32),
                                     _stream()), "rii_rotate")
    return y


def rii_assign(index: Index, codes: torch.Tensor, coarse: torch.Tensor) -> torch.Tensor:
    n, K = codes.shape[0], coarse.shape[0]
    out = torch.empty(n, dtype=torch.int32, device=codes.device)
    _check(load_library().rii_assign(index.handle, _dp(codes, torch.uint8), i64(n), _dp(coarse, torch.uint8), K,
                                     _dp(out), _stream()), "rii_assign")
    return out


def rii_index_read_scan_counters(index: Index):
    """The tallies of the whole-database scan kernels since the last call (a list of
    RII_SCAN_COUNTERS integers, see rii_bench.h); resets them."""
    out = (ctypes.c_uint64 * RII_SCAN_COUNTERS)()
    _check(load_library().rii_index_read_scan_counters(index.handle, out), "rii_index_read_scan_counters")
    return [int(v) for v in out]


def rii_scan_linear_plan(index: Index, Q: int, topk: int):
    """(queries per block, row chunks per query group) of the launch rii_adc_scan_linear would make."""
    qpb, chunks = ctypes.c_int(0), ctypes.c_int64(0)
    _check(load_library().rii_scan_linear_plan(index.handle, Q, topk, ctypes.byref(qpb), ctypes.byref(chunks)),
           "rii_scan_linear_plan")
    return qpb.value, chunks.value


def rii_bench_lds_lookups(width: int, blocks: int, threads: int, iters: int, lds_bytes: int = 98 * 1024) -> int:
    """Measurement aid: launch the LDS look-up ceiling kernel on the current stream (time it with
    events); returns the number of look-ups it performs."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    _check(load_library().rii_bench_lds_lookups(width, blocks, threads, iters, lds_bytes, _dp(sink), _stream()),
           "rii_bench_lds_lookups")
    return blocks * threads * 32 * iters


def rii_bench_scan_linear_half(index: Index, lut: torch.Tensor, topk: int, out=None):
    """Measurement aid: rii_adc_scan_linear through the half-precision-table variant of the batched kernel."""
    Q = lut.shape[0]
    ids, dist = out if out is not None else _out(Q, max(topk, 1), lut.device)
    _check(load_library().rii_bench_scan_linear_half(index.handle, _dp(lut, torch.float32), Q, topk, _dp(ids, torch.int32),
                                                     _dp(dist, torch.float32), _stream()), "rii_bench_scan_linear_half")
    return ids, dist


def rii_bench_lds_reads(width: int, blocks: int, threads: int, iters: int, lds_bytes: int = 64 * 1024) -> int:
    """Measurement aid: launch the LDS read ceiling kernel on the current stream; returns the number of reads."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    _check(load_library().rii_bench_lds_reads(width, blocks, threads, iters, lds_bytes, _dp(sink), _stream()),
           "rii_bench_lds_reads")
    return blocks * threads * iters * {4: 16, 8: 8, 16: 4}[width]


def rii_index_set_scan_events(index: Index, start_event, stop_event):
    """Measurement aid: raw hipEvent_t handles (ints or None) recorded around the linear-scan kernel."""
    s = ctypes.c_void_p(start_event) if start_event else None
    e = ctypes.c_void_p(stop_event) if stop_event else None
    _check(load_library().rii_index_set_scan_events(index.handle, s, e), "rii_index_set_scan_events")
