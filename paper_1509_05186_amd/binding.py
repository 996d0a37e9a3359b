"""ctypes binding of include/etf.h.  Method names are the C entry points without the prefix."""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

ETF_MAX_M = 16
ETF_MAX_TOPK = 1024
ETF_MODE_FLAT, ETF_MODE_TREE, ETF_MODE_FOREST = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "lib", "libetf.so")
_lib = None

EXPORTS = [
    "etf_create", "etf_destroy", "etf_set_stream", "etf_strerror", "etf_last_error", "etf_set_option",
    "etf_pq_train", "etf_pq_set_codebooks", "etf_pq_get_codebooks", "etf_pq_encode",
    "etf_pq_set_rotation", "etf_pq_get_rotation", "etf_rotate", "etf_rotate_workspace_bytes", "etf_rotate_device", "etf_opq_train",
    "etf_index_build", "etf_index_set_leaf_term", "etf_index_set_leaf_bytes", "etf_index_set_chunk_order", "etf_suggest_chunk_order", "etf_suggest_partition", "etf_index_stats", "etf_index_device_bytes", "etf_index_upload",
    "etf_index_layout", "etf_index_export",
    "etf_encode_workspace_bytes", "etf_pq_encode_device",
    "etf_index_build_device_bytes", "etf_index_build_device",
    "etf_workspace_bytes", "etf_lut_build", "etf_adc", "etf_search", "etf_last_fallback_count",
    "etf_static_scratch_bytes", "etf_search_static",
    "etf_profile_enable", "etf_profile_read", "etf_probe_bandwidth",
    "etf_ivf_set_coarse", "etf_ivf_assign_workspace_bytes", "etf_ivf_assign_device", "etf_ivf_build", "etf_ivf_stats",
    "etf_ivf_device_bytes", "etf_ivf_upload", "etf_ivf_workspace_bytes", "etf_ivf_search",
]
ETF_PROBE_READ, ETF_PROBE_WRITE, ETF_PROBE_COPY, ETF_PROBE_ROWS, ETF_PROBE_LDS, ETF_PROBE_LDS_SCATTER = 0, 1, 2, 3, 4, 5
ETF_PROBE_VALU_F32, ETF_PROBE_VALU_ADD3, ETF_PROBE_VALU_PK16, ETF_PROBE_MFMA_F32 = 6, 7, 8, 9
KERNEL_CLASSES = ["lut", "level", "leaf", "flat", "reduce", "tau", "select", "exact", "sample", "lds", "encode",
                  "ivf_coarse", "ivf_scan", "lds16"]


class EtfStats(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int32), ("K", ctypes.c_int32), ("T", ctypes.c_int32),
        ("chunk_begin", ctypes.c_int32 * (ETF_MAX_M + 1)),
        ("N", ctypes.c_int64), ("n_distinct", ctypes.c_int64), ("max_dup", ctypes.c_int64),
        ("nI", (ctypes.c_int64 * ETF_MAX_M) * ETF_MAX_M),
        ("nL", (ctypes.c_int64 * ETF_MAX_M) * ETF_MAX_M),
        ("L1", ctypes.c_int64 * ETF_MAX_M), ("L2", ctypes.c_int64 * ETF_MAX_M),
        ("sumP", ctypes.c_int64 * ETF_MAX_M), ("lookups", ctypes.c_int64 * ETF_MAX_M),
        ("paper_bytes", ctypes.c_int64 * ETF_MAX_M),
        ("device_bytes", ctypes.c_int64),
        ("chunk_order", ctypes.c_int32 * ETF_MAX_M),
    ]

    def as_dict(self) -> dict:
        T = self.T
        cb = [int(self.chunk_begin[t]) for t in range(T + 1)]
        trees = []
        for t in range(T):
            D = cb[t + 1] - cb[t]
            trees.append({
                "chunks": (cb[t], cb[t + 1]), "D": D,
                "nI": [int(self.nI[t][l]) for l in range(D)], "nL": [int(self.nL[t][l]) for l in range(D)],
                "L1": int(self.L1[t]), "L2": int(self.L2[t]), "sumP": int(self.sumP[t]),
                "lookups": int(self.lookups[t]), "paper_bytes": int(self.paper_bytes[t]),
            })
        return {"M": self.M, "K": self.K, "T": T, "N": int(self.N), "n_distinct": int(self.n_distinct),
                "max_dup": int(self.max_dup), "device_bytes": int(self.device_bytes), "trees": trees,
                "chunk_order": [int(self.chunk_order[j]) for j in range(self.M)]}


class EtfIvfStats(ctypes.Structure):
    _fields_ = [("cells", ctypes.c_int32), ("N", ctypes.c_int64), ("entries", ctypes.c_int64), ("max_list", ctypes.c_int64),
                ("max_dup", ctypes.c_int64), ("tree_lookups", ctypes.c_int64), ("flat_lookups", ctypes.c_int64),
                ("device_bytes", ctypes.c_int64)]

    def as_dict(self) -> dict:
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


_Grid64 = (ctypes.c_int64 * ETF_MAX_M) * ETF_MAX_M
_Grid32 = (ctypes.c_int32 * ETF_MAX_M) * ETF_MAX_M


class EtfLayout(ctypes.Structure):
    _fields_ = [
        ("total", ctypes.c_int64),
        ("codebooks", ctypes.c_int64), ("codes", ctypes.c_int64), ("ids_in", ctypes.c_int64),
        ("ids_sorted", ctypes.c_int64), ("ebegin", ctypes.c_int64), ("enc_of_pos", ctypes.c_int64),
        ("ecodes", ctypes.c_int64), ("sample_enc", ctypes.c_int64), ("sample_pos", ctypes.c_int64),
        ("n_sample_enc", ctypes.c_int64), ("n_sample_pos", ctypes.c_int64),
        ("leaf_of", ctypes.c_int64 * ETF_MAX_M),
        ("icode", _Grid64), ("iparent", _Grid64), ("lcodes", _Grid64), ("lparent", _Grid64), ("lrow", _Grid64),
        ("lstride", _Grid32),
        ("rec0", ctypes.c_int64), ("rec0_stride", ctypes.c_int32),
        ("trec", ctypes.c_int64 * ETF_MAX_M), ("trec_stride", ctypes.c_int32 * ETF_MAX_M),
        ("cb_centered", ctypes.c_int64), ("cb_norm", ctypes.c_int64), ("cb_mean", ctypes.c_int64),
        ("sample_enc_codes", ctypes.c_int64), ("sample_pos_codes", ctypes.c_int64),
        ("cb_row", ctypes.c_int32),
        ("eterm", ctypes.c_int64), ("pterm", ctypes.c_int64),
    ]


class EtfError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("etf error %d: %s" % (code, message))
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads lib/libetf.so.  Raises if it has not been built: there is no other implementation."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("HIP library %s is missing: run `python -m paper_1509_05186_amd.build`" % _LIB_PATH)
    try:
        # torch first: the library must bind to the HIP runtime torch brings along (whichever of the two is
        # loaded first decides), or its calls see no device in a process where torch holds the GPU
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_LIB_PATH)
    P, I, L = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    sig = {
        "etf_create": (I, [ctypes.POINTER(P), I, P]),
        "etf_destroy": (None, [P]),
        "etf_set_stream": (I, [P, P]),
        "etf_strerror": (ctypes.c_char_p, [I]),
        "etf_last_error": (ctypes.c_char_p, [P]),
        "etf_set_option": (I, [P, ctypes.c_char_p, L]),
        "etf_pq_train": (I, [P, P, L, I, I, I, I, ctypes.c_uint64]),
        "etf_pq_set_codebooks": (I, [P, P, I, I, I]),
        "etf_pq_get_codebooks": (I, [P, P]),
        "etf_pq_encode": (I, [P, P, L, P]),
        "etf_pq_set_rotation": (I, [P, P, I]),
        "etf_pq_get_rotation": (I, [P, P]),
        "etf_rotate": (I, [P, P, L, P]),
        "etf_rotate_workspace_bytes": (L, [P]),
        "etf_rotate_device": (I, [P, P, L, P, P, L]),
        "etf_opq_train": (I, [P, P, L, I, I, I, I, I, ctypes.c_uint64]),
        "etf_index_build": (I, [P, P, L, P, I, P]),
        "etf_index_set_chunk_order": (I, [P, P]),
        "etf_index_set_leaf_term": (I, [P, P, L]),
        "etf_index_set_leaf_bytes": (I, [P, P, L, ctypes.c_float, ctypes.c_float]),
        "etf_suggest_chunk_order": (I, [P, P, L, I, P, P, ctypes.POINTER(L), ctypes.POINTER(L)]),
        "etf_suggest_partition": (I, [P, P, L, I, P, P, ctypes.POINTER(L), ctypes.POINTER(L)]),
        "etf_index_stats": (I, [P, ctypes.POINTER(EtfStats)]),
        "etf_index_device_bytes": (L, [P]),
        "etf_index_upload": (I, [P, P, L]),
        "etf_index_layout": (I, [P, ctypes.POINTER(EtfLayout)]),
        "etf_index_export": (I, [P, P, L]),
        "etf_encode_workspace_bytes": (L, [P]),
        "etf_pq_encode_device": (I, [P, P, L, P, P, L]),
        "etf_index_build_device_bytes": (I, [P, L, I, P, ctypes.POINTER(L), ctypes.POINTER(L)]),
        "etf_index_build_device": (I, [P, P, L, P, I, P, P, L, P, L]),
        "etf_workspace_bytes": (L, [P, L, I, I]),
        "etf_lut_build": (I, [P, P, L, P]),
        "etf_adc": (I, [P, P, L, I, P, P, L]),
        "etf_search": (I, [P, P, L, I, I, P, P, P, L]),
        "etf_last_fallback_count": (I, [P, ctypes.POINTER(L)]),
        "etf_static_scratch_bytes": (L, []),
        "etf_search_static": (I, [P, P, L, I, I, P, P]),
        "etf_profile_enable": (I, [P, I]),
        "etf_profile_read": (I, [P, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(L)]),
        "etf_probe_bandwidth": (I, [P, I, P, P, L]),
        "etf_ivf_set_coarse": (I, [P, P, I]),
        "etf_ivf_assign_workspace_bytes": (L, [P, L]),
        "etf_ivf_assign_device": (I, [P, P, L, P, P, P, L]),
        "etf_ivf_build": (I, [P, P, P, L, P]),
        "etf_ivf_stats": (I, [P, ctypes.POINTER(EtfIvfStats)]),
        "etf_ivf_device_bytes": (L, [P]),
        "etf_ivf_upload": (I, [P, P, L]),
        "etf_ivf_workspace_bytes": (L, [P, L, I, I]),
        "etf_ivf_search": (I, [P, P, L, I, I, P, P, P, L]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    _lib = lib
    return lib


def _host(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dev(t) -> int:
    """Device pointer of a torch tensor (contiguous, on the GPU)."""
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous GPU tensor")
    return t.data_ptr()


class Context:
    """One etf_ctx.  device=None makes a host-only context (train / encode / build / stats)."""

    def __init__(self, device: Optional[int] = 0, stream: Optional[int] = None):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        rc = self._lib.etf_create(ctypes.byref(self._h), -1 if device is None else int(device), stream)
        if rc != 0:
            raise EtfError(rc, self._lib.etf_strerror(rc).decode())
        self._keep = {}     # device buffers the library refers to (index image)

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._lib.etf_destroy(self._h)
            self._h = ctypes.c_void_p()
            self._keep = {}

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ck(self, rc: int):
        if rc < 0:
            raise EtfError(int(rc), self._lib.etf_last_error(self._h).decode())
        return rc

    # ---- context
    def set_stream(self, stream: Optional[int]):
        self._ck(self._lib.etf_set_stream(self._h, stream))

    def set_option(self, name: str, value: int):
        self._ck(self._lib.etf_set_option(self._h, name.encode(), int(value)))

    # ---- product quantiser (host)
    def pq_train(self, x: np.ndarray, M: int, K: int, iters: int, seed: int):
        x = np.ascontiguousarray(x, dtype=np.float32)
        self._ck(self._lib.etf_pq_train(self._h, _host(x), x.shape[0], x.shape[1], M, K, iters, seed))
        self._shape = (x.shape[1], M, K)

    def pq_set_codebooks(self, cb: np.ndarray):
        cb = np.ascontiguousarray(cb, dtype=np.float32)
        M, K, ds = cb.shape
        self._ck(self._lib.etf_pq_set_codebooks(self._h, _host(cb), M * ds, M, K))
        self._shape = (M * ds, M, K)

    def pq_set_rotation(self, R: Optional[np.ndarray]):
        """R: [d][d] float32 (the quantiser's space is y = R x), or None to clear."""
        if R is None:
            self._ck(self._lib.etf_pq_set_rotation(self._h, None, 0))
            self._rot_d = 0
            return
        R = np.ascontiguousarray(R, dtype=np.float32)
        if R.ndim != 2 or R.shape[0] != R.shape[1]:
            raise ValueError("expected a square matrix")
        self._ck(self._lib.etf_pq_set_rotation(self._h, _host(R), R.shape[0]))
        self._rot_d = R.shape[0]

    def pq_get_rotation(self) -> np.ndarray:
        d = getattr(self, "_rot_d", 0)
        R = np.zeros((d, d), dtype=np.float32)
        self._ck(self._lib.etf_pq_get_rotation(self._h, _host(R) if d else None))
        return R

    def rotate(self, x: np.ndarray) -> np.ndarray:
        """Host: [n][d] float32 -> R x, float32."""
        x = np.ascontiguousarray(x, dtype=np.float32)
        out = np.empty_like(x)
        if x.ndim != 2 or x.shape[1] != getattr(self, "_rot_d", 0):
            raise ValueError("expected [n][%d] vectors" % getattr(self, "_rot_d", 0))
        self._ck(self._lib.etf_rotate(self._h, _host(x) if len(x) else None, x.shape[0], _host(out) if len(x) else None))
        return out

    def rotate_workspace_bytes(self) -> int:
        return self._ck(self._lib.etf_rotate_workspace_bytes(self._h))

    def rotate_device(self, x, out=None, ws=None):
        """x: float32 device tensor [n][d]; returns R x as a float32 device tensor."""
        import torch
        d = getattr(self, "_rot_d", 0)
        if x.dim() != 2 or x.shape[1] != d or x.dtype != torch.float32 or not x.is_contiguous():
            raise ValueError("expected a contiguous float32 tensor [n][%d]" % d)
        n = x.shape[0]
        if out is None:
            out = torch.empty_like(x)
        if ws is None:
            ws = torch.empty(self.rotate_workspace_bytes() + 256, dtype=torch.uint8, device=x.device)
        p, nb = self._ws(ws)
        self._ck(self._lib.etf_rotate_device(self._h, _dev(x) if n else None, n, _dev(out) if n else None, p, nb))
        return out

    def opq_train(self, x: np.ndarray, M: int, K: int, iters: int, rounds: int, seed: int):
        x = np.ascontiguousarray(x, dtype=np.float32)
        self._ck(self._lib.etf_opq_train(self._h, _host(x), x.shape[0], x.shape[1], M, K, iters, rounds, seed))
        self._shape = (x.shape[1], M, K)
        self._rot_d = x.shape[1]

    def pq_get_codebooks(self) -> np.ndarray:
        d, M, K = self._shape
        cb = np.zeros((M, K, d // M), dtype=np.float32)
        self._ck(self._lib.etf_pq_get_codebooks(self._h, _host(cb)))
        return cb

    def pq_encode(self, x: np.ndarray) -> np.ndarray:
        x = np.ascontiguousarray(x, dtype=np.float32)
        d, M, K = self._shape
        if x.ndim != 2 or x.shape[1] != d:
            raise ValueError("expected [n][%d] vectors" % d)
        codes = np.zeros((x.shape[0], M), dtype=np.uint8)
        self._ck(self._lib.etf_pq_encode(self._h, _host(x), x.shape[0], _host(codes)))
        return codes

    # ---- index (host)
    def index_build(self, codes: np.ndarray, ids: Optional[np.ndarray] = None, T: int = 1,
                    chunk_begin: Optional[Sequence[int]] = None):
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        d, M, K = self._shape
        if codes.ndim != 2 or codes.shape[1] != M:
            raise ValueError("expected [N][%d] codes" % M)
        ids_a = None if ids is None else np.ascontiguousarray(ids, dtype=np.int32)
        cb = None if chunk_begin is None else np.ascontiguousarray(chunk_begin, dtype=np.int32)
        if cb is not None and cb.shape != (T + 1,):
            raise ValueError("chunk_begin must have T+1 entries")
        self._ck(self._lib.etf_index_build(self._h, _host(codes), codes.shape[0], _host(ids_a), T, _host(cb)))
        self._N = codes.shape[0]

    def index_set_leaf_term(self, term: Optional[np.ndarray]):
        """Additive float32 term per vector for the next index_build (None clears a pending one)."""
        t = None if term is None else np.ascontiguousarray(term, dtype=np.float32)
        self._ck(self._lib.etf_index_set_leaf_term(self._h, _host(t), 0 if t is None else t.shape[0]))

    def index_set_leaf_bytes(self, b: Optional[np.ndarray], scale: float, offset: float):
        """One byte per vector: the next index_build attaches offset + scale * b[n]."""
        a = None if b is None else np.ascontiguousarray(b, dtype=np.uint8)
        self._ck(self._lib.etf_index_set_leaf_bytes(self._h, _host(a), 0 if a is None else a.shape[0], scale, offset))

    def index_set_chunk_order(self, order: Optional[Sequence[int]]):
        """Chunk order of the next index build (a permutation of 0..M-1; None = as given)."""
        o = None if order is None else np.ascontiguousarray(order, dtype=np.int32)
        if o is not None and o.shape != (self._shape[1],):
            raise ValueError("order must have M entries")
        self._ck(self._lib.etf_index_set_chunk_order(self._h, _host(o)))

    def suggest_chunk_order(self, codes: np.ndarray, T: int = 1, chunk_begin: Optional[Sequence[int]] = None):
        """(order, lookups in the given order, lookups in the suggested order) for host codes [N][M]."""
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        M = self._shape[1]
        if codes.ndim != 2 or codes.shape[1] != M:
            raise ValueError("expected [N][%d] codes" % M)
        cb = None if chunk_begin is None else np.ascontiguousarray(chunk_begin, dtype=np.int32)
        if cb is not None and cb.shape != (T + 1,):
            raise ValueError("chunk_begin must have T+1 entries")
        order = np.zeros(M, dtype=np.int32)
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        self._ck(self._lib.etf_suggest_chunk_order(self._h, _host(codes), codes.shape[0], T, _host(cb), _host(order),
                                                   ctypes.byref(a), ctypes.byref(b)))
        return order, int(a.value), int(b.value)

    def suggest_partition(self, codes: np.ndarray, T: int):
        """(chunk_begin, order, lookups with the equal cut, lookups with the suggested cut) for host codes [N][M]."""
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        M = self._shape[1]
        if codes.ndim != 2 or codes.shape[1] != M:
            raise ValueError("expected [N][%d] codes" % M)
        cb = np.zeros(T + 1, dtype=np.int32)
        order = np.zeros(M, dtype=np.int32)
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        self._ck(self._lib.etf_suggest_partition(self._h, _host(codes), codes.shape[0], T, _host(cb), _host(order),
                                                 ctypes.byref(a), ctypes.byref(b)))
        return cb, order, int(a.value), int(b.value)

    def index_stats(self) -> dict:
        st = EtfStats()
        self._ck(self._lib.etf_index_stats(self._h, ctypes.byref(st)))
        return st.as_dict()

    def index_device_bytes(self) -> int:
        return self._ck(self._lib.etf_index_device_bytes(self._h))

    def index_layout(self) -> EtfLayout:
        lay = EtfLayout()
        self._ck(self._lib.etf_index_layout(self._h, ctypes.byref(lay)))
        return lay

    def index_export(self) -> np.ndarray:
        """The device image as a host byte array (what index_upload copies to the GPU)."""
        buf = np.zeros(self.index_device_bytes(), dtype=np.uint8)
        self._ck(self._lib.etf_index_export(self._h, _host(buf), buf.size))
        return buf

    def index_upload(self, dev_buf=None):
        """Uploads the index into dev_buf (uint8 GPU tensor); allocates one with torch if None."""
        import torch
        n = self.index_device_bytes()
        if dev_buf is None:
            dev_buf = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
        off = (-dev_buf.data_ptr()) % 256
        self._ck(self._lib.etf_index_upload(self._h, dev_buf.data_ptr() + off, dev_buf.numel() - off))
        self._keep["index"] = dev_buf
        return dev_buf

    # ---- device
    def workspace_bytes(self, Q: int, k: int, mode: int) -> int:
        return self._ck(self._lib.etf_workspace_bytes(self._h, Q, k, mode))

    def alloc_workspace(self, Q: int, k: int, mode: int):
        import torch
        n = self.workspace_bytes(Q, k, mode)
        return torch.empty(n + 256, dtype=torch.uint8, device="cuda")

    @staticmethod
    def _ws(ws):
        off = (-ws.data_ptr()) % 256
        return ws.data_ptr() + off, ws.numel() - off

    def encode_workspace_bytes(self) -> int:
        return self._ck(self._lib.etf_encode_workspace_bytes(self._h))

    def pq_encode_device(self, x, codes=None, ws=None):
        """x: float32 device tensor [n][d]; returns uint8 device tensor [n][M]."""
        import torch
        d, M, K = self._shape
        if x.dim() != 2 or x.shape[1] != d or x.dtype != torch.float32 or not x.is_contiguous():
            raise ValueError("expected a contiguous float32 tensor [n][%d]" % d)
        n = x.shape[0]
        if codes is None:
            codes = torch.empty((n, M), dtype=torch.uint8, device=x.device)
        if ws is None:
            ws = torch.empty(self.encode_workspace_bytes() + 256, dtype=torch.uint8, device=x.device)
        p, nb = self._ws(ws)
        self._ck(self._lib.etf_pq_encode_device(self._h, _dev(x) if n else None, n, _dev(codes) if n else None, p, nb))
        return codes

    def index_build_device_bytes(self, N: int, T: int = 1, chunk_begin: Optional[Sequence[int]] = None):
        """(image bytes that always suffice, workspace bytes) of a device-side build of N vectors."""
        a, b = ctypes.c_int64(0), ctypes.c_int64(0)
        cb = None if chunk_begin is None else np.ascontiguousarray(chunk_begin, dtype=np.int32)
        if cb is not None and cb.shape != (T + 1,):
            raise ValueError("chunk_begin must have T+1 entries")
        self._ck(self._lib.etf_index_build_device_bytes(self._h, N, T, _host(cb), ctypes.byref(a), ctypes.byref(b)))
        return int(a.value), int(b.value)

    def index_build_device(self, codes, ids=None, T: int = 1, chunk_begin: Optional[Sequence[int]] = None,
                           image=None, ws=None):
        """codes: uint8 device tensor [N][M]; ids: int32 device tensor [N] or None.  Returns the image tensor."""
        import torch
        d, M, K = self._shape
        if codes.dim() != 2 or codes.shape[1] != M or codes.dtype != torch.uint8 or not codes.is_contiguous():
            raise ValueError("expected a contiguous uint8 tensor [N][%d]" % M)
        N = codes.shape[0]
        if ids is not None and (ids.dtype != torch.int32 or ids.shape != (N,) or not ids.is_contiguous()):
            raise ValueError("expected a contiguous int32 tensor [N]")
        cb = None if chunk_begin is None else np.ascontiguousarray(chunk_begin, dtype=np.int32)
        if cb is not None and cb.shape != (T + 1,):
            raise ValueError("chunk_begin must have T+1 entries")
        nimg, nws = self.index_build_device_bytes(N, T, chunk_begin)
        if image is None:
            image = torch.empty(nimg + 256, dtype=torch.uint8, device=codes.device)
        if ws is None:
            ws = torch.empty(nws + 256, dtype=torch.uint8, device=codes.device)
        pi, ni = self._ws(image)
        pw, nw = self._ws(ws)
        self._ck(self._lib.etf_index_build_device(self._h, _dev(codes), N, None if ids is None else _dev(ids), T,
                                                  _host(cb), pi, ni, pw, nw))
        self._keep["index"] = image
        self._N = N
        return image

    def lut_build(self, queries, lut=None):
        import torch
        d, M, K = self._shape
        Q = queries.shape[0]
        if lut is None:
            lut = torch.empty((Q, M, K), dtype=torch.float32, device=queries.device)
        self._ck(self._lib.etf_lut_build(self._h, _dev(queries), Q, _dev(lut)))
        return lut

    def adc(self, queries, mode: int, dist=None, ws=None):
        import torch
        Q = queries.shape[0]
        if dist is None:
            dist = torch.empty((Q, self._N), dtype=torch.float32, device=queries.device)
        if ws is None:
            ws = self.alloc_workspace(Q, 0, mode)
        p, n = self._ws(ws)
        self._ck(self._lib.etf_adc(self._h, _dev(queries), Q, mode, _dev(dist), p, n))
        return dist

    def search(self, queries, k: int, mode: int, out_ids=None, out_dist=None, ws=None):
        import torch
        Q = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((Q, k), dtype=torch.int32, device=queries.device)
        if out_dist is None:
            out_dist = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
        if ws is None:
            ws = self.alloc_workspace(Q, k, mode)
        p, n = self._ws(ws)
        self._ck(self._lib.etf_search(self._h, _dev(queries), Q, k, mode, _dev(out_ids), _dev(out_dist), p, n))
        return out_ids, out_dist

    def search_static(self, queries, k: int, mode: int, out_ids, out_dist):
        """etf_search_static: the caller passes inputs and outputs only; nothing is allocated by the call."""
        self._ck(self._lib.etf_search_static(self._h, _dev(queries), queries.shape[0], k, mode, _dev(out_ids), _dev(out_dist)))
        return out_ids, out_dist

    def last_fallback_count(self) -> int:
        v = ctypes.c_int64(0)
        self._ck(self._lib.etf_last_fallback_count(self._h, ctypes.byref(v)))
        return int(v.value)

    # ---- IVFADC
    def ivf_set_coarse(self, centroids: np.ndarray):
        c = np.ascontiguousarray(centroids, dtype=np.float32)
        if c.ndim != 2 or c.shape[1] != self._shape[0]:
            raise ValueError("expected [cells][%d] centroids" % self._shape[0])
        self._ck(self._lib.etf_ivf_set_coarse(self._h, _host(c), c.shape[0]))

    def ivf_assign_device(self, x, ws=None):
        """x: float32 device tensor [n][d]; returns (cells int32 [n], codes uint8 [n][M]) device tensors."""
        import torch
        d, M, K = self._shape
        if x.dim() != 2 or x.shape[1] != d or x.dtype != torch.float32 or not x.is_contiguous():
            raise ValueError("expected a contiguous float32 tensor [n][%d]" % d)
        n = x.shape[0]
        cells = torch.empty((n,), dtype=torch.int32, device=x.device)
        codes = torch.empty((n, M), dtype=torch.uint8, device=x.device)
        if ws is None:
            ws = torch.empty(self._ck(self._lib.etf_ivf_assign_workspace_bytes(self._h, n)) + 256, dtype=torch.uint8, device=x.device)
        p, nb = self._ws(ws)
        self._ck(self._lib.etf_ivf_assign_device(self._h, _dev(x) if n else None, n, _dev(cells) if n else None,
                                                 _dev(codes) if n else None, p, nb))
        return cells, codes

    def ivf_build(self, cells: np.ndarray, codes: np.ndarray, ids: Optional[np.ndarray] = None):
        cells = np.ascontiguousarray(cells, dtype=np.int32)
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        if codes.ndim != 2 or codes.shape[1] != self._shape[1] or cells.shape != (codes.shape[0],):
            raise ValueError("expected cells [N] and codes [N][%d]" % self._shape[1])
        ids_a = None if ids is None else np.ascontiguousarray(ids, dtype=np.int32)
        self._ck(self._lib.etf_ivf_build(self._h, _host(cells), _host(codes), codes.shape[0], _host(ids_a)))

    def ivf_stats(self) -> dict:
        st = EtfIvfStats()
        self._ck(self._lib.etf_ivf_stats(self._h, ctypes.byref(st)))
        return st.as_dict()

    def ivf_upload(self, dev_buf=None):
        import torch
        n = self._ck(self._lib.etf_ivf_device_bytes(self._h))
        if dev_buf is None:
            dev_buf = torch.empty(n + 256, dtype=torch.uint8, device="cuda")
        off = (-dev_buf.data_ptr()) % 256
        self._ck(self._lib.etf_ivf_upload(self._h, dev_buf.data_ptr() + off, dev_buf.numel() - off))
        self._keep["ivf"] = dev_buf
        return dev_buf

    def ivf_workspace_bytes(self, Q: int, k: int, w: int) -> int:
        return self._ck(self._lib.etf_ivf_workspace_bytes(self._h, Q, k, w))

    def ivf_search(self, queries, k: int, w: int, out_ids=None, out_dist=None, ws=None):
        import torch
        Q = queries.shape[0]
        if out_ids is None:
            out_ids = torch.empty((Q, k), dtype=torch.int32, device=queries.device)
        if out_dist is None:
            out_dist = torch.empty((Q, k), dtype=torch.float32, device=queries.device)
        if ws is None:
            ws = torch.empty(self.ivf_workspace_bytes(Q, k, w) + 256, dtype=torch.uint8, device=queries.device)
        p, n = self._ws(ws)
        self._ck(self._lib.etf_ivf_search(self._h, _dev(queries), Q, k, w, _dev(out_ids), _dev(out_dist), p, n))
        return out_ids, out_dist

    def probe_bandwidth(self, kind: int, a, b, nbytes: int):
        """One launch of a streaming probe kernel over the uint8 device tensors a and b (256-byte aligned)."""
        self._ck(self._lib.etf_probe_bandwidth(self._h, kind, _dev(a), _dev(b), nbytes))

    def profile_enable(self, on: bool):
        self._ck(self._lib.etf_profile_enable(self._h, 1 if on else 0))

    def profile_read(self) -> dict:
        """{kernel class: (milliseconds, launches)} since the last read."""
        n = len(KERNEL_CLASSES)
        ms = (ctypes.c_double * n)()
        cnt = (ctypes.c_int64 * n)()
        self._ck(self._lib.etf_profile_read(self._h, ms, cnt))
        return {name: (float(ms[i]), int(cnt[i])) for i, name in enumerate(KERNEL_CLASSES)}
