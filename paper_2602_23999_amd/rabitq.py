"""Thin Python binding of librabitq_hip.so (argument marshalling only).

Every function has the name of the C entry point it calls (include/rabitq.h) without
the ``rabitq_`` prefix.  PyTorch is used for device memory and streams only: tensors are
allocated here, their ``data_ptr()`` and the current stream are handed to the library,
and every step of the search runs in the library's HIP kernels.  There is no fallback:
a missing library or a failing call raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librabitq_hip.so")
FLT_MAX = float(np.finfo(np.float32).max)
MAX_K = 128
QUERY_BITS = 4
TILE = 64

EXPORTS = [
    "rabitq_index_upload", "rabitq_index_build", "rabitq_index_export", "rabitq_index_free", "rabitq_search", "rabitq_search_noalloc", "rabitq_set_option", "rabitq_index_info",
    "rabitq_stage_ms", "rabitq_rotate", "rabitq_query_prep", "rabitq_qhat_stride", "rabitq_coarse_probe",
    "rabitq_probe_list_scratch_words", "rabitq_probe_select_variant", "rabitq_cand_capacity", "rabitq_build_probe_lists", "rabitq_seed_threshold", "rabitq_scan",
    "rabitq_merge", "rabitq_last_error",
]


class RabitqError(RuntimeError):
    pass


class _Desc(C.Structure):
    _fields_ = [("dim", C.c_int32), ("nlist", C.c_int32), ("n", C.c_int64), ("total_bits", C.c_int32),
                ("metric", C.c_int32), ("rotation", C.c_void_p), ("centroids", C.c_void_p),
                ("offsets", C.c_void_p), ("short_codes", C.c_void_p), ("short_factors", C.c_void_p),
                ("long_codes", C.c_void_p), ("long_factors", C.c_void_p), ("ids", C.c_void_p),
                ("mean", C.c_void_p)]


class _QueryRepr(C.Structure):
    _fields_ = [("planes", C.c_void_p), ("delta", C.c_void_p), ("sum_qhat", C.c_void_p), ("sum_q", C.c_void_p),
                ("sq_norm", C.c_void_p), ("qhat8", C.c_void_p), ("q_stage", C.c_void_p), ("lut", C.c_void_p)]


class _BuildParams(C.Structure):
    _fields_ = [("dim", C.c_int32), ("nlist", C.c_int32), ("n", C.c_int64), ("total_bits", C.c_int32),
                ("metric", C.c_int32), ("kmeans_iters", C.c_int32), ("train_size", C.c_int64),
                ("epsilon0", C.c_float), ("rotation", C.c_void_p), ("center", C.c_int32)]


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree shared library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RabitqError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.rabitq_last_error.restype = C.c_char_p
    lib.rabitq_last_error.argtypes = []
    lib.rabitq_index_upload.argtypes = [C.POINTER(_Desc), C.POINTER(vp), vp]
    lib.rabitq_index_build.argtypes = [C.POINTER(_BuildParams), vp, C.POINTER(vp), vp]
    lib.rabitq_index_export.argtypes = [vp] * 10
    lib.rabitq_index_free.argtypes = [vp]
    lib.rabitq_search.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    lib.rabitq_search_noalloc.argtypes = [vp, vp, i64, i32, i32, vp, vp, vp]
    lib.rabitq_set_option.argtypes = [vp, C.c_char_p, i64]
    lib.rabitq_index_info.argtypes = [vp, C.c_char_p]
    lib.rabitq_index_info.restype = i64
    lib.rabitq_stage_ms.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
    lib.rabitq_rotate.argtypes = [vp, vp, i64, vp, vp]
    lib.rabitq_query_prep.argtypes = [vp, vp, i64, C.POINTER(_QueryRepr), vp]
    lib.rabitq_qhat_stride.argtypes = [i32]
    lib.rabitq_qhat_stride.restype = i32
    lib.rabitq_coarse_probe.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, vp, vp]
    lib.rabitq_probe_list_scratch_words.argtypes = [i32, i64]
    lib.rabitq_probe_list_scratch_words.restype = i64
    lib.rabitq_cand_capacity.argtypes = [i32]
    lib.rabitq_probe_select_variant.argtypes = [i32, i32]
    lib.rabitq_probe_select_variant.restype = i32
    lib.rabitq_cand_capacity.restype = i32
    lib.rabitq_build_probe_lists.argtypes = [vp, vp, i64, i32, vp, vp, vp, vp]
    lib.rabitq_seed_threshold.argtypes = [vp, C.POINTER(_QueryRepr), vp, vp, vp, i64, i32, i32, vp, vp]
    lib.rabitq_scan.argtypes = [vp, C.POINTER(_QueryRepr), vp, vp, vp, vp, vp, i64, i32, i32, vp, vp, vp, vp, vp]
    lib.rabitq_merge.argtypes = [vp, vp, vp, i64, i32, i32, vp, vp, vp]
    for name in EXPORTS:
        if name not in ("rabitq_last_error", "rabitq_index_info", "rabitq_probe_list_scratch_words",
                        "rabitq_cand_capacity", "rabitq_qhat_stride", "rabitq_probe_select_variant"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int):
    if rc != 0:
        raise RabitqError(f"rabitq error {rc}: {load_library().rabitq_last_error().decode()}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> int:
    if not (t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise RabitqError(f"expected a contiguous CUDA tensor of {dtype}, got {t.dtype} on {t.device}")
    return t.data_ptr()


class Index:
    """An uploaded index.  ``arrays`` holds host numpy arrays in the layout of
    rabitq_index_desc (see include/rabitq.h)."""

    def __init__(self, *, dim, nlist, n, total_bits, metric, rotation, centroids, offsets, short_codes,
                 short_factors, ids, long_codes=None, long_factors=None, mean=None):
        lib = load_library()
        if not torch.cuda.is_available():
            raise RabitqError("no HIP device: the search path has no CPU fallback")

        def host(a, dt):
            return None if a is None else np.ascontiguousarray(a, dtype=dt)
        self._keep = dict(rotation=host(rotation, np.float32), centroids=host(centroids, np.float32),
                          offsets=host(offsets, np.int64), short_codes=host(short_codes, np.uint32),
                          short_factors=host(short_factors, np.float32), long_codes=host(long_codes, np.uint32),
                          long_factors=host(long_factors, np.float32), ids=host(ids, np.int32),
                          mean=host(mean, np.float32))
        k = self._keep
        if k["rotation"].size != dim * dim or k["centroids"].size != nlist * dim or k["offsets"].size != nlist + 1:
            raise RabitqError("rotation / centroids / offsets have the wrong size")
        if k["mean"] is not None and k["mean"].size != dim:
            raise RabitqError("mean must hold D elements")
        counts = np.diff(k["offsets"])
        n_tiles = int(((counts + TILE - 1) // TILE).sum())
        W = dim // 32
        F = 0 if total_bits == 1 else next(f for f in (2, 4, 8) if total_bits <= f)
        want = dict(short_codes=n_tiles * W * TILE, short_factors=n_tiles * 3 * TILE, ids=n_tiles * TILE)
        if total_bits > 1:
            want.update(long_codes=n_tiles * TILE * dim * F // 32, long_factors=n_tiles * TILE * 2)
        for name, sz in want.items():
            if k[name] is None or k[name].size != sz:
                raise RabitqError(f"{name} must hold {sz} elements")
        p = lambda a: None if a is None else a.ctypes.data
        desc = _Desc(dim, nlist, n, total_bits, {"l2": 0, "ip": 1}[metric], p(k["rotation"]), p(k["centroids"]),
                     p(k["offsets"]), p(k["short_codes"]), p(k["short_factors"]), p(k["long_codes"]),
                     p(k["long_factors"]), p(k["ids"]), p(k["mean"]))
        h = C.c_void_p()
        _check(lib.rabitq_index_upload(C.byref(desc), C.byref(h), _stream()))
        self._h = h
        self._keep = None
        self.dim, self.nlist, self.n, self.total_bits, self.metric = dim, nlist, n, total_bits, metric
        self.W = W

    @classmethod
    def build(cls, data: torch.Tensor, nlist: int, total_bits: int, rotation, metric: str = "l2",
              kmeans_iters: int = 10, train_size: int = 0, epsilon0: float = 1.9, center: bool = False) -> "Index":
        """rabitq_index_build: builds the index on the device from raw vectors `data` [n, D]
        (CUDA fp32) and a host rotation matrix [D, D]; `center` builds on the vectors minus
        their mean (L2 only)."""
        lib = load_library()
        n, dim = data.shape
        rot = np.ascontiguousarray(rotation, dtype=np.float32)
        if rot.shape != (dim, dim):
            raise RabitqError("rotation must be [D, D]")
        prm = _BuildParams(dim, nlist, n, total_bits, {"l2": 0, "ip": 1}[metric], kmeans_iters, train_size, epsilon0,
                           rot.ctypes.data, int(bool(center)))
        h = C.c_void_p()
        _check(lib.rabitq_index_build(C.byref(prm), _dev(data, torch.float32), C.byref(h), _stream()))
        self = cls.__new__(cls)
        self._h, self._keep = h, None
        self.dim, self.nlist, self.n, self.total_bits, self.metric, self.W = dim, nlist, n, total_bits, metric, dim // 32
        return self

    def export(self) -> dict:
        """rabitq_index_export: host numpy arrays in the layout of rabitq_index_desc."""
        lib = load_library()
        D, nlist, W = self.dim, self.nlist, self.W
        tiles, slots, F = self.index_info("n_tiles"), self.index_info("n_slots"), self.index_info("long_field_bits")
        out = dict(dim=D, nlist=nlist, n=self.n, total_bits=self.total_bits, metric=self.metric,
                   rotation=np.empty((D, D), np.float32), centroids=np.empty((nlist, D), np.float32),
                   offsets=np.empty(nlist + 1, np.int64), short_codes=np.empty(tiles * W * TILE, np.uint32),
                   short_factors=np.empty(tiles * 3 * TILE, np.float32), ids=np.empty(slots, np.int32),
                   long_codes=None, long_factors=None, mean=np.empty(D, np.float32))
        if self.total_bits > 1:
            out["long_codes"] = np.empty(slots * D * F // 32, np.uint32)
            out["long_factors"] = np.empty(slots * 2, np.float32)
        p = lambda a: None if a is None else a.ctypes.data
        _check(lib.rabitq_index_export(self._h, p(out["rotation"]), p(out["centroids"]), p(out["offsets"]),
                                       p(out["short_codes"]), p(out["short_factors"]), p(out["long_codes"]),
                                       p(out["long_factors"]), p(out["ids"]), p(out["mean"])))
        return out

    def save(self, path: str):
        """Writes the exported arrays to an .npz file (plain arrays, no pickled objects)."""
        out = self.export()
        np.savez(path, **{k: (np.asarray(v) if v is not None else np.zeros(0, np.uint32)) for k, v in out.items()})

    @classmethod
    def load(cls, path: str) -> "Index":
        """Uploads an index written by save()."""
        with np.load(path, allow_pickle=False) as z:
            d = {k: z[k] for k in z.files}
        scal = {k: int(d.pop(k)) for k in ("dim", "nlist", "n", "total_bits")}
        metric = str(d.pop("metric"))
        for k in ("long_codes", "long_factors"):
            if d[k].size == 0:
                d[k] = None
        return cls(metric=metric, **scal, **d)

    def close(self):
        if getattr(self, "_h", None):
            _check(load_library().rabitq_index_free(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- whole path -------------------------------------------------------------
    def search(self, queries: torch.Tensor, k: int, nprobe: int, out_ids=None, out_dists=None):
        nq = queries.shape[0]
        dev = queries.device
        if out_ids is None:
            out_ids = torch.empty((nq, k), dtype=torch.int64, device=dev)
        if out_dists is None:
            out_dists = torch.empty((nq, k), dtype=torch.float32, device=dev)
        _check(load_library().rabitq_search(self._h, _dev(queries, torch.float32), nq, k, nprobe,
                                            _dev(out_ids, torch.int64), _dev(out_dists, torch.float32), _stream()))
        return out_ids, out_dists

    def search_noalloc(self, queries: torch.Tensor, k: int, nprobe: int, out_ids: torch.Tensor, out_dists: torch.Tensor):
        """rabitq_search_noalloc: the caller supplies the outputs; nothing is allocated here or in the library."""
        _check(load_library().rabitq_search_noalloc(self._h, _dev(queries, torch.float32), queries.shape[0], k, nprobe,
                                                    _dev(out_ids, torch.int64), _dev(out_dists, torch.float32), _stream()))
        return out_ids, out_dists

    def set_option(self, name: str, value: int):
        _check(load_library().rabitq_set_option(self._h, name.encode(), value))

    def index_info(self, name: str) -> int:
        v = load_library().rabitq_index_info(self._h, name.encode())
        if v < 0:
            _check(int(v))
        return int(v)

    STAGES = ["rotate", "query_prep", "coarse_gemm", "probe_select", "list_build", "seed", "scan_setup", "scan",
              "merge", "scan_estimate"]

    def stage_ms(self):
        """Mean per-stage milliseconds over the searches recorded since set_option("profile", n)."""
        buf = (C.c_float * 10)()
        calls = C.c_int32(0)
        _check(load_library().rabitq_stage_ms(self._h, buf, C.byref(calls)))
        return dict(zip(self.STAGES, [float(x) for x in buf])), int(calls.value)

    # ---- stages -----------------------------------------------------------------
    def rotate(self, queries):
        out = torch.empty_like(queries)
        _check(load_library().rabitq_rotate(self._h, _dev(queries, torch.float32), queries.shape[0],
                                            _dev(out, torch.float32), _stream()))
        return out

    @staticmethod
    def _repr_struct(prep: dict) -> "_QueryRepr":
        return _QueryRepr(_dev(prep["planes"], torch.int32), _dev(prep["delta"], torch.float32),
                          _dev(prep["sum_qhat"], torch.int32), _dev(prep["sum_q"], torch.float32),
                          _dev(prep["sq_norm"], torch.float32), _dev(prep["qhat8"], torch.int8),
                          _dev(prep["q_stage"], torch.float32),
                          _dev(prep["lut"], torch.float16) if prep.get("lut") is not None else None)

    def query_prep(self, q_rot):
        """rabitq_query_prep: the per-query representation as a dict of device tensors."""
        nq, dev = q_rot.shape[0], q_rot.device
        stride = load_library().rabitq_qhat_stride(self.dim)
        prep = dict(planes=torch.empty((nq, QUERY_BITS, self.W), dtype=torch.int32, device=dev),
                    delta=torch.empty(nq, dtype=torch.float32, device=dev),
                    sum_qhat=torch.empty(nq, dtype=torch.int32, device=dev),
                    sum_q=torch.empty(nq, dtype=torch.float32, device=dev),
                    sq_norm=torch.empty(nq, dtype=torch.float32, device=dev),
                    qhat8=torch.empty((nq, stride), dtype=torch.int8, device=dev),
                    q_stage=torch.empty((nq, self.dim), dtype=torch.float32, device=dev),
                    lut=torch.empty((nq, self.dim // 4, 16), dtype=torch.float16, device=dev))
        r = self._repr_struct(prep)
        _check(load_library().rabitq_query_prep(self._h, _dev(q_rot, torch.float32), nq, C.byref(r), _stream()))
        return prep

    def coarse_probe(self, q_rot, sq_norm, nprobe):
        nq, dev = q_rot.shape[0], q_rot.device
        scores = torch.empty((nq, self.nlist), dtype=torch.float32, device=dev)
        ids = torch.empty((nq, nprobe), dtype=torch.int32, device=dev)
        G = torch.empty((nq, nprobe), dtype=torch.float32, device=dev)
        E = torch.empty((nq, nprobe), dtype=torch.float32, device=dev)
        _check(load_library().rabitq_coarse_probe(self._h, _dev(q_rot, torch.float32), _dev(sq_norm, torch.float32),
                                                  nq, nprobe, scores.data_ptr(), ids.data_ptr(), G.data_ptr(),
                                                  E.data_ptr(), _stream()))
        return dict(probe_ids=ids, probe_G=G, probe_E=E, scores=scores)

    def build_probe_lists(self, probe_ids):
        nq, nprobe = probe_ids.shape
        dev = probe_ids.device
        words = load_library().rabitq_probe_list_scratch_words(self.nlist, nq)
        scratch = torch.empty(max(int(words), 1), dtype=torch.int32, device=dev)
        pair_off = torch.empty(self.nlist + 1, dtype=torch.int32, device=dev)
        pair_ids = torch.empty(nq * nprobe, dtype=torch.int32, device=dev)
        _check(load_library().rabitq_build_probe_lists(self._h, _dev(probe_ids, torch.int32), nq, nprobe,
                                                       pair_off.data_ptr(), pair_ids.data_ptr(), scratch.data_ptr(),
                                                       _stream()))
        return pair_off, pair_ids

    def seed_threshold(self, prep, probes, k):
        nq, nprobe = probes["probe_ids"].shape
        tau = torch.empty(nq, dtype=torch.float32, device=probes["probe_ids"].device)
        r = self._repr_struct(prep)
        _check(load_library().rabitq_seed_threshold(
            self._h, C.byref(r), _dev(probes["probe_ids"], torch.int32), _dev(probes["probe_G"], torch.float32),
            _dev(probes["probe_E"], torch.float32), nq, k, nprobe, tau.data_ptr(), _stream()))
        return tau

    def scan(self, prep, probes, pair_off, pair_ids, tau, k, dbg_off=None):
        nq, nprobe = probes["probe_G"].shape
        dev = tau.device
        cap = load_library().rabitq_cand_capacity(k)
        if cap < 0:
            _check(cap)
        cand_keys = torch.empty((nq * nprobe, cap), dtype=torch.int64, device=dev)
        cand_cnt = torch.empty(nq * nprobe, dtype=torch.int32, device=dev)
        dbg_ip = None
        if dbg_off is not None:
            dbg_ip = torch.zeros(int(dbg_off[-1].item()), dtype=torch.int32, device=dev)
        r = self._repr_struct(prep)
        _check(load_library().rabitq_scan(
            self._h, C.byref(r), _dev(probes["probe_G"], torch.float32), _dev(probes["probe_E"], torch.float32),
            _dev(pair_off, torch.int32), _dev(pair_ids, torch.int32), _dev(tau, torch.float32), nq, k, nprobe,
            cand_keys.data_ptr(), cand_cnt.data_ptr(), None if dbg_ip is None else dbg_ip.data_ptr(),
            None if dbg_off is None else _dev(dbg_off, torch.int64), _stream()))
        return cand_keys, cand_cnt, dbg_ip

    def merge(self, cand_keys, cand_cnt, nq, k, nprobe):
        dev = cand_keys.device
        out_ids = torch.empty((nq, k), dtype=torch.int64, device=dev)
        out_d = torch.empty((nq, k), dtype=torch.float32, device=dev)
        _check(load_library().rabitq_merge(self._h, _dev(cand_keys, torch.int64), _dev(cand_cnt, torch.int32), nq, k,
                                           nprobe, out_ids.data_ptr(), out_d.data_ptr(), _stream()))
        return out_ids, out_d


def index_from_arrays(meta: dict, dev: dict) -> Index:
    """Uploads an index given its scalar description and device-layout arrays
    (keys as in rabitq_index_desc)."""
    return Index(dim=meta["dim"], nlist=meta["nlist"], n=meta["n"], total_bits=meta["total_bits"],
                 metric=meta["metric"], rotation=meta["P"], centroids=meta["centroids_rot"], offsets=meta["offsets"],
                 short_codes=dev["short_codes"], short_factors=dev["short_factors"], ids=dev["ids"],
                 long_codes=dev["long_codes"], long_factors=dev["long_factors"], mean=meta.get("mean"))
