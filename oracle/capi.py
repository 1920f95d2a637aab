"""ctypes wrapper of the compiled C oracle (test infrastructure only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < max(os.path.getmtime(x) for x in _build.SRCS):
            path = _build.build()
        L = C.CDLL(path)
        i64p, i32p = C.POINTER(C.c_int64), C.POINTER(C.c_int32)
        L.oob_oracle_create.restype = C.c_void_p
        L.oob_oracle_create.argtypes = [i64p, i64p, i64p, i64p, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_int64, C.c_int]
        L.oob_oracle_destroy.argtypes = [C.c_void_p]
        L.oob_oracle_destroy.restype = None
        for name in ("smax", "ndelta"):
            getattr(L, f"oob_oracle_{name}").argtypes = [C.c_void_p]
            getattr(L, f"oob_oracle_{name}").restype = C.c_int
        for name in ("states", "candidates", "evaluated"):
            getattr(L, f"oob_oracle_{name}").argtypes = [C.c_void_p]
            getattr(L, f"oob_oracle_{name}").restype = C.c_int64
        L.oob_oracle_valid.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oob_oracle_valid.restype = C.c_int
        L.oob_oracle_threads.restype = C.c_int
        L.oob_oracle_get_block.argtypes = [C.c_void_p, C.c_int, C.c_int, i32p, i64p, i64p, i64p,
                                           i64p, i32p, i32p, i32p, i32p]
        L.oob_oracle_get_block.restype = C.c_int
        L.oob_oracle_templates.argtypes = [C.c_void_p, C.c_int, C.c_int, i32p, i32p, i32p, i64p,
                                           i64p, i64p, i64p, i64p, i32p, i32p, i32p]
        L.oob_oracle_templates.restype = None
        L.oob_oracle_coverage.argtypes = [i32p, C.c_int, C.c_int, C.c_int, i32p, i32p, C.c_int]
        L.oob_oracle_coverage.restype = None
        L.oob_oracle_instantiate.argtypes = [i32p, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_uint16),
                                             C.c_int64, C.POINTER(C.c_int64)]
        L.oob_oracle_instantiate.restype = C.c_int64
        _lib = L
    return _lib


def _p64(a):
    return a.ctypes.data_as(C.POINTER(C.c_int64))


def _p32(a):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


class Oracle:
    """All DP tables of one planning job, computed on the CPU."""

    def __init__(self, inp, threads: int = 0):
        self.inp = inp
        self.L, self.M = inp.L, inp.gpus_per_node
        fwd = np.ascontiguousarray(inp.fwd_ns, dtype=np.int64)
        bwd = np.ascontiguousarray(inp.bwd_ns, dtype=np.int64)
        mem = np.ascontiguousarray(inp.mem_bytes, dtype=np.int64)
        bnd = np.ascontiguousarray(inp.boundary_ns, dtype=np.int64)
        self._h = lib().oob_oracle_create(_p64(fwd), _p64(bwd), _p64(mem), _p64(bnd), self.L,
                                          inp.n_max, self.M, inp.microbatches, inp.mem_cap,
                                          threads)
        if not self._h:
            raise ValueError("oracle: bad arguments")
        self.Smax = lib().oob_oracle_smax(self._h)
        self.D = lib().oob_oracle_ndelta(self._h)
        self.states = lib().oob_oracle_states(self._h)
        self.candidates = lib().oob_oracle_candidates(self._h)
        self.evaluated = lib().oob_oracle_evaluated(self._h)

    def close(self):
        if self._h:
            lib().oob_oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def valid(self, S: int, delta: int) -> bool:
        return bool(lib().oob_oracle_valid(self._h, S, delta))

    def block(self, S: int, delta: int) -> Dict[str, np.ndarray]:
        """Records of one (S', delta), each array [(L+1), (L+1)] indexed [u, v]."""
        W = self.L + 1
        a32 = {k: np.zeros((W, W), dtype=np.int32) for k in ("exists", "kstar", "s", "k", "m")}
        a64 = {k: np.zeros((W, W), dtype=np.int64) for k in ("T", "T1", "T3", "tmax")}
        ok = lib().oob_oracle_get_block(self._h, S, delta, _p32(a32["exists"]), _p64(a64["T"]),
                                        _p64(a64["T1"]), _p64(a64["T3"]), _p64(a64["tmax"]),
                                        _p32(a32["kstar"]), _p32(a32["s"]), _p32(a32["k"]),
                                        _p32(a32["m"]))
        if not ok:
            raise KeyError((S, delta))
        a32.update(a64)
        return a32

    def templates(self, n_min: int, n_max: int) -> Dict[str, np.ndarray]:
        cnt = n_max - n_min + 1
        cap = cnt * max(1, self.Smax)
        r = {k: np.zeros(cnt, dtype=np.int32) for k in ("feasible", "S", "kstar")}
        r.update({k: np.zeros(cnt, dtype=np.int64) for k in ("T", "T1", "T2", "T3", "tmax")})
        r["stage_off"] = np.zeros(cnt + 1, dtype=np.int32)
        r["stage_begin"] = np.zeros(cap + cnt, dtype=np.int32)
        r["stage_gpus"] = np.zeros(cap, dtype=np.int32)
        lib().oob_oracle_templates(self._h, n_min, cnt, _p32(r["feasible"]), _p32(r["S"]),
                                   _p32(r["kstar"]), _p64(r["T"]), _p64(r["T1"]), _p64(r["T2"]),
                                   _p64(r["T3"]), _p64(r["tmax"]), _p32(r["stage_off"]),
                                   _p32(r["stage_begin"]), _p32(r["stage_gpus"]))
        return r


def coverage(feasible: np.ndarray, n_min: int, f: int) -> Dict[str, np.ndarray]:
    feasible = np.ascontiguousarray(feasible, dtype=np.int32)
    cnt = int(feasible.shape[0])
    hdr = np.zeros(8, dtype=np.int32)
    ln = max(cnt, f + 1)
    mp = np.zeros(ln, dtype=np.int32)
    lib().oob_oracle_coverage(_p32(feasible), n_min, cnt, f, _p32(hdr), _p32(mp), ln)
    return {"hdr": hdr, "maxpipes": mp}


def plan(inp, threads: int = 0) -> dict:
    """Whole hot path on the CPU: tables, templates, coverage."""
    o = Oracle(inp, threads)
    try:
        t = o.templates(inp.n_min, inp.n_max)
        c = coverage(t["feasible"], inp.n_min, inp.f)
        t["cover_hdr"] = c["hdr"]
        t["cover_maxpipes"] = c["maxpipes"]
        t["states"], t["candidates"], t["evaluated"] = o.states, o.candidates, o.evaluated
        return t
    finally:
        o.close()


def template_stages(t: dict, i: int):
    """(stage_begin list of S+1 entries, stage_gpus list of S entries) of template i."""
    S = int(t["S"][i])
    off = int(t["stage_off"][i])
    return (list(map(int, t["stage_begin"][off + i: off + i + S + 1])),
            list(map(int, t["stage_gpus"][off: off + S])))
