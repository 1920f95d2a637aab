"""Thin Python binding of the C ABI in include/oob_plan.h.

Argument marshalling only: every step of the planning path runs in the HIP
kernels of liboob_plan.so.  PyTorch supplies device memory and the stream.
There is no CPU fallback: if the library is missing, loading fails.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "liboob_plan.so")

OOB_OK, OOB_EINVAL, OOB_ECAPACITY, OOB_EOVERFLOW, OOB_EHIP = 0, -1, -2, -3, -4
OOB_FORBIDDEN = 1 << 62
_ERR = {OOB_EINVAL: "OOB_EINVAL", OOB_ECAPACITY: "OOB_ECAPACITY", OOB_EOVERFLOW: "OOB_EOVERFLOW",
        OOB_EHIP: "OOB_EHIP"}

SYMBOLS = ["oob_plan_max_stages", "oob_plan_workspace_size", "oob_plan_create",
           "oob_plan_templates", "oob_plan_templates_batch", "oob_plan_destroy", "oob_plan_export_block",
           "oob_plan_level_timing", "oob_plan_last_level_ms", "oob_plan_export_flags", "oob_plan_valu_peak", "oob_plan_valu_peak_f64",
           "oob_plan_set_option", "oob_plan_layout_selftest"]
OOB_OPT_PLAIN_SPLIT, OOB_OPT_XCD_ORDER, OOB_OPT_ONE_STREAM = 1, 2, 3
OOB_OPT_SELECT8_FROM, OOB_OPT_FUSE_FROM = 4, 5
INST_SYMBOLS = ["oob_inst_workspace_size", "oob_inst_count", "oob_inst_enumerate", "oob_inst_keep_wide_table",
                "oob_inst_enumerate_static"]
OOB_INST_STATIC_BYTES = 4 << 20
RECONF_SYMBOLS = ["oob_reconf_simulate"]
DIST_SYMBOLS = ["oob_dist_solve", "oob_dist_choose"]
EXACT_SYMBOLS = ["oob_exact_workspace_size", "oob_exact_minimum", "oob_exact_staged_workspace_size",
                 "oob_exact_minimum_staged"]
OOB_EXACT_LIMIT_CAN_BIND = -2
OOB_DIST_OK, OOB_DIST_TOO_FEW_MICROBATCHES, OOB_DIST_TOO_MANY_TEMPLATES, OOB_DIST_BAD_TIME, OOB_DIST_NO_PIPELINE = range(5)
RECONF_ROWS = ("survived", "reinstantiated", "borrowed", "merges", "alive", "nodes", "violations", "stop")


class oob_profile(C.Structure):
    _fields_ = [("fwd_ns", C.c_void_p), ("bwd_ns", C.c_void_p), ("mem_bytes", C.c_void_p),
                ("boundary_ns", C.c_void_p)]


class oob_templates(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("feasible", "S", "kstar", "T", "T1", "T2", "T3", "tmax", "stage_off", "stage_begin",
                 "stage_gpus", "cover_hdr", "cover_maxpipes", "status")] + \
               [("states", C.c_int64), ("candidates", C.c_int64)]


_lib = None


def load():
    """Loads liboob_plan.so (built by paper_2309_08125_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2309_08125_amd.build` "
                               "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        L.oob_plan_max_stages.argtypes = [C.c_int] * 4
        L.oob_plan_max_stages.restype = C.c_int
        L.oob_plan_layout_selftest.argtypes = [C.c_int]
        L.oob_plan_layout_selftest.restype = C.c_int
        L.oob_plan_workspace_size.argtypes = [C.c_int] * 3
        L.oob_plan_workspace_size.restype = C.c_size_t
        L.oob_plan_create.argtypes = [C.POINTER(C.c_void_p), C.c_int, C.c_int, C.c_int, C.c_void_p,
                                      C.c_size_t]
        L.oob_plan_create.restype = C.c_int
        L.oob_plan_templates.argtypes = [C.c_void_p, C.POINTER(oob_profile), C.c_int, C.c_int,
                                         C.c_int, C.c_int, C.c_int, C.c_int64, C.c_int,
                                         C.POINTER(oob_templates), C.c_void_p]
        L.oob_plan_templates.restype = C.c_int
        L.oob_plan_templates_batch.argtypes = [C.c_void_p, C.c_int, C.POINTER(oob_profile),
                                               C.POINTER(C.c_int), C.POINTER(C.c_int),
                                               C.POINTER(C.c_int), C.POINTER(C.c_int),
                                               C.POINTER(C.c_int), C.POINTER(C.c_int64),
                                               C.POINTER(C.c_int), C.POINTER(oob_templates),
                                               C.c_void_p]
        L.oob_plan_templates_batch.restype = C.c_int
        L.oob_plan_destroy.argtypes = [C.c_void_p]
        L.oob_plan_destroy.restype = C.c_int
        L.oob_plan_level_timing.argtypes = [C.c_void_p, C.c_int]
        L.oob_plan_level_timing.restype = C.c_int
        L.oob_plan_last_level_ms.argtypes = [C.c_void_p, C.POINTER(C.c_float)]
        L.oob_plan_last_level_ms.restype = C.c_int
        L.oob_plan_export_flags.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_plan_export_flags.restype = C.c_int
        L.oob_plan_export_block.argtypes = [C.c_void_p, C.c_int, C.c_int] + [C.c_void_p] * 7
        L.oob_plan_export_block.restype = C.c_int
        L.oob_plan_valu_peak.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        L.oob_plan_valu_peak.restype = C.c_int
        L.oob_plan_valu_peak_f64.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
        L.oob_plan_valu_peak_f64.restype = C.c_int
        L.oob_plan_set_option.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.oob_plan_set_option.restype = C.c_int
        L.oob_inst_enumerate_static.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p,
                                                C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_inst_enumerate_static.restype = C.c_int
        L.oob_inst_keep_wide_table.argtypes = [C.c_int]
        L.oob_inst_keep_wide_table.restype = C.c_int
        L.oob_inst_workspace_size.argtypes = [C.c_int] * 3
        L.oob_inst_workspace_size.restype = C.c_size_t
        spec = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_size_t]
        L.oob_inst_count.argtypes = spec + [C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_inst_count.restype = C.c_int
        L.oob_inst_enumerate.argtypes = spec + [C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_inst_enumerate.restype = C.c_int
        L.oob_reconf_simulate.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_void_p, C.c_int,
                                          C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                          C.c_void_p]
        L.oob_reconf_simulate.restype = C.c_int
        L.oob_dist_solve.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p, C.c_int, C.c_void_p,
                                     C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_dist_solve.restype = C.c_int
        L.oob_dist_choose.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_dist_choose.restype = C.c_int
        L.oob_exact_workspace_size.argtypes = [C.c_int] * 3
        L.oob_exact_workspace_size.restype = C.c_size_t
        L.oob_exact_minimum.argtypes = [C.POINTER(oob_profile), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int64,
                                        C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oob_exact_minimum.restype = C.c_int
        L.oob_exact_staged_workspace_size.argtypes = [C.c_int] * 4
        L.oob_exact_staged_workspace_size.restype = C.c_size_t
        L.oob_exact_minimum_staged.argtypes = L.oob_exact_minimum.argtypes
        L.oob_exact_minimum_staged.restype = C.c_int
        _lib = L
    return _lib


def check(rc: int, what: str):
    if rc != OOB_OK:
        raise RuntimeError(f"{what}: {_ERR.get(rc, rc)}")


# ---- the C entry points under their own names (thin wrappers) ----------------------------
def oob_plan_max_stages(L, n_max, gpus_per_node, microbatches) -> int:
    return load().oob_plan_max_stages(L, n_max, gpus_per_node, microbatches)


def oob_plan_layout_selftest(L) -> int:
    return load().oob_plan_layout_selftest(L)


def oob_plan_workspace_size(max_L, max_nodes, max_gpus_per_node) -> int:
    return load().oob_plan_workspace_size(max_L, max_nodes, max_gpus_per_node)


def oob_plan_create(max_L, max_nodes, max_gpus_per_node, dev_workspace_ptr, workspace_bytes):
    h = C.c_void_p()
    rc = load().oob_plan_create(C.byref(h), max_L, max_nodes, max_gpus_per_node,
                                C.c_void_p(dev_workspace_ptr), workspace_bytes)
    return rc, h


def oob_plan_templates(h, profile: oob_profile, L, n_min, n_max, gpus_per_node, microbatches,
                       mem_cap, f, out: oob_templates, stream_ptr) -> int:
    return load().oob_plan_templates(h, C.byref(profile), L, n_min, n_max, gpus_per_node,
                                     microbatches, mem_cap, f, C.byref(out),
                                     C.c_void_p(stream_ptr))


def oob_plan_templates_batch(h, profiles, Ls, n_mins, n_maxs, gpus, microbatches, mem_caps, fs, outs,
                             stream_ptr) -> int:
    """profiles: list of oob_profile, outs: list of oob_templates (filled in place), the rest
    lists of ints."""
    n = len(profiles)
    prof_arr = (oob_profile * n)(*profiles)
    out_arr = (oob_templates * n)(*outs)
    ints = lambda xs: (C.c_int * n)(*xs)
    rc = load().oob_plan_templates_batch(h, n, prof_arr, ints(Ls), ints(n_mins), ints(n_maxs), ints(gpus),
                                         ints(microbatches), (C.c_int64 * n)(*mem_caps), ints(fs), out_arr,
                                         C.c_void_p(stream_ptr))
    for i in range(n):  # host fields written by the library
        outs[i].states, outs[i].candidates = out_arr[i].states, out_arr[i].candidates
    return rc


def oob_plan_destroy(h) -> int:
    return load().oob_plan_destroy(h)


def oob_inst_workspace_size(p, N_hi, f) -> int:
    return load().oob_inst_workspace_size(p, N_hi, f)


def oob_inst_count(sizes_ptr, p, n0, N_lo, N_hi, f, dev_workspace_ptr, workspace_bytes, offsets_ptr,
                   status_ptr, stream_ptr) -> int:
    return load().oob_inst_count(C.c_void_p(sizes_ptr), p, n0, N_lo, N_hi, f, C.c_void_p(dev_workspace_ptr),
                                 workspace_bytes, C.c_void_p(offsets_ptr), C.c_void_p(status_ptr),
                                 C.c_void_p(stream_ptr))


def oob_inst_enumerate(sizes_ptr, p, n0, N_lo, N_hi, f, dev_workspace_ptr, workspace_bytes, x_ptr, capacity,
                       offsets_ptr, status_ptr, stream_ptr) -> int:
    return load().oob_inst_enumerate(C.c_void_p(sizes_ptr), p, n0, N_lo, N_hi, f,
                                     C.c_void_p(dev_workspace_ptr), workspace_bytes, C.c_void_p(x_ptr),
                                     capacity, C.c_void_p(offsets_ptr), C.c_void_p(status_ptr),
                                     C.c_void_p(stream_ptr))


def oob_inst_enumerate_static(sizes_ptr, p, n0, N_lo, N_hi, f, x_ptr, capacity, offsets_ptr, status_ptr,
                              stream_ptr) -> int:
    return load().oob_inst_enumerate_static(C.c_void_p(sizes_ptr), p, n0, N_lo, N_hi, f, C.c_void_p(x_ptr), capacity,
                                            C.c_void_p(offsets_ptr), C.c_void_p(status_ptr), C.c_void_p(stream_ptr))


def oob_reconf_simulate(sizes0_ptr, c0, n0, n_hi, f, draws_ptr, steps, burst, T, trace_ptr, final_sizes_ptr,
                        summary_ptr, status_ptr, stream_ptr) -> int:
    return load().oob_reconf_simulate(C.c_void_p(sizes0_ptr), c0, n0, n_hi, f, C.c_void_p(draws_ptr), steps, burst,
                                      T, C.c_void_p(trace_ptr), C.c_void_p(final_sizes_ptr),
                                      C.c_void_p(summary_ptr), C.c_void_p(status_ptr), C.c_void_p(stream_ptr))


def oob_dist_solve(x_ptr, count, capacity, p, template_T_ptr, Q, vx_ptr, slowest_ptr, base_ptr, extra_ptr,
                   status_ptr, stream_ptr) -> int:
    return load().oob_dist_solve(C.c_void_p(x_ptr), count, capacity, p, C.c_void_p(template_T_ptr), Q,
                                 C.c_void_p(vx_ptr), C.c_void_p(slowest_ptr), C.c_void_p(base_ptr),
                                 C.c_void_p(extra_ptr), C.c_void_p(status_ptr), C.c_void_p(stream_ptr))


def oob_dist_choose(offsets_ptr, segments, count, slowest_ptr, status_ptr, best_ptr, stream_ptr) -> int:
    return load().oob_dist_choose(C.c_void_p(offsets_ptr), segments, count, C.c_void_p(slowest_ptr),
                                  C.c_void_p(status_ptr), C.c_void_p(best_ptr), C.c_void_p(stream_ptr))


def oob_exact_workspace_size(L, n_max, gpus_per_node) -> int:
    return load().oob_exact_workspace_size(L, n_max, gpus_per_node)


def oob_exact_minimum(profile, L, n_min, n_max, gpus_per_node, microbatches, mem_cap, dev_workspace_ptr,
                      workspace_bytes, best_ptr, status_ptr, stream_ptr) -> int:
    return load().oob_exact_minimum(C.byref(profile) if profile is not None else None, L, n_min, n_max,
                                    gpus_per_node, microbatches, mem_cap, C.c_void_p(dev_workspace_ptr),
                                    workspace_bytes, C.c_void_p(best_ptr), C.c_void_p(status_ptr),
                                    C.c_void_p(stream_ptr))


def oob_exact_staged_workspace_size(L, n_max, gpus_per_node, microbatches) -> int:
    return load().oob_exact_staged_workspace_size(L, n_max, gpus_per_node, microbatches)


def oob_exact_minimum_staged(profile, L, n_min, n_max, gpus_per_node, microbatches, mem_cap, dev_workspace_ptr,
                             workspace_bytes, best_ptr, status_ptr, stream_ptr) -> int:
    return load().oob_exact_minimum_staged(C.byref(profile) if profile is not None else None, L, n_min, n_max,
                                           gpus_per_node, microbatches, mem_cap, C.c_void_p(dev_workspace_ptr),
                                           workspace_bytes, C.c_void_p(best_ptr), C.c_void_p(status_ptr),
                                           C.c_void_p(stream_ptr))


# ---- convenience layer over torch device memory ------------------------------------------
class DeviceProfile:
    """A PlanInput's arrays resident in HBM: one device buffer, one host-to-device copy."""

    KEYS = ("fwd_ns", "bwd_ns", "mem_bytes", "boundary_ns")

    def __init__(self, inp, device="cuda:0"):
        import numpy as np
        import torch

        self.inp = inp
        parts = [np.ascontiguousarray(a, dtype=np.int64).reshape(-1)
                 for a in (inp.fwd_ns, inp.bwd_ns, inp.mem_bytes, inp.boundary_ns)]
        self.base = torch.from_numpy(np.concatenate(parts)).to(device)
        self.t, o = {}, 0
        for k, a in zip(self.KEYS, parts):
            self.t[k] = self.base[o: o + a.size]
            o += a.size
        self.c = oob_profile(*(self.t[k].data_ptr() for k in self.KEYS))


class DeviceTemplates:
    """Result buffers in HBM for `count` templates of at most Smax stages: views of one device buffer,
    so that the results come back in one device-to-host copy."""

    I32 = ("feasible", "S", "kstar", "stage_off", "stage_begin", "stage_gpus", "cover_hdr",
           "cover_maxpipes", "status")
    I64 = ("T", "T1", "T2", "T3", "tmax")

    def __init__(self, count: int, Smax: int, f: int, device="cuda:0"):
        import torch

        sizes = {"feasible": count, "S": count, "kstar": count, "stage_off": count + 1,
                 "stage_begin": count * (Smax + 1), "stage_gpus": count * Smax, "cover_hdr": 8,
                 "cover_maxpipes": max(count, f + 1), "status": 1}
        # the 64-bit arrays first, then the 32-bit ones, every array on an 8-byte boundary
        self.layout, o = {}, 0
        for k in self.I64:
            self.layout[k] = (o, count, torch.int64)
            o += 8 * count
        for k in self.I32:
            n = max(1, sizes[k])
            self.layout[k] = (o, n, torch.int32)
            o += (4 * n + 7) // 8 * 8
        self.base = torch.zeros(o, dtype=torch.uint8, device=device)
        self.t = {k: self.base[off: off + n * (8 if dt == torch.int64 else 4)].view(dt)
                  for k, (off, n, dt) in self.layout.items()}
        self.c = oob_templates()
        for k in self.I32 + self.I64:
            setattr(self.c, k, self.t[k].data_ptr())

    def to_host(self) -> Dict[str, "object"]:
        import torch

        host = self.base.cpu()  # waits for the stream's work, then one copy
        r = {k: host[off: off + n * (8 if dt == torch.int64 else 4)].view(dt).numpy()
             for k, (off, n, dt) in self.layout.items()}
        r["states"], r["candidates"] = int(self.c.states), int(self.c.candidates)
        return r


class Planner:
    """Owns a workspace tensor and a handle sized for the given maxima; `lanes` > 1 sizes the
    workspace for that many jobs side by side in plan_batch."""

    def __init__(self, max_L: int, max_nodes: int, max_gpus_per_node: int, device="cuda:0", lanes: int = 1):
        import torch

        self.device = torch.device(device)
        nbytes = oob_plan_workspace_size(max_L, max_nodes, max_gpus_per_node)
        if nbytes == 0:
            raise ValueError("oob_plan_workspace_size: dimensions out of range")
        nbytes = (nbytes + 255) // 256 * 256 * max(1, lanes)
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        rc, self.h = oob_plan_create(max_L, max_nodes, max_gpus_per_node,
                                     self.workspace.data_ptr(), nbytes)
        check(rc, "oob_plan_create")

    def close(self):
        if getattr(self, "h", None):
            oob_plan_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def level_timing(self, enable: bool = True):
        check(load().oob_plan_level_timing(self.h, int(enable)), "oob_plan_level_timing")

    def last_level_ms(self) -> float:
        ms = C.c_float()
        check(load().oob_plan_last_level_ms(self.h, C.byref(ms)), "oob_plan_last_level_ms")
        return float(ms.value)

    def valu_peak(self, f64_mix: bool = False) -> float:
        """Measured lane-operations per second: 32-bit add / compare / select (oob_plan_valu_peak) or
        the fp64 mix of a candidate (oob_plan_valu_peak_f64)."""
        import torch

        v = C.c_double()
        s = torch.cuda.current_stream(self.device)
        fn = load().oob_plan_valu_peak_f64 if f64_mix else load().oob_plan_valu_peak
        check(fn(self.h, C.c_void_p(s.cuda_stream), C.byref(v)), "oob_plan_valu_peak")
        return float(v.value)

    def new_outputs(self, inp) -> DeviceTemplates:
        Smax = oob_plan_max_stages(inp.L, inp.n_max, inp.gpus_per_node, inp.microbatches)
        return DeviceTemplates(inp.n_max - inp.n_min + 1, Smax, inp.f, self.device)

    def enqueue(self, prof: DeviceProfile, out: DeviceTemplates, stream=None) -> None:
        """oob_plan_templates on `stream` (default: torch's current stream); no sync."""
        import torch

        inp = prof.inp
        s = stream if stream is not None else torch.cuda.current_stream(self.device)
        rc = oob_plan_templates(self.h, prof.c, inp.L, inp.n_min, inp.n_max, inp.gpus_per_node,
                                inp.microbatches, inp.mem_cap, inp.f, out.c, s.cuda_stream)
        check(rc, "oob_plan_templates")
        self.last_L = inp.L

    def plan_batch(self, inps) -> List[Dict[str, "object"]]:
        """Independent jobs through oob_plan_templates_batch (one after the other on the stream)."""
        import torch

        profs = [DeviceProfile(inp, self.device) for inp in inps]
        outs = [self.new_outputs(inp) for inp in inps]
        s = torch.cuda.current_stream(self.device)
        rc = oob_plan_templates_batch(self.h, [p.c for p in profs], [i.L for i in inps],
                                      [i.n_min for i in inps], [i.n_max for i in inps],
                                      [i.gpus_per_node for i in inps], [i.microbatches for i in inps],
                                      [i.mem_cap for i in inps], [i.f for i in inps],
                                      [o.c for o in outs], s.cuda_stream)
        check(rc, "oob_plan_templates_batch")
        self.last_L = inps[-1].L if inps else 0
        torch.cuda.synchronize(self.device)
        return [o.to_host() for o in outs]

    def plan(self, inp) -> Dict[str, "object"]:
        import torch

        prof = DeviceProfile(inp, self.device)
        out = self.new_outputs(inp)
        self.enqueue(prof, out)
        torch.cuda.synchronize(self.device)
        return out.to_host()

    def set_option(self, option: int, value: int):
        check(load().oob_plan_set_option(self.h, option, value), "oob_plan_set_option")

    def flags(self):
        """[keyed split kernel used, reserved x3] of the last call."""
        import torch

        buf = torch.zeros(4, dtype=torch.int32, device=self.device)
        s = torch.cuda.current_stream(self.device)
        check(load().oob_plan_export_flags(self.h, buf.data_ptr(), C.c_void_p(s.cuda_stream)),
              "oob_plan_export_flags")
        return buf.cpu().numpy().tolist()

    def block(self, S: int, delta: int) -> Optional[Dict[str, "object"]]:
        """Records of (S', delta) left by the last call, arrays [n, n] indexed [u, v - S']."""
        import torch

        n = self.last_L - S + 1
        if n < 1:
            return None
        bufs = {k: torch.empty(n * n, dtype=torch.float64, device=self.device)
                for k in ("T", "T1", "tmax", "T3")}
        bufs.update({k: torch.empty(n * n, dtype=torch.int32, device=self.device)
                     for k in ("kstar", "choice")})
        s = torch.cuda.current_stream(self.device)
        rc = load().oob_plan_export_block(self.h, S, delta, *(bufs[k].data_ptr() for k in
                                          ("T", "T1", "tmax", "T3", "kstar", "choice")),
                                          C.c_void_p(s.cuda_stream))
        if rc != OOB_OK:
            return None
        return {k: v.cpu().numpy().reshape(n, n) for k, v in bufs.items()}


class Instantiator:
    """Device buffers for oob_inst_count / oob_inst_enumerate of one (sizes, N' range, f)."""

    def __init__(self, sizes, N_lo: int, N_hi: int, f: int, n0: int = 0, p: int = 0, device="cuda:0"):
        """sizes: list of template sizes, or None for the consecutive sizes n0 .. n0+p-1."""
        import torch

        self.device = torch.device(device)
        self.sizes = None if sizes is None else torch.tensor(list(sizes), dtype=torch.int32, device=self.device)
        self.p = p if sizes is None else len(sizes)
        self.n0, self.N_lo, self.N_hi, self.f = n0, N_lo, N_hi, f
        nbytes = oob_inst_workspace_size(self.p, N_hi, f)
        if nbytes == 0:
            raise ValueError("oob_inst_workspace_size: arguments out of range")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self.offsets = torch.zeros(N_hi - N_lo + 2, dtype=torch.int64, device=self.device)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.device)

    def _spec(self):
        return (self.sizes.data_ptr() if self.sizes is not None else 0, self.p, self.n0, self.N_lo, self.N_hi,
                self.f, self.workspace.data_ptr(), self.workspace.numel())

    def count(self):
        """Offsets per N' (host array, last entry = total) and the device status."""
        import torch

        s = torch.cuda.current_stream(self.device)
        check(oob_inst_count(*self._spec(), self.offsets.data_ptr(), self.status.data_ptr(), s.cuda_stream),
              "oob_inst_count")
        torch.cuda.synchronize(self.device)
        return self.offsets.cpu().numpy(), int(self.status.item())

    def enqueue(self, x, capacity: int) -> None:
        """oob_inst_enumerate into the 16-bit tensor x ([p, capacity], read as uint16) on the current stream;
        count() must have run for this object before."""
        import torch

        s = torch.cuda.current_stream(self.device)
        check(oob_inst_enumerate(*self._spec(), x.data_ptr() if x is not None else 0, capacity,
                                 self.offsets.data_ptr(), self.status.data_ptr(), s.cuda_stream),
              "oob_inst_enumerate")

    def enumerate(self):
        """(offsets, vectors [total, p] as a host array in list order, status)."""
        import torch

        off, st = self.count()
        total = int(off[-1])
        if st != OOB_OK:
            return off, None, st
        x = torch.empty((self.p, max(total, 1)), dtype=torch.int16, device=self.device)  # uint16 bits
        self.enqueue(x, total)
        torch.cuda.synchronize(self.device)
        return off, x.cpu().numpy().view("uint16")[:, :total].T.copy(), int(self.status.item())


class FailureSimulator:
    """Device buffers for oob_reconf_simulate: T trajectories of `steps` steps of `burst` failures."""

    def __init__(self, sizes0, n0: int, n_hi: int, f: int, draws, trace: bool = True, device="cuda:0"):
        """draws: uint32 host array [steps, burst, T] (inputs.failure_draws)."""
        import numpy as np
        import torch

        self.device = torch.device(device)
        self.steps, self.burst, self.T = (int(v) for v in draws.shape)
        self.n0, self.n_hi, self.f = n0, n_hi, f
        self.sizes0 = torch.tensor([int(v) for v in sizes0], dtype=torch.int32, device=self.device)
        self.c0 = self.sizes0.numel()
        self.draws = torch.from_numpy(np.ascontiguousarray(draws).view(np.int32)).to(self.device)  # uint32 bits
        self.trace = torch.zeros((self.steps, self.T), dtype=torch.int32, device=self.device) if trace else None
        self.final_sizes = torch.zeros((self.c0, self.T), dtype=torch.int32, device=self.device)
        self.summary = torch.zeros((len(RECONF_ROWS), self.T), dtype=torch.int32, device=self.device)
        self.status = torch.full((1,), -99, dtype=torch.int32, device=self.device)

    def enqueue(self) -> None:
        import torch

        s = torch.cuda.current_stream(self.device)
        check(oob_reconf_simulate(self.sizes0.data_ptr(), self.c0, self.n0, self.n_hi, self.f,
                                  self.draws.data_ptr(), self.steps, self.burst, self.T,
                                  self.trace.data_ptr() if self.trace is not None else 0,
                                  self.final_sizes.data_ptr(), self.summary.data_ptr(), self.status.data_ptr(),
                                  s.cuda_stream), "oob_reconf_simulate")

    def run(self):
        """(status, summary rows by name, final sizes [c0, T], trace words [steps, T] as uint32)."""
        import torch

        self.enqueue()
        torch.cuda.synchronize(self.device)
        summary = {k: self.summary[i].cpu().numpy() for i, k in enumerate(RECONF_ROWS)}
        trace = self.trace.cpu().numpy().view("uint32") if self.trace is not None else None
        return int(self.status.item()), summary, self.final_sizes.cpu().numpy(), trace


class ExactMinimum:
    """Device buffers for oob_exact_minimum (staged=False) or oob_exact_minimum_staged of one planning job."""

    def __init__(self, inp, staged: bool = False, device="cuda:0", workspace_bytes: int = 0):
        import torch

        self.device = torch.device(device)
        self.inp, self.staged = inp, staged
        self.prof = DeviceProfile(inp, self.device)
        nbytes = (oob_exact_staged_workspace_size(inp.L, inp.n_max, inp.gpus_per_node, inp.microbatches) if staged
                  else oob_exact_workspace_size(inp.L, inp.n_max, inp.gpus_per_node))
        if nbytes == 0:
            raise ValueError("oob_exact_workspace_size: dimensions out of range")
        self.workspace = torch.empty(workspace_bytes or nbytes, dtype=torch.uint8, device=self.device)
        self.best = torch.full((inp.n_max - inp.n_min + 1,), -99, dtype=torch.int64, device=self.device)
        self.status = torch.full((1,), -99, dtype=torch.int32, device=self.device)

    def enqueue(self) -> int:
        import torch

        i = self.inp
        s = torch.cuda.current_stream(self.device)
        fn = oob_exact_minimum_staged if self.staged else oob_exact_minimum
        return fn(self.prof.c, i.L, i.n_min, i.n_max, i.gpus_per_node, i.microbatches, i.mem_cap,
                  self.workspace.data_ptr(), self.workspace.numel(), self.best.data_ptr(),
                  self.status.data_ptr(), s.cuda_stream)

    def run(self):
        """(status, exact minimum per template as a list: None where no pipeline exists,
        OOB_EXACT_LIMIT_CAN_BIND where the entry point without stage counts does not answer)."""
        import torch

        check(self.enqueue(), "oob_exact_minimum")
        torch.cuda.synchronize(self.device)
        return int(self.status.item()), [None if v == -1 else int(v) for v in self.best.cpu().numpy()]


class Distributor:
    """Device buffers for oob_dist_solve / oob_dist_choose over `count` plans of p templates."""

    def __init__(self, x, count: int, template_T, Q: int, distribution: bool = True, device="cuda:0"):
        """x: int16 device tensor [p, capacity] (uint16 bits, as Instantiator.enqueue fills it) or a host
        array [count, p] of counts; template_T: p times per microbatch."""
        import numpy as np
        import torch

        self.device = torch.device(device)
        if not torch.is_tensor(x):
            x = torch.from_numpy(np.ascontiguousarray(np.asarray(x, dtype=np.uint16).T).view(np.int16)).to(self.device)
        self.x, self.count, self.Q = x, count, Q
        self.p, self.capacity = int(x.shape[0]), int(x.shape[1])
        self.template_T = torch.tensor([int(v) for v in template_T], dtype=torch.int64, device=self.device)
        n = max(count, 1)
        self.vx = torch.zeros((n, 2), dtype=torch.int64, device=self.device)
        self.slowest = torch.zeros(n, dtype=torch.int64, device=self.device)
        self.status = torch.full((n,), -99, dtype=torch.int32, device=self.device)
        self.base = torch.zeros_like(x) if distribution else None
        self.extra = torch.zeros_like(x) if distribution else None

    def enqueue(self) -> None:
        import torch

        s = torch.cuda.current_stream(self.device)
        check(oob_dist_solve(self.x.data_ptr(), self.count, self.capacity, self.p, self.template_T.data_ptr(), self.Q,
                             self.vx.data_ptr(), self.slowest.data_ptr(),
                             self.base.data_ptr() if self.base is not None else 0,
                             self.extra.data_ptr() if self.extra is not None else 0,
                             self.status.data_ptr(), s.cuda_stream), "oob_dist_solve")

    def solve(self):
        """(status [count], vx [count] as Python ints, slowest [count], base [count, p], extra [count, p])."""
        import torch

        self.enqueue()
        torch.cuda.synchronize(self.device)
        w = self.vx.cpu().numpy().view("uint64")[: self.count]
        vx = [(int(hi) << 64) | int(lo) for lo, hi in w]
        cut = lambda t: None if t is None else t.cpu().numpy().view("uint16")[:, : self.count].T.copy()
        return (self.status.cpu().numpy()[: self.count], vx, self.slowest.cpu().numpy()[: self.count],
                cut(self.base), cut(self.extra))

    def choose(self, offsets):
        """Index of the best plan of every group offsets[g] .. offsets[g+1]-1 (host array in, host array out)."""
        import numpy as np
        import torch

        off = torch.from_numpy(np.asarray(offsets, dtype=np.int64)).to(self.device)
        best = torch.full((len(offsets) - 1,), -99, dtype=torch.int64, device=self.device)
        s = torch.cuda.current_stream(self.device)
        check(oob_dist_choose(off.data_ptr(), len(offsets) - 1, self.count, self.slowest.data_ptr(),
                              self.status.data_ptr(), best.data_ptr(), s.cuda_stream), "oob_dist_choose")
        torch.cuda.synchronize(self.device)
        return best.cpu().numpy()

    def time_choose(self, offsets, reps: int = 20) -> float:
        """Seconds per oob_dist_choose call, from events on the stream the kernels are launched on."""
        import numpy as np
        import torch

        off = torch.from_numpy(np.asarray(offsets, dtype=np.int64)).to(self.device)
        best = torch.full((len(offsets) - 1,), -99, dtype=torch.int64, device=self.device)
        s = torch.cuda.current_stream(self.device)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        args = (off.data_ptr(), len(offsets) - 1, self.count, self.slowest.data_ptr(), self.status.data_ptr(),
                best.data_ptr(), s.cuda_stream)
        check(oob_dist_choose(*args), "oob_dist_choose")
        ev[0].record(s)
        for _ in range(reps):
            check(oob_dist_choose(*args), "oob_dist_choose")
        ev[1].record(s)
        torch.cuda.synchronize(self.device)
        return ev[0].elapsed_time(ev[1]) / reps * 1e-3


def template_stages(r: dict, i: int):
    S = int(r["S"][i])
    off = int(r["stage_off"][i])
    return (list(map(int, r["stage_begin"][off + i: off + i + S + 1])),
            list(map(int, r["stage_gpus"][off: off + S])))
