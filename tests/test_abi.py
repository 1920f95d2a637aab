"""Host logic of the C ABI that needs no GPU: the library loads, exports every declared
symbol, validates arguments before touching the device, and sizes its workspace."""
import ctypes as C
import os
import re

import paper_2309_08125_amd as P
from paper_2309_08125_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(header="oob_plan.h", prefix="oob_plan_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = P.load()
    names = declared_symbols()
    assert len(names) >= 7
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(B.SYMBOLS) == names
    inst = declared_symbols("oob_inst.h", "oob_inst_")
    assert len(inst) == 5
    for name in inst:
        assert hasattr(lib, name), name
    assert sorted(B.INST_SYMBOLS) == inst
    reconf = declared_symbols("oob_reconf.h", "oob_reconf_")
    assert reconf == ["oob_reconf_simulate"] and hasattr(lib, reconf[0]) and sorted(B.RECONF_SYMBOLS) == reconf
    dist = declared_symbols("oob_dist.h", "oob_dist_")
    assert dist == ["oob_dist_choose", "oob_dist_solve"] and all(hasattr(lib, n) for n in dist)
    assert sorted(B.DIST_SYMBOLS) == dist
    exact = declared_symbols("oob_exact.h", "oob_exact_")
    assert exact == ["oob_exact_minimum", "oob_exact_minimum_staged", "oob_exact_staged_workspace_size",
                     "oob_exact_workspace_size"] and all(hasattr(lib, n) for n in exact)
    assert sorted(B.EXACT_SYMBOLS) == exact
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["oob_dist.h", "oob_exact.h", "oob_inst.h", "oob_plan.h",
                                                                  "oob_reconf.h"]


def test_exact_minimum_entry_point_validates_arguments_without_touching_the_gpu():
    assert P.oob_exact_workspace_size(98, 64, 8) > 0 and P.oob_exact_workspace_size(98, 64, 8) % 256 == 0
    assert P.oob_exact_workspace_size(256, 1, 1) == 0 and P.oob_exact_workspace_size(10, 600, 8) == 0
    prof = B.oob_profile(1, 1, 1, 1)
    fake = 0x10000
    call = lambda **kw: P.oob_exact_minimum(kw.get("prof", prof), kw.get("L", 12), kw.get("n_min", 1), kw.get("n_max", 4),
                                            kw.get("M", 2), kw.get("nb", 8), kw.get("cap", 1 << 30), kw.get("ws", fake),
                                            kw.get("nbytes", 1 << 40), kw.get("best", fake), kw.get("st", fake), 0)
    for bad in (dict(prof=None), dict(L=0), dict(L=256), dict(n_min=0), dict(n_min=5), dict(M=0), dict(cap=0),
                dict(ws=0), dict(ws=0x10001), dict(best=0), dict(st=0), dict(nb=-1)):
        assert call(**bad) == P.OOB_EINVAL, bad
    assert call(nbytes=1024) == P.OOB_ECAPACITY
    # the workspace of the entry point without stage counts is the two stage-time tables while its tables
    # fit LDS; the staged entry point wants at least 16 workgroups' worth of tables
    assert P.oob_exact_workspace_size(98, 64, 8) < (2 << 20) and P.oob_exact_workspace_size(250, 16, 8) > (1 << 28)
    assert P.oob_exact_staged_workspace_size(40, 8, 4, 16) % 256 == 0 and P.oob_exact_staged_workspace_size(40, 8, 4, -1) == 0
    staged = lambda **kw: P.oob_exact_minimum_staged(prof, 12, 1, 4, 2, kw.get("nb", 3), 1 << 30, fake,
                                                     kw.get("nbytes", 1 << 40), fake, fake, 0)
    assert staged(nb=-1) == P.OOB_EINVAL and staged(nbytes=4096) == P.OOB_ECAPACITY


def test_reconfiguration_entry_point_validates_arguments_without_touching_the_gpu():
    fake = 0x10000  # never dereferenced: every call below fails its host-side checks
    call = lambda **kw: P.oob_reconf_simulate(kw.get("sizes0", fake), kw.get("c0", 4), kw.get("n0", 2),
                                              kw.get("n_hi", 5), kw.get("f", 1), kw.get("draws", fake),
                                              kw.get("steps", 3), kw.get("burst", 1), kw.get("T", 100), fake, fake,
                                              kw.get("summary", fake), kw.get("status", fake), 0)
    for bad in (dict(sizes0=0), dict(summary=0), dict(status=0), dict(c0=0), dict(c0=65), dict(n0=0), dict(n_hi=1),
                dict(n_hi=65536), dict(f=-1), dict(steps=-1), dict(burst=0), dict(burst=256), dict(T=0),
                dict(draws=0), dict(f=40000)):
        assert call(**bad) == P.OOB_EINVAL, bad


def test_instantiation_entry_points_validate_arguments_without_touching_the_gpu():
    ws = P.oob_inst_workspace_size(57, 128, 8)
    assert ws >= 64 * 129 * 10 * 12 and ws % 256 == 0
    assert P.oob_inst_workspace_size(0, 10, 1) == 0
    assert P.oob_inst_workspace_size(3, 5000, 1) == 0
    assert P.oob_inst_workspace_size(3, 10, 255) == 0
    fake = 0x10000  # never dereferenced: every call below fails its host-side checks
    call = lambda **kw: P.oob_inst_count(kw.get("sizes", fake), kw.get("p", 3), kw.get("n0", 0),
                                         kw.get("N_lo", 0), kw.get("N_hi", 10), kw.get("f", 1),
                                         kw.get("ws", fake), kw.get("nbytes", 1 << 20), kw.get("off", fake),
                                         kw.get("st", fake), 0)
    assert call(p=0) == P.OOB_EINVAL
    assert call(N_lo=11) == P.OOB_EINVAL
    assert call(N_hi=4096) == P.OOB_EINVAL
    assert call(f=-1) == P.OOB_EINVAL
    assert call(ws=0) == P.OOB_EINVAL
    assert call(ws=0x10001) == P.OOB_EINVAL          # not 256-byte aligned
    assert call(off=0) == P.OOB_EINVAL
    assert call(st=0) == P.OOB_EINVAL
    assert call(sizes=0, n0=0) == P.OOB_EINVAL        # consecutive sizes need n0 >= 1
    assert call(nbytes=64) == P.OOB_ECAPACITY
    rc = P.oob_inst_enumerate(fake, 3, 0, 0, 10, 1, fake, 1 << 20, 0, 5, fake, fake, 0)
    assert rc == P.OOB_EINVAL                        # capacity > 0 without an output array


def test_distribution_entry_points_validate_arguments_without_touching_the_gpu():
    fake = 0x10000  # never dereferenced: every call below fails its host-side checks or has nothing to do
    solve = lambda **kw: P.oob_dist_solve(kw.get("x", fake), kw.get("count", 1), kw.get("capacity", 1), kw.get("p", 1),
                                          kw.get("tT", fake), kw.get("Q", 1), kw.get("vx", fake), kw.get("slowest", fake),
                                          kw.get("base", 0), kw.get("extra", 0), kw.get("status", fake), 0)
    for bad in (dict(x=0), dict(tT=0), dict(vx=0), dict(slowest=0), dict(status=0), dict(count=-1),
                dict(count=2, capacity=1), dict(p=0), dict(p=1024), dict(Q=0), dict(Q=65536),
                dict(base=fake), dict(extra=fake)):
        assert solve(**bad) == P.OOB_EINVAL, bad
    assert solve(count=0, capacity=0) == P.OOB_OK
    assert P.oob_dist_choose(0, 1, 1, fake, fake, fake, 0) == P.OOB_EINVAL
    assert P.oob_dist_choose(fake, -1, 1, fake, fake, fake, 0) == P.OOB_EINVAL
    assert P.oob_dist_choose(fake, 1, -1, fake, fake, fake, 0) == P.OOB_EINVAL
    assert P.oob_dist_choose(fake, 1, 1, fake, fake, 0, 0) == P.OOB_EINVAL
    assert P.oob_dist_choose(fake, 0, 1, fake, fake, fake, 0) == P.OOB_OK


def test_max_stages_and_workspace_size():
    assert P.oob_plan_max_stages(98, 64, 8, 128) == 98
    assert P.oob_plan_max_stages(12, 4, 1, 8) == 4
    assert P.oob_plan_max_stages(128, 32, 8, 64) == 64
    assert P.oob_plan_max_stages(0, 1, 1, 1) == P.OOB_EINVAL
    small, big = P.oob_plan_workspace_size(12, 4, 1), P.oob_plan_workspace_size(98, 64, 8)
    assert 0 < small < big
    # 40 bytes per record slot of the blocked (u, v) planes plus the per-split minima
    assert 0.5e9 < big < 2e9
    assert P.oob_plan_workspace_size(2000, 4, 1) == 0  # beyond OOB_MAX_L


def test_create_and_call_reject_bad_arguments_without_touching_the_gpu():
    rc, h = P.oob_plan_create(12, 4, 1, 0, 1 << 20)
    assert rc == P.OOB_EINVAL  # null workspace
    rc, h = P.oob_plan_create(12, 4, 1, 0x1001, 1 << 30)
    assert rc == P.OOB_EINVAL  # not 256-byte aligned
    rc, h = P.oob_plan_create(12, 4, 1, 0x10000, 16)
    assert rc == P.OOB_ECAPACITY  # workspace too small
    need = P.oob_plan_workspace_size(12, 4, 1)
    rc, h = P.oob_plan_create(12, 4, 1, 0x10000, need)  # a fake address: never dereferenced here
    assert rc == P.OOB_OK
    prof = B.oob_profile(1, 1, 1, 1)
    out = B.oob_templates()
    for name, _ in B.oob_templates._fields_[:14]:
        setattr(out, name, 1)
    call = lambda **kw: P.oob_plan_templates(h, prof, kw.get("L", 12), kw.get("n_min", 1),
                                             kw.get("n_max", 4), kw.get("M", 1), kw.get("nb", 8),
                                             kw.get("cap", 1 << 30), kw.get("f", 1), out, 0)
    assert call(L=0) == P.OOB_EINVAL
    assert call(n_min=0) == P.OOB_EINVAL
    assert call(n_min=3, n_max=2) == P.OOB_EINVAL
    assert call(M=0) == P.OOB_EINVAL
    assert call(nb=-1) == P.OOB_EINVAL
    assert call(f=-1) == P.OOB_EINVAL
    assert call(cap=0) == P.OOB_EINVAL
    assert call(L=13) == P.OOB_ECAPACITY
    assert call(n_max=5) == P.OOB_ECAPACITY
    assert call(M=2) == P.OOB_ECAPACITY
    out.status = None
    assert call() == P.OOB_EINVAL  # null output pointer
    assert P.load().oob_plan_export_block(h, 1, 0, 1, 1, 1, 1, 1, 1, None) == P.OOB_EINVAL  # no call yet
    assert P.oob_plan_destroy(h) == P.OOB_OK


def test_table_layout_and_task_lists_for_every_depth():
    """Host side of the table layout (block columns shifted so that v = L ends a block) and of the
    per-level task lists (split ranges cut into segments of equal length): for every depth up to 160
    layers and a few beyond, every state of every level lies in exactly one enumerated block and at
    a record of its own, every enumerated block holds a state, the segments of a block partition
    its split range, and the counts stay within the bounds that size a handle's workspace."""
    for L in list(range(1, 161)) + [255, 256, 257, 383]:
        assert P.oob_plan_layout_selftest(L) == 0, L
    assert P.oob_plan_layout_selftest(0) == P.OOB_EINVAL
    assert P.oob_plan_layout_selftest(1 << 20) == P.OOB_EINVAL
    # a workspace sized for a depth serves every smaller depth: sizes grow with every maximum
    sizes = [P.oob_plan_workspace_size(L, 16, 4) for L in range(8, 140)]
    assert all(a <= b for a, b in zip(sizes, sizes[1:]))
