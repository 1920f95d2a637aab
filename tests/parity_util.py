"""Element-by-element comparison of the HIP path's results with the CPU oracle's."""
import numpy as np

TEMPLATE_KEYS = ("feasible", "S", "kstar", "T", "T1", "T2", "T3", "tmax")


def canonical_templates(res: dict, count: int, f: int) -> bytes:
    """Canonical byte form of everything compare_templates compares, for stored digests: the
    per-template scalars, the stage lists of every template, the coverage header and array, and
    the work counters."""
    parts = [np.asarray(res[k])[:count].astype("<i8").tobytes() for k in TEMPLATE_KEYS]
    off = np.asarray(res["stage_off"])[:count + 1].astype("<i8")
    total = int(off[count])
    parts.append(off.tobytes())
    parts.append(np.asarray(res["stage_gpus"])[:total].astype("<i8").tobytes())
    parts.append(np.asarray(res["stage_begin"])[:total + count].astype("<i8").tobytes())
    parts.append(np.asarray(res["cover_hdr"]).astype("<i8").tobytes())
    parts.append(np.asarray(res["cover_maxpipes"])[:max(count, f + 1)].astype("<i8").tobytes())
    parts.append(np.array([res["states"], res["candidates"]], dtype="<i8").tobytes())
    return b"".join(parts)


def compare_templates(got: dict, want: dict, count: int):
    """Bit-exact: per-template scalars, stage lists, coverage, work counters."""
    assert int(got["status"][0]) == 0, f"device status {int(got['status'][0])}"
    for k in TEMPLATE_KEYS:
        g, w = np.asarray(got[k])[:count], np.asarray(want[k])[:count]
        assert np.array_equal(g.astype(np.int64), w.astype(np.int64)), \
            f"{k}: first mismatch at template {int(np.flatnonzero(g != w)[0])}: {g} vs {w}"
    assert np.array_equal(np.asarray(got["stage_off"])[:count + 1],
                          np.asarray(want["stage_off"])[:count + 1])
    total = int(want["stage_off"][count])
    assert np.array_equal(np.asarray(got["stage_gpus"])[:total], np.asarray(want["stage_gpus"])[:total])
    assert np.array_equal(np.asarray(got["stage_begin"])[:total + count],
                          np.asarray(want["stage_begin"])[:total + count])
    assert np.array_equal(np.asarray(got["cover_hdr"]), np.asarray(want["cover_hdr"]))
    ln = len(want["cover_maxpipes"])
    assert np.array_equal(np.asarray(got["cover_maxpipes"])[:ln], np.asarray(want["cover_maxpipes"]))
    assert (got["states"], got["candidates"]) == (want["states"], want["candidates"])


def compare_block(gblk: dict, oblk: dict, S: int, L: int):
    """One (S', delta) block: existence, T, T1, T3, tmax, k*, and the winning (s, k, m) of every
    state; padding entries must read as "no such state".  gblk arrays are [n, n] indexed
    [u, v - S'], oblk arrays are [L+1, L+1] indexed [u, v]."""
    n = L - S + 1
    assert gblk["T"].shape == (n, n)
    u = np.arange(n)[:, None]
    j = np.arange(n)[None, :]
    v = j + S
    state = j >= u
    ex = np.zeros((n, n), dtype=bool)
    ex[state] = oblk["exists"][np.broadcast_to(u, (n, n))[state], np.broadcast_to(v, (n, n))[state]] != 0
    gex = np.isfinite(gblk["T"])
    assert np.array_equal(gex, ex), f"existence differs at S'={S}: {np.argwhere(gex != ex)[:5]}"
    uu, vv = np.broadcast_to(u, (n, n))[ex], np.broadcast_to(v, (n, n))[ex]
    for key in ("T", "T1", "T3", "tmax"):
        g = gblk[key][ex]
        bad = ~((g == np.floor(g)) & (np.abs(g) < 2.0**53))
        if bad.any():
            i = int(np.flatnonzero(bad)[0])
            raise AssertionError(f"{key} is not an exact integer at S'={S} u={int(uu[i])} v={int(vv[i])}: "
                                 f"{g[i]!r} (oracle {int(oblk[key][uu[i], vv[i]])}); {int(bad.sum())} such records")
        w = oblk[key][uu, vv]
        if not np.array_equal(g.astype(np.int64), w):
            i = int(np.flatnonzero(g.astype(np.int64) != w)[0])
            raise AssertionError(f"{key} differs at S'={S} u={int(uu[i])} v={int(vv[i])}: {int(g[i])} vs oracle "
                                 f"{int(w[i])}; {int((g.astype(np.int64) != w).sum())} such records")
    assert np.array_equal(gblk["kstar"][ex], oblk["kstar"][uu, vv]), f"kstar differs at S'={S}"
    if S > 1:
        ch = gblk["choice"][ex]
        assert np.array_equal(ch & 1023, oblk["s"][uu, vv]), f"s differs at S'={S}"
        assert np.array_equal((ch >> 10) & 2047, oblk["k"][uu, vv]), f"k differs at S'={S}"
        assert np.array_equal((ch >> 21) & 1023, oblk["m"][uu, vv]), f"m differs at S'={S}"
    return int(ex.sum())


def canonical_oracle_block(oblk: dict, S: int, L: int):
    """Canonical byte form of one oracle block (states in row-major (u, v) order)."""
    n = L - S + 1
    u, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    st = j >= u
    uu, vv = u[st], (j + S)[st]
    ex = oblk["exists"][uu, vv] != 0
    parts = [ex.astype(np.uint8).tobytes()]
    for key in ("T", "T1", "T3", "tmax"):
        parts.append(oblk[key][uu, vv][ex].astype("<i8").tobytes())
    for key in ("kstar", "s", "k", "m"):
        parts.append(oblk[key][uu, vv][ex].astype("<i4").tobytes())
    return b"".join(parts)


def canonical_gpu_block(gblk: dict, S: int, L: int):
    """Same canonical form from the HIP path's block arrays."""
    n = L - S + 1
    u, j = np.meshgrid(np.arange(n), np.arange(n), indexing="ij")
    st = j >= u
    ex = np.isfinite(gblk["T"][st])
    parts = [ex.astype(np.uint8).tobytes()]
    for key in ("T", "T1", "T3", "tmax"):
        parts.append(gblk[key][st][ex].astype("<i8").tobytes())
    ch = gblk["choice"][st][ex]
    parts.append(gblk["kstar"][st][ex].astype("<i4").tobytes())
    for val in (ch & 1023, (ch >> 10) & 2047, (ch >> 21) & 1023):
        parts.append(val.astype("<i4").tobytes())
    return b"".join(parts)
