"""Writes the stored expected values for the full-size configurations.

Calls only the CPU oracle (oracle/) and the input generators (inputs/).  Output:
tests/golden/<name>_expected.json with the templates, the coverage and one SHA-256 per
stage-count level over the canonical form of every state record of that level
(tests/parity_util.canonical_oracle_block).  Takes minutes for configuration 4.

    python tests/golden/make_golden.py cfg4
    python tests/golden/make_golden.py cfg4_paper_nb     (configuration 4 with N_b = 4 S' per state)
    python tests/golden/make_golden.py cfg5 <instance> [<instance> ...]
    python tests/golden/make_golden.py cfg4_exact        (exact minimum of the cost per template, about a minute)
    python tests/golden/make_golden.py cfg5_all [threads] (all 256 instances of the batched configuration: per
                                                          instance T, S, feasibility and one SHA-256 over everything
                                                          parity_util.compare_templates compares; about an hour)
"""
import hashlib
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))
sys.path.insert(0, os.path.dirname(HERE))

import inputs  # noqa: E402
from oracle import capi  # noqa: E402
import parity_util as PU  # noqa: E402


def expected(inp) -> dict:
    t0 = time.time()
    o = capi.Oracle(inp)
    t = o.templates(inp.n_min, inp.n_max)
    c = capi.coverage(t["feasible"], inp.n_min, inp.f)
    out = {k: [int(x) for x in v] for k, v in t.items()}
    out["cover_hdr"] = [int(x) for x in c["hdr"]]
    out["cover_maxpipes"] = [int(x) for x in c["maxpipes"]]
    out["states"], out["candidates"] = int(o.states), int(o.candidates)
    digests = {}
    for S in range(1, o.Smax + 1):
        h = hashlib.sha256()
        for delta in range(o.D):
            if o.valid(S, delta):
                h.update(PU.canonical_oracle_block(o.block(S, delta), S, inp.L))
        digests[str(S)] = h.hexdigest()
    out["level_sha256"] = digests
    out["_meta"] = {"name": inp.name, "L": inp.L, "n_min": inp.n_min, "n_max": inp.n_max,
                    "M": inp.gpus_per_node, "microbatches": inp.microbatches, "f": inp.f,
                    "oracle_seconds": round(time.time() - t0, 1),
                    "written_by": "tests/golden/make_golden.py (CPU oracle only)"}
    o.close()
    return out


def main():
    which = sys.argv[1]
    if which == "cfg4":
        inp = inputs.config(4)
        json.dump(expected(inp), open(os.path.join(HERE, "cfg4_expected.json"), "w"))
    elif which == "cfg4_paper_nb":
        import dataclasses

        inp = dataclasses.replace(inputs.config(4), microbatches=0, name="cfg4_gpt175b_paper_nb")
        json.dump(expected(inp), open(os.path.join(HERE, "cfg4_paper_nb_expected.json"), "w"))
    elif which == "cfg5":
        insts = inputs.config(5)
        for idx in map(int, sys.argv[2:]):
            json.dump(expected(insts[idx]),
                      open(os.path.join(HERE, f"cfg5_{idx}_expected.json"), "w"))
    elif which == "cfg5_all":
        threads = int(sys.argv[2]) if len(sys.argv) > 2 else 0
        insts = inputs.config(5)
        path = os.path.join(HERE, "cfg5_all_templates.json")
        done = json.load(open(path))["instances"] if os.path.exists(path) else {}
        t0 = time.time()
        for idx, inp in enumerate(insts):
            if str(idx) in done:
                continue
            t = capi.plan(inp, threads)
            cnt = inp.n_max - inp.n_min + 1
            done[str(idx)] = {"name": inp.name, "L": inp.L, "f": inp.f,
                              "feasible": [int(x) for x in t["feasible"]], "S": [int(x) for x in t["S"]],
                              "T": [int(x) for x in t["T"]],
                              "sha256": hashlib.sha256(PU.canonical_templates(t, cnt, inp.f)).hexdigest()}
            print(f"instance {idx} L={inp.L} f={inp.f}: {time.time() - t0:.0f} s", flush=True)
            json.dump({"source": "oracle/capi.plan on inputs.config(5); sha256 over "
                                 "tests/parity_util.canonical_templates", "instances": done},
                      open(path + ".tmp", "w"))
            os.replace(path + ".tmp", path)
    elif which == "cfg4_exact":
        from oracle import exact_minimum

        inp = inputs.config(4)
        json.dump({"source": "oracle/exact_minimum.py on inputs.config(4)", "n_min": inp.n_min,
                   "exact_minimum": exact_minimum.exact_minimum(inp)},
                  open(os.path.join(HERE, "cfg4_exact_minimum.json"), "w"))
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main()
