#!/usr/bin/env python3
"""Writes tests/golden/instance_times.json: the measured launch time of every compiled kernel instance that
serves each benchmark shape (the seven benchmark configurations, the paper's five unbalanced GEMMs and its
three Conv2d shapes), on one MI355X.

This is a MEASUREMENT fixture, not oracle output: it is what pins the library's analytical cost model (which
instance it ranks first, and how its ranking correlates with the hardware) to something that shares no code
with it.  tests/test_cost_model_measured.py reads it on the CPU.

Run on the GPU machine from the repository root, after building:
    python tests/golden/make_instance_times.py
Protocol per (shape, instance): launches that settle the shader clock (15 ms), then the median of 3
event-bracketed batches of at least 10 launches (about 3 ms each).  Instances the cost model prices above
SKIP_FACTOR times its cheapest instance for the shape are not timed (they would only lengthen the run).
Boxes differ by a few percent, and not uniformly over the instances (one box ran the 256x256 tiles 5 % faster
than another and the 128x128 tiles of 64x32 waves the same), so the file keeps every run: a new run on the same
instance list is appended (`us_runs`), and `us` is the mean over the runs.
"""
import json
import os
import subprocess
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
SKIP_FACTOR = 6.0
PROBLEM_FIELDS = ("op", "in_dtype", "out_dtype", "transA", "transB", "batch", "M", "N", "K", "n", "c", "h", "w", "k", "r", "s",
                  "stride", "pad")


def merge(path, new):
    """Append this run to the runs the file already holds, if they describe the same instances."""
    for sh in new["shapes"].values():
        for r in sh["instances"].values():
            r["us_runs"] = [r["us"]]
    new["runs"] = [{"device": new["device"], "commit": new["commit"]}]
    if not os.path.exists(path):
        return new
    old = json.load(open(path))
    try:
        for name, sh in new["shapes"].items():
            for idx, r in sh["instances"].items():
                o = old["shapes"][name]["instances"].get(idx)
                if o is None:
                    continue
                if o["coords"] != r["coords"] or o["stages"] != r["stages"] or o["direct"] != r["direct"]:
                    raise KeyError(idx)
                r["us_runs"] = list(o.get("us_runs", [o["us"]])) + r["us_runs"]
                r["us"] = round(sum(r["us_runs"]) / len(r["us_runs"]), 3)
        new["runs"] = list(old.get("runs", [{"device": old.get("device"), "commit": old.get("commit")}])) + new["runs"]
    except KeyError:
        print("the existing file describes other instances: starting over", flush=True)
        for sh in new["shapes"].values():
            for r in sh["instances"].values():
                r["us_runs"] = r["us_runs"][-1:]
                r["us"] = r["us_runs"][0]
        new["runs"] = new["runs"][-1:]
    return new


def main():
    import torch
    from bench import Case
    from paper_2502_11407_amd import binding as gs, inputs

    shapes = list(inputs.all_configs().items())
    shapes += [("u%d" % i, None) for i in range(len(inputs.UNBALANCED_GEMMS))]
    shapes += [("C%d" % (i + 1), None) for i in range(len(inputs.PAPER_CONVS))]
    out = {"device": torch.cuda.get_device_properties(0).name,
           "commit": subprocess.run(["git", "rev-parse", "HEAD"], capture_output=True, text=True, cwd=ROOT).stdout.strip() or "unknown",
           "command": "python tests/golden/make_instance_times.py",
           "protocol": "clock settle 15 ms, median of 3 batches of >= 10 launches (~3 ms each), HIP events on the launch stream",
           "num_instances": gs.num_instances(), "shapes": {}}
    t_all = time.time()
    for name, wl in shapes:
        if wl is None:
            wl = inputs.unbalanced_gemm(int(name[1:])) if name[0] == "u" else inputs.paper_conv(int(name[1:]) - 1)
        c = Case(gs, inputs, wl)
        p = c.p
        picked = c.sched.kernel_id
        cands = []
        for idx in range(gs.num_instances()):
            s = gs.instance_schedule(idx, p)
            if s is None:
                continue
            if c.is_gemm and s.direct_lds and wl.K % s.tile[2][0] != 0:
                continue
            us = gs.predict_us(s, p)
            if us > 0:
                cands.append((us, idx, s))
        cheapest = min(u for u, _, _ in cands)
        rows = {}
        for us, idx, s in cands:
            if us > SKIP_FACTOR * cheapest and idx != picked:
                continue
            c.sched, c.ws = s, None
            if not c.is_gemm:
                c.ws = gs.conv_workspace(p, s)
            try:
                ms = c.time_median_ms(batches=3, min_launches=10, settle_ms=15.0, batch_ms=3.0)
            except gs.GensorError as e:          # an instance that cannot take this problem after all (alignment, extent limits)
                print(name, "instance", idx, "refused:", e, flush=True)
                continue
            rows[str(idx)] = {"us": round(ms * 1e3, 3), "predicted_us": round(us, 3),
                              "coords": [s.tile[0][0], s.tile[1][0], s.tile[2][0], s.tile[0][1], s.tile[1][1], s.tile[2][1],
                                         s.vthread[0], s.vthread[1]],
                              "stages": s.stages, "direct": s.direct_lds, "vec": 1 if s.vec_bytes == 16 else 0}
        best = min(rows, key=lambda k: rows[k]["us"])
        out["shapes"][name] = {"workload": wl.name, "problem": {f: int(getattr(p, f)) for f in PROBLEM_FIELDS},
                               "picked_when_measured": picked, "instances": rows}
        print("%s: %d instances timed, best %s %.1f us, picked %d %.1f us (%.1f s so far)" % (
            name, len(rows), best, rows[best]["us"], picked, rows[str(picked)]["us"], time.time() - t_all), flush=True)
        del c, wl
        torch.cuda.empty_cache()
    path = os.path.join(ROOT, "tests", "golden", "instance_times.json")
    out = merge(path, out)
    with open(path, "w") as f:
        json.dump(out, f, indent=0, sort_keys=True)
    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", "instance_times.json"), "w") as f:
        json.dump(out, f, indent=0, sort_keys=True)
    print("wrote", path, flush=True)


if __name__ == "__main__":
    main()
