"""The library's host logic (decision core, virtual-time driver, network planner, launch planner) under AddressSanitizer
and UndefinedBehaviorSanitizer.  The host sources are compiled into an executable (`tests/host_sanitize/driver.cpp`) with
both sanitizers on the host side; it reads a text script, drives the C ABI in DARIS_NO_DEVICE | DARIS_VIRTUAL_TIME mode and
prints traces, stage cuts and launch plans, which must equal what the oracle / the regular build give.  A sanitizer report
makes the executable exit non-zero.

Script lines: `init FLAGS`, `partition N_CU N_STREAMS`, `layer OP C_IN C_OUT K STRIDE PAD GROUPS ACT IN_FROM RES_FROM`,
`task PERIOD DEADLINE PRIO DTYPE C H W K AFET...` (registers the layers given since the last task), `et TASK STAGE PART N V...`,
`release T TASK`, `migrate TASK PART`, `run`, `stats TASK`, `shutdown`."""
import os
import subprocess

import numpy as np
import pytest

import paper_2504_08795_amd as D
import workloads as wl
from lib_helpers import Session
from oracle import des, staging
from sched_helpers import golden_flags, load_golden, model_from_golden

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(ROOT, "paper_2504_08795_amd", "csrc")
EXE = os.path.join(HERE, "host_sanitize", "driver_asan_ubsan")
HOST = D.VIRTUAL_TIME | D.NO_DEVICE
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


@pytest.fixture(scope="module")
def driver():
    """Builds the sanitized executable (about a minute; reused while it is newer than every source)."""
    srcs = [os.path.join(CSRC, f) for f in ("aql.cpp", "launch.cpp", "sched_core.cpp", "net_plan.cpp", "daris_api.cpp")] + \
           [os.path.join(HERE, "host_sanitize", "driver.cpp")]
    deps = srcs + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [os.path.join(ROOT, "include", "daris.h")]
    blob, scratch = os.path.join(CSRC, "kernels_blob.o"), os.path.join(CSRC, "static_scratch.hip.o")
    if not (os.path.exists(blob) and os.path.exists(scratch)):
        pytest.skip("library objects not built (python -m paper_2504_08795_amd.build)")
    if not os.path.exists(EXE) or any(os.path.getmtime(d) > os.path.getmtime(EXE) for d in deps):
        hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
        objs = []
        for s in srcs:
            o = os.path.join(HERE, "host_sanitize", os.path.basename(s) + ".san.o")
            subprocess.check_call([hipcc, "-O1", "-g", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-omit-frame-pointer"] + SAN + ["-c", s, "-o", o],
                                  stderr=subprocess.DEVNULL)
            objs.append(o)
        subprocess.check_call([hipcc, "--offload-arch=gfx950"] + SAN + ["-o", EXE] + objs + [blob, scratch, "-L/opt/rocm/lib", "-lhsa-runtime64", "-lpthread", "-ldl"],
                              stderr=subprocess.DEVNULL)
    return EXE


def run_script(exe, lines, tmp_path):
    path = os.path.join(str(tmp_path), "script.txt")
    with open(path, "w") as f:
        f.write("\n".join(lines) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0:exitcode=23", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1:exitcode=24")
    r = subprocess.run([exe, path], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"driver exited with {r.returncode}:\n{r.stderr[-3000:]}"
    out = {"rec": [], "cuts": {}, "plan": {}, "decision": [], "stats": {}}
    for ln in r.stdout.splitlines():
        p = ln.split()
        if p[0] == "rec":
            out["rec"].append(tuple(int(v) for v in p[1:]))
        elif p[0] == "cuts":
            out["cuts"][int(p[1])] = [int(v) for v in p[2:]]
        elif p[0] == "plan":
            out["plan"][(int(p[1]), int(p[2]))] = [int(v) for v in p[3:]]
        elif p[0] == "decision":
            out["decision"].append((int(p[1]), int(p[2])))
        elif p[0] == "stats":
            out["stats"][int(p[1])] = [int(v) for v in p[2:]]
    return out


def plain_task_lines(tasks):
    """Tasks as chains of 1x1 convolutions, one layer per stage (what lib_helpers.register_plain_tasks builds)."""
    lines = []
    for t in tasks:
        k = len(t["afet"])
        for i in range(k):
            lines.append(f"layer 0 4 4 1 1 0 1 0 {i - 1} -1")
        lines.append(f"task {t['period']} {t['deadline']} {t['prio']} 0 4 2 2 {k} " + " ".join(str(a) for a in t["afet"]))
    return lines


def et_lines(et, n_parts):
    return [f"et {i} {j} {k} {len(per_part[k])} " + " ".join(str(int(v)) for v in per_part[k])
            for i, per_stage in enumerate(et) for j, per_part in enumerate(per_stage) for k in range(n_parts)]


def command_lines(cmds):
    return [f"release {c[1]} {c[2]}" if c[0] == "release" else f"migrate {c[2]} {c[3]}" for c in cmds]


@pytest.mark.parametrize("name", ["sched_single_task.json", "sched_hp_preempts_lp.json", "sched_admission_migration.json",
                                  "sched_migration_target_choice.json", "sched_forced_migration_at_boundary.json", "sched_hp_admission.json"])
def test_golden_traces_under_sanitizers(driver, tmp_path, name):
    g, cmds, et, want = load_golden(name)
    lib_flags = {"no_last": D.NO_LAST, "no_prior": D.NO_PRIOR, "no_fixed": D.NO_FIXED, "hp_admission": D.HP_ADMISSION}
    flags = HOST | sum(lib_flags[f] for f in g.get("flags", []))
    lines = [f"init {flags}"] + [f"partition 8 {ns}" for ns in g["partitions"]] + plain_task_lines(g["tasks"]) + \
        et_lines(et, len(g["partitions"])) + command_lines(cmds) + ["run", "shutdown"]
    out = run_script(driver, lines, tmp_path)
    assert out["rec"] == want


@pytest.mark.parametrize("config,load,flags,ns", [(2, 25.0, 0, 1), (3, 18.0, 0, 2), (4, 22.0, D.NO_FIXED, 1), (2, 45.0, D.HP_ADMISSION, 1), (5, 12.0, 0, 1)])
def test_benchmark_shaped_sets_under_sanitizers(driver, tmp_path, config, load, flags, ns):
    ts = wl.make_taskset(config, n_jobs=40 if config != 5 else 25)
    et = wl.virtual_et_table(ts, load_scale=load)
    afet = [[int(np.mean(et[i][j][0][:8])) for j in range(t.n_stages)] for i, t in enumerate(ts.tasks)]
    rel = ts.releases()
    cmds = [("release", t, i) for t, i, _ in rel] + [("migrate", rel[n][0], (n // 7) % len(ts.tasks), (n // 3) % len(ts.partitions)) for n in range(25, len(rel), 61)]
    cmds.sort(key=lambda c: c[1])
    oflags = (des.F_NO_FIXED if flags & D.NO_FIXED else 0) | (des.F_HP_ADMISSION if flags & D.HP_ADMISSION else 0)
    tasks = [des.TaskParam(t.period_ns, t.deadline_ns, t.priority, list(afet[i])) for i, t in enumerate(ts.tasks)]
    m = des.SchedulerModel([ns] * len(ts.partitions), tasks, flags=oflags)
    want = des.run_virtual(m, cmds, et)
    lines = [f"init {HOST | flags}"] + [f"partition 8 {ns}"] * len(ts.partitions) + \
        plain_task_lines([dict(period=t.period, deadline=t.deadline, prio=t.prio, afet=t.afet) for t in tasks]) + et_lines(et, len(ts.partitions)) + \
        command_lines(cmds) + ["run"] + [f"stats {i}" for i in range(len(tasks))] + ["shutdown"]
    out = run_script(driver, lines, tmp_path)
    assert out["rec"] == want and len(want) > 100
    for i, o in enumerate(m.stats()):
        assert out["stats"][i] == [o["released"], o["accepted"], o["completed"], o["missed"], o["rejected_admission"], o["rejected_overrun"], o["ctx"]]


@pytest.mark.parametrize("net,dtype", [("tiny", 0), ("resnet18", 0), ("resnet50", 1), ("vgg16", 0), ("mobilenet_v2", 0), ("resnet50", 0)])
def test_network_planning_under_sanitizers(driver, tmp_path, net, dtype):
    """Registration of every configured network (shape inference, slots, launch plans, joint launches) and its stage split:
    the sanitized build must give the cuts of the oracle and the launch plans of the regular build."""
    layers, shp = wl.build_net(net)
    macs = wl.net_macs(layers, shp)
    legal = staging.legal_cuts(layers)
    ks = [k for k in (1, 2, 3, 4) if k - 1 <= len(legal)]
    lines = [f"init {HOST}", "partition 64 1"]
    for k in ks:
        lines += [f"layer {L.op} {L.c_in} {L.c_out} {L.k} {L.stride} {L.pad} {L.groups} {L.act} {L.in_from} {L.res_from}" for L in layers]
        lines.append(f"task 10000000 10000000 0 {dtype} {shp[0]} {shp[1]} {shp[2]} {k}")
    out = run_script(driver, lines + ["shutdown"], tmp_path)
    with Session(HOST):
        D.daris_create_partition(64)
        dnn, keep = D.make_dnn(layers, None, shp, "bf16" if dtype else "fp32")
        t = D.daris_register_task(dnn, 10**7, 10**7, D.LP)
        plans = [list(D.daris_get_launch_plan(t, l).values()) for l in range(len(layers))]
    for i, k in enumerate(ks):
        assert out["cuts"][i] == staging.split(macs, legal, k), (net, k)
        for l in range(len(layers)):
            assert out["plan"][(i, l)] == plans[l], (net, l)
