"""The host-only half of the library (network validation, cost model, planner, stage layout, schedule creation) built
with AddressSanitizer and UndefinedBehaviorSanitizer on the host side and driven through the C ABI by
tests/host_sanitize.cpp: every workload, valid and invalid plans.  No GPU is touched; the results must equal the
regular library's."""
import glob
import os
import subprocess

import pytest

import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2207_11019_amd", "csrc")
FIELDS = ("kind", "cin", "cout", "kh", "kw", "stride", "pad", "h_in", "w_in", "flags", "src", "add_src", "cut_allowed_after",
          "d_in", "kd", "pad_d")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    exe = str(out / "host_sanitize")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
    flags = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument"]
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.cpp")) + glob.glob(os.path.join(CSRC, "*.hip"))) + [os.path.join(ROOT, "tests", "host_sanitize.cpp")]
    procs = []
    for s in srcs:
        obj = str(out / (os.path.basename(s) + ".o"))
        procs.append((obj, subprocess.Popen(["hipcc", "-x", "hip", "-c", s, "-o", obj] + flags + san, stderr=subprocess.PIPE, text=True)))
    for obj, p in procs:
        _, err = p.communicate()
        assert p.returncode == 0, err[-2000:]
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe] + [o for o, _ in procs])
    return exe


def _net(layers, lpm):
    arr = lpm.layers_from_dicts(layers)
    lines = ["net %d" % len(arr)]
    for l in arr:
        lines.append(" ".join(str(getattr(l, f)) for f in FIELDS))
    return lines


def test_host_code_under_sanitizers(driver):
    import paper_2207_11019_amd as lpm
    cmds, expect = [], []
    configs = dict(wl.CONFIGS, **wl.EXTRA_CONFIGS)
    for name, (builder, batch, M, Z, dt, fixed) in configs.items():
        L = builder()
        m = batch // M
        cp = dict(lpm.MI355X_COST[dt], link_byte_per_us=153000, microbatch=m, n_microbatch=M)
        cmds += _net(L, lpm)
        expect.append("net %d" % len(L))
        cmds.append("cost %d %d %d %d %d %d" % (cp["flop_per_us"], cp["hbm_byte_per_us"], cp["link_byte_per_us"], cp["elem_bytes"], m, M))
        expect.append("cost ok")
        allowed = sum(l["cut_after"] for l in L[:-1])
        for z in range(1, min(5, allowed + 1) + 1):
            starts, costs = lpm.lpm_partition(L, z, cp)
            cmds.append("plan %d" % z)
            expect.append("plan 0 " + " ".join(map(str, starts)) + " | " + " ".join(map(str, costs)))
            cmds.append("fixed %d %s" % (z, " ".join(map(str, starts))))
            expect.append("fixed 0 " + " ".join(map(str, starts)) + " | " + " ".join(map(str, costs)))
        # plans that point outside the layer list, reversed plans, too many stages
        for bad in ([0, 100000, len(L)], [0, len(L), len(L)], [0, len(L) + 5, len(L)], [0, -3, len(L)]):
            cmds.append("fixed 2 %s" % " ".join(map(str, bad)))
            expect.append("fixed -6")
        cmds.append("plan %d" % (len(L) + 1)); expect.append("plan -1")
        cmds.append("plan 0"); expect.append("plan -1")
        for i in (0, len(L) // 2, len(L) - 1):
            cmds.append("lcost %d" % i); expect.append("lcost 0 %d" % lpm.lpm_layer_cost(L, i, cp))
        cmds.append("lcost %d" % len(L)); expect.append("lcost -1 0")
        lc = [lpm.lpm_layer_cost(L, i, cp) for i in range(len(L))]
        zz = min(Z, allowed + 1)
        cmds.append("costs %d %s" % (zz, " ".join(map(str, lc))))
        expect.append("costs 0 " + " ".join(map(str, lpm.lpm_partition_costs(L, zz, cp, lc)[0])) + " | " +
                      " ".join(map(str, lpm.lpm_partition_costs(L, zz, cp, lc)[1])))
        dtype = lpm.BF16 if dt == "bf16" else lpm.F32
        plan = list(fixed) if fixed is not None else lpm.lpm_partition(L, Z, cp)[0]
        for z in range(len(plan) - 1):
            s = lpm.Stage(L, plan[z], plan[z + 1], m, dtype)
            cmds.append("stage %d %d %d %d" % (plan[z], plan[z + 1], m, dtype))
            expect.append("stage 0 %d %d %d %d %d %d %d %d" % (s.param_bytes, s.lowp_bytes, s.grad_bytes, s.stash_bytes, s.fwd_ws_bytes,
                                                                s.bwd_ws_bytes, s.in_bytes, s.out_bytes))
        cmds.append("stage %d %d %d %d" % (0, len(L) + 3, m, dtype)); expect.append("stage -1")
        cmds.append("stage %d %d %d %d" % (2, 2, m, dtype)); expect.append("stage -1")
        # (creating a schedule makes HIP events: without a GPU the call gets as far as that and reports LPM_EHIP)
        cmds.append("sched %d %s %d %d %d 2" % (len(plan) - 1, " ".join(map(str, plan)), m, M, dtype)); expect.append(("sched 0", "sched -5"))
        cmds.append("sched %d %s %d %d %d 9" % (len(plan) - 1, " ".join(map(str, plan)), m, M, dtype)); expect.append("sched -1")
    r = subprocess.run([driver], input="\n".join(cmds) + "\n", capture_output=True, text=True, timeout=300)
    assert "AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr and "LeakSanitizer" not in r.stderr, r.stderr[-4000:]
    assert r.returncode == 0, (r.returncode, r.stderr[-2000:])
    got = r.stdout.strip().split("\n")
    assert got[-1].startswith("done")
    assert len(got) - 1 == len(expect), (len(got), len(expect))
    for g, e in zip(got, expect):
        assert g.startswith(e), (g, e)          # (str.startswith takes a tuple of alternatives)
