"""The C-ABI from plain C: tests/c_client/client.c (gcc, no Python, no torch, no HIP call of its own) loads a
scenario, searches it through chm_search_best, chm_search_best_static, a bounded search and chm_search_best_batch on
the default stream, and its printed plans must be the oracle's."""
import os
import subprocess

import numpy as np
import pytest

from oracle import oracle as O
from paper_2508_21613_amd import synth

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _write(sc, path):
    with open(path, "w") as fh:
        head = [sc["L"], sc["PP"], sc["DP"], sc["M"], len(sc["failed_nodes"]), sc["comm_us"], sc["mem_cap_mib"],
                sc.get("reroute_cap", 0), sc["horizon_steps"]] + list(sc["reconf_us"])
        fh.write(" ".join(str(int(x)) for x in head) + "\n")
        fh.write("%d %d\n" % (sc["xfer_us_per_mib"], 0 if sc.get("speed_q16") is None else 1))
        for key in ("fwd_us", "bwd_us", "mem_mib", "failed_nodes"):
            fh.write(" ".join(str(int(x)) for x in sc[key]) + "\n")
        if sc.get("speed_q16") is not None:
            fh.write(" ".join(str(int(x)) for x in sc["speed_q16"]) + "\n")


def _line(what, rc, b):
    reroute = ",".join(str(x) for row in b["reroute"] for x in row)
    return "%s rc=%d index=%d cost=%d strategy=%d stages=%d cuts=%s t_step=%d t_trans=%d reroute=%s" % (
        what, rc, b["index"], b["cost"], b["strategy"], b["stages"], ",".join(str(x) for x in b["cuts"]), b["t_step_us"],
        b["t_trans_us"], reroute)


@pytest.mark.parametrize("name", ["config1", "hetero_two_failures"])
def test_plain_c_caller(tmp_path, name):
    sc = synth.config1() if name == "config1" else synth.small_random(2008, L=14, PP=6, DP=4, M=7, n_failed=4, hetero=True, cap=9)
    exe = tmp_path / "client"
    lib_dir = os.path.join(ROOT, "paper_2508_21613_amd")
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-I", os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "c_client", "client.c"),
                    "-o", str(exe), "-L", lib_dir, "-lchm", "-Wl,-rpath," + lib_dir], check=True)
    path = tmp_path / "scenario.txt"
    _write(sc, str(path))
    out = subprocess.run([str(exe), str(path)], check=True, capture_output=True, text=True, timeout=120).stdout.splitlines()
    o = O.Scenario(sc)
    assert out[0] == "space families=%d plans=%d" % (len(o.families), o.n_plans)
    rc_all, best_all = o.search(7)
    want = {"exhaustive": (rc_all, best_all), "static": (rc_all, best_all), "bounded": (rc_all, best_all), "batch": (rc_all, best_all)}
    for k in range(3):
        want["strategy%d" % k] = o.search(1 << k)
    seen = set()
    for line in out[1:]:
        what = line.split(" ")[0]
        rc, b = want[what]
        seen.add(what)
        if rc == O.OK:
            assert line == _line(what, rc, b), (line, _line(what, rc, b))
        else:
            assert line.startswith("%s rc=%d " % (what, rc)), line
    assert seen == set(want)
