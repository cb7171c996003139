"""Host logic without a GPU: the launch plans and workspace layouts of csrc/plan.hpp.

A small C++ program (tests/plan_check.cpp, host compiler only) walks a grid of geometries and checks
that every key tile is owned by exactly one split, that no split is empty, that rows are padded to
whole workgroups and that the workspace regions are aligned and disjoint; the sizes it derives from the
layouts are then compared with what the C ABI's mage_workspace_bytes() reports for the same shapes.
"""
import os
import subprocess

from paper_2602_14209_amd import binding as mb

HERE = os.path.dirname(os.path.abspath(__file__))


def test_plans_and_workspace_layouts(tmp_path):
    exe = str(tmp_path / "plan_check")
    subprocess.run(["g++", "-std=c++17", "-O1", "-o", exe, os.path.join(HERE, "plan_check.cpp")], check=True)
    r = subprocess.run([exe], capture_output=True, text=True)
    lines = r.stdout.splitlines()
    fails = [ln for ln in lines if ln.startswith("FAIL")]
    assert r.returncode == 0 and lines[-1] == "OK", "\n".join(fails[:20])
    checked = 0
    for ln in lines:
        if not ln.startswith("NEED"):
            continue
        B, Hq, Hkv, d, L, k, dt, need = (int(x) for x in ln.split()[1:])
        shape = mb.make_shape(B, Hq, Hkv, d, L, k, "bf16" if dt == 1 else "f32")
        got = mb.mage_workspace_bytes(shape)
        # B*G beyond 2^20 rows etc. never occur in this grid: every shape is supported
        assert got == need, (ln, got)
        checked += 1
    assert checked > 1000
