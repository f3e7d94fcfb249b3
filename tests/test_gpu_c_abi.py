"""The C ABI called from a C program (tests/c_abi/gcn_layer_from_c.c, built by build()): preprocessing,
plan, one GCN layer forward and backward, then one GAT layer in every caching variant, each checked inside
the program against the dense definition."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi")


def test_gcn_layer_from_a_c_program():
    exe = os.path.join(HERE, "gcn_layer_from_c")
    assert os.path.exists(exe), "tests/c_abi/gcn_layer_from_c is not built: run __graft_entry__.build()"
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.startswith("ok: GCN layer from C")
    assert r.stdout.count("ok: GAT layer from C") == 4, r.stdout
