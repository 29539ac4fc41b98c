"""The plain-C demo of the boundary: built by the build step with gcc -std=c99, run on the GPU."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
DEMO = os.path.join(ROOT, "examples", "c_abi_demo")


def test_c_demo_source_is_plain_c():
    src = open(DEMO + ".c").read()
    assert '#include "tardis.h"' in src
    for word in ("class ", "template", "namespace", "std::", "torch"):
        assert word not in src


@pytest.mark.gpu
def test_c_demo_identities_hold_on_the_gpu():
    """Empty ranges: every neuron repaired, the folded path equals the unmodified FFN; identity
    activation with its exact line: nothing flagged, same equality.  (No reference needed.)"""
    assert os.path.exists(DEMO), "run python -m paper_2501_10054_amd.build first"
    import torch
    if torch.cuda.is_initialized():
        pytest.skip("this process already drives the GPU; the demo is started from a process that does not")
    r = subprocess.run([DEMO], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip().endswith("c_abi_demo: OK")
