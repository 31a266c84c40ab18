"""The C ABI used from a plain C++ program (examples/detox_step_main.cpp: HIP runtime and
libdetox.so only, no Python in the process): its printed results against the oracle, bit for bit
(the inputs are small integers, so every sum is exact)."""
import os
import subprocess

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROGRAM = os.path.join(ROOT, "examples", "detox_step_main")
AGG = {"multikrum": 0, "bulyan": 1, "coord_median": 2, "geomedian": 3, "trimmed_mean": 4}


def _input(n, r, d, seed):
    """The matrix the program builds (see its header comment)."""
    state = seed & 0xFFFFFFFF
    G = np.empty((n, d), dtype=np.float32)
    c = np.arange(d, dtype=np.uint64)
    for g in range(n // r):
        state = (1103515245 * state + 12345) & 0x7FFFFFFF
        a = state % 29 + 1
        state = (1103515245 * state + 12345) & 0x7FFFFFFF
        b = state % 31
        row = ((a * c + b) % 31).astype(np.float32) - np.float32(15.0)
        for k in range(r):
            G[g * r + k] = 9.0 if (r >= 3 and g % 3 == 0 and k == 1) else row
    return G


@pytest.mark.parametrize("n,r,d,B,agg,f,m", [(45, 3, 10007, 5, "multikrum", 1, 3), (45, 3, 4099, 5, "coord_median", 0, 0),
                                             (45, 3, 5000, 15, "bulyan", 1, 0), (27, 3, 777, 3, "trimmed_mean", 1, 0),
                                             (30, 5, 2048, 6, "multikrum", 1, 2)])
def test_program_output_equals_the_oracle(n, r, d, B, agg, f, m):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    assert os.path.exists(PROGRAM), "run __graft_entry__.build() first"
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.path.join(ROOT, "paper_1907_12205_amd") + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([PROGRAM, str(n), str(r), str(d), str(B), str(AGG[agg]), str(f), str(m), "2019"],
                         capture_output=True, text=True, timeout=100, env=env)
    assert run.returncode == 0, run.stderr
    lines = run.stdout.split("\n")
    winner = [int(l[2:]) for l in lines if l.startswith("w ")]
    out = np.array([int(l[2:], 16) for l in lines if l.startswith("x ")], dtype=np.uint32).view(np.float32)
    G = _input(n, r, d, 2019)
    kw = dict(f=f) if agg in ("bulyan", "trimmed_mean") else (dict(f=f, m=m) if agg == "multikrum" else {})
    ref_out, ref_w, _ = oracle.detox_step(G, r, B, agg, **kw)
    assert winner == ref_w.tolist()
    assert out.tobytes() == ref_out.astype(np.float32).tobytes()
