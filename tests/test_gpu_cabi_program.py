"""The C ABI used from a plain C++ program (examples/detox_step_main.cpp: HIP runtime and
libdetox.so only, no Python in the process): its printed results against the oracle, bit for bit
(the inputs are small integers, so every sum is exact)."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import workloads

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


CALLS = os.path.join(ROOT, "examples", "detox_calls_main")


@pytest.mark.parametrize("n,r,d,B", [(45, 3, 6007, 5), (36, 3, 2500, 4), (105, 5, 3001, 7)])
def test_separate_calls_through_the_bare_c_abi(n, r, d, B):
    """examples/detox_calls_main.cpp: filter, block means and every aggregator called one by one
    from C++, the deployed hierarchy and the signSGD pairing; each printed result against the
    oracle (integer inputs: exact everywhere but the iterated geometric median)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    assert os.path.exists(CALLS), "run __graft_entry__.build() first"
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.path.join(ROOT, "paper_1907_12205_amd") + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    run = subprocess.run([CALLS, str(n), str(r), str(d), str(B), "2019"], capture_output=True, text=True, timeout=200, env=env)
    assert run.returncode == 0, run.stderr
    got = {}
    for line in run.stdout.split("\n"):
        if line:
            tag, val = line.split()
            got.setdefault(tag, []).append(val)
    f32 = lambda tag: np.array([int(v, 16) for v in got[tag]], dtype=np.uint32).view(np.float32)
    i32 = lambda tag: np.array([int(v) for v in got[tag]], dtype=np.int64)
    G = _input(n, r, d, 2019)
    V = n // r
    winner, Z = oracle.majority_filter(G, r, materialise=True)
    assert i32("w").tolist() == winner.tolist()
    Zhat = oracle.block_mean(G, winner, B)
    assert f32("z").tobytes() == Zhat.tobytes() and f32("zf").tobytes() == Zhat.tobytes()
    assert f32("med").tobytes() == oracle.coord_median(Zhat).tobytes()
    assert f32("trim").tobytes() == oracle.trimmed_mean(Zhat, B // 4).astype(np.float32).tobytes()
    gm = oracle.geomedian(Zhat, iters=20, eps=1e-8)
    assert np.linalg.norm(f32("gm") - gm) <= 1e-5 * np.linalg.norm(gm)
    D = np.array([int(v, 16) for v in got["dist"]], dtype=np.uint64).view(np.float64).reshape(V, V)
    assert (D == oracle.pairwise_sqdist(Z)).all()
    ref_out, ref_sel, _ = oracle.multikrum(Z, 1, V - 3)
    assert i32("mksel").tolist() == ref_sel.tolist() and f32("mk").tobytes() == ref_out.astype(np.float32).tobytes()
    ref_out, ref_sel = oracle.bulyan(Z, 1)
    assert i32("bulsel").tolist() == ref_sel.tolist() and f32("bul").tobytes() == ref_out.astype(np.float32).tobytes()
    assert f32("medmany").tobytes() == oracle.coord_median(G).tobytes()
    ref_out, ref_w, _, ref_sels = oracle.detox_step_robust_blocks(G, r, 2, "multikrum", 1, -1)
    assert i32("rbw").tolist() == ref_w.tolist()
    sel = i32("rbsel")
    for b, rs in enumerate(ref_sels):
        lo = (b * V) // 2
        assert sel[lo: lo + len(rs)].tolist() == rs.tolist()
    assert np.linalg.norm(f32("rb") - ref_out) <= 1e-6 * np.linalg.norm(ref_out)
    S = workloads.pack_signs(G)
    ref, ref_w = oracle.sign_majority(S, d, r, B)
    assert i32("sw").tolist() == ref_w.tolist()
    pos = np.array([int(v) for v in got["sp"]], dtype=np.int64).astype(np.uint32)
    neg = np.array([int(v) for v in got["sn"]], dtype=np.int64).astype(np.uint32)
    bits = lambda m: np.unpackbits(m.view(np.uint8), bitorder="little")[:d].astype(np.int8)
    assert ((bits(pos) - bits(neg)) == ref).all()
