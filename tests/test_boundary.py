"""CPU checks of the C-ABI boundary: the library loads, exports every declared symbol, sizes
workspaces, and rejects bad arguments on the host before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dx():
    import paper_1907_12205_amd as dx
    if not os.path.exists(dx.library_path()):
        from paper_1907_12205_amd import build
        build.build()
    return dx


def test_exports_match_the_header(dx):
    header = open(os.path.join(ROOT, "include", "detox.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:detox|robust)_[a-z_0-9]+)\s*\(", body))
    assert {"detox_majority_filter", "detox_block_mean", "robust_multikrum", "robust_bulyan",
            "robust_coord_median", "robust_geomedian"} <= declared
    L = ctypes.CDLL(dx.library_path())
    for name in declared:
        assert hasattr(L, name), name


def test_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_1907_12205_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower().replace("test infrastructure", ""), f


def test_workspace_sizes(dx):
    assert dx.workspace_bytes("block_mean", 15, 1000) == 0
    assert dx.workspace_bytes("coord_median", 15, 1000) == 0
    assert dx.workspace_bytes("filter", 15, 1000) % 256 == 0 and dx.workspace_bytes("filter", 15, 1000) >= 15 * 8
    a, b = dx.workspace_bytes("multikrum", 5, 1000), dx.workspace_bytes("multikrum", 45, 1000)
    assert 0 < a and 0 < b
    assert dx.workspace_bytes("multikrum", 129, 1000) == 0          # beyond the build's limit
    assert dx.workspace_bytes("step", 45, 1000, 5) == dx.workspace_bytes("filter", 45, 1000) + a
    # the hierarchy with a robust aggregator inside vote groups: sized by its own selector, from the
    # number of votes and of vote groups; 15 votes carry the in-pass Gram workspace on top
    rb15, rb21 = dx.workspace_bytes("step_robust_blocks", 15, 1000, 2), dx.workspace_bytes("step_robust_blocks", 21, 1000, 3)
    assert rb15 > dx.workspace_bytes("filter", 15, 1000) + dx.workspace_bytes("multikrum", 8, 1000) + dx.workspace_bytes("multikrum", 15, 1000)
    assert rb21 > dx.workspace_bytes("filter", 21, 1000) + dx.workspace_bytes("multikrum", 7, 1000)
    assert rb15 % 256 == 0 and dx.workspace_bytes("step_robust_blocks", 15, 1000, 16) == 0      # more groups than votes
    # the Gram partial sums are one tile set per wavefront: the size does not grow with d
    assert dx.workspace_bytes("multikrum", 105, 25_000_000) == dx.workspace_bytes("multikrum", 105, 1000)


def test_argument_validation_happens_on_the_host(dx):
    L = dx.lib()
    OK, EINVAL, EPRECOND, EWS = 0, 1, 2, 3
    p = ctypes.c_void_p(256)      # never dereferenced: every call below must fail before any launch
    big = 1 << 30
    assert L.detox_majority_filter(None, 9, 10, 10, 3, None, p, None, 0, p, big, None) == EINVAL
    assert L.detox_majority_filter(p, 9, 10, 9, 3, None, p, None, 0, p, big, None) == EINVAL      # ld < d
    assert L.detox_majority_filter(p, 10, 10, 10, 3, None, p, None, 0, p, big, None) == EINVAL    # r does not divide n
    assert L.detox_majority_filter(p, 24, 10, 10, 12, None, p, None, 0, p, big, None) == EINVAL   # r beyond the limit
    assert L.detox_majority_filter(p, 9, 10, 10, 3, None, p, None, 0, None, 0, None) == EWS
    assert L.detox_majority_filter(p, 9, 10, 10, 3, None, p, None, 0, ctypes.c_void_p(260), big, None) == EWS
    assert L.detox_majority_filter(p, 9, 10, 10, 3, None, p, None, 0, p, 8, None) == EWS
    assert L.detox_block_mean(p, 10, 10, p, 5, 6, None, p, 10, None) == EINVAL                    # more blocks than votes
    assert L.robust_multikrum(p, 6, 10, 10, 2, 1, p, p, None, p, big, None) == EPRECOND           # 6 < 2*2+3
    assert L.robust_multikrum(p, 7, 10, 10, 2, 6, p, p, None, p, big, None) == EPRECOND           # m > count - f
    assert L.robust_multikrum(p, 7, 10, 10, 2, 5, p, p, None, p, 16, None) == EWS
    assert L.robust_multikrum(p, 200, 10, 10, 2, 5, p, p, None, p, big, None) == EINVAL
    assert L.robust_bulyan(p, 10, 10, 10, 2, p, p, p, big, None) == EPRECOND                      # 10 < 4*2+3
    assert L.robust_coord_median(p, 0, 10, 10, p, None) == EINVAL
    assert L.robust_geomedian(p, 7, 10, 10, 50, ctypes.c_double(0.0), p, p, big, None) == EINVAL  # eps must be > 0
    assert L.detox_step(p, 45, 10, 10, 3, 5, None, 5, None, 1, 1, -1, 50, ctypes.c_double(1e-8),
                        p, p, 10, p, p, p, big, None) == EPRECOND                                 # Bulyan on 5 rows, f = 1
    assert L.detox_step(p, 45, 10, 10, 3, 5, None, 16, None, 0, 1, 3, 50, ctypes.c_double(1e-8),
                        p, p, 10, p, p, p, big, None) == EINVAL                                   # B > n/r
    assert L.detox_step(p, 45, 10, 10, 3, 5, None, 5, None, 0, -1, -1, 50, ctypes.c_double(1e-8),
                        p, p, 10, p, p, p, big, None) == EPRECOND      # derived f = 2 needs 7 rows for Multi-Krum
    assert L.detox_step_robust_blocks(p, 45, 10, 10, 3, None, 2, None, 0, 2, 3, p, p, 10, p, p, p,
                                      dx.workspace_bytes("step_robust_blocks", 15, 10, 2) - 256, None) == EWS
    assert L.detox_step_robust_blocks(p, 45, 10, 10, 3, None, 2, None, 0, 3, 3, p, p, 10, p, p, p, big, None) == EPRECOND
    # the variant on the library's own scratch array: a step that needs more than the array holds
    # is refused on the host (120 rows for the aggregator: 8 row tiles of Gram partials)
    header = open(os.path.join(ROOT, "include", "detox.h")).read()
    assert int(re.search(r"DETOX_STATIC_SCRATCH_BYTES \(\(size_t\)(\d+) << 20\)", header).group(1)) << 20 < \
        dx.workspace_bytes("step", 360, 10, 120)
    assert L.detox_step_static(p, 360, 10, 10, 3, 5, None, 120, None, 2, -1, -1, 50, ctypes.c_double(1e-8),
                               p, None, 0, p, p, None) == EWS
    assert L.detox_step_static(p, 45, 10, 10, 3, 5, None, 16, None, 0, 1, 3, 50, ctypes.c_double(1e-8),
                               p, p, 10, p, p, None) == EINVAL
    for code in range(5):
        assert dx.strerror(code)


def test_calls_fail_loudly_without_the_library(monkeypatch, dx):
    from paper_1907_12205_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libdetox.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.lib()
