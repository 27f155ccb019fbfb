"""CPU-side checks of libskm: it loads, exports what include/skm.h declares, its host-side rules
agree with the oracle's, and argument errors are reported as error codes (no GPU call is made)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def skm():
    from paper_2603_20009_amd import skm as m
    if not os.path.exists(m.LIB_PATH):
        from paper_2603_20009_amd import build
        build.build(verbose=False)
    m.lib()
    return m


def test_every_declared_symbol_is_exported(skm):
    hdr = open(os.path.join(ROOT, "include", "skm.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(skm_[a-z_0-9]+)\s*\(", hdr)))
    assert len(names) >= 14
    L = skm.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(skm.EXPORTS) == names
    assert skm.version().startswith("skm")


def test_struct_sizes_match_header(skm):
    # sizes implied by include/skm.h on LP64: catches a field added on one side only
    assert C.sizeof(skm.TraceRow) == 3 * 8 + 10 * 8 + 2 * 4 + 32 * 8 + 6 * 4
    assert C.sizeof(skm.Trace) == 4 * 4 + 8 * 4 + 8
    assert C.sizeof(skm.Params) == 10 * 4 + 2 * 8 + 6 * 4 + 4 * 8 + 8 + 2 * 4 + 2 * 4 + 2 * 8 + 4 * 4
    p = skm.Params()
    skm.lib().skm_params_default(C.byref(p))
    assert (p.dprime_frac, p.adjust_dprime, p.final_assign, p.rotate, p.etr) == (0.125, 1, 1, 1, 0)
    assert p.eps0 == pytest.approx(2.1) and p.nq == 1000 and p.topk == 10 and p.etr_patience == 2
    assert p.adj_lo == pytest.approx(0.95) and p.adj_hi == pytest.approx(0.97) and p.adj_step == pytest.approx(0.2)


def test_host_rules_agree_with_the_oracle(skm, orc):
    for d in (16, 100, 128, 384, 768, 1536, 3072):
        assert skm.dprime_init(d) == orc.dprime_init(d)
        for t in range(16, d + 1, 16):
            assert skm.theta_ratio(d, t, 2.1) == pytest.approx(orc.theta_ratio(d, t, float(np.float32(2.1))), rel=1e-6)
        assert skm.theta_ratio(d, 16, float("inf")) == 1.0
        for dp in range(16, d + 1, 16):
            for f in (0.5, 0.949, 0.96, 0.971, 0.999):
                assert skm.dprime_adjust(d, dp, f) == orc.dprime_adjust(d, dp, f)
    for seed, n, k in ((42, 20_000, 100), (1, 1000, 1000), (7, 10**6, 1024), (2**63 + 5, 333, 17)):
        assert skm.sample_rows(seed, n, k) == orc.sample_rows(seed, n, k).tolist()
    # hierarchical fit: number of meso-clusters and the shares of k
    for k in (1, 2, 3, 10, 99, 1024, 16384, 32768, 2**24):
        assert skm.hier_meso_count(k) == orc.hier_meso_count(k)
    rng = np.random.default_rng(11)
    for _ in range(200):
        km = int(rng.integers(1, 200))
        sizes = rng.integers(0, 50_000, km) * (rng.random(km) > 0.05)
        sizes[int(rng.integers(0, km))] += km + 5
        k = int(rng.integers(km, min(int(sizes.sum()), 40 * km) + 1))
        assert skm.hier_alloc(sizes.tolist(), k) == orc.hier_alloc(sizes, k).tolist()
    assert skm.lib().skm_hier_alloc(None, 3, 5, None) == -1


def test_argument_errors_are_codes_not_crashes(skm):
    L = skm.lib()
    one = C.c_void_p(16)   # never dereferenced: every call below fails validation first
    assert L.skm_fit(None, 10, 16, 2, 1, 0, one, None) == -1
    assert L.skm_fit(one, 10, 8, 2, 1, 0, one, None) == -1          # d < 16
    assert L.skm_fit(one, 10, 16, 11, 1, 0, one, None) == -1        # k > n
    assert L.skm_fit(one, 10, 16, 2, 0, 0, one, None) == -1         # iters < 1
    assert L.skm_fit(one, 10, 16, 2, 1, 0, None, None) == -1        # no output
    assert L.skm_assign(one, 0, 16, one, 2, None, one, None) == -1  # n < 1
    assert L.skm_assign_exact(one, 10, 16, None, 2, None, one, None) == -1
    assert L.skm_update(one, 10, 16, None, 2, None, one, None) == -1
    assert L.skm_sample_rows(1, 5, 6, one) == -1
    assert b"invalid" in L.skm_strerror(-1) and L.skm_last_error() != b""
    assert L.skm_strerror(0) == b"ok"


def test_workspace_size_query(skm):
    L = skm.lib()
    assert L.skm_workspace_bytes(0, 16, 1, None) == -1 and L.skm_workspace_bytes(10, 8, 2, None) == -1
    assert L.skm_workspace_bytes(10, 16, 11, None) > 0      # an assignment step may have k > n
    small = skm.workspace_bytes(1000, 64, 10)
    big = skm.workspace_bytes(1_000_000, 1536, 1024)
    # two copies of the rotated points, their split-fp16 copy and the prefix-norm table dominate
    assert small > 0 and 3 * 1_000_000 * 1536 * 4 < big < 6 * 1_000_000 * 1536 * 4
    p = skm.Params()
    L.skm_params_default(C.byref(p))
    p.etr, p.nq, p.topk = 1, 1000, 10
    assert skm.workspace_bytes(1_000_000, 1536, 1024, p) > big
