"""CPU-side checks of the product: the C-ABI library loads and exports what the header
declares, host-side validation returns the documented status codes before any GPU call,
and the synthetic workloads have the documented shapes.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2207_04604_amd import binding as B
from paper_2207_04604_amd.synth import CONFIGS, closed_neighbourhood_groups

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2207_04604_amd import build
        build.build_library()
    return B.lib()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "d2mhe.h")).read()
    declared = sorted(set(re.findall(r"\b(d2mhe_[a-z0-9_]+)\s*\(", header)))
    assert declared == sorted(B.SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_strerror_covers_all_codes(lib):
    seen = {B.strerror(code) for code in range(0, -8, -1)}
    assert len(seen) == 8 and "unknown status" not in seen
    assert B.strerror(-99) == "unknown status"


def _params(log2n=10, q=(1073707009,), t=12289, eta=21, f=8, kmax=4):
    return B.make_params(log2n, list(q), t, eta, f, kmax, 1)


def test_parameter_validation(lib):
    good, keep = _params()
    assert B.workspace_bytes(good) > 0
    bad = [
        _params(log2n=9), _params(log2n=17),
        _params(q=(1073707009, 1073707009)),              # duplicate prime
        _params(q=(1073707011,)),                          # not 1 mod 2N
        _params(q=(2049 * 2048 + 1,)),                     # 1 mod 2N but composite (divisible by 7)
        _params(q=((1 << 61) + 20 * 2048 + 1,)),           # above 2^61
        _params(t=12290), _params(t=1073707009),           # t not prime-congruent / t >= q
        _params(eta=0), _params(eta=33), _params(f=31), _params(kmax=0),
        # a 31-bit prime t = 1 mod 2N below a 36-bit prime q: valid BFV, above the library's t < 2^30
        _params(q=(68719464449,), t=2147473409),
    ]
    ok36, keep36 = _params(q=(68719464449,), t=1073707009)   # the same shape with a 30-bit t is accepted
    assert B.workspace_bytes(ok36) > 0
    for prm, keep2 in bad:
        assert B.workspace_bytes(prm) == 0
        handle = C.c_void_p()
        fake = np.zeros(64, dtype=np.uint64)
        st = lib.d2mhe_create(C.byref(prm), fake.ctypes.data, fake.nbytes, None, C.byref(handle))
        assert st == B.ERR_BAD_PARAMS and not handle
    # 17 limbs
    p17, keep3 = B.make_params(10, [1073707009] * 17, 12289, 21, 8, 4, 1)
    assert B.workspace_bytes(p17) == 0


def test_create_argument_checks(lib):
    prm, keep = _params()
    need = B.workspace_bytes(prm)
    handle = C.c_void_p()
    fake = np.zeros(64, dtype=np.uint64)
    assert lib.d2mhe_create(None, fake.ctypes.data, need, None, C.byref(handle)) == B.ERR_NULL
    assert lib.d2mhe_create(C.byref(prm), None, need, None, C.byref(handle)) == B.ERR_NULL
    assert lib.d2mhe_create(C.byref(prm), fake.ctypes.data, need, None, None) == B.ERR_NULL
    assert lib.d2mhe_create(C.byref(prm), fake.ctypes.data + 8, need, None, C.byref(handle)) == B.ERR_ALIGN
    assert lib.d2mhe_create(C.byref(prm), fake.ctypes.data, need - 1, None, C.byref(handle)) == B.ERR_WORKSPACE
    # entry points refuse a NULL context
    assert lib.d2mhe_ntt_forward(None, fake.ctypes.data, 1, None) == B.ERR_NULL
    assert lib.d2mhe_encrypt(None, None, None, 1, 0, 0, 0, None, None) == B.ERR_NULL
    assert lib.d2mhe_round_scratch_bytes(None, 4, 1, 4096) == 0


def test_workspace_size_formula(lib):
    for name, cfg in CONFIGS.items():
        prm, keep = B.make_params(cfg.log2_n, cfg.q, cfg.t, cfg.eta, cfg.frac_bits, max(cfg.max_group, 1), cfg.seed)
        need = B.workspace_bytes(prm)
        moduli = cfg.L + (1 if cfg.t else 0)
        tables = moduli * 2 * cfg.N * 16
        crs = 2 * cfg.L * cfg.N * 8 if cfg.t else 0
        assert tables + crs <= need <= tables + crs + 4096, name


def test_workload_shapes():
    expect = {"C1": (1, 4, 4, 16 * 1024), "C2": (16, 5, 25, 192 * 1024), "C3": (32, 7, 153, 512 * 1024),
              "C4": (1, 8, 684, 2 * 1024 * 1024)}
    for name, (G, K, Cn, ct_bytes) in expect.items():
        cfg = CONFIGS[name]
        groups = cfg.groups()
        assert len(groups) == G and all(len(g) == K for g in groups) and cfg.max_group == K
        assert cfg.C == Cn and 2 * cfg.L * cfg.N * 8 == ct_bytes
        for g in groups:
            assert g == sorted(g)
    c3 = CONFIGS["C3"]
    adj = c3.adjacency()
    assert all(len(a) == 6 and i not in a for i, a in enumerate(adj))
    assert all(i in adj[j] for i, a in enumerate(adj) for j in a)          # symmetric
    seen, todo = {0}, [0]
    while todo:
        for j in adj[todo.pop()]:
            if j not in seen:
                seen.add(j)
                todo.append(j)
    assert len(seen) == 32                                                  # connected
    g = CONFIGS["C2"].gradients(parties=2, n_values=1000)
    assert g[0].dtype == np.float32 and g[0].shape == (1000,) and abs(float(g[0].std()) - 0.01) < 0.002
    assert CONFIGS["C5"].L == 16 and CONFIGS["C5"].batch == 64 and all(q % (1 << 17) == 1 for q in CONFIGS["C5"].q)


def test_grouping_merges_identical_neighbourhoods():
    adj = [[1, 2], [0, 2], [0, 1], [4], [3]]
    groups, owner = closed_neighbourhood_groups(adj)
    assert groups == [[0, 1, 2], [3, 4]] and owner == [0, 0, 0, 1, 1]


def test_bench_reads_kernel_traffic_from_the_committed_profiles():
    """bench.py takes roofline.traffic from the rocprofv3 summaries under profiles/: every round configuration it
    times by default has a k_encrypt line there, the C5 leg its four kernels, and unknown kernels give None."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    bench = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(bench)
    for wl in ("C2", "C3", "C4"):
        got = bench.profiled_traffic(wl, "k_encrypt")
        assert got is not None and got[0] > 0 and got[1] > 0 and got[2].startswith("profiles/")
        cfg = CONFIGS[wl]
        jobs = sum(len(g) for g in cfg.groups())
        launches = -(-jobs // bench.JOBS_PER_LAUNCH)
        written = jobs * cfg.C * 16 * cfg.L * cfg.N / launches          # the ciphertexts of one launch
        assert written <= got[1] <= 2.0 * written, (wl, got, written)
    for k in ("k_head_forward", "k_tail_forward", "k_tail_inverse", "k_head_inverse"):
        rd, wr, _ = bench.profiled_traffic("C5", k)
        assert 0.95 * 2 ** 29 <= wr <= 1.1 * 2 ** 29 and rd >= 0.95 * 2 ** 29
    assert bench.profiled_traffic("C3", "k_no_such_kernel") is None
    assert bench.ops_per_butterfly(1 << 29)[0] == 8 and bench.ops_per_butterfly((1 << 54) - 1)[0] == 15


def test_arithmetic_policies_hold_their_contracts_on_the_host(tmp_path):
    """The modular-arithmetic header of the kernels, built for the host (its plain-C side, the same formulas the
    device code pins with assembly) and checked against 128-bit integers on the ends of every documented range:
    tests/arith_host_check.cpp."""
    import shutil
    import subprocess
    cxx = shutil.which("amdclang++") or "/opt/rocm/llvm/bin/clang++"
    exe = str(tmp_path / "arith_host_check")
    subprocess.check_call([cxx, "-O2", "-std=c++17", "-w", "-o", exe, os.path.join(ROOT, "tests", "arith_host_check.cpp")])
    run = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout[-2000:]
    assert "all arithmetic policies hold their contracts" in run.stdout
