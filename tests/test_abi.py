"""Host-only checks of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and its planner agrees with the oracle's independently written geometry."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_00277_amd import binding, build
    if not os.path.exists(binding.LIB_PATH) or not os.path.exists(binding.MEASURE_LIB_PATH):
        build.build(verbose=False)
    binding.lib()
    return binding


def _declared(header_name):
    header = open(os.path.join(ROOT, "include", header_name)).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    return set(re.findall(r"\b(ftar_[a-z_0-9]+)\s*\(", header))


def _exported(path):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return {line.split()[-1] for line in out.splitlines() if re.search(r" [TW] ftar_[a-z_0-9]+$", line)}


def test_exports_every_declared_symbol(B):
    # the product header: exactly the method's calls, all in libftar.so
    declared = _declared("ftar.h")
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    raw = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(raw, name) is not None, name
    # the measurement header: two hooks in libftar.so, the probe kernels in the bench-only library
    measure = _declared("ftar_measure.h")
    assert measure == set(B.MEASURE_HOOKS) | set(B.MEASURE_EXPORTS), measure
    assert not (measure & declared)
    for name in B.MEASURE_HOOKS:
        assert getattr(raw, name) is not None, name
    # libftar.so exports no C entry point that neither header declares; the probe is not in it
    assert _exported(B.LIB_PATH) == declared | set(B.MEASURE_HOOKS)
    assert _exported(B.MEASURE_LIB_PATH) == set(B.MEASURE_EXPORTS)


def test_status_strings_and_classes(B):
    for s in (0, 1, 2, 3, 4, 5, 16, 17, 32):
        assert B.ftar_status_str(s) and B.ftar_status_str(s) != "unknown status"
    assert B.ftar_status_is_retryable(B.FTAR_ERR_STALE_PLAN) and B.ftar_status_is_retryable(B.FTAR_ERR_SKIPPED)
    assert not any(B.ftar_status_is_retryable(s) for s in (0, 1, 2, 3, 4, 5, 32))


def test_plan_rejects_bad_arguments(B):
    cases = [((0, 1, 10, 1), B.FTAR_ERR_INVALID_ARG), ((65, 1, 10, 1), B.FTAR_ERR_INVALID_ARG),
             ((4, 0, 10, 1), B.FTAR_ERR_NO_LIVE), ((4, 0x10, 10, 1), B.FTAR_ERR_BAD_MASK),
             ((4, 0xF, 0, 1), B.FTAR_ERR_INVALID_ARG), ((4, 0xF, 10, 0), B.FTAR_ERR_INVALID_ARG)]
    for args, status in cases:
        with pytest.raises(B.FtarError) as e:
            B.ftar_plan(*args)
        assert e.value.status == status, args


def test_planner_matches_oracle_geometry(B, oracle):
    cases = [(16, 0xFFFF, 1 << 28, 16384), (16, 0xFDFF, 1 << 28, 16384), (8, 0xF7, 1000, 16),
             (5, 0b10101, 17, 4), (6, 0b111111, 3, 1), (4, 0xF, 100, 1000),
             (64, (1 << 64) - 1, 12345, 7), (8, 0xFF, 2_000_000_000, 16384), (3, 0b101, 1, 1)]
    for n, mask, count, chunk in cases:
        p = B.ftar_plan(n, mask, count, chunk)
        ring = oracle.live_ring(n, mask)
        N = len(ring)
        assert p.n_live == N and p.n_steps == N - 1 and p.acc_bytes == count * 4
        sb = oracle.geometry(n, mask, count, chunk)
        for k in range(N):
            b, e, owner = p.segment(k)
            assert (b, e) == (sb[k], sb[k + 1])
            assert owner == ring[(k + N - 1) % N]
        import numpy as np
        assert np.float32(p.scale) == oracle.scale(N)
        p.destroy()


def test_plan_is_pure(B):
    a = B.ftar_plan(16, 0xFDFF, 1 << 28, 16384)
    b = B.ftar_plan(16, 0xFDFF, 1 << 28, 16384)
    assert [a.segment(k) for k in range(15)] == [b.segment(k) for k in range(15)]


def test_oracle_is_not_reachable_from_the_product(B):
    # the package must not import the oracle, and the oracle must not import the package
    pkg = os.path.join(ROOT, "paper_2602_00277_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "ftar_oracle" not in src and "oracle/" not in src, f
    osrc = open(os.path.join(ROOT, "oracle", "ftar_oracle.py")).read() + \
        open(os.path.join(ROOT, "oracle", "ftar_oracle.cpp")).read()
    assert "paper_2602_00277_amd" not in osrc and "ftar.h" not in osrc and "libftar.so" not in osrc


def test_lr_factors_match_the_oracle(B, oracle):
    # host-only call: no GPU needed
    L = B.lib()
    for n, live, zmask in [(8, 0xFF, 0), (16, 0x01FF, 0), (16, 0x00FF, 0x000F), (7, 0b1010101, 0b0000100),
                           (64, (1 << 64) - 1, 1 << 63), (3, 0b011, 0b011)]:
        plan = L.ftar_plan(n, live, 1000, 10)
        assert plan
        assert L.ftar_plan_set_zero_mask(plan, zmask, 0) == 0
        lin, root = ctypes.c_float(), ctypes.c_float()
        assert L.ftar_plan_lr_factors(plan, ctypes.byref(lin), ctypes.byref(root)) == 0
        want_lin, want_root = oracle.lr_factors(n, live, zmask)
        assert lin.value == float(want_lin) and root.value == float(want_root), (n, hex(live), hex(zmask))
        assert L.ftar_plan_lr_factors(plan, None, None) == 0
        L.ftar_plan_destroy(plan)
    assert L.ftar_plan_lr_factors(None, None, None) == B.FTAR_ERR_INVALID_ARG


def test_gate_units_match_the_definition(B, oracle):
    # host-only: slots without the flag; with rows of chunks, per partition (2N-2) x the largest number of
    # chunks any portion has (paper section 4.2: a step is pipelined over the chunks of a portion)
    L = B.lib()
    for n, mask, count, chunk, part in [(8, 0xFF, 8 * 8192 * 6, 8192, 0), (8, 0xF7, 7 * 4096 * 5 + 4096 * 3 + 100, 4096, 0),
                                        (16, 0xFFFF, 1 << 28, 16384, 0), (16, 0xFDFF, 1 << 28, 16384, 4 << 20),
                                        (6, 0x3F, 6 * 8192 * 10 + 8192 * 2, 8192, 6 * 8192 * 4), (12, 0xFFF, 4096 * 5, 4096, 0),
                                        (2, 3, 1000, 7, 0), (1, 1, 1000, 7, 0)]:
        plan = L.ftar_plan(n, mask, count, chunk)
        assert plan
        if part:
            assert L.ftar_plan_set_partition(plan, part) == 0
        N = bin(mask).count("1")
        want = 0
        P = part if part else count
        for p0 in range(0, count, P):
            sb = oracle.geometry(n, mask, min(P, count - p0), chunk)
            want += (2 * N - 2) * max(-(-(sb[k + 1] - sb[k]) // chunk) for k in range(N))
        assert L.ftar_plan_n_gate_units(plan, B.FTAR_PERSIST_CHUNKS) == want, (n, hex(mask), count, chunk, part)
        assert L.ftar_plan_n_gate_units(plan, 0) == L.ftar_plan_n_slots(plan)
        L.ftar_plan_destroy(plan)
    assert L.ftar_plan_n_gate_units(None, 0) == 0
