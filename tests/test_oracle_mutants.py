"""CPU: do the oracle's pins bite?  Each case plants ONE plausible mistake in a copy of the oracle's source (a
dropped term, a wrong sign, a wrong index, a transposed direction, a wrong divisor, a wrong rounding), builds
that copy, and runs the pin tests of tests/test_oracle_*.py against it: at least one of them must fail.  The
mistakes are planted in the oracle, on the CPU; nothing of the HIP path is involved."""
import importlib.util
import itertools
import os
import shutil
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")
PIN_MODULES = ["test_oracle_reduce", "test_oracle_ring", "test_oracle_zero", "test_oracle_variants", "test_oracle_bf16"]

# (what is planted, text of the source as it stands, text that replaces its first occurrence)
MUTANTS = [
    ("one-shot reduce: the second live replica is dropped",
     "for (int j = 1; j < N; ++j) a = a + load_f32(bufs[ring[j]], i, dtype);",
     "for (int j = 2; j < N; ++j) a = a + load_f32(bufs[ring[j]], i, dtype);"),
    ("one-shot reduce: a term is subtracted",
     "for (int j = 1; j < N; ++j) a = a + load_f32(bufs[ring[j]], i, dtype);",
     "for (int j = 1; j < N; ++j) a = a - load_f32(bufs[ring[j]], i, dtype);"),
    ("scale: divided by N + 1",
     "float mean_scale(int N) { return 1.0f / static_cast<float>(N); }",
     "float mean_scale(int N) { return 1.0f / static_cast<float>(N + 1); }"),
    ("bf16 narrowing: ties go up instead of to even",
     "u += 0x7fffu + keep_lsb;",
     "u += 0x8000u;"),
    ("bf16 narrowing: truncation",
     "u += 0x7fffu + keep_lsb;",
     "u += 0u;"),
    ("ring closed form: a portion absorbs its ring positions in the other direction",
     "for (int m = 1; m < N; ++m) a = a + load_f32(bufs[ring[(k + m) % N]], j, dtype);\n        if (N > 1) a = a * scale;",
     "for (int m = 1; m < N; ++m) a = a + load_f32(bufs[ring[(k + N - m) % N]], j, dtype);\n        if (N > 1) a = a * scale;"),
    ("message-passing ring: data arrives from the right neighbour",
     "int left = (p + N - 1) % N;\n            recv[p] = send[left];\n            recv_seg[p] = send_seg[left];\n        }\n        const bool last",
     "int left = (p + 1) % N;\n            recv[p] = send[left];\n            recv_seg[p] = send_seg[left];\n        }\n        const bool last"),
    ("message-passing ring: the last step forgets the scale",
     "                    r = r * scale;\n",
     ""),
    ("message-passing ring: intermediate results are also written to the user buffer",
     "                    send[p][j] = r;  // result kept only in the send buffer\n",
     "                    send[p][j] = r; store_cvt(local, sb[k] + j, dtype, r);\n"),
    ("one-shot reduce with zero participants: the divisor policy is ignored",
     "const int divisor = contributors_only ? N - Z : N;",
     "const int divisor = N;"),
    ("one-shot reduce with zero participants: the divisor counts the zero ones instead",
     "const int divisor = contributors_only ? N - Z : N;",
     "const int divisor = contributors_only ? (Z > 0 ? Z : N) : N;"),
    ("zero participants in the ring: the divisor policy is ignored",
     "  const float scale = 1.0f / static_cast<float>(divisor);\n  std::vector<size_t> sb(N + 1);",
     "  const float scale = 1.0f / static_cast<float>(N);\n  std::vector<size_t> sb(N + 1);"),
    ("zero participants in the ring: the other divisor is applied under the default policy too",
     "  const float scale = 1.0f / static_cast<float>(divisor);\n  std::vector<size_t> sb(N + 1);",
     "  const float scale = 1.0f / static_cast<float>(N - Z > 0 ? N - Z : N);\n  std::vector<size_t> sb(N + 1);"),
    ("zero participants in the ring: the first one of a portion is read after all",
     "float a = ((zero_mask >> r0) & 1u) ? 0.0f : load_f32(bufs[r0], j, dtype);",
     "float a = load_f32(bufs[r0], j, dtype);"),
    ("portions: boundaries not on whole chunks",
     "unsigned __int128 b = q * chunk;",
     "unsigned __int128 b = static_cast<unsigned __int128>(k) * count / static_cast<unsigned>(N);"),
    ("partial sums in flight: one ring position too many",
     "for (int m = 1; m <= rs_steps; ++m) a = a + load_f32(bufs[ring[(k + m) % N]], j, dtype);",
     "for (int m = 1; m <= rs_steps + 1; ++m) a = a + load_f32(bufs[ring[(k + m) % N]], j, dtype);"),
    ("learning-rate factors: the square root taken in single precision of the rounded ratio",
     "*root = static_cast<float>(std::sqrt(static_cast<double>(healthy) / static_cast<double>(n)));",
     "*root = std::sqrt(static_cast<float>(healthy) / static_cast<float>(n));"),
    ("learning-rate factors: catching-up replicas counted as healthy",
     "healthy += ((zero_mask >> ring[j]) & 1u) ? 0 : 1;",
     "healthy += 1;"),
]


def _load_mutant(tmp_path, idx, old, new):
    d = tmp_path / ("mutant_%d" % idx)
    d.mkdir()
    src = open(os.path.join(ORACLE_DIR, "ftar_oracle.cpp")).read()
    assert old in src, "the text to replace is not in the oracle any more: update this case"
    (d / "ftar_oracle.cpp").write_text(src.replace(old, new, 1))
    shutil.copy(os.path.join(ORACLE_DIR, "ftar_oracle.py"), d / "ftar_oracle.py")
    spec = importlib.util.spec_from_file_location("ftar_oracle_mutant_%d" % idx, str(d / "ftar_oracle.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.build(force=True)
    return mod


def _pin_calls():
    """Every pin test of the oracle with its parameters spelled out: (name, function, keyword arguments)."""
    if HERE not in sys.path:
        sys.path.insert(0, HERE)
    calls = []
    for name in PIN_MODULES:
        mod = importlib.import_module(name)
        for attr in sorted(dir(mod)):
            fn = getattr(mod, attr)
            if not attr.startswith("test_") or not callable(fn):
                continue
            axes = []
            for mark in getattr(fn, "pytestmark", []):
                if mark.name == "parametrize":
                    names = [a.strip() for a in mark.args[0].split(",")]
                    axes.append([dict(zip(names, v if isinstance(v, (tuple, list)) and len(names) > 1 else (v,)))
                                 for v in mark.args[1]])
            for combo in itertools.product(*axes) if axes else [()]:
                kw = {}
                for part in combo:
                    kw.update(part)
                calls.append(("%s.%s%s" % (name, attr, kw if kw else ""), fn, kw))
    return calls


def test_the_unmutated_oracle_passes_when_called_this_way(oracle):
    # the harness below must not be what makes a mutant fail
    for what, fn, kw in _pin_calls():
        fn(oracle=oracle, **kw)


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, idx):
    what, old, new = MUTANTS[idx]
    mutant = _load_mutant(tmp_path, idx, old, new)
    killed_by = None
    for name, fn, kw in _pin_calls():
        try:
            fn(oracle=mutant, **kw)
        except (AssertionError, Exception) as e:  # a pin bit (an error raised by the oracle's wrapper counts too)
            killed_by = "%s: %s" % (name, type(e).__name__)
            break
    assert killed_by is not None, "no pin notices: " + what
    print("%s -> %s" % (what, killed_by))
