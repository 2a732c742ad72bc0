"""Do the pins bind?  Each case plants one plausible mistake in a copy of the oracle's source (a dropped term, a
wrong sign, a wrong boundary, a reversed order), builds it, and runs the oracle's pin tests against that build in
a child process: some pin must fail.  The mistakes live on the CPU, in the oracle's copy, never in the GPU path."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "pxchg_oracle.c")

FP16, REDUCE, UPDATE, STATS = ("test_oracle_fp16.py", "test_oracle_reduce.py", "test_oracle_update.py",
                               "test_oracle_stats.py")

# (name, text in the oracle, replacement, pin file that must notice)
MUTANTS = [
    ("tie rounds up instead of to even (normal range)",
     "rest == 0x1000u && (h & 1u)", "rest == 0x1000u", FP16),
    ("tie rounds up instead of to even (subnormal range)",
     "rest == half && (h & 1u)", "rest == half", FP16),
    ("overflow threshold one binade late",
     "if (e >= 16) return", "if (e >= 17) return", FP16),
    ("flush to zero one binade early",
     "if (e < -25) return sign;", "if (e < -24) return sign;", FP16),
    ("subnormal shift off by one",
     "int shift = -e - 1;", "int shift = -e;", FP16),
    ("infinity becomes NaN",
     "if (mag == 0x7f800000u) return (uint16_t)(sign | 0x7c00u);",
     "if (mag == 0x7f800000u) return (uint16_t)(sign | 0x7e00u);", FP16),
    ("sign dropped in the narrowing",
     "uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);", "uint16_t sign = 0; (void)x;", FP16),
    ("float32 contributions summed in reverse order",
     "for (int i = 1; i < k; ++i) s = s + ((const float *)contrib[i])[j];",
     "for (int i = k - 1; i >= 1; --i) s = s + ((const float *)contrib[i])[j];", REDUCE),
    ("half contributions summed in reverse order",
     "for (int i = 1; i < k; ++i) s = s + widen(((const uint16_t *)contrib[i])[j]);",
     "for (int i = k - 1; i >= 1; --i) s = s + widen(((const uint16_t *)contrib[i])[j]);", REDUCE),
    ("running sum starts from zero",
     "s = ((const float *)contrib[0])[j];", "s = 0.0f + ((const float *)contrib[0])[j];", REDUCE),
    ("last contribution dropped",
     "for (int i = 1; i < k; ++i) s = s + ((const float *)contrib[i])[j];",
     "for (int i = 1; i < k - 1; ++i) s = s + ((const float *)contrib[i])[j];", REDUCE),
    ("average multiplies by a rounded reciprocal",
     "? s / kf : s;", "? s * (1.0f / kf) : s;", REDUCE),
    ("sum mode divides too",
     "(mode == ORACLE_AVG) ? s / kf : s;", "s / kf;", REDUCE),
    ("half output truncated instead of rounded",
     "else ((uint16_t *)out)[j] = narrow(a);",
     "else ((uint16_t *)out)[j] = (uint16_t)(narrow(a) & 0xfffeu);", REDUCE),
    ("weight decay taken from the velocity",
     "float dw = wd * w[j];", "float dw = wd * v[j];", UPDATE),
    ("weight decay dropped",
     "float gg = g + dw;", "float gg = g; (void)dw;", UPDATE),
    ("gradient step with the wrong sign",
     "float vn = mv - lg;", "float vn = mv + lg;", UPDATE),
    ("velocity subtracted from the weights",
     "w[j] = w[j] + vn;", "w[j] = w[j] - vn;", UPDATE),
    ("momentum applied to the new gradient too",
     "float lg = lr * gg;", "float lg = lr * gg * mu;", UPDATE),
    ("fused multiply-add in the velocity",
     "float vn = mv - lg;", "float vn = __builtin_fmaf(-lr, gg, mv); (void)lg;", UPDATE),
    ("fused multiply-add in the decay term",
     "float gg = g + dw;", "float gg = __builtin_fmaf(wd, w[j], g); (void)dw;", UPDATE),
    ("fused multiply-add in the elastic pull",
     "x[j] = x[j] - d;", "x[j] = __builtin_fmaf(-alpha, diff, x[j]);", UPDATE),
    ("elastic difference reversed",
     "float diff = x[j] - c[j];", "float diff = c[j] - x[j];", UPDATE),
    ("center pushed away from the worker",
     "c[j] = c[j] + d;", "c[j] = c[j] - d;", UPDATE),
    ("worker moves twice as far as the center",
     "x[j] = x[j] - d;", "x[j] = x[j] - d - d;", UPDATE),
    ("diagnostics count NaN but not infinity",
     "if ((bits_of(x) & 0x7f800000u) == 0x7f800000u) {", "if (x != x) {", UPDATE),
    ("diagnostics take the signed maximum",
     "float ax = x < 0.0f ? -x : x;", "float ax = x;", UPDATE),
    ("diagnostics sum magnitudes instead of squares",
     "ss = ss + (double)x * (double)x;", "ss = ss + (double)ax;", UPDATE),
    ("diagnostics square in binary32",
     "ss = ss + (double)x * (double)x;", "ss = ss + (double)(x * x);", UPDATE),
    ("ordered sum: lane taken from the element, not from its 16-byte piece",
     "double *slot = wave_acc + (i / piece) % 64;", "double *slot = wave_acc + i % 64;", STATS),
    ("ordered sum: binary16 pieces as short as binary32 ones",
     "const int piece = (dtype == ORACLE_F32) ? 4 : 8;", "const int piece = 4;", STATS),
    ("ordered sum: lanes do not wrap after 64 pieces",
     "double *slot = wave_acc + (i / piece) % 64;", "double *slot = wave_acc + ((i / piece) < 64 ? (i / piece) : 63);", STATS),
    ("ordered sum: a block's chunks dealt to the waves in runs instead of round-robin",
     "double *wave_acc = acc + 64 * (j % waves);", "double *wave_acc = acc + 64 * (int)((int64_t)j * waves / block_chunks);", STATS),
    ("ordered sum: chunks run on across tensor boundaries",
     "const int j = (int)(g % block_chunks);", "const int j = (int)((g - t) % block_chunks);", STATS),
    ("ordered sum: butterfly steps in ascending order",
     "for (int off = 32; off >= 1; off /= 2) {", "for (int off = 1; off <= 32; off *= 2) {", STATS),
    ("ordered sum: lanes added one after the other instead of the butterfly",
     "for (int l = 0; l < 64; ++l) tmp[l] = lane[l] + lane[l ^ off];",
     "for (int l = 0; l < 64; ++l) tmp[l] = (l == 0 && off == 1) ? lane[0] : lane[l]; if (off == 1) for (int l = 1; l < 64; ++l) tmp[0] = tmp[0] + lane[l];", STATS),
    ("ordered sum: group 1 added last instead of second",
     "total = (grp == 0) ? lane[0] : total + lane[0];",
     "total = (grp == 0) ? lane[0] : (grp == 1 ? total : total + lane[0]); "
     "if (grp >= 1 && grp == threads / 64 - 1) total = total + a[64];", STATS),
    ("ordered sum: a combine thread takes a run of values instead of every T-th",
     "for (int64_t i = t; i < n; i += threads) a[t] = a[t] + values[i];",
     "for (int64_t i = t * ((n + threads - 1) / threads); i < (t + 1) * ((n + threads - 1) / threads) && i < n; ++i) a[t] = a[t] + values[i];", STATS),
    ("ordered sum: the last, incomplete block is dropped",
     "if (j == block_chunks - 1 || g == n_chunks - 1) {", "if (j == block_chunks - 1) {", STATS),
    ("ordered sum: squares taken in binary32",
     "*slot = *slot + (double)x * (double)x;", "*slot = *slot + (double)(x * x);", STATS),
    ("ordered sum: an element that is not finite is added",
     "if (!finite) { ++bad; continue; }", "if (!finite) { ++bad; }", STATS),
    ("ordered sum: largest magnitude keeps its sign",
     "float mag = x < 0.0f ? -x : x;", "float mag = x;", STATS),
]


def _run_pins(lib_path, pins):
    env = dict(os.environ, PXCHG_ORACLE_LIB=str(lib_path))
    return subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                           os.path.join(HERE, pins)], env=env, capture_output=True, text=True, cwd=ROOT, timeout=600)


@pytest.fixture(scope="module")
def mutant_runs(tmp_path_factory):
    """Builds every mutant and runs its pin file, four at a time; name -> finished child process."""
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    text = open(SRC).read()
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    base = tmp_path_factory.mktemp("mutants")

    def one(job):
        i, (name, old, new, pins) = job
        if text.count(old) != 1:
            return name, None
        c, so = base / f"mutant{i}.c", base / f"libmutant{i}.so"
        c.write_text(text.replace(old, new))
        subprocess.run(["gcc", *flags, str(c), "-o", str(so)], check=True)
        return name, _run_pins(so, pins)

    with ThreadPoolExecutor(max_workers=4) as pool:
        return dict(pool.map(one, enumerate(MUTANTS)))


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_some_pin(mutant_runs, name):
    run = mutant_runs[name]
    assert run is not None, "the oracle no longer contains exactly one copy of this mutant's text: update MUTANTS"
    assert run.returncode == 1, f"no pin noticed: {name}\n{run.stdout[-2000:]}"
    assert " failed" in run.stdout


def test_the_unmodified_oracle_passes_in_the_same_harness(tmp_path):
    """The child-process harness itself: the untouched source, built the same way, passes every pin."""
    import oracle
    so = tmp_path / "liboracle.so"
    flags = [f for f in oracle.CFLAGS if f not in ("-Wall", "-Wextra")]
    subprocess.run(["gcc", *flags, SRC, "-o", str(so)], check=True)
    for pins in (FP16, REDUCE, UPDATE, STATS):
        run = _run_pins(so, pins)
        assert run.returncode == 0, run.stdout[-2000:]
