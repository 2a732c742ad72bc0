"""CPU-only checks of the C-ABI library: it loads without a GPU, exports every
function that include/pxchg.h declares, and its host-side logic (chunk planning,
options, argument validation that happens before any GPU call) behaves."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pxchg.h")


@pytest.fixture(scope="module")
def px():
    import paper_1605_08325_amd as px
    if not os.path.exists(px.library_path()):
        from paper_1605_08325_amd import build
        build.build_lib()
    px.load()
    return px


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pxchg_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for n in ("pxchg_pack_fp16", "pxchg_reduce_avg", "pxchg_sgd_momentum", "pxchg_easgd"):
        assert n in names


def test_library_exports_every_declared_symbol(px):
    lib = ctypes.CDLL(px.library_path())
    names = declared_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in pxchg.h but not exported"


def test_binding_covers_every_declared_symbol(px):
    from paper_1605_08325_amd import binding
    assert sorted(binding.SIGNATURES) == declared_functions()


def test_no_fallback_when_library_is_missing(px, monkeypatch):
    from paper_1605_08325_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", os.path.join(ROOT, "no_such_dir", "libpxchg.so"))
    with pytest.raises(ImportError):
        binding.load()


def test_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_1605_08325_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU or eager fallback", ""), f
    oracle_src = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + \
        open(os.path.join(ROOT, "oracle", "pxchg_oracle.c")).read()
    assert "paper_1605_08325_amd" not in oracle_src and "hip" not in oracle_src.lower().replace("the hip library", "")


def test_status_strings_and_version(px):
    assert px.version() >= 200
    assert px.status_string(0) == "ok"
    for s in range(1, 8):
        assert px.status_string(s) not in ("ok", "unknown status")
    assert px.status_string(99) == "unknown status"


def test_options_validate_their_values(px):
    old = [px.get_option(o) for o in range(5)]
    assert old == [512, 0, 1, -1, 0]          # the documented defaults
    try:
        px.set_option(px.OPT_CENTER_RESIDENT, 1)
        assert px.get_option(px.OPT_CENTER_RESIDENT) == 1
        px.set_option(px.OPT_CHUNK_ELEMS, 4096)
        assert px.get_option(px.OPT_CHUNK_ELEMS) == 4096
        for bad in (0, 100, 513, 1 << 21, -512):
            with pytest.raises(px.PxchgError):
                px.set_option(px.OPT_CHUNK_ELEMS, bad)
        for opt, bad in ((px.OPT_BLOCKS_PER_CU, -1), (px.OPT_BLOCKS_PER_CU, 65), (px.OPT_CHECK_RANGES, 2),
                         (px.OPT_NONTEMPORAL, 6), (px.OPT_NONTEMPORAL, -2), (px.OPT_CENTER_RESIDENT, 2),
                         (px.OPT_CENTER_RESIDENT, -1), (17, 0)):
            with pytest.raises(px.PxchgError):
                px.set_option(opt, bad)
        assert px.get_option(17) == -1
    finally:
        for o, v in enumerate(old):
            px.set_option(o, v)


def test_plan_chunks_covers_every_element_exactly_once(px):
    counts = [1, 0, 511, 512, 513, 5000, 0, 1024 * 3, 70_001]
    for chunk in (512, 1024, 8192):
        t, s, ln = px.plan_chunks(counts, chunk)
        covered = {i: 0 for i in range(len(counts))}
        prev = (-1, -1)
        for ti, si, li in zip(t, s, ln):
            assert 0 < li <= chunk and si % chunk == 0 and si + li <= counts[ti]
            assert (ti, si) > prev                     # tensor-major, ascending
            prev = (ti, si)
            covered[ti] += li
        assert [covered[i] for i in range(len(counts))] == counts
        assert len(t) == sum((c + chunk - 1) // chunk for c in counts)


def test_plan_chunks_matches_the_alexnet_table(px):
    import workloads as wl
    t, s, ln = px.plan_chunks(wl.alexnet_counts(), 512)
    assert len(t) == 119_076 and sum(ln) == wl.ALEXNET_PARAMS


def test_plan_groups_cuts_the_tensor_list_into_runs_of_a_minimum_size(px):
    import workloads as wl
    counts = wl.alexnet_counts()
    # from the last tensor backwards: fc8 + fc7 (20.9 M), fc6 (37.8 M), the five convolutions (2.3 M, what is left)
    assert px.plan_groups(counts, 8_000_000) == [(12, 4), (10, 2), (0, 10)]
    assert px.plan_groups(counts, 8_000_000, reverse=False) == [(0, 11), (11, 2), (13, 3)]
    assert px.plan_groups(counts, 10 ** 9) == [(0, 16)]
    assert px.plan_groups(counts, 1) == [(t, 1) for t in reversed(range(16))]
    assert px.plan_groups(counts, 0, reverse=False) == [(t, 1) for t in range(16)]
    for min_elems in (1, 5000, 300_000, 8_000_000, 40_000_000):
        for reverse in (True, False):
            groups = px.plan_groups(counts, min_elems, reverse)
            covered = sorted(t for f, m in groups for t in range(f, f + m))
            assert covered == list(range(16))                                   # every tensor once
            assert all(sum(counts[f:f + m]) >= min_elems for f, m in groups[:-1])   # all but the last are big enough
    assert px.plan_groups([0, 0, 5, 0], 3) == [(2, 2), (0, 2)]                 # empty tensors ride along
    lib = px.load()
    n = ctypes.c_int(0)
    c = (ctypes.c_int64 * 2)(4, -1)
    assert lib.pxchg_plan_groups(2, c, 1, 1, 0, None, None, ctypes.byref(n)) == 1       # negative count
    c = (ctypes.c_int64 * 2)(4, 4)
    assert lib.pxchg_plan_groups(2, c, 1, 1, 2, None, None, ctypes.byref(n)) == 1       # room claimed, no arrays
    assert lib.pxchg_plan_groups(0, c, 1, 1, 0, None, None, ctypes.byref(n)) == 1
    assert lib.pxchg_plan_groups(2, c, -1, 1, 0, None, None, ctypes.byref(n)) == 1


def test_plan_chunks_rejects_bad_arguments(px):
    lib = px.load()
    n = ctypes.c_int64(0)
    arr = (ctypes.c_int64 * 2)(5, -1)
    assert lib.pxchg_plan_chunks(2, arr, 512, 0, None, None, None, ctypes.byref(n)) == 1    # negative count
    arr = (ctypes.c_int64 * 2)(5, 7)
    assert lib.pxchg_plan_chunks(2, arr, 500, 0, None, None, None, ctypes.byref(n)) == 1    # bad chunk size
    assert lib.pxchg_plan_chunks(0, arr, 512, 0, None, None, None, ctypes.byref(n)) == 1
    assert lib.pxchg_plan_chunks(2, None, 512, 0, None, None, None, ctypes.byref(n)) == 1
    assert lib.pxchg_plan_chunks(2, arr, 512, 4, None, None, None, ctypes.byref(n)) == 1    # cap without arrays


def test_host_side_argument_validation_needs_no_gpu(px):
    """These paths return before any HIP call, so they behave the same here."""
    lib = px.load()
    h = ctypes.c_void_p()
    arr = (ctypes.c_int64 * 2)(5, 7)
    assert lib.pxchg_table_create(2, arr, None) == 1
    assert lib.pxchg_table_create(0, arr, ctypes.byref(h)) == 1
    assert lib.pxchg_table_create(2, None, ctypes.byref(h)) == 1
    neg = (ctypes.c_int64 * 2)(5, -7)
    assert lib.pxchg_table_create(2, neg, ctypes.byref(h)) == 1
    assert h.value is None
    # null handles
    assert lib.pxchg_table_destroy(None) == 0 and lib.pxchg_bufset_destroy(None) == 0
    assert lib.pxchg_table_total(None) == -1 and lib.pxchg_table_n_tensors(None) == -1
    assert lib.pxchg_table_n_chunks(None) == -1
    assert lib.pxchg_reduce_avg(None, 2, None, None, 0, None) == 1
    assert lib.pxchg_sgd_momentum(None, None, None, None, 0.1, 0.9, 0.0, None) == 1
    assert lib.pxchg_easgd(None, None, None, 0.1, None) == 1
    assert lib.pxchg_pack_fp16(None, 1, None, None, None) == 1
    assert lib.pxchg_bufset_create(None, 0, None, ctypes.byref(h)) == 1


def test_table_create_without_a_gpu_reports_no_device(px):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(px.PxchgError) as e:
        px.Table([10, 20])
    assert e.value.status == 4


def test_header_is_plain_c(tmp_path):
    """The boundary must be usable from C: the header compiles as C99 and as C++ with no other include."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "pxchg.h"\nint main(void) { pxchg_stats s; s.nonfinite = 0; return (int)s.nonfinite + PXCHG_OK; }\n')
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        r = subprocess.run([cc, std, "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x",
                            "c" if cc == "gcc" else "c++", "-I", inc, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
