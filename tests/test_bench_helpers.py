"""bench.py's host-side helpers that the benchmark line depends on (no GPU): the HBM traffic figures are parsed at
run time from the committed counter summary, so a change of that file's layout must not silently turn them into
nulls or into figures below the algorithmic bytes."""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def test_traffic_is_read_from_the_counter_summary_and_is_not_below_the_algorithmic_bytes():
    import bench
    n, k = 60_965_224, 8
    algorithmic = {"pack": 6 * k * n, "reduce": (2 * k + 2) * n, "update": 18 * n, "elastic": 16 * n,
                   "fused_reduce_update": (2 * k + 16) * n, "fused_elastic_round": (8 * k + 8) * n}
    traffic = bench.measured_traffic()
    assert set(traffic) == set(algorithmic), "a row of the summary was not found"
    for stage, want in algorithmic.items():
        assert want <= traffic[stage] <= 1.03 * want, (stage, traffic[stage], want)


def test_rotation_makes_every_operand_set_wait_for_a_gigabyte_of_other_traffic():
    import bench
    for per_set in (20 * 2 ** 20, 182 * 10 ** 6, 1_200_000_000, 3_600_000_000):
        sets = bench.rotation(per_set)
        assert sets >= 2 and (sets - 1) * per_set >= min(bench.COLD_BYTES, 63 * per_set)
    assert bench.rotation(1) == 64          # capped


def test_host_threads_reports_what_is_used_and_what_is_there(monkeypatch):
    import bench
    monkeypatch.setenv("OMP_NUM_THREADS", "3")
    used, available = bench.host_threads()
    assert used == min(3, available) and available == len(os.sched_getaffinity(0))
    monkeypatch.delenv("OMP_NUM_THREADS")
    assert bench.host_threads() == (available, available)


def test_every_tuning_alternative_names_a_hook_that_the_kernel_source_has():
    """paper_1605_08325_amd/tune.py builds its alternatives with -D flags; a flag whose macro the source no longer
    tests would build the shipped library under another name and the A/B table would compare it with itself."""
    import re
    from paper_1605_08325_amd import tune
    csrc = os.path.join(ROOT, "paper_1605_08325_amd", "csrc")
    source = "".join(open(os.path.join(csrc, f)).read() for f in os.listdir(csrc) if f.endswith((".hip", ".h"))) + \
        open(os.path.join(ROOT, "include", "pxchg.h")).read()
    assert tune.VARIANTS["shipped"] == []
    for name, flags in tune.VARIANTS.items():
        for flag in flags:
            m = re.fullmatch(r"-D(PXCHG_[A-Z0-9_]+)(=\d+)?", flag)
            assert m, (name, flag)
            assert re.search(r"#\s*(ifdef|ifndef|if|elif)\b[^\n]*\b" + m.group(1) + r"\b", source), (name, m.group(1))
