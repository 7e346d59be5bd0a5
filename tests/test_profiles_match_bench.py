"""The instruction counts and HBM traffic that bench.py prices its kernels with are readings of
rocprofv3 counters, kept as text summaries under profiles/.  This test ties the constants in
bench.py to those summaries, so that neither can change without the other."""
import os
import re

import bench

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def readings(path, counter):
    """{(configuration, op): per-launch value} from lines `<name> <eval|gen> <counter> per_launch=<value>`."""
    out = {}
    for line in open(os.path.join(ROOT, "profiles", path)):
        m = re.match(rf"(\w+) (eval|gen) {counter} per_launch=(\d+)", line)
        if m:
            out[(m.group(1), m.group(2))] = int(m.group(3))
    return out


def test_issued_instruction_counts_are_the_profiled_ones():
    lds = readings("configs_sq_counters.txt", "SQ_INSTS_LDS")
    valu = readings("configs_sq_counters.txt", "SQ_INSTS_VALU")
    assert set(bench.ISSUED) == set(bench.CONFIG_NAMES) == {name for name, _ in lds}
    for name, ops in bench.ISSUED.items():
        for op, counts in ops.items():
            assert counts["lds"] == lds[(name, op)], (name, op)
            assert counts["valu"] == valu[(name, op)], (name, op)


def test_bank_conflict_counters_read_zero():
    for counter in ("SQ_LDS_BANK_CONFLICT", "SQ_LDS_ADDR_CONFLICT"):
        r = readings("configs_sq_counters.txt", counter)
        assert len(r) == 2 * len(bench.CONFIG_NAMES) and not any(r.values()), counter


def test_hbm_traffic_is_the_profiled_one_and_equals_the_algorithmic_bytes():
    hbm = readings("hbm_counters.txt", "HBM_BYTES")
    assert "config5" in bench.MEASURED_HBM_BYTES
    shapes = {"config2": ("eq", 32, 1 << 20), "config3": ("cmp", 32, 64 * 112 * 112), "config5": ("cmp", 32, 1 << 22)}
    for name, ops in bench.MEASURED_HBM_BYTES.items():
        kind, n, batch = shapes[name]
        for op, measured in ops.items():
            assert measured == hbm[(name, op)], (name, op)
            algorithmic = batch * bench.hbm_bytes(kind, op, n)
            assert abs(measured / algorithmic - 1) < 0.01, (name, op, measured / algorithmic)       # no wasted re-reads


def test_issued_lookups_never_exceed_what_table_driven_aes_needs():
    """Sharing of coinciding lookups only removes work: issued <= algorithmic, and not by more than a fifth."""
    shapes = {"config1": ("cmp", 32, 16384), "config2": ("eq", 32, 1 << 20), "config3": ("cmp", 32, 64 * 112 * 112),
              "config4": ("cmp", 32, 64 * 56 * 56), "config5": ("cmp", 32, 1 << 22), "n16": ("cmp", 16, 1 << 22)}
    for name, (kind, n, batch) in shapes.items():
        for op in ("eval", "gen"):
            algorithmic = batch * bench.aes_blocks(kind, op, n) * bench.LOOKUPS_PER_BLOCK
            issued = bench.ISSUED[name][op]["lds"] * 64
            # the quad layout issues 64-lane instructions for 16 elements, each lane a quarter of a block
            assert 0.8 * algorithmic < issued <= 1.02 * algorithmic, (name, op, issued / algorithmic)


def test_work_model_matches_the_papers_sizes():
    assert bench.hbm_bytes("cmp", "eval", 32) == 812 and bench.hbm_bytes("eq", "eval", 32) == 548
    assert bench.hbm_bytes("cmp", "gen", 32) == 40 + 2 * 808 and bench.hbm_bytes("eq", "gen", 32) == 40 + 2 * 544
    assert bench.aes_blocks("cmp", "eval", 32) == 64 and bench.aes_blocks("cmp", "gen", 32) == 192
