"""Host-side checks that need no GPU: the shared library loads, exports every symbol the header
declares, and its pure-arithmetic entry points (layout size, schedule, workspace, argument
checks) behave as documented."""
import os
import re

import numpy as np
import pytest

from paper_2511_14881_amd import binding as st
from tests.helpers import read_golden

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "silvertorch.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_symbols()
    assert len(names) >= 14
    lib = st.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert sorted(st.EXPORTS) == names
    assert lib.st_version() >= 100


def test_index_size_is_items_times_bits_over_eight():
    # paper Sec. 6.2.2: 40M items at 512/768/1024/2048 bits -> 2.56/3.84/5/10 GB (+ tile padding)
    for row in read_golden("paper_arithmetic.txt"):
        if row[0] != "bytes":
            continue
        n, m, nbytes = int(row[1]), int(row[2]), float(row[3])
        got = st.st_bloom_layout_bytes(n, m)
        assert got >= nbytes and got - nbytes < 1024 * m / 8 + 1
    assert st.st_bloom_layout_bytes(1024, 64) == 1024 * 64 // 8
    assert st.st_bloom_layout_bytes(1, 64) == 1024 * 64 // 8
    assert st.st_bloom_layout_bytes(0, 64) == 0
    with pytest.raises(st.StError) as e:
        st.st_bloom_layout_bytes(10, 0)
    assert e.value.code == st.ST_EINVAL
    with pytest.raises(st.StError):
        st.st_bloom_layout_bytes(1 << 31, 64)


@pytest.mark.parametrize("n,B,K", [(0, 1, 1), (1, 1, 10), (10_000, 1, 10), (1_000_000, 64, 100),
                                   (10_000_000, 256, 500), (5_000_000, 128, 200),
                                   (20_000_000, 1024, 1000), (123_457, 7, 16384), (3_000_000, 16, 100_000),
                                   (2**31 - 1, 4, 5)])
@pytest.mark.parametrize("q_split", [1, 2, 8])
def test_schedule_covers_the_corpus_once(n, B, K, q_split):
    levels, groups, cap = st.st_search_plan(n, B, K, q_split)
    assert groups == 1024 and cap in (64, 128, 256, 512)
    assert groups * cap >= 2 * K + 2048
    assert levels[0, 0] == 0 and levels[-1, 1] == n
    seeded = levels[0, 2] == 0 and n > 0
    for i, (b, e, seg) in enumerate(levels):
        assert e >= b and seg % 64 == 0 and seg <= 2048  # seg = items a workgroup takes per visit
        if i == 1 and seeded:
            # the seed pass only yields thresholds: the level after it starts over at item 0
            assert b == 0 and e > levels[0, 1]
        elif i:
            assert b == levels[i - 1, 1] and e > b and b % 1024 == 0
    b, e, seg = levels[0]
    if seeded:
        # small batch, large corpus: the prefix is scanned by the per-query seed kernel
        assert B <= 128 and n >= 8 * 32768 and e == 32768
    elif n == 0:
        assert len(levels) == 1
    else:
        # level 0: `cap` items per workgroup at most, so its regions cannot overflow
        assert seg == cap and (e - b + seg - 1) // seg <= groups // q_split
    assert len(levels) <= 32


def test_workspace_size_and_argument_checks():
    a = st.st_search_workspace_bytes(1_000_000, 128, 64, 1, 100)
    assert a > 0 and a % 256 == 0
    assert st.st_search_workspace_bytes(1_000_000, 128, 128, 1, 100) > a
    for bad in [(-1, 128, 1, 1, 1), (10, 100, 1, 1, 1), (10, 0, 1, 1, 1), (10, 128, 0, 1, 1),
                (10, 128, 5000, 1, 1), (10, 128, 1, 0, 1), (10, 128, 1, 9, 1), (10, 128, 1, 1, 0),
                (10, 128, 1, 1, 200000), (10, 8192, 1, 1, 1)]:
        with pytest.raises(st.StError) as e:
            st.st_search_workspace_bytes(*bad)
        assert e.value.code == st.ST_EINVAL
        assert st.last_error()


def test_expression_workspace_adds_mask_rows_and_tables():
    base = st.st_search_workspace_bytes(1_000_000, 128, 64, 1, 100)
    a = st.st_search_expr_workspace_bytes(1_000_000, 128, 64, 1, 100, 0)
    # one 128-byte line per query and 1024-item tile, plus the (here nearly empty) tables
    assert a >= base + 977 * 64 * 128 and a - base - 977 * 64 * 128 < 4096
    b = st.st_search_expr_workspace_bytes(1_000_000, 128, 64, 1, 100, 64 * 8)
    assert b > a and b - a <= 64 * 8 * 17 * 4 + 256
    for bad in [(-1, 128, 64, 1, 100, 0), (1000, 128, 64, 1, 100, -1), (1000, 128, 64, 1, 100, 64 * 256 + 1)]:
        with pytest.raises(st.StError) as e:
            st.st_search_expr_workspace_bytes(*bad)
        assert e.value.code == st.ST_EINVAL


def test_null_arguments_are_rejected_without_touching_a_gpu():
    lib = st.lib()
    assert lib.st_bloom_free(None) == 0
    assert lib.st_bloom_bytes(None) == st.ST_EINVAL
    assert lib.st_bloom_build(None, None, 0, 64, 2, None, None) == st.ST_EINVAL
    assert lib.st_search(None, None, None, 0, 16, None, None, 1, None, None, 1, None, None, None, None, 0,
                         None) == st.ST_EINVAL
    assert lib.st_bloom_mask_expr(None, None, None, None, 0, None, None) == st.ST_EINVAL
    assert lib.st_search_expr(None, None, None, 0, 16, None, None, 1, 1, None, None, None, None, 1, None, None,
                              None, None, 0, None) == st.ST_EINVAL
    assert lib.st_score_pairs(None, None, 16, None, None, None, None, 0, None, None, None) == st.ST_EINVAL
    assert lib.st_set_scoring_path(0) in (0, 1, 2)


def _plan(n, d, batch, tasks, K, m, k, filters):
    ids, off = [], [0]
    for f in filters:
        ids += list(f)
        off.append(len(ids))
    return st.st_search_host_plan(n, d, batch, tasks, K, m, k, np.array(ids, dtype=np.uint64),
                                  np.array(off, dtype=np.int64))


def test_host_plan_groups_queries_by_their_filter_as_a_set():
    # Sec. 4.2: a filter is the conjunction of its terms, so the order of the terms, and a term
    # given twice, make no new filter; queries of one filter share one group
    rng = np.random.default_rng(3)
    pool = [tuple(int(x) for x in rng.integers(1, 1 << 40, 2)) for _ in range(8)]
    same_order = [pool[q % 8] for q in range(64)]
    mixed_order = [pool[q % 8][::-1] if q % 2 else pool[q % 8] for q in range(64)]
    a = _plan(1_000_000, 128, 64, 1, 100, 256, 3, same_order)
    b = _plan(1_000_000, 128, 64, 1, 100, 256, 3, mixed_order)
    assert a == b
    assert a["distinct_filters"] == 8 and a["mfma_groups"] == 8 and a["dot_groups"] == 0
    assert a["levels"] == 2 and a["seed_pass"] == 1 and a["q_split"] == 1 and a["waves"] == 4
    c = _plan(1_000_000, 128, 4, 1, 100, 256, 3, [(7, 7), (), (9,), ()])
    assert c["distinct_filters"] == 3  # {7}, the empty filter (twice), {9}
    d = _plan(1_000_000, 128, 3, 1, 100, 256, 3, [(7, 7), (7,), (7, 7, 7)])
    assert d["distinct_filters"] == 1


def test_host_plan_routes_groups_by_size_and_shape():
    # one query per filter: nothing to share, every group goes to the wavefront-dot form
    solo = _plan(1_000_000, 128, 64, 1, 100, 256, 3, [(i + 1,) for i in range(64)])
    assert solo["distinct_filters"] == 64 and solo["mfma_groups"] == 0 and solo["dot_groups"] == 64
    # the four benchmark shapes: level counts as st_search_plan gives them, the large batches in
    # 8-wavefront workgroups without a seed pass, batch 1024 split over two passes of query rows
    pool = [(11 * i + 1, 13 * i + 2) for i in range(8)]
    large = _plan(10_000_000, 256, 256, 1, 500, 512, 4, [pool[q % 8] for q in range(256)])
    assert (large["mfma_groups"], large["waves"], large["levels"], large["seed_pass"]) == (8, 8, 2, 0)
    multi = _plan(5_000_000, 128, 128, 4, 200, 256, 3, [pool[q % 8] for q in range(128)])
    assert (multi["mfma_groups"], multi["waves"], multi["levels"], multi["seed_pass"]) == (8, 8, 2, 0)
    dense = _plan(20_000_000, 128, 1024, 1, 1000, 128, 2, [pool[q % 2][:1] for q in range(1024)])
    assert dense["distinct_filters"] == 2 and dense["q_split"] == 2 and dense["levels"] == 3
    for p, shape in ((large, (10_000_000, 256, 500)), (multi, (5_000_000, 128 * 4, 200)),
                     (dense, (20_000_000, 1024, 1000))):
        levels, _, _ = st.st_search_plan(*shape, p["q_split"])
        assert p["levels"] == len(levels)
    # the per-call tables stay small: they are what one call uploads before its first launch
    assert 0 < large["table_bytes"] < 64 * 1024 and 0 < dense["table_bytes"] < 64 * 1024


def test_host_plan_rejects_bad_arguments():
    with pytest.raises(ValueError):
        _plan(1_000_000, 128, 2, 1, 100, 256, 3, [(1,)])  # offsets shorter than the batch: the binding refuses
    with pytest.raises(st.StError) as e:
        st.st_search_host_plan(1_000_000, 100, 1, 1, 100, 256, 3, np.array([1], dtype=np.uint64),
                               np.array([0, 1], dtype=np.int64))
    assert e.value.code == st.ST_EINVAL
    with pytest.raises(st.StError):
        st.st_search_host_plan(1_000_000, 128, 1, 1, 200_000, 256, 3, np.array([1], dtype=np.uint64),
                               np.array([0, 1], dtype=np.int64))


def test_optimistic_keep_bounds_the_chance_of_a_too_tight_threshold(tmp_path):
    # The planner lets the selection after a prefix keep r < K keys; the r-th best key of the
    # prefix is a valid threshold unless the prefix holds r or more of the K best items of the
    # corpus.  With item order carrying no information that count is hypergeometric; the planner
    # promises a chance below 1e-12.  Checked against scipy's exact tail, not the planner's bound.
    import shutil
    import subprocess
    from scipy.stats import hypergeom
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "plan_keep")
    src = os.path.join(ROOT, "tests", "plan_keep_host_test.cpp")
    inc = os.path.join(ROOT, "paper_2511_14881_amd", "csrc")
    subprocess.run([cxx, "-std=c++17", "-O1", "-I", inc, src, "-o", exe], check=True)
    cases = [(500, 65536, 10_000_000), (200, 65536, 5_000_000), (1000, 32768, 20_000_000), (100, 32768, 1_000_000),
             (10_000, 65536, 1_000_000), (100_000, 262144, 1_000_000), (2048, 9_357_312, 40_000_000),
             (500, 65536, 2**31 - 1), (500, 65536, 300_000), (16, 65536, 131072), (1, 65536, 10_000_000),
             (500, 9_999_999, 10_000_000), (500, 10_000_000, 10_000_000), (500, 20_000_000, 10_000_000)]
    out = subprocess.run([exe] + [str(x) for c in cases for x in c], capture_output=True, text=True, check=True)
    keeps = [int(x) for x in out.stdout.split()]
    assert len(keeps) == len(cases)
    for (K, prefix, n), r in zip(cases, keeps):
        assert 1 <= r <= K
        if prefix >= n:
            assert r == K
            continue
        if r < K:  # P(at least r of the K best lie in the prefix)
            assert hypergeom.sf(r - 1, n, K, prefix) < 1e-12, (K, prefix, n, r)
        mean = K * prefix / n
        assert r >= mean  # never below the expected count
    # the benchmark shapes get thresholds far tighter than the K-th best of the prefix
    assert keeps[0] <= 32 and keeps[1] <= 32 and keeps[2] <= 32


def test_first_level_is_halved_only_where_the_last_selection_stays_small(tmp_path):
    # A search that samples its first level may take it at half the size when two levels remain and
    # the second would hand the final selection at most 3500 keys per query (K + what it admits).
    import shutil
    import subprocess
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host C++ compiler")
    exe = str(tmp_path / "plan_levels")
    src = os.path.join(ROOT, "tests", "plan_keep_host_test.cpp")
    inc = os.path.join(ROOT, "paper_2511_14881_amd", "csrc")
    subprocess.run([cxx, "-std=c++17", "-O1", "-I", inc, src, "-o", exe], check=True)
    cases = [(5_000_000, 200, 1), (5_000_000, 200, 0), (10_000_000, 500, 1), (20_000_000, 1000, 1), (1_000_000, 100, 1),
             (40_000, 10, 1)]
    out = subprocess.run([exe, "levels"] + [str(x) for c in cases for x in c], capture_output=True, text=True, check=True)
    rows = [tuple(int(v) for v in line.split()) for line in out.stdout.splitlines()]
    assert rows[0] == (2, 32768)        # Multi's sizes: halved
    assert rows[1] == (2, 65536)        # ... not for a search that keeps the prefix
    assert rows[2] == (2, 65536)        # Large: 18 * 304 + 500 keys would be too many
    assert rows[3][0] == 3 and rows[3][1] == 65536   # three levels: left alone
    assert rows[4] == (2, 32768)        # K = 100 on 1 M items: 27 * 29.5 + 100
    assert rows[5][1] == 40_000         # a corpus smaller than the first level: one level
    for (n, K, small), (levels, end0) in zip(cases, rows):
        if small and levels == 2 and end0 == 32768:
            keep = int(subprocess.run([exe, str(K), str(end0), str(n)], capture_output=True, text=True, check=True).stdout)
            assert K + keep * (n / end0 - 1) <= 3500
