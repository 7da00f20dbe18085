"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same
seeded inputs.  Bit-exact for Bloom signatures and masks, int32 dots, fp32 scores, top-K ids and
counts (the tolerance the problem statement fixes: none)."""
import sys

import numpy as np
import pytest
import torch

from oracle import st_oracle as O
from paper_2511_14881_amd import binding as st
from paper_2511_14881_amd import synth as S

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _np(t):
    return t.detach().cpu().numpy()


def _u64(t):
    return _np(t).view(np.uint64)


def oracle_index(w, m=None, k=None):
    cfg = w.cfg
    return O.bloom_build(_np(w.feat_offsets), _np(w.feat_ids).view(np.uint64), m or cfg.m_bits,
                         k or cfg.k_hashes)


def check_search(w, K, sigs=None, queries=None, path=0, label="", fast_path_only=False, slow_path=None):
    """Runs the GPU search on the whole batch and compares the chosen queries with the oracle.
    fast_path_only: also require that no query fell back to the slow exact path (a schedule that
    overflows candidate regions on an ordinary workload is a performance bug, not a wrong result).
    slow_path: (queries that must have fallen back, queries that must not have)."""
    cfg = w.cfg
    say(f"[parity] {label or cfg.name}: N={cfg.n_items} d={cfg.d} B={cfg.batch} T={cfg.n_tasks} "
        f"m={cfg.m_bits} k={cfg.k_hashes} K={K} path={path}")
    dev = [t.cuda() for t in (w.items, w.item_scale, w.feat_offsets, w.feat_ids, w.queries, w.query_scale)]
    items, iscale, foff, fids, q, qs = dev
    bloom = st.st_bloom_build(foff, fids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    old = st.st_set_scoring_path(path)
    buf = st.SearchBuffers(cfg.n_items, cfg.d, cfg.batch, max(cfg.n_tasks, 1), K)
    try:
        if cfg.n_tasks > 0:
            ids, scores, count = st.st_search_multitask(bloom, items, iscale, q, qs, w.task_weight,
                                                        w.filt_ids, w.filt_offsets, K, buffers=buf)
        else:
            ids, scores, count = st.st_search(bloom, items, iscale, q, qs, w.filt_ids, w.filt_offsets, K,
                                              buffers=buf)
        torch.cuda.synchronize()
    finally:
        st.st_set_scoring_path(old)
    if fast_path_only:
        slow = np.nonzero(_np(buf.overflow_flags()))[0]
        assert slow.size == 0, f"queries {slow[:8].tolist()}... took the slow exact path"
    if slow_path is not None:
        flags = _np(buf.overflow_flags())
        assert all(flags[b] == 1 for b in slow_path[0]) and all(flags[b] == 0 for b in slow_path[1]), flags
    ids, scores, count = _np(ids), _np(scores), _np(count)
    if sigs is None:
        sigs = oracle_index(w)
    sel = list(range(cfg.batch)) if queries is None else list(queries)
    fo = w.filt_offsets
    sub_ids = np.concatenate([w.filt_ids[fo[b]:fo[b + 1]] for b in sel]) if sel else np.zeros(0, np.uint64)
    sub_off = np.concatenate([[0], np.cumsum([fo[b + 1] - fo[b] for b in sel])]).astype(np.int64)
    oi, os_, oc = O.search(sigs, cfg.m_bits, cfg.k_hashes, _np(w.items), _np(w.item_scale),
                           _np(w.queries)[sel], _np(w.query_scale)[sel], sub_ids, sub_off, K,
                           task_weight=w.task_weight)
    for j, b in enumerate(sel):
        assert count[b] == oc[j], f"query {b}: count {count[b]} vs oracle {oc[j]}"
        bad = np.nonzero(ids[b] != oi[j])[0]
        assert bad.size == 0, (f"query {b}: first id mismatch at rank {bad[0]}: gpu {ids[b][bad[0]]} "
                               f"score {scores[b][bad[0]]} vs oracle {oi[j][bad[0]]} score {os_[j][bad[0]]}")
        assert np.array_equal(scores[b].view(np.uint32), os_[j].view(np.uint32)), f"query {b}: score bits differ"
    bloom.free()
    return ids, scores, count


def ragged_workload(seed, n, d, B, vocab, max_feats, m, k, T=0, dist="gauss"):
    """A corpus with ragged (also empty) feature lists and one random 1-2 term filter per query."""
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, max_feats + 1, n)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ids = rng.integers(0, vocab, int(off[-1])).astype(np.int64)
    cfg = S.Config(f"ragged{seed}", n, d, B, T, m, k, 2, 10, max_feats, vocab, 0.0, dist, 0.0, B)
    items = S.gen_int8(seed, S.S_ITEMS, n, d, dist)
    iscale = S.gen_scale(seed, S.S_ISCALE, n)
    Tn = max(T, 1)
    q = S.gen_int8(seed, S.S_QUERIES, B * Tn, d, dist)
    qs = S.gen_scale(seed, S.S_QSCALE, B * Tn)
    wts = None
    if T:
        q, qs = q.reshape(B, T, d), qs.reshape(B, T)
        wts = rng.uniform(0, 1, T).astype(np.float32)
    filters = [list(rng.integers(0, vocab, rng.integers(0, 3))) for _ in range(B)]
    fid = np.array([x for f in filters for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filters])]).astype(np.int64)
    return S.Workload(cfg, items, iscale, torch.from_numpy(off), torch.from_numpy(ids), q, qs, wts, fid,
                      foff, filters)


# ------------------------------------------------------------------ Bloom index
@pytest.mark.parametrize("n,m,k,host", [(1, 64, 2, True), (1000, 64, 2, False), (1025, 100, 3, True),
                                        (70_001, 256, 3, False), (5000, 768, 5, False), (3000, 1, 1, True)])
def test_bloom_signatures_and_masks_match_oracle(n, m, k, host):
    say(f"[bloom] n={n} m={m} k={k} host_csr={host}")
    w = ragged_workload(100 + n, n, 16, 6, 30, 7, m, k)
    off, ids = w.feat_offsets, w.feat_ids
    if not host:
        off, ids = off.cuda(), ids.cuda()
    bloom = st.st_bloom_build(off, ids, n, m, k)
    assert bloom.nbytes == st.st_bloom_layout_bytes(n, m) == ((n + 1023) // 1024) * 1024 * m // 8
    sigs = oracle_index(w, m, k)
    got = _u64(st.st_bloom_export_signatures(bloom))
    torch.cuda.synchronize()
    assert np.array_equal(got, sigs)
    filters = [[], [3], [3, 7], [1, 2, 29], [12345678901234567], [0]]
    fid = np.array([x for f in filters for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filters])]).astype(np.int64)
    masks = _u64(st.st_bloom_mask(bloom, fid, foff))
    for j, f in enumerate(filters):
        assert np.array_equal(masks[j], O.bloom_mask(sigs, m, k, f)), f"mask of filter {f} differs"
    bloom.free()


def test_bloom_index_of_tiny_config_has_no_false_negatives():
    w = S.make_workload(S.CONFIGS["tiny"])
    cfg = w.cfg
    bloom = st.st_bloom_build(w.feat_offsets.cuda(), w.feat_ids.cuda(), cfg.n_items, cfg.m_bits, cfg.k_hashes)
    mask = _u64(st.st_bloom_mask(bloom, w.filt_ids, w.filt_offsets[:2]))[0]
    exact = O.exact_mask(_np(w.feat_offsets), _u64(w.feat_ids), w.filt_ids)
    assert not (exact & ~mask).any()
    assert np.array_equal(mask, O.bloom_mask(oracle_index(w), cfg.m_bits, cfg.k_hashes, w.filt_ids))


# ------------------------------------------------------------------ scoring arithmetic
@pytest.mark.parametrize("d", [16, 64, 128, 256, 48])
def test_int32_dots_and_rescaled_scores_are_bit_exact(d):
    say(f"[pairs] d={d}")
    rng = np.random.default_rng(d)
    n, B, P = 4096, 8, 20_000
    items = torch.from_numpy(rng.integers(-128, 128, (n, d)).astype(np.int8))
    q = torch.from_numpy(rng.integers(-128, 128, (B, d)).astype(np.int8))
    items[0] = -128
    q[0] = -128
    isc = torch.from_numpy(rng.uniform(0.5, 1.5, n).astype(np.float32))
    qsc = torch.from_numpy(rng.uniform(0.5, 1.5, B).astype(np.float32))
    pi = torch.from_numpy(rng.integers(0, n, P).astype(np.int64))
    pq = torch.from_numpy(rng.integers(0, B, P).astype(np.int32))
    pi[0], pq[0] = 0, 0
    dots, scores = st.st_score_pairs(items.cuda(), isc.cuda(), q.cuda(), qsc.cuda(), pi.cuda(), pq.cuda())
    torch.cuda.synchronize()
    want = (items.numpy().astype(np.int64)[pi.numpy()] * q.numpy().astype(np.int64)[pq.numpy()]).sum(axis=1)
    assert np.array_equal(_np(dots).astype(np.int64), want)
    assert _np(dots)[0] == d * 128 * 128
    ws = np.array([O.rescale(int(want[i]), qsc[pq[i]].item(), isc[pi[i]].item()) for i in range(2000)],
                  dtype=np.float32)
    assert np.array_equal(_np(scores)[:2000].view(np.uint32), ws.view(np.uint32))


# ------------------------------------------------------------------ search: the five workloads
def test_tiny_config():
    check_search(S.make_workload(S.CONFIGS["tiny"]), S.CONFIGS["tiny"].top_k)


# scoring path: 0 = the library's own choice, 1 = wavefront dot product only, 2 = MFMA for every
# group whose shape allows it (also groups of a single query)
PATHS = [0, 1, 2]


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("n", [3_000, 100_003])
def test_mid_recipe_small(n, path):
    cfg = S.scaled(S.CONFIGS["mid"], n)
    check_search(S.make_workload(cfg), cfg.top_k, path=path)


def test_mid_recipe_with_literal_feature_ids():
    # correctness-only variant of the input recipe: rank r gets id r - 1 (popular ids are then
    # XOR-neighbours, which the hash family h_j(f) = splitmix64(f ^ j) must not trip over)
    cfg = S.scaled(S.CONFIGS["mid"], 100_003, scatter_ids=False)
    check_search(S.make_workload(cfg), cfg.top_k)


@pytest.mark.parametrize("name,n", [("mid", 200_000), ("multi", 120_000), ("large", 300_000)])
def test_all_distinct_filters_stress_batch(name, n):
    # every query of the batch carries its own filter (pool = batch): no query rows to share, so
    # the groups go to the wavefront dot-product scorer (or ride along in the MFMA scan)
    base = S.CONFIGS[name]
    cfg = S.scaled(base, n, pool=base.batch)
    w = S.make_workload(cfg)
    fo = w.filt_offsets
    assert len({tuple(w.filt_ids[fo[b]:fo[b + 1]]) for b in range(base.batch)}) > base.batch // 2
    for path in (0, 2):
        # (short levels of a search that uses both scorers once crowded a query's candidates into
        # four regions: the fast path has to hold here too)
        check_search(w, cfg.top_k, path=path, label=f"{name} with {base.batch} distinct filters", fast_path_only=True)


@pytest.mark.parametrize("path", PATHS)
def test_multitask_recipe_small(path):
    cfg = S.scaled(S.CONFIGS["multi"], 60_000, batch=16)
    check_search(S.make_workload(cfg), cfg.top_k, path=path)


@pytest.mark.parametrize("path", PATHS)
def test_large_recipe_small(path):
    cfg = S.scaled(S.CONFIGS["large"], 50_000, batch=32)
    check_search(S.make_workload(cfg), cfg.top_k, path=path)


@pytest.mark.parametrize("path", PATHS)
def test_mfma_recipe_small(path):
    cfg = S.scaled(S.CONFIGS["mfma"], 40_000, batch=64, top_k=300)
    check_search(S.make_workload(cfg), cfg.top_k, path=path)


def test_large_batch_splits_query_rows_over_workgroup_rows():
    # 1024 query rows of 128 bytes exceed one workgroup's resident-query budget: the rows are
    # split over two rows of workgroups, each scanning the corpus for its own queries
    cfg = S.scaled(S.CONFIGS["mfma"], 70_000, batch=1024, top_k=100)
    check_search(S.make_workload(cfg), cfg.top_k, queries=range(0, 1024, 37))


@pytest.mark.parametrize("T,d", [(1, 64), (2, 64), (4, 256), (2, 512), (3, 128)])
def test_multitask_shapes(T, d):
    w = ragged_workload(900 + T + d, 20_000, d, 24, 6, 3, 128, 2, T=T)
    check_search(w, 64, path=2, label=f"multitask T={T} d={d}")


def test_mid_config_full_size_every_query():
    # the configuration bench.py times, at full size, all 64 queries against the oracle
    cfg = S.CONFIGS["mid"]
    w = S.make_workload(cfg, device="cuda")
    check_search(w, cfg.top_k, fast_path_only=True)


@pytest.mark.parametrize("name", ["large", "multi", "mfma"])
def test_big_configs_full_size_sampled_queries(name):
    # full-size corpus and batch through the library; the oracle recomputes 64 queries spread
    # over the batch (every distinct filter of the batch is among them)
    cfg = S.CONFIGS[name]
    w = S.make_workload(cfg, device="cuda")
    step = max(cfg.batch // 64, 1)
    check_search(w, cfg.top_k, queries=range(0, cfg.batch, step), fast_path_only=True)


# ------------------------------------------------------------------ Large: the selectivity sweep
# The Large workload is specified with its filters' selectivity swept from 0.1 % to the broadest
# conjunction the frequent ids allow (about 15 %): almost every 16-item unit is padding at the low
# end, the candidate queues and regions are under the most pressure at the high end.
@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("target", S.LARGE_SWEEP)
def test_large_selectivity_sweep_small(target, path):
    cfg = S.scaled(S.CONFIGS["large"], 150_000, batch=64, target_sel=target)
    w = S.make_workload(cfg)
    check_search(w, cfg.top_k, path=path, label=f"large recipe, selectivity target {target:g}")


_LARGE_FULL = {}


@pytest.mark.parametrize("target", S.LARGE_SWEEP)
def test_large_selectivity_sweep_full_size(target):
    # full-size corpus and batch in the launch configuration bench.py times; the oracle recomputes
    # 32 queries spread over the batch (every distinct filter of the batch is among them)
    if "w" not in _LARGE_FULL:
        _LARGE_FULL["w"] = S.make_workload(S.CONFIGS["large"], device="cuda")
    w = S.refilter(_LARGE_FULL["w"], target)
    sels = set(tuple(f) for f in w.pool)
    assert len(sels) == w.cfg.pool
    check_search(w, w.cfg.top_k, queries=range(0, w.cfg.batch, 8), fast_path_only=True,
                 label=f"large at full size, selectivity target {target:g}")
    if target == S.LARGE_SWEEP[-1]:
        _LARGE_FULL.clear()


@pytest.mark.parametrize("d,T,all_pass", [(128, 0, False), (128, 0, True), (64, 2, False), (48, 0, False), (256, 4, False)])
def test_seed_pass_small_batch_large_corpus(d, T, all_pass):
    # few query rows over a corpus of at least 8 x 32768 items: the prefix is scanned by one
    # workgroup per query.  With every item passing, the prefix holds more candidates than fit
    # in LDS and the selection runs through global memory.
    w = ragged_workload(4000 + d + T, 270_001, d, 6, 9, 4, 128, 2, T=T)
    if all_pass:
        w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(7, np.int64)
    check_search(w, 150, label=f"seed pass d={d} T={T} all_pass={all_pass}")


# ------------------------------------------------------------------ search: edges
@pytest.mark.parametrize("n,d,B,K,T", [(1, 16, 1, 1, 0), (63, 16, 3, 5, 0), (64, 32, 2, 64, 0),
                                       (65, 48, 2, 100, 0), (1023, 64, 5, 7, 0), (1025, 64, 5, 2000, 0),
                                       (40_000, 32, 20, 50, 0), (33_000, 16, 40, 10, 0),
                                       (5000, 32, 6, 20, 3), (5000, 64, 3, 6000, 0), (2000, 16, 4, 9, 8)])
@pytest.mark.parametrize("path", [0, 2])
def test_ragged_sizes_and_filters(n, d, B, K, T, path):
    # ragged and empty feature lists, empty filters, filters nothing passes, K above the
    # number of passing items and above the corpus size, more distinct filters than one pass holds
    w = ragged_workload(n + d, n, d, B, 12, 4, 100, 3, T=T)
    ids, scores, count = check_search(w, K, path=path, label=f"ragged n={n} d={d} B={B} K={K} T={T}")
    for b in range(B):
        assert (ids[b, count[b]:] == -1).all() and np.isneginf(scores[b, count[b]:]).all()


@pytest.mark.parametrize("seed,n,d,B,K,T,vocab", [
    (101, 90_000, 64, 130, 1, 0, 12), (102, 150_000, 64, 200, 10, 0, 30), (103, 260_000, 128, 256, 100, 0, 8),
    (104, 400_000, 64, 140, 1000, 0, 12), (105, 400_000, 64, 136, 3000, 0, 6), (106, 180_000, 128, 66, 40, 2, 12),
    (107, 300_000, 128, 40, 200, 4, 10), (108, 300_000, 64, 100, 7, 0, 40), (109, 500_000, 64, 24, 500, 0, 12),
    (110, 270_000, 256, 160, 64, 0, 20), (111, 131_073, 64, 129, 2048, 0, 5), (112, 350_000, 64, 512, 30, 0, 16)])
def test_levels_with_tight_thresholds_on_mixed_selectivities(seed, n, d, B, K, T, vocab):
    # Plans of two and more levels (with and without a seed pass) on batches whose filters range
    # from "every item" over a few percent down to a handful of items and none at all: selections
    # that keep fewer than K keys meet queries with more, with fewer and with no passing items in
    # the first level (the last two admit without a threshold), K above and below what passes, one
    # to four tasks.  Every query is compared with the oracle, and none may need the slow path.
    w = ragged_workload(seed, n, d, B, vocab, 3, 128, 2, T=T)
    levels, _, _ = st.st_search_plan(n, B * max(T, 1), K)
    assert len(levels) >= 2
    ids, scores, count = check_search(w, K, label=f"mixed selectivities seed={seed}", fast_path_only=True)
    for b in range(B):
        assert (ids[b, count[b]:] == -1).all()


@pytest.mark.parametrize("K,B", [(5000, 6), (16384, 2), (50_000, 3), (100_000, 2)])
def test_top_k_above_the_lds_sort_size(K, B):
    # K above 2048: the running top-K lives in global memory, is carried unordered from level to
    # level and ordered once at the end (in LDS up to 16384 keys, in global memory above: the
    # paper's pre-filter sizes of 10^4 - 10^5 items, Sec. 5.1)
    n = 300_000 if K <= 16384 else 700_000
    w = ragged_workload(31 + K, n, 64, B, 12, 4, 100, 3)
    w.filt_ids = np.array([3], dtype=np.uint64)           # query 0 filtered, the others take every item
    w.filt_offsets = np.array([0] + [1] * B, dtype=np.int64)
    levels, _, _ = st.st_search_plan(n, B, K)
    assert len(levels) >= 2
    check_search(w, K, label=f"K={K}")


@pytest.mark.parametrize("B,T,d", [(48, 0, 64), (24, 2, 128), (300, 0, 64)])
def test_many_distinct_filters_through_the_mfma_scorer(B, T, d):
    # more filter groups than one pass of the MFMA scan holds (8), most of them with one or two
    # queries: several filter batches per segment, single-block groups, padding rows
    n = 120_000
    w = ragged_workload(500 + B, n, d, B, 30, 4, 128, 2, T=T)
    check_search(w, 64, path=2, label=f"many filters B={B} T={T} d={d}")


def test_empty_corpus_and_no_passing_items():
    w = ragged_workload(5, 500, 16, 3, 10, 3, 4096, 2)
    w.filt_ids = np.array([10**15, 10**15 + 16, 10**15 + 32], dtype=np.uint64)  # ids no item holds
    w.filt_offsets = np.array([0, 1, 2, 3], dtype=np.int64)
    ids, scores, count = check_search(w, 10, label="nothing passes")
    assert (count == 0).all() and (ids == -1).all()


def test_all_scores_tie_lower_id_wins():
    w = ragged_workload(6, 50_000, 32, 4, 10, 3, 64, 2)
    w.queries = torch.zeros_like(w.queries)
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(5, np.int64)
    ids, scores, _ = check_search(w, 300, label="zero queries")
    assert np.array_equal(ids, np.tile(np.arange(300), (4, 1)))
    assert (scores == 0).all()


def test_duplicate_rows_tie_in_id_order():
    w = ragged_workload(7, 30_000, 32, 3, 10, 3, 64, 2)
    w.items = w.items[:100].repeat(300, 1).contiguous()
    w.item_scale = w.item_scale[:100].repeat(300).contiguous()
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(4, np.int64)
    check_search(w, 700, label="300 copies of 100 rows")


def test_three_distinct_rows_on_the_seeded_path_stay_exact():
    # small batch, large corpus: the seed pass takes its thresholds from the best few distinct scores
    # of its slices; a corpus of three distinct rows has fewer than that, so the pass must fall back
    # to the exact selection (and the flood of equal scores that follows to the slow exact path)
    n, d, B = 300_000, 64, 4
    w = ragged_workload(21, n, d, B, 10, 3, 64, 2)
    w.items = w.items[:3].repeat(n // 3, 1).contiguous()
    w.item_scale = w.item_scale[:3].repeat(n // 3).contiguous()
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(B + 1, np.int64)
    check_search(w, 50, label="three distinct rows, seeded path")


def test_rising_scores_overflow_the_regions_and_take_the_exact_slow_path():
    # every later item beats every earlier one, so each level admits everything it scans:
    # the candidate regions overflow and the affected queries are recomputed by the slow path
    n, d, B = 150_000, 16, 3
    w = ragged_workload(8, n, d, B, 10, 3, 64, 2)
    w.items = torch.ones((n, d), dtype=torch.int8)
    w.queries = torch.ones((B, d), dtype=torch.int8)
    w.queries[1] = -1            # for this query scores fall with the id: no overflow
    w.item_scale = (0.5 + torch.arange(n, dtype=torch.float32) / n).contiguous()
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(B + 1, np.int64)
    for path in (1, 2):
        ids, _, _ = check_search(w, 50, path=path, label="rising scores", slow_path=([0], [1]))
        assert ids[0, 0] == n - 1 and ids[1, 0] == 0


def test_best_items_at_the_head_of_the_corpus_defeat_the_tight_threshold_and_take_the_exact_slow_path():
    # Batches too large for the seed pass keep fewer than K keys after the first level (the planner's
    # optimistic_keep), i.e. they admit by a threshold tighter than the K-th best so far.  That
    # threshold is too tight exactly when the best items crowd the first level: here scores fall with
    # the id, the K best are items 0..K-1, and nothing of the second level reaches the threshold.  The
    # last selection sees fewer than K keys at or above it and recomputes the query exactly.
    # Query 1 has its scores rise with the id (the regions overflow instead); both must be exact.
    n, d, B, K = 300_000, 64, 130, 500
    levels, _, _ = st.st_search_plan(n, B, K)
    assert len(levels) == 2 and levels[0, 2] != 0  # two cooperative levels, no seed pass
    w = ragged_workload(9, n, d, B, 10, 3, 64, 2)
    w.items = torch.ones((n, d), dtype=torch.int8)
    w.queries = torch.ones((B, d), dtype=torch.int8)
    w.queries[1::2] = -1
    w.item_scale = (1.5 - torch.arange(n, dtype=torch.float32) / n).contiguous()
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(B + 1, np.int64)
    for path in (0, 1):
        ids, _, count = check_search(w, K, queries=[0, 1, 2, 3, 128, 129], path=path, label="falling scores",
                                     slow_path=(list(range(B)), []))
        assert ids[0, 0] == 0 and ids[1, 0] == n - 1 and (count == K).all()


@pytest.mark.parametrize("d,B,seeded", [(256, 256, False), (64, 16, True)])
def test_scores_along_a_trend_keep_the_fast_path_where_the_first_level_is_a_sample(d, B, seeded):
    # Large batches served by the 8-wavefront MFMA scan alone take their first level as segments
    # spread evenly over the corpus, not as a prefix, and so does the seed pass of small batches
    # with its tiles.  Here the item scales fall twentyfold along the item order (a corpus ordered
    # by age or popularity), so the best items of every query crowd the head of the corpus: a
    # prefix holds far more of the final top-K than its share, and a threshold drawn from it would
    # be too tight.  The sample sees the trend like the rest of the corpus does, and no query
    # needs the slow exact path.
    n, K = 300_000, 500
    summary = st.st_search_host_plan(n, d, B, 1, K, 64, 2, np.zeros(0, np.uint64), np.zeros(B + 1, np.int64))
    assert summary["levels"] == 2 and summary["seed_pass"] == (1 if seeded else 0)
    assert seeded or summary["waves"] == 8
    w = ragged_workload(11, n, d, B, 10, 3, 64, 2)
    w.item_scale = (4.0 * torch.exp(-3.0 * torch.arange(n, dtype=torch.float32) / n)).contiguous()
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(B + 1, np.int64)
    ids, _, count = check_search(w, K, queries=range(0, B, 16), label="scores along a trend, sampled first level",
                                 slow_path=([], list(range(B))))
    assert (count == K).all()
    # the premise: the prefix a plain first level would scan holds well over its share of the results
    prefix = 32768 if seeded else 65536
    assert np.mean(ids[::16] < prefix) > 2.5 * prefix / n


def test_hot_items_exactly_where_the_seed_pass_looks_defeat_it_and_take_the_exact_slow_path():
    # Small batches take their first threshold from the seed pass over 512 words of 64 items spread
    # evenly over the corpus, and that threshold too is tighter than the K-th best of what the pass
    # has seen.  Here exactly the words the pass looks at carry a scale sixteen times that of the
    # rest (a period in the corpus that matches the stride of the sample), so the K best of the
    # corpus all lie inside the sample: the threshold lands among them, fewer than K keys of the
    # corpus reach it, and the last selection recomputes every query exactly.  A block of hot
    # items anywhere else (second call) is seen in proportion and stays on the fast path.
    n, d, B, K = 300_000, 64, 6, 500
    levels, _, _ = st.st_search_plan(n, B, K)
    assert levels[0, 2] == 0 and len(levels) == 2  # seed pass, then one level over the corpus
    pass_words = int(levels[0, 1]) // 64
    stride = (n // 64) // pass_words
    assert stride >= 2
    w = ragged_workload(10, n, d, B, 10, 3, 64, 2)
    w.filt_ids, w.filt_offsets = np.zeros(0, np.uint64), np.zeros(B + 1, np.int64)
    word = torch.arange(n) // 64
    sampled = (word % stride == 0) & (word // stride < pass_words)
    w.item_scale = torch.where(sampled, torch.tensor(4.0), torch.tensor(0.25)).contiguous()
    for path in (0, 1):
        ids, _, count = check_search(w, K, path=path, label="hot items at the sampled words",
                                     slow_path=(list(range(B)), []))
        assert (count == K).all() and sampled.numpy()[ids].all()
    scale = torch.full((n,), 0.25, dtype=torch.float32)
    scale[:32768] = 4.0
    w.item_scale = scale.contiguous()
    ids, _, count = check_search(w, K, label="a block of hot items", slow_path=([], list(range(B))))
    assert (count == K).all() and (ids < 32768).all()


@pytest.mark.parametrize("B", [16, 48])
def test_loose_threshold_admits_most_pairs_of_a_later_level(B):
    # K is close to the number of items of the first level that pass the filter, so the threshold
    # the second level starts with admits most of its (query, item) pairs: with three query blocks
    # in one filter group a single 16-item unit yields more admissions than a wavefront's queue
    # holds, and the scan has to fall back from its pipelined loop without losing or doubling any
    n = 150_000
    w = ragged_workload(77, n, 64, B, 40, 3, 256, 2)
    w.filt_ids, w.filt_offsets = np.full(B, 7, np.uint64), np.arange(B + 1, dtype=np.int64)
    levels, _, _ = st.st_search_plan(n, B, 2000)
    assert len(levels) >= 2
    check_search(w, 2000, label=f"loose threshold B={B}")


@pytest.mark.parametrize("kind", ["loguniform", "tiny", "mixed"])
@pytest.mark.parametrize("B", [8, 40])
def test_wide_range_of_scales_keeps_the_exact_ranking(kind, B):
    # admission is tested against a bound derived from the threshold and the two scales; the
    # ranking must stay the exact fp32 one whatever the magnitudes (also where the scale of an
    # item is so small that the bound is not trusted and the item takes the exact test alone)
    n, d = 200_000, 64
    w = ragged_workload(91, n, d, B, 40, 3, 256, 2)
    rng = np.random.default_rng(5)
    if kind == "loguniform":
        isc = np.exp(rng.uniform(np.log(1e-3), np.log(1e3), n))
        qsc = np.exp(rng.uniform(np.log(1e-3), np.log(1e3), B))
    elif kind == "tiny":
        isc = rng.choice([1e-35, 3e-33, 1e-39], n)
        qsc = rng.uniform(0.5e6, 1.5e6, B)
    else:
        isc = rng.uniform(0.5, 1.5, n)
        pick = rng.uniform(0, 1, n)
        isc[pick < 0.02] = 1e-39
        isc[(pick >= 0.02) & (pick < 0.04)] = 1e-35
        isc[(pick >= 0.04) & (pick < 0.06)] = 1e-20
        isc[(pick >= 0.06) & (pick < 0.065)] = 1e20
        qsc = rng.uniform(0.5, 1.5, B)
        qsc[0] = 1e-32
    w.item_scale = torch.from_numpy(isc.astype(np.float32))
    w.query_scale = torch.from_numpy(qsc.astype(np.float32))
    w.filt_ids, w.filt_offsets = np.full(B, 7, np.uint64), np.arange(B + 1, dtype=np.int64)
    check_search(w, 300, label=f"scales {kind} B={B}")


def test_results_are_deterministic():
    cfg = S.scaled(S.CONFIGS["mid"], 80_000)
    w = S.make_workload(cfg)
    a = check_search(w, cfg.top_k, queries=[0, 1], label="determinism run 1")
    b = check_search(w, cfg.top_k, queries=[0, 1], label="determinism run 2")
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_concurrent_searches_on_two_streams():
    # two host threads, each with its own stream, workspace and outputs, share one index
    import threading
    cfg = S.scaled(S.CONFIGS["mid"], 150_000)
    w = S.make_workload(cfg, device="cuda")
    bloom = st.st_bloom_build(w.feat_offsets, w.feat_ids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    ref = [t.clone() for t in st.st_search(bloom, w.items, w.item_scale, w.queries, w.query_scale,
                                           w.filt_ids, w.filt_offsets, cfg.top_k)]
    torch.cuda.synchronize()
    errors = []

    def worker(i):
        try:
            stream = torch.cuda.Stream()
            buf = st.SearchBuffers(cfg.n_items, cfg.d, cfg.batch, 1, cfg.top_k)
            for _ in range(30):
                ids, scores, count = st.st_search(bloom, w.items, w.item_scale, w.queries, w.query_scale,
                                                  w.filt_ids, w.filt_offsets, cfg.top_k, buffers=buf, stream=stream)
            stream.synchronize()
            for a, b in zip((ids, scores, count), ref):
                if not torch.equal(a, b):
                    errors.append(f"thread {i}: results differ")
        except Exception as e:  # noqa: BLE001
            errors.append(f"thread {i}: {e!r}")

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    bloom.free()


# ------------------------------------------------------------------ search: argument errors
def test_error_paths_return_codes():
    w = ragged_workload(9, 2000, 16, 2, 10, 3, 64, 2)
    items, isc, q, qs = w.items.cuda(), w.item_scale.cuda(), w.queries.cuda(), w.query_scale.cuda()
    bloom = st.st_bloom_build(w.feat_offsets, w.feat_ids, 2000, 64, 2)
    buf = st.SearchBuffers(2000, 16, 2, 1, 10)
    small = st.SearchBuffers(2000, 16, 2, 1, 10)
    small.nbytes = 1024
    with pytest.raises(st.StError) as e:
        st.st_search(bloom, items, isc, q, qs, w.filt_ids, w.filt_offsets, 10, buffers=small)
    assert e.value.code == st.ST_EWORKSPACE
    with pytest.raises(st.StError) as e:  # corpus size differs from the index
        st.st_search(bloom, items[:1000].contiguous(), isc[:1000].contiguous(), q, qs, w.filt_ids,
                     w.filt_offsets, 10, buffers=buf)
    assert e.value.code == st.ST_EINVAL
    wide = st.st_bloom_build(w.feat_offsets, w.feat_ids, 2000, 8192, 2)
    many = np.arange(0, 16 * 40, 16, dtype=np.uint64)  # 40 terms x 2 hashes > 64 signature bits
    with pytest.raises(st.StError) as e:
        st.st_search(wide, items, isc, q, qs, np.concatenate([many, many]), np.array([0, 40, 80]), 10,
                     buffers=buf)
    assert e.value.code == st.ST_EINVAL
    wide.free()
    # the library is still usable afterwards
    st.st_search(bloom, items, isc, q, qs, w.filt_ids, w.filt_offsets, 10, buffers=buf)
    torch.cuda.synchronize()
    bloom.free()


def test_overflow_in_the_level_after_the_seed_pass_is_caught():
    # The seed pass looks at 512 words of 64 items spread over the corpus only.  Here no item of
    # those words passes the filter of the even queries, so their threshold stays open and the one
    # level after the seed pass admits a whole dense block of passing items: far more than the
    # candidate regions hold.  Those queries must be flagged and recomputed by the slow exact path,
    # not silently truncated.
    n, d, B, K = 300_000, 64, 6, 50
    w = ragged_workload(91, n, d, B, 30, 3, 128, 3)
    off = np.arange(n + 1, dtype=np.int64)
    ids = np.full(n, 2000, dtype=np.int64)
    ids[100_000:160_000] = 1000
    levels, _, _ = st.st_search_plan(n, B, K)
    assert levels[0, 2] == 0  # seed pass
    stride = (n // 64) // (int(levels[0, 1]) // 64)
    ids[(np.arange(n) // 64) % stride == 0] = 2000  # nothing the pass looks at passes filter 1000
    filters = [[1000] if b % 2 == 0 else [2000] for b in range(B)]
    w.feat_offsets, w.feat_ids = torch.from_numpy(off), torch.from_numpy(ids)
    w.filt_ids = np.array([x for f in filters for x in f], dtype=np.uint64)
    w.filt_offsets = np.arange(B + 1, dtype=np.int64)
    w.pool = filters
    check_search(w, K, label="dense block behind an empty prefix", slow_path=([0, 2, 4], []))
