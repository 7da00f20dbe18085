"""GPU parity of the boolean filter expressions (paper Sec. 4 query form, Sec. 4.3 operation
array on a stack): masks and searches through the C ABI against the CPU oracle, bit-exact."""
import numpy as np
import pytest
import torch

from oracle import st_oracle as O
from paper_2511_14881_amd import binding as st
from paper_2511_14881_amd import synth as S
from tests.test_gpu_parity import _np, _u64, oracle_index, ragged_workload, say
from tests.test_oracle_expr_pins import postfix, random_tree

pytestmark = pytest.mark.gpu


def pack(programs):
    ops = np.array([o for p in programs for o in p[0]], dtype=np.int32)
    ids = np.array([i for p in programs for i in p[1]], dtype=np.uint64)
    off = np.concatenate([[0], np.cumsum([len(p[0]) for p in programs])]).astype(np.int64)
    return ops, ids, off


def random_programs(seed, n, vocab, depth=4):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        out.append(([], []) if i % 7 == 3 else postfix(random_tree(rng, vocab, depth)))
    return out


def check_expr_search(w, programs_per_query, K, sigs=None, queries=None, path=0, label="", fast_path_only=False):
    """GPU st_search_expr on the whole batch against the oracle on the chosen queries."""
    cfg = w.cfg
    ops, ids, off = pack(programs_per_query)
    say(f"[expr] {label or cfg.name}: N={cfg.n_items} d={cfg.d} B={cfg.batch} T={cfg.n_tasks} K={K} path={path} "
        f"entries={ops.size}")
    items, iscale, foff, fids, q, qs = [t.cuda() for t in (w.items, w.item_scale, w.feat_offsets, w.feat_ids,
                                                         w.queries, w.query_scale)]
    bloom = st.st_bloom_build(foff, fids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    T = max(cfg.n_tasks, 1)
    buf = st.SearchBuffers(cfg.n_items, cfg.d, cfg.batch, T, K, n_expr_entries=int(off[-1]))
    old = st.st_set_scoring_path(path)
    try:
        g_ids, g_scores, g_count = st.st_search_expr(bloom, items, iscale, q, qs, ops, ids, off, K,
                                                     task_weight=w.task_weight, buffers=buf)
        torch.cuda.synchronize()
    finally:
        st.st_set_scoring_path(old)
    if fast_path_only:
        slow = np.nonzero(_np(buf.overflow_flags()))[0]
        assert slow.size == 0, f"queries {slow[:8].tolist()}... took the slow exact path"
    g_ids, g_scores, g_count = _np(g_ids), _np(g_scores), _np(g_count)
    if sigs is None:
        sigs = oracle_index(w)
    sel = list(range(cfg.batch)) if queries is None else list(queries)
    s_ops, s_ids, s_off = pack([programs_per_query[b] for b in sel])
    oi, os_, oc = O.search_expr(sigs, cfg.m_bits, cfg.k_hashes, _np(w.items), _np(w.item_scale),
                                _np(w.queries)[sel], _np(w.query_scale)[sel], s_ops, s_ids, s_off, K,
                                task_weight=w.task_weight)
    for j, b in enumerate(sel):
        assert g_count[b] == oc[j], f"query {b}: count {g_count[b]} vs oracle {oc[j]}"
        bad = np.nonzero(g_ids[b] != oi[j])[0]
        assert bad.size == 0, f"query {b}: first id mismatch at rank {bad[0]}: gpu {g_ids[b][bad[0]]} vs {oi[j][bad[0]]}"
        assert np.array_equal(g_scores[b].view(np.uint32), os_[j].view(np.uint32)), f"query {b}: score bits differ"
    bloom.free()
    return g_ids, g_scores, g_count


# ------------------------------------------------------------------ masks
@pytest.mark.parametrize("n,m,k", [(1, 64, 2), (1000, 64, 2), (1025, 100, 3), (70_001, 256, 3), (5000, 768, 5)])
def test_expression_masks_match_oracle(n, m, k):
    say(f"[expr-mask] n={n} m={m} k={k}")
    w = ragged_workload(300 + n, n, 16, 6, 30, 7, m, k)
    bloom = st.st_bloom_build(w.feat_offsets.cuda(), w.feat_ids.cuda(), n, m, k)
    sigs = oracle_index(w, m, k)
    programs = random_programs(n, 40, 30)
    # the deepest stack the library allows: sixteen leaves, then fifteen operators
    programs.append(([O.LEAF] * 16 + [O.OR, O.AND] * 7 + [O.OR], list(range(16)) + [0] * 15))
    programs.append(([O.LEAF, O.NOT], [12345678901234567, 0]))
    ops, ids, off = pack(programs)
    masks = _u64(st.st_bloom_mask_expr(bloom, ops, ids, off))
    for j, (o, i) in enumerate(programs):
        assert np.array_equal(masks[j], O.expr_mask(sigs, m, k, o, i)), f"mask of program {j} {o} differs"
    bloom.free()


def test_ill_formed_programs_are_rejected():
    w = ragged_workload(7, 500, 16, 4, 30, 5, 64, 2)
    bloom = st.st_bloom_build(w.feat_offsets.cuda(), w.feat_ids.cuda(), 500, 64, 2)
    items, iscale, q, qs = w.items.cuda(), w.item_scale.cuda(), w.queries.cuda(), w.query_scale.cuda()
    good = ([O.LEAF], [1])
    for bad in (([O.AND], [0]), ([O.LEAF, O.LEAF], [1, 2]), ([O.LEAF, O.NOT, O.OR], [1, 0, 0]), ([9], [0]),
                ([O.LEAF] * 17 + [O.AND] * 16, [1] * 33), ([O.LEAF] + [O.NOT] * 256, [1] * 257)):
        ops, ids, off = pack([good, bad])
        with pytest.raises(st.StError) as e:
            st.st_bloom_mask_expr(bloom, ops, ids, off)
        assert e.value.code == st.ST_EINVAL
        ops, ids, off = pack([good, good, bad, good])
        with pytest.raises(st.StError) as e:
            st.st_search_expr(bloom, items, iscale, q, qs, ops, ids, off, 10)
        assert e.value.code == st.ST_EINVAL
    # a workspace sized for the plain search is too small
    ops, ids, off = pack([good] * 4)
    with pytest.raises(st.StError) as e:
        st.st_search_expr(bloom, items, iscale, q, qs, ops, ids, off, 10, buffers=st.SearchBuffers(500, 16, 4, 1, 10))
    assert e.value.code == st.ST_EWORKSPACE
    torch.cuda.synchronize()
    bloom.free()


# ------------------------------------------------------------------ search
@pytest.mark.parametrize("path", [0, 1, 2])
@pytest.mark.parametrize("n,d,B,T,K", [(3000, 64, 9, 0, 20), (70_001, 128, 33, 0, 100), (20_000, 128, 12, 3, 50),
                                       (50_000, 64, 40, 4, 64)])
def test_expression_search_matches_oracle(n, d, B, T, K, path):
    w = ragged_workload(400 + n, n, d, B, 24, 6, 128, 3, T=T)
    programs = random_programs(n + B, B, 24, depth=3)
    check_expr_search(w, programs, K, path=path, label=f"ragged n={n}")


def test_conjunction_programs_give_the_plain_search_result():
    w = ragged_workload(55, 30_000, 64, 16, 20, 6, 128, 3)
    programs = []
    for f in w.pool:
        f = [int(x) for x in f]
        programs.append(([], []) if not f else ([O.LEAF] + [x for _ in f[1:] for x in (O.LEAF, O.AND)],
                                                [f[0]] + [x for g in f[1:] for x in (g, 0)]))
    g_ids, g_scores, g_count = check_expr_search(w, programs, 40, label="conjunctions")
    items, iscale, q, qs = w.items.cuda(), w.item_scale.cuda(), w.queries.cuda(), w.query_scale.cuda()
    bloom = st.st_bloom_build(w.feat_offsets.cuda(), w.feat_ids.cuda(), 30_000, 128, 3)
    p_ids, p_scores, p_count = st.st_search(bloom, items, iscale, q, qs, w.filt_ids, w.filt_offsets, 40)
    torch.cuda.synchronize()
    assert np.array_equal(_np(p_ids), g_ids) and np.array_equal(_np(p_count), g_count)
    assert np.array_equal(_np(p_scores).view(np.uint32), g_scores.view(np.uint32))
    bloom.free()


def test_every_query_its_own_program():
    # more distinct programs than the MFMA scorer takes filter groups: both scorers in one search
    w = ragged_workload(66, 40_000, 128, 160, 40, 6, 256, 3)
    programs = [postfix(("and", ("leaf", b % 40), ("not", ("leaf", (b * 7 + 1) % 40)))) if b % 2 else
                postfix(("or", ("leaf", b % 40), ("leaf", (b // 40 + b + 3) % 40))) for b in range(160)]
    check_expr_search(w, programs, 30, label="160 programs")


@pytest.mark.parametrize("name,n", [("mid", 200_000), ("multi", 150_000)])
def test_query_form_recipe_scaled(name, n):
    cfg = S.scaled(S.CONFIGS[name], n)
    w = S.make_workload(cfg)
    ops, ids, off, pool = S.gen_filter_programs(cfg)
    programs = [(ops[off[b]:off[b + 1]].tolist(), ids[off[b]:off[b + 1]].tolist()) for b in range(cfg.batch)]
    check_expr_search(w, programs, cfg.top_k, label=f"{name} query form", queries=range(0, cfg.batch, 3))


def test_query_form_recipe_mid_full_size():
    cfg = S.CONFIGS["mid"]
    w = S.make_workload(cfg)
    ops, ids, off, pool = S.gen_filter_programs(cfg)
    programs = [(ops[off[b]:off[b + 1]].tolist(), ids[off[b]:off[b + 1]].tolist()) for b in range(cfg.batch)]
    # one query per program of the pool (the oracle scans 1M items per query)
    seen, sel = set(), []
    for b in range(cfg.batch):
        key = tuple(programs[b][0]) + tuple(programs[b][1])
        if key not in seen:
            seen.add(key)
            sel.append(b)
    check_expr_search(w, programs, cfg.top_k, label="mid query form, full size", queries=sel, fast_path_only=True)


# ------------------------------------------------------------------ cluster probing (IVF)
def check_ivf(w, programs_per_query, n_clusters, n_probe, K, queries=None, path=0, label="", fast_path_only=False):
    cfg = w.cfg
    ops, ids, off = pack(programs_per_query)
    say(f"[ivf] {label or cfg.name}: N={cfg.n_items} d={cfg.d} B={cfg.batch} K={K} clusters={n_clusters} "
        f"probes={n_probe} path={path}")
    cent, cs, coff = S.gen_clusters(cfg, n_clusters)
    items, iscale, foff, fids, q, qs = [t.cuda() for t in (w.items, w.item_scale, w.feat_offsets, w.feat_ids,
                                                         w.queries, w.query_scale)]
    bloom = st.st_bloom_build(foff, fids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    buf = st.IvfBuffers(cfg.n_items, cfg.d, cfg.batch, K, n_clusters, n_probe, int(off[-1]))
    old = st.st_set_scoring_path(path)
    try:
        g = st.st_search_ivf(bloom, items, iscale, cent.cuda(), cs.cuda(), coff.cuda(), n_probe, q, qs, ops, ids, off,
                             K, buffers=buf)
        torch.cuda.synchronize()
    finally:
        st.st_set_scoring_path(old)
    if fast_path_only:
        slow = np.nonzero(_np(buf.overflow_flags()))[0]
        assert slow.size == 0, f"queries {slow[:8].tolist()}... took the slow exact path"
    g_ids, g_scores, g_count, g_probes = [_np(t) for t in g]
    sigs = oracle_index(w)
    sel = list(range(cfg.batch)) if queries is None else list(queries)
    s_ops, s_ids, s_off = pack([programs_per_query[b] for b in sel])
    oi, os_, oc, op = O.search_ivf(sigs, cfg.m_bits, cfg.k_hashes, _np(w.items), _np(w.item_scale), _np(cent),
                                   _np(cs), _np(coff), n_probe, _np(w.queries)[sel], _np(w.query_scale)[sel],
                                   s_ops, s_ids, s_off, K)
    for j, b in enumerate(sel):
        assert np.array_equal(g_probes[b], op[j]), f"query {b}: probed clusters differ"
        assert g_count[b] == oc[j], f"query {b}: count {g_count[b]} vs oracle {oc[j]}"
        bad = np.nonzero(g_ids[b] != oi[j])[0]
        assert bad.size == 0, f"query {b}: first id mismatch at rank {bad[0]}: gpu {g_ids[b][bad[0]]} vs {oi[j][bad[0]]}"
        assert np.array_equal(g_scores[b].view(np.uint32), os_[j].view(np.uint32)), f"query {b}: score bits differ"
    bloom.free()


@pytest.mark.parametrize("path", [0, 1, 2])
@pytest.mark.parametrize("n,d,B,n_c,n_p,K", [(3000, 64, 9, 7, 3, 20), (70_001, 128, 33, 300, 40, 100),
                                             (20_000, 64, 12, 50, 50, 30), (50_000, 128, 20, 2000, 1, 64),
                                             (40_000, 32, 5, 3, 8, 50), (30_000, 64, 6, 1500, 600, 40),
                                             (20_000, 64, 4, 50, 20, 3000), (90_000, 48, 7, 512, 512, 10),
                                             (200_000, 64, 5, 5000, 40, 50), (100_000, 32, 3, 4096, 700, 30),
                                             (70_000, 16, 2, 65536, 100, 20)])
def test_probing_search_matches_oracle(n, d, B, n_c, n_p, K, path):
    # path 0: up to 512 probes run per query over the probed ranges; more probes, and the forced
    # scorers (1, 2), take the route through per-query mask rows and the fused scan.  From 4096
    # clusters on the centroid scoring is split over several workgroups per query.
    w = ragged_workload(500 + n, n, d, B, 24, 6, 128, 3)
    programs = random_programs(n + B + 1, B, 24, depth=3)
    check_ivf(w, programs, n_c, n_p, K, path=path, label=f"ragged n={n}")


def test_probing_search_mid_recipe_scaled_and_full():
    for n, step in ((200_000, 4), (1_000_000, 9)):
        cfg = S.scaled(S.CONFIGS["mid"], n)
        w = S.make_workload(cfg)
        ops, ids, off, pool = S.gen_filter_programs(cfg)
        programs = [(ops[off[b]:off[b + 1]].tolist(), ids[off[b]:off[b + 1]].tolist()) for b in range(cfg.batch)]
        check_ivf(w, programs, 1024, 64, cfg.top_k, queries=range(0, cfg.batch, step), label=f"mid@{n}",
                  fast_path_only=True)


def test_probing_search_with_multitask_queries_returns_task_specific_lists():
    # Sec. 5.2: the task embeddings of a request are batched against the one index and every task
    # gets its own list; here each of the T = 4 embeddings of a query probes its own clusters with
    # the query's filter program (the multi-task recipe flattened to B * T single-task queries)
    cfg = S.scaled(S.CONFIGS["multi"], 150_000, batch=12)
    w = S.make_workload(cfg)
    ops, ids, off, _ = S.gen_filter_programs(cfg)
    w2, (f_ops, f_ids, f_off) = S.flatten_tasks(w, (ops, ids, off))
    assert w2.cfg.batch == 48 and w2.queries.shape == (48, cfg.d)
    programs = [(f_ops[f_off[b]:f_off[b + 1]].tolist(), f_ids[f_off[b]:f_off[b + 1]].tolist()) for b in range(48)]
    assert programs[0] == programs[3] and programs[4] == programs[7]  # the tasks of a query share its filter
    check_ivf(w2, programs, 256, 16, cfg.top_k, label="multi recipe, task-specific lists", fast_path_only=True)


def test_probing_search_on_an_empty_corpus_and_with_empty_clusters_only():
    B, d, K, n_c = 3, 32, 5, 4
    q = torch.zeros((B, d), dtype=torch.int8, device="cuda")
    qs = torch.ones(B, dtype=torch.float32, device="cuda")
    cent = torch.ones((n_c, d), dtype=torch.int8, device="cuda")
    cs = torch.ones(n_c, dtype=torch.float32, device="cuda")
    ops, ids, off = pack([([], [])] * B)
    # no items at all
    bloom = st.st_bloom_build(np.zeros(1, np.int64), np.zeros(0, np.uint64), 0, 64, 2)
    items = torch.zeros((0, d), dtype=torch.int8, device="cuda")
    iscale = torch.zeros(0, dtype=torch.float32, device="cuda")
    coff = torch.zeros(n_c + 1, dtype=torch.int64, device="cuda")
    g_ids, g_scores, g_count, g_probes = st.st_search_ivf(bloom, items, iscale, cent, cs, coff, 2, q, qs, ops, ids, off, K)
    torch.cuda.synchronize()
    assert (_np(g_count) == 0).all() and (_np(g_ids) == -1).all() and np.isneginf(_np(g_scores)).all()
    assert _np(g_probes).tolist() == [[0, 1]] * B  # equal scores: lower cluster ids first
    bloom.free()
    # items exist, but the probed clusters (ids 0 and 1) are empty
    n = 100
    bloom = st.st_bloom_build(np.arange(n + 1, dtype=np.int64), np.zeros(n, np.uint64), n, 64, 2)
    items = torch.ones((n, d), dtype=torch.int8, device="cuda")
    iscale = torch.ones(n, dtype=torch.float32, device="cuda")
    coff = torch.tensor([0, 0, 0, 50, 100], dtype=torch.int64, device="cuda")
    g_ids, g_scores, g_count, g_probes = st.st_search_ivf(bloom, items, iscale, cent, cs, coff, 2, q, qs, ops, ids, off, K)
    torch.cuda.synchronize()
    assert (_np(g_count) == 0).all() and (_np(g_ids) == -1).all()
    bloom.free()
