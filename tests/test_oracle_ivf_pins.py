"""Pins of the oracle's cluster probing (paper Sec. 4.2 and Alg. 1 phases 1-4) against things other
than itself: numpy argsort of centroid scores with hand-built range masks, the plain search when
every cluster is probed, order independence of probing and filtering, and the paper's
probed-fraction arithmetic.  CPU only."""
import numpy as np
import pytest

from oracle import st_oracle as O
from tests.helpers import topk_reference
from tests.test_oracle_expr_pins import eval_tree, postfix, ragged_corpus

LEAF, AND, OR, NOT = O.LEAF, O.AND, O.OR, O.NOT


def workload(seed, n=900, d=32, B=6, n_c=12, vocab=12, max_feats=4, empty_clusters=True):
    rng = np.random.default_rng(seed)
    off, ids = ragged_corpus(rng, n, vocab, max_feats)
    items = rng.integers(-127, 128, (n, d)).astype(np.int8)
    iscale = rng.uniform(0.5, 1.5, n).astype(np.float32)
    q = rng.integers(-127, 128, (B, d)).astype(np.int8)
    qs = rng.uniform(0.5, 1.5, B).astype(np.float32)
    cent = rng.integers(-127, 128, (n_c, d)).astype(np.int8)
    cs = rng.uniform(0.5, 1.5, n_c).astype(np.float32)
    cuts = np.sort(rng.integers(0, n + 1, n_c - 1))
    if empty_clusters and n_c > 3:
        cuts[1] = cuts[0]  # an empty cluster
    coff = np.concatenate([[0], cuts, [n]]).astype(np.int64)
    return rng, off, ids, items, iscale, q, qs, cent, cs, coff


def pack(programs):
    ops = np.array([o for p in programs for o in p[0]], dtype=np.int32)
    pid = np.array([i for p in programs for i in p[1]], dtype=np.uint64)
    offs = np.concatenate([[0], np.cumsum([len(p[0]) for p in programs])]).astype(np.int64)
    return ops, pid, offs


TREES = [("leaf", 1), ("or", ("leaf", 2), ("leaf", 3)), None, ("and", ("leaf", 5), ("not", ("leaf", 1))),
         ("and", ("or", ("leaf", 0), ("leaf", 7)), ("leaf", 4)), ("not", ("leaf", 2))]


@pytest.mark.parametrize("n_probe", [1, 3, 12, 20])
def test_probing_is_argsort_of_centroid_scores_then_masked_search(n_probe):
    rng, off, ids, items, iscale, q, qs, cent, cs, coff = workload(41)
    n, B, K, n_c = items.shape[0], q.shape[0], 30, cent.shape[0]
    m, k = 128, 3
    sigs = O.bloom_build(off, ids, m, k)
    programs = [([], []) if t is None else postfix(t) for t in TREES]
    ops, pid, offs = pack(programs)
    gi, gs, gc, gp = O.search_ivf(sigs, m, k, items, iscale, cent, cs, coff, n_probe, q, qs, ops, pid, offs, K)
    leaf = lambda f: O.mask_to_bool(O.bloom_mask(sigs, m, k, [f]), n)
    cdots = q.astype(np.int32) @ cent.astype(np.int32).T
    dots = q.astype(np.int32) @ items.astype(np.int32).T
    for b in range(B):
        cscore = (cdots[b].astype(np.float32) * qs[b]) * cs
        order = np.lexsort((np.arange(n_c), -cscore.astype(np.float64)))[: min(n_probe, n_c)]
        assert gp[b][: order.size].tolist() == order.tolist()
        assert (gp[b][order.size:] == -1).all()
        in_probe = np.zeros(n, bool)
        for c in order:
            in_probe[coff[c]:coff[c + 1]] = True
        passing = np.ones(n, bool) if TREES[b] is None else eval_tree(TREES[b], leaf)
        scores = (dots[b].astype(np.float32) * qs[b]) * iscale
        # filter-then-probe and probe-then-filter are one conjunction (Sec. 4.3)
        wi, ws, wc = topk_reference(scores, passing & in_probe, K)
        assert np.array_equal(gi[b], wi)
        assert np.array_equal(gs[b], ws)
        assert gc[b] == min(K, wc)


def test_probing_every_cluster_is_the_brute_force_search():
    _, off, ids, items, iscale, q, qs, cent, cs, coff = workload(42)
    m, k, K = 64, 2, 25
    sigs = O.bloom_build(off, ids, m, k)
    programs = [([], []) if t is None else postfix(t) for t in TREES]
    ops, pid, offs = pack(programs)
    a = O.search_ivf(sigs, m, k, items, iscale, cent, cs, coff, cent.shape[0], q, qs, ops, pid, offs, K)
    b = O.search_expr(sigs, m, k, items, iscale, q, qs, ops, pid, offs, K)
    for x, y in zip(a[:3], b):
        assert np.array_equal(x, y)
    # more probes than clusters changes nothing
    c = O.search_ivf(sigs, m, k, items, iscale, cent, cs, coff, cent.shape[0] + 5, q, qs, ops, pid, offs, K)
    for x, y in zip(c[:3], b):
        assert np.array_equal(x, y)


def test_centroid_ties_go_to_the_lower_cluster_id():
    _, off, ids, items, iscale, q, qs, cent, cs, coff = workload(43, n_c=8, empty_clusters=False)
    cent[5] = cent[2]
    cs[5] = cs[2]
    cent[7] = cent[2]
    cs[7] = cs[2]
    q[0] = cent[2]  # cluster 2 (and its copies) is the best match of query 0
    sigs = O.bloom_build(off, ids, 64, 2)
    ops, pid, offs = pack([([], [])] * q.shape[0])
    _, _, _, probes = O.search_ivf(sigs, 64, 2, items, iscale, cent, cs, coff, 3, q, qs, ops, pid, offs, 5)
    assert probes[0].tolist() == [2, 5, 7]


def test_probed_fraction_arithmetic_of_the_paper():
    # Sec. 4.3: 81 million items in 9,000 clusters, 256 probes -> about 2.3 million items, 2.8 %
    assert round(81_000_000 / 9_000 * 256) == 2_304_000
    assert abs(256 / 9_000 - 0.028) < 0.001
    # the same ratio on equal clusters through the oracle: items returned with K = N are the probed ones
    n, n_c, n_p, d = 900, 90, 7, 16
    rng = np.random.default_rng(44)
    items = rng.integers(-127, 128, (n, d)).astype(np.int8)
    cent = rng.integers(-127, 128, (n_c, d)).astype(np.int8)
    q = rng.integers(-127, 128, (3, d)).astype(np.int8)
    ones = lambda x: np.ones(x, np.float32)
    coff = np.arange(0, n + 1, n // n_c).astype(np.int64)
    sigs = O.bloom_build(np.zeros(n + 1, np.int64), np.zeros(0, np.uint64), 64, 2)
    ops, pid, offs = pack([([], [])] * 3)
    ids, _, count, probes = O.search_ivf(sigs, 64, 2, items, ones(n), cent, ones(n_c), coff, n_p, q, ones(3),
                                         ops, pid, offs, n)
    assert (count == n_p * (n // n_c)).all()
    for b in range(3):
        got = np.sort(ids[b][: count[b]])
        want = np.sort(np.concatenate([np.arange(coff[c], coff[c + 1]) for c in probes[b]]))
        assert np.array_equal(got, want)


def test_ill_formed_program_is_rejected():
    _, off, ids, items, iscale, q, qs, cent, cs, coff = workload(45)
    sigs = O.bloom_build(off, ids, 64, 2)
    ops, pid, offs = pack([([LEAF, LEAF], [1, 2])] * q.shape[0])
    with pytest.raises(ValueError):
        O.search_ivf(sigs, 64, 2, items, iscale, cent, cs, coff, 3, q, qs, ops, pid, offs, 5)
