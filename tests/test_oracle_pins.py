"""Pins for the CPU oracle: each test ties one part of it to something other than itself --
published hash outputs, brute force on raw id sets, closed forms, numpy library routines,
exact rational arithmetic -- so that a dropped term, wrong sign, wrong index or transposed
operand anywhere in oracle/st_oracle.c fails at least one of them."""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import st_oracle as O
from paper_2511_14881_amd import synth as S
from tests.helpers import f32_fma, f32_mul, read_golden, round_f32, topk_reference

GAMMA = 0x9E3779B97F4A7C15
M64 = (1 << 64) - 1


# ---------------------------------------------------------------- hash
def test_splitmix64_published_vectors():
    rows = read_golden("splitmix64_vectors.txt")
    assert len(rows) == 8
    for seed, idx, val in rows:
        x = (int(seed) + int(idx) * GAMMA) & M64
        assert O.splitmix64(x) == int(val, 0)


def _py_splitmix64(x):
    z = (x + GAMMA) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


@pytest.mark.parametrize("m", [1, 7, 64, 100, 256, 768, 1 << 20])
def test_bit_index_is_hash_of_xor_mod_m(m):
    rng = np.random.default_rng(1)
    for f in [0, 1, 2, 3, M64, 1 << 63] + [int(v) for v in rng.integers(0, 1 << 62, 20)]:
        for j in range(5):
            assert O.bit_index(f, j, m) == _py_splitmix64(f ^ j) % m


# ---------------------------------------------------------------- signatures
@pytest.mark.parametrize("m,k", [(64, 2), (100, 3), (256, 3), (768, 5), (512, 4)])
def test_signature_bits(m, k):
    rng = np.random.default_rng(m * 31 + k)
    ids = rng.integers(0, 1 << 40, 9).astype(np.uint64)
    sig = O.signature(ids, m, k)
    assert sig.size == (m + 63) // 64
    want = set(_py_splitmix64(int(f) ^ j) % m for f in ids for j in range(k))
    got = {w * 64 + b for w in range(sig.size) for b in range(64) if (int(sig[w]) >> b) & 1}
    assert got == want
    assert len(got) <= k * ids.size
    # duplicates are harmless, the empty list gives the zero signature, order does not matter
    assert np.array_equal(O.signature(np.concatenate([ids, ids[::-1]]), m, k), sig)
    assert not O.signature(np.zeros(0, np.uint64), m, k).any()


def test_sibling_ids_share_bits_for_k2():
    # consequence of hashing f XOR j: for k = 2, ids 2a and 2a+1 have identical bit sets
    for a in [0, 5, 12345]:
        assert np.array_equal(O.signature([2 * a], 256, 2), O.signature([2 * a + 1], 256, 2))
    assert not np.array_equal(O.signature([2], 256, 2), O.signature([4], 256, 2))


def _ragged_corpus(rng, n_items, vocab, max_feats):
    lens = rng.integers(0, max_feats + 1, n_items)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ids = rng.integers(0, vocab, int(off[-1])).astype(np.uint64)
    return off, ids


def test_bloom_build_is_per_item_signature():
    rng = np.random.default_rng(3)
    off, ids = _ragged_corpus(rng, 300, 50, 6)
    sigs = O.bloom_build(off, ids, 100, 3)
    for i in [0, 1, 17, 299]:
        assert np.array_equal(sigs[i], O.signature(ids[off[i]:off[i + 1]], 100, 3))


# ---------------------------------------------------------------- Bloom test vs exact sets
def _py_exact(off, ids, filt):
    n = off.size - 1
    return np.array([set(int(x) for x in filt) <= set(int(x) for x in ids[off[i]:off[i + 1]])
                     for i in range(n)])


@pytest.mark.parametrize("m,k", [(64, 2), (256, 3), (100, 4)])
def test_no_false_negatives_and_exact_mask(m, k):
    rng = np.random.default_rng(m + k)
    off, ids = _ragged_corpus(rng, 1000, 14, 8)
    sigs = O.bloom_build(off, ids, m, k)
    for filt in ([3], [3, 7], [1, 2, 3], [13, 0]):
        ex = O.mask_to_bool(O.exact_mask(off, ids, filt), 1000)
        assert np.array_equal(ex, _py_exact(off, ids, filt))
        bl = O.mask_to_bool(O.bloom_mask(sigs, m, k, filt), 1000)
        assert ex.sum() > 0
        assert not (ex & ~bl).any(), "Bloom test dropped an item that holds every filter id"


def test_huge_filter_equals_exact_set_match():
    rng = np.random.default_rng(11)
    # ids spaced by 16 so that no two distinct ids are XOR-neighbours
    off, ids = _ragged_corpus(rng, 600, 30, 5)
    ids = ids * np.uint64(16)
    m, k = 1 << 20, 3
    sigs = O.bloom_build(off, ids, m, k)
    for filt in ([16], [32, 48], [0, 16, 64]):
        ex = O.exact_mask(off, ids, filt)
        assert np.array_equal(O.bloom_mask(sigs, m, k, filt), ex)


def test_empty_filter_passes_everything_and_tail_bits_are_zero():
    rng = np.random.default_rng(5)
    for n in (1, 63, 64, 65, 130):
        off, ids = _ragged_corpus(rng, n, 10, 3)
        mask = O.bloom_mask(O.bloom_build(off, ids, 64, 2), 64, 2, [])
        assert mask.size == (n + 63) // 64
        assert O.mask_to_bool(mask, n).all()
        total = sum(bin(int(w)).count("1") for w in mask)
        assert total == n


@pytest.mark.parametrize("m,k,n_feat,n_items,n_queries", [
    (64, 2, 4, 2_000, 1_000),     # Tiny's filter: closed form 1.381e-2
    (256, 3, 8, 4_000, 1_500),    # Mid's: 7.17e-4
    (512, 4, 16, 6_000, 2_500),   # Large's: 1.91e-4
])
def test_false_positive_rate_near_closed_form(m, k, n_feat, n_items, n_queries):
    """Single-term queries on ids no item holds, ids spaced by 16 so that none are XOR-neighbours:
    the empirical pass rate must sit within 10% of (1-e^{-kn/m})^k."""
    rng = np.random.default_rng(m)
    vocab = 1 << 30
    ids = (rng.choice(vocab, size=(n_items, n_feat), replace=True).astype(np.uint64) * np.uint64(16))
    off = np.arange(0, n_items * n_feat + 1, n_feat, dtype=np.int64)
    sigs = O.bloom_build(off, ids.reshape(-1), m, k)
    set_bits = np.unpackbits(sigs.view(np.uint8), axis=1).sum(axis=1)
    p = float(set_bits.mean()) / m
    assert p == pytest.approx(1.0 - math.exp(-k * n_feat / m), rel=0.02)
    hits = {True: 0, False: 0}
    count = {True: 0, False: 0}
    for qi in range(n_queries):
        f = (vocab + 1 + qi) * 16  # never present in any item
        distinct = len({_py_splitmix64(f ^ j) % m for j in range(k)}) == k
        hits[distinct] += int(O.mask_to_bool(O.bloom_mask(sigs, m, k, [np.uint64(f)]), n_items).sum())
        count[distinct] += 1
    closed = (1.0 - math.exp(-k * n_feat / m)) ** k
    # The textbook derivation treats the k probes as independent draws (collisions among a
    # query's own hashes included), so it is the rate over ALL queries that it predicts.
    overall = (hits[True] + hits[False]) / (n_items * n_queries)
    assert abs(overall - closed) <= 0.10 * closed, (overall, closed)
    # queries probing k distinct bits pass a little less often than that, colliding ones far more
    rate_distinct = hits[True] / (n_items * count[True])
    assert 0.80 * closed <= rate_distinct <= overall
    if count[False]:
        assert hits[False] / (n_items * count[False]) > 3 * closed


def test_paper_layout_arithmetic():
    for row in read_golden("paper_arithmetic.txt"):
        if row[0] == "words":
            n, words = int(row[1]), int(row[2])
            assert (n + 63) // 64 == words
        elif row[0] == "bytes":
            n, m, nbytes = int(row[1]), int(row[2]), float(row[3])
            assert n * O.sig_words(m) * 8 == pytest.approx(nbytes, rel=1e-12)
        elif row[0] == "heuristic":
            a, b, c, d = map(int, row[1:])
            assert a * b * c == d
    # the oracle's item-major index has exactly that size
    sigs = O.bloom_build(np.arange(0, 129, dtype=np.int64), np.arange(128, dtype=np.uint64), 768, 5)
    assert sigs.nbytes == 128 * 768 // 8


# ---------------------------------------------------------------- dot products and rescale
def test_dot_against_wide_integers():
    rng = np.random.default_rng(7)
    for d in (16, 64, 128, 256):
        q = rng.integers(-128, 128, d).astype(np.int8)
        e = rng.integers(-128, 128, d).astype(np.int8)
        assert O.dot(q, e) == int(q.astype(np.int64) @ e.astype(np.int64))
    q = np.full(256, -128, np.int8)
    assert O.dot(q, q) == 256 * 128 * 128
    assert O.dot(q, np.full(256, 127, np.int8)) == -256 * 128 * 127
    # not symmetric data: a transposed / swapped operand would still pass, a wrong index would not
    a = np.arange(-8, 8, dtype=np.int8)
    b = np.array([1] + [0] * 15, dtype=np.int8)
    assert O.dot(a, b) == -8


def test_rescale_is_two_rounded_multiplies_left_to_right():
    rng = np.random.default_rng(9)
    found_order_sensitive = 0
    for _ in range(4000):
        d = int(rng.integers(-4_000_000, 4_000_000))
        sq = np.float32(rng.uniform(0.5, 1.5))
        si = np.float32(rng.uniform(0.5, 1.5))
        left = f32_mul(f32_mul(np.float32(d), sq), si)
        right = f32_mul(np.float32(d), f32_mul(sq, si))
        once = round_f32(Fraction(d) * Fraction(float(sq)) * Fraction(float(si)))
        got = O.rescale(d, sq, si)
        assert got == left
        found_order_sensitive += int(left != right) + int(left != once)
    assert found_order_sensitive > 100  # the sample really distinguishes the orders


# ---------------------------------------------------------------- search
def _small_workload(seed, n=700, d=32, B=5, vocab=12, max_feats=4):
    rng = np.random.default_rng(seed)
    off, ids = _ragged_corpus(rng, n, vocab, max_feats)
    items = rng.integers(-127, 128, (n, d)).astype(np.int8)
    iscale = rng.uniform(0.5, 1.5, n).astype(np.float32)
    q = rng.integers(-127, 128, (B, d)).astype(np.int8)
    qs = rng.uniform(0.5, 1.5, B).astype(np.float32)
    return off, ids, items, iscale, q, qs


def test_unfiltered_unit_scale_search_is_matmul_plus_stable_argsort():
    off, ids, items, _, q, _ = _small_workload(21)
    n, B, K = items.shape[0], q.shape[0], 50
    sigs = O.bloom_build(off, ids, 64, 2)
    ones_i = np.ones(n, np.float32)
    ones_q = np.ones(B, np.float32)
    got_i, got_s, got_c = O.search(sigs, 64, 2, items, ones_i, q, ones_q, [], np.zeros(B + 1, np.int64), K)
    dots = q.astype(np.int32) @ items.astype(np.int32).T
    for b in range(B):
        order = np.argsort(-dots[b], kind="stable")[:K]
        assert np.array_equal(got_i[b], order)
        assert np.array_equal(got_s[b], dots[b][order].astype(np.float32))
        assert got_c[b] == K


@pytest.mark.parametrize("m,k", [(64, 2), (1 << 20, 3)])
def test_filtered_search_equals_score_everything_then_mask(m, k):
    # order independence of the two predicates (paper Sec. 4.3): mask-then-score == score-then-mask
    off, ids, items, iscale, q, qs = _small_workload(22)
    n, B, K = items.shape[0], q.shape[0], 40
    filters = [[1], [2, 3], [], [5, 1], [11]]
    if m == 1 << 20:  # space the ids so that XOR-neighbours cannot alias: Bloom == exact set
        ids = ids * np.uint64(16)
        filters = [[16 * x for x in f] for f in filters]
    sigs = O.bloom_build(off, ids, m, k)
    fid = np.array([x for f in filters for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filters])]).astype(np.int64)
    got_i, got_s, got_c = O.search(sigs, m, k, items, iscale, q, qs, fid, foff, K)
    dots = q.astype(np.int32) @ items.astype(np.int32).T
    for b in range(B):
        all_scores = (dots[b].astype(np.float32) * qs[b]) * iscale  # numpy fp32, left to right
        passing = O.mask_to_bool(O.bloom_mask(sigs, m, k, filters[b]), n)
        if m == 1 << 20:
            passing_exact = _py_exact(off, ids, filters[b])
            assert np.array_equal(passing, passing_exact)
        wi, ws, wc = topk_reference(all_scores, passing, K)
        assert np.array_equal(got_i[b], wi)
        assert np.array_equal(got_s[b], ws)
        assert got_c[b] == min(K, wc)


def test_ties_break_to_lower_id():
    off, ids, items, iscale, q, qs = _small_workload(23, n=200)
    sigs = O.bloom_build(off, ids, 64, 2)
    zero_q = np.zeros_like(q)
    gi, gs, gc = O.search(sigs, 64, 2, items, iscale, zero_q, qs, [], np.zeros(q.shape[0] + 1, np.int64), 17)
    assert np.array_equal(gi, np.tile(np.arange(17), (q.shape[0], 1)))
    assert (gs == 0).all() and not np.signbit(gs).any()
    # duplicated rows with equal scales: the copies tie and must come out in id order
    items2 = np.concatenate([items[:50], items[:50], items[:50]])
    sc2 = np.concatenate([iscale[:50]] * 3)
    off2 = np.zeros(151, np.int64)
    sigs2 = O.bloom_build(off2, np.zeros(0, np.uint64), 64, 2)
    gi, gs, _ = O.search(sigs2, 64, 2, items2, sc2, q[:1], qs[:1], [], np.zeros(2, np.int64), 150)
    trip = gi[0].reshape(50, 3)
    assert (trip[:, 1] == trip[:, 0] + 50).all() and (trip[:, 2] == trip[:, 0] + 100).all()
    assert (np.diff(gs[0]) <= 0).all()


def test_short_and_empty_results_are_padded():
    off, ids, items, iscale, q, qs = _small_workload(24, n=100, vocab=8)
    ids = ids * np.uint64(16)
    sigs = O.bloom_build(off, ids, 1 << 16, 2)
    B = q.shape[0]
    absent = [999_999 * 16]
    some = [48]
    filters = [absent, some, [], absent, some]
    fid = np.array([x for f in filters for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filters])]).astype(np.int64)
    K = 150  # above the corpus size
    gi, gs, gc = O.search(sigs, 1 << 16, 2, items, iscale, q, qs, fid, foff, K)
    n_some = int(_py_exact(off, ids, some).sum())
    assert list(gc) == [0, n_some, 100, 0, n_some]
    for b in range(B):
        assert (gi[b, gc[b]:] == -1).all() and np.isneginf(gs[b, gc[b]:]).all()
        assert (gi[b, :gc[b]] >= 0).all()
    # K = 1 returns the arg-max
    gi1, gs1, _ = O.search(sigs, 1 << 16, 2, items, iscale, q, qs, fid, foff, 1)
    assert np.array_equal(gi1[:, 0], gi[:, 0]) and np.array_equal(gs1[:, 0], gs[:, 0])


# ---------------------------------------------------------------- multi-task aggregation
def test_single_task_weight_one_reduces_to_plain_search():
    off, ids, items, iscale, q, qs = _small_workload(25)
    sigs = O.bloom_build(off, ids, 64, 2)
    B = q.shape[0]
    foff = np.arange(B + 1, dtype=np.int64)
    fid = np.array([1, 2, 3, 4, 5], dtype=np.uint64)
    a = O.search(sigs, 64, 2, items, iscale, q, qs, fid, foff, 30)
    b = O.search(sigs, 64, 2, items, iscale, q[:, None, :], qs[:, None], fid, foff, 30,
                 task_weight=np.ones(1, np.float32))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_aggregation_is_fma_chain_in_task_order():
    rng = np.random.default_rng(26)
    n, d, B, T, K = 60, 16, 3, 4, 60
    items = rng.integers(-127, 128, (n, d)).astype(np.int8)
    iscale = rng.uniform(0.5, 1.5, n).astype(np.float32)
    q = rng.integers(-127, 128, (B, T, d)).astype(np.int8)
    qs = rng.uniform(0.5, 1.5, (B, T)).astype(np.float32)
    w = rng.uniform(0, 1, T).astype(np.float32)
    sigs = O.bloom_build(np.zeros(n + 1, np.int64), np.zeros(0, np.uint64), 64, 2)
    gi, gs, gc = O.search(sigs, 64, 2, items, iscale, q, qs, [], np.zeros(B + 1, np.int64), K,
                          task_weight=w)
    differs_from_unfused = 0
    for b in range(B):
        agg = np.zeros(n, np.float32)
        unfused = np.zeros(n, np.float32)
        dbl = np.zeros(n, np.float64)
        for i in range(n):
            a = np.float32(0.0)
            u = np.float32(0.0)
            for t in range(T):
                dot = int(q[b, t].astype(np.int64) @ items[i].astype(np.int64))
                st = f32_mul(f32_mul(np.float32(dot), qs[b, t]), iscale[i])
                a = f32_fma(w[t], st, a)
                u = np.float32(u + f32_mul(w[t], st))
                dbl[i] += float(w[t]) * float(dot) * float(qs[b, t]) * float(iscale[i])
            agg[i], unfused[i] = a, u
        differs_from_unfused += int((agg != unfused).sum())
        wi, ws, _ = topk_reference(agg, np.ones(n, bool), K)
        assert np.array_equal(gi[b], wi)
        assert np.array_equal(gs[b], ws)
        # and within 1e-6 relative of the double-precision value of the same sum
        got = np.empty(n)
        got[gi[b]] = gs[b]
        assert np.allclose(got, dbl, rtol=1e-6, atol=1e-6 * np.abs(dbl).max())
    assert differs_from_unfused > 0  # the chain is really fused, not mul-then-add


# ---------------------------------------------------------------- the workloads themselves
def test_tiny_config_end_to_end_against_numpy():
    w = S.make_workload(S.CONFIGS["tiny"])
    cfg = w.cfg
    off, ids = w.feat_offsets.numpy(), w.feat_ids.numpy().astype(np.uint64)
    items, iscale = w.items.numpy(), w.item_scale.numpy()
    sigs = O.bloom_build(off, ids, cfg.m_bits, cfg.k_hashes)
    gi, gs, gc = O.search(sigs, cfg.m_bits, cfg.k_hashes, items, iscale, w.queries.numpy(),
                          w.query_scale.numpy(), w.filt_ids, w.filt_offsets, cfg.top_k)
    passing = O.mask_to_bool(O.bloom_mask(sigs, cfg.m_bits, cfg.k_hashes, w.filt_ids), cfg.n_items)
    exact = _py_exact(off, ids, w.filt_ids)
    assert not (exact & ~passing).any()
    # about 0.4% true matches plus about 1.4% false positives (and the sibling id's items)
    assert 0.008 < passing.mean() < 0.04
    dots = w.queries.numpy().astype(np.int32) @ items.astype(np.int32).T
    scores = (dots[0].astype(np.float32) * w.query_scale.numpy()[0]) * iscale
    wi, ws, _ = topk_reference(scores, passing, cfg.top_k)
    assert np.array_equal(gi[0], wi) and np.array_equal(gs[0], ws) and gc[0] == cfg.top_k
