"""Pins of the oracle's boolean filter expressions (paper Sec. 4 query form, Sec. 4.3 operation
array and stack) against things other than itself: a recursive evaluation of the expression
tree on per-feature masks, raw id sets of a hand-written corpus, algebraic laws, and the already
pinned conjunction filter.  CPU only."""
import numpy as np
import pytest

from oracle import st_oracle as O
from tests.helpers import topk_reference

LEAF, AND, OR, NOT = O.LEAF, O.AND, O.OR, O.NOT


# ---------------------------------------------------------------- expression trees (test side)
# A tree is ("leaf", id) | ("not", t) | ("and", a, b) | ("or", a, b).
def postfix(tree):
    """Operation array of a tree: operands first, operator last."""
    kind = tree[0]
    if kind == "leaf":
        return [LEAF], [tree[1]]
    if kind == "not":
        ops, ids = postfix(tree[1])
        return ops + [NOT], ids + [0]
    lo, li = postfix(tree[1])
    ro, ri = postfix(tree[2])
    return lo + ro + [AND if kind == "and" else OR], li + ri + [0]


def eval_tree(tree, leaf_value):
    """Recursive evaluation; leaf_value(id) -> bool array over the items."""
    kind = tree[0]
    if kind == "leaf":
        return leaf_value(tree[1])
    if kind == "not":
        return ~eval_tree(tree[1], leaf_value)
    a, b = eval_tree(tree[1], leaf_value), eval_tree(tree[2], leaf_value)
    return (a & b) if kind == "and" else (a | b)


def random_tree(rng, vocab, depth):
    r = rng.random()
    if depth == 0 or r < 0.25:
        return ("leaf", int(rng.integers(0, vocab)))
    if r < 0.45:
        return ("not", random_tree(rng, vocab, depth - 1))
    return ("and" if r < 0.72 else "or", random_tree(rng, vocab, depth - 1), random_tree(rng, vocab, depth - 1))


def ragged_corpus(rng, n_items, vocab, max_feats):
    lens = rng.integers(0, max_feats + 1, n_items)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    ids = rng.integers(0, vocab, int(off[-1])).astype(np.uint64)
    return off, ids


def has_feature(off, ids, f):
    return np.array([f in set(int(x) for x in ids[off[i]:off[i + 1]]) for i in range(off.size - 1)])


# ---------------------------------------------------------------- well-formedness
def test_program_depth_and_ill_formed_programs():
    assert O.expr_depth([]) == 0
    assert O.expr_depth([LEAF]) == 1
    assert O.expr_depth([LEAF, LEAF, AND]) == 2
    assert O.expr_depth([LEAF, LEAF, LEAF, OR, AND]) == 3
    assert O.expr_depth([LEAF, NOT, NOT]) == 1
    for bad in ([AND], [NOT], [LEAF, AND], [LEAF, LEAF], [LEAF, LEAF, AND, OR], [7], [LEAF, -1]):
        assert O.expr_depth(bad) == -1, bad
    sigs = O.bloom_build([0, 1], [3], 64, 2)
    with pytest.raises(ValueError):
        O.expr_mask(sigs, 64, 2, [LEAF, LEAF], [1, 2])


# ---------------------------------------------------------------- the paper's example, by hand
def test_country_and_language_example_on_a_hand_written_corpus():
    # Query of the form  country = US AND (lang = EN OR lang = ES)  [Sec. 4, concrete example].
    # Feature ids spaced by 16 and a signature far wider than the corpus needs: no two ids share a
    # hash bit here (checked below), so the Bloom result must equal the set semantics.
    US, CA, EN, ES, FR = 16, 32, 48, 64, 80
    corpus = [
        [US, EN],      # 0 pass
        [US, ES],      # 1 pass
        [US, FR],      # 2 wrong language
        [CA, EN],      # 3 wrong country
        [US],          # 4 no language
        [EN, ES],      # 5 no country
        [US, EN, ES],  # 6 pass (both languages)
        [],            # 7 nothing
        [CA, FR],      # 8
        [US, FR, ES],  # 9 pass
    ]
    expected = [True, True, False, False, False, False, True, False, False, True]
    off = np.concatenate([[0], np.cumsum([len(c) for c in corpus])]).astype(np.int64)
    ids = np.array([x for c in corpus for x in c], dtype=np.uint64)
    m, k = 4096, 3
    bits = [O.bit_index(f, j, m) for f in (US, CA, EN, ES, FR) for j in range(k)]
    assert len(set(bits)) == len(bits)
    sigs = O.bloom_build(off, ids, m, k)
    # operands first: US EN ES OR AND
    ops, pid = [LEAF, LEAF, LEAF, OR, AND], [US, EN, ES, 0, 0]
    got = O.mask_to_bool(O.expr_mask(sigs, m, k, ops, pid), len(corpus))
    assert got.tolist() == expected
    # the other operand order (EN ES OR US AND) is the same predicate
    got2 = O.mask_to_bool(O.expr_mask(sigs, m, k, [LEAF, LEAF, OR, LEAF, AND], [EN, ES, 0, US, 0]), len(corpus))
    assert got2.tolist() == expected
    # NOT: country = US AND NOT lang = FR
    got3 = O.mask_to_bool(O.expr_mask(sigs, m, k, [LEAF, LEAF, NOT, AND], [US, FR, 0, 0]), len(corpus))
    assert got3.tolist() == [True, True, False, False, True, False, True, False, False, False]


# ---------------------------------------------------------------- stack machine vs tree recursion
@pytest.mark.parametrize("m,k,seed", [(64, 2, 1), (100, 3, 2), (256, 4, 3)])
def test_operation_array_equals_recursive_tree_evaluation(m, k, seed):
    rng = np.random.default_rng(seed)
    n = 777  # ragged last word
    off, ids = ragged_corpus(rng, n, 16, 6)
    sigs = O.bloom_build(off, ids, m, k)
    # a leaf is the (pinned) Bloom test of a one-id filter
    leaf = lambda f: O.mask_to_bool(O.bloom_mask(sigs, m, k, [f]), n)
    seen_not = seen_deep = False
    for _ in range(60):
        tree = random_tree(rng, 16, 4)
        ops, pid = postfix(tree)
        want = eval_tree(tree, leaf)
        mask = O.expr_mask(sigs, m, k, ops, pid)
        assert np.array_equal(O.mask_to_bool(mask, n), want), tree
        # nothing past the last item, also under NOT
        assert sum(bin(int(w)).count("1") for w in mask) == int(want.sum())
        seen_not |= NOT in ops
        seen_deep |= O.expr_depth(ops) >= 3
    assert seen_not and seen_deep


def test_operand_order_matters_where_it_should():
    # a AND NOT b differs from b AND NOT a: a mistake in which operand NOT applies to shows here
    rng = np.random.default_rng(9)
    n = 500
    off, ids = ragged_corpus(rng, n, 8, 3)
    m, k = 512, 3
    sigs = O.bloom_build(off, ids, m, k)
    a, b = 2, 5
    la = O.mask_to_bool(O.bloom_mask(sigs, m, k, [a]), n)
    lb = O.mask_to_bool(O.bloom_mask(sigs, m, k, [b]), n)
    assert (la & ~lb).sum() > 0 and (lb & ~la).sum() > 0 and not np.array_equal(la & ~lb, lb & ~la)
    got = O.mask_to_bool(O.expr_mask(sigs, m, k, [LEAF, LEAF, NOT, AND], [a, b, 0, 0]), n)
    assert np.array_equal(got, la & ~lb)
    got = O.mask_to_bool(O.expr_mask(sigs, m, k, [LEAF, NOT, LEAF, AND], [a, 0, b, 0]), n)
    assert np.array_equal(got, ~la & lb)


def test_conjunction_program_is_the_conjunction_filter():
    # AND of one-id leaves sets exactly the bits of the whole id list: Eq. 4 with Q = {a, b, c}
    rng = np.random.default_rng(4)
    n = 900
    off, ids = ragged_corpus(rng, n, 12, 6)
    for m, k in ((64, 2), (256, 3)):
        sigs = O.bloom_build(off, ids, m, k)
        for filt in ([3], [3, 7], [1, 2, 3], [5, 5]):
            ops = [LEAF] + [x for _ in filt[1:] for x in (LEAF, AND)]
            pid = [filt[0]] + [x for f in filt[1:] for x in (f, 0)]
            assert np.array_equal(O.expr_mask(sigs, m, k, ops, pid), O.bloom_mask(sigs, m, k, filt))
        assert np.array_equal(O.expr_mask(sigs, m, k, [], []), O.bloom_mask(sigs, m, k, []))


def test_de_morgan_and_double_negation():
    rng = np.random.default_rng(6)
    n = 640
    off, ids = ragged_corpus(rng, n, 10, 5)
    m, k = 128, 2
    sigs = O.bloom_build(off, ids, m, k)
    a, b = 1, 4
    lhs = O.expr_mask(sigs, m, k, [LEAF, LEAF, OR, NOT], [a, b, 0, 0])
    rhs = O.expr_mask(sigs, m, k, [LEAF, NOT, LEAF, NOT, AND], [a, 0, b, 0, 0])
    assert np.array_equal(lhs, rhs)
    lhs = O.expr_mask(sigs, m, k, [LEAF, LEAF, AND, NOT], [a, b, 0, 0])
    rhs = O.expr_mask(sigs, m, k, [LEAF, NOT, LEAF, NOT, OR], [a, 0, b, 0, 0])
    assert np.array_equal(lhs, rhs)
    assert np.array_equal(O.expr_mask(sigs, m, k, [LEAF, NOT, NOT], [a, 0, 0]), O.expr_mask(sigs, m, k, [LEAF], [a]))


def test_error_direction_against_raw_id_sets():
    # Narrow signatures give false positives at the leaves.  Without NOT the program can only pass
    # too many items (no false negatives); a negated leaf can only pass too few.
    rng = np.random.default_rng(8)
    n = 1500
    off, ids = ragged_corpus(rng, n, 40, 8)
    m, k = 64, 2
    sigs = O.bloom_build(off, ids, m, k)
    exact_leaf = lambda f: has_feature(off, ids, f)
    widened = narrowed = 0
    for _ in range(25):
        # NOT-free tree
        tree = random_tree(rng, 40, 3)
        while NOT in postfix(tree)[0]:
            tree = random_tree(rng, 40, 3)
        ops, pid = postfix(tree)
        bl = O.mask_to_bool(O.expr_mask(sigs, m, k, ops, pid), n)
        ex = eval_tree(tree, exact_leaf)
        assert not (ex & ~bl).any()
        widened += int((bl & ~ex).sum())
        f = int(rng.integers(0, 40))
        bl = O.mask_to_bool(O.expr_mask(sigs, m, k, [LEAF, NOT], [f, 0]), n)
        ex = ~exact_leaf(f)
        assert not (bl & ~ex).any()
        narrowed += int((ex & ~bl).sum())
    assert widened > 0 and narrowed > 0  # the signatures really were narrow enough to err


# ---------------------------------------------------------------- search with programs
def _workload(seed, n=700, d=32, B=6, vocab=12, max_feats=4):
    rng = np.random.default_rng(seed)
    off, ids = ragged_corpus(rng, n, vocab, max_feats)
    items = rng.integers(-127, 128, (n, d)).astype(np.int8)
    iscale = rng.uniform(0.5, 1.5, n).astype(np.float32)
    q = rng.integers(-127, 128, (B, d)).astype(np.int8)
    qs = rng.uniform(0.5, 1.5, B).astype(np.float32)
    return rng, off, ids, items, iscale, q, qs


def _pack(programs):
    ops = np.array([o for p in programs for o in p[0]], dtype=np.int32)
    pid = np.array([i for p in programs for i in p[1]], dtype=np.uint64)
    offs = np.concatenate([[0], np.cumsum([len(p[0]) for p in programs])]).astype(np.int64)
    return ops, pid, offs


def test_search_with_programs_equals_score_everything_then_mask():
    rng, off, ids, items, iscale, q, qs = _workload(31)
    n, B, K = items.shape[0], q.shape[0], 40
    m, k = 128, 3
    sigs = O.bloom_build(off, ids, m, k)
    trees = [("leaf", 1), ("or", ("leaf", 2), ("leaf", 3)), None,
             ("and", ("leaf", 5), ("not", ("leaf", 1))),
             ("and", ("or", ("leaf", 0), ("leaf", 7)), ("or", ("leaf", 4), ("not", ("leaf", 9)))),
             ("not", ("or", ("leaf", 2), ("leaf", 3)))]
    programs = [([], []) if t is None else postfix(t) for t in trees]
    ops, pid, offs = _pack(programs)
    got_i, got_s, got_c = O.search_expr(sigs, m, k, items, iscale, q, qs, ops, pid, offs, K)
    leaf = lambda f: O.mask_to_bool(O.bloom_mask(sigs, m, k, [f]), n)
    dots = q.astype(np.int32) @ items.astype(np.int32).T
    for b in range(B):
        all_scores = (dots[b].astype(np.float32) * qs[b]) * iscale
        passing = np.ones(n, bool) if trees[b] is None else eval_tree(trees[b], leaf)
        wi, ws, wc = topk_reference(all_scores, passing, K)
        assert np.array_equal(got_i[b], wi)
        assert np.array_equal(got_s[b], ws)
        assert got_c[b] == min(K, wc)


def test_search_with_conjunction_programs_is_the_plain_search():
    _, off, ids, items, iscale, q, qs = _workload(32)
    B, K = q.shape[0], 25
    m, k = 64, 2
    sigs = O.bloom_build(off, ids, m, k)
    filters = [[1], [2, 3], [], [5, 1], [11], [4, 6, 8]]
    programs = []
    for f in filters:
        if not f:
            programs.append(([], []))
        else:
            programs.append(([LEAF] + [x for _ in f[1:] for x in (LEAF, AND)],
                             [f[0]] + [x for g in f[1:] for x in (g, 0)]))
    ops, pid, offs = _pack(programs)
    fid = np.array([x for f in filters for x in f], dtype=np.uint64)
    foff = np.concatenate([[0], np.cumsum([len(f) for f in filters])]).astype(np.int64)
    a = O.search_expr(sigs, m, k, items, iscale, q, qs, ops, pid, offs, K)
    b = O.search(sigs, m, k, items, iscale, q, qs, fid, foff, K)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # and with tasks: same weighted aggregation as the plain multi-task search
    rng = np.random.default_rng(33)
    T = 3
    qt = rng.integers(-127, 128, (B, T, items.shape[1])).astype(np.int8)
    qst = rng.uniform(0.5, 1.5, (B, T)).astype(np.float32)
    w = rng.uniform(0, 1, T).astype(np.float32)
    a = O.search_expr(sigs, m, k, items, iscale, qt, qst, ops, pid, offs, K, task_weight=w)
    b = O.search(sigs, m, k, items, iscale, qt, qst, fid, foff, K, task_weight=w)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    with pytest.raises(ValueError):
        O.search_expr(sigs, m, k, items, iscale, q, qs, [LEAF, LEAF] * 6, [1] * 12, np.arange(0, 13, 2), K)
