"""Pins of the oracle's Value Model formulas (paper Sec. 5.2): hand-worked programs, exact rational
arithmetic for the rounded operations, recursive evaluation of random formula trees, the weighted
sum as a special case.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import st_oracle as O
from tests.helpers import f32_mul, round_f32

T, C = O.vm_task, O.VM_CONST


def run(scores, prog):
    ops = [p[0] if isinstance(p, tuple) else p for p in prog]
    consts = [p[1] if isinstance(p, tuple) else 0.0 for p in prog]
    return O.value_model(np.asarray(scores, np.float32), ops, consts)


def test_hand_worked_programs():
    s = [[0.5, 2.0, -1.0], [3.0, 0.25, 4.0]]
    # 2 * like + share
    assert run(s, [(C, 2.0), T(0), O.VM_MUL, T(1), O.VM_ADD]).tolist() == [3.0, 6.25]
    # operand order of SUB: like - share
    assert run(s, [T(0), T(1), O.VM_SUB]).tolist() == [-1.5, 2.75]
    # min / max
    assert run(s, [T(0), T(2), O.VM_MIN]).tolist() == [-1.0, 3.0]
    assert run(s, [T(0), T(2), O.VM_MAX]).tolist() == [0.5, 4.0]
    # condition: if comment > 0 then like else share
    assert run(s, [T(2), (C, 0.0), O.VM_GT, T(0), T(1), O.VM_SELECT]).tolist() == [2.0, 3.0]
    # GT pushes 1 or 0
    assert run(s, [T(0), T(1), O.VM_GT]).tolist() == [0.0, 1.0]
    # a single entry
    assert run(s, [T(1)]).tolist() == [2.0, 0.25]
    assert run(s, [(C, 7.5)]).tolist() == [7.5, 7.5]


def test_each_operation_rounds_once():
    rng = np.random.default_rng(3)
    s = rng.uniform(0.1, 3.0, (50, 2)).astype(np.float32)
    w = np.float32(0.3)
    got = run(s, [(C, float(w)), T(0), O.VM_MUL, T(1), O.VM_ADD])
    for i in range(50):
        prod = f32_mul(w, s[i, 0])
        want = round_f32(Fraction(float(prod)) + Fraction(float(s[i, 1])))
        assert got[i] == want


def tree_eval(t, row):
    k = t[0]
    if k == "task":
        return np.float32(row[t[1]])
    if k == "const":
        return np.float32(t[1])
    if k == "select":
        c, x, y = (tree_eval(u, row) for u in t[1:])
        return x if c != 0 else y
    a, b = tree_eval(t[1], row), tree_eval(t[2], row)
    if k == "add":
        return np.float32(a + b)
    if k == "sub":
        return np.float32(a - b)
    if k == "mul":
        return np.float32(a * b)
    if k == "min":
        return a if a < b else b
    if k == "max":
        return a if a > b else b
    return np.float32(1.0 if a > b else 0.0)


CODE = {"add": O.VM_ADD, "sub": O.VM_SUB, "mul": O.VM_MUL, "min": O.VM_MIN, "max": O.VM_MAX, "gt": O.VM_GT}


def tree_postfix(t):
    k = t[0]
    if k == "task":
        return [T(t[1])]
    if k == "const":
        return [(C, t[1])]
    if k == "select":
        return tree_postfix(t[1]) + tree_postfix(t[2]) + tree_postfix(t[3]) + [O.VM_SELECT]
    return tree_postfix(t[1]) + tree_postfix(t[2]) + [CODE[k]]


def random_formula(rng, n_tasks, depth):
    r = rng.random()
    if depth == 0 or r < 0.2:
        return ("task", int(rng.integers(0, n_tasks))) if rng.random() < 0.7 else ("const", float(np.float32(rng.uniform(-2, 2))))
    if r < 0.3:
        return ("select", random_formula(rng, n_tasks, depth - 1), random_formula(rng, n_tasks, depth - 1),
                random_formula(rng, n_tasks, depth - 1))
    k = ["add", "sub", "mul", "min", "max", "gt"][int(rng.integers(0, 6))]
    return (k, random_formula(rng, n_tasks, depth - 1), random_formula(rng, n_tasks, depth - 1))


def test_program_equals_recursive_tree_evaluation():
    rng = np.random.default_rng(4)
    s = rng.uniform(-2, 2, (40, 4)).astype(np.float32)
    for _ in range(60):
        tree = random_formula(rng, 4, 3)
        got = run(s, tree_postfix(tree))
        want = np.array([tree_eval(tree, row) for row in s], dtype=np.float32)
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), tree


def test_ill_formed_programs():
    for bad, nt in (([O.VM_ADD], 2), ([T(0), O.VM_ADD], 2), ([T(0), T(1)], 2), ([T(2)], 2), ([99], 2),
                    ([T(0), T(1), O.VM_SELECT], 2), ([T(0)] * 17 + [O.VM_ADD] * 16, 1), ([], 1)):
        assert O.vm_depth(bad, nt) == -1, bad
    assert O.vm_depth([T(0), T(1), T(0), O.VM_SELECT], 2) == 3
    with pytest.raises(ValueError):
        O.value_model(np.zeros((2, 2), np.float32), [T(0), T(1)], [0, 0])
