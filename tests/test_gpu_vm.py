"""GPU parity of the Value Model formulas (paper Sec. 5.2) through the C ABI: bit-identical to the
CPU oracle on hand-written and random formulas."""
import numpy as np
import pytest
import torch

from oracle import st_oracle as O
from paper_2511_14881_amd import binding as st
from tests.test_gpu_parity import say
from tests.test_oracle_vm_pins import random_formula, tree_postfix

pytestmark = pytest.mark.gpu
T, C = O.vm_task, O.VM_CONST


def split(prog):
    ops = [p[0] if isinstance(p, tuple) else p for p in prog]
    consts = [p[1] if isinstance(p, tuple) else 0.0 for p in prog]
    return ops, consts


def check(scores, prog, label):
    ops, consts = split(prog)
    say(f"[vm] {label}: n={scores.shape[0]} T={scores.shape[1]} entries={len(ops)}")
    got = st.st_value_model(torch.from_numpy(scores).cuda(), ops, consts)
    torch.cuda.synchronize()
    want = O.value_model(scores, ops, consts)
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


@pytest.mark.parametrize("n,n_tasks", [(1, 1), (1000, 3), (70_001, 4), (300_000, 8)])
def test_random_formulas_match_oracle(n, n_tasks):
    rng = np.random.default_rng(n + n_tasks)
    scores = rng.uniform(-3, 3, (n, n_tasks)).astype(np.float32)
    scores[rng.random((n, n_tasks)) < 0.05] = 0.0  # exact zeros exercise the conditions
    for _ in range(12):
        check(scores, tree_postfix(random_formula(rng, n_tasks, 4)), "random tree")
    # a long weighted sum, and the deepest stack allowed
    ws = [(C, 0.25), T(0), O.VM_MUL]
    for t in range(1, n_tasks):
        ws += [(C, 0.1 * t), T(t), O.VM_MUL, O.VM_ADD]
    check(scores, ws, "weighted sum")
    check(scores, [T(0)] * 16 + [O.VM_ADD, O.VM_MAX, O.VM_MUL] * 5, "depth 16")


def test_ill_formed_formulas_are_rejected():
    s = torch.zeros((4, 2), dtype=torch.float32, device="cuda")
    for bad in ([O.VM_ADD], [T(0), O.VM_ADD], [T(0), T(1)], [T(2)], [99], [T(0), T(1), O.VM_SELECT],
                [T(0)] * 17 + [O.VM_ADD] * 16, [T(0)] + [T(0), O.VM_ADD] * 32):
        with pytest.raises(st.StError) as e:
            st.st_value_model(s, bad, [0.0] * len(bad))
        assert e.value.code == st.ST_EINVAL
    with pytest.raises(st.StError):
        st.st_value_model(s, [C], [float("nan")])
    out = st.st_value_model(torch.zeros((0, 2), dtype=torch.float32, device="cuda"), [T(1)], [0.0])
    assert out.numel() == 0
