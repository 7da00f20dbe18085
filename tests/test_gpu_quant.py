"""GPU parity of the publish-time quantisation (paper Sec. 4.2) through the C ABI: int8 codes, row
scales and min / max bit-identical to the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import st_oracle as O
from paper_2511_14881_amd import binding as st
from tests.test_gpu_parity import say

pytestmark = pytest.mark.gpu


def check(x, label):
    say(f"[quant] {label}: shape {tuple(x.shape)}")
    q, rs, mm = st.st_quantize_global(torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    oq, ors, (omn, omx) = O.quantize_global(x)
    assert np.array_equal(q.cpu().numpy(), oq), "codes differ"
    assert np.array_equal(rs.cpu().numpy().view(np.uint32), ors.view(np.uint32)), "scales differ"
    got = mm.cpu().numpy()
    assert got[0] == omn and got[1] == omx


@pytest.mark.parametrize("n,d", [(1, 1), (7, 5), (300, 48), (1000, 128), (70_001, 16), (33, 1000), (1_000_000, 128)])
def test_quantisation_matches_oracle(n, d):
    rng = np.random.default_rng(n + d)
    x = (rng.standard_normal((n, d)) * rng.uniform(0.01, 30.0)).astype(np.float32)
    check(x, "normal")


def test_special_tables():
    check(np.zeros((5, 16), np.float32), "all zero")
    check(np.zeros((0, 16), np.float32), "empty")
    check(np.full((3, 17), -2.5, np.float32), "constant negative")
    x = np.linspace(-1.0, 3.0, 4096, dtype=np.float32).reshape(64, 64)  # many exact ties at .5 steps of s
    check(x, "ramp")
    x = np.array([[1e-30, -3e-30, 2e-30, 0.0]], dtype=np.float32)
    check(x, "tiny magnitudes")
    x = np.array([[3e38, -1e38, 5.0, 0.0]], dtype=np.float32)
    check(x, "huge magnitudes")


def test_quantised_table_feeds_the_search():
    # quantise items and queries on the GPU, search with the per-row scales it wrote, and compare
    # with the oracle run on the oracle's own quantisation of the same fp32 tables
    rng = np.random.default_rng(12)
    n, d, B, K = 20_000, 64, 8, 20
    xi = rng.standard_normal((n, d)).astype(np.float32)
    xq = rng.standard_normal((B, d)).astype(np.float32)
    qi, si, _ = st.st_quantize_global(torch.from_numpy(xi).cuda())
    qq, sq, _ = st.st_quantize_global(torch.from_numpy(xq).cuda())
    off = torch.arange(n + 1, dtype=torch.int64)
    ids = torch.from_numpy(rng.integers(0, 6, n).astype(np.int64))
    bloom = st.st_bloom_build(off.cuda(), ids.cuda(), n, 64, 2)
    fid = np.array([b % 6 for b in range(B)], dtype=np.uint64)
    foff = np.arange(B + 1, dtype=np.int64)
    g_ids, g_scores, g_count = st.st_search(bloom, qi, si, qq, sq, fid, foff, K)
    torch.cuda.synchronize()
    oqi, osi, _ = O.quantize_global(xi)
    oqq, osq, _ = O.quantize_global(xq)
    sigs = O.bloom_build(off.numpy(), ids.numpy().view(np.uint64), 64, 2)
    oi, os_, oc = O.search(sigs, 64, 2, oqi, osi, oqq, osq, fid, foff, K)
    assert np.array_equal(g_ids.cpu().numpy(), oi) and np.array_equal(g_count.cpu().numpy(), oc)
    assert np.array_equal(g_scores.cpu().numpy().view(np.uint32), os_.view(np.uint32))
    bloom.free()
