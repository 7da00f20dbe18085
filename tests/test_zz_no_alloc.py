"""The entry point that allocates nothing (st_search_static): its results against st_search's on
the same inputs, bit for bit, on two calls in a row that share the library's fixed workspace, the
second with a smaller input; and the size limit."""
import sys

import numpy as np
import pytest
import torch

from paper_2511_14881_amd import binding as st
from paper_2511_14881_amd import synth as S

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def both(w, bloom, K):
    cfg = w.cfg
    ref = [t.clone() for t in st.st_search(bloom, w.items, w.item_scale, w.queries, w.query_scale, w.filt_ids,
                                           w.filt_offsets, K)]
    torch.cuda.synchronize()
    out = (torch.full((cfg.batch, K), -7, dtype=torch.int64, device="cuda"),
           torch.full((cfg.batch, K), 7.0, dtype=torch.float32, device="cuda"),
           torch.full((cfg.batch,), -7, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = st.st_search_static(bloom, w.items, w.item_scale, w.queries, w.query_scale, w.filt_ids, w.filt_offsets, K,
                              out=out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for name, a, b in zip(("ids", "scores", "count"), got, ref):
        a, b = a.cpu().numpy(), b.cpu().numpy()
        if a.dtype == np.float32:
            a, b = a.view(np.uint32), b.view(np.uint32)
        assert np.array_equal(a, b), f"{name} differ between st_search_static and st_search"


def test_static_workspace_search_matches_st_search_twice_in_a_row():
    say("[no-alloc] first call: mid recipe at 200,000 items, batch 32")
    cfg1 = S.scaled(S.CONFIGS["mid"], 200_000, batch=32)
    w1 = S.make_workload(cfg1, device="cuda")
    b1 = st.st_bloom_build(w1.feat_offsets, w1.feat_ids, cfg1.n_items, cfg1.m_bits, cfg1.k_hashes)
    both(w1, b1, cfg1.top_k)
    say("[no-alloc] second call: smaller corpus, batch and K on the same workspace")
    cfg2 = S.scaled(S.CONFIGS["mid"], 30_001, batch=5, top_k=17)
    w2 = S.make_workload(cfg2, device="cuda")
    b2 = st.st_bloom_build(w2.feat_offsets, w2.feat_ids, cfg2.n_items, cfg2.m_bits, cfg2.k_hashes)
    both(w2, b2, cfg2.top_k)
    say("[no-alloc] and the first shape again")
    both(w1, b1, cfg1.top_k)
    b1.free()
    b2.free()


def test_static_workspace_rejects_sizes_beyond_its_limit():
    cfg = S.scaled(S.CONFIGS["mid"], 50_000, batch=256)
    assert st.st_search_workspace_bytes(cfg.n_items, cfg.d, cfg.batch, 1, cfg.top_k) > st.ST_STATIC_SCRATCH_BYTES
    w = S.make_workload(cfg, device="cuda")
    bloom = st.st_bloom_build(w.feat_offsets, w.feat_ids, cfg.n_items, cfg.m_bits, cfg.k_hashes)
    with pytest.raises(st.StError) as e:
        st.st_search_static(bloom, w.items, w.item_scale, w.queries, w.query_scale, w.filt_ids, w.filt_offsets, cfg.top_k)
    assert e.value.code == st.ST_EWORKSPACE
    bloom.free()
