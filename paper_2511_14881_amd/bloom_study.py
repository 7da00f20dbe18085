#!/usr/bin/env python3
"""Bloom index parameter study (paper Sec. 6.2.2): false-positive rate, index size, build time and
filter latency against the number of signature bits, on a synthetic corpus of the paper's shape
(tens of feature values per item, at most 120, five hash functions).

    python -m paper_2511_14881_amd.bloom_study [--n-items 10000000] [--bits 512,768,1024,2048]

Prints one JSON line per bit width.  The false-positive rate is measured against the exact answer
(does the item's feature list hold the queried id), and printed beside the closed form
mean_i (1 - exp(-k n_i / m))^k over the items' list lengths n_i.  Latency is that of the 1-bit mask
export for a batch of single-id filters: it reads k rows per filter whatever m is.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--n-items", type=int, default=10_000_000)
    ap.add_argument("--bits", default="512,768,1024,2048")
    ap.add_argument("--k", type=int, default=5)
    ap.add_argument("--queries", type=int, default=64)
    ap.add_argument("--vocab", type=int, default=1_000_000)
    ap.add_argument("--max-values", type=int, default=120, help="list lengths are uniform on [0, max-values]")
    ap.add_argument("--seed", type=int, default=20251114)
    args = ap.parse_args()

    import torch
    from paper_2511_14881_amd import binding as st
    from paper_2511_14881_amd import synth

    if not torch.cuda.is_available():
        print("bloom_study needs a GPU", file=sys.stderr)
        sys.exit(2)
    st.lib()
    n = args.n_items
    dev = "cuda"
    idx = torch.arange(n, device=dev, dtype=torch.int64)
    lens = (synth._lsr(synth.rand_u64(args.seed, 21, idx), 11) % (args.max_values + 1))
    off = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    off[1:] = torch.cumsum(lens, 0)
    nnz = int(off[-1])
    ids = torch.empty(nnz, dtype=torch.int64, device=dev)
    chunk = 1 << 26
    for a in range(0, nnz, chunk):  # in pieces: the generator's temporaries are several times the output
        b = min(nnz, a + chunk)
        ids[a:b] = synth._lsr(synth.rand_u64(args.seed, 22, torch.arange(a, b, device=dev, dtype=torch.int64)), 11) % args.vocab
    qz = synth._lsr(synth.rand_u64(args.seed, 23, torch.arange(args.queries, dtype=torch.int64)), 11) % args.vocab
    q_ids = qz.numpy().astype(np.uint64)
    q_off = np.arange(args.queries + 1, dtype=np.int64)
    n_words = (n + 63) // 64

    # exact answer per query: the item's list holds the id (prefix sums of the hits at the list ends)
    exact_bits = []
    for f in q_ids.tolist():
        c = torch.zeros(nnz + 1, dtype=torch.int32, device=dev)
        c[1:] = torch.cumsum((ids == int(f)).to(torch.int32), 0, dtype=torch.int32)
        exact_bits.append((c[off[1:]] - c[off[:-1]]) > 0)
        del c
    lens_f = lens.to(torch.float64)
    shifts = torch.arange(64, device=dev, dtype=torch.int64)

    for m in [int(x) for x in args.bits.split(",")]:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        bloom = st.st_bloom_build(off, ids, n, m, args.k)
        torch.cuda.synchronize()
        build_s = time.perf_counter() - t0
        masks = st.st_bloom_mask(bloom, q_ids, q_off)  # warm-up, and the masks for the rate
        torch.cuda.synchronize()
        reps = 5
        t0 = time.perf_counter()
        for _ in range(reps):
            st.st_bloom_mask(bloom, q_ids, q_off)
        torch.cuda.synchronize()
        mask_ms = (time.perf_counter() - t0) * 1e3 / reps
        fp = neg = fn = 0
        for j in range(args.queries):
            bits = ((masks[j].unsqueeze(1) >> shifts) & 1).reshape(-1)[:n].bool()
            ex = exact_bits[j]
            fp += int((bits & ~ex).sum())
            fn += int((ex & ~bits).sum())
            neg += int((~ex).sum())
        closed = float(((1.0 - torch.exp(-args.k * lens_f / m)) ** args.k).mean())
        out = {
            "study": "bloom bits", "n_items": n, "m_bits": m, "k_hashes": args.k, "queries": args.queries,
            "mean_values_per_item": nnz / n, "max_values_per_item": args.max_values,
            "index_bytes": bloom.nbytes, "index_bytes_at_40M_items": st.st_bloom_layout_bytes(40_000_000, m),
            "build_seconds": build_s, "build_items_per_s": n / build_s,
            "mask_ms_per_batch": mask_ms, "mask_GBs": args.queries * args.k * n_words * 8 / (mask_ms * 1e-3) / 1e9,
            "false_positive_rate": fp / max(neg, 1), "closed_form": closed, "false_negatives": fn,
            "bits_heuristic": args.max_values * args.k * 3,
        }
        print(json.dumps(out), flush=True)
        bloom.free()
        del masks


if __name__ == "__main__":
    main()
