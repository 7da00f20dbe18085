"""Seeded synthetic inputs shaped like the paper's retrieval workloads.

This module holds no arithmetic of the retrieval method (no Bloom hashing, no
scoring, no selection): it only draws corpora, feature lists, queries and
filters.  Both the GPU library's tests and the CPU oracle's tests take their
inputs from here, so the two sides always see the same bytes.

Everything is a pure function of (seed, stream, index) through a counter-based
generator built from integer tensor ops, so the same values come out on the CPU
and on the GPU, in any chunking.  The generator's mixer is the 64-bit finaliser
of MurmurHash3, deliberately not the hash the Bloom index uses.

The paper's own pools are production data (80M / 10M / 20M / 40M items, d=128,
a handful of feature values per item, broad filters, large top-k; Sec. 6); the
five configurations below stand in for them.
"""
from __future__ import annotations

import itertools
from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 20251114
_M64 = (1 << 64) - 1
# stream tags
S_ITEMS, S_ISCALE, S_FEATS, S_QUERIES, S_QSCALE, S_FILTERS, S_WEIGHTS = 1, 2, 3, 4, 5, 6, 7


def _s64(x: int) -> int:
    """Python int (mod 2^64) as the signed value torch.int64 stores."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


_C1 = _s64(0xFF51AFD7ED558CCD)
_C2 = _s64(0xC4CEB9FE1A85EC53)
_GOLD = 0x9E3779B97F4A7C15


def _lsr(z: torch.Tensor, s: int) -> torch.Tensor:
    return (z >> s) & ((1 << (64 - s)) - 1)


def _fmix(z: torch.Tensor) -> torch.Tensor:
    z = (z ^ _lsr(z, 33)) * _C1
    z = (z ^ _lsr(z, 33)) * _C2
    return z ^ _lsr(z, 33)


def _fmix_int(z: int) -> int:
    z &= _M64
    z = ((z ^ (z >> 33)) * 0xFF51AFD7ED558CCD) & _M64
    z = ((z ^ (z >> 33)) * 0xC4CEB9FE1A85EC53) & _M64
    return z ^ (z >> 33)


def stream_key(seed: int, stream: int) -> int:
    return _fmix_int((seed * _GOLD + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _M64)


def rand_u64(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """64 random bits per index (int64 tensor holding the bit pattern)."""
    key = _s64(stream_key(seed, stream))
    return _fmix(_fmix(idx * _s64(_GOLD) + key) ^ key)


def rand_unit(seed: int, stream: int, idx: torch.Tensor) -> torch.Tensor:
    """Uniform float64 in [0, 1) from the top 53 bits."""
    return _lsr(rand_u64(seed, stream, idx), 11).to(torch.float64) * (1.0 / (1 << 53))


def _arange(lo: int, hi: int, device) -> torch.Tensor:
    return torch.arange(lo, hi, dtype=torch.int64, device=device)


_GAUSS_TABLE = None


def _gauss_table() -> torch.Tensor:
    """int8 quantile table: entry u is clip(round_half_even(40 * Phi^-1((u+.5)/65536)), +-127)."""
    global _GAUSS_TABLE
    if _GAUSS_TABLE is None:
        from scipy.special import ndtri
        z = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
        _GAUSS_TABLE = torch.from_numpy(np.clip(np.rint(40.0 * z), -127, 127).astype(np.int8))
    return _GAUSS_TABLE


def gen_int8(seed: int, stream: int, n_rows: int, d: int, dist: str, device="cpu",
             chunk_rows: int = 1 << 20) -> torch.Tensor:
    """[n_rows, d] int8.  dist 'uniform': 255 values in [-127,127]; 'gauss': N(0,40^2) rounded
    and clipped to +-127.  Four values come from each 64-bit draw (16 bits apiece)."""
    assert d % 4 == 0
    out = torch.empty((n_rows, d), dtype=torch.int8, device=device)
    table = _gauss_table().to(device) if dist == "gauss" else None
    per_row = d // 4
    shifts = torch.tensor([0, 16, 32, 48], dtype=torch.int64, device=device)
    for r0 in range(0, n_rows, chunk_rows):
        r1 = min(n_rows, r0 + chunk_rows)
        z = rand_u64(seed, stream, _arange(r0 * per_row, r1 * per_row, device))
        u16 = (z.unsqueeze(1) >> shifts) & 0xFFFF  # [n, 4]
        if dist == "gauss":
            v = table[u16.reshape(-1)]
        elif dist == "uniform":
            v = (((u16 * 255) >> 16) - 127).to(torch.int8).reshape(-1)
        else:
            raise ValueError(dist)
        out[r0:r1] = v.reshape(r1 - r0, d)
    return out


def gen_scale(seed: int, stream: int, n: int, device="cpu") -> torch.Tensor:
    """fp32 in [0.5, 1.5)."""
    return (0.5 + rand_unit(seed, stream, _arange(0, n, device))).to(torch.float32)


def zipf_cdf(vocab: int, s: float) -> np.ndarray:
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


_SCATTER_A = 48271


def rank_to_id(rank0, vocab: int, scatter: bool):
    """Zipf rank (0-based) -> feature id.  The scatter map keeps popular ids from
    being numeric neighbours."""
    return (rank0 * _SCATTER_A) % vocab if scatter else rank0


@dataclass
class Config:
    name: str
    n_items: int
    d: int
    batch: int
    n_tasks: int           # 0 = single-task entry point
    m_bits: int
    k_hashes: int
    n_terms: int           # filter arity
    top_k: int
    feats_per_item: int
    vocab: int
    zipf_s: float          # 0 = uniform vocabulary
    item_dist: str         # 'uniform' | 'gauss'
    target_sel: float      # wanted exact-set selectivity of a filter (ignored for uniform vocab)
    pool: int              # number of distinct filters in a batch
    query_scale_one: bool = False
    seed: int = BASE_SEED
    scatter_ids: bool = True
    extra: dict = field(default_factory=dict)


CONFIGS = {
    "tiny": Config("tiny", 10_000, 64, 1, 0, 64, 2, 1, 10, 4, 1_000, 0.0, "uniform", 0.0, 1,
                   query_scale_one=True),
    "mid": Config("mid", 1_000_000, 128, 64, 0, 256, 3, 2, 100, 8, 100_000, 1.1, "gauss", 0.10, 8),
    "large": Config("large", 10_000_000, 256, 256, 0, 512, 4, 3, 500, 16, 1_000_000, 1.05, "gauss",
                    0.05, 8),
    "multi": Config("multi", 5_000_000, 128, 128, 4, 256, 3, 2, 200, 8, 100_000, 1.1, "gauss",
                    0.10, 8),
    "mfma": Config("mfma", 20_000_000, 128, 1024, 0, 128, 2, 1, 1000, 8, 100_000, 1.1, "gauss",
                   0.50, 2),
}


def scaled(cfg: Config, n_items: int, **kw) -> Config:
    """Same recipe on a smaller corpus (for parity cases the oracle finishes in seconds)."""
    d = dict(cfg.__dict__)
    d.update(n_items=n_items, name=f"{cfg.name}@{n_items}")
    d.update(kw)
    return Config(**d)


def gen_features(cfg: Config, device="cpu", chunk: int = 1 << 22):
    """CSR feature lists: offsets int64 [N+1], ids int64 (values < vocab) [N*n].
    n ids per item, drawn with replacement."""
    n = cfg.feats_per_item
    total = cfg.n_items * n
    ids = torch.empty(total, dtype=torch.int64, device=device)
    cdf = None
    if cfg.zipf_s > 0:
        cdf = torch.from_numpy(zipf_cdf(cfg.vocab, cfg.zipf_s)).to(device)
    for a in range(0, total, chunk):
        b = min(total, a + chunk)
        u = rand_unit(cfg.seed, S_FEATS, _arange(a, b, device))
        if cdf is None:
            r = (u * cfg.vocab).to(torch.int64).clamp_(max=cfg.vocab - 1)
            ids[a:b] = r
        else:
            r = torch.searchsorted(cdf, u, right=True).clamp_(max=cfg.vocab - 1)
            ids[a:b] = rank_to_id(r, cfg.vocab, cfg.scatter_ids)
    offsets = torch.arange(0, total + 1, n, dtype=torch.int64, device=device)
    return offsets, ids


def choose_filter_pool(cfg: Config, feat_ids_sample: np.ndarray) -> list[tuple[int, ...]]:
    """Pick cfg.pool distinct conjunctions of cfg.n_terms ids whose exact-set selectivity,
    counted on a sample of items, is closest to cfg.target_sel.  Candidates are the 32 most
    frequent ids (Zipf vocab) -- recommendation filters are few and broad (paper Sec. 7)."""
    n = cfg.feats_per_item
    if cfg.zipf_s <= 0:
        # uniform vocabulary: any id is as good as another; take the pool from the filter stream
        z = rand_u64(cfg.seed, S_FILTERS, _arange(1 << 20, (1 << 20) + cfg.pool * cfg.n_terms, "cpu"))
        v = (_lsr(z, 11) % cfg.vocab).reshape(cfg.pool, cfg.n_terms).tolist()
        return [tuple(int(x) for x in row) for row in v]
    rows = feat_ids_sample.reshape(-1, n)
    head = [int(rank_to_id(r, cfg.vocab, cfg.scatter_ids)) for r in range(32)]
    pres = np.stack([(rows == h).any(axis=1) for h in head], axis=1).astype(np.float32)  # [S, 32]
    n_s = float(pres.shape[0])
    if cfg.n_terms == 1:
        count = {(i,): c for i, c in enumerate(pres.sum(axis=0))}
    elif cfg.n_terms == 2:
        c2 = pres.T @ pres
        count = {(i, j): c2[i, j] for i, j in itertools.combinations(range(32), 2)}
    elif cfg.n_terms == 3:
        count = {}
        for i in range(32):
            c3 = (pres * pres[:, i:i + 1]).T @ pres
            for j, l in itertools.combinations(range(i + 1, 32), 2):
                count[(i, j, l)] = c3[j, l]
    else:
        raise ValueError("filter arity above 3 is not part of any workload")
    scored = []
    for combo, c in count.items():
        sel = float(c) / n_s
        scored.append((abs(np.log(max(sel, 1e-9) / cfg.target_sel)), combo, sel))
    scored.sort(key=lambda t: (t[0], t[1]))
    pool = [tuple(head[c] for c in combo) for _, combo, _ in scored[: cfg.pool]]
    return pool


def gen_filters(cfg: Config, pool: list[tuple[int, ...]]):
    """Per-query conjunctions as CSR (ids uint64 [sum], offsets int64 [B+1])."""
    z = rand_u64(cfg.seed, S_FILTERS, _arange(0, cfg.batch, "cpu"))
    pick = (_lsr(z, 11) % len(pool)).tolist()
    ids, off = [], [0]
    for b in range(cfg.batch):
        ids.extend(pool[pick[b]])
        off.append(len(ids))
    return np.asarray(ids, dtype=np.uint64), np.asarray(off, dtype=np.int64)


@dataclass
class Workload:
    cfg: Config
    items: torch.Tensor         # [N, d] int8
    item_scale: torch.Tensor    # [N] fp32
    feat_offsets: torch.Tensor  # [N+1] int64
    feat_ids: torch.Tensor      # [nnz] int64 (non-negative; reinterpret as uint64)
    queries: torch.Tensor       # [B, d] or [B, T, d] int8
    query_scale: torch.Tensor   # [B] or [B, T] fp32
    task_weight: np.ndarray | None  # [T] fp32, host
    filt_ids: np.ndarray        # uint64, host
    filt_offsets: np.ndarray    # int64 [B+1], host
    pool: list


def make_workload(cfg: Config, device="cpu") -> Workload:
    items = gen_int8(cfg.seed, S_ITEMS, cfg.n_items, cfg.d, cfg.item_dist, device)
    item_scale = gen_scale(cfg.seed, S_ISCALE, cfg.n_items, device)
    off, ids = gen_features(cfg, device)
    T = max(cfg.n_tasks, 1)
    q = gen_int8(cfg.seed, S_QUERIES, cfg.batch * T, cfg.d, cfg.item_dist, device)
    if cfg.query_scale_one:
        qs = torch.ones(cfg.batch * T, dtype=torch.float32, device=device)
    else:
        qs = gen_scale(cfg.seed, S_QSCALE, cfg.batch * T, device)
    w = None
    if cfg.n_tasks > 0:
        q = q.reshape(cfg.batch, T, cfg.d)
        qs = qs.reshape(cfg.batch, T)
        w = rand_unit(cfg.seed, S_WEIGHTS, _arange(0, T, "cpu")).to(torch.float32).numpy()
    sample_items = min(cfg.n_items, 200_000)
    sample = ids[: sample_items * cfg.feats_per_item].cpu().numpy()
    pool = choose_filter_pool(cfg, sample)
    fid, foff = gen_filters(cfg, pool)
    return Workload(cfg, items, item_scale, off, ids, q, qs, w, fid, foff, pool)


def refilter(w: Workload, target_sel: float, name: str | None = None) -> Workload:
    """The same corpus and queries with another filter pool: conjunctions whose exact-set
    selectivity is closest to target_sel (1.0 = the broadest the 32 most frequent ids allow).
    Shares every tensor with w; only the config and the host filter arrays are new."""
    cfg = scaled(w.cfg, w.cfg.n_items, target_sel=target_sel,
                 name=name or f"{w.cfg.name}+sel{target_sel:g}")
    sample_items = min(cfg.n_items, 200_000)
    sample = w.feat_ids[: sample_items * cfg.feats_per_item].cpu().numpy()
    pool = choose_filter_pool(cfg, sample)
    fid, foff = gen_filters(cfg, pool)
    return Workload(cfg, w.items, w.item_scale, w.feat_offsets, w.feat_ids, w.queries, w.query_scale,
                    w.task_weight, fid, foff, pool)


# selectivity targets of the Large workload's sweep (the last one: the broadest available)
LARGE_SWEEP = (0.001, 0.01, 0.05, 1.0)


# operation codes of a filter program (postfix order), as the library's header defines them
OP_LEAF, OP_AND, OP_OR, OP_NOT = 0, 1, 2, 3


def gen_filter_programs(cfg: Config, pool: int = 8, with_not: bool = True):
    """Per-query filters of the paper's query form (Sec. 4): a broad term AND an OR-group of two
    narrower terms, every second program of the pool also AND NOT a further term.  Terms come
    from the 32 most frequent ids.  Returns (ops int32 [sum], ids uint64 [sum], offsets int64
    [B+1], programs) with programs[p] = (ops, ids) of pool entry p; query b uses entry
    u64(filters, 2^21 + b) mod pool."""
    head = [int(rank_to_id(r, cfg.vocab, cfg.scatter_ids)) for r in range(32)] if cfg.zipf_s > 0 else \
           [int(x) % cfg.vocab for x in range(32)]
    z = _lsr(rand_u64(cfg.seed, S_FILTERS, _arange(3 << 20, (3 << 20) + 4 * pool, "cpu")), 11).reshape(pool, 4).tolist()
    programs = []
    for p in range(pool):
        a = head[z[p][0] % 4]
        b = head[2 + z[p][1] % 14]
        c = head[2 + (z[p][1] % 14 + 1 + z[p][2] % 13) % 14]  # differs from b
        ops = [OP_LEAF, OP_LEAF, OP_LEAF, OP_OR, OP_AND]
        ids = [a, b, c, 0, 0]
        if with_not and p % 2 == 1:
            ops += [OP_LEAF, OP_NOT, OP_AND]
            ids += [head[z[p][3] % 8], 0, 0]
        programs.append((ops, ids))
    pick = (_lsr(rand_u64(cfg.seed, S_FILTERS, _arange(2 << 20, (2 << 20) + cfg.batch, "cpu")), 11) % pool).tolist()
    all_ops, all_ids, off = [], [], [0]
    for b in range(cfg.batch):
        all_ops.extend(programs[pick[b]][0])
        all_ids.extend(programs[pick[b]][1])
        off.append(len(all_ops))
    return (np.asarray(all_ops, dtype=np.int32), np.asarray(all_ids, dtype=np.uint64),
            np.asarray(off, dtype=np.int64), programs)


def flatten_tasks(w: Workload, prog):
    """A multi-task workload as single-task queries: every task embedding of a query becomes a
    query of its own with the original query's filter program (the paper batches the tasks of a
    request against one index and gets task-specific lists, Sec. 5.2).  prog = (ops, ids, offsets)
    per original query; returns the flattened workload and programs."""
    cfg = w.cfg
    T = max(cfg.n_tasks, 1)
    ops, ids, off = prog
    f_ops, f_ids, f_off = [], [], [0]
    for b in range(cfg.batch):
        for _ in range(T):
            f_ops.extend(ops[off[b]:off[b + 1]].tolist())
            f_ids.extend(ids[off[b]:off[b + 1]].tolist())
            f_off.append(len(f_ops))
    fo = w.filt_offsets
    fid = np.concatenate([np.tile(w.filt_ids[fo[b]:fo[b + 1]], T) for b in range(cfg.batch)]) if cfg.batch else w.filt_ids
    foff = np.concatenate([[0], np.cumsum(np.repeat(fo[1:] - fo[:-1], T))]).astype(np.int64)
    c2 = scaled(cfg, cfg.n_items, batch=cfg.batch * T, n_tasks=0, name=cfg.name)
    w2 = Workload(c2, w.items, w.item_scale, w.feat_offsets, w.feat_ids, w.queries.reshape(cfg.batch * T, cfg.d),
                  w.query_scale.reshape(cfg.batch * T), None, fid.astype(np.uint64), foff, w.pool)
    return w2, (np.asarray(f_ops, dtype=np.int32), np.asarray(f_ids, dtype=np.uint64), np.asarray(f_off, dtype=np.int64))


S_CLUSTERS = 11  # random stream of the cluster layout and the centroids


def gen_clusters(cfg: Config, n_clusters: int, device="cpu"):
    """A cluster layout for the probing search: the corpus cut into n_clusters contiguous ranges
    at sorted random positions (so sizes vary, a few clusters may be empty), centroids drawn from
    the item family with scales U(0.5, 1.5).  No clustering is trained: the probing cost and the
    exactness of the result do not depend on where the centroids are.  Returns (centroids int8
    [n_c, d], scales fp32 [n_c], offsets int64 [n_c + 1])."""
    cent = gen_int8(cfg.seed, S_CLUSTERS, n_clusters, cfg.d, cfg.item_dist, device)
    cs = gen_scale(cfg.seed, S_CLUSTERS + 1, n_clusters, device)
    z = _lsr(rand_u64(cfg.seed, S_CLUSTERS + 2, _arange(0, max(n_clusters - 1, 0), "cpu")), 11)
    cuts = torch.sort(z % (cfg.n_items + 1)).values if n_clusters > 1 else torch.zeros(0, dtype=torch.int64)
    off = torch.cat([torch.zeros(1, dtype=torch.int64), cuts.to(torch.int64),
                     torch.full((1,), cfg.n_items, dtype=torch.int64)]).to(device)
    return cent, cs, off
