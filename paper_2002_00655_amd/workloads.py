"""Seeded synthetic inputs for the parameter-server / blocked-SGD path.

This module only draws random numbers and lays out arrays.  It contains none
of the method's arithmetic (no parameter-server semantics, no SGD step, no
blocking of ratings), so that the CPU oracle and the HIP library can both be
fed from it without sharing any code of the method.

The matrix-factorization inputs stand in for the datasets of Section 4.1
(Table "ML tasks, models, and datasets"), none of which is available: a sparse
m x n matrix with N revealed entries whose row / column degrees are uniform or
long-tailed, and whose values come from a planted low-rank model plus noise.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = [
    "MFWorkload", "KGEWorkload", "MF_CONFIGS", "make_mf", "mf_config",
    "zipf_probs", "equal_bounds", "balanced_bounds", "cyclic_schedule",
    "random_schedule", "make_kge", "partition_by_relation",
]


# --------------------------------------------------------------------------
# degree distributions
# --------------------------------------------------------------------------
def zipf_probs(size: int, s: float, cap: float, rng: np.random.Generator) -> np.ndarray:
    """Probabilities proportional to rank**(-s), truncated so none exceeds
    ``cap`` (the excess is spread over the others in proportion, i.e. by
    water-filling), then assigned to ids through a random permutation."""
    w = np.arange(1, size + 1, dtype=np.float64) ** (-float(s))
    w /= w.sum()
    if cap * size < 1.0:
        raise ValueError("cap too small for the number of ids")
    # t = number of leading (largest) entries clamped to cap.
    tail = np.concatenate([np.cumsum(w[::-1])[::-1], [0.0]])  # tail[t] = sum_{i>=t} w_i
    t = 0
    while t < size:
        rest = tail[t]
        scale = (1.0 - t * cap) / rest if rest > 0 else 0.0
        if w[t] * scale <= cap * (1 + 1e-12):
            break
        # jump ahead: every entry i with w[i]*scale > cap must be clamped too
        nxt = int(np.searchsorted(-w * scale, -cap, side="left"))
        t = max(t + 1, nxt)
    p = w.copy()
    if t > 0:
        rest = tail[t]
        p[:t] = cap
        p[t:] = w[t:] * ((1.0 - t * cap) / rest)
    p /= p.sum()
    return p[rng.permutation(size)]


def _cuda():
    """torch's CUDA device if there is one (only used to speed up sorting and
    searching of the drawn numbers; results are identical to the numpy path)."""
    try:
        import torch
        if torch.cuda.is_available():
            return torch
    except ImportError:
        pass
    return None


def _cdf(p: np.ndarray) -> np.ndarray:
    cdf = np.cumsum(p)
    cdf[-1] = 1.0
    return cdf


def _sample(p: Optional[np.ndarray], size: int, count: int, rng: np.random.Generator) -> np.ndarray:
    """``count`` ids drawn from probabilities ``p`` (uniform if None) by inverting the CDF."""
    if p is None:
        return rng.integers(0, size, size=count, dtype=np.int64)
    out = np.searchsorted(_cdf(p), rng.random(count), side="right")
    np.minimum(out, size - 1, out=out)
    return out.astype(np.int64, copy=False)


def _unique_positions(m, n, nnz, p_row, p_col, rng):
    """Draw (row, col) pairs with independent marginals until ``nnz`` distinct
    cells exist; return them sorted by (row, col)."""
    if p_row is None and p_col is None and m * n < (1 << 62):
        flat = rng.choice(m * n, size=nnz, replace=False)
        flat.sort()
        return flat // n, flat % n
    torch = _cuda()
    have = np.empty(0, dtype=np.int64)
    if torch is not None:
        have_t = torch.empty(0, dtype=torch.int64, device="cuda")
        cdf_r = None if p_row is None else torch.from_numpy(_cdf(p_row)).cuda()
        cdf_c = None if p_col is None else torch.from_numpy(_cdf(p_col)).cuda()
    need = nnz
    over = 1.08
    size = 0
    for _ in range(64):
        cnt = int(need * over) + 1024
        if torch is None:
            r = _sample(p_row, m, cnt, rng)
            c = _sample(p_col, n, cnt, rng)
            have = np.unique(np.concatenate([have, r * n + c]))
            size = have.size
        else:   # same draws, same arithmetic, sorted on the device
            def draw(cdf, dim):
                if cdf is None:
                    return torch.from_numpy(rng.integers(0, dim, size=cnt, dtype=np.int64)).cuda()
                u = torch.from_numpy(rng.random(cnt)).cuda()
                return torch.searchsorted(cdf, u, right=True).clamp_(max=dim - 1)
            r = draw(cdf_r, m)
            c = draw(cdf_c, n)
            have_t = torch.unique(torch.cat([have_t, r * n + c]))
            del r, c
            size = int(have_t.numel())
        if size >= nnz:
            break
        need = nnz - size
        over = min(over * 1.5, 8.0)
    else:
        raise RuntimeError("could not reach the requested number of distinct cells")
    if torch is not None:
        have = have_t.cpu().numpy()
        del have_t
    if have.size > nnz:
        drop = rng.choice(have.size, size=have.size - nnz, replace=False)
        keep = np.ones(have.size, dtype=bool)
        keep[drop] = False
        have = have[keep]
    return have // n, have % n


def _planted_dot(U: np.ndarray, V: np.ndarray, rows: np.ndarray, cols: np.ndarray) -> np.ndarray:
    """sum_k U[rows,k]*V[cols,k] in float32, in chunks (input preparation only)."""
    out = np.empty(rows.size, dtype=np.float32)
    try:
        import torch
        Ut, Vt = torch.from_numpy(U), torch.from_numpy(V)
        dev = torch.device("cuda") if torch.cuda.is_available() else torch.device("cpu")
        Ut, Vt = Ut.to(dev), Vt.to(dev)
        step = 1 << 22 if dev.type == "cuda" else 1 << 20
        for a in range(0, rows.size, step):
            ri = torch.from_numpy(rows[a:a + step]).to(dev)
            ci = torch.from_numpy(cols[a:a + step]).to(dev)
            out[a:a + step] = (Ut[ri] * Vt[ci]).sum(1).cpu().numpy()
        return out
    except ImportError:  # numpy only
        step = 1 << 19
        for a in range(0, rows.size, step):
            out[a:a + step] = np.einsum("ij,ij->i", U[rows[a:a + step]], V[cols[a:a + step]])
        return out


# --------------------------------------------------------------------------
# matrix factorization workloads
# --------------------------------------------------------------------------
@dataclass
class MFWorkload:
    name: str
    m: int
    n: int
    rank: int
    d_row: int
    d_col: int
    lr: float
    lam: float
    epochs: int
    rows: np.ndarray            # int32 [nnz], sorted by (row, col)
    cols: np.ndarray            # int32 [nnz]
    vals: np.ndarray            # float32 [nnz]
    W0: np.ndarray              # float32 [m, rank]  initial row factors
    H0: np.ndarray              # float32 [n, rank]  initial column factors
    row_bounds: np.ndarray = field(default=None)   # int64 [d_row+1]
    col_bounds: np.ndarray = field(default=None)   # int64 [d_col+1]
    noise_std: float = 0.1

    @property
    def nnz(self) -> int:
        return int(self.rows.size)

    @property
    def num_keys(self) -> int:
        return self.m + self.n


# name -> recipe.  "cap" is the largest allowed expected degree as a fraction
# of the other dimension (no row can hold more entries than there are columns).
MF_CONFIGS = {
    # 1,000 x 1,000, 100k entries at uniform cells, planted rank 8, rank 16, 4x4
    "tiny": dict(m=1000, n=1000, nnz=100_000, row=None, col=None, planted=8, rank=16,
                 d=4, epochs=1, values="real", seed=0),
    # 100,000 x 10,000, 10M entries, Zipf(1.0) both sides, planted 32, rank 50, 64x64
    "medium": dict(m=100_000, n=10_000, nnz=10_000_000, row=1.0, col=1.0, planted=32, rank=50,
                   d=64, epochs=5, values="real", seed=0),
    # 480,189 x 17,770, ~100M entries, long-tailed both sides, values 1..5, rank 100, 256x256
    "large": dict(m=480_189, n=17_770, nnz=100_000_000, row=1.0, col=1.0, planted=100, rank=100,
                  d=256, epochs=1, values="stars", seed=0),
    # 10M x 1M, 500M entries, uniform rows, Zipf(1.1) columns, rank 100
    "wide": dict(m=10_000_000, n=1_000_000, nnz=500_000_000, row=None, col=1.1, planted=100,
                 rank=100, d=256, epochs=1, values="real", seed=0),
}


def mf_config(name: str, scale: float = 1.0) -> dict:
    """Recipe of a named configuration; ``scale`` < 1 shrinks m, n and nnz by
    that factor (same degree laws, same rank and blocking) for quick runs."""
    cfg = dict(MF_CONFIGS[name])
    if scale != 1.0:
        cfg["m"] = max(cfg["d"], int(round(cfg["m"] * scale)))
        cfg["n"] = max(cfg["d"], int(round(cfg["n"] * scale)))
        cfg["nnz"] = max(1, int(round(cfg["nnz"] * scale)))
    cfg["name"] = name if scale == 1.0 else f"{name}@{scale:g}"
    return cfg


def make_mf(name: str = "tiny", scale: float = 1.0, seed: Optional[int] = None,
            lr: float = 0.01, lam: float = 0.05, **override) -> MFWorkload:
    cfg = mf_config(name, scale)
    cfg.update(override)
    if seed is not None:
        cfg["seed"] = seed
    m, n, nnz, rank = cfg["m"], cfg["n"], cfg["nnz"], cfg["rank"]
    nnz = min(nnz, (m * n) // 2)
    ss = np.random.SeedSequence(cfg["seed"])
    g_deg_r, g_deg_c, g_pos, g_fac, g_noise, g_init = [np.random.default_rng(s) for s in ss.spawn(6)]

    p_row = None if cfg["row"] is None else zipf_probs(m, cfg["row"], 0.5 * n / nnz, g_deg_r)
    p_col = None if cfg["col"] is None else zipf_probs(n, cfg["col"], 0.5 * m / nnz, g_deg_c)
    r64, c64 = _unique_positions(m, n, nnz, p_row, p_col, g_pos)

    kp = cfg["planted"]
    sf = kp ** -0.5
    U = (g_fac.standard_normal((m, kp), dtype=np.float32) * np.float32(sf))
    V = (g_fac.standard_normal((n, kp), dtype=np.float32) * np.float32(sf))
    dot = _planted_dot(U, V, r64, c64)
    noise = g_noise.standard_normal(r64.size, dtype=np.float32) * np.float32(0.1)
    if cfg["values"] == "stars":
        # unit-variance planted score shifted to the middle of a 1..5 scale
        vals = np.rint(np.clip(3.6 + dot * np.float32(kp ** 0.5) + noise, 1.0, 5.0)).astype(np.float32)
    else:
        vals = (dot + noise).astype(np.float32)
    del U, V, dot, noise

    a = np.float32(rank ** -0.5)
    W0 = ((g_init.random((m, rank), dtype=np.float32) - np.float32(0.5)) * a).astype(np.float32)
    H0 = ((g_init.random((n, rank), dtype=np.float32) - np.float32(0.5)) * a).astype(np.float32)
    d = cfg["d"]
    return MFWorkload(name=cfg["name"], m=m, n=n, rank=rank, d_row=d, d_col=d, lr=lr, lam=lam,
                      epochs=cfg["epochs"], rows=r64.astype(np.int32), cols=c64.astype(np.int32),
                      vals=vals, W0=W0, H0=H0, row_bounds=equal_bounds(m, d), col_bounds=equal_bounds(n, d))


# --------------------------------------------------------------------------
# block boundaries and stratum schedules (inputs of the method, not part of it)
# --------------------------------------------------------------------------
def equal_bounds(size: int, d: int) -> np.ndarray:
    """Range partition into d blocks of floor(size/d) or ceil(size/d) ids."""
    return (np.arange(d + 1, dtype=np.int64) * size) // d


def _split_by_weight(cum: np.ndarray, lo: int, hi: int, parts: int) -> np.ndarray:
    """Inner boundaries (parts - 1 of them) that cut indices [lo, hi) into `parts` stretches of roughly equal weight;
    cum[i] = weight of the indices before i."""
    targets = cum[lo] + np.arange(1, parts, dtype=np.float64) * ((cum[hi] - cum[lo]) / parts)
    b = lo + np.searchsorted(cum[lo:hi + 1], targets, side="left")
    return np.clip(b, lo, hi).astype(np.int64)


def balanced_bounds(ids: np.ndarray, size: int, d: int, per_id: float = 0.0, solo_frac: float = 1.0) -> np.ndarray:
    """Contiguous ranges holding roughly equal numbers of entries each.  per_id > 0: ranges of roughly equal
    weight, where an index weighs its number of entries plus per_id (for blocks whose processing time has a
    part per row or column on top of the part per entry).  An index with more entries than solo_frac times what
    an average range has gets a range of its own - next to anything else it would only make the heaviest range
    heavier (a range is cut where the running weight passes a multiple of the average, so an index of that
    size makes its range that much larger) -, and the other ranges are dealt out to the stretches between such
    indices in proportion to their weights."""
    deg = np.bincount(ids, minlength=size).astype(np.float64) + float(per_id)
    cum = np.concatenate([[0], np.cumsum(deg)])
    solo = np.flatnonzero(deg - float(per_id) > float(solo_frac) * ids.size / d)   # by entries alone, whatever else weighs
    if solo.size:
        # the stretches between the heavy indices, and how many ranges each gets: one each, the rest by weight
        starts = np.concatenate([[0], solo + 1])
        ends = np.concatenate([solo, [size]])
        nonempty = ends > starts
        spare = d - solo.size - int(nonempty.sum())
        if spare >= 0:
            weight = np.where(nonempty, cum[ends] - cum[starts], 0.0)
            share = weight / weight.sum() * spare if weight.sum() > 0 else np.zeros(starts.size)
            parts = np.floor(share).astype(np.int64)
            order = np.argsort(-(share - parts), kind="stable")
            order = order[nonempty[order]]
            left = spare - int(parts.sum())
            for j in range(left if order.size else 0):     # (more than one round only if stretches weigh nothing)
                parts[order[j % order.size]] += 1
            parts[nonempty] += 1
            firsts = []                                    # first index of every range, in order
            for k in range(starts.size):
                if nonempty[k]:
                    firsts.append(np.array([starts[k]], dtype=np.int64))
                    firsts.append(_split_by_weight(cum, int(starts[k]), int(ends[k]), int(parts[k])))
                if k < solo.size:
                    firsts.append(np.array([solo[k]], dtype=np.int64))
            out = np.concatenate(firsts + [np.array([size], dtype=np.int64)])
            if out.size == d + 1:
                return out
        # (too few ranges to set every heavy index apart: cut by weight alone)
    targets = np.arange(d + 1, dtype=np.float64) * (cum[-1] / d)
    b = np.searchsorted(cum, targets, side="left").astype(np.int64)
    b[0], b[-1] = 0, size
    return np.maximum.accumulate(b)


def cyclic_schedule(d: int) -> np.ndarray:
    """int32 [d strata, d tasks, 3] of (worker, row block, column block): in
    stratum s worker b keeps row block b and takes column block (b+s) mod d."""
    b = np.arange(d, dtype=np.int32)
    out = np.empty((d, d, 3), dtype=np.int32)
    for s in range(d):
        out[s, :, 0] = b
        out[s, :, 1] = b
        out[s, :, 2] = (b + s) % d
    return out


def random_schedule(d: int, rng: np.random.Generator) -> np.ndarray:
    """A random exact cover of the d x d blocks by d strata (a random Latin
    square built from shuffled cyclic shifts), with shuffled task order and a
    random worker assignment per stratum."""
    rp, cp, sp = rng.permutation(d), rng.permutation(d), rng.permutation(d)
    out = np.empty((d, d, 3), dtype=np.int32)
    for k, s in enumerate(sp):
        order = rng.permutation(d)
        out[k, :, 0] = rng.permutation(d)
        out[k, :, 1] = rp[order]
        out[k, :, 2] = cp[(order + s) % d]
    return out


# --------------------------------------------------------------------------
# knowledge-graph-embedding workload (Appendix A, "Knowledge graph embeddings")
# --------------------------------------------------------------------------
@dataclass
class KGEWorkload:
    name: str
    num_entities: int
    num_relations: int
    dim: int                    # complex dimension; an embedding holds 2*dim floats
    subj: np.ndarray            # int32 [T]
    rel: np.ndarray             # int32 [T]
    obj: np.ndarray             # int32 [T]
    neg_subj: np.ndarray        # int32 [T, n_neg_s]  replacement subjects
    neg_obj: np.ndarray         # int32 [T, n_neg_o]  replacement objects
    E0: np.ndarray              # float32 [num_entities, 2*dim]
    R0: np.ndarray              # float32 [num_relations, 2*dim]
    lr: float = 0.1
    eps: float = 1e-10


def make_kge(num_entities=500_000, num_relations=600, triples=3_000_000, dim=100,
             n_neg_s=5, n_neg_o=5, s=1.0, seed=0, name="complex") -> KGEWorkload:
    ss = np.random.SeedSequence(seed)
    g_p, g_t, g_n, g_i = [np.random.default_rng(x) for x in ss.spawn(4)]
    p_e = zipf_probs(num_entities, s, min(1.0, 0.02 + 1.0 / num_entities * 4), g_p)
    p_r = zipf_probs(num_relations, s, min(1.0, 0.2 + 1.0 / num_relations * 4), g_p)
    subj = _sample(p_e, num_entities, triples, g_t).astype(np.int32)
    obj = _sample(p_e, num_entities, triples, g_t).astype(np.int32)
    rel = _sample(p_r, num_relations, triples, g_t).astype(np.int32)
    neg_s = g_n.integers(0, num_entities, size=(triples, n_neg_s), dtype=np.int64).astype(np.int32)
    neg_o = g_n.integers(0, num_entities, size=(triples, n_neg_o), dtype=np.int64).astype(np.int32)
    E0 = (g_i.standard_normal((num_entities, 2 * dim), dtype=np.float32) * np.float32(0.1))
    R0 = (g_i.standard_normal((num_relations, 2 * dim), dtype=np.float32) * np.float32(0.1))
    return KGEWorkload(name=name, num_entities=num_entities, num_relations=num_relations, dim=dim,
                       subj=subj, rel=rel, obj=obj, neg_subj=neg_s, neg_obj=neg_o, E0=E0, R0=R0)


def partition_by_relation(w: KGEWorkload, parts: int):
    """The triples grouped by worker, all triples of a relation with one worker (Appendix A of the paper: the
    training data is partitioned by relation): relations are dealt to the workers by decreasing frequency, each
    to the worker with the fewest triples so far; inside a worker's part the triples keep their order.
    Returns (a copy of the workload with the triples reordered, part_ptr of parts + 1 offsets)."""
    counts = np.bincount(w.rel, minlength=w.num_relations)
    load = np.zeros(parts, np.int64)
    owner = np.zeros(w.num_relations, np.int64)
    for r in np.argsort(-counts, kind="stable"):
        p = int(np.argmin(load))
        owner[r] = p
        load[p] += counts[r]
    part = owner[w.rel]
    order = np.argsort(part, kind="stable")
    part_ptr = np.concatenate([[0], np.cumsum(np.bincount(part, minlength=parts))]).astype(np.int64)
    out = KGEWorkload(name=w.name, num_entities=w.num_entities, num_relations=w.num_relations, dim=w.dim,
                      subj=w.subj[order], rel=w.rel[order], obj=w.obj[order], neg_subj=w.neg_subj[order],
                      neg_obj=w.neg_obj[order], E0=w.E0, R0=w.R0)
    return out, part_ptr
