"""Nested-loop workloads: a synthetic directed graph in compressed sparse row form and the
PageRank iteration / sparse matrix-vector product over it, as plain data.

Stands in for the graph of the paper's PageRank experiments (Sec. 7.4, 7.5), which the paper
does not name; the shape follows the social / web graphs such experiments use: a heavy-tailed
in-degree distribution with mean about 11.5 (a few vertices with 1e5 and more in-edges, a
fifth of the vertices with one, a quarter with none), and sources that are partly close to
the destination in vertex order and partly anywhere.

Like workloads/configs.py this module holds input generation and loop descriptions only: no
arithmetic of the method.  Every value is a function of (seed, stream, position), built
from torch integer / correctly rounded f64 operations, so host and device generation give
identical bits.
"""
import torch

from . import rng
from .ir import NestedProgram

SEED = 6
DAMPING = 0.85
PAGERANK_VERTICES = 4_800_000        # full size: about 5.5e7 edges


def make_graph(n_vertices, device="cpu", seed=SEED, max_degree=None, offsets="i64"):
    """CSR by destination: row i lists the sources of the edges into vertex i.

    Returns (rowptr [n+1], src [E] int32, weight [E] f64, outdeg [n] int64).
    In-degree of vertex i: floor(4 / u^0.75) - 4 for u uniform in (0,1] (a power law with
    exponent 7/3), capped at max_degree (default n/16): a quarter of the vertices get no
    in-edge, a fifth exactly one, the mean is about 11.5 and at full size the largest rows
    hold 3e5 edges.  Source of edge e into vertex i: with probability 1/2 within +-512 of
    i, otherwise uniform over all vertices.
    """
    n = int(n_vertices)
    cap = int(max_degree) if max_degree is not None else max(4, n // 16)
    u = 1.0 - rng.unit_f64(seed, 0, 0, n, device)                    # (0, 1]
    s4 = torch.sqrt(torch.sqrt(u))                                   # u^(3/4) from correctly rounded steps
    deg = (torch.floor(4.0 / (s4 * s4 * s4)).to(torch.int64) - 4).clamp(min=0, max=cap)
    rowptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    rowptr[1:] = torch.cumsum(deg, 0)
    n_edges = int(rowptr[-1].item()) if n else 0
    dst = torch.repeat_interleave(torch.arange(n, dtype=torch.int64, device=device), deg)
    near = rng.uniform_int(seed, 1, 0, n_edges, -512, 512, device)
    far = rng.uniform_int(seed, 2, 0, n_edges, 0, max(n - 1, 0), device)
    pick = rng.unit_f64(seed, 3, 0, n_edges, device)
    src = torch.where(pick < 0.5, torch.remainder(dst + near, max(n, 1)), far)
    weight = rng.uniform_f64(seed, 4, 0, n_edges, 0.5, 1.5, device)
    outdeg = torch.bincount(src, minlength=n) if n_edges else torch.zeros(n, dtype=torch.int64, device=device)
    if offsets == "i32":
        rowptr = rowptr.to(torch.int32)
    return rowptr, src.to(torch.int32), weight, outdeg


def program_pagerank(n_vertices, offsets="i64"):
    """One PageRank iteration in pull form over CSR-by-destination:

        new_rank[i] = (1 - d) / n + d * sum over edges (j -> i) of contrib[j]

    with contrib[j] = rank[j] / outdeg[j] (0 for vertices without out-edges) computed by the
    loop of program_contrib.  Outer vectors: row start, row end; inner vector: src; gather vector:
    contrib.  Outer builders: vecbuilder (the new ranks) and a merger (their sum)."""
    p = NestedProgram([offsets, offsets], 0, 1, ["i32"], ["f64"], "f64", "add")
    q = p.inner
    q.merge(0, q.lookup(0, q.col(0)))
    o = p.outer
    base = o.const("f64", (1.0 - DAMPING) / float(n_vertices))
    new_rank = o.bin("add", base, o.bin("mul", o.const("f64", DAMPING), o.inner()))
    o.merge(o.vecbuilder("f64"), new_rank)
    o.merge(o.merger("f64", "add"), new_rank)
    return p


def program_spmv(offsets="i64"):
    """y = A x over CSR: y[i] = sum over the row's entries of weight * x[col]."""
    p = NestedProgram([offsets, offsets], 0, 1, ["i32", "f64"], ["f64"], "f64", "add")
    q = p.inner
    q.merge(0, q.bin("mul", q.col(1), q.lookup(0, q.col(0))))
    o = p.outer
    o.merge(o.vecbuilder("f64"), o.inner())
    return p


def program_contrib():
    """contrib[j] = rank[j] / outdeg[j] if outdeg[j] > 0 else 0: the map between two PageRank
    iterations, an ordinary (not nested) loop over (rank f64, outdeg i64)."""
    from .ir import Program
    p = Program(["f64", "i64"])
    rank, deg = p.col(0), p.col(1)
    has = p.bin("gt", deg, p.const("i64", 0))
    safe = p.select(has, p.un("cast", deg, to="f64"), p.const("f64", 1.0))
    p.merge(p.vecbuilder("f64"), p.select(has, p.bin("div", rank, safe), p.const("f64", 0.0)))
    return p
