"""The five benchmark loops and the paper's printed examples, as plain data.

Each entry gives (a) the recipe of its seeded synthetic columns and (b) the
loop body / builders as a `workloads.ir.Program`.  Nothing here evaluates a
body: the oracle and the HIP library do that, independently of each other.

The synthetic columns stand in for the datasets the paper measures on, which
are not available: the city/crime frame of Sec. 2.1 (C1), the Black-Scholes
records of Sec. 7.1 (C2), TPC-H lineitem-like columns for Q6 and Q1 of
Sec. 7.1/7.4 (C3, C4) and the zip-code cleaning file of Sec. 7.1 (C5).
"""
import numpy as np
import torch

from . import rng
from .ir import Program

FULL_ROWS = {"C1": 1_000_000, "C2": 50_000_000, "C3": 200_000_000,
             "C4": 200_000_000, "C5": 100_000_000}
SEEDS = {"C1": 1, "C2": 2, "C3": 3, "C4": 4, "C5": 5}

INV_SQRT2 = 0.70710678118654752440   # nearest double to 1/sqrt(2)
RATE = 0.02


# ----------------------------------------------------------------------
# programs
# ----------------------------------------------------------------------
def program_c1():
    """filter x>0.5, map x*y+1.0, merger<f64,+> and merger<i64,+> count."""
    p = Program(["f64", "f64"])
    x, y = p.col(0), p.col(1)
    pred = p.bin("gt", x, p.const("f64", 0.5))
    v = p.bin("add", p.bin("mul", x, y), p.const("f64", 1.0))
    one = p.const("i64", 1)
    p.merge(p.merger("f64", "add"), v, pred=pred)
    p.merge(p.merger("i64", "add"), one, pred=pred)
    return p


def program_c2():
    """European option prices; two unconditional vecbuilders (call, put).

    d1 = (ln(S/K) + (r + s^2/2) T) / (s sqrt T),  d2 = d1 - s sqrt T,
    N(x) = 1/2 + 1/2 erf(x/sqrt 2),  N(-x) = 1/2 - 1/2 erf(x/sqrt 2),
    call = S N(d1) - K e^{-rT} N(d2),  put = K e^{-rT} N(-d2) - S N(-d1).
    """
    p = Program(["f64", "f64", "f64", "f64"])
    S, K, T, vol = p.col(0), p.col(1), p.col(2), p.col(3)
    half = p.const("f64", 0.5)
    r = p.const("f64", RATE)
    isq2 = p.const("f64", INV_SQRT2)
    sqrt_t = p.un("sqrt", T)
    vol_sqrt_t = p.bin("mul", vol, sqrt_t)
    ln_sk = p.un("log", p.bin("div", S, K))
    half_var = p.bin("mul", p.bin("mul", vol, vol), half)
    drift = p.bin("mul", p.bin("add", r, half_var), T)
    d1 = p.bin("div", p.bin("add", ln_sk, drift), vol_sqrt_t)
    d2 = p.bin("sub", d1, vol_sqrt_t)
    e1 = p.un("erf", p.bin("mul", d1, isq2))
    e2 = p.un("erf", p.bin("mul", d2, isq2))
    he1 = p.bin("mul", half, e1)
    he2 = p.bin("mul", half, e2)
    n_d1 = p.bin("add", half, he1)
    n_d2 = p.bin("add", half, he2)
    n_md1 = p.bin("sub", half, he1)
    n_md2 = p.bin("sub", half, he2)
    disc = p.un("exp", p.un("neg", p.bin("mul", r, T)))
    k_disc = p.bin("mul", K, disc)
    call = p.bin("sub", p.bin("mul", S, n_d1), p.bin("mul", k_disc, n_d2))
    put = p.bin("sub", p.bin("mul", k_disc, n_md2), p.bin("mul", S, n_md1))
    p.merge(p.vecbuilder("f64"), call)
    p.merge(p.vecbuilder("f64"), put)
    p.named = {"d1": d1, "d2": d2, "call": call, "put": put}
    return p


def program_c3():
    """365<=day<730 and 0.05<=discount<=0.07 and quantity<24; sum price*discount."""
    p = Program(["i32", "f64", "f64", "f64"])
    day, disc, qty, price = p.col(0), p.col(1), p.col(2), p.col(3)
    c = p.bin("ge", day, p.const("i32", 365))
    c = p.bin("and", c, p.bin("lt", day, p.const("i32", 730)))
    c = p.bin("and", c, p.bin("ge", disc, p.const("f64", 0.05)))
    c = p.bin("and", c, p.bin("le", disc, p.const("f64", 0.07)))
    c = p.bin("and", c, p.bin("lt", qty, p.const("f64", 24.0)))
    v = p.bin("mul", price, disc)
    p.merge(p.merger("f64", "add"), v, pred=c)
    return p


def program_c4(capacity=8):
    """filter day<=2400; group by (flag,status); four f64 sums and a count."""
    p = Program(["i8", "i8", "i32", "f64", "f64", "f64", "f64"])
    flag, status, day = p.col(0), p.col(1), p.col(2)
    qty, price, disc, tax = p.col(3), p.col(4), p.col(5), p.col(6)
    pred = p.bin("le", day, p.const("i32", 2400))
    one = p.const("f64", 1.0)
    disc_price = p.bin("mul", price, p.bin("sub", one, disc))
    charge = p.bin("mul", disc_price, p.bin("add", one, tax))
    cnt = p.const("i64", 1)
    d = p.dictmerger(["i8", "i8"], ["f64", "f64", "f64", "f64", "i64"], "add", capacity)
    p.merge(d, [qty, price, disc_price, charge, cnt], keys=[flag, status], pred=pred)
    return p


def program_c5(capacity=100_000):
    """filter code>0, map code mod 100000; vecbuilder + dictmerger count."""
    p = Program(["i64"])
    code = p.col(0)
    pred = p.bin("gt", code, p.const("i64", 0))
    v = p.bin("mod", code, p.const("i64", 100_000))
    one = p.const("i64", 1)
    p.merge(p.vecbuilder("i64"), v, pred=pred)
    p.merge(p.dictmerger(["i64"], ["i64"], "add", capacity), [one], keys=[v], pred=pred)
    return p


EXAMPLES = {}


def program_group_by_zip(capacity=100_000):
    """filter code>0; groupbuilder: the codes grouped by code mod 100000 (the C5 column)."""
    p = Program(["i64"])
    code = p.col(0)
    p.merge(p.groupbuilder(["i64"], "i64", capacity), code, keys=[p.bin("mod", code, p.const("i64", 100_000))],
            pred=p.bin("gt", code, p.const("i64", 0)))
    return p


PROGRAMS = {"C1": program_c1, "C2": program_c2, "C3": program_c3,
            "C4": program_c4, "C5": program_c5}

# algorithmic bytes per row (every input column once, every mandatory output once)
IN_BYTES = {"C1": 16, "C2": 32, "C3": 28, "C4": 38, "C5": 8}
OUT_BYTES = {"C1": 0.0, "C2": 16.0, "C3": 0.0, "C4": 0.0, "C5": 7.2}


# ----------------------------------------------------------------------
# the loops printed in the paper (Listing "Examples of using builders",
# Listing "for operating over multiple builders", Listing "after loop fusion")
# ----------------------------------------------------------------------
def example_merge_values():
    p = Program(["i32"])
    p.merge(p.vecbuilder("i32"), p.col(0))
    return p


def example_map_plus_one():
    p = Program(["i32"])
    p.merge(p.vecbuilder("i32"), p.bin("add", p.col(0), p.const("i32", 1)))
    return p


def example_zip_filter():
    p = Program(["i32", "i32"])
    a, b = p.col(0), p.col(1)
    pred = p.bin("gt", a, p.const("i32", 1))
    p.merge(p.vecbuilder("i32"), p.bin("add", a, b), pred=pred)
    return p


def example_two_builders():
    p = Program(["i32"])
    x = p.col(0)
    p.merge(p.vecbuilder("i32"), p.bin("add", x, p.const("i32", 1)))
    p.merge(p.merger("i32", "add"), x)
    return p


def example_filter_sum(threshold=500000):
    p = Program(["i64"])
    x = p.col(0)
    p.merge(p.merger("i64", "add"), x, pred=p.bin("gt", x, p.const("i64", threshold)))
    return p


# ----------------------------------------------------------------------
# columns
# ----------------------------------------------------------------------
def _zipf_tables(seed, nkeys=100_000, s=1.1):
    """Host-side tables: cumulative Zipf weights and a seeded key permutation."""
    w = 1.0 / np.power(np.arange(1, nkeys + 1, dtype=np.float64), s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    order = rng.bits64(seed, 100, 0, nkeys).numpy()
    perm = np.argsort(order, kind="stable").astype(np.int64)
    return torch.from_numpy(cdf), torch.from_numpy(perm)


def make_columns(name, n, device="cpu", seed=None):
    """Seeded synthetic columns of config `name`, `n` rows, on `device`."""
    seed = SEEDS[name] if seed is None else seed
    g = lambda c, lo, hi: rng.uniform_int(seed, c, 0, n, lo, hi, device)
    f = lambda c, lo, hi: rng.uniform_f64(seed, c, 0, n, lo, hi, device)
    if name == "C1":
        return [rng.unit_f64(seed, 0, 0, n, device), rng.unit_f64(seed, 1, 0, n, device)]
    if name == "C2":
        return [f(0, 10.0, 100.0), f(1, 10.0, 100.0), f(2, 0.1, 2.0), f(3, 0.1, 0.5)]
    if name == "C3":
        return [g(0, 0, 2556).to(torch.int32),
                g(1, 0, 10).to(torch.float64) / 100.0,
                g(2, 1, 50).to(torch.float64),
                f(3, 900.0, 105000.0)]
    if name == "C4":
        return [g(0, 0, 2).to(torch.int8), g(1, 0, 1).to(torch.int8),
                g(2, 0, 2556).to(torch.int32),
                g(3, 1, 50).to(torch.float64), f(4, 900.0, 105000.0),
                g(5, 0, 10).to(torch.float64) / 100.0,
                g(6, 0, 8).to(torch.float64) / 100.0]
    if name == "C5":
        cdf, perm = _zipf_tables(seed)
        cdf, perm = cdf.to(device), perm.to(device)
        u = rng.unit_f64(seed, 0, 0, n, device)
        rank = torch.clamp(torch.searchsorted(cdf, u, right=True), max=perm.numel() - 1)
        key = perm[rank]
        hi = g(1, 0, 999)
        code = hi * 100_000 + key
        code = torch.where(code < 10_000, g(2, 1, 999) * 100_000 + key, code)
        kind = rng.unit_f64(seed, 3, 0, n, device)
        neg = -g(4, 1, 99_999_999)
        code = torch.where(kind < 0.05, torch.zeros_like(code), code)
        code = torch.where((kind >= 0.05) & (kind < 0.10), neg, code)
        return [code]
    raise KeyError(name)


def checksum(t):
    """Wrapping 64-bit sum of the raw bytes of a column (padded to 8 bytes)."""
    b = t.detach().cpu().contiguous().view(torch.uint8).numpy()
    pad = (-b.size) % 8
    if pad:
        b = np.concatenate([b, np.zeros(pad, np.uint8)])
    with np.errstate(over="ignore"):
        return int(b.view(np.uint64).sum(dtype=np.uint64))


EXAMPLES.update({"merge_5_6": example_merge_values, "map_plus_one": example_map_plus_one,
                 "zip_filter": example_zip_filter, "two_builders": example_two_builders})
