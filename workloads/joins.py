"""A hash join followed by a small group-by, shaped like TPC-H Q12 (the paper runs Q12 among its
TPC-H queries, Sec. 7.4; its tables are not available): `orders` is the build side, `lineitem`
the probe side.

    build : dict[orderkey -> {1 if the order's priority is urgent or high else 0}]
    probe : lineitem rows with shipmode in {MAIL, SHIP}, commitdate < receiptdate,
            shipdate < commitdate and receiptdate inside one year look their order up and count,
            per shipmode, the high-priority and the other orders' lines.

Synthetic columns with the table shapes of scale factor 10 (1.5e7 orders, 6e7 line items, one to
seven lines per order): plain data and seeded generators only, no arithmetic of the method.
"""
import torch

from . import rng
from .ir import Program

SEED = 7
ORDERS = 15_000_000
LINEITEMS = 60_000_000
YEAR_START, YEAR_END = 731, 1096          # receipt dates inside the second of seven years


def make_tables(n_orders=ORDERS, n_lines=LINEITEMS, device="cpu", seed=SEED):
    """orders: (orderkey i32, priority i8 in 0..4); lineitem: (orderkey i32, shipmode i8 in 0..6,
    commitdate, receiptdate, shipdate: i32 day numbers in 0..2556).  Order keys are the numbers
    0..n_orders-1 times 4 (sparse, like the benchmark's) in a seeded random order; a line's
    order is uniform over the orders."""
    g = lambda c, lo, hi, m: rng.uniform_int(seed, c, 0, m, lo, hi, device)
    perm = torch.argsort(rng.bits64(seed, 0, 0, n_orders, device))
    orderkey = (perm * 4).to(torch.int32)
    priority = g(1, 0, 4, n_orders).to(torch.int8)
    l_order = (g(2, 0, max(n_orders - 1, 0), n_lines) * 4).to(torch.int32)
    shipmode = g(3, 0, 6, n_lines).to(torch.int8)
    ship = g(4, 0, 2400, n_lines)
    commit = ship + g(5, -30, 60, n_lines)
    receipt = ship + g(6, 1, 30, n_lines)
    return ([orderkey, priority],
            [l_order, shipmode, commit.to(torch.int32), receipt.to(torch.int32), ship.to(torch.int32)])


def program_build(capacity=ORDERS):
    p = Program(["i32", "i8"])
    high = p.un("cast", p.bin("lt", p.col(1), p.const("i8", 2)), to="i64")
    p.merge(p.dictmerger(["i32"], ["i64"], "add", capacity), [high], keys=[p.col(0)])
    return p


def program_probe():
    p = Program(["i32", "i8", "i32", "i32", "i32"], dicts=[{"key_types": ["i32"], "val_types": ["i64"]}])
    okey, mode, commit, receipt, ship = [p.col(i) for i in range(5)]
    pred = p.bin("or", p.bin("eq", mode, p.const("i8", 2)), p.bin("eq", mode, p.const("i8", 5)))
    pred = p.bin("and", pred, p.bin("lt", commit, receipt))
    pred = p.bin("and", pred, p.bin("lt", ship, commit))
    pred = p.bin("and", pred, p.bin("ge", receipt, p.const("i32", YEAR_START)))
    pred = p.bin("and", pred, p.bin("lt", receipt, p.const("i32", YEAR_END)))
    high = p.dictlookup(0, 0, [okey])
    low = p.bin("sub", p.const("i64", 1), high)
    p.merge(p.dictmerger(["i8"], ["i64", "i64"], "add", 8), [high, low], keys=[mode], pred=pred)
    return p
