"""Shared comparison rules for the GPU parity tests (test infrastructure).

Tolerances:
  * integer, count, compaction-order and key-set outputs: bit-exact;
  * f64 merger / dictmerger sums: 1e-9 relative to the correctly rounded sum;
  * f64 min / max: bit-exact (order independent);
  * f64 map outputs (vecbuilder of f64): 1e-12 relative per element, with an
    absolute floor `map_floor` (0 unless a test states why it needs one).
"""
import numpy as np

from oracle import interp

SUM_RTOL = 1e-9
MAP_RTOL = 1e-12


def sorted_dict(res, idx):
    """A dictmerger result sorted by key (the library leaves the order of the entries unspecified)."""
    kcols, vcols = res.dict(idx)
    if len(kcols[0]):
        order = np.lexsort(tuple(reversed(kcols)))
        kcols = [k[order] for k in kcols]
        vcols = [v[order] for v in vcols]
    return kcols, vcols


def sorted_groups(res, idx):
    """A groupbuilder result with the groups ordered by key and the values of each group ascending
    (the library leaves both orders unspecified)."""
    kcols, offsets, values = res.groups(idx)
    ng = len(kcols[0])
    if ng:
        sizes = np.diff(offsets)
        gid = np.repeat(np.arange(ng), sizes)                     # group of every value, storage order
        rank = np.empty(ng, dtype=np.int64)
        order = np.lexsort(tuple(reversed(kcols)))
        rank[order] = np.arange(ng)                                # position of each group once sorted by key
        by = np.lexsort((values, rank[gid]))                       # by group (sorted), then by value
        values = values[by]
        kcols = [k[order] for k in kcols]
        offsets = np.concatenate([[0], np.cumsum(sizes[order])]).astype(np.int64)
    return kcols, offsets, values


def oracle_results(prog, cols_gpu, inits=None):
    host_inits = {b: t.cpu().numpy() for b, t in (inits or {}).items()}
    return interp.run(prog, [c.cpu().numpy() for c in cols_gpu], sums="exact", inits=host_inits)


def _close_sum(got, want, func):
    got, want = float(got), float(want)
    if func in ("min", "max"):
        return got == want
    return abs(got - want) <= SUM_RTOL * abs(want)


def assert_matches(prog, res, want, map_floor=0.0, label=""):
    res.check()
    for b, spec in enumerate(prog.builders):
        tag = "%s builder %d (%s)" % (label, b, spec["kind"])
        if spec["kind"] == "merger":
            got = res.merger(b)
            if spec["type"] == "f64":
                assert _close_sum(got, want[b], spec["func"]), (tag, got, want[b])
            else:
                assert int(got) == int(want[b]), (tag, got, want[b])
        elif spec["kind"] == "vecmerger":
            got = res.vec_host(b)
            assert len(got) == spec["length"], tag
            if spec["type"] == "f64" and spec["func"] in ("add", "mul"):
                # cells are sums in some order: relative to the cell, floored at the largest cell
                scale = np.maximum(np.abs(want[b]), np.max(np.abs(want[b])) if len(got) else 0.0)
                assert np.all(np.abs(got - want[b]) <= SUM_RTOL * scale), tag
            else:
                assert np.array_equal(got, want[b]), tag
        elif spec["kind"] == "groupbuilder":
            # groups and the values inside a group come back in no particular order: compare the
            # groups sorted by key and every group's values as a sorted list (values are moved,
            # never computed with: bit-exact)
            keys, offsets, values = sorted_groups(res, b)
            wkeys, woff, wvals = want[b]
            assert len(keys[0]) == len(wkeys[0]), (tag, len(keys[0]), len(wkeys[0]))
            for g, w in zip(keys, wkeys):
                assert np.array_equal(g, w), tag + " keys"
            assert np.array_equal(offsets, woff), tag + " group sizes"
            gid = np.repeat(np.arange(len(woff) - 1), np.diff(woff))
            wsorted = wvals[np.lexsort((wvals, gid))]
            assert np.array_equal(values.view(np.uint8), wsorted.view(np.uint8)), tag + " values"
        elif spec["kind"] == "vecbuilder":
            got = res.vec_host(b)
            assert len(got) == len(want[b]), (tag, len(got), len(want[b]))
            if spec["type"] == "f64":
                bound = MAP_RTOL * np.maximum(np.abs(want[b]), map_floor)
                bad = np.flatnonzero(~(np.abs(got - want[b]) <= bound))
                assert bad.size == 0, (tag, bad[:5], got[bad[:5]], want[b][bad[:5]])
            else:
                assert np.array_equal(got, want[b]), tag
        else:
            keys, vals = sorted_dict(res, b)
            wkeys, wvals = want[b]
            assert len(keys[0]) == len(wkeys[0]), (tag, len(keys[0]), len(wkeys[0]))
            for g, w in zip(keys, wkeys):
                assert np.array_equal(g, w), tag + " keys"
            for t, g, w in zip(spec["val_types"], vals, wvals):
                if t == "f64":
                    if spec["func"] in ("min", "max"):
                        assert np.array_equal(g, w), tag + " values"
                    else:
                        assert np.all(np.abs(g - w) <= SUM_RTOL * np.abs(w)), (tag, g, w)
                else:
                    assert np.array_equal(g, w), tag + " values"
