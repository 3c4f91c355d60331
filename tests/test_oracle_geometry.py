"""Pins for oracle/geometry.py: the worked examples of App. B.1, the App. C
parameter table, and the check values of the benchmark configurations."""
import os

import pytest

from oracle import geometry as geo
from oracle import layers

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_examples():
    examples, cur = {}, None
    for line in open(os.path.join(GOLDEN, "halo_examples.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        tok = line.split()
        if tok[0] == "example":
            cur = dict(workers=[])
            examples[tok[1]] = cur
        elif tok[0] == "params":
            cur["params"] = {k: int(v) for k, v in (t.split("=") for t in tok[1:])}
        else:
            ins, outs = line.split("|")
            cur["workers"].append((ins.split()[2:], [int(t) for t in outs.split()[1:]]))
    return examples


EXAMPLES = _read_examples()


@pytest.mark.parametrize("name", sorted(EXAMPLES))
def test_worked_examples_buffers_and_outputs(name):
    ex = EXAMPLES[name]
    p = ex["params"]
    ws = geo.dim_geometry(p["n"], p["k"], p["s"], p["p"], p["dil"], p["P"])
    assert len(ws) == len(ex["workers"])
    for g, (drawn_in, drawn_out) in zip(ws, ex["workers"]):
        first = g["in_start"] - g["halo"][0] - g["pad"][0]
        cells = []
        for c in range(g["buf"]):
            gi = first + c
            cells.append("-" if gi < 0 or gi >= p["n"] else str(gi))
        assert cells == drawn_in
        roots = [j * p["s"] - p["p"] + ((p["k"] - 1) // 2) * p["dil"]
                 for j in range(g["out_start"], g["out_start"] + g["out_size"])]
        assert roots == drawn_out


def test_prose_halo_widths():
    for line in open(os.path.join(GOLDEN, "halo_widths.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        name, w, hl, hr, el, er = line.split()
        p = EXAMPLES[name]["params"]
        g = geo.dim_geometry(p["n"], p["k"], p["s"], p["p"], p["dil"], p["P"])[int(w)]
        assert g["halo"] == (int(hl), int(hr))
        assert g["extra"] == (int(el), int(er))


def test_unbalanced_conv_output_length_and_split():
    # App. B.1 second example: m = 7, split 3,2,2; fourth example 20 -> 4,4,3,3,3,3
    assert geo.output_length(11, 5, 1, 0, 1) == 7
    assert [z for _, z in geo.balanced_split(7, 3)] == [3, 2, 2]
    assert [z for _, z in geo.balanced_split(20, 6)] == [4, 4, 3, 3, 3, 3]
    assert [z for _, z in geo.balanced_split(10, 6)] == [2, 2, 2, 2, 1, 1]


def test_lenet_table_shapes():
    """App. C table: 2x2 weight partitions of 120x400, 84x120, 10x84; bias on
    workers 0 and 2 (column j = 0 of the row-major P_fo x P_fi grid)."""
    full = dict(C5=(120, 400), F6=(84, 120), OUT=(10, 84))
    for line in open(os.path.join(GOLDEN, "lenet_param_shapes.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        layer, kind, worker, wshape, bshape = line.split()
        worker = int(worker)
        if kind == "conv":
            # learnable conv parameters live on one worker only (P_r = 1 x 1)
            assert (wshape == "none") == (worker != 0)
            continue
        n_fo, n_fi = full[layer]
        i, j = divmod(worker, 2)                       # row-major P_fo x P_fi
        rows = layers.feature_blocks(n_fo, 2)[i]
        cols = layers.feature_blocks(n_fi, 2)[j]
        shape = (rows.stop - rows.start, cols.stop - cols.start)
        assert shape == tuple(int(t) for t in wshape.split(","))
        has_bias = (j == 0)
        assert (bshape != "none") == has_bias
        if has_bias:
            assert int(bshape) == shape[0]


CONFIG_DIMS = [
    # (n,k,s,p,P), m, per worker (padL, haloL, extraL, extraR, haloR, padR), bulk sizes, buf sizes
    ((64, 3, 1, 1, 4), 64, [(1, 0, 0, 0, 1, 0), (0, 1, 0, 0, 1, 0), (0, 1, 0, 0, 1, 0), (0, 1, 0, 0, 0, 1)],
     [16] * 4, [18] * 4),
    ((256, 3, 1, 1, 2), 256, [(1, 0, 0, 0, 1, 0), (0, 1, 0, 0, 0, 1)], [128] * 2, [130] * 2),
    ((28, 5, 1, 2, 2), 28, [(2, 0, 0, 0, 2, 0), (0, 2, 0, 0, 0, 2)], [14] * 2, [18] * 2),
    ((28, 2, 2, 0, 2), 14, [(0, 0, 0, 0, 0, 0)] * 2, [14] * 2, [14] * 2),
    ((14, 5, 1, 0, 2), 10, [(0, 0, 0, 0, 2, 0), (0, 2, 0, 0, 0, 0)], [7] * 2, [9] * 2),
    ((10, 2, 2, 0, 2), 5, [(0, 0, 0, 0, 1, 0), (0, 0, 1, 0, 0, 0)], [5] * 2, [6, 5]),
    ((256, 5, 2, 2, 4), 128, [(2, 0, 0, 0, 1, 0), (0, 2, 0, 0, 1, 0), (0, 2, 0, 0, 1, 0), (0, 2, 0, 0, 0, 1)],
     [64] * 4, [67] * 4),
    ((250, 5, 2, 2, 4), 125, [(2, 0, 0, 0, 2, 0), (0, 1, 0, 0, 1, 0), (0, 2, 0, 0, 1, 0), (0, 2, 0, 0, 0, 1)],
     [63, 63, 62, 62], [67, 65, 65, 65]),
]


@pytest.mark.parametrize("params,m,widths,bulks,bufs", CONFIG_DIMS)
def test_config_geometry(params, m, widths, bulks, bufs):
    n, k, s, p, P = params
    assert geo.output_length(n, k, s, p, 1) == m
    ws = geo.dim_geometry(n, k, s, p, 1, P)
    got = [(g["pad"][0], g["halo"][0], g["extra"][0], g["extra"][1], g["halo"][1], g["pad"][1]) for g in ws]
    assert got == widths
    assert [g["in_size"] for g in ws] == bulks
    assert [g["buf"] for g in ws] == bufs
    for g in ws:
        assert g["origin"] == g["extra"][0]


def test_needed_range_is_exactly_covered():
    """Brute force: for random parameters the buffer of every worker covers
    exactly the taps its outputs read, plus its own extra cells."""
    import random
    rnd = random.Random(0)
    done = 0
    while done < 300:
        P = rnd.randint(1, 5)
        k, s, dil = rnd.randint(1, 5), rnd.randint(1, 3), rnd.randint(1, 2)
        p = rnd.randint(0, 3)
        n = rnd.randint(P * 4, P * 12)
        try:
            ws = geo.dim_geometry(n, k, s, p, dil, P)
        except ValueError:
            continue
        done += 1
        covered_out = []
        for g in ws:
            first = g["in_start"] - g["halo"][0] - g["pad"][0]
            taps = set()
            for j in range(g["out_start"], g["out_start"] + g["out_size"]):
                covered_out.append(j)
                for t in range(k):
                    gi = j * s - p + t * dil
                    taps.add(gi)
                    c = g["origin"] + (j - g["out_start"]) * s + t * dil
                    assert first + c == gi and 0 <= c < g["buf"]
            owned = set(range(g["in_start"], g["in_start"] + g["in_size"]))
            assert min(taps | owned) == first
            assert max(taps | owned) == first + g["buf"] - 1
        assert covered_out == list(range(geo.output_length(n, k, s, p, dil)))


def test_errors():
    with pytest.raises(geo.EmptyPartition):
        geo.dim_geometry(3, 1, 1, 0, 1, 4)
    with pytest.raises(geo.HaloTooWide):
        geo.dim_geometry(8, 7, 1, 3, 1, 4)     # halo 3 > neighbour bulk 2
    with pytest.raises(geo.HaloTooWide):
        geo.explicit_dim_geometry([2, 5], [(0, 0), (3, 0)])


def test_row_major_worker_numbering():
    part = geo.Partition.explicit([[5, 6], [7, 4]], [[(0, 2), (4, 0)], [(0, 0), (3, 0)]])
    assert part.neighbour(0, 0, 1) == 2 and part.neighbour(0, 1, 1) == 1
    assert part.neighbour(3, 0, 0) == 1 and part.neighbour(3, 1, 0) == 2
    assert part.neighbour(0, 0, 0) is None
    assert [part.coords(w) for w in range(4)] == [(0, 0), (0, 1), (1, 0), (1, 1)]
