"""Host logic of the library, checked without a GPU: the work partition of the persistent shared-block kernel must
cover every (column, stage) position exactly once within the partial results it promises, for any level shape, CU
count and workspace; the suffix planner must respect its limits.  The walk below is the kernel's own rule (mode 0:
team t owns flattened positions [t*quota, (t+1)*quota), part index = team - floor(column * n_c / quota); mode 1: ranges
aligned to the columns), restated in Python."""
import itertools

import numpy as np
import pytest

from paper_2402_05099_amd import binding as hb


def walk(plan):
    """pieces[(column)] = list of (first stage, stages, part index, team) in the order the teams produce them"""
    n_c, ncols, quota = plan["n_c"], plan["ncols"], plan["quota"]
    total = ncols * n_c
    pieces = {}
    nteams = 8 * plan["tpx"]
    for team in range(nteams):
        if plan["mode"] == 2:
            f0, f1, sp = plan["starts"][team], plan["starts"][team + 1], plan["first_part"][team]
        elif plan["mode"] == 0:
            f0, f1 = team * quota, (team + 1) * quota
            sp = team - (f0 // n_c * n_c) // quota
        elif ncols <= nteams:
            c = team * ncols // nteams
            tf = -(-c * nteams // ncols)
            nt = -(-(c + 1) * nteams // ncols) - tf
            sp = team - tf
            f0, f1 = c * n_c + sp * n_c // nt, c * n_c + (sp + 1) * n_c // nt
        else:
            f0, f1 = team * ncols // nteams * n_c, (team + 1) * ncols // nteams * n_c
            sp = 0
        f0, f1 = min(f0, total), min(f1, total)
        c, k0 = divmod(f0, n_c) if f0 < f1 else (0, 0)
        while f0 < f1:
            ln = min(n_c - k0, f1 - f0)
            pieces.setdefault(c, []).append((k0, ln, sp, team))
            f0 += ln
            c += 1
            k0 = 0
            sp = 0          # a later piece of the same team starts its column
    return pieces


SHAPES = [
    # n_blocks, max_rows, max_seqs, Hkv, rows_per_seq
    (1, 16384, 1024, 40, 1), (1, 4096, 512, 8, 8), (1, 2048, 256, 40, 1), (16, 512, 128, 40, 1), (1, 1024, 2048, 40, 1),
    (1, 16384, 1024, 1, 8), (3, 77, 300, 2, 4), (1, 1, 129, 1, 1), (1, 33, 257, 3, 1), (5, 1000, 9000, 4, 2), (1, 31, 40000, 1, 1),
    (2, 100000, 130, 8, 1), (7, 65, 200, 5, 6),
]


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("slots", [1, 3, 4, 12, 20, 32])
@pytest.mark.parametrize("max_parts", [1, 2, 3, 24, 64])
@pytest.mark.parametrize("D", [128, 64])
def test_wide_plan_covers_every_stage_once(shape, slots, max_parts, D):
    n_blocks, max_rows, max_seqs, Hkv, rps = shape
    plan = hb.hg_debug_wide_plan(n_blocks, max_rows, max_seqs, Hkv, rps, max_parts, slots, D)
    assert plan is not None, "one part per row always fits"
    rows = max_seqs * rps
    mtiles = -(-rows // 256)
    assert plan["n_c"] == -(-max_rows // (32 if D == 128 else 64))      # a stage is 8 KiB of K at either head dimension
    assert plan["rowgroups"] * plan["T"] >= mtiles and (plan["rowgroups"] - 1) * plan["T"] < mtiles
    assert plan["T"] <= plan["slots"] == slots and plan["tpx"] == slots // plan["T"] >= 1
    assert plan["ncols"] == n_blocks * Hkv * plan["rowgroups"]
    assert 1 <= plan["nparts"] <= max_parts
    pieces = walk(plan)
    assert sorted(pieces) == list(range(plan["ncols"])), "every column is visited"
    for c, ps in pieces.items():
        ps.sort()
        assert ps[0][0] == 0 and sum(p[1] for p in ps) == plan["n_c"], "the pieces of a column tile its stages"
        for (k0, ln, _, _), (k1, _, _, _) in zip(ps, ps[1:]):
            assert k0 + ln == k1
        assert [p[2] for p in ps] == list(range(len(ps))), "part indices count the pieces of the column from 0"
        assert len(ps) <= plan["nparts"]
    # the teams that exist can take the whole space
    if plan["mode"] == 0:
        assert 8 * plan["tpx"] * plan["quota"] >= plan["ncols"] * plan["n_c"]


def test_wide_plan_aligns_short_pieces_to_columns():
    """Config 2's shape (40 columns of 64 stages on 256 teams): ranges of 10 stages would cut 32 teams' ranges at a
    column boundary (two pieces, each with its fixed price); aligned ranges give every team one piece of 9..11 stages."""
    plan = hb.hg_debug_wide_plan(1, 2048, 256, 40, 1, 24, 32)
    assert plan["mode"] == 1 and plan["nparts"] == 7
    pieces = walk(plan)
    per_team = {}
    for c, ps in pieces.items():
        for (k0, ln, sp, team) in ps:
            per_team.setdefault(team, []).append(ln)
    assert all(len(v) == 1 for v in per_team.values()) and len(per_team) == 256
    assert max(v[0] for v in per_team.values()) == 11 and min(v[0] for v in per_team.values()) == 9


def test_wide_plan_gives_ranges_of_equal_cost():
    """Config 3 at 16K keys (40 columns of 512 stages on 64 teams): equal ranges of 320 stages put a column boundary into
    every second team's range.  Ranges of equal cost, a boundary counting as nine stages: 325 stages without a boundary,
    316 with one (321 for a team that ends its column), every (column, stage) still covered once, three parts at most."""
    plan = hb.hg_debug_wide_plan(1, 16384, 1024, 40, 1, 24, 32)
    assert plan["mode"] == 2 and plan["nparts"] == 3 and plan["quota"] == 325
    starts = plan["starts"]
    assert starts[0] == 0 and starts[-1] == 40 * 512 and all(a <= b for a, b in zip(starts, starts[1:]))
    for t in range(64):
        f0, f1 = starts[t], starts[t + 1]
        inner = (f1 - 1) // 512 - f0 // 512
        assert inner <= 1 and (f1 - f0) + 9 * inner <= 325
        assert (f1 - f0) + 9 * inner >= 321                      # nobody is short of work either
    # when every team has a boundary (or none has) the equal ranges stay: config 5's root, config 4
    assert hb.hg_debug_wide_plan(1, 1024, 2048, 40, 1, 24, 32)["mode"] == 0
    assert hb.hg_debug_wide_plan(1, 4096, 512, 8, 8, 24, 32)["mode"] == 0


def test_wide_plan_rejects_what_it_cannot_run():
    assert hb.hg_debug_wide_plan(1, 0, 100, 1, 1, 4, 32) is None      # no keys
    assert hb.hg_debug_wide_plan(1, 100, 100, 1, 1, 0, 32) is None     # no room for a result
    assert hb.hg_debug_wide_plan(1, 100, 100, 1, 1, 4, 33) is None     # more CUs per XCD than there are
    assert hb.hg_debug_wide_plan(1, 100, 100, 1, 1, 4, 0) is None
    assert hb.hg_debug_wide_plan(1, 100, 100, 1, 1, 4, 32, 96) is None  # head dimensions other than 64 and 128


@pytest.mark.parametrize("B,nq,Hq,Hkv,D,max_len,ps", [
    (1024, 1, 40, 40, 128, 128, 0), (512, 1, 64, 8, 128, 512, 0), (512, 1, 64, 8, 128, 512, 16), (4, 1, 4, 4, 64, 16, 0),
    (1024, 4, 40, 40, 128, 128, 0), (2048, 1, 40, 40, 128, 64, 0), (3, 1, 8, 1, 128, 5000, 0), (256, 1, 40, 40, 128, 4096, 16),
    (1, 1, 1, 1, 64, 1, 0), (7, 6, 8, 2, 64, 300, 32), (512, 2, 16, 16, 128, 512, 0), (512, 1, 24, 8, 128, 100, 0),
    (512, 1, 16, 8, 128, 512, 0), (512, 1, 16, 8, 128, 128, 0), (512, 1, 16, 8, 128, 256, 16), (64, 1, 32, 32, 128, 383, 0),
    (64, 1, 32, 32, 128, 384, 0),
])
def test_suffix_plan_limits(B, nq, Hq, Hkv, D, max_len, ps):
    p = hb.hg_debug_suffix_plan(B, nq, Hq, Hkv, D, max_len, ps)
    assert p is not None
    assert p["chunk"] % 32 == 0 and p["chunk"] >= 32
    assert p["nchunks"] * p["chunk"] >= max_len and (p["nchunks"] - 1) * p["chunk"] < max(max_len, 1)
    G = Hq // Hkv
    several = nq >= 2 or G >= 3 or (G == 2 and max_len >= 256) or (D == 128 and max_len >= 384)   # ... or long rows to stream
    assert p["mfma"] == int(several), "matrix cores when a KV head serves several rows of a sequence"
    assert G % p["gt"] == 0 and p["gt"] in (1, 2, 4, 8)
    if ps and not p["mfma"]:
        assert p["chunk"] <= 32 * ps, "a vector-ALU work item covers at most 32 pages"


def test_suffix_plan_rejects_bad_arguments():
    assert hb.hg_debug_suffix_plan(4, 1, 6, 4, 128, 10) is None     # Hq not a multiple of Hkv
    assert hb.hg_debug_suffix_plan(4, 1, 4, 4, 96, 10) is None      # unsupported head dimension
    assert hb.hg_debug_suffix_plan(0, 1, 4, 4, 128, 10) is None
