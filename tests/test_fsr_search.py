"""Host logic of the selection loop (the paper's Algorithm 1 over tile configurations) with a scripted backend:
no GPU, no library calls."""
from paper_2506_09092_amd import fsr_search
from paper_2506_09092_amd.fsr_search import Candidate, Problem, neighbours, search


def scripted(latency, rejected=(), mismatch=()):
    calls = dict(runs=[], validates=[], latency=[])

    def runs(c):
        calls["runs"].append(c)
        return c not in rejected

    def validates(c):
        calls["validates"].append(c)
        return c not in mismatch

    def lat(c):
        calls["latency"].append(c)
        return latency(c)

    return runs, validates, lat, calls


def test_neighbours_stay_in_range():
    assert neighbours(Candidate(0, 1), 3) == [Candidate(1, 1), Candidate(0, 2)]
    assert neighbours(Candidate(2, 64), 3) == [Candidate(1, 64), Candidate(2, 32)]
    assert neighbours(Candidate(1, 4), 3) == [Candidate(2, 4), Candidate(0, 4), Candidate(1, 8), Candidate(1, 2)]
    assert neighbours(Candidate(1, 1), 4, max_slices=1) == [Candidate(2, 1), Candidate(0, 1)]


def test_neighbours_follow_a_chain_of_likeness():
    # bf16 candidate numbers are not in order of tile size: the chain is; a tile that is not on it falls back to +-1
    chain = fsr_search.TILE_CHAIN["bf16"]
    assert sorted(chain) == list(range(11))
    assert neighbours(Candidate(0, 1), 11, 1, chain) == [Candidate(5, 1), Candidate(1, 1)]       # 256 x 256: 192 x 256, general 256 x 256
    assert neighbours(Candidate(8, 1), 11, 1, chain) == [Candidate(6, 1), Candidate(7, 1)]       # 192 x 192: 128 x 256, 256 x 192
    assert neighbours(Candidate(4, 1), 11, 1, chain) == [Candidate(3, 1)] and neighbours(Candidate(1, 1), 11, 1, chain) == [Candidate(0, 1)]
    assert neighbours(Candidate(10, 1), 11, 1, chain) == [Candidate(2, 1), Candidate(9, 1)]     # direct-to-LDS 128 x 128: the general 128 x 128, 256 x 128
    assert neighbours(Candidate(2, 1), 3, 1, (5, 6)) == [Candidate(1, 1)]
    # the search reaches a minimum that plain numbering would need many rounds for: 0 -> 5 -> 7
    lat = lambda c: {7: 1.0, 5: 2.0, 0: 3.0}.get(c.tile, 9.0)
    runs, validates, latency, _ = scripted(lat)
    assert search(Candidate(0, 1), 11, runs, validates, latency, rounds=3, per_round=4, max_slices=1, chain=chain)["best"] == Candidate(7, 1)


def test_walks_downhill_to_the_minimum():
    # latency has one minimum at tile 2, 8 slices; the start is three refinement steps away
    lat = lambda c: abs(c.tile - 2) + abs(c.slices.bit_length() - 4)
    runs, validates, latency, calls = scripted(lat)
    r = search(Candidate(1, 1), 3, runs, validates, latency, rounds=4, per_round=4)
    assert r["best"] == Candidate(2, 8) and r["best_latency"] == 0
    assert len(r["rounds"]) == 4 and all(len(x["candidates"]) <= 4 for x in r["rounds"])
    assert len(set(calls["runs"])) == len(calls["runs"])                 # no candidate is tried twice
    # every round's winner is the fastest of its valid candidates
    for x in r["rounds"]:
        assert x["latency"][x["winner"]] == min(x["latency"].values())


def test_invalid_candidates_are_never_timed_and_never_win():
    lat = lambda c: 10 - c.tile           # the fastest tiles are the ones that fail
    runs, validates, latency, calls = scripted(lat, rejected={Candidate(3, 1)}, mismatch={Candidate(2, 1)})
    r = search(Candidate(1, 1), 4, runs, validates, latency, rounds=3, per_round=4, max_slices=1)
    assert r["best"] == Candidate(1, 1)
    assert r["visited"][Candidate(2, 1)] == "mismatch" and r["visited"].get(Candidate(3, 1), "rejected") == "rejected"
    assert Candidate(2, 1) not in calls["latency"] and Candidate(3, 1) not in calls["latency"]
    assert Candidate(3, 1) not in calls["validates"]                     # validation only for candidates that run


def test_a_round_without_valid_candidates_does_not_count():
    # the start and its neighbours all fail; the loop proposes their neighbours and still delivers `rounds` rounds
    bad = {Candidate(1, 1), Candidate(2, 1), Candidate(0, 1), Candidate(1, 2)}
    runs, validates, latency, calls = scripted(lambda c: c.slices + c.tile, rejected=bad)
    r = search(Candidate(1, 1), 3, runs, validates, latency, rounds=2, per_round=4)
    assert r["rounds"][0]["valid"] == [] and r["rounds"][0]["winner"] is None
    counted = [x for x in r["rounds"] if x["winner"] is not None]
    assert len(counted) == 2
    assert r["best"] is not None and r["best"] not in bad
    assert r["best_latency"] == min(latency for x in counted for latency in x["latency"].values())


def test_the_incumbent_survives_slower_rounds():
    # the start is the global minimum: later rounds only find slower candidates
    lat = lambda c: 0.0 if c == Candidate(1, 1) else 5.0 + c.tile + c.slices
    runs, validates, latency, _ = scripted(lat)
    r = search(Candidate(1, 1), 3, runs, validates, latency, rounds=3, per_round=2)
    assert r["best"] == Candidate(1, 1) and r["best_latency"] == 0.0
    assert r["rounds"][1]["winner"] != Candidate(1, 1)


def test_ends_when_the_space_is_exhausted():
    runs, validates, latency, calls = scripted(lambda c: 1.0)
    r = search(Candidate(0, 1), 2, runs, validates, latency, rounds=50, per_round=4, max_slices=2)
    assert set(r["visited"]) == {Candidate(t, s) for t in (0, 1) for s in (1, 2)}
    assert len(r["rounds"]) < 50


def test_ties_are_broken_deterministically():
    runs, validates, latency, _ = scripted(lambda c: 1.0)
    a = search(Candidate(1, 2), 3, runs, validates, latency)
    b = search(Candidate(1, 2), 3, runs, validates, latency)
    assert a["best"] == b["best"] == min(a["rounds"][0]["valid"])


def test_table_row_format():
    assert fsr_search.table_row(Problem("bf16", 0, 1, 2048, 2048, 2048), False, Candidate(2, 1)) == \
        "    {1, 0, 1, 2048, 2048, 2048, 0, 2, 1},"
    assert fsr_search.table_row(Problem("f32", 1, 0, 1, 4096, 4096), True, Candidate(2, 16)).startswith("    {0, 1, 0, 1, 4096, 4096, 1, 2, 16}")
