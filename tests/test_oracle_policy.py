"""Pins for oracle/policy.py: the paper's printed example, Eq. 1 on sweeps, minimality by
counting, the strawman as negative control.  CPU only."""
import itertools
import os

import pytest

from oracle import policy as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "walkthrough_w32_g8.txt")


def load_golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        k, v = [x.strip() for x in line.split("=")]
        out[k] = int(v) if v.lstrip("-").isdigit() else v
    return out


def at_sync(w):
    """Every survivor has finished its quota: the state in which the paper detects failures."""
    for r in w.alive():
        w.contributed[r] = w.target[r]


def eq1(w):
    return sum(w.target[r] for r in w.contributors())


def test_walkthrough_example_printed_by_the_paper():
    g = load_golden()
    w = P.World(g["W_init"], g["G_init"])
    assert w.B == g["B"]
    at_sync(w)
    d = w.on_failure([g["failed_first"] - 1])
    assert d["W_cur"] == g["W_cur_after_first"]
    assert d["C_cur"] == g["C_cur"]
    assert d["at_boundary"] == g["at_boundary"]
    assert d["G_ext"] == g["G_ext"] and d["n_bdry"] == g["n_bdry"] == d["n_bm"]
    assert d["loop_bound"] == g["loop_bound_after"]
    assert d["restore_mode"] == P.RESTORE_NONBLOCKING
    alive_t = [d["target"][r] for r in w.alive()]
    assert alive_t.count(g["quota_major_extended"]) == g["majors_extended"] == d["n_maj"]
    assert alive_t.count(g["quota_boundary_minor"]) == g["n_bdry"]
    assert sum(alive_t) == g["B"]
    assert d["epoch"] == 1
    at_sync(w)
    w.commit()
    d = w.advance()
    for k in ("G_cur", "n_maj", "R_cur", "n_min", "n_ms", "n_mi"):
        assert d[k] == g[k], k
    assert d["role"][g["minor_is"] - 1] == P.MINOR
    assert d["role"][g["minor_spare_is"] - 1] == P.MINOR_SPARE
    assert d["role"][:28] == [P.MAJOR] * 28 and d["role"][29] == P.MAJOR_SPARE
    assert d["n_maj"] * d["G_cur"] + d["n_min"] * d["R_cur"] == g["B"]
    at_sync(w)
    d = w.on_failure([g["failed_second"] - 1])
    assert d["at_boundary"] == g["at_boundary_second"]
    assert d["role"][g["promoted_second"] - 1] == P.MINOR
    assert d["restore_mode"] == P.RESTORE_BLOCKING
    assert d["loop_bound"] == g["loop_bound_second"]
    assert d["epoch"] == 2 and d["C_cur"] == g["B"] and eq1(w) == g["B"]


def test_advancement_matches_its_definition():
    for W in range(1, 40):
        for B in (W, 2 * W, 7 * W, 8 * W + 3, 256):
            if B >= W:
                check_advancement(W, B)


def check_advancement(W, B):
    lay = P.policy_advancement(W, B)
    G = lay["G_cur"]
    assert W * G >= B and (G == 1 or W * (G - 1) < B)            # smallest such G
    assert G == -(-B // W)
    assert lay["n_maj"] == B // G and lay["R_cur"] == B - lay["n_maj"] * G
    assert 0 <= lay["R_cur"] < G
    assert lay["n_min"] == (1 if lay["R_cur"] else 0)
    spare = W - lay["n_maj"] - lay["n_min"]
    assert spare >= 0 and lay["n_ms"] + lay["n_mi"] == spare
    assert lay["n_mi"] == (1 if lay["n_min"] == 1 and spare >= 2 else 0)
    assert lay["n_maj"] * G + lay["n_min"] * lay["R_cur"] == B   # Eq. 1 in the steady state
    if lay["R_cur"] == 0:                                        # main-text wording of the rule
        assert lay["n_mi"] == 0 and lay["n_ms"] == W - lay["n_maj"]


def test_boundary_extension_matches_its_definition():
    for B in (8, 31, 256):
        for W in range(1, 12):
            for C in range(0, B):
                check_extension(C, W, B)


def check_extension(C, W, B):
    G_ext, n_bdry = P.boundary_extension(C, W, B)
    assert G_ext >= 1 and C + W * G_ext >= B
    assert G_ext == 1 or C + W * (G_ext - 1) < B
    assert G_ext == max(1, -(-(B - C) // W))
    assert 0 <= n_bdry < W
    assert C + (W - n_bdry) * G_ext + n_bdry * (G_ext - 1) == B


def run_attrition(W, G, schedule, check):
    """schedule: list of failure sets (indices into the current alive list), one per iteration."""
    w = P.World(W, G)
    for picks in schedule:
        at_sync(w)
        assert sum(w.contributed[r] for r in w.contributors()) == w.B
        alive = w.alive()
        failed = sorted({alive[k % len(alive)] for k in picks})
        if len(failed) == len(alive):
            with pytest.raises(P.NoSurvivor):
                w.on_failure(failed)
            return
        if failed:
            d = w.on_failure(failed)
            check(w, d)
            assert eq1(w) == w.B                                  # quotas sum to B again
            assert all(w.role[r] == P.DEAD for r in failed)
            if d["at_boundary"]:
                assert d["restore_mode"] == P.RESTORE_NONBLOCKING and d["G_ext"] >= 1
            else:
                assert d["restore_mode"] == P.RESTORE_BLOCKING and d["G_ext"] == 0
            at_sync(w)
            assert w.C_cur() == w.B
        w.commit()
        d = w.advance()
        assert eq1(w) == w.B
        assert all(w.target[r] == w.quota_of_role(w.role[r]) for r in w.alive())


def test_eq1_exhaustive_small_worlds():
    """Every (W <= 6, G <= 3), every sequence of up to three failure sets of size <= 2."""
    n = 0
    for W in range(1, 7):
        for G in range(1, 4):
            sets = [()] + [(a,) for a in range(W)] + list(itertools.combinations(range(W), 2))
            for seq in itertools.product(sets, repeat=3):
                run_attrition(W, G, seq, lambda w, d: None)
                n += 1
    assert n > 1000


def test_eq1_heavy_attrition_64_replicas():
    seq = [(2 * t, 2 * t + 1) for t in range(16)]
    seen = {"boundary": 0, "promotion": 0}

    def check(w, d):
        seen["boundary" if d["at_boundary"] else "promotion"] += 1

    w = P.World(64, 2)
    for t in range(16):
        at_sync(w)
        alive = w.alive()
        d = w.on_failure(alive[:2])
        check(w, d)
        assert eq1(w) == 128
        at_sync(w)
        w.commit()
        w.advance()
        assert eq1(w) == 128
    assert len(w.alive()) == 32
    assert seen["boundary"] >= 1 and seen["promotion"] >= 1
    assert w.G_cur == 4 and all(w.role[r] == P.MAJOR for r in w.alive())


def test_promotion_needs_a_spare_of_the_same_role():
    w = P.World(32, 8)
    at_sync(w)
    w.on_failure([31])
    at_sync(w)
    w.commit()
    w.advance()                      # 28 majors, minor r28, major-spare r29, minor-spare r30
    at_sync(w)
    d = w.on_failure([0])            # a major fails: the major-spare takes over
    assert not d["at_boundary"] and d["role"][29] == P.MAJOR and d["n_ms"] == 0
    at_sync(w)
    d = w.on_failure([1])            # next major: only a minor-spare is left -> boundary
    assert d["at_boundary"] and d["role"][30] == P.MINOR_SPARE
    assert eq1(w) == 256
    assert 30 not in w.contributors()            # the spare stays masked at a boundary


def test_spare_stays_masked_when_the_minor_fails_without_a_minor_spare():
    """B = 256 with 30 survivors: 28 majors @9, one minor @4, one spare (a major-spare).
    Losing the minor is a boundary; admitting the spare's 9 microbatches would overshoot."""
    w = P.World(32, 8)
    at_sync(w)
    w.on_failure([30, 31])
    at_sync(w)
    w.commit()
    d = w.advance()
    assert (d["G_cur"], d["n_maj"], d["R_cur"], d["n_ms"], d["n_mi"]) == (9, 28, 4, 1, 0)
    at_sync(w)
    d = w.on_failure([28])
    assert d["at_boundary"] and d["C_cur"] == 252
    assert d["G_ext"] == 1 and d["n_bdry"] == 24
    assert eq1(w) == 256


def test_lost_spare_changes_nothing_but_the_epoch():
    w = P.World(32, 8)
    at_sync(w)
    w.on_failure([31])
    at_sync(w)
    w.commit()
    w.advance()
    before = list(w.target)
    at_sync(w)
    d = w.on_failure([29])           # the major-spare
    assert not d["at_boundary"] and d["epoch"] == 2 and d["restore_mode"] == P.RESTORE_BLOCKING
    before[29] = before[29]
    assert [w.target[r] for r in w.alive()] == [before[r] for r in w.alive()]


def test_no_survivor():
    w = P.World(3, 2)
    with pytest.raises(P.NoSurvivor):
        w.on_failure([0, 1, 2])


def test_adaptive_strawman_shrinks_the_batch():
    """Alg. 8: never a boundary, blocking restore, the committed count drops below B."""
    w = P.World(8, 4, static=False)
    at_sync(w)
    d = w.on_failure([3])
    assert not d["at_boundary"] and d["restore_mode"] == P.RESTORE_BLOCKING
    assert d["loop_bound"] == 4
    assert w.C_cur() == 28 < w.B
    w.commit()
    w.advance()
    assert w.G_cur == 4 and eq1(w) == 28
