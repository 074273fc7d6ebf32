"""The failure-schedule generator/consumer: a pure function of its arguments, YAML round trip,
location weights, and schedules consumed by the CPU oracle keep Eq. 1.  CPU only."""
import numpy as np

from oracle.proto import Proto
from paper_2605_11215_amd import schedule
from tests.driver import run_iteration, view_oracle


def test_schedule_is_a_pure_function_of_its_arguments():
    a = schedule.generate(16, 8, 3, 40, (5, 60), {"mb": 1, "sync": 3}, max_microbatch=8)
    b = schedule.generate(16, 8, 3, 40, (5, 60), {"mb": 1, "sync": 3}, max_microbatch=8)
    assert a == b and len(a) == 40
    assert a != schedule.generate(16, 8, 4, 40, (5, 60), {"mb": 1, "sync": 3}, max_microbatch=8)
    assert all(5 <= e["step"] <= 60 and 0 <= e["replica"] < 16 and 0 <= e["local_rank"] < 8 for e in a)
    assert [e["step"] for e in a] == sorted(e["step"] for e in a)
    assert schedule.generate(16, 8, 3, 10, (5, 60))[:0] == []
    # a longer schedule extends a shorter one (entry i depends on i only)
    short = schedule.generate(16, 8, 3, 10, (5, 60), {"mb": 1, "sync": 3})
    assert all(e in a for e in short)


def test_yaml_round_trip():
    a = schedule.generate(64, 8, 11, 25, (0, 99), {"mb": 1, "sync": 1})
    text = schedule.to_yaml(a)
    assert "failures:" in text and schedule.from_yaml(text) == a
    assert schedule.from_yaml("") == []


def test_location_weights():
    a = schedule.generate(8, 1, 5, 4000, (0, 9), {"mb": 1, "sync": 3}, max_microbatch=4)
    mb = [e for e in a if e["location"].startswith("mb:")]
    assert abs(len(mb) / 4000 - 0.25) < 0.03
    assert {int(e["location"][3:]) for e in mb} == {0, 1, 2, 3, 4}
    assert all(0 <= int(e["location"][5:]) <= 100 for e in a if e["location"].startswith("sync:"))
    reps = np.bincount([e["replica"] for e in a], minlength=8)
    assert reps.min() > 400                                       # every replica is hit about equally
    assert all(e["location"].startswith("sync:") for e in schedule.generate(8, 1, 5, 50, (0, 9)))


def test_consumed_schedule_keeps_eq1_on_the_oracle():
    W, G, off = 12, 3, [0, 5, 9, 40]
    entries = schedule.generate(W, 4, 2, 14, (0, 9), {"mb": 1, "sync": 1}, max_microbatch=G)
    o = Proto(W, G, off, dtype=np.float64)
    o.set_state(np.zeros(off[-1], np.float32))
    g = lambda t, mb: np.full(off[-1], 0.25, np.float32)
    lost = 0
    for t in range(10):
        v = view_oracle(o)
        dying, fid = schedule.for_step(entries, t, v["alive"], v["target"], 3)
        assert len(dying) < len(v["alive"]) and 0 <= fid <= 3
        out = run_iteration(o, view_oracle, t, g, W, dying=dying, fidelity_k=fid)
        assert sum(len(x) for x in out["ids"].values()) == W * G
        assert np.all(o.grad_out == 0.25)
        lost += len(dying)
    assert lost >= 5 and len(o.world.alive()) == W - lost
