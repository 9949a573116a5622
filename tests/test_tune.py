"""The schedule game's host logic (no GPU): moves, reward, greedy play on synthetic timers."""
import math

import pytest

from paper_2501_08071_amd import tune


def test_grid_and_moves():
    states = tune.all_states()
    assert len(states) == len(set(states)) == 31
    assert tune.START in states and tune.SHIPPED in states and all(tune.valid(s) for s in states)
    for s in states:
        for n in tune.neighbours(s):
            assert n in states and sum(a != b for a, b in zip(s, n)) == 1      # one knob, one step
            assert s in tune.neighbours(n)                                      # every move can be taken back
    # (0,2,2,4,32) is not valid (two blocks between barriers need eight buffers), nor is (0,1,2,4,64) (blocks of
    # 64 keys exist in the alternating-phase loop only)
    assert set(tune.neighbours(tune.START)) == {(1, 1, 2, 4, 32, 4, 0), (0, 1, 4, 4, 32, 4, 0), (0, 1, 2, 8, 32, 4, 0)}
    assert set(tune.neighbours((1, 1, 2, 8, 32, 4, 0))) == {(0, 1, 2, 8, 32, 4, 0), (1, 2, 2, 8, 32, 4, 0), (1, 1, 4, 8, 32, 4, 0),
                                                            (1, 1, 2, 4, 32, 4, 0), (1, 1, 2, 8, 64, 4, 0)}
    # the 64-row kernel is one move away from the shipped schedule and from nowhere else; the deeper read-ahead is a move of
    # the alternating-phase loop with 64-key blocks only
    assert tune.SHIPPED[:-1] + (1,) in tune.neighbours(tune.SHIPPED)
    assert [s for s in states if s[-1] == 1] == [tune.SHIPPED[:-1] + (1,)]
    assert all(s[0] == 1 and s[4] == 64 for s in states if s[5] == 8)
    assert tune.state_flags(tune.SHIPPED) == ["-DATTN_PINGPONG=1", "-DATTN_BARRIER_EVERY=2", "-DATTN_FETCH=4", "-DATTN_NBUF=8",
                                              "-DATTN_PP_KEYS=64", "-DATTN_PP_FETCH=4", "-DATTN_ROWS64=0"]


def test_the_shipped_state_is_the_one_the_headers_default_to():
    import os
    import re
    text = open(os.path.join(os.path.dirname(tune.HERE), "paper_2501_08071_amd", "csrc", "attn_launch.h")).read()
    for (macro, _), value in zip(tune.KNOBS.values(), tune.SHIPPED):
        m = re.search(rf"#ifndef {macro}\n#define {macro} (\d+)", text)
        assert m and int(m.group(1)) == value, macro


def test_reward_is_the_papers():
    # Section 3.6: R = (T_prev - T) / T_0 * 100; rewards of a trajectory add up to the total gain in percent of T_0
    assert tune.reward(2.0, 1.5, 4.0) == pytest.approx(12.5)
    ts = [4.0, 3.0, 2.9, 2.0]
    assert sum(tune.reward(a, b, ts[0]) for a, b in zip(ts, ts[1:])) == pytest.approx((ts[0] - ts[-1]) / ts[0] * 100)


def _separable(s):
    d = dict(zip(tune.KNOBS, s))
    return 1.0 - 0.2 * d["pingpong"] - 0.05 * (d["fetch"] == 4) - 0.1 * (d["nbuf"] == 8) - 0.02 * (d["barrier_every"] == 2)


def test_greedy_play_takes_the_biggest_gain_first_and_stops_at_the_noise():
    calls = []

    def timer(s):
        calls.append(s)
        return _separable(s)

    r = tune.play_game(timer)
    tail = "_prefetch4_rows640"
    assert [m["to"] for m in r["moves"]] == ["pingpong1_barrier_every1_fetch2_nbuf4_block32" + tail, "pingpong1_barrier_every1_fetch2_nbuf8_block32" + tail,
                                             "pingpong1_barrier_every1_fetch4_nbuf8_block32" + tail,
                                             "pingpong1_barrier_every2_fetch4_nbuf8_block32" + tail]
    assert [round(m["reward"], 6) for m in r["moves"]] == [20.0, 10.0, 5.0, 2.0]
    assert r["total_reward"] == pytest.approx(37.0) and r["speedup"] == pytest.approx(1 / 0.63)
    assert len(calls) == len(set(calls))                # no schedule is measured twice
    # with a noise floor above the smallest gain the last move is not taken
    r2 = tune.play_game(_separable, noise_pct=3.0)
    assert r2["final"] == "pingpong1_barrier_every1_fetch4_nbuf8_block32" + tail
    # deterministic: same timer, same trajectory
    assert tune.play_game(_separable)["moves"] == r["moves"]


def test_a_schedule_that_fails_its_check_is_never_entered():
    def timer(s):
        return math.inf if dict(zip(tune.KNOBS, s))["pingpong"] == 1 else _separable(s)

    r = tune.play_game(timer)
    assert "pingpong1" not in r["final"] and all("pingpong1" not in m["to"] for m in r["moves"])
    with pytest.raises(RuntimeError):
        tune.play_game(lambda s: math.inf)


def test_local_optimum_ends_the_game():
    # a timer whose only improvement needs two knobs at once: greedy single moves cannot reach it
    def timer(s):
        d = dict(zip(tune.KNOBS, s))
        return 0.5 if (d["pingpong"] == 1 and d["nbuf"] == 8) else 1.0 + 0.01 * (d["pingpong"] + (d["nbuf"] == 8))

    r = tune.play_game(timer)
    assert r["moves"] == [] and r["final"] == tune.state_name(tune.START)
