"""CPU model of how the four waves of a block agree, without meeting, on the tile after which
they flush the parked aggregate at a common instant (csrc/stream_pass.h, "When to flush").

The kernel's rules, restated as small state machines whose every access to the two shared LDS
words is one atomic step:

  wave 0, at the flush point of tile t:
      if it has no announcement pending and the clock has passed the next instant:
          announce "flush after tile t + 2"          (store flush_after)
      publish progress = t + 1                        (store, after the announcement)
      flush now if t is the announced tile (or the staging is full, or the piece ends)
  any other wave, at the flush point of tile t:
      wait until progress >= t - 1                    (wave 0 has been through tile t - 2)
      flush now if flush_after == t (or full, or end)
  a flush is: barrier, stores, barrier; after an on-time flush wave 0 forgets its announcement

The model explores every interleaving of the waves' steps and every choice of the tiles at which
the clock fires (exhaustively for three waves and for four on a short piece, randomly for four
on a long one) and checks that whenever the
block's barrier releases, all waves stand at the same barrier of the same tile with the same
number of parked tiles, and that no reachable state is stuck.  Planted mistakes (a gate one tile
too lax, an announcement one tile too early, the progress published before the announcement)
must each be caught.
"""
import random

import pytest

NEVER = 10 ** 9


class Rules:
    """The protocol's constants; tests plant mistakes by changing them."""
    gate_lag = 1            # other waves wait for progress >= t - gate_lag
    announce_ahead = 2      # wave 0 announces the flush for tile t + announce_ahead
    progress_first = False  # True: progress is published before the announcement (wrong order)


def initial(nwaves):
    # per wave: (tile, pc, parked tiles, pending announcement or, for the other waves, the tile
    # they saw announced); shared: progress, flush_after, waves parked at the barrier
    waves = tuple((0, "tile", 0, NEVER) for _ in range(nwaves))
    return (waves, 0, NEVER, 0)


def wave0_order(rules):
    """The pcs wave 0 goes through at a flush point."""
    return ("publish", "clock", "decide") if rules.progress_first else ("clock", "publish", "decide")


def steps(state, tiles, capacity, rules, fires_left):
    """All successors (new_state, fires_left) of a state: one per wave that can move, two for wave
    0's clock read when the clock may fire.  Raises AssertionError when the barrier releases waves
    that do not stand at the same place."""
    waves, progress, flush_after, parked = state
    n = len(waves)
    order0 = wave0_order(rules)
    out = []

    def put(i, w, progress=progress, flush_after=flush_after, parked=parked, fires=fires_left):
        out.append(((waves[:i] + (w,) + waves[i + 1:], progress, flush_after, parked), fires))

    for i, (t, pc, staged, ann) in enumerate(waves):
        more = t + 1 < tiles
        if pc == "tile":                      # pass 1 of tile t is done and G is parked
            put(i, (t, order0[0] if i == 0 else "gate", staged + 1, ann))
        elif pc == "clock":                   # wave 0 reads the clock and may announce
            nxt = order0[order0.index("clock") + 1]
            put(i, (t, nxt, staged, ann))
            if ann == NEVER and fires_left > 0:
                a = t + rules.announce_ahead
                put(i, (t, nxt, staged, a), flush_after=a, fires=fires_left - 1)
        elif pc == "publish":                 # wave 0: progress = t + 1
            put(i, (t, order0[order0.index("publish") + 1], staged, ann), progress=t + 1)
        elif pc == "gate":                    # the other waves wait for wave 0
            if progress >= t - rules.gate_lag:
                put(i, (t, "decide", staged, ann))
        elif pc == "decide":
            on_time = (t == ann) if i == 0 else (flush_after == t)
            if on_time or staged == capacity or not more:
                put(i, (t, "barrier1", staged, t if on_time else ann))
            else:
                put(i, (t + 1, "tile", staged, ann))
        elif pc in ("barrier1", "barrier2"):  # arrive; the last wave in releases all of them
            if parked + 1 < n:
                put(i, (t, pc + " parked", staged, ann), parked=parked + 1)
                continue
            others = [(w[0], w[1].split()[0], w[2]) for j, w in enumerate(waves) if j != i]
            assert all(o == (t, pc, staged) for o in others), (
                "the barrier released waves that stand at different places", (t, pc, staged), others)
            released = []
            for tj, _, sj, aj in waves:
                if pc == "barrier1":
                    released.append((tj, "barrier2", sj, aj))
                elif tj + 1 >= tiles:
                    released.append((tj, "done", 0, NEVER))
                else:   # flushed: nothing parked; an on-time flush uses the announcement up
                    released.append((tj + 1, "tile", 0, NEVER if aj == tj else aj))
            out.append(((tuple(released), progress, flush_after, 0), fires_left))
        # (waves parked at a barrier, and waves that are done, do not move by themselves)
    return out


def explore(nwaves, tiles, capacity, rules, fires):
    """Every reachable state, depth first; returns how many there are."""
    start = (initial(nwaves), fires)
    seen = {start}
    stack = [start]
    while stack:
        state, fl = stack.pop()
        if all(w[1] == "done" for w in state[0]):
            continue
        succ = steps(state, tiles, capacity, rules, fl)
        assert succ, ("stuck: no wave can move", state)
        for s in succ:
            if s not in seen:
                seen.add(s)
                stack.append(s)
    return len(seen)


def random_walk(nwaves, tiles, capacity, rules, fires, rng):
    """One random interleaving to the end; returns the number of flushes."""
    state, fl = initial(nwaves), fires
    flushes = 0
    for _ in range(100000):
        if all(w[1] == "done" for w in state[0]):
            return flushes
        succ = steps(state, tiles, capacity, rules, fl)
        assert succ, ("stuck: no wave can move", state)
        was_parked = state[3]
        state, fl = rng.choice(succ)
        if was_parked and state[3] == 0 and state[0][0][1] in ("tile", "done"):
            flushes += 1
    raise AssertionError("did not finish")


def test_three_waves_every_interleaving():
    # capacity 4 tiles, 9 tiles in the piece, the clock may fire at up to two tiles of wave 0
    visited = explore(3, tiles=9, capacity=4, rules=Rules(), fires=2)
    assert visited > 10000
    # other capacities, among them one where forced and timed flushes fall on neighbouring tiles
    for cap in (1, 2, 3):
        explore(3, tiles=7, capacity=cap, rules=Rules(), fires=2)


def test_four_waves_every_interleaving_of_a_short_piece():
    assert explore(4, tiles=6, capacity=4, rules=Rules(), fires=1) > 100000
    with pytest.raises(AssertionError):
        explore(4, tiles=6, capacity=4, rules=planted(gate_lag=2), fires=1)


def test_four_waves_random_interleavings():
    rng = random.Random(1)
    total = 0
    for rep in range(300):
        total += random_walk(4, tiles=40, capacity=rng.choice([3, 5, 8]), rules=Rules(),
                             fires=rng.choice([0, 1, 3, 6]), rng=rng)
    assert total > 300 * 5      # the walks did flush, timed flushes among them


def planted(**kw):
    r = Rules()
    for k, v in kw.items():
        setattr(r, k, v)
    return r


@pytest.mark.parametrize("rules", [planted(gate_lag=2), planted(announce_ahead=1),
                                   planted(progress_first=True)],
                         ids=["gate one tile too lax", "announcement one tile too early",
                              "progress published before the announcement"])
def test_planted_mistakes_are_caught(rules):
    with pytest.raises(AssertionError):
        explore(3, tiles=9, capacity=4, rules=rules, fires=2)


def test_a_stricter_gate_still_works_but_a_gate_on_the_same_tile_blocks():
    explore(3, tiles=9, capacity=4, rules=planted(gate_lag=0), fires=2)     # waits longer, same result
    # waiting for wave 0 to be through tile t + 1 cannot work: wave 0 may be parked in the flush
    # barrier of tile t, which the others never reach
    with pytest.raises(AssertionError):
        explore(3, tiles=9, capacity=4, rules=planted(gate_lag=-2), fires=2)
