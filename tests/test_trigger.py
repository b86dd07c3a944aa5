"""Host logic of the time-based trigger (no GPU): driven by a simulated clock it must reproduce the
timeline the oracle derives from Alg. 1 / Alg. 2."""
import pytest

from oracle import model as omodel
from paper_2305_09887_amd.aggregation import AggregationTrigger


class FakeClock:
    def __init__(self):
        self.t = 0.0

    def __call__(self):
        return self.t


def simulate(step_time, n_trainers, dt_int, dt_train):
    """Discrete-event run of M trainers against an AggregationTrigger.  A trainer looks at the flag only
    when a step of its own ends (Alg. 2); a round completes when every trainer has joined."""
    clock = FakeClock()
    trig = AggregationTrigger(dt_int, dt_train, clock)
    ends = [step_time(i, 0) for i in range(n_trainers)]   # time at which each trainer's current step ends
    steps = [0] * n_trainers
    joined = [False] * n_trainers
    rounds = []
    while True:
        i = min((k for k in range(n_trainers) if not joined[k]), key=lambda k: ends[k])
        if ends[i] > dt_train and not any(joined):         # stop flag is up before this step would be seen
            pass
        clock.t = ends[i]
        steps[i] += 1
        if trig.should_aggregate() and clock.t - 0.0 <= dt_train + max(step_time(k, 0) for k in range(n_trainers)) \
                and trig.t_agg + dt_int <= dt_train:
            joined[i] = True
            if all(joined):
                trig.mark_aggregated()                     # weights returned at the time the slowest one delivered
                rounds.append(list(steps))
                joined = [False] * n_trainers
                ends = [clock.t + step_time(k, steps[k]) for k in range(n_trainers)]
            continue
        if trig.should_stop() or (trig.t_agg + dt_int > dt_train and clock.t > dt_train):
            ends[i] = float("inf")
            joined[i] = True                                # out of the loop
            if all(joined):
                break
            continue
        ends[i] = clock.t + step_time(i, steps[i])
    return rounds, steps


@pytest.mark.parametrize("speeds,dt_int,dt_train", [
    ([1.0, 1.0, 1.0], 10.5, 35.0),
    ([1.0, 1.0, 1.4], 10.5, 25.0),
    ([0.7, 1.3, 1.0, 2.1], 7.3, 50.0),
])
def test_trigger_reproduces_oracle_rounds(speeds, dt_int, dt_train):
    st = lambda i, k: speeds[i]
    want_rounds, _ = omodel.tma_schedule(st, len(speeds), dt_int, dt_train)
    got_rounds, _ = simulate(st, len(speeds), dt_int, dt_train)
    assert got_rounds == want_rounds


def test_trigger_basics():
    clock = FakeClock()
    trig = AggregationTrigger(2.0, 5.0, clock)
    assert not trig.should_aggregate() and not trig.should_stop()
    clock.t = 2.0
    assert trig.should_aggregate()                 # >= : fires exactly at the interval
    clock.t = 2.5
    trig.mark_aggregated()                         # T_agg is reset when the weights are back
    clock.t = 4.4
    assert not trig.should_aggregate()
    clock.t = 4.5
    assert trig.should_aggregate()
    clock.t = 5.0
    assert not trig.should_stop()                  # strict > for the training budget
    clock.t = 5.01
    assert trig.should_stop() and trig.rounds == 1
    with pytest.raises(ValueError):
        AggregationTrigger(0.0, 1.0)
