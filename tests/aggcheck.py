"""Invariant of every aggregation round (Alg. 1 aggregation line, Alg. 2 overwrite; Sec. 4.4 for failed trainers),
checked on the parameters a ModelAggregation recorded on its aggregation stream (test helper)."""
import numpy as np


def check_recorded_rounds(agg, n_rounds, active_mask):
    """For each recorded round: the mean equals the arithmetic mean of the ACTIVE trainers' parameters as they were
    right before phi (so every active trainer's last step had finished), every active trainer holds exactly that
    mean right after it, inactive ones are untouched, and the next step of no trainer slipped in between."""
    M = agg.M
    active = [i for i in range(M) if (active_mask >> i) & 1]
    before = agg.rec_before[:n_rounds].cpu().numpy().astype(np.float64)
    after = agg.rec_after[:n_rounds].cpu().numpy()
    glob = agg.rec_global[:n_rounds].cpu().numpy()
    for r in range(n_rounds):
        mean = before[r, active].mean(axis=0)                      # the definition of phi, in fp64
        scale = max(np.abs(mean).max(), 1e-30)
        assert np.abs(glob[r] - mean).max() <= 1e-6 * scale, f"round {r}: W_global is not the mean of the inputs"
        for i in range(M):
            if i in active:
                assert np.array_equal(after[r, i], glob[r]), f"round {r}: trainer {i} does not hold the mean"
            else:
                assert np.array_equal(after[r, i], before[r, i].astype(np.float32)), f"round {r}: inactive trainer {i} changed"
        if r + 1 < n_rounds and len(active) > 1:
            # between two rounds the trainers trained on different data: their parameters must have moved apart again
            assert any(not np.array_equal(before[r + 1, i], before[r + 1, active[0]]) for i in active[1:]) or \
                agg.history[r + 1] == agg.history[r], f"round {r + 1}: no trainer moved since round {r}"
