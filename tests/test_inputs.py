"""CPU: the seeded input recipe (kvtrim_inputs) - repetitions of a workload are other draws of the same recipe."""
import numpy as np

import kvtrim_inputs as ki


def test_seed_index_gives_another_draw_of_the_same_shape():
    a = ki.workload("tiny", prefill=256)
    b = ki.workload("tiny", prefill=256, seed_index=1)
    assert ki.workload("tiny", prefill=256, seed_index=0) == a and a.seed != b.seed
    assert (a.nseg, a.budget, a.prefill) == (b.nseg, b.budget, b.prefill)
    ca, _ = ki.ragged_cache(a, [40] * a.nseg)
    cb, _ = ki.ragged_cache(b, [40] * b.nseg)
    ca2, _ = ki.ragged_cache(ki.workload("tiny", prefill=256), [40] * a.nseg)
    assert np.array_equal(ca["log_beta"].numpy(), ca2["log_beta"].numpy())         # seeded: the same bytes every time
    assert ca["log_beta"].shape == cb["log_beta"].shape
    assert not np.array_equal(ca["log_beta"].numpy(), cb["log_beta"].numpy())
    assert not np.array_equal(ca["k"].float().numpy(), cb["k"].float().numpy())
