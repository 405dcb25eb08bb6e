"""How a chained stream of decode steps is compared when evicted-slot sets have to be bit-exact
while utilities only agree to rel 1e-4 (two fp32 summation orders can order a near-tie
differently):

  1. exact, every step: the oracle's eviction applied to the tested side's OWN pre-step
     utility bits must give exactly the tested side's evicted slots;
  2. the free-running oracle trajectory is compared too (utilities rel 1e-4, attention output
     to its tolerance).  At the first step - and any later one - where its own eviction differs
     from the tested side's, the two candidates must be a near-tie in the oracle's state
     (relative utility gap <= 1e-4); the tested side's choice is then adopted so that both
     trajectories keep holding the same entries, and the comparison goes on.

No arithmetic of the method lives here: the eviction itself is the oracle's.
"""
import numpy as np

from oracle import pikv_oracle as orc

NEAR_TIE_RTOL = 1e-4


def reconcile_eviction(ref_utility, ref_n, S, mask, got_idx, got_cnt, u_before, n_before, step):
    """Returns (idx, cnt, n_adopted): the eviction to apply to the oracle's trajectory this step.
    ref_n is updated in place (as orc.evict does); raises AssertionError on a real mismatch."""
    # 1. exact on identical bits
    ub, nb = u_before.copy(), n_before.copy()
    pidx, pcnt = orc.evict(ub, nb, S - 1, shard_mask=mask, max_evict=1)
    np.testing.assert_array_equal(got_cnt, pcnt, err_msg="step %d: evicted counts" % step)
    np.testing.assert_array_equal(got_idx[pcnt == 1], pidx[pcnt == 1],
                                  err_msg="step %d: evicted slots on the tested side's own bits" % step)
    # 2. free running
    ridx, rcnt = orc.evict(ref_utility, ref_n, S - 1, shard_mask=mask, max_evict=1)
    np.testing.assert_array_equal(rcnt, pcnt, err_msg="step %d: which shards were full" % step)
    adopted = 0
    out = ridx.copy()
    for b, e in zip(*np.nonzero((rcnt == 1) & (ridx[:, :, 0] != got_idx[:, :, 0]))):
        mine, theirs = int(ridx[b, e, 0]), int(got_idx[b, e, 0])
        a, c = float(ref_utility[b, e, mine]), float(ref_utility[b, e, theirs])
        gap = abs(a - c)
        assert gap <= NEAR_TIE_RTOL * max(abs(a), abs(c)) + 1e-12, (
            "step %d shard (%d,%d): the tested side evicted slot %d (oracle utility %.9g), the oracle "
            "slot %d (%.9g): not a near-tie" % (step, b, e, theirs, c, mine, a))
        out[b, e, 0] = theirs
        adopted += 1
    return out, rcnt, adopted
