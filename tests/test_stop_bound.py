"""The inequality the selection kernel's read-ahead limit rests on, checked on the CPU against the oracle's own
P_acc curves: after n blocks of a ranking, with AS_acc and AS_min as they stand, the stop rule of Algorithm 1
(lines 13-18) must fire at the first tested position n* with N - n* < (AS_acc / AS_min) (1 - eps) / eps at the
latest, because AS_acc only grows and AS_min only shrinks from there on.  The kernel publishes that position (with
a safety factor and rounded up to whole chunks) as the point beyond which keys are not worth reading; a stop
beyond it would mean keys the rule needs were never read.  Nothing of the kernel is executed here: the test pins
the mathematics, on the oracle's curves, for every head, every n and several thresholds."""
import math

import numpy as np
import pytest

import np_reference as ref
from oracle import psa_oracle as po


def _bound(as_blocks: np.ndarray, n: int, N: int, eps: float, m: int) -> int:
    """The latest position the stop can take, judged after the first n blocks (natural-log AS values)."""
    acc = np.logaddexp.reduce(as_blocks[:n])
    mn = as_blocks[:n].min()
    room = math.exp(acc - mn) * (1.0 - eps) / eps if eps > 0 else math.inf
    # smallest n* >= n + 1 with N - n* < room, then the next tested position (a multiple of m, or N)
    nstar = max(n + 1, N - (math.ceil(room) - 1) if math.isfinite(room) else 0)
    nstar = min(N, -(-nstar // m) * m)
    return nstar


@pytest.mark.parametrize("eps,m", [(0.5, 1), (0.9, 1), (0.95, 4), (0.99, 3), (0.999, 1)])
def test_the_stop_never_lies_beyond_the_bound_computed_from_any_earlier_state(eps, m):
    rng = np.random.default_rng(7)
    pb = ref.random_problem(rng, B=3, Hq=8, Hkv=2, d=16, T=4, ctx=(160, 61, 7), dtype=po.BF16)
    res = po.psa_decode(pb, eps, m, curves=True)
    G = 4
    checked = 0
    for r in range(3):
        N = int(pb.num_blocks()[r])
        for hq in range(8):
            stop = int(res.n_selected[r, hq])
            lse = res.block_lse[r, hq, :N]                  # log AS of the n-th block in rank order
            for n in range(1, stop + 1):
                assert stop <= _bound(lse, n, N, eps, m), (r, hq, n, stop)
                checked += 1
            # and the bound is attained: judged at the stop itself it names the stop
            assert _bound(lse, stop, N, eps, m) >= stop
    assert checked > 100
