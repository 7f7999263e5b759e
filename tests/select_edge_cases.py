"""Score vectors that sit exactly on a selection cut (Sec. 3.3, strategies 1 and 3) or one fp32 ulp beside it, with the
selection a strict ">" in double arithmetic must give.  Used as a pin of the oracle (CPU) and as a function-parity
case of the selection kernel (GPU)."""
import numpy as np

from oracle import round_attention as ora


def select_edge_cases():
    """List of (scores, oracle keyword arguments, expected selection or None where no hand value is claimed)."""
    f32 = np.float32
    up = lambda x: np.nextafter(f32(x), f32(2.0))
    dn = lambda x: np.nextafter(f32(x), f32(-1.0))
    cases = []   # (scores, params, expected selection or None = whatever the oracle says)
    # THRESHOLD at a value fp32 holds exactly: at the cut is out, one ulp above is in, one below is out
    thr = dict(strategy=ora.THRESHOLD, threshold=0.125, min_rounds=0)
    cases += [([0.125, 0.5, 0.25, 0.125], thr, [1, 2]),
              ([up(0.125), 0.5, 0.25, 0.125], thr, [0, 1, 2]),
              ([dn(0.125), 0.5, up(0.125), 0.125], thr, [1, 2])]
    # the paper's v = 0.1 is not an fp32 number: float32(0.1) lies above the double 0.1, its predecessor below
    thr01 = dict(strategy=ora.THRESHOLD, threshold=0.1, min_rounds=0)
    cases += [([f32(0.1), dn(f32(0.1)), 0.7, 0.1], thr01, [0, 2, 3])]
    # ADAPTIVE, lambda = 0: the mean of {1/4, 1/4, 1/2, 0} is exactly 1/4
    mean = dict(strategy=ora.ADAPTIVE, lam=0.0, min_rounds=0)
    cases += [([0.25, 0.25, 0.5, 0.0], mean, [2]),
              ([up(0.25), 0.25, 0.5, 0.0], mean, [0, 2]),        # the mean moves up by a quarter ulp only
              ([dn(0.25), 0.25, 0.5, 0.0], mean, [1, 2])]        # ... and down: the untouched 1/4 is now above it
    # ADAPTIVE, lambda = 1: {1/2, 1/2, 0, 0} has mean 1/4 and std 1/4, the cut is exactly 1/2: nothing passes,
    # min_rounds = 1 falls back to the best round, ties to the lower index
    one = dict(strategy=ora.ADAPTIVE, lam=1.0)
    cases += [([0.5, 0.5, 0.0, 0.0], one, [0]),
              ([0.5, up(0.5), 0.0, 0.0], one, None),
              ([dn(0.5), 0.5, 0.0, 0.0], one, None),
              ([0.5, 0.5, 0.0, 0.0], dict(strategy=ora.ADAPTIVE, lam=1.0, min_rounds=0), [])]
    # a longer vector whose population std is exact: 16 x {3/32 or 1/32} -> mean 1/16, std 1/32, cut 3/32
    v = [3 / 32] * 8 + [1 / 32] * 8
    cases += [(v, one, [0]), ([up(3 / 32)] + v[1:], one, None), (v[:-1] + [dn(1 / 32)], one, None)]
    return cases
