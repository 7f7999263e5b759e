"""The oracle's whole path on the smallest benchmark configuration, against scalar brute force."""
import math

import numpy as np

from oracle import pipeline
from oracle import round_attention as ra
from synth import make_workload


def test_config1_pipeline_against_scalar_brute_force():
    w = make_workload("cfg1")
    res = pipeline.run(w)[0]
    q0, q1 = w.q(0)[0, 0].astype(float), w.q(1)[0, 0].astype(float)
    R, Hq, G, d, scale = 8, w.Hq, w.G, w.d, w.scale
    # scores: plain loops over heads, rounds, tokens
    P = np.zeros((Hq, R))
    for h in range(Hq):
        for r in range(R):
            k = w.k_round(0, 0, r).astype(float)
            P[h, r] = sum(math.exp(scale * float(np.dot(q0[h], k[j, h // G]))) for j in range(k.shape[0]))
        P[h] /= P[h].sum()
    assert np.allclose(res.P, P, rtol=1e-11)
    S = P.mean(axis=0)
    cut = S.mean() + S.std()
    assert res.sel == [r for r in range(R) if S[r] > cut]
    # attention over the selected rounds of the post-watershed layer
    O = np.zeros((Hq, d))
    for h in range(Hq):
        z = 0.0
        for r in res.sel:
            k, v = w.k_round(0, 1, r).astype(float), w.v_round(0, 1, r).astype(float)
            for j in range(k.shape[0]):
                e = math.exp(scale * float(np.dot(q1[h], k[j, h // G])))
                z += e
                O[h] += e * v[j, h // G]
        O[h] /= z
    assert np.allclose(res.out[1][0], O, rtol=1e-11, atol=1e-13)
    assert ra.row_error(res.out[1][0], O) < 1e-12


def test_selection_margins_of_the_decode_configs_are_well_conditioned():
    w = make_workload("cfg2", B=3)
    for b in range(3):
        _, S = pipeline.scores_for_sequence(w, b)
        _, info = ra.select_rounds(S)
        assert info["margin"] > 1e-4
