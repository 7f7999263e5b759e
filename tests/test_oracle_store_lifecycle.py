"""Pins of the oracle's turn-end / dropping models (Sec. 3.2 last step, Alg. 1 last line, Sec. 3.4)."""
import numpy as np
import pytest

from oracle import store_lifecycle as sl
from synth import make_workload, pack_round_host


def test_addresses_of_a_hand_worked_round():
    # 2 layers, 2 kv heads, 2 channels, 3 tokens: a layer holds 3 key rows and one 16-token value
    # tile per head = (3 + 16) * 2 * 2 = 76 elements.
    Hkv, d, n = 2, 2, 3
    assert sl.round_tensor_elems(2, Hkv, d, n) == 152
    assert sl.key_address(0, 0, 0, 0, Hkv, d, n) == 0
    assert sl.key_address(0, 1, 0, 0, Hkv, d, n) == 6            # head 1 starts after 3 rows of 2
    assert sl.key_address(1, 1, 2, 1, Hkv, d, n) == 76 + 11
    assert sl.value_address(0, 0, 0, 0, Hkv, d, n) == 12         # right after the 12 key elements
    assert sl.value_address(0, 0, 1, 0, Hkv, d, n) == 13         # next token of the same channel is adjacent
    assert sl.value_address(0, 0, 0, 1, Hkv, d, n) == 12 + 16    # next channel is 16 further
    assert sl.value_address(0, 1, 2, 1, Hkv, d, n) == 12 + 32 + 16 + 2
    assert sl.value_address(1, 0, 0, 0, Hkv, d, n) == 76 + 12


@pytest.mark.parametrize("n", [1, 15, 16, 17, 37])
def test_addresses_tile_the_tensor_exactly_once(n):
    L, Hkv, d = 2, 2, 4
    seen = np.zeros(sl.round_tensor_elems(L, Hkv, d, n), dtype=np.int32)
    for layer in range(L):
        for g in range(Hkv):
            for c in range(d):
                for t in range(n):
                    seen[sl.key_address(layer, g, t, c, Hkv, d, n)] += 1
                for t in range(16 * ((n + 15) // 16)):
                    seen[sl.value_address(layer, g, t, c, Hkv, d, n)] += 1
    assert (seen == 1).all()


@pytest.mark.parametrize("cfg,kw", [("cfg1", {}), ("cfg2", dict(B=1, R=3, length=("fixed", 37))),
                                    ("cfg2", dict(B=1, R=2, length=("fixed", 16)))])
def test_reader_inverts_the_input_packer(cfg, kw):
    """The packer of the synthetic inputs and the oracle's reader are written separately; one must
    undo the other, values and zero padding alike."""
    w = make_workload(cfg, **kw)
    layers = list(range(1, w.n_post_layers + 1))
    for r in range(min(w.n_rounds(0), 3)):
        buf = pack_round_host(w, 0, r, layers)
        n = int(w.lens[0][r])
        K, V, pad = sl.read_round_tensor(buf, len(layers), w.Hkv, w.d, n)
        for i, layer in enumerate(layers):
            k, v = w.k_round(0, layer, r), w.v_round(0, layer, r)
            if w.dtype == "bf16":
                from synth.workloads import to_bf16_bits
                k, v = to_bf16_bits(k), to_bf16_bits(v)
            assert np.array_equal(K[i], k) and np.array_equal(V[i], v)
        assert (pad == 0).all()


def test_activity_ledger_hand_example():
    led = sl.ActivityLedger()
    for r in range(4):
        led.add_round(r)
    led.record_selection([1, 3])
    led.add_round(4)                       # a new round joins after the first turn
    led.record_selection([3])
    led.record_selection([3, 4])
    assert led.turns == {0: 3, 1: 3, 2: 3, 3: 3, 4: 2}
    assert led.hits == {0: 0, 1: 1, 2: 0, 3: 3, 4: 1}
    assert led.inactive(min_turns=3) == [0, 2]
    assert led.inactive(min_turns=4) == []
    led.drop([0, 2])
    led.record_selection([1])
    assert led.turns == {1: 4, 3: 4, 4: 3} and led.hits == {1: 2, 3: 3, 4: 1}
    with pytest.raises(AssertionError):
        led.record_selection([0])           # a dropped round can no longer be selected
