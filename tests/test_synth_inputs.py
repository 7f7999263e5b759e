"""Host-side checks of the seeded input generators and the packed layouts."""
import numpy as np

from synth import make_workload, pack_layer, to_bf16_bits, bf16_bits_to_f32
import torch


def test_bf16_rounding_matches_library_round_to_nearest_even():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65280.0, 1e-30], dtype=np.float32)])
    ours = bf16_bits_to_f32(to_bf16_bits(x))
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, ref)


def test_workloads_are_deterministic_and_lazily_sliceable():
    a, b = make_workload("cfg2", B=2), make_workload("cfg2", B=2)
    assert all(np.array_equal(x, y) for x, y in zip(a.lens, b.lens))
    assert np.array_equal(a.k_round(1, 0, 3), b.k_round(1, 0, 3))
    assert np.array_equal(a.q(1), b.q(1))
    assert not np.array_equal(a.k_round(1, 0, 3), a.k_round(1, 1, 3))
    k = a.k_round(0, 1, 2)
    assert k.shape == (a.lens[0][2], 8, 128) and k.dtype == np.float32
    assert np.array_equal(bf16_bits_to_f32(to_bf16_bits(k)), k)      # values are exactly bf16
    assert all(200 <= n <= 1000 for n in a.lens[0])


def test_length_recipes():
    w3 = make_workload("cfg3", B=2)
    assert all(int(l.sum()) == 32768 and l.min() >= 1 and len(l) == 60 for l in w3.lens)
    w1 = make_workload("cfg1")
    assert w1.lens[0].tolist() == [64] * 8 and w1.dtype == "f32"


def test_relevant_rounds_carry_the_bias():
    w = make_workload("cfg1")
    q = w.q(1)[0, 0]                                              # [Hq, d]
    rel = set(w.relevant[0].tolist())
    for r in range(8):
        k = w.k_round(0, 1, r)
        proj = np.mean([(k[:, h // 2, :] @ q[h]).mean() for h in range(4)])
        assert (proj > 5.0) == (r in rel)


def test_contiguous_and_paged_packing_hold_the_same_values():
    w = make_workload("cfg2", B=2, R=5, length=("uniform", 3, 40))
    pc = pack_layer(w, 1, block_size=0, threads=1)
    pp = pack_layer(w, 1, block_size=16, threads=2)
    Hkv, d = w.Hkv, w.d
    kc, vc, vp = pc.k.reshape(-1, d), pc.v, pp.v.reshape(-1, Hkv, d, 16)
    for b in range(2):
        for r in range(5):
            n = int(w.lens[b][r])
            kr, vr = to_bf16_bits(w.k_round(b, 1, r)), to_bf16_bits(w.v_round(b, 1, r))
            assert pc.seg_len[b, r] == n == pp.seg_len[b, r]
            for g in (0, Hkv - 1):
                for t in (0, n // 2, n - 1):
                    row = (pc.seg_off[b, r] * Hkv + g * n + t)
                    assert np.array_equal(kc[row], kr[t, g])
                    blk = pp.block_table[b, pp.seg_off[b, r] + t // 16]
                    assert np.array_equal(vp[blk, g, :, t % 16], vr[t, g])
                    L16 = 16 * (-(-n // 16))
                    base = (pc.seg_off_v[b, r] * Hkv + g * L16 + (t // 16) * 16) * d + t % 16
                    assert np.array_equal(vc[base + 16 * np.arange(d)], vr[t, g])
    used = pp.block_table[pp.block_table >= 0]
    assert len(set(used.tolist())) == len(used)                    # no physical block is shared
