"""GPU tests of the KV store's turn-end write-back and of round dropping (Sec. 3.2 last step, Alg. 1
last line, Sec. 3.4): the new round leaves the GPU as one host tensor per sequence, can be selected
on the next turn, and rounds that were never selected are dropped."""
import numpy as np
import pytest
import torch

import paper_2502_15294_amd as ra
from oracle import round_attention as ora
from oracle import store_lifecycle as sl
from synth import make_workload, pack_round_host
from synth.device import Engine, to_device
from synth.workloads import to_bf16_bits

pytestmark = pytest.mark.gpu
STREAM_TOL = 5e-5


def _pinned(arr):
    return torch.from_numpy(arr.view(np.int16) if arr.dtype == np.uint16 else arr).pin_memory()


def _bits(x, dtype):
    return to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def _host_array(t, dtype):
    a = t.numpy()
    return a.view(np.uint16) if dtype == "bf16" else a


def _store(w, R_max, pool_bytes):
    dt = ra.RA_BF16 if w.dtype == "bf16" else ra.RA_F32
    return ra.ra_kv_store_create(0, w.n_post_layers, w.B, R_max, w.Hkv, w.d, dt, pool_bytes)


def _padded_cur(w, layers, cur_cap):
    """Device tensors [B][cur_cap][Hkv][d] per layer whose first cur_len rows are the workload's
    current round and whose tail is junk that must never reach the host tensor."""
    ks, vs = [], []
    for layer in layers:
        for src, dst in ((w.cur_k(layer), ks), (w.cur_v(layer), vs)):
            full = np.full((w.B, cur_cap, w.Hkv, w.d), 7.0, dtype=np.float32)
            full[:, :w.cur_len] = src
            dst.append(to_device(full, w.dtype))
    return ks, vs


@pytest.mark.parametrize("cfg,kw,new_lens", [
    ("cfg4", dict(B=3, R=6, n_post_layers=3, cur_len=37, length=("uniform", 20, 90)), [37, 16, 5]),
    ("cfg4", dict(B=2, R=4, n_post_layers=2, cur_len=130, length=("uniform", 20, 90)), [130, -1]),
    ("cfg1", dict(B=2, n_post_layers=2, cur_len=21), [21, 0]),
])
def test_save_round_writes_the_round_tensor(cfg, kw, new_lens):
    """The tensor written to pinned host memory, read back element by element through the oracle's
    address definition, holds exactly the current round's keys and values and zero padding."""
    w = make_workload(cfg, **kw)
    print(f"save case {cfg} {kw} lens={new_lens}", flush=True)
    layers = list(range(1, w.n_post_layers + 1))
    R_new = w.R_max
    store = _store(w, R_new + 1, 64 << 20)
    cur_cap = w.cur_len + 11
    ks, vs = _padded_cur(w, layers, cur_cap)
    skip = [n < 0 for n in new_lens]
    lens = [max(n, 0) for n in new_lens]
    el = torch.int16 if w.dtype == "bf16" else torch.float32
    hosts = [None if skip[b] else
             torch.full((ra.ra_kv_store_round_bytes(store, lens[b]) // (2 if w.dtype == "bf16" else 4) + 1,), 3,
                        dtype=el).pin_memory() for b in range(w.B)]
    rounds = torch.tensor([-1 if skip[b] else R_new for b in range(w.B)], dtype=torch.int32)
    side = torch.cuda.Stream()
    ra.ra_kv_store_save_round(store, rounds, torch.tensor(lens, dtype=torch.int32), ks, vs, hosts, None, side)
    saved = ra.ra_kv_store_save_wait(store)
    assert saved == sum(ra.ra_kv_store_round_bytes(store, lens[b]) for b in range(w.B) if not skip[b])
    for b in range(w.B):
        if skip[b]:
            with pytest.raises(ra.RaError) as e:
                ra.ra_kv_store_round_activity(store, b, R_new)
            assert e.value.code == ra.RA_ERR_STATE
            continue
        n = lens[b]
        buf = _host_array(hosts[b], w.dtype)
        assert buf[-1] == 3                                        # nothing written past the tensor
        K, V, pad = sl.read_round_tensor(buf[:-1], len(layers), w.Hkv, w.d, n)
        for i, layer in enumerate(layers):
            assert np.array_equal(K[i], _bits(w.cur_k(layer)[b, :n], w.dtype)), (b, layer)
            assert np.array_equal(V[i], _bits(w.cur_v(layer)[b, :n], w.dtype)), (b, layer)
        assert (pad == 0).all()
        assert ra.ra_kv_store_round_activity(store, b, R_new) == (0, 0)
    ra.ra_kv_store_destroy(store)


def test_two_turns_save_select_and_drop():
    """Turn 1 stages a selection and decodes with the current round, then saves that round; turn 2
    selects the saved round together with an old one and decodes from the staged copies.  The
    activity counters follow the oracle's ledger, dropping removes exactly the never-selected
    rounds, and a selection that still names a dropped round attends over the others only."""
    w = make_workload("cfg4", B=3, R=7, n_post_layers=2, cur_len=45, length=("lognormal", 60.0, 0.8, 400))
    layers = [1, 2]
    R = w.R_max
    store = _store(w, R + 1, 64 << 20)
    keep = {}
    ledgers = [sl.ActivityLedger() for _ in range(w.B)]
    for b in range(w.B):
        for r in range(w.n_rounds(b)):
            keep[b, r] = _pinned(pack_round_host(w, b, r, layers))
            ra.ra_kv_store_register_round(store, b, r, keep[b, r], int(w.lens[b][r]))
            ledgers[b].add_round(r)
    eng = Engine(w, extra_tokens=64)
    ctx = eng.ctx
    side = torch.cuda.Stream()
    new_lens = [45, 17, 32]
    cur_cap = 48
    ks, vs = _padded_cur(w, layers, cur_cap)
    cur_len = torch.tensor(new_lens, dtype=torch.int32, device="cuda")

    # ---- turn 1 -----------------------------------------------------------------------------
    sel1 = [[1, 4], [0], [2, 3, 5]]
    sel_t = torch.full((w.B, R + 1), -1, dtype=torch.int32)
    for b, s in enumerate(sel1):
        sel_t[b, :len(s)] = torch.tensor(s, dtype=torch.int32)
        ledgers[b].record_selection(s)
    n_t = torch.tensor([len(s) for s in sel1], dtype=torch.int32)
    ra.ra_kv_store_stage(store, sel_t, n_t, ra.RA_STAGE_LAYER_MAJOR, side)
    for li, layer in enumerate(layers):
        ra.ra_kv_store_wait_layer(store, li)
        q = to_device(w.q(layer)[:, 0], w.dtype)
        out, _ = ra.ra_round_sparse_attn_decode(ctx, q, ra.ra_kv_store_layer_view(store, li), cur_k=ks[li],
                                                cur_v=vs[li], cur_len=cur_len, scale=w.scale)
        for b in range(w.B):
            kr = [w.k_round(b, layer, r) if r in sel1[b] else None for r in range(w.n_rounds(b))]
            vr = [w.v_round(b, layer, r) if r in sel1[b] else None for r in range(w.n_rounds(b))]
            n = new_lens[b]
            ro, _ = ora.sparse_attention(w.q(layer)[b], kr, vr, sel1[b], w.scale, w.cur_k(layer)[b, :n],
                                         w.cur_v(layer)[b, :n])
            assert ora.row_error(out[b].cpu().numpy(), ro[0]) < STREAM_TOL, (b, layer)
    hosts = [torch.empty(ra.ra_kv_store_round_bytes(store, n) // 2, dtype=torch.int16).pin_memory() for n in new_lens]
    new_round = torch.tensor([w.n_rounds(b) for b in range(w.B)], dtype=torch.int32)
    ra.ra_kv_store_save_round(store, new_round, torch.tensor(new_lens, dtype=torch.int32), ks, vs, hosts, None, side)
    for b in range(w.B):
        ledgers[b].add_round(int(new_round[b]))
    ra.ra_kv_store_release(store)

    # ---- turn 2: no host wait between the save and the stage that reads the saved tensors ---------
    sel2 = [[4, int(new_round[0])], [int(new_round[1])], [0, 5, int(new_round[2])]]
    sel_t.fill_(-1)
    for b, s in enumerate(sel2):
        sel_t[b, :len(s)] = torch.tensor(s, dtype=torch.int32)
        ledgers[b].record_selection(s)
    n_t = torch.tensor([len(s) for s in sel2], dtype=torch.int32)
    ra.ra_kv_store_stage(store, sel_t, n_t, ra.RA_STAGE_ROUND_MAJOR, side)

    def rounds_of(b, layer, sel, dropped=()):
        nr = w.n_rounds(b)
        kr, vr = [None] * (nr + 1), [None] * (nr + 1)
        for r in sel:
            if r in dropped:
                kr[r] = np.zeros((0, w.Hkv, w.d), dtype=np.float32)
                vr[r] = np.zeros((0, w.Hkv, w.d), dtype=np.float32)
            elif r == nr:
                kr[r], vr[r] = w.cur_k(layer)[b, :new_lens[b]], w.cur_v(layer)[b, :new_lens[b]]
            else:
                kr[r], vr[r] = w.k_round(b, layer, r), w.v_round(b, layer, r)
        return kr, vr

    for li, layer in enumerate(layers):
        ra.ra_kv_store_wait_layer(store, li)
        q = to_device(w.q(layer)[:, 0], w.dtype)
        out, _ = ra.ra_round_sparse_attn_decode(ctx, q, ra.ra_kv_store_layer_view(store, li), scale=w.scale)
        for b in range(w.B):
            kr, vr = rounds_of(b, layer, sel2[b])
            ro, _ = ora.sparse_attention(w.q(layer)[b], kr, vr, sel2[b], w.scale, None, None)
            assert ora.row_error(out[b].cpu().numpy(), ro[0]) < STREAM_TOL, (b, layer)
    torch.cuda.synchronize()
    for b in range(w.B):
        for r in ledgers[b].turns:
            assert ra.ra_kv_store_round_activity(store, b, r) == (ledgers[b].turns[r], ledgers[b].hits[r]), (b, r)

    # ---- dropping ---------------------------------------------------------------------------------
    with pytest.raises(ra.RaError) as e:                      # still staged
        ra.ra_kv_store_drop_inactive(store, 2, w.B, R + 1)
    assert e.value.code == ra.RA_ERR_STATE
    ra.ra_kv_store_release(store)
    _, before, _ = ra.ra_kv_store_stats(store)
    idx, n = ra.ra_kv_store_drop_inactive(store, 2, w.B, R + 1)
    freed = 0
    dropped = []
    for b in range(w.B):
        expect = ledgers[b].inactive(2)
        assert idx[b, :n[b]].tolist() == expect and (idx[b, n[b]:] == -1).all(), b
        assert int(new_round[b]) not in expect                  # one turn only: below the threshold
        freed += sum(ra.ra_kv_store_round_bytes(store, int(w.lens[b][r])) for r in expect)
        ledgers[b].drop(expect)
        dropped.append(set(expect))
        for r in expect:
            del keep[b, r]                                      # the host tensors may go now
    assert sum(len(d) for d in dropped) > 0
    _, after, _ = ra.ra_kv_store_stats(store)
    assert before - after == freed
    idx2, n2 = ra.ra_kv_store_drop_inactive(store, 2, w.B, R + 1)    # nothing left to drop
    assert int(n2.sum()) == 0 and (idx2 == -1).all()

    # ---- turn 3: a stale selection names a dropped round --------------------------------------------
    sel3 = []
    for b in range(w.B):
        gone = sorted(dropped[b])
        alive = sorted(ledgers[b].turns)
        sel3.append(sorted(set(gone[:1] + alive[:2])))
    sel_t.fill_(-1)
    for b, s in enumerate(sel3):
        sel_t[b, :len(s)] = torch.tensor(s, dtype=torch.int32)
    n_t = torch.tensor([len(s) for s in sel3], dtype=torch.int32)
    ra.ra_kv_store_stage(store, sel_t, n_t, ra.RA_STAGE_ROUND_MAJOR, side)
    ra.ra_kv_store_wait_layer(store, 0)
    out, _ = ra.ra_round_sparse_attn_decode(ctx, to_device(w.q(1)[:, 0], w.dtype), ra.ra_kv_store_layer_view(store, 0),
                                            scale=w.scale)
    for b in range(w.B):
        kr, vr = rounds_of(b, 1, sel3[b], dropped[b])
        ro, _ = ora.sparse_attention(w.q(1)[b], kr, vr, sel3[b], w.scale, None, None)
        assert ora.row_error(out[b].cpu().numpy(), ro[0]) < STREAM_TOL, b
    staged, _, _ = ra.ra_kv_store_stats(store)
    assert staged == sum(ra.ra_kv_store_round_bytes(store, new_lens[b] if r == w.n_rounds(b) else int(w.lens[b][r]))
                         for b in range(w.B) for r in sel3[b] if r not in dropped[b])
    ra.ra_kv_store_release(store)
    ra.ra_kv_store_destroy(store)
    eng.close()


def test_save_round_error_paths():
    w = make_workload("cfg2", B=1, R=2, n_post_layers=2, cur_len=20, lens=[[20, 30]])
    store = _store(w, 3, 1 << 20)
    ks, vs = _padded_cur(w, [1, 2], 32)
    one = torch.tensor([2], dtype=torch.int32)
    n20 = torch.tensor([20], dtype=torch.int32)
    good = torch.empty(ra.ra_kv_store_round_bytes(store, 20) // 2, dtype=torch.int16).pin_memory()
    with pytest.raises(ra.RaError) as e:                               # host tensor not pinned
        ra.ra_kv_store_save_round(store, one, n20, ks, vs, [torch.empty(good.numel(), dtype=torch.int16)])
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    with pytest.raises(ra.RaError) as e:                               # longer than the current-round buffer
        ra.ra_kv_store_save_round(store, one, torch.tensor([33], dtype=torch.int32), ks, vs, [good])
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    with pytest.raises(ra.RaError) as e:                               # round index out of range
        ra.ra_kv_store_save_round(store, torch.tensor([3], dtype=torch.int32), n20, ks, vs, [good])
    assert e.value.code == ra.RA_ERR_INVALID_ARG
    small = _store(w, 3, 64 << 10)                                     # pool smaller than the round
    with pytest.raises(ra.RaError) as e:
        ra.ra_kv_store_save_round(small, one, n20, ks, vs, [good])
    assert e.value.code == ra.RA_ERR_OOM
    with pytest.raises(ra.RaError) as e:                               # nothing was registered by the failures
        ra.ra_kv_store_round_activity(store, 0, 2)
    assert e.value.code == ra.RA_ERR_STATE
    with pytest.raises(ra.RaError) as e:
        ra.ra_kv_store_drop_round(store, 0, 2)
    assert e.value.code == ra.RA_ERR_STATE
    ra.ra_kv_store_save_round(store, one, n20, ks, vs, [good])
    ra.ra_kv_store_drop_round(store, 0, 2)                             # waits for the copy, then forgets the round
    assert ra.ra_kv_store_stats(store)[1] == 0
    ra.ra_kv_store_destroy(small)
    ra.ra_kv_store_destroy(store)


@pytest.mark.parametrize("seed", range(4))
def test_random_turns_against_the_ledger_and_the_oracle(seed):
    """Six turns of a random dialogue: each turn stages a random selection (in either copy order), decodes one
    layer from the staged view, saves a new round of random length, and now and then drops the rounds that were
    never selected.  Counters follow the oracle's ledger, bytes follow the selection, attention follows the oracle."""
    rng = np.random.default_rng(500 + seed)
    B, R0, turns = 2, 4, 6
    cur_cap = 40
    w = make_workload("cfg4", B=B, R=R0, n_post_layers=2, cur_len=cur_cap, length=("uniform", 1, 120))
    layers = [1, 2]
    R_max = R0 + turns
    store = _store(w, R_max, 64 << 20)
    eng = Engine(w, extra_tokens=turns * cur_cap + 64)
    side = torch.cuda.Stream()
    ledgers = [sl.ActivityLedger() for _ in range(B)]
    # per sequence: round index -> (length, keys per layer, values per layer) as float arrays; host tensors kept alive
    content = [dict() for _ in range(B)]
    keep = {}
    for b in range(B):
        for r in range(R0):
            keep[b, r] = _pinned(pack_round_host(w, b, r, layers))
            ra.ra_kv_store_register_round(store, b, r, keep[b, r], int(w.lens[b][r]))
            content[b][r] = (int(w.lens[b][r]), [w.k_round(b, l, r) for l in layers], [w.v_round(b, l, r) for l in layers])
            ledgers[b].add_round(r)
    dropped = [set() for _ in range(B)]
    for turn in range(turns):
        n_now = R0 + turn
        # ---- a random selection among the rounds that exist (dropped ones may be named: they are empty) ----------
        sels = [sorted(rng.choice(n_now, size=int(rng.integers(1, n_now + 1)), replace=False).tolist()) for _ in range(B)]
        sel_t = torch.full((B, R_max), -1, dtype=torch.int32)
        for b, s in enumerate(sels):
            sel_t[b, :len(s)] = torch.tensor(s, dtype=torch.int32)
            ledgers[b].record_selection([r for r in s if r not in dropped[b]])
        n_t = torch.tensor([len(s) for s in sels], dtype=torch.int32)
        order = [ra.RA_STAGE_ROUND_MAJOR, ra.RA_STAGE_LAYER_MAJOR, ra.RA_STAGE_GROUPED][int(rng.integers(3))]
        ra.ra_kv_store_stage(store, sel_t, n_t, order, side)
        li = int(rng.integers(0, 2))
        ra.ra_kv_store_wait_layer(store, li)
        q_np = rng.standard_normal((B, 1, w.Hq, w.d)).astype(np.float32)
        q = to_device(q_np[:, 0], w.dtype)
        q_np = q.float().cpu().numpy()[:, None]                     # the values the GPU really sees
        out, _ = ra.ra_round_sparse_attn_decode(eng.ctx, q, ra.ra_kv_store_layer_view(store, li), scale=w.scale)
        torch.cuda.synchronize()
        staged, registered, _ = ra.ra_kv_store_stats(store)
        want_bytes = 0
        for b in range(B):
            live = [r for r in sels[b] if r not in dropped[b]]
            want_bytes += sum(ra.ra_kv_store_round_bytes(store, content[b][r][0]) for r in live)
            n_keys = sum(content[b][r][0] for r in live)
            if n_keys == 0:
                assert np.all(out[b].cpu().numpy() == 0)
                continue
            kr = {r: content[b][r][1][li] for r in live}
            vr = {r: content[b][r][2][li] for r in live}
            n_all = max(live) + 1
            ro, _ = ora.sparse_attention(q_np[b], [kr.get(r) for r in range(n_all)], [vr.get(r) for r in range(n_all)], live,
                                         w.scale, None, None)
            assert ora.row_error(out[b].cpu().numpy()[None], ro) < STREAM_TOL, (turn, b)
        assert staged == want_bytes
        # ---- the turn ends: a new round of random length goes to host memory ---------------------------------
        new_lens = [int(rng.integers(0, cur_cap + 1)) for _ in range(B)]
        k_np = [rng.standard_normal((B, cur_cap, w.Hkv, w.d)).astype(np.float32) for _ in layers]
        v_np = [rng.standard_normal((B, cur_cap, w.Hkv, w.d)).astype(np.float32) for _ in layers]
        ks, vs = [to_device(x, w.dtype) for x in k_np], [to_device(x, w.dtype) for x in v_np]
        hosts = [torch.empty(max(ra.ra_kv_store_round_bytes(store, n) // 2, 1), dtype=torch.int16).pin_memory()
                 for n in new_lens]
        ra.ra_kv_store_save_round(store, torch.full((B,), n_now, dtype=torch.int32),
                                  torch.tensor(new_lens, dtype=torch.int32), ks, vs, hosts, None, side)
        for b in range(B):
            keep[b, n_now] = hosts[b]
            n = new_lens[b]
            content[b][n_now] = (n, [k.float().cpu().numpy()[b, :n] for k in ks], [v.float().cpu().numpy()[b, :n] for v in vs])
            ledgers[b].add_round(n_now)
        ra.ra_kv_store_release(store)
        for b in range(B):
            for r in ledgers[b].turns:
                assert ra.ra_kv_store_round_activity(store, b, r) == (ledgers[b].turns[r], ledgers[b].hits[r]), (turn, b, r)
        # ---- every other turn: drop what was never selected in at least two turns -------------------------------
        if turn % 2 == 1:
            idx, n = ra.ra_kv_store_drop_inactive(store, 2, B, R_max)
            for b in range(B):
                expect = ledgers[b].inactive(2)
                assert idx[b, :n[b]].tolist() == expect, (turn, b)
                ledgers[b].drop(expect)
                dropped[b] |= set(expect)
                for r in expect:
                    content[b][r] = (0, content[b][r][1], content[b][r][2])
                    keep.pop((b, r), None)
    ra.ra_kv_store_save_wait(store)
    ra.ra_kv_store_destroy(store)
    eng.close()
