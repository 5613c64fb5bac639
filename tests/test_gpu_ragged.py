"""GPU parity for batches whose sequences differ: prompt lengths, positions,
budgets per sequence, sequences that sit a step out, per-sequence cosines.
The oracle works one (layer, sequence, KV head) unit at a time, so it needs no
notion of a ragged batch: each unit is simply given its own lengths."""
import os

import numpy as np
import pytest
import torch

from oracle import sqa_oracle as O
from paper_2404_04793_amd import workloads as W
from tests.harness import (TOL, check_step_scores, export_state, import_state, np64, rel_err, round_scores_f32,
                           uses_matrix_cores)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sqa():
    from paper_2404_04793_amd import binding
    return binding


def _i32(x):
    return torch.tensor(x, dtype=torch.int32, device=DEV)


@pytest.mark.parametrize("dtype,d", [("f32", 256), ("bf16", 1024)])
def test_layer_importance_per_sequence(sqa, dtype, d):
    L, lens = 3, [37, 1, 0, 260, 5]
    T = sum(lens)
    wl = W.scaled(W.WORKLOADS["tiny"], L=L, hidden=d, dtype=dtype, B=1, P=T)
    hs = [W.hidden_states(wl, l, DEV) for l in range(L)]
    h_in = torch.stack([x[0] for x in hs]).contiguous()
    h_out = torch.stack([x[1] for x in hs]).contiguous()
    start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cos = sqa.layer_importance_seq(h_in, h_out, _i32(start.tolist())).cpu().numpy().astype(np.float64)
    a, b = np64(h_in), np64(h_out)
    for s, n in enumerate(lens):
        if n == 0:
            assert np.all(cos[:, s] == 0.0)
            continue
        ref = O.layer_importance(a[:, start[s]:start[s + 1]], b[:, start[s]:start[s + 1]])
        assert np.max(np.abs(cos[:, s] - ref) / np.maximum(np.abs(ref), 1e-3)) < 1e-5
    # one segment covering everything == the plain call, bit for bit
    whole = sqa.layer_importance_seq(h_in, h_out, _i32([0, T]))[:, 0].cpu().numpy()
    plain = sqa.layer_importance(h_in, h_out).cpu().numpy()
    assert np.array_equal(whole.view(np.uint32), plain.view(np.uint32))


@pytest.mark.parametrize("dtype,D,g", [("f32", 64, 2), ("bf16", 128, 1), ("bf16", 128, 4)])
def test_prefill_scores_ragged(sqa, dtype, D, g):
    B, Hkv, P = 3, 2, 200
    plen = [200, 77, 1]
    wl = W.scaled(W.WORKLOADS["tiny"], L=1, Hq=Hkv * g, Hkv=Hkv, D=D, B=B, P=P, dtype=dtype)
    K, _ = W.prompt_kv(wl, 0, DEV)
    Q = W.prompt_q(wl, 0, DEV)
    got = sqa.prefill_scores(Q, K, opts=sqa.batch_opts(prompt_len=_i32(plen))).cpu().numpy().astype(np.float64)
    Qn, Kn = np64(Q), np64(K)
    for b in range(B):
        for h in range(Hkv):
            n = plen[b]
            ref = O.prefill_scores(Qn[b, h * g:(h + 1) * g, :n], Kn[b, h, :n])
            assert rel_err(got[b, h, :n], ref) < TOL[dtype]
            assert np.all(got[b, h, n:] == 0.0)


@pytest.mark.parametrize("policy,g,packed", [("sliding", 2, False), ("streaming", 2, True), ("h2o", 2, False),
                                              ("h2o", 2, True), ("h2o", 8, True), ("sliding", 8, False)])
def test_ragged_batch_end_to_end(sqa, policy, g, packed):
    """Three sequences with different prompt lengths and budgets through scores ->
    compress -> decode (teacher forced), one of them sitting out some steps.  g = 8 takes the
    matrix-core variant of the decode kernel; packed: every unit owns exactly the slots its own
    budget needs (unit_offset) instead of the layer's maximum."""
    lo = {"sliding": 1, "streaming": 5, "h2o": 2}[policy]
    _ragged_case(sqa, policy, g, packed, False, "bf16", 128, 2, 2, 3, 150, 7, [150, 61, 9],
                 [[40, 13, max(lo, 6)], [153, 70, 12]], lambda b, t: [True, t % 3 != 1, t < 5][b])


def _random_ragged_cases(n, seed=515):
    r = np.random.default_rng(seed)
    out = []
    for k in range(n):
        dtype = ["bf16", "f32"][int(r.integers(2))]
        D = [64, 128][int(r.integers(2))]
        g = [1, 2, 4, 8][int(r.integers(4))]
        Hkv, B, L = int(r.integers(1, 4)), int(r.integers(2, 6)), int(r.integers(1, 4))
        P, S = int(r.choice([40, 97, 150, 260, 420])), int(r.integers(3, 8))
        policy = ["sliding", "streaming", "h2o"][int(r.integers(3))]
        lo = {"sliding": 1, "streaming": 5, "h2o": 2}[policy]
        plen = [P] + [int(r.integers(1, P + 1)) for _ in range(B - 1)]
        budget_seq = [[int(max(lo, r.choice([r.integers(lo, lo + 8), r.integers(lo, P), plen[b], plen[b] + 3])))
                       for b in range(B)] for _ in range(L)]
        layout = int(r.integers(3))
        out.append(("rag%02d_%s_%s_D%d_g%d_%s" % (k, policy, dtype, D, g, ["dense", "packed", "blocked"][layout]),
                    policy, g, layout == 1, layout == 2, dtype, D, L, Hkv, B, P, S, plen, budget_seq, int(r.integers(2, 5))))
    return out


# (SQA_RANDOM_CASES=1500 python -m pytest tests/test_gpu_ragged.py -m gpu -k random  runs a longer campaign)
RANDOM_RAGGED = _random_ragged_cases(max(1, int(os.environ.get("SQA_RANDOM_CASES", "28")) // 2))


@pytest.mark.parametrize("case", RANDOM_RAGGED, ids=[c[0] for c in RANDOM_RAGGED])
def test_ragged_random_batches(sqa, case):
    """Seeded random batches: 2-5 sequences with their own prompt lengths and per-layer budgets (below, at
    and above their lengths), sitting out every 2nd-4th step in turn, in the dense, packed or blocked layout."""
    _, policy, g, packed, blocked, dtype, D, L, Hkv, B, P, S, plen, budget_seq, sit_mod = case
    _ragged_case(sqa, policy, g, packed, blocked, dtype, D, L, Hkv, B, P, S, plen, budget_seq,
                 lambda b, t: (b + t) % sit_mod != sit_mod - 1 or b == 0)


def _ragged_case(sqa, policy, g, packed, blocked, dtype, D, L, Hkv, B, P, S, plen, budget_seq, is_active):
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    Hq = Hkv * g
    layer_budget = [max(r) for r in budget_seq]
    wl = W.scaled(W.WORKLOADS["tiny"], L=L, Hq=Hq, Hkv=Hkv, D=D, B=B, P=P, S=S, dtype=dtype, policy=policy)
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, DEV)
    unit_caps = [[min(budget_seq[l][b], plen[b] + S) for b in range(B) for _ in range(Hkv)] for l in range(L)]
    caches = sqa.LayerCaches(layer_budget, [max(c) for c in unit_caps] if packed else [min(b, P + S) for b in layer_budget],
                             B, Hkv, D, tdt, DEV, True, unit_capacities=unit_caps if packed else None,
                             blocked=blocked, block_seed=P)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    plen_d, bseq_d = _i32(plen), _i32(budget_seq)
    opts_pre = sqa.batch_opts(prompt_len=plen_d, budget_seq=bseq_d, status=status)
    Ks, Vs, Ss, qkv = [], [], [], []
    for l in range(L):
        K, V = W.prompt_kv(wl, l, DEV, u_dirs, mask)
        Q = W.prompt_q(wl, l, DEV, u_dirs)
        Ks.append(K); Vs.append(V)
        Ss.append(sqa.prefill_scores(Q, K, opts=opts_pre))
        qkv.append(W.decode_qkv(wl, l, DEV, u_dirs, mask))
    sqa.prefill_compress_layers(Ks, Vs, Ss if policy == "h2o" else None, policy, wl.n_sink, caches, opts=opts_pre)
    assert int(status.item()) == 0
    state = {}
    for l in range(L):
        Kn, Vn, Sn = np64(Ks[l]), np64(Vs[l]), np64(Ss[l])
        for b in range(B):
            for h in range(Hkv):
                n = plen[b]
                want = O.prefill_compress(Kn[b, h, :n], Vn[b, h, :n], Sn[b, h, :n], budget_seq[l][b], policy, wl.n_sink)
                got = export_state(caches, l, b, h)
                assert got["pos"].tolist() == want["pos"].tolist(), ("compress", l, b, h)
                assert np.array_equal(got["K"], want["K"]) and np.array_equal(got["V"], want["V"])
                if policy == "h2o":
                    assert np.array_equal(got["score"], want["score"])
                state[l, b, h] = want
    q_all = torch.stack([x[0] for x in qkv], 1).contiguous()
    k_all = torch.stack([x[1] for x in qkv], 1).contiguous()
    v_all = torch.stack([x[2] for x in qkv], 1).contiguous()
    qn, kn, vn = np64(q_all), np64(k_all), np64(v_all)
    ws = sqa.decode_workspace(caches, Hq, policy)
    pos_now = list(plen)
    worst = 0.0
    for t in range(S):
        active = [is_active(b, t) for b in range(B)]
        new_pos = [pos_now[b] if active[b] else -1 for b in range(B)]
        for key, c in state.items():
            import_state(caches, key[0], key[1], key[2], c)
        out = torch.full((L, B, Hq, D), 7.0, dtype=tdt, device=DEV)
        sqa.decode_step(q_all[t], k_all[t], v_all[t], 0, policy, wl.n_sink, caches, out, ws,
                        opts=sqa.batch_opts(budget_seq=bseq_d, new_pos_seq=_i32(new_pos)))
        assert sqa.read_device_status(ws) == 0
        o = np64(out)
        for (l, b, h), c in state.items():
            got = export_state(caches, l, b, h)
            if not active[b]:
                assert np.all(o[l, b] == 7.0)                              # untouched
                assert got["pos"].tolist() == c["pos"].tolist() and np.array_equal(got["K"], c["K"])
                continue
            want_out, c2 = O.decode_step(c, qn[t, l, b, h * g:(h + 1) * g], kn[t, l, b, h], vn[t, l, b, h],
                                         new_pos[b], budget_seq[l][b], policy, wl.n_sink)
            assert got["pos"].tolist() == c2["pos"].tolist(), (t, l, b, h)
            assert np.array_equal(got["K"], c2["K"]) and np.array_equal(got["V"], c2["V"])
            worst = max(worst, rel_err(o[l, b, h * g:(h + 1) * g], want_out))
            if policy == "h2o":
                check_step_scores(got, c, c2, uses_matrix_cores(dtype, D, g), (t, l, b, h))
            state[l, b, h] = round_scores_f32(c2)
        for b in range(B):
            pos_now[b] += 1 if active[b] else 0
    assert worst < TOL[dtype]
    for l in range(L):                                   # the sorted view, in the layout of pos
        kept = sqa.kept_idx_sorted(caches, l).cpu().numpy()
        for b in range(B):
            for h in range(Hkv):
                want = state[l, b, h]["pos"].tolist()
                if packed:
                    lo = caches.offsets_host[l][b * Hkv + h]
                    hi = caches.offsets_host[l][b * Hkv + h + 1]
                    row = kept[lo:hi]
                else:
                    row = kept[b, h]
                assert row[:len(want)].tolist() == want and np.all(row[len(want):] == -1)


def test_out_of_range_per_sequence_values_are_reported(sqa):
    B, Hkv, D, P = 2, 1, 64, 32
    K = torch.randn(B, Hkv, P, D, device=DEV); V = torch.randn(B, Hkv, P, D, device=DEV)
    caches = sqa.LayerCaches([8], [9], B, Hkv, D, torch.float32, DEV, True)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    # sequence 1: prompt longer than the tensors
    sqa.prefill_compress_layers([K], [V], None, "sliding", 4, caches,
                                opts=sqa.batch_opts(prompt_len=_i32([32, 33]), status=status))
    assert int(status.item()) == 2 and caches.lens[0][:, 0].tolist() == [8, 0]
    status.zero_()
    # sequence 0: budget above the layer's maximum
    sqa.prefill_compress_layers([K], [V], None, "sliding", 4, caches,
                                opts=sqa.batch_opts(budget_seq=_i32([[9, 3]]), status=status))
    assert int(status.item()) == 5 and caches.lens[0][:, 0].tolist() == [0, 3]
    # decode: same bad budget -> status word, unit untouched, out zeroed
    ws = sqa.decode_workspace(caches, Hkv, "sliding")
    q = torch.randn(1, B, Hkv, D, device=DEV); out = torch.full_like(q, 3.0)
    sqa.decode_step(q, q, q, 40, "sliding", 4, caches, out, ws, opts=sqa.batch_opts(budget_seq=_i32([[9, 3]])))
    assert sqa.read_device_status(ws) == 5
    assert caches.lens[0][:, 0].tolist() == [0, 3] and bool((out[0, 0] == 0).all()) and not bool((out[0, 1] == 0).any())
    # packed units: a unit that was given fewer slots than its budget keeps is reported and left empty
    small = sqa.LayerCaches([8], [8], B, Hkv, D, torch.float32, DEV, True, unit_capacities=[[8, 5]])
    status.zero_()
    sqa.prefill_compress_layers([K], [V], None, "sliding", 4, small, opts=sqa.batch_opts(status=status))
    assert int(status.item()) == 6 and small.lens[0][:, 0].tolist() == [8, 0]


def test_decode_with_an_empty_packed_unit(sqa):
    """Packed units where one unit was given no slot at all: that unit is reported (no free slot) and its
    out rows are zeroed; its neighbours, whose slot ranges touch it on both sides, step normally.  The
    unit owns no memory, so nothing may be read through its (empty) range."""
    B, Hkv, D, b = 3, 1, 64, 6
    for empty in (0, 1, 2):                      # first, middle and last unit of the layer
        caps = [b, b, b]
        caps[empty] = 0
        caches = sqa.LayerCaches([b], [b], B, Hkv, D, torch.float32, DEV, True, unit_capacities=[caps])
        ws = sqa.decode_workspace(caches, Hkv, "h2o")
        r = np.random.default_rng(empty)
        state = {u: O.new_cache(np.zeros((0, D)), np.zeros((0, D))) for u in range(B) if u != empty}
        for t in range(3):
            q = torch.from_numpy(r.standard_normal((1, B, Hkv, D)).astype(np.float32)).to(DEV)
            k = torch.from_numpy(r.standard_normal((1, B, Hkv, D)).astype(np.float32)).to(DEV)
            v = torch.from_numpy(r.standard_normal((1, B, Hkv, D)).astype(np.float32)).to(DEV)
            out = torch.full_like(q, 5.0)
            sqa.decode_step(q, k, v, t, "h2o", 4, caches, out, ws)
            assert sqa.read_device_status(ws) == 6           # SQA_ERR_CAPACITY, from the empty unit
            assert bool((out[0, empty] == 0).all()) and int(caches.lens[0][empty, 0]) == 0
            for u in state:
                want, state[u] = O.decode_step(state[u], np64(q)[0, u], np64(k)[0, u, 0], np64(v)[0, u, 0], t, b, "h2o")
                assert rel_err(np64(out)[0, u], want) < 1e-5
                assert export_state(caches, 0, u, 0)["pos"].tolist() == state[u]["pos"].tolist()


@pytest.mark.parametrize("blocked", [True, False], ids=["blocked", "dense"])
def test_a_new_sequence_takes_a_finished_ones_place(sqa, blocked):
    """A running batch of three sequences: after some decode steps sequence 1 is finished and another prompt,
    with its own length and its own per-layer budgets, takes its batch slot.  With blocked allocation the
    leaving sequence's K/V blocks go back to the layer's free list (sqa_block_pool) and the newcomer is dealt
    blocks from it -- in another order, more of them in one layer and fewer in the other -- without anything
    of the other sequences moving.  Only the newcomer's prompt is compressed
    (a batch-of-one call on the same memory); every sequence is checked against the oracle throughout."""
    dtype, L, Hkv, g, D, B, P, S = "bf16", 2, 2, 2, 128, 3, 120, 14
    Hq = Hkv * g
    policy, join_at = "h2o", 6
    budget_a = [[50, 50, 50], [90, 90, 90]]                     # [L][B] before the change
    new_len, new_budget = 77, [64, 40]                          # the newcomer: prompt length and budgets per layer
    layer_budget = [64, 90]
    wl = W.scaled(W.WORKLOADS["tiny"], L=L, Hq=Hq, Hkv=Hkv, D=D, B=B, P=P, S=S, dtype=dtype, policy=policy)
    wl2 = W.scaled(wl, B=1, P=new_len)
    caps = [min(b, P + S) for b in layer_budget]
    caches = sqa.LayerCaches(layer_budget, caps, B, Hkv, D, torch.bfloat16, DEV, True, blocked=blocked, block_seed=3,
                             spare_blocks=12)
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, DEV)
    bseq = _i32(budget_a)
    Ks, Vs, Ss, qkv = [], [], [], []
    for l in range(L):
        K, V = W.prompt_kv(wl, l, DEV, u_dirs, mask)
        Ks.append(K); Vs.append(V)
        Ss.append(sqa.prefill_scores(W.prompt_q(wl, l, DEV, u_dirs), K))
        qkv.append(W.decode_qkv(wl, l, DEV, u_dirs, mask))
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    sqa.prefill_compress_layers(Ks, Vs, Ss, policy, 4, caches, opts=sqa.batch_opts(budget_seq=bseq, status=status))
    assert int(status.item()) == 0
    state = {(l, b, h): O.prefill_compress(np64(Ks[l])[b, h], np64(Vs[l])[b, h], np64(Ss[l])[b, h], budget_a[l][b], policy, 4)
             for l in range(L) for b in range(B) for h in range(Hkv)}
    q_all = torch.stack([x[0] for x in qkv], 1).contiguous()
    k_all = torch.stack([x[1] for x in qkv], 1).contiguous()
    v_all = torch.stack([x[2] for x in qkv], 1).contiguous()
    qn, kn, vn = np64(q_all), np64(k_all), np64(v_all)
    ws = sqa.decode_workspace(caches, Hq, policy)
    budget_now = [row[:] for row in budget_a]
    pos_now = [P, P, P]
    out = torch.empty(L, B, Hq, D, dtype=torch.bfloat16, device=DEV)
    worst = 0.0
    for t in range(S):
        if t == join_at:
            # ---- sequence 1 leaves, the newcomer takes batch slot 1 ---------------------------------------
            Kn, Vn, Sn = [], [], []
            for l in range(L):
                K2, V2 = W.prompt_kv(wl2, l, DEV, u_dirs, W.hh_mask(wl2, DEV))
                K2 = (K2.float() + 0.5).to(torch.bfloat16)              # (other values than the first prompts')
                Kn.append(K2); Vn.append(V2)
                Sn.append(sqa.prefill_scores(W.prompt_q(wl2, l, DEV, u_dirs), K2))
            if blocked:
                for l in range(L):
                    tbl = caches.block_table[l]
                    n_blocks = caches.K[l].shape[0]
                    # the layer's free list (sqa_block_pool), brought to the state of the running batch: every
                    # block taken, the spare ones (in no unit's table row) given back
                    pool = sqa.BlockPool(n_blocks)
                    pool.take(n_blocks)
                    in_use = set(tbl.flatten().tolist())
                    pool.give(sorted(set(range(n_blocks)) - in_use))
                    leaving = tbl[1 * Hkv:2 * Hkv].flatten().tolist()
                    pool.give(leaving)                                                 # sequence 1 gives its blocks back
                    need = (min(new_budget[l], new_len + S) + sqa.SQA_BLOCK_SLOTS - 1) // sqa.SQA_BLOCK_SLOTS
                    for h in range(Hkv):
                        mine = pool.take(need)                                         # last given back, first reused
                        tbl[1 * Hkv + h, :need] = torch.tensor(mine, dtype=torch.int32, device=DEV)
                        tbl[1 * Hkv + h, need:] = -1                                   # (never read: beyond the unit's budget)
                    assert pool.free_count() == n_blocks - len(in_use) + len(leaving) - Hkv * need
                    pool.close()
            budget_now = [[budget_a[l][0], new_budget[l], budget_a[l][2]] for l in range(L)]
            bseq = _i32(budget_now)
            one = sqa.batch_opts(budget_seq=_i32([[new_budget[l]] for l in range(L)]), status=status)
            sqa.prefill_compress_layers(Kn, Vn, Sn, policy, 4, caches, opts=one, table=caches.sequence_table(1))
            assert int(status.item()) == 0
            for l in range(L):
                for h in range(Hkv):
                    state[l, 1, h] = O.prefill_compress(np64(Kn[l])[0, h], np64(Vn[l])[0, h], np64(Sn[l])[0, h],
                                                        new_budget[l], policy, 4)
                    got = export_state(caches, l, 1, h)
                    assert got["pos"].tolist() == state[l, 1, h]["pos"].tolist()
                    assert np.array_equal(got["K"], state[l, 1, h]["K"]) and np.array_equal(got["score"], state[l, 1, h]["score"])
            pos_now[1] = new_len
        # every step: the GPU runs on its own state, the oracle steps from the exported state
        before = {key: export_state(caches, *key) for key in state}
        sqa.decode_step(q_all[t], k_all[t], v_all[t], 0, policy, 4, caches, out, ws,
                        opts=sqa.batch_opts(budget_seq=bseq, new_pos_seq=_i32(pos_now)))
        assert sqa.read_device_status(ws) == 0
        o = np64(out)
        for (l, b, h) in state:
            want, c2 = O.decode_step(before[l, b, h], qn[t, l, b, h * g:(h + 1) * g], kn[t, l, b, h], vn[t, l, b, h],
                                     pos_now[b], budget_now[l][b], policy, 4)
            got = export_state(caches, l, b, h)
            assert got["pos"].tolist() == c2["pos"].tolist(), (t, l, b, h)
            assert np.array_equal(got["K"], c2["K"]) and np.array_equal(got["V"], c2["V"]), (t, l, b, h)
            check_step_scores(got, before[l, b, h], c2, False, (t, l, b, h))
            worst = max(worst, rel_err(o[l, b, h * g:(h + 1) * g], want))
        pos_now = [p + 1 for p in pos_now]
    assert worst < TOL[dtype]
    if blocked:                                                  # no block belongs to two units
        for l in range(L):
            used = [x for x in caches.block_table[l].flatten().tolist() if x >= 0]
            need1 = (min(new_budget[l], new_len + S) + 15) // 16
            assert len(set(used)) == len(used) and len(used) == 2 * Hkv * caches.block_table[l].shape[1] + Hkv * need1


def test_packed_units_smaller_than_the_layer_budget_and_next_to_the_prompt(sqa):
    """Two things the host cannot know with packed units and per-sequence values, and must therefore not
    refuse: (1) the largest unit of a layer may have fewer slots than min(P, the layer's budget) -- a long
    prompt with a small budget beside a short prompt with a large one; (2) the packed cache ends at
    unit_offset[B*Hkv], far before B*Hkv*capacity rows, so a prompt tensor that follows it directly in memory
    does not overlap it.  (Both were rejected with SQA_ERR_CAPACITY / SQA_ERR_SHAPE before.)"""
    dtype, Hkv, D, B, P, S, policy = "bf16", 1, 128, 2, 40, 4, "sliding"
    plen, budget_seq = [40, 6], [[5, 30]]
    unit_caps = [[min(budget_seq[0][b], plen[b] + S) for b in range(B)]]          # [5, 10]: capacity 10 < min(40, 30)
    caches = sqa.LayerCaches([30], [max(unit_caps[0])], B, Hkv, D, torch.bfloat16, DEV, True, unit_capacities=unit_caps)
    total = caches.total_slots(0)
    assert total == 15 and B * Hkv * caches.capacities[0] > total
    wl = W.scaled(W.WORKLOADS["tiny"], L=1, Hq=Hkv, Hkv=Hkv, D=D, B=B, P=P, S=S, dtype=dtype, policy=policy)
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, DEV)
    K0, V0 = W.prompt_kv(wl, 0, DEV, u_dirs, mask)
    # one buffer: the 15 rows of the packed K cache, then the prompt's K rows right behind them
    big = torch.zeros(total + B * Hkv * P, D, dtype=torch.bfloat16, device=DEV)
    Kp = big[total:].view(B, Hkv, P, D)
    Kp.copy_(K0)
    caches.K[0] = big[:total]
    caches.table[0].K = caches.K[0].data_ptr()
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    opts = sqa.batch_opts(prompt_len=_i32(plen), budget_seq=_i32(budget_seq), status=status)
    sqa.prefill_compress_layers([Kp], [V0], None, policy, wl.n_sink, caches, opts=opts)
    assert int(status.item()) == 0
    assert torch.equal(Kp, K0)                                                   # the prompt behind the cache is untouched
    Kn, Vn = np64(K0), np64(V0)
    for b in range(B):
        want = O.prefill_compress(Kn[b, 0, :plen[b]], Vn[b, 0, :plen[b]], None, budget_seq[0][b], policy, wl.n_sink)
        got = export_state(caches, 0, b, 0)
        assert got["pos"].tolist() == want["pos"].tolist()
        assert np.array_equal(got["K"], want["K"]) and np.array_equal(got["V"], want["V"])
