"""GPU parity in the export direction: the library runs on its own from the compressed prompt -- nothing
is ever written into its caches by the test -- and before every step the test reads the GPU's own unit
state, lets the oracle take one step from exactly that state (Algorithm 1 steps 14-21), and compares
what the GPU holds afterwards: kept positions bit for bit, K/V rows bit for bit, accumulated scores
element by element, outputs per vector.

This is the check of what a unit carries from step to step: under H2O the kernel decides the next
eviction at the end of a step and stores it in the unit record (evict_hint); a teacher-forced test
overwrites that record, this one does not.  The decision is also compared directly: the token the record
says will go next must be the token the oracle's selection drops when the next token is appended.
Covered: the vector-ALU kernel with 4 waves per unit (whole and split units) and one wave per unit, the
matrix-core kernel (4 and 8 query heads per KV head; whole, split, one wave per unit), both orders of a
step, fp32 and bf16."""
import os

import numpy as np
import pytest
import torch

from oracle import sqa_oracle as O
from paper_2404_04793_amd import workloads as W
from tests.harness import (TOL, carried_victim_pos, check_step_scores, export_light, near_tie_swap, np64,
                           oracle_next_victim_pos, oracle_view, rel_err, unit_kv, uses_matrix_cores)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sqa():
    from paper_2404_04793_amd import binding
    return binding


def _step_and_compare(sqa, caches, ws, budgets, policy, order, dtype, D, g, P, S, q_all, k_all, v_all, rows, sample,
                      n_sink=4):
    """rows[(l, b, h)] = (K rows by position [P + S, D], V rows by position) in fp64.  Returns counters."""
    ae = order == "attend_then_evict"
    opts = sqa.batch_opts(order=order) if ae else None
    mc = uses_matrix_cores(dtype, D, g)
    L, B, Hq = q_all.shape[1], q_all.shape[2], q_all.shape[3]
    qn, kn, vn = np64(q_all), np64(k_all), np64(v_all)
    out = torch.empty(L, B, Hq, D, dtype=q_all.dtype, device=DEV)
    seen = {"leaver_goes": 0, "heavy_goes": 0, "evictions": 0, "near_ties": 0, "worst_out": 0.0, "worst_score": 0.0}
    for t in range(S):
        before = {key: export_light(caches, *key, *rows[key]) for key in sample}
        sqa.decode_step(q_all[t], k_all[t], v_all[t], P + t, policy, n_sink, caches, out, ws, opts=opts)
        o = np64(out)
        for key in sample:
            l, b, h = key
            c = before[key]
            want_out, c2 = O.decode_step(oracle_view(c), qn[t, l, b, h * g:(h + 1) * g], kn[t, l, b, h], vn[t, l, b, h],
                                         P + t, budgets[l], policy, n_sink, order)
            got = export_light(caches, l, b, h, *rows[key])
            seen["worst_out"] = max(seen["worst_out"], rel_err(o[l, b, h * g:(h + 1) * g], want_out))
            if len(c["pos"]) == budgets[l]:
                seen["evictions"] += 1
            if got["pos"].tolist() != c2["pos"].tolist():
                assert ae and policy == "h2o", (t, key, sorted(set(got["pos"]) ^ set(c2["pos"])))
                _, full = O.decode_step(oracle_view(c), qn[t, l, b, h * g:(h + 1) * g], kn[t, l, b, h], vn[t, l, b, h],
                                        P + t, 1 << 30, policy, n_sink, order)
                assert near_tie_swap(got["pos"].tolist(), c2["pos"].tolist(), c, full, budgets[l] - budgets[l] // 2, mc), (t, key)
                seen["near_ties"] += 1
                continue
            # the rows the GPU holds are the rows of those positions
            n = len(got["pos"])
            Kn, Vn = unit_kv(caches, l, b, h, n)
            order_idx = np.argsort(got["raw_pos"], kind="stable")
            assert np.array_equal(Kn[order_idx], c2["K"]) and np.array_equal(Vn[order_idx], c2["V"]), (t, key)
            if policy == "h2o":
                seen["worst_score"] = max(seen["worst_score"], check_step_scores(got, c, c2, mc, (t, key)))
                if not ae and len(got["pos"]) == budgets[l]:
                    # the decision the unit carries to the next step, against the oracle's selection
                    carried = carried_victim_pos(got, budgets[l])
                    assert carried is not None, (t, key, got["hint"])
                    assert carried == oracle_next_victim_pos(got, budgets[l]), (t, key, got["hint"])
                    seen["leaver_goes" if got["hint"] == -1 else "heavy_goes"] += 1
                if ae:
                    assert got["hint"] == -2
    assert sqa.read_device_status(ws) == 0
    assert seen["worst_out"] < TOL[dtype], seen
    return seen


def _rows_by_position(Kp, Vp, k_all, v_all, l, b, h):
    return (np.concatenate([np64(Kp[b, h]), np64(k_all[:, l, b, h])]), np.concatenate([np64(Vp[b, h]), np64(v_all[:, l, b, h])]))


STEPPING = [
    # name, dtype, Hq, Hkv, D, B, P, S, policy, budgets, order
    # budgets: 300 = a whole unit shared by 4 waves, 700 = split into 3 chunks over 3 workgroups, 37 = shorter than one pass
    ("h2o_bf16_mha", "bf16", 2, 2, 128, 2, 750, 48, "h2o", [300, 700, 37], "evict_then_attend"),
    ("h2o_bf16_gqa4_matrix", "bf16", 8, 2, 128, 2, 750, 48, "h2o", [300, 700, 37], "evict_then_attend"),
    ("h2o_bf16_gqa8_matrix", "bf16", 16, 2, 128, 2, 750, 48, "h2o", [300, 700, 37], "evict_then_attend"),
    ("h2o_f32_d64_gqa2", "f32", 4, 2, 64, 1, 500, 40, "h2o", [310, 520, 21], "evict_then_attend"),
    ("h2o_bf16_mha_attend_first", "bf16", 2, 2, 128, 2, 750, 40, "h2o", [300, 700, 37], "attend_then_evict"),
    ("h2o_bf16_gqa8_matrix_attend_first", "bf16", 16, 2, 128, 2, 750, 40, "h2o", [300, 700, 37], "attend_then_evict"),
    ("streaming_bf16_gqa4_matrix", "bf16", 8, 2, 128, 1, 750, 40, "streaming", [300, 700, 37], "evict_then_attend"),
    # units that fill up while decoding (budget above the prompt length)
    ("h2o_bf16_mha_filling", "bf16", 2, 2, 128, 1, 300, 44, "h2o", [310, 330, 400], "evict_then_attend"),
]


@pytest.mark.parametrize("case", STEPPING, ids=[c[0] for c in STEPPING])
def test_stepping_from_the_gpus_own_state(sqa, case):
    _run_case(sqa, case)


@pytest.mark.parametrize("order", ["evict_then_attend", "attend_then_evict"])
def test_stepping_whole_long_units_in_a_small_call(sqa, order):
    """208 units of 600 slots in one call: few enough workgroups that units stay whole although they are
    long, and that all four waves of a workgroup stay for the unit's tail (score update, eviction
    decision) instead of leaving it to the first wave."""
    _run_case(sqa, ("h2o_bf16_mha_whole_long_units", "bf16", 8, 8, 128, 26, 640, 24, "h2o", [600], order), stride=19)


def test_stepping_matrix_core_units_at_the_lds_limit(sqa):
    """8 query heads per KV head, 208 whole units per layer.  1050 slots: the largest units whose per-head
    probabilities of a step (33 tiles x 8 heads x 68 bytes) all fit in LDS next to the stage buffers; 1200 and
    2300 slots: the leading 33 tiles stay in LDS, the other 5 / 39 pass through the workspace."""
    _run_case(sqa, ("h2o_bf16_gqa8_matrix_lds_limit", "bf16", 64, 8, 128, 26, 2400, 10, "h2o", [1050, 1200, 2300],
                    "evict_then_attend"), stride=37)


def test_stepping_matrix_core_long_units_attend_first_blocked(sqa):
    """The same split of a unit's probabilities between LDS and workspace under attend-then-evict, with K and V
    in 16-row blocks (the staged block numbers take their share of the LDS: 32 tiles stay)."""
    _run_case(sqa, ("h2o_bf16_gqa8_matrix_lds_limit_ae", "bf16", 64, 8, 128, 26, 1500, 8, "h2o", [1100, 1400],
                    "attend_then_evict"), stride=41, blocked=True)


@pytest.mark.parametrize("case", [STEPPING[0], STEPPING[2], STEPPING[3], STEPPING[5], STEPPING[7]],
                         ids=[STEPPING[i][0] for i in (0, 2, 3, 5, 7)])
def test_stepping_with_blocked_allocation(sqa, case):
    """K and V rows in 16-row blocks of shared pools, the blocks of a unit scattered by a block table."""
    _run_case(sqa, case, blocked=True)


def _run_case(sqa, case, stride=1, blocked=False, need_both_outcomes=True):
    """need_both_outcomes: the case is built so that units evict and, under H2O, both results of the carried
    decision occur (the random shapes make no such promise: a budget above everything never evicts)."""
    name, dtype, Hq, Hkv, D, B, P, S, policy, budgets, order = case
    L, g = len(budgets), Hq // Hkv
    wl = W.scaled(W.WORKLOADS["tiny"], L=L, Hq=Hq, Hkv=Hkv, D=D, B=B, P=P, S=S, dtype=dtype, policy=policy)
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, DEV)
    Kp, Vp, qkv = [], [], []
    caches = sqa.LayerCaches(budgets, [min(b, P + S) for b in budgets], B, Hkv, D, wl.torch_dtype, DEV, True,
                             blocked=blocked, block_seed=P + S)
    for l in range(L):
        K, V = W.prompt_kv(wl, l, DEV, u_dirs, mask)
        Kp.append(K); Vp.append(V)
        sc = sqa.prefill_scores(W.prompt_q(wl, l, DEV, u_dirs), K) if policy == "h2o" else None
        sqa.prefill_compress(K, V, sc, policy, wl.n_sink, caches, l)
        qkv.append(W.decode_qkv(wl, l, DEV, u_dirs, mask))
    q_all = torch.stack([x[0] for x in qkv], 1).contiguous()
    k_all = torch.stack([x[1] for x in qkv], 1).contiguous()
    v_all = torch.stack([x[2] for x in qkv], 1).contiguous()
    sample = [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)][::stride]
    rows = {key: _rows_by_position(Kp[key[0]], Vp[key[0]], k_all, v_all, *key) for key in sample}
    ws = sqa.decode_workspace(caches, Hq, policy)
    seen = _step_and_compare(sqa, caches, ws, budgets, policy, order, dtype, D, g, P, S, q_all, k_all, v_all, rows, sample,
                             wl.n_sink)
    print(name, order, seen)
    if not need_both_outcomes:
        return
    assert seen["evictions"] > 0
    if policy == "h2o" and order == "evict_then_attend":
        assert seen["leaver_goes"] > 0 and seen["heavy_goes"] > 0, seen       # both outcomes of the carried decision


@pytest.mark.parametrize("dtype,D,g,order,blocked", [
    ("bf16", 128, 1, "evict_then_attend", False), ("bf16", 128, 4, "evict_then_attend", False),
    ("bf16", 128, 8, "evict_then_attend", False), ("bf16", 128, 8, "attend_then_evict", False),
    ("f32", 64, 1, "evict_then_attend", False), ("bf16", 128, 1, "evict_then_attend", True),
    ("bf16", 128, 8, "evict_then_attend", True)])
def test_stepping_one_wave_per_unit(sqa, dtype, D, g, order, blocked):
    """4096 short units in one call: every wave owns a unit and carries its eviction decision alone.
    40 steps on the GPU's own state, a sample of units against the oracle every step."""
    policy, B, Hkv, L, P, S = "h2o", 64, 8, 8, 40, 40
    Hq = Hkv * g
    budgets = [6, 17, 33, 40, 41, 64, 200, 9]
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    gen = torch.Generator(device="cpu").manual_seed(1000 + 10 * D + g)
    mk = lambda *shape: torch.randn(*shape, generator=gen).to(tdt).to(DEV)
    Ks, Vs = [mk(B, Hkv, P, D) for _ in range(L)], [mk(B, Hkv, P, D) for _ in range(L)]
    Ss = [torch.rand(B, Hkv, P, generator=gen).to(DEV) for _ in range(L)]
    q_all, k_all, v_all = mk(S, L, B, Hq, D), mk(S, L, B, Hkv, D), mk(S, L, B, Hkv, D)
    caches = sqa.LayerCaches(budgets, [min(b, P + S) for b in budgets], B, Hkv, D, tdt, DEV, True, blocked=blocked)
    sqa.prefill_compress_layers(Ks, Vs, Ss, policy, 4, caches)
    ws = sqa.decode_workspace(caches, Hq, policy)
    units = [(l, b, h) for l in range(L) for b in range(B) for h in range(Hkv)]
    sample = units[::151] + units[-2:]
    rows = {key: _rows_by_position(Ks[key[0]], Vs[key[0]], k_all, v_all, *key) for key in sample}
    seen = _step_and_compare(sqa, caches, ws, budgets, policy, order, dtype, D, g, P, S, q_all, k_all, v_all, rows, sample)
    print(dtype, D, g, order, seen)
    assert seen["evictions"] > 0
    if order == "evict_then_attend":
        assert seen["leaver_goes"] > 0 and seen["heavy_goes"] > 0, seen


def _random_stepping_cases(n, seed=808):
    """Seeded random larger shapes: prompts to 2100 tokens, 1-3 layers, 1-208 units, every group size and policy,
    both orders, dense or blocked rows; about six units of each are followed."""
    r = np.random.default_rng(seed)
    out = []
    for k in range(n):
        dtype = ["bf16", "bf16", "f32"][int(r.integers(3))]
        D = 128 if dtype == "bf16" and r.integers(4) else [64, 128][int(r.integers(2))]
        g = [1, 2, 4, 8][int(r.integers(4))]
        Hkv, B = int(r.choice([1, 2, 4, 8])), int(r.choice([1, 2, 4, 13, 26]))
        P, S = int(r.choice([200, 330, 700, 1250, 2100])), int(r.integers(6, 14))
        policy = ["h2o", "h2o", "sliding", "streaming"][int(r.integers(4))]
        lo = {"sliding": 1, "streaming": 5, "h2o": 2}[policy]
        budgets = [int(max(lo, r.choice([r.integers(lo, 70), r.integers(100, min(400, P)), r.integers(min(400, P - 1), P),
                                         P - 3, P + 2]))) for _ in range(int(r.integers(1, 4)))]
        order = ["evict_then_attend", "attend_then_evict"][int(r.integers(2))]
        blocked = bool(r.integers(2))
        out.append((("step%02d_%s_%s_D%d_g%d" % (k, policy, dtype, D, g), dtype, Hkv * g, Hkv, D, B, P, S, policy, budgets, order),
                    max(1, B * Hkv * len(budgets) // 6), blocked))
    return out


# (SQA_RANDOM_CASES=1500 python -m pytest tests/test_gpu_stepping.py -m gpu -k random  runs a longer campaign)
RANDOM_STEPPING = _random_stepping_cases(max(1, int(os.environ.get("SQA_RANDOM_CASES", "28")) // 4))


@pytest.mark.parametrize("case,stride,blocked", RANDOM_STEPPING, ids=[c[0][0] for c in RANDOM_STEPPING])
def test_stepping_random_shapes(sqa, case, stride, blocked):
    _run_case(sqa, case, stride=stride, blocked=blocked, need_both_outcomes=False)
