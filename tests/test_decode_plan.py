"""The launch plan of the decode step (sqa_decode_plan: host arithmetic, no GPU): the configurations that
bench.py times and the profiles describe, and invariants over random shapes."""
import ctypes as C

import numpy as np
import pytest

from paper_2404_04793_amd import binding as sqa
from paper_2404_04793_amd import workloads as W

# budgets of the five workloads (their group sizes and the budget rule are pinned in the oracle tests)
BUDGETS = {
    "llama2_7b": [2271, 2271] + [143] * 28 + [2271, 2271],
    "stress_7b": [571, 571] + [35] * 28 + [571, 571],
    "mistral_7b": [1987] * 2 + [1987] * 14 + [368] * 15 + [1987],          # 17 important layers, 15 unimportant
    "llama2_70b": [3439] * 10 + [491] * 27 + [3439] + [491] * 15 + [3439] + [491] * 18 + [3439] * 8,
}


def _plan(name, policy=None, blocked=False, layers=None):
    wl = W.WORKLOADS[name]
    b = BUDGETS[name] if layers is None else [BUDGETS[name][i] for i in layers]
    assert layers is not None or len(b) == wl.L
    caps = [min(x, wl.P + wl.S) for x in b]
    return sqa.decode_plan(b, caps, wl.B, wl.Hq, wl.Hkv, wl.D, "bf16", policy or wl.policy, blocked), b, wl


def test_llama2_7b_launch_is_the_one_the_profile_describes():
    p, b, wl = _plan("llama2_7b")
    units = wl.B * wl.Hkv
    assert p["workgroups"] == 4 * units + 28 * units // 4 == 2816           # whole long units, four short units per workgroup
    assert p["matrix_cores"] == 0 and p["wide_tail"] == 0 and p["table_entries"] == 0
    for lay, x in zip(p["layers"], b):
        assert lay["wave_per_unit"] == (1 if x == 143 else 0)
        assert lay["workgroups_per_unit"] == (0 if x == 143 else 1)         # no unit is split
    assert p["lds_bytes"] == 2304 * 4                                        # the step's logits of one 2271-token unit
    one, _, _ = _plan("llama2_7b", layers=[0])
    assert one["workgroups"] == units and one["wide_tail"] == 1 and one["layers"][0]["workgroups_per_unit"] == 1
    short, _, _ = _plan("llama2_7b", layers=[5])
    assert short["workgroups"] == units and short["layers"][0]["wave_per_unit"] == 0   # 256 units: too few for one wave each


def test_stress_mistral_70b_launches():
    p, b, wl = _plan("stress_7b")
    units = wl.B * wl.Hkv
    assert p["workgroups"] == 4 * units + 28 * units // 4 == 78848
    p, b, wl = _plan("mistral_7b")
    assert p["matrix_cores"] == 1 and p["workgroups"] == 32 * wl.B * wl.Hkv == 8192
    assert all(l["workgroups_per_unit"] == 1 and l["probs_in_lds"] == 0 for l in p["layers"])
    p, b, wl = _plan("llama2_70b")
    assert p["matrix_cores"] == 1 and p["workgroups"] == 80 * wl.B * wl.Hkv == 10240
    # H2O with grouped queries: probabilities stay in LDS where 2 bytes x heads x tokens fit beside the stage buffers
    p, b, _ = _plan("mistral_7b", policy="h2o")
    assert all(l["probs_in_lds"] == 1 for l in p["layers"])
    p, b, _ = _plan("llama2_70b", policy="h2o")
    # (a 3439-token unit keeps what fits -- its leading tiles -- and passes the rest through the workspace)
    assert [l["probs_in_lds"] for l in p["layers"]] == [1 if x == 491 else 2 for x in b]
    assert p["lds_bytes"] <= 160 * 1024 // 3                                  # three workgroups per CU


def test_blocked_allocation_adds_the_staged_table():
    dense, b, _ = _plan("llama2_7b")
    blk, _, _ = _plan("llama2_7b", blocked=True)
    assert blk["table_entries"] == (2271 + 15) // 16
    assert blk["lds_bytes"] == dense["lds_bytes"] + 4 * blk["table_entries"]
    assert blk["workgroups"] == dense["workgroups"]
    small = sqa.decode_plan([35] * 32, [35] * 32, 224, 32, 32, 128, "bf16", "h2o", True)
    assert small["table_entries"] == 4 * (256 // 16) or small["table_entries"] >= 4 * 3   # a row per wave


@pytest.mark.parametrize("seed", range(60))
def test_plan_invariants_on_random_shapes(seed):
    r = np.random.default_rng(seed)
    L = int(r.integers(1, 81))
    Hkv = int(r.choice([1, 2, 4, 8, 32]))
    g = int(r.choice([1, 2, 4, 8]))
    B = int(r.choice([1, 2, 8, 16, 64, 224]))
    D = int(r.choice([64, 128]))
    dtype = str(r.choice(["bf16", "f32"]))
    policy = str(r.choice(["h2o", "sliding", "streaming"]))
    budgets = [int(x) for x in r.choice([8, 35, 143, 368, 571, 2271, 3439, 9000, 40000], size=L)]
    caps = [min(b, int(r.choice([b, b, 300, 5000]))) for b in budgets]
    blocked = bool(r.integers(0, 2)) and max(min(b, c) for b, c in zip(budgets, caps)) <= 16 * 1024
    try:
        p = sqa.decode_plan(budgets, caps, B, g * Hkv, Hkv, D, dtype, policy, blocked)
    except sqa.SqaError as e:
        assert e.code == 6                                                    # only: does not fit (LDS, counters)
        return
    units = B * Hkv
    total = 0
    for lay, b, c in zip(p["layers"], budgets, caps):
        n = min(b, c) + 1                                                     # attend-then-evict attends one more
        assert lay["slots_per_workgroup"] % 64 == 0
        if lay["wave_per_unit"]:
            assert lay["workgroups_per_unit"] == 0 and n <= lay["slots_per_workgroup"] and units * L >= 4096
            total += (units + 3) // 4
        else:
            k = lay["workgroups_per_unit"]
            assert k >= 1 and k * lay["slots_per_workgroup"] >= n > (k - 1) * lay["slots_per_workgroup"]
            total += units * k
        assert not lay["probs_in_lds"] or (p["matrix_cores"] and policy == "h2o")
    assert p["workgroups"] == total
    assert p["lds_bytes"] <= 160 * 1024
    assert p["matrix_cores"] == int(dtype == "bf16" and D == 128 and g >= 4)
    assert p["wide_tail"] == int(total <= 512)
    assert (p["table_entries"] > 0) == blocked
    t = (sqa.LayerCacheStruct * L)()
    for i in range(L):
        t[i].capacity, t[i].budget = caps[i], budgets[i]
    assert p["workspace_bytes"] <= sqa._lib.sqa_decode_workspace_bytes(t, L, B, g * Hkv, Hkv, D, sqa.POLICY[policy])


def test_plan_argument_errors():
    lib = sqa._lib
    t = (sqa.LayerCacheStruct * 1)()
    t[0].capacity, t[0].budget = 8, 8
    info = sqa.DecodePlanInfo()
    call = lambda **kw: lib.sqa_decode_plan(kw.get("t", t), kw.get("n", 1), kw.get("B", 1), kw.get("Hq", 4), kw.get("Hkv", 4),
                                            kw.get("D", 128), kw.get("dt", 1), kw.get("pol", 2), kw.get("info", C.byref(info)), None)
    assert call() == 0 and info.workgroups == 4
    assert call(t=None) == 1 and call(info=None) == 1
    assert call(dt=4) == 3 and call(pol=9) == 4
    assert call(Hq=6) == 2 and call(D=100) == 2 and call(n=0) == 2 and call(B=0) == 2
    t[0].budget = 0
    assert call() == 5
    t[0].budget, t[0].capacity = 8, 0
    assert call() == 6
