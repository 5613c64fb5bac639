"""configs[0] end to end: the stored oracle run (tests/golden/tiny_end_to_end.json,
written by tests/golden/make_tiny_golden.py from the oracle alone) must be
reproduced by the oracle here (CPU) and by the HIP path running on its own (GPU)."""
import importlib.util
import json
import os

import numpy as np
import pytest
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = json.load(open(os.path.join(HERE, "golden", "tiny_end_to_end.json")))


def test_oracle_reproduces_the_stored_run():
    spec = importlib.util.spec_from_file_location("make_tiny_golden", os.path.join(HERE, "golden", "make_tiny_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    now = mod.compute()
    assert now["budgets"] == GOLD["budgets"] == [85, 17, 17, 85] and now["groups"] == GOLD["groups"]
    assert np.allclose(now["cos"], GOLD["cos"], atol=1e-7)
    assert np.allclose(GOLD["cos"], [0.4472, 0.9578, 0.9578, 0.5547], atol=5e-3)     # 1/sqrt(1+a^2), a = 2, .3, .3, 1.5
    for key, g in GOLD["units"].items():
        n = now["units"][key]
        assert n["kept_after_prefill"] == g["kept_after_prefill"] and n["kept_after_step"] == g["kept_after_step"]
        assert np.allclose(n["out_last_step_first4"], g["out_last_step_first4"], rtol=1e-8)
        l = int(key.split(",")[0])
        b = GOLD["budgets"][l]
        assert len(g["kept_after_prefill"]) == b and all(len(s) == b for s in g["kept_after_step"].values())
        # the recent half is always there, the first prompt token (causal mass >= 1) stays a heavy hitter
        assert g["kept_after_step"]["15"][-(b - b // 2):] == list(range(272 - (b - b // 2), 272))
        assert g["kept_after_step"]["15"][0] == 0


@pytest.mark.gpu
def test_hip_path_reproduces_the_stored_run():
    from paper_2404_04793_amd import binding as sqa
    from paper_2404_04793_amd import workloads as W
    from paper_2404_04793_amd.session import Session
    wl = W.WORKLOADS["tiny"]
    sess = Session(wl, "cuda:0")
    cos = sess.probe_and_allocate()
    assert np.allclose(cos, GOLD["cos"], atol=1e-5)
    assert sess.budgets == GOLD["budgets"] and sess.groups == GOLD["groups"]
    sess.compress_prompt()
    for key, g in GOLD["units"].items():
        l, h = map(int, key.split(","))
        n = len(g["kept_after_prefill"])
        assert sqa.kept_idx_sorted(sess.caches, l)[0, h, :n].cpu().tolist() == g["kept_after_prefill"]
    for t in range(wl.S):
        sess.decode(steps=1, start=t)
        kept = [sqa.kept_idx_sorted(sess.caches, l).cpu() for l in range(wl.L)]
        for key, g in GOLD["units"].items():
            l, h = map(int, key.split(","))
            if str(t) in g["kept_after_step"]:
                want = g["kept_after_step"][str(t)]
                assert kept[l][0, h, :len(want)].tolist() == want, (key, t)
    assert sqa.read_device_status(sess.dec_ws) == 0
    for key, g in GOLD["units"].items():
        l, h = map(int, key.split(","))
        got = sess.out[wl.S - 1, l, 0, h, :4].double().cpu().numpy()
        ref = np.array(g["out_last_step_first4"])
        assert np.abs(got - ref).max() < 1e-5 * max(np.abs(ref).max(), 0.05)
        tot = float(sess.caches.score[l][0, h, :sess.budgets[l]].double().sum())
        assert abs(tot - g["score_sum_end"]) < 1e-5 * g["score_sum_end"]
