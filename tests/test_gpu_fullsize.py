"""Full-size parity in the launch configuration bench.py times (one decode
launch over all layers of the workload), on sampled outputs the oracle can
compute one by one, teacher-forced per step: the oracle's state before step t
(scores rounded once to the fp32 the accumulator stores) is imported into the
sampled units, the GPU runs the step for the WHOLE batch, and the sampled
units are compared.  Plus properties that hold for every unit at any size."""
import numpy as np
import pytest
import torch

from oracle import sqa_oracle as O
from paper_2404_04793_amd import workloads as W
from tests.harness import (TOL, carried_victim_pos, check_step_scores, clustering_margin, export_light, export_state,
                           import_state, near_tie_swap, np64, oracle_next_victim_pos, oracle_view, rel_err,
                           round_scores_f32, uses_matrix_cores)

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_fullsize(wl, sample_layers, units, check_steps, cos_layers, order="evict_then_attend", probe_tokens=None,
                  blocked=False):
    """check_steps are teacher-forced (the oracle's state is written into the sampled units first, which also
    discards the eviction decision the unit carried: the kernel decides afresh); at every other step the test
    only READS the sampled units' state before the step and lets the oracle take the same step from it, so the
    state the GPU carries from step to step -- ring position, carried eviction decision -- is what is checked."""
    from paper_2404_04793_amd import binding as sqa
    from paper_2404_04793_amd.session import Session
    sess = Session(wl, DEV, keep_prompt_q=True, order=order, probe_tokens=probe_tokens, blocked=blocked)
    ae = order == "attend_then_evict"
    g, tol = wl.g, TOL[wl.dtype]
    h2o = wl.policy == "h2o"
    mc = uses_matrix_cores(wl.dtype, wl.D, g)

    # ---- probe + budgets --------------------------------------------------
    cos = np.array(sess.probe_and_allocate(), dtype=np.float32)
    for l in cos_layers:
        ref = O.layer_importance(np64(sess.h_in[l:l + 1]), np64(sess.h_out[l:l + 1]))[0]
        assert abs(float(cos[l]) - ref) / max(abs(ref), 1e-3) < 1e-5, (l, cos[l], ref)
    want_b, want_g = O.allocate_budgets(cos, wl.total_budget, wl.p)
    assert sess.budgets == want_b and sess.groups == want_g and sum(want_b) == wl.total_budget
    budgets = sess.budgets
    # budgets from GPU cosines may only be compared when fp32 noise cannot flip the clustering
    assert clustering_margin(cos) > 1e-6, clustering_margin(cos)

    # ---- prompt scores + compression on sampled units -----------------------
    sample = [(l, b, h) for l in sample_layers for (b, h) in units]
    state = {}
    for (l, b, h) in sample:
        Kn, Vn = np64(sess.Kp[l][b, h]), np64(sess.Vp[l][b, h])
        if h2o:
            s_ref = O.prefill_scores(np64(sess.Qp[l][b, h * g:(h + 1) * g]), Kn)
            assert rel_err(np64(sess.scores[l][b, h])[None], s_ref[None]) < tol
            s32 = s_ref.astype(np.float32)
            sess.scores[l][b, h] = torch.from_numpy(s32).to(DEV)      # both sides select on these
            s0 = s32.astype(np.float64)
        else:
            s0 = np.zeros(wl.P)
        state[l, b, h] = O.prefill_compress(Kn, Vn, s0, budgets[l], wl.policy, wl.n_sink)
    sess.Qp = None
    sess.compress_prompt()
    for key, c in state.items():
        got = export_state(sess.caches, *key)
        assert got["pos"].tolist() == c["pos"].tolist(), key
        assert np.array_equal(got["K"], c["K"]) and np.array_equal(got["V"], c["V"])
        if h2o:
            assert np.array_equal(got["score"], c["score"])
    for l in range(wl.L):
        assert bool((sess.caches.lens[l] == min(wl.P, budgets[l])).all())
    # what the run holds resident is what the size model says for these budgets
    if not blocked:                                        # (pools hold whole 16-row blocks and a few spare ones)
        assert sess.resident_kv_bytes() == W.squeezed_cache_bytes(wl, budgets)

    # ---- decode: the GPU runs every step for the whole batch ---------------------
    qn = {k: np64(sess.q[:, k[0], k[1], k[2] * g:(k[2] + 1) * g]) for k in sample}
    kn = {k: np64(sess.k_new[:, k[0], k[1], k[2]]) for k in sample}
    vn = {k: np64(sess.v_new[:, k[0], k[1], k[2]]) for k in sample}
    rows = {k: (np.concatenate([np64(sess.Kp[k[0]][k[1], k[2]]), kn[k]]),
                np.concatenate([np64(sess.Vp[k[0]][k[1], k[2]]), vn[k]])) for k in sample}     # K, V rows by position
    worst_out, worst_sc = 0.0, 0.0
    seen = {"leaver_goes": 0, "heavy_goes": 0, "near_ties": 0}
    first_divergence = None
    for t in range(wl.S):
        teacher = t in check_steps
        if teacher:
            for key, c in state.items():
                import_state(sess.caches, key[0], key[1], key[2], c)
            before = dict(state)
        else:
            before = {key: export_light(sess.caches, *key, *rows[key]) for key in sample}
            for key in sample:                  # information only: where the run on its own left the teacher's path
                if first_divergence is None and before[key]["pos"].tolist() != state[key]["pos"].tolist():
                    first_divergence = (t, key)
        sess.decode(steps=1, start=t)
        for key in sample:
            l, b, h = key
            c = before[key]
            args = (qn[key][t], kn[key][t], vn[key][t], wl.P + t)
            want_out, c2 = O.decode_step(oracle_view(c), *args, budgets[l], wl.policy, wl.n_sink, order)
            state[key] = round_scores_f32(c2)
            got = export_state(sess.caches, l, b, h) if teacher else export_light(sess.caches, l, b, h, *rows[key])
            worst_out = max(worst_out, rel_err(np64(sess.out[t, l, b, h * g:(h + 1) * g]), want_out))
            if ae and h2o and got["pos"].tolist() != c2["pos"].tolist():
                # decided on scores updated in this very step (fp32 there, fp64 here): only two candidates the
                # arithmetic cannot tell apart may be swapped
                _, full = O.decode_step(oracle_view(c), *args, 1 << 30, wl.policy, wl.n_sink, order)
                bl = budgets[l]
                assert near_tie_swap(got["pos"].tolist(), c2["pos"].tolist(), c, full, bl - bl // 2, mc), (key, t)
                seen["near_ties"] += 1
                continue
            assert got["pos"].tolist() == c2["pos"].tolist(), (key, t)
            if teacher:
                assert np.array_equal(got["K"], c2["K"]) and np.array_equal(got["V"], c2["V"]), (key, t)
            if h2o:
                worst_sc = max(worst_sc, check_step_scores(got, c, c2, mc, (key, t)))
                if not teacher and not ae and len(got["pos"]) == budgets[l]:
                    carried = carried_victim_pos(got, budgets[l])
                    assert carried is not None and carried == oracle_next_victim_pos(got, budgets[l]), (key, t, got["hint"])
                    seen["leaver_goes" if got["hint"] == -1 else "heavy_goes"] += 1
    print("%s %s: worst out %.2e (allowed %.0e), worst score error %.2f of its bound, %s, first step at which the "
          "free-running units differ from the teacher-forced path: %s" % (wl.name, order, worst_out, tol, worst_sc, seen, first_divergence))
    assert worst_out < tol, worst_out
    assert sqa.read_device_status(sess.dec_ws) == 0
    if h2o and not ae and len(check_steps) < wl.S:
        assert seen["leaver_goes"] + seen["heavy_goes"] > 0

    # ---- properties of every unit -------------------------------------------
    end = wl.P + wl.S
    for l in range(wl.L):
        n = min(end, budgets[l])
        assert bool((sess.caches.lens[l] == n).all()), l
        kept = sqa.kept_idx_sorted(sess.caches, l)[:, :, :n].to(torch.int64)
        assert bool((kept[:, :, 1:] > kept[:, :, :-1]).all())           # unique, ascending
        assert int(kept.min()) >= 0 and int(kept.max()) == end - 1
        if n == budgets[l]:
            if wl.policy == "sliding":
                rec = n
            elif wl.policy == "streaming":
                rec = n - wl.n_sink
                assert bool((kept[:, :, :wl.n_sink] == torch.arange(wl.n_sink, device=DEV)).all())  # sinks stay
            else:
                rec = n - n // 2
            want = torch.arange(end - rec, end, device=DEV)
            assert bool((kept[:, :, n - rec:] == want).all()), l           # the recent window
    assert all(bool(torch.isfinite(sess.out[t]).all()) for t in range(wl.S))
    if h2o:
        for l in range(wl.L):
            tot = sess.caches.score[l][:, :, :min(end, budgets[l])].double().sum(-1)
            assert bool((tot <= g * end * (1 + 1e-4)).all()) and bool((tot > 0).all())


def test_llama2_7b_full_size():
    """configs[1] exactly as bench.py runs it."""
    wl = W.WORKLOADS["llama2_7b"]
    _run_fullsize(wl, sample_layers=[0, 5, 17, 31], units=[(0, 0), (7, 31)],
                  check_steps={0, 1, 2, 100, 222, 223, 224, 225, 255}, cos_layers=[0, 16, 31])


def test_llama2_7b_full_size_blocked_allocation():
    """configs[1] with K and V in pools of 16-row blocks scattered by a block table (the layout a serving loop
    with sequences joining and leaving would use), 64 decode steps."""
    wl = W.scaled(W.WORKLOADS["llama2_7b"], S=64)
    _run_fullsize(wl, sample_layers=[0, 5, 31], units=[(0, 0), (7, 31)], check_steps={0, 1, 40, 63}, cos_layers=[16],
                  blocked=True)


def test_llama2_7b_full_size_attend_then_evict():
    """configs[1] in the other order of a step, 48 decode steps (the 2271-slot layers never fill, the
    143-slot layers evict from the first step on)."""
    wl = W.scaled(W.WORKLOADS["llama2_7b"], S=48)
    _run_fullsize(wl, sample_layers=[0, 5, 31], units=[(0, 0), (7, 31)], check_steps={0, 1, 2, 30, 47},
                  cos_layers=[16], order="attend_then_evict")


def test_mistral_7b_full_size():
    """configs[2] at its real batch (32) and layer count, in the launch bench.py times; 8 decode steps; the
    probe sees 4096 token rows per layer so that the hidden states stay small."""
    wl = W.scaled(W.WORKLOADS["mistral_7b"], S=8)
    _run_fullsize(wl, sample_layers=[0, 9, 20, 31], units=[(0, 0), (31, 7)], check_steps={0, 7}, cos_layers=[1, 20],
                  probe_tokens=4096)


def test_mistral_7b_full_size_under_h2o():
    """The Mistral shape at its real batch and layer count under H2O (the policy configs[2] does not use; a leg
    of bench.py): 4 query heads per KV head on the matrix cores, every unit's probabilities of a step in LDS."""
    wl = W.scaled(W.WORKLOADS["mistral_7b"], S=6, policy="h2o")
    _run_fullsize(wl, sample_layers=[0, 20], units=[(0, 0), (31, 7)], check_steps={0, 5}, cos_layers=[1],
                  probe_tokens=4096)


def test_llama2_70b_full_size():
    """configs[3] at its real batch (16) and all 80 layers, in the launch bench.py times; 8 decode steps."""
    wl = W.scaled(W.WORKLOADS["llama2_70b"], S=8)
    _run_fullsize(wl, sample_layers=[0, 40, 79], units=[(0, 0), (15, 7)], check_steps={0, 7}, cos_layers=[0, 79],
                  probe_tokens=2048)


def test_stress_7b_full_size():
    """configs[4] at its real batch (224), 70 decode steps: the 571-slot layers fill at step 59 and evict
    from then on; the 35-slot layers (one wave per unit) evict from the first step."""
    wl = W.scaled(W.WORKLOADS["stress_7b"], S=70)
    _run_fullsize(wl, sample_layers=[0, 12, 31], units=[(0, 0), (223, 31)], check_steps={0, 1, 60, 69}, cos_layers=[0, 12],
                  probe_tokens=4096)


def test_mistral_7b_gqa_streaming_reduced_batch():
    """configs[2] at batch 4 (prompt, heads, budgets and decode length as given)."""
    wl = W.scaled(W.WORKLOADS["mistral_7b"], B=4, S=64)
    _run_fullsize(wl, sample_layers=[0, 9, 20], units=[(0, 0), (3, 7)], check_steps={0, 1, 31, 63}, cos_layers=[1, 20])


def test_llama2_70b_gqa8_sliding_reduced():
    """configs[3] at batch 2, 40 layers, 32 decode steps (head shape, prompt and budgets as given)."""
    wl = W.scaled(W.WORKLOADS["llama2_70b"], B=2, S=32, L=40, hidden=2048)
    _run_fullsize(wl, sample_layers=[0, 20, 39], units=[(0, 0), (1, 7)], check_steps={0, 1, 31}, cos_layers=[0, 39])


@pytest.mark.parametrize("B,L", [(16, 24), (2, 8)])
def test_llama2_70b_shape_gqa8_h2o(B, L):
    """The 70B head shape, prompt and budgets under H2O (the policy configs[3] does not use): 8 query heads per KV
    head accumulate into one score per token.  Batch 16: the 3439-token units stay whole (one workgroup walks
    the unit and its stored probabilities); batch 2: the same units are split over several workgroups."""
    wl = W.scaled(W.WORKLOADS["llama2_70b"], B=B, S=12, L=L, hidden=1024, policy="h2o")
    _run_fullsize(wl, sample_layers=[0, L // 2, L - 1], units=[(0, 0), (B - 1, 7)], check_steps={0, 1, 11},
                  cos_layers=[0, L - 1])


def test_stress_7b_reduced_batch():
    """configs[4] at batch 16, 128 decode steps (short prompt, small budgets: 35 / 571)."""
    wl = W.scaled(W.WORKLOADS["stress_7b"], B=16, S=128)
    _run_fullsize(wl, sample_layers=[0, 12, 30], units=[(0, 0), (15, 31)], check_steps={0, 1, 59, 60, 61, 127},
                  cos_layers=[0, 12])


def test_llama2_7b_ragged_batch():
    """configs[1] with prompt lengths from 2048 down to 1152: per-sequence cosines and budgets, ragged
    scores and compression, per-sequence positions -- the path `bench.py --ragged` times."""
    from paper_2404_04793_amd import binding as sqa
    from paper_2404_04793_amd.session import Session
    wl = W.scaled(W.WORKLOADS["llama2_7b"], S=24)
    plen = [wl.P - (b * wl.P) // (2 * wl.B) for b in range(wl.B)]
    sess = Session(wl, DEV, keep_prompt_q=True, prompt_len=plen)
    g, tol = wl.g, TOL[wl.dtype]
    sess.probe_and_allocate()
    starts = np.concatenate([[0], np.cumsum(plen)])
    cos = sqa.layer_importance_seq(sess.h_in, sess.h_out, sess.seq_start).cpu().numpy()
    for l, b in [(0, 0), (17, 3), (31, 7)]:
        ref = O.layer_importance(np64(sess.h_in[l:l + 1, starts[b]:starts[b + 1]]),
                                 np64(sess.h_out[l:l + 1, starts[b]:starts[b + 1]]))[0]
        assert abs(float(cos[l, b]) - ref) / max(abs(ref), 1e-3) < 1e-5
    for b in range(wl.B):
        total = wl.L * (plen[b] * wl.budget_pct // 100)
        want = O.allocate_budgets(cos[:, b], total, wl.p)[0]
        assert [sess.budget_seq[l][b] for l in range(wl.L)] == want and sum(want) == total
    sample = [(l, b, h) for l in (0, 9, 31) for (b, h) in ((0, 0), (4, 13), (7, 31))]
    state = {}
    for (l, b, h) in sample:
        n = plen[b]
        Kn, Vn = np64(sess.Kp[l][b, h, :n]), np64(sess.Vp[l][b, h, :n])
        s_ref = O.prefill_scores(np64(sess.Qp[l][b, h * g:(h + 1) * g, :n]), Kn)
        assert rel_err(np64(sess.scores[l][b, h, :n])[None], s_ref[None]) < tol
        assert bool((sess.scores[l][b, h, n:] == 0).all())
        s32 = s_ref.astype(np.float32)
        sess.scores[l][b, h, :n] = torch.from_numpy(s32).to(DEV)
        state[l, b, h] = O.prefill_compress(Kn, Vn, s32.astype(np.float64), sess.budget_seq[l][b], wl.policy, wl.n_sink)
    sess.compress_prompt()
    assert int(sess.status.item()) == 0
    for key, c in state.items():
        got = export_state(sess.caches, *key)
        assert got["pos"].tolist() == c["pos"].tolist(), key
        assert np.array_equal(got["K"], c["K"]) and np.array_equal(got["score"], c["score"])
    check = {0, 1, 23}
    worst = 0.0
    for t in range(wl.S):
        if t in check:
            for key, c in state.items():
                import_state(sess.caches, key[0], key[1], key[2], c)
        sess.decode(steps=1, start=t)
        for (l, b, h) in sample:
            state_before = state[l, b, h]
            want_out, c2 = O.decode_step(state_before, np64(sess.q[t, l, b, h * g:(h + 1) * g]), np64(sess.k_new[t, l, b, h]),
                                         np64(sess.v_new[t, l, b, h]), plen[b] + t, sess.budget_seq[l][b], wl.policy, wl.n_sink)
            state[l, b, h] = round_scores_f32(c2)
            if t in check:
                got = export_state(sess.caches, l, b, h)
                assert got["pos"].tolist() == c2["pos"].tolist(), (l, b, h, t)
                assert np.array_equal(got["K"], c2["K"]) and np.array_equal(got["V"], c2["V"])
                check_step_scores(got, state_before, c2, False, (l, b, h, t))
                worst = max(worst, rel_err(np64(sess.out[t, l, b, h * g:(h + 1) * g]), want_out))
    assert worst < tol and sqa.read_device_status(sess.dec_ws) == 0
    for l in range(wl.L):                                    # every unit: its own length and newest position
        kept_all = sqa.kept_idx_sorted(sess.caches, l)       # packed like pos: unit u starts at unit_offset[u]
        off = sess.caches.offsets_host[l]
        for b in range(wl.B):
            n = min(plen[b] + wl.S, sess.budget_seq[l][b])
            assert bool((sess.caches.lens[l][b] == n).all())
            for h in range(wl.Hkv):
                lo = off[b * wl.Hkv + h]
                assert off[b * wl.Hkv + h + 1] - lo == n     # exact fit
                kept = kept_all[lo:lo + n]
                assert int(kept[-1]) == plen[b] + wl.S - 1 and bool((kept[1:] > kept[:-1]).all())
    dense = sum(wl.B * wl.Hkv * c for c in sess.caches.capacities)
    assert sum(sess.caches.total_slots(l) for l in range(wl.L)) < 0.85 * dense      # the memory the packing saves
