"""sqa_decode_step_static -- the decode step for callers that cannot allocate (its scratch is a device array
inside the library) -- against sqa_decode_step_ex with a caller's workspace: same inputs, two copies of the
caches, every byte of out, K, V, positions, scores and unit records equal after every step.  Two runs in a
row share the library's array, the second with a smaller input whose launch plan lays the scratch out
differently (fewer layers, other split counts): stale contents of the first run must not matter.
Collected last on purpose (the file name sorts after the other tests)."""
import pytest
import torch

from paper_2404_04793_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def sqa():
    from paper_2404_04793_amd import binding
    return binding


def _inputs(wl):
    u_dirs, mask = W.unit_dirs(wl), W.hh_mask(wl, DEV)
    Kp, Vp, Qp, qkv = [], [], [], []
    for l in range(wl.L):
        K, V = W.prompt_kv(wl, l, DEV, u_dirs, mask)
        Kp.append(K); Vp.append(V); Qp.append(W.prompt_q(wl, l, DEV, u_dirs))
        qkv.append(W.decode_qkv(wl, l, DEV, u_dirs, mask))
    q = torch.stack([x[0] for x in qkv], 1).contiguous()
    k = torch.stack([x[1] for x in qkv], 1).contiguous()
    v = torch.stack([x[2] for x in qkv], 1).contiguous()
    return Kp, Vp, Qp, q, k, v


def _run_both(sqa, wl, budgets, order="evict_then_attend", blocked=False):
    """Runs wl.S steps through both entry points on separate copies of the caches and compares every byte
    after every step."""
    Kp, Vp, Qp, q_all, k_all, v_all = _inputs(wl)
    caps = [min(b, wl.P + wl.S) for b in budgets]
    h2o = wl.policy == "h2o"
    opts = None if order == "evict_then_attend" else sqa.batch_opts(order=order)
    both = []
    for _ in range(2):
        c = sqa.LayerCaches(budgets, caps, wl.B, wl.Hkv, wl.D, wl.torch_dtype, DEV, True, blocked=blocked)
        for l in range(wl.L):
            sc = sqa.prefill_scores(Qp[l], Kp[l]) if h2o else None
            sqa.prefill_compress(Kp[l], Vp[l], sc, wl.policy, wl.n_sink, c, l)
        both.append(c)
    ref, sta = both
    ws = sqa.decode_workspace(ref, wl.Hq, wl.policy)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out_ref = torch.empty(wl.L, wl.B, wl.Hq, wl.D, dtype=wl.torch_dtype, device=DEV)
    out_sta = torch.empty_like(out_ref)
    for t in range(wl.S):
        out_ref.fill_(1.0); out_sta.fill_(2.0)
        sqa.decode_step(q_all[t], k_all[t], v_all[t], wl.P + t, wl.policy, wl.n_sink, ref, out_ref, ws, opts=opts)
        sqa.decode_step_static(q_all[t], k_all[t], v_all[t], wl.P + t, wl.policy, wl.n_sink, sta, out_sta, status, opts=opts)
        torch.cuda.synchronize()
        assert torch.equal(out_ref.view(torch.int16 if wl.dtype == "bf16" else torch.int32),
                           out_sta.view(torch.int16 if wl.dtype == "bf16" else torch.int32)), t
        for l in range(wl.L):
            assert torch.equal(ref.state[l], sta.state[l]), (t, l)
            assert torch.equal(ref.pos[l], sta.pos[l]), (t, l)
            assert torch.equal(ref.score[l].view(torch.int32), sta.score[l].view(torch.int32)), (t, l)
            assert torch.equal(ref.K[l].view(torch.uint8), sta.K[l].view(torch.uint8)), (t, l)
            assert torch.equal(ref.V[l].view(torch.uint8), sta.V[l].view(torch.uint8)), (t, l)
    assert sqa.read_device_status(ws) == 0 and int(status.item()) == 0
    assert bool(torch.isfinite(out_sta.float()).all())


def test_static_scratch_entry_point_matches_the_workspace_one(sqa):
    # first run: three layers, long units split over 3 and 2 workgroups (partials, counters, H2O logits in scratch)
    big = W.scaled(W.WORKLOADS["tiny"], L=3, Hq=4, Hkv=2, D=128, B=3, P=800, S=6, dtype="bf16", policy="h2o")
    _run_both(sqa, big, [700, 41, 520])
    # second run, smaller: one layer, other chunking; the counters it uses lie where the first run's did,
    # everything else of the array still holds the first run's data
    small = W.scaled(W.WORKLOADS["tiny"], L=1, Hq=2, Hkv=2, D=64, B=2, P=450, S=5, dtype="f32", policy="h2o")
    _run_both(sqa, small, [420])
    # third: the matrix-core variant (its per-head probabilities go through the scratch for every unit),
    # the other order of a step, then a sliding-window call
    mf = W.scaled(W.WORKLOADS["tiny"], L=2, Hq=16, Hkv=2, D=128, B=2, P=700, S=4, dtype="bf16", policy="h2o")
    _run_both(sqa, mf, [650, 90], order="attend_then_evict")
    sl = W.scaled(W.WORKLOADS["tiny"], L=2, Hq=8, Hkv=2, D=128, B=1, P=900, S=4, dtype="bf16", policy="sliding")
    _run_both(sqa, sl, [777, 30])
    # and with K / V in blocks named by a block table
    _run_both(sqa, big, [700, 41, 520], blocked=True)


def test_static_scratch_entry_point_limits_and_status(sqa):
    """A call whose scratch exceeds the array is refused on the host (nothing runs); device-side conditions
    land in the caller's status word."""
    # one unit of 600000 slots with 8 heads under H2O: 8 x 600000 x 4 bytes of probabilities > 15 MiB
    B, Hkv, D, g = 1, 1, 128, 8
    huge = sqa.LayerCaches([600000], [600000], B, Hkv, D, torch.bfloat16, DEV, True)
    q = torch.zeros(1, B, Hkv * g, D, dtype=torch.bfloat16, device=DEV)
    kv = torch.zeros(1, B, Hkv, D, dtype=torch.bfloat16, device=DEV)
    out = torch.empty_like(q)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(sqa.SqaError) as e:
        sqa.decode_step_static(q, kv, kv, 5, "h2o", 4, huge, out, status)
    assert e.value.code == 6                                  # SQA_ERR_CAPACITY
    assert int(huge.lens[0][0, 0]) == 0 and int(status.item()) == 0
    # device-side: a unit longer than its budget on entry -> SQA_ERR_STATE in the caller's word
    c = sqa.LayerCaches([4], [8], 1, 1, 64, torch.float32, DEV, True)
    c.lens[0][0, 0] = 6
    q = torch.randn(1, 1, 1, 64, device=DEV); out = torch.ones_like(q)
    sqa.decode_step_static(q, q, q, 9, "sliding", 4, c, out, status)
    torch.cuda.synchronize()
    assert int(status.item()) == 8 and float(out.abs().sum()) == 0.0 and int(c.lens[0][0, 0]) == 6
