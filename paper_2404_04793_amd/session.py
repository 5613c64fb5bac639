"""One synthetic generation job on one GPU, driven through the binding:
inputs resident in HBM, then Algorithm 1 end to end -- probe, budgets, prompt
compression, S decode steps.  Used by bench.py and the full-size parity tests;
holds no arithmetic of the method (that is all in libsqa)."""
from __future__ import annotations

from typing import Dict, List, Optional

import torch

from . import binding as sqa
from . import workloads as W


class Session:
    def __init__(self, wl: W.Workload, device="cuda:0", keep_prompt_q: bool = False, uniform_budget: bool = False,
                 full_cache: bool = False, probe_tokens: Optional[int] = None, fused_probe: bool = False,
                 order: str = "evict_then_attend", prompt_len: Optional[List[int]] = None, blocked: bool = False):
        """probe_tokens: hidden-state rows per layer given to the probe (default: all B*P prompt tokens;
        a smaller number keeps the hidden states of the largest workloads within HBM).
        fused_probe: the probe runs inside the residual add that writes h_out (Sec. 3).
        prompt_len: a ragged batch -- sequence b's prompt is its first prompt_len[b] <= P tokens (the
        tensors stay padded to P); each sequence is then probed and budgeted on its own
        (sqa_layer_importance_seq, one sqa_allocate_budgets per sequence) and decodes at its own position.
        blocked: K and V of every layer live in pools of 16-row blocks that a block table deals to the units
        (in a seeded random order, so that no unit is contiguous)."""
        self.wl, self.dev = wl, device
        self.blocked = blocked
        assert not (blocked and prompt_len is not None)
        self.fused_probe = fused_probe
        self.order = order
        self.opts = None if order == "evict_then_attend" else sqa.batch_opts(order=order)
        self.ragged = prompt_len is not None
        if self.ragged:
            assert len(prompt_len) == wl.B and all(1 <= x <= wl.P for x in prompt_len)
            assert not (uniform_budget or full_cache or fused_probe or probe_tokens)
            self.prompt_len = [int(x) for x in prompt_len]
            self.plen_dev = torch.tensor(self.prompt_len, dtype=torch.int32, device=device)
            starts = [0]
            for x in self.prompt_len:
                starts.append(starts[-1] + x)                 # the hidden-state rows of the sequences, packed
            self.seq_start = torch.tensor(starts, dtype=torch.int32, device=device)
            self.pos_steps = (self.plen_dev[None, :] + torch.arange(wl.S, dtype=torch.int32, device=device)[:, None]).contiguous()
            self.status = torch.zeros(1, dtype=torch.int32, device=device)
            self.budget_seq = None
        self.uniform_budget, self.full_cache = uniform_budget, full_cache
        self.u, self.mask = W.unit_dirs(wl), W.hh_mask(wl, device)
        L = wl.L
        # hidden states before / after self-attention, all layers: [L, T, hidden]
        T = wl.B * wl.P if probe_tokens is None else int(probe_tokens)
        self.probe_tokens = T
        self.h_in = torch.empty(L, T, wl.hidden, dtype=wl.torch_dtype, device=device)
        self.h_out = torch.empty_like(self.h_in)
        for l in range(L):
            a, b = W.hidden_states(wl, l, device, n_tokens=T)
            self.h_in[l], self.h_out[l] = a, b
        # the attention block's output, so that h_in + attn_out reproduces the generated h_out (up to rounding)
        self.attn_out = (self.h_out.float() - self.h_in.float()).to(wl.torch_dtype) if fused_probe else None
        # prompt K, V (kept resident: every pass compresses them again) and H2O prompt scores
        self.Kp, self.Vp, self.scores, self.Qp = [], [], [], []
        for l in range(L):
            K, V = W.prompt_kv(wl, l, device, self.u, self.mask)
            self.Kp.append(K); self.Vp.append(V)
            if wl.policy == "h2o":
                Q = W.prompt_q(wl, l, device, self.u)
                self.scores.append(sqa.prefill_scores(Q, K, opts=sqa.batch_opts(prompt_len=self.plen_dev)
                                                      if self.ragged else None))
                if keep_prompt_q:
                    self.Qp.append(Q)
                del Q
            else:
                self.scores.append(None)
        # decode inputs for all steps: [S, L, B, H, D]
        self.q = torch.empty(wl.S, L, wl.B, wl.Hq, wl.D, dtype=wl.torch_dtype, device=device)
        self.k_new = torch.empty(wl.S, L, wl.B, wl.Hkv, wl.D, dtype=wl.torch_dtype, device=device)
        self.v_new = torch.empty_like(self.k_new)
        for l in range(L):
            q, k, v = W.decode_qkv(wl, l, device, self.u, self.mask)
            self.q[:, l], self.k_new[:, l], self.v_new[:, l] = q, k, v
        self.out = torch.empty(wl.S, L, wl.B, wl.Hq, wl.D, dtype=wl.torch_dtype, device=device)
        self.cos_dev = torch.empty(L, dtype=torch.float32, device=device)
        self.cos_host = torch.empty(L, dtype=torch.float32, pin_memory=True)
        n = sqa._lib.sqa_layer_importance_workspace_bytes(L, T, wl.hidden)
        self.imp_ws = torch.empty(max(n, 8), dtype=torch.uint8, device=device)
        self.dec_ws = None
        self.dec_ws_layer = None
        self.caches: Optional[sqa.LayerCaches] = None
        self.budgets: Optional[List[int]] = None
        self.groups: Optional[List[int]] = None
        torch.cuda.synchronize()

    # -- Algorithm 1 steps 1-11 ------------------------------------------------
    def probe_and_allocate(self):
        wl = self.wl
        if self.ragged:
            return self._probe_and_allocate_ragged()
        if self.fused_probe:
            sqa.residual_add_importance(self.h_in, self.attn_out, self.h_out, self.cos_dev, self.imp_ws)
        else:
            sqa.layer_importance(self.h_in, self.h_out, self.cos_dev, self.imp_ws)
        self.cos_host.copy_(self.cos_dev, non_blocking=False)
        cos = self.cos_host.tolist()
        if self.full_cache:
            budgets, groups = [wl.P + wl.S] * wl.L, [1] * wl.L
        elif self.uniform_budget:
            budgets, groups = sqa.allocate_budgets(cos, wl.total_budget, 1.0)
        else:
            budgets, groups = sqa.allocate_budgets(cos, wl.total_budget, wl.p)
        if self.caches is None or budgets != self.budgets:
            caps = [min(b, wl.P + wl.S) for b in budgets]
            self.caches = sqa.LayerCaches(budgets, caps, wl.B, wl.Hkv, wl.D, wl.torch_dtype, self.dev,
                                          wl.policy == "h2o", blocked=self.blocked)
            self.dec_ws = sqa.decode_workspace(self.caches, wl.Hq, wl.policy)
            self.dec_ws_layer = [sqa.decode_workspace(self.caches, wl.Hq, wl.policy, l, 1) for l in range(wl.L)]
        self.budgets, self.groups = budgets, groups
        return cos

    def _probe_and_allocate_ragged(self):
        wl = self.wl
        cos = sqa.layer_importance_seq(self.h_in, self.h_out, self.seq_start).cpu()       # [L, B]
        per_seq = []
        for b in range(wl.B):
            total = wl.L * max(self.prompt_len[b] * wl.budget_pct // 100, 8)
            per_seq.append(sqa.allocate_budgets(cos[:, b].tolist(), total, wl.p)[0])
        budget_seq = [[per_seq[b][l] for b in range(wl.B)] for l in range(wl.L)]         # [L][B]
        budgets = [max(row) for row in budget_seq]                                       # the layers' maxima
        if self.caches is None or budget_seq != self.budget_seq:
            # packed units: every (sequence, head) owns exactly the slots its own budget can fill
            unit_caps = [[min(budget_seq[l][b], self.prompt_len[b] + wl.S) for b in range(wl.B) for _ in range(wl.Hkv)]
                         for l in range(wl.L)]
            self.caches = sqa.LayerCaches(budgets, [max(c) for c in unit_caps], wl.B, wl.Hkv, wl.D, wl.torch_dtype,
                                          self.dev, wl.policy == "h2o", unit_capacities=unit_caps)
            self.dec_ws = sqa.decode_workspace(self.caches, wl.Hq, wl.policy)
            self.dec_ws_layer = [sqa.decode_workspace(self.caches, wl.Hq, wl.policy, l, 1) for l in range(wl.L)]
            self.bseq_dev = torch.tensor(budget_seq, dtype=torch.int32, device=self.dev)
            self.opts_pre = sqa.batch_opts(prompt_len=self.plen_dev, budget_seq=self.bseq_dev, status=self.status)
            self.opts_step = [sqa.batch_opts(budget_seq=self.bseq_dev, new_pos_seq=self.pos_steps[t], order=self.order)
                              for t in range(wl.S)]
        self.budget_seq, self.budgets, self.groups = budget_seq, budgets, None
        return cos.mean(dim=1).tolist()

    # -- steps 12 + 16-17 on the prompt ---------------------------------------
    def compress_prompt(self):
        wl = self.wl
        sqa.prefill_compress_layers(self.Kp, self.Vp, self.scores, wl.policy, wl.n_sink, self.caches,
                                    opts=self.opts_pre if self.ragged else None)

    # -- steps 14-21 -----------------------------------------------------------
    def decode(self, steps: Optional[int] = None, per_layer: bool = False, start: int = 0):
        wl = self.wl
        S = wl.S if steps is None else steps
        for t in range(start, start + S):
            opts = self.opts_step[t] if self.ragged else self.opts
            if per_layer:
                assert not self.ragged        # (budget_seq rows are addressed from the call's first layer)
                for l in range(wl.L):
                    sqa.decode_step(self.q[t, l], self.k_new[t, l], self.v_new[t, l], wl.P + t, wl.policy, wl.n_sink,
                                    self.caches, self.out[t, l], self.dec_ws_layer[l], layer0=l, n_layers=1,
                                    opts=opts)
            else:
                sqa.decode_step(self.q[t], self.k_new[t], self.v_new[t], wl.P + t, wl.policy, wl.n_sink,
                                self.caches, self.out[t], self.dec_ws, opts=opts)

    # -- the same steps replayed from a HIP graph ---------------------------------
    def capture_step_graph(self, per_layer: bool = True):
        """Records one decode step (one launch per layer, or one launch in all) into a HIP graph whose
        inputs are fixed buffers: q/k/v of the step are copied in, the position comes from a device
        array (sqa_batch_opts.new_pos_seq), so the recorded launches never change.  Nothing in the
        recorded work is a memset."""
        wl = self.wl
        self.g_q = torch.empty_like(self.q[0]); self.g_k = torch.empty_like(self.k_new[0])
        self.g_v = torch.empty_like(self.v_new[0]); self.g_out = torch.empty_like(self.out[0])
        self.g_pos = torch.zeros(wl.B, dtype=torch.int32, device=self.dev)
        order = "evict_then_attend" if self.opts is None else "attend_then_evict"
        self.g_opts = sqa.batch_opts(new_pos_seq=self.g_pos, order=order)

        def step():
            if per_layer:
                for l in range(wl.L):
                    sqa.decode_step(self.g_q[l], self.g_k[l], self.g_v[l], 0, wl.policy, wl.n_sink, self.caches,
                                    self.g_out[l], self.dec_ws_layer[l], layer0=l, n_layers=1, opts=self.g_opts)
            else:
                sqa.decode_step(self.g_q, self.g_k, self.g_v, 0, wl.policy, wl.n_sink, self.caches, self.g_out,
                                self.dec_ws, opts=self.g_opts)

        # one eager run first (with every sequence sitting out, so no state changes): it performs the
        # one-time per-kernel set-up that must not happen during capture
        self.g_pos.fill_(-1)
        step()
        torch.cuda.synchronize()
        self.graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(self.graph):
            step()
        torch.cuda.synchronize()

    def decode_graph(self, steps: Optional[int] = None, start: int = 0):
        wl = self.wl
        S = wl.S if steps is None else steps
        for t in range(start, start + S):
            self.g_q.copy_(self.q[t]); self.g_k.copy_(self.k_new[t]); self.g_v.copy_(self.v_new[t])
            self.g_pos.fill_(wl.P + t)
            self.graph.replay()
            self.out[t].copy_(self.g_out)

    def run_pass(self):
        """The whole hot path once over this batch."""
        self.probe_and_allocate()
        self.compress_prompt()
        self.decode()

    # -- accounting (bytes the method must move; Sec. 2.1 KV size model) --------
    def decode_bytes_per_step(self) -> List[int]:
        """Algorithmic HBM bytes of each decode step (see workloads.decode_bytes_per_step)."""
        if self.ragged:
            return W.decode_bytes_per_step_ragged(self.wl, self.budget_seq, self.prompt_len)
        return W.decode_bytes_per_step(self.wl, self.budgets)

    def probe_bytes(self) -> int:
        wl = self.wl
        rows = sum(self.prompt_len) if self.ragged else self.probe_tokens
        return (3 if self.fused_probe else 2) * wl.L * rows * wl.hidden * wl.elem_bytes

    def compress_bytes(self) -> int:
        wl = self.wl
        row = wl.D * wl.elem_bytes
        tot = 0
        for l, b in enumerate(self.budgets):
            for s in range(wl.B):
                P = self.prompt_len[s] if self.ragged else wl.P
                n = min(P, self.budget_seq[l][s] if self.ragged else b)
                tot += wl.Hkv * ((4 * P if wl.policy == "h2o" else 0) + 2 * 2 * n * row)
        return tot

    def resident_kv_bytes(self) -> int:
        return W.resident_cache_bytes(self.wl, [self.caches.total_slots(l) for l in range(self.wl.L)])
