"""Thin ctypes binding over libsqa.so (the C ABI of include/sqa.h).

Argument marshalling only: every step of the path runs in the HIP library.
PyTorch supplies device memory and the current stream.  There is no fallback:
if the library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsqa.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libsqa.so is not built: run `python -m paper_2404_04793_amd.build` "
        "(there is no CPU or PyTorch fallback for the HIP path)")
_lib = C.CDLL(LIB_PATH)

SQA_OK = 0
ERR = {1: "NULL", 2: "SHAPE", 3: "DTYPE", 4: "POLICY", 5: "BUDGET", 6: "CAPACITY", 7: "HIP", 8: "STATE"}
SQA_F32, SQA_BF16 = 0, 1
POLICY = {"sliding": 0, "streaming": 1, "h2o": 2}
SQA_MAX_LAYERS = 128
SQA_BLOCK_SLOTS = 16


class SqaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        _lib.sqa_status_str.restype = C.c_char_p
        msg = _lib.sqa_status_str(C.c_int(code)).decode()
        super().__init__("%s: SQA_ERR_%s (%s)" % (where, ERR.get(code, str(code)), msg))


class LayerCacheStruct(C.Structure):
    """Mirror of sqa_layer_cache."""
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("score_acc", C.c_void_p), ("pos", C.c_void_p),
                ("unit_state", C.c_void_p), ("unit_offset", C.c_void_p), ("block_table", C.c_void_p),
                ("capacity", C.c_int32), ("budget", C.c_int32), ("blocks_per_unit", C.c_int32), ("n_blocks", C.c_int32)]


class DecodePlanInfo(C.Structure):
    """Mirror of sqa_decode_plan_info."""
    _fields_ = [("workgroups", C.c_int64), ("workspace_bytes", C.c_int64), ("lds_bytes", C.c_int32),
                ("matrix_cores", C.c_int32), ("wide_tail", C.c_int32), ("table_entries", C.c_int32)]


class DecodeLayerPlan(C.Structure):
    """Mirror of sqa_decode_layer_plan."""
    _fields_ = [("workgroups_per_unit", C.c_int32), ("slots_per_workgroup", C.c_int32),
                ("wave_per_unit", C.c_int32), ("probs_in_lds", C.c_int32)]


class BatchOptsStruct(C.Structure):
    """Mirror of sqa_batch_opts."""
    _fields_ = [("prompt_len", C.c_void_p), ("budget_seq", C.c_void_p), ("new_pos_seq", C.c_void_p),
                ("status", C.c_void_p), ("order", C.c_int32)]


ORDER = {"evict_then_attend": 0, "attend_then_evict": 1}

_vp, _i, _i64, _sz, _f64 = C.c_void_p, C.c_int, C.c_int64, C.c_size_t, C.c_double
_LCp = C.POINTER(LayerCacheStruct)
_BOp = C.POINTER(BatchOptsStruct)

_lib.sqa_layer_importance_workspace_bytes.restype = _sz
_lib.sqa_layer_importance_workspace_bytes.argtypes = [_i, _i64, _i]
_lib.sqa_layer_importance.restype = _i
_lib.sqa_layer_importance.argtypes = [_vp, _vp, _i, _i, _i64, _i, _vp, _vp, _sz, _vp]
_lib.sqa_residual_add_importance.restype = _i
_lib.sqa_residual_add_importance.argtypes = [_vp, _vp, _vp, _i, _i, _i64, _i, _vp, _vp, _sz, _vp]
_lib.sqa_layer_importance_seq.restype = _i
_lib.sqa_layer_importance_seq.argtypes = [_vp, _vp, _i, _i, _i64, _i, _vp, _i, _vp, _vp, _sz, _vp]
_lib.sqa_allocate_budgets.restype = _i
_lib.sqa_allocate_budgets.argtypes = [C.POINTER(C.c_float), _i, _i64, _f64, C.POINTER(C.c_int32), C.POINTER(C.c_int8)]
_lib.sqa_prefill_scores_workspace_bytes.restype = _sz
_lib.sqa_prefill_scores_workspace_bytes.argtypes = [_i, _i, _i, _i, _i]
_lib.sqa_prefill_scores.restype = _i
_lib.sqa_prefill_scores.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp]
_lib.sqa_prefill_scores_ex.restype = _i
_lib.sqa_prefill_scores_ex.argtypes = [_vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp, _BOp]
_lib.sqa_prefill_scores_lse.restype = _i
_lib.sqa_prefill_scores_lse.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _vp, _vp, _sz, _vp, _BOp]
_lib.sqa_prefill_compress.restype = _i
_lib.sqa_prefill_compress.argtypes = [_vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _i, _LCp, _vp]
_lib.sqa_prefill_compress_layers.restype = _i
_lib.sqa_prefill_compress_layers.argtypes = [C.POINTER(_vp), C.POINTER(_vp), _i, C.POINTER(_vp), _i, _i, _i, _i, _i, _i,
                                             _LCp, _i, _vp]
_lib.sqa_prefill_compress_layers_ex.restype = _i
_lib.sqa_prefill_compress_layers_ex.argtypes = [C.POINTER(_vp), C.POINTER(_vp), _i, C.POINTER(_vp), _i, _i, _i, _i, _i,
                                                _i, _LCp, _i, _vp, _BOp]
_lib.sqa_decode_workspace_bytes.restype = _sz
_lib.sqa_decode_workspace_bytes.argtypes = [_LCp, _i, _i, _i, _i, _i, _i]
_lib.sqa_decode_workspace_init.restype = _i
_lib.sqa_decode_workspace_init.argtypes = [_vp, _sz, _vp]
_lib.sqa_decode_step.restype = _i
_lib.sqa_decode_step.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, C.c_int32, _i, _i, _LCp, _vp, _i,
                                 _vp, _vp, _sz, _vp]
_lib.sqa_decode_step_ex.restype = _i
_lib.sqa_decode_step_ex.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, C.c_int32, _i, _i, _LCp, _vp, _i,
                                    _vp, _vp, _sz, _vp, _BOp]
_lib.sqa_decode_step_static.restype = _i
_lib.sqa_decode_step_static.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, C.c_int32, _i, _i, _LCp, _vp, _i,
                                        _vp, _vp, _vp, _BOp]
_lib.sqa_clear_device_status.restype = _i
_lib.sqa_clear_device_status.argtypes = [_vp, _vp]
_lib.sqa_read_device_status.restype = _i
_lib.sqa_read_device_status.argtypes = [_vp, _vp, C.POINTER(C.c_int32)]
_lib.sqa_kept_idx_sorted.restype = _i
_lib.sqa_kept_idx_sorted.argtypes = [_LCp, _i, _i, _vp, _vp]
_lib.sqa_decode_plan.argtypes = [_LCp, _i, _i, _i, _i, _i, _i, _i, C.POINTER(DecodePlanInfo), C.POINTER(DecodeLayerPlan)]
_lib.sqa_block_pool_create.argtypes = [C.c_int32]
_lib.sqa_block_pool_create.restype = _vp
_lib.sqa_block_pool_destroy.argtypes = [_vp]
_lib.sqa_block_pool_destroy.restype = None
_lib.sqa_block_pool_free_count.argtypes = [_vp]
_lib.sqa_block_pool_free_count.restype = C.c_int32
_lib.sqa_block_pool_take.argtypes = [_vp, C.c_int32, C.POINTER(C.c_int32)]
_lib.sqa_block_pool_give.argtypes = [_vp, C.POINTER(C.c_int32), C.c_int32]


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SQA_F32
    if t.dtype == torch.bfloat16:
        return SQA_BF16
    return -1


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def batch_opts(prompt_len: Optional[torch.Tensor] = None, budget_seq: Optional[torch.Tensor] = None,
               new_pos_seq: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
               order: str = "evict_then_attend") -> BatchOptsStruct:
    """sqa_batch_opts from int32 device tensors (the caller keeps them alive until the work has run)."""
    for t in (prompt_len, budget_seq, new_pos_seq, status):
        if t is not None and (t.dtype != torch.int32 or not t.is_contiguous()):
            raise TypeError("per-sequence arrays are contiguous int32 tensors")
    return BatchOptsStruct(_ptr(prompt_len), _ptr(budget_seq), _ptr(new_pos_seq), _ptr(status), ORDER[order])


def _opts(o: Optional[BatchOptsStruct]):
    return None if o is None else C.byref(o)


def _check(code: int, where: str):
    if code != SQA_OK:
        raise SqaError(code, where)


# --------------------------------------------------------------------------

def layer_importance(h_in: torch.Tensor, h_out: torch.Tensor, cos_out: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """h_in, h_out [L, T, hidden] (contiguous, device) -> cos [L] fp32 (device)."""
    L, T, d = h_in.shape
    if cos_out is None:
        cos_out = torch.empty(L, dtype=torch.float32, device=h_in.device)
    need = _lib.sqa_layer_importance_workspace_bytes(L, T, d)
    if workspace is None:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=h_in.device)
    _check(_lib.sqa_layer_importance(_ptr(h_in), _ptr(h_out), _dt(h_in), L, T, d, _ptr(cos_out),
                                     _ptr(workspace), workspace.numel(), _stream()), "sqa_layer_importance")
    return cos_out


def residual_add_importance(h_in: torch.Tensor, attn_out: torch.Tensor, h_out: torch.Tensor,
                            cos_out: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """h_out = h_in + attn_out written (h_out may be h_in or attn_out itself) and cos [L] of
    (h_in, h_out) returned, one pass.  All [L, T, hidden], contiguous, device."""
    L, T, d = h_in.shape
    if cos_out is None:
        cos_out = torch.empty(L, dtype=torch.float32, device=h_in.device)
    need = _lib.sqa_layer_importance_workspace_bytes(L, T, d)
    if workspace is None:
        workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=h_in.device)
    _check(_lib.sqa_residual_add_importance(_ptr(h_in), _ptr(attn_out), _ptr(h_out), _dt(h_in), L, T, d,
                                            _ptr(cos_out), _ptr(workspace), workspace.numel(), _stream()),
           "sqa_residual_add_importance")
    return cos_out


def layer_importance_seq(h_in: torch.Tensor, h_out: torch.Tensor, seq_start: torch.Tensor) -> torch.Tensor:
    """h_in, h_out [L, T, hidden]; seq_start int32 [n_seq + 1] (device) -> cos [L, n_seq] fp32."""
    L, T, d = h_in.shape
    n_seq = seq_start.numel() - 1
    cos_out = torch.empty(L, n_seq, dtype=torch.float32, device=h_in.device)
    need = n_seq * _lib.sqa_layer_importance_workspace_bytes(L, T, d)
    workspace = torch.empty(max(need, 8), dtype=torch.uint8, device=h_in.device)
    _check(_lib.sqa_layer_importance_seq(_ptr(h_in), _ptr(h_out), _dt(h_in), L, T, d, _ptr(seq_start), n_seq,
                                         _ptr(cos_out), _ptr(workspace), workspace.numel(), _stream()),
           "sqa_layer_importance_seq")
    return cos_out


def allocate_budgets(cos: Sequence[float], total_budget: int, p: float) -> Tuple[List[int], List[int]]:
    """cos: host floats (rounded to fp32 here) -> (budget[L], group[L])."""
    L = len(cos)
    c = (C.c_float * L)(*[float(x) for x in cos])
    b = (C.c_int32 * L)()
    g = (C.c_int8 * L)()
    _check(_lib.sqa_allocate_budgets(c, L, int(total_budget), float(p), b, g), "sqa_allocate_budgets")
    return list(b), list(g)


def prefill_scores(Q: torch.Tensor, K: torch.Tensor, scores_out: Optional[torch.Tensor] = None,
                   opts: Optional[BatchOptsStruct] = None, row_lse: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Q [B, Hq, P, D], K [B, Hkv, P, D] -> scores [B, Hkv, P] fp32.  row_lse [B, Hq, P] fp32 (optional): the
    natural-log softmax normalisers of the prompt's causal attention, if the caller has them
    (sqa_prefill_scores_lse: one pass instead of two)."""
    B, Hq, P, D = Q.shape
    Hkv = K.shape[1]
    if scores_out is None:
        scores_out = torch.empty(B, Hkv, P, dtype=torch.float32, device=Q.device)
    need = _lib.sqa_prefill_scores_workspace_bytes(B, Hq, Hkv, P, D)
    ws = torch.empty(max(need, 8), dtype=torch.uint8, device=Q.device)
    if row_lse is None:
        _check(_lib.sqa_prefill_scores_ex(_ptr(Q), _ptr(K), _dt(Q), B, Hq, Hkv, P, D, _ptr(scores_out), _ptr(ws),
                                          ws.numel(), _stream(), _opts(opts)), "sqa_prefill_scores")
    else:
        if row_lse.dtype != torch.float32 or not row_lse.is_contiguous() or tuple(row_lse.shape) != (B, Hq, P):
            raise TypeError("row_lse is a contiguous fp32 tensor [B, Hq, P]")
        _check(_lib.sqa_prefill_scores_lse(_ptr(Q), _ptr(K), _ptr(row_lse), _dt(Q), B, Hq, Hkv, P, D, _ptr(scores_out),
                                           _ptr(ws), ws.numel(), _stream(), _opts(opts)), "sqa_prefill_scores_lse")
    return scores_out


def decode_plan(budgets: Sequence[int], capacities: Sequence[int], B: int, Hq: int, Hkv: int, D: int,
                dtype: str, policy: str, blocked: bool = False) -> dict:
    """sqa_decode_plan: the launch a decode call over these layers would make (host arithmetic, no GPU).
    dtype: "bf16" or "f32"."""
    n = len(budgets)
    t = (LayerCacheStruct * n)()
    for i in range(n):
        t[i].capacity, t[i].budget = int(capacities[i]), int(budgets[i])
        if blocked:
            t[i].block_table = 0x1000                     # (only "is it NULL" is looked at)
            t[i].blocks_per_unit = (min(int(capacities[i]), int(budgets[i])) + SQA_BLOCK_SLOTS - 1) // SQA_BLOCK_SLOTS
            t[i].n_blocks = 1
    info, per = DecodePlanInfo(), (DecodeLayerPlan * n)()
    _check(_lib.sqa_decode_plan(t, n, B, Hq, Hkv, D, {"f32": 0, "bf16": 1}[dtype], POLICY[policy], C.byref(info), per),
           "sqa_decode_plan")
    out = {f: int(getattr(info, f)) for f, _ in DecodePlanInfo._fields_}
    out["layers"] = [{f: int(getattr(per[i], f)) for f, _ in DecodeLayerPlan._fields_} for i in range(n)]
    return out


class BlockPool:
    """sqa_block_pool: the free list of one layer's K/V block numbers (host book-keeping)."""

    def __init__(self, n_blocks: int):
        self._p = _lib.sqa_block_pool_create(n_blocks)
        if not self._p:
            raise ValueError("sqa_block_pool_create(%d) failed" % n_blocks)

    def free_count(self) -> int:
        return int(_lib.sqa_block_pool_free_count(self._p))

    def take(self, n: int) -> List[int]:
        ids = (C.c_int32 * max(n, 1))()
        _check(_lib.sqa_block_pool_take(self._p, n, ids), "sqa_block_pool_take")
        return list(ids[:n])

    def give(self, ids: Sequence[int]) -> None:
        arr = (C.c_int32 * max(len(ids), 1))(*ids)
        _check(_lib.sqa_block_pool_give(self._p, arr, len(ids)), "sqa_block_pool_give")

    def close(self) -> None:
        if self._p:
            _lib.sqa_block_pool_destroy(self._p)
            self._p = None

    def __del__(self):
        self.close()


class LayerCaches:
    """Device memory of the compact caches of a range of layers, plus the
    sqa_layer_cache table on the host and its copy on the device."""

    def __init__(self, budgets: Sequence[int], capacities: Sequence[int], B: int, Hkv: int, D: int,
                 dtype: torch.dtype, device, with_scores: bool = True,
                 unit_capacities: Optional[Sequence[Sequence[int]]] = None, blocked: bool = False,
                 block_seed: Optional[int] = 0, spare_blocks: int = 3):
        """unit_capacities[l][b*Hkv + h] (optional): packed units -- every unit gets exactly that many
        slots (sqa_layer_cache.unit_offset); K, V, score, pos of a layer are then flat over the slots and
        `capacities[l]` must be the largest of them.
        blocked: K and V of a layer are pools of 16-row blocks and every unit owns the blocks its table row
        names (sqa_layer_cache.block_table); the blocks are dealt out in a seeded random order (block_seed;
        None = in order), with a few spare blocks in between, so that no unit is contiguous.
        Use unit(l, b, h) / unit_kv_rows(l, b, h) to address a unit whatever the layout."""
        self.L, self.B, self.Hkv, self.D, self.dtype = len(budgets), B, Hkv, D, dtype
        self.budgets, self.capacities = list(budgets), list(capacities)
        self.blocked = blocked
        assert not (blocked and unit_capacities is not None)
        self.K, self.V, self.score, self.pos, self.state = [], [], [], [], []
        self.lens, self.head, self.hint = [], [], []        # views of the [B, Hkv, 4] unit_state records
        self.offsets: List[Optional[torch.Tensor]] = []
        self.offsets_host: List[Optional[List[int]]] = []
        self.block_table: List[Optional[torch.Tensor]] = []
        self.table = (LayerCacheStruct * self.L)()
        for i, (b, cap) in enumerate(zip(budgets, capacities)):
            bpu = n_blocks = 0
            tbl = None
            if blocked:
                bpu = (cap + SQA_BLOCK_SLOTS - 1) // SQA_BLOCK_SLOTS
                n_blocks = B * Hkv * bpu + spare_blocks
                if block_seed is None:
                    perm = torch.arange(n_blocks)
                else:
                    perm = torch.randperm(n_blocks, generator=torch.Generator().manual_seed(block_seed + 7919 * i))
                tbl = perm[:B * Hkv * bpu].to(torch.int32).view(B * Hkv, bpu).contiguous().to(device)
                shape_rows, shape_flat = (n_blocks, SQA_BLOCK_SLOTS, D), (B, Hkv, cap)
                self.offsets.append(None); self.offsets_host.append(None)
            elif unit_capacities is None:
                shape_rows, shape_flat = (B, Hkv, cap, D), (B, Hkv, cap)
                self.offsets.append(None); self.offsets_host.append(None)
            else:
                caps_u = [int(x) for x in unit_capacities[i]]
                assert len(caps_u) == B * Hkv and max(caps_u) == cap
                off = [0]
                for x in caps_u:
                    off.append(off[-1] + x)
                shape_rows, shape_flat = (off[-1], D), (off[-1],)
                self.offsets_host.append(off)
                self.offsets.append(torch.tensor(off, dtype=torch.int64, device=device))
            self.block_table.append(tbl)
            self.K.append(torch.zeros(*shape_rows, dtype=dtype, device=device))
            self.V.append(torch.zeros(*shape_rows, dtype=dtype, device=device))
            self.score.append(torch.zeros(*shape_flat, dtype=torch.float32, device=device) if with_scores else None)
            self.pos.append(torch.full(shape_flat, -1, dtype=torch.int32, device=device))
            st = torch.zeros(B, Hkv, 4, dtype=torch.int32, device=device)
            st[..., 2] = -2
            self.state.append(st)
            self.lens.append(st[..., 0]); self.head.append(st[..., 1]); self.hint.append(st[..., 2])
            t = self.table[i]
            t.K, t.V = self.K[i].data_ptr(), self.V[i].data_ptr()
            t.score_acc = self.score[i].data_ptr() if with_scores else None
            t.pos, t.unit_state = self.pos[i].data_ptr(), self.state[i].data_ptr()
            t.unit_offset = None if self.offsets[i] is None else self.offsets[i].data_ptr()
            t.block_table = None if tbl is None else tbl.data_ptr()
            t.capacity, t.budget, t.blocks_per_unit, t.n_blocks = int(cap), int(b), int(bpu), int(n_blocks)
        raw = bytes(memoryview(self.table))
        self.table_dev = torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(device)

    def unit(self, layer: int, b: int, h: int):
        """(K, V, score or None, pos) views of unit (b, h): [slots, D], [slots, D], [slots], [slots].
        With blocked allocation K and V are None here: address their rows through unit_kv_rows."""
        sc = self.score[layer]
        if self.blocked:
            return None, None, None if sc is None else sc[b, h], self.pos[layer][b, h]
        if self.offsets_host[layer] is None:
            return self.K[layer][b, h], self.V[layer][b, h], None if sc is None else sc[b, h], self.pos[layer][b, h]
        u = b * self.Hkv + h
        lo, hi = self.offsets_host[layer][u], self.offsets_host[layer][u + 1]
        return self.K[layer][lo:hi], self.V[layer][lo:hi], None if sc is None else sc[lo:hi], self.pos[layer][lo:hi]

    def unit_kv_rows(self, layer: int, b: int, h: int):
        """(K rows [all rows of the layer, D], V rows likewise, index of the row of each of the unit's slots):
        slot s of the unit is row idx[s] of both, whatever the layout."""
        Kf, Vf = self.K[layer].view(-1, self.D), self.V[layer].view(-1, self.D)
        dev = Kf.device
        u = b * self.Hkv + h
        cap = self.capacities[layer]
        if self.blocked:
            s = torch.arange(cap, device=dev)
            blk = self.block_table[layer][u].to(torch.int64)
            return Kf, Vf, blk[s // SQA_BLOCK_SLOTS] * SQA_BLOCK_SLOTS + s % SQA_BLOCK_SLOTS
        if self.offsets_host[layer] is None:
            return Kf, Vf, torch.arange(u * cap, (u + 1) * cap, device=dev)
        lo, hi = self.offsets_host[layer][u], self.offsets_host[layer][u + 1]
        return Kf, Vf, torch.arange(lo, hi, device=dev)

    def sequence_table(self, b: int):
        """sqa_layer_cache records (host) that describe sequence b alone as a batch of one: the same memory,
        the per-unit arrays entered at the sequence's first unit.  For calls that concern one sequence of a
        running batch -- compressing the prompt of a sequence that takes a finished one's place."""
        assert all(o is None for o in self.offsets_host), "not for packed units"
        t = (LayerCacheStruct * self.L)()
        es = self.K[0].element_size()
        for i in range(self.L):
            u0, cap, src = b * self.Hkv, self.capacities[i], self.table[i]
            t[i].K = src.K if self.blocked else src.K + u0 * cap * self.D * es
            t[i].V = src.V if self.blocked else src.V + u0 * cap * self.D * es
            t[i].score_acc = None if not src.score_acc else src.score_acc + u0 * cap * 4
            t[i].pos, t[i].unit_state = src.pos + u0 * cap * 4, src.unit_state + u0 * 16
            t[i].unit_offset = None
            t[i].block_table = None if not self.blocked else src.block_table + u0 * src.blocks_per_unit * 4
            t[i].capacity, t[i].budget = src.capacity, src.budget
            t[i].blocks_per_unit, t[i].n_blocks = src.blocks_per_unit, src.n_blocks
        return t

    def total_slots(self, layer: int) -> int:
        if self.blocked:
            return self.K[layer].shape[0] * SQA_BLOCK_SLOTS
        off = self.offsets_host[layer]
        return self.B * self.Hkv * self.capacities[layer] if off is None else off[-1]

    def struct_ptr(self, layer: int = 0):
        return C.cast(C.byref(self.table, layer * C.sizeof(LayerCacheStruct)), _LCp)

    def dev_ptr(self, layer: int = 0):
        return self.table_dev.data_ptr() + layer * C.sizeof(LayerCacheStruct)


def prefill_compress(K: torch.Tensor, V: torch.Tensor, attn_scores: Optional[torch.Tensor], policy: str,
                     n_sink: int, caches: LayerCaches, layer: int) -> None:
    """K, V [B, Hkv, P, D] of one layer -> caches' layer `layer`."""
    B, Hkv, P, D = K.shape
    _check(_lib.sqa_prefill_compress(_ptr(K), _ptr(V), _dt(K), _ptr(attn_scores), B, Hkv, P, D, POLICY[policy],
                                     n_sink, caches.struct_ptr(layer), _stream()), "sqa_prefill_compress")


def prefill_compress_layers(K: Sequence[torch.Tensor], V: Sequence[torch.Tensor],
                            attn_scores: Optional[Sequence[Optional[torch.Tensor]]], policy: str, n_sink: int,
                            caches: LayerCaches, layer0: int = 0, opts: Optional[BatchOptsStruct] = None,
                            table=None) -> None:
    """K[i], V[i] [B, Hkv, P, D] of layer layer0 + i -> caches' layers layer0 .. layer0 + len(K) - 1.
    table: sqa_layer_cache records to use instead of the caches' own (LayerCaches.sequence_table)."""
    n = len(K)
    B, Hkv, P, D = K[0].shape
    Ks = (_vp * n)(*[t.data_ptr() for t in K])
    Vs = (_vp * n)(*[t.data_ptr() for t in V])
    Ss = None if attn_scores is None or attn_scores[0] is None else (_vp * n)(*[t.data_ptr() for t in attn_scores])
    layers = caches.struct_ptr(layer0) if table is None else C.cast(C.byref(table, layer0 * C.sizeof(LayerCacheStruct)), _LCp)
    _check(_lib.sqa_prefill_compress_layers_ex(Ks, Vs, _dt(K[0]), Ss, B, Hkv, P, D, POLICY[policy], n_sink,
                                               layers, n, _stream(), _opts(opts)),
           "sqa_prefill_compress_layers")


def decode_workspace(caches: "LayerCaches", Hq: int, policy: str, layer0: int = 0,
                     n_layers: Optional[int] = None) -> torch.Tensor:
    """Scratch for sqa_decode_step over layers [layer0, layer0 + n_layers) of `caches`, zero-filled."""
    n_layers = caches.L - layer0 if n_layers is None else n_layers
    need = _lib.sqa_decode_workspace_bytes(caches.struct_ptr(layer0), n_layers, caches.B, Hq, caches.Hkv, caches.D,
                                           POLICY[policy])
    if need == 0:
        raise SqaError(2, "sqa_decode_workspace_bytes")
    ws = torch.empty(need, dtype=torch.uint8, device=caches.K[0].device)
    _check(_lib.sqa_decode_workspace_init(_ptr(ws), need, _stream()), "sqa_decode_workspace_init")
    return ws


def decode_step(q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, new_pos: int, policy: str,
                n_sink: int, caches: LayerCaches, out: torch.Tensor, workspace: torch.Tensor,
                layer0: int = 0, n_layers: Optional[int] = None, use_dev_table: bool = True,
                opts: Optional[BatchOptsStruct] = None) -> torch.Tensor:
    """q [n_layers, B, Hq, D], k_new / v_new [n_layers, B, Hkv, D] -> out like q."""
    n_layers = caches.L - layer0 if n_layers is None else n_layers
    B, Hq, D = q.shape[-3], q.shape[-2], q.shape[-1]
    Hkv = k_new.shape[-2]
    if opts is None:
        _check(_lib.sqa_decode_step(_ptr(q), _ptr(k_new), _ptr(v_new), _dt(q), B, Hq, Hkv, D, int(new_pos),
                                    POLICY[policy], n_sink, caches.struct_ptr(layer0),
                                    caches.dev_ptr(layer0) if use_dev_table else None, n_layers, _ptr(out),
                                    _ptr(workspace), workspace.numel(), _stream()), "sqa_decode_step")
    else:
        _check(_lib.sqa_decode_step_ex(_ptr(q), _ptr(k_new), _ptr(v_new), _dt(q), B, Hq, Hkv, D, int(new_pos),
                                       POLICY[policy], n_sink, caches.struct_ptr(layer0),
                                       caches.dev_ptr(layer0) if use_dev_table else None, n_layers, _ptr(out),
                                       _ptr(workspace), workspace.numel(), _stream(), C.byref(opts)),
               "sqa_decode_step_ex")
    return out


def decode_step_static(q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor, new_pos: int, policy: str,
                       n_sink: int, caches: LayerCaches, out: torch.Tensor, status: torch.Tensor,
                       layer0: int = 0, n_layers: Optional[int] = None, use_dev_table: bool = True,
                       opts: Optional[BatchOptsStruct] = None) -> torch.Tensor:
    """sqa_decode_step_static: decode_step without a workspace (the library's own scratch array);
    status: int32 device tensor of one element that receives the device-side status."""
    n_layers = caches.L - layer0 if n_layers is None else n_layers
    B, Hq, D = q.shape[-3], q.shape[-2], q.shape[-1]
    Hkv = k_new.shape[-2]
    _check(_lib.sqa_decode_step_static(_ptr(q), _ptr(k_new), _ptr(v_new), _dt(q), B, Hq, Hkv, D, int(new_pos),
                                       POLICY[policy], n_sink, caches.struct_ptr(layer0),
                                       caches.dev_ptr(layer0) if use_dev_table else None, n_layers, _ptr(out),
                                       _ptr(status), _stream(), _opts(opts)), "sqa_decode_step_static")
    return out


def clear_device_status(workspace: torch.Tensor) -> None:
    _check(_lib.sqa_clear_device_status(_ptr(workspace), _stream()), "sqa_clear_device_status")


def read_device_status(workspace: torch.Tensor) -> int:
    v = C.c_int32(0)
    _check(_lib.sqa_read_device_status(_ptr(workspace), _stream(), C.byref(v)), "sqa_read_device_status")
    return v.value


def kept_idx_sorted(caches: LayerCaches, layer: int) -> torch.Tensor:
    """-> int32 [B, Hkv, capacity]: kept positions ascending, -1 padded."""
    shape = (caches.B, caches.Hkv, caches.capacities[layer]) if caches.offsets_host[layer] is None \
        else (caches.total_slots(layer),)
    out = torch.empty(*shape, dtype=torch.int32, device=caches.K[layer].device)
    _check(_lib.sqa_kept_idx_sorted(caches.struct_ptr(layer), caches.B, caches.Hkv, _ptr(out), _stream()),
           "sqa_kept_idx_sorted")
    return out
