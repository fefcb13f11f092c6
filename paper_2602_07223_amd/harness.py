"""Device-memory plumbing around the binding: upload a synthetic layer, allocate outputs and
workspace with torch, and issue verify -> select -> draft through the C ABI.  No arithmetic of the
method lives here; torch is used for allocation, copies and streams only."""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np
import torch

from . import binding as vb
from .synth import LayerInputs

PAGE = 16


def bf16_to_device(bits: np.ndarray, device) -> torch.Tensor:
    """uint16 bf16 bit patterns -> torch.bfloat16 tensor on ``device`` (bit-exact)."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def bf16_to_host_f64(t: torch.Tensor) -> np.ndarray:
    """torch.bfloat16 tensor -> float64 NumPy array (exact)."""
    bits = t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


@dataclasses.dataclass
class DeviceLayer:
    q_verify: torch.Tensor      # bf16 [B, G, Hq, D]
    q_draft: torch.Tensor       # bf16 [G, B, Hq, D]
    k_cache: torch.Tensor       # bf16 [P, 16, Hkv, D]
    v_cache: torch.Tensor
    block_table: torch.Tensor   # int32 [B, max_blocks]
    seq_lens: torch.Tensor      # int32 [B]
    k_new: Optional[torch.Tensor] = None     # bf16 [steps, B, 1, Hkv, D]: rows the live drafting phase appends
    v_new: Optional[torch.Tensor] = None
    seq_lens_live: Optional[torch.Tensor] = None   # int32 [B]: the lengths the live drafting phase advances

    @staticmethod
    def upload(L: LayerInputs, device="cuda:0") -> "DeviceLayer":
        dl = DeviceLayer(
            q_verify=bf16_to_device(L.q_verify, device), q_draft=bf16_to_device(L.q_draft, device),
            k_cache=bf16_to_device(L.k_cache, device), v_cache=bf16_to_device(L.v_cache, device),
            block_table=torch.from_numpy(L.block_table).to(device), seq_lens=torch.from_numpy(L.seq_lens).to(device))
        if L.k_new is not None:
            dl.k_new, dl.v_new = bf16_to_device(L.k_new, device), bf16_to_device(L.v_new, device)
            dl.seq_lens_live = dl.seq_lens.clone()
        return dl


class VegasPath:
    """One layer's verify -> select -> draft calls with preallocated outputs and workspace."""

    def __init__(self, *, batch: int, num_q_heads: int, num_kv_heads: int, num_queries: int, max_blocks: int,
                 max_seq_len: int, num_pages: int, budget_tokens: int, softmax_scale: float,
                 collect_rows: int = vb.COLLECT_ALL_ROWS, head_dim: int = 128, device="cuda:0",
                 verify_chunk: int = 0, draft_chunk: int = 0, max_sel_blocks: int = 0,
                 score_metric: int = vb.METRIC_PAGE_WEIGHTS, token_granular: bool = False, window: int = 0,
                 growth: int = 0):
        """token_granular: the paper's own variant -- verification collects averaged logits per token,
        selection picks single tokens, drafting walks one-token pages (Sec. 3.3, Sec. 4).
        window > 0: verification of a banded layer (local masking; needs collect_rows = COLLECT_NONE)."""
        self.device = torch.device(device)
        self.token_granular = token_granular
        if token_granular:
            score_metric = vb.METRIC_TOKEN_LOGITS
        self.B, self.Hq, self.Hkv, self.G, self.D = batch, num_q_heads, num_kv_heads, num_queries, head_dim
        self.budget_tokens = budget_tokens
        max_pages = (max_seq_len + PAGE - 1) // PAGE
        want = max(min((budget_tokens + PAGE - 1) // PAGE, max_pages), (num_queries + PAGE - 2) // PAGE + 1)
        if token_granular:                                   # sel_table rows hold token slots
            want = min(max(budget_tokens, num_queries), max_seq_len)
        # two entries of slack; a row of token slots also needs room for the tokens a live drafting phase appends
        self.max_sel_blocks = max_sel_blocks or (want + 2 + (growth if token_granular else 0))
        common = dict(batch=batch, num_q_heads=num_q_heads, num_kv_heads=num_kv_heads, num_queries=num_queries,
                      max_blocks=max_blocks, max_sel_blocks=self.max_sel_blocks, num_pages=num_pages,
                      softmax_scale=softmax_scale, head_dim=head_dim)
        self.desc_verify = vb.make_desc(max_seq_len=max_seq_len, collect_rows=collect_rows,
                                        kv_chunk_tokens=verify_chunk, score_metric=score_metric, window=window,
                                        **common)
        if token_granular:
            draft_common = dict(common, max_blocks=self.max_sel_blocks, num_pages=num_pages * PAGE)
            # (a selection that holds the whole sequence grows past max_seq_len while drafting)
            self.desc_draft = vb.make_desc(max_seq_len=min(self.max_sel_blocks, max_seq_len + growth), collect_rows=vb.COLLECT_NONE,
                                           kv_chunk_tokens=draft_chunk, page_size=1, **draft_common)
        else:
            draft_len = min(self.max_sel_blocks * PAGE, max_blocks * PAGE)
            self.desc_draft = vb.make_desc(max_seq_len=draft_len, collect_rows=vb.COLLECT_NONE,
                                           kv_chunk_tokens=draft_chunk, **common)
        nbytes = max(vb.vegas_workspace_bytes(self.desc_verify), vb.vegas_workspace_bytes(self.desc_draft))
        if nbytes == 0:
            raise ValueError("descriptor rejected by vegas_workspace_bytes")
        dev = self.device
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.out_verify = torch.empty((batch, num_queries, num_q_heads, head_dim), dtype=torch.bfloat16, device=dev)
        per_page = PAGE if score_metric == vb.METRIC_TOKEN_LOGITS else 1       # token scores: one per token slot
        self.block_scores = torch.empty((batch, max_blocks * per_page), dtype=torch.float32, device=dev)
        self.sel_table = torch.empty((batch, self.max_sel_blocks), dtype=torch.int32, device=dev)
        self.sel_seq_lens = torch.empty((batch,), dtype=torch.int32, device=dev)
        self.out_draft = torch.empty((num_queries, batch, num_q_heads, head_dim), dtype=torch.bfloat16, device=dev)

        # the K/V append of a live drafting phase may take every sequence up to `growth` tokens past max_seq_len
        self.desc_append = vb.make_desc(max_seq_len=min(max_seq_len + growth, max_blocks * PAGE),
                                        collect_rows=vb.COLLECT_NONE, **common)
        # growing the selection: the block table's geometry with the selection's page size
        ext = dict(common, num_pages=num_pages * PAGE) if token_granular else common
        self.desc_extend = vb.make_desc(max_seq_len=min(max_seq_len + growth, max_blocks * PAGE),
                                        collect_rows=vb.COLLECT_NONE, page_size=1 if token_granular else PAGE, **ext)

    @classmethod
    def for_layer(cls, L: LayerInputs, budget_tokens: Optional[int] = None, **kw) -> "VegasPath":
        s = L.spec
        return cls(batch=s.batch, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads,
                   num_queries=s.num_queries, max_blocks=L.max_blocks,
                   max_seq_len=max(int(L.seq_lens.max()), 1), num_pages=L.num_pages,
                   budget_tokens=budget_tokens if budget_tokens is not None else s.budget_tokens,
                   softmax_scale=L.softmax_scale, head_dim=s.head_dim, **kw)

    def stream(self) -> int:
        return int(torch.cuda.current_stream(self.device).cuda_stream)

    # The calls below pass raw device addresses (cached per DeviceLayer) so that the host cost of one
    # call stays at a few microseconds: at batch 1 the kernels are that short.
    def _addrs(self, dl: DeviceLayer):
        a = getattr(dl, "_addrs", None)
        if a is None:
            # checked once per layer, since the calls below hand over addresses: both descriptors' cache extents
            for desc in (self.desc_verify, self.desc_draft):
                need = vb.cache_extent_bytes(desc)
                for name in ("k_cache", "v_cache"):
                    have = vb._avail_bytes(getattr(dl, name))
                    if have < need:
                        raise ValueError(f"{name} spans {have} bytes, the descriptor needs {need}")
            B, G = self.B, self.G
            if (dl.q_verify.numel() < B * G * self.Hq * self.D or dl.q_draft.numel() < G * B * self.Hq * self.D or
                    dl.block_table.numel() < B * self.desc_verify.max_blocks or dl.seq_lens.numel() < B):
                raise ValueError("layer tensors are smaller than the descriptor's shapes")
            step_bytes = dl.q_draft[0].numel() * dl.q_draft.element_size()
            a = dict(qv=dl.q_verify.data_ptr(), k=dl.k_cache.data_ptr(), v=dl.v_cache.data_ptr(),
                     bt=dl.block_table.data_ptr(), sl=dl.seq_lens.data_ptr(),
                     qd=[dl.q_draft.data_ptr() + i * step_bytes for i in range(dl.q_draft.shape[0])])
            dl._addrs = a
        return a

    def _own(self):
        o = getattr(self, "_own_addrs", None)
        if o is None:
            step_bytes = self.out_draft[0].numel() * self.out_draft.element_size()
            o = dict(ws=self.workspace.data_ptr(), wsn=self.workspace.numel(), ov=self.out_verify.data_ptr(),
                     bs=self.block_scores.data_ptr(), st=self.sel_table.data_ptr(), ssl=self.sel_seq_lens.data_ptr(),
                     od=[self.out_draft.data_ptr() + i * step_bytes for i in range(self.out_draft.shape[0])])
            self._own_addrs = o
        return o

    def verify(self, dl: DeviceLayer, stream=None, stages: int = 0) -> None:
        a, o = self._addrs(dl), self._own()
        vb.vegas_verify_attention(self.desc_verify, a["qv"], a["k"], a["v"], a["bt"], a["sl"], o["ov"], o["bs"],
                                  o["ws"], stream=self.stream() if stream is None else stream,
                                  workspace_bytes=o["wsn"], stages=stages)

    def select(self, dl: DeviceLayer, block_scores: Optional[torch.Tensor] = None, budgets=None, stream=None) -> None:
        a, o = self._addrs(dl), self._own()
        if self.token_granular:
            vb.vegas_select_tokens(self.desc_verify, o["bs"] if block_scores is None else block_scores,
                                   a["bt"], a["sl"], self.budget_tokens, o["st"], o["ssl"], o["ws"], budgets=budgets,
                                   stream=self.stream() if stream is None else stream, workspace_bytes=o["wsn"])
            return
        vb.vegas_select_blocks(self.desc_verify, o["bs"] if block_scores is None else block_scores,
                               a["bt"], a["sl"], self.budget_tokens, o["st"], o["ssl"], budgets=budgets,
                               stream=self.stream() if stream is None else stream)

    def draft(self, dl: DeviceLayer, step: int, stream=None, stages: int = 0) -> None:
        a, o = self._addrs(dl), self._own()
        vb.vegas_draft_attention(self.desc_draft, a["qd"][step], a["k"], a["v"], o["st"], o["ssl"], o["od"][step],
                                 o["ws"], stream=self.stream() if stream is None else stream,
                                 workspace_bytes=o["wsn"], stages=stages)

    def live_iteration(self, dl: DeviceLayer, fused: bool = True) -> None:
        """One decoding iteration with a live drafting phase (Sec. 2.3): verify and select at the layer's lengths,
        then per draft step the new token's K/V is appended, the selection grows by it (Sec. 3.2, last sentence)
        and the draft call attends over the grown selection.  The live lengths are rewound first (one small device
        copy), so every iteration starts from the same state; the appended slots are simply overwritten.
        fused: append and growth in one launch (vegas_append_kv_extend) instead of two calls."""
        st = self.stream()
        a, o = self._addrs(dl), self._own()
        dl.seq_lens_live.copy_(dl.seq_lens)
        self.verify(dl, st)
        self.select(dl, stream=st)
        sll = dl.seq_lens_live.data_ptr()
        row = dl.k_new[0].numel() * dl.k_new.element_size()
        for s in range(self.G):
            if fused:
                vb.vegas_append_kv_extend(self.desc_append, dl.k_new.data_ptr() + s * row, dl.v_new.data_ptr() + s * row,
                                          1, a["bt"], sll, a["k"], a["v"], o["st"], o["ssl"],
                                          self.desc_extend.page_size, stream=st)
            else:
                vb.vegas_append_kv(self.desc_append, dl.k_new.data_ptr() + s * row, dl.v_new.data_ptr() + s * row, 1,
                                   a["bt"], sll, a["k"], a["v"], stream=st)
                vb.vegas_extend_selection(self.desc_extend, a["bt"], sll, 1, o["st"], o["ssl"], stream=st)
            self.draft(dl, s, st)

    def iteration(self, dl: DeviceLayer) -> None:
        """One decoding iteration's attention work for one layer: verify, select, G draft steps."""
        st = self.stream()
        self.verify(dl, st)
        self.select(dl, stream=st)
        for s in range(self.G):
            self.draft(dl, s, st)
