"""vegas_draft_attention_static (the entry point that allocates nothing: its chunk partials live in a scratch
array inside the library's device image) against vegas_draft_attention with a caller's workspace, through the
C ABI: same kernels, so the outputs must agree bit for bit -- on two calls in a row, the second one smaller, since
every call on a device shares the one array and finds the previous call's contents in it.  The first call is also
held to the oracle's bar, so that "both wrong in the same way" cannot pass."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16


def selection_of(L, rng, keep_pages):
    """A random ascending selection of `keep_pages` 16-token pages per sequence (the last page always in it)."""
    B = L.spec.batch
    rows, lens = [], []
    for b in range(B):
        n = int(L.seq_lens[b])
        npg = (n + PAGE - 1) // PAGE
        logical = np.sort(rng.choice(npg - 1, size=min(keep_pages - 1, npg - 1), replace=False))
        logical = np.concatenate([logical, [npg - 1]]).astype(np.int64)
        rows.append(L.block_table[b, logical])
        lens.append(PAGE * (len(logical) - 1) + (n - PAGE * (npg - 1)))
    msb = max(len(r) for r in rows) + 2
    sel = np.full((B, msb), -1, dtype=np.int32)
    for b, r in enumerate(rows):
        sel[b, :len(r)] = r
    return sel, np.array(lens, dtype=np.int32)


def both_ways(L, sel, ssl):
    s = L.spec
    dev = torch.device("cuda:0")
    B, msb = sel.shape
    desc = vb.make_desc(batch=B, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                        max_blocks=msb, max_sel_blocks=msb, max_seq_len=msb * PAGE, num_pages=L.num_pages,
                        softmax_scale=L.softmax_scale, head_dim=s.head_dim)
    assert vb.vegas_workspace_bytes(desc) <= vb.vegas_static_scratch_bytes()
    args = (harness.bf16_to_device(L.q_draft[0], dev), harness.bf16_to_device(L.k_cache, dev),
            harness.bf16_to_device(L.v_cache, dev), torch.from_numpy(sel).to(dev), torch.from_numpy(ssl).to(dev))
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    want = torch.full((B, s.num_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=dev)
    got = torch.full_like(want, float("nan"))
    vb.vegas_draft_attention(desc, *args, want, ws)
    vb.vegas_draft_attention_static(desc, *args, got)
    torch.cuda.synchronize()
    return want, got


def test_static_scratch_draft_equals_workspace_draft_on_two_calls_in_a_row():
    rng = np.random.default_rng(20260)
    # first call: three sequences, 130-page selections (several chunks per KV head and a merge kernel)
    big = synth.make_layer(synth.scaled(synth.CONFIGS["ctx4k"], batch=3, seq_len=4096 - 5, hitters=8))
    sel, ssl = selection_of(big, rng, 130)
    print(f"[case] static scratch, first call: batch 3, ssl={list(ssl)}", flush=True)
    want, got = both_ways(big, sel, ssl)
    assert torch.equal(want.view(torch.int16), got.view(torch.int16))
    ref = O.draft_attention(big.q_draft[0], big.k_cache, big.v_cache, sel, ssl, big.softmax_scale)
    U.check_out("static.first", got, ref, U.vmax_visible(big))
    # second call, smaller: one sequence, 40 pages -- the array still holds the first call's partials
    small = synth.make_layer(synth.scaled(synth.CONFIGS["ctx4k"], seq_len=1500, hitters=4))
    sel2, ssl2 = selection_of(small, rng, 40)
    print(f"[case] static scratch, second call: batch 1, ssl={list(ssl2)}", flush=True)
    want2, got2 = both_ways(small, sel2, ssl2)
    assert torch.equal(want2.view(torch.int16), got2.view(torch.int16))
    ref2 = O.draft_attention(small.q_draft[0], small.k_cache, small.v_cache, sel2, ssl2, small.softmax_scale)
    U.check_out("static.second", got2, ref2, U.vmax_visible(small))
