"""GPU parity: per-sequence budgets from a sparsity ratio (App. C) and growth of a selection by freshly
appended tokens while drafting (Sec. 3.2, last sentence), both against the CPU oracle (integer work: bit-exact)."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16


@pytest.mark.parametrize("ratio", [0.07, 0.5, 0.013])
def test_ratio_budgets_pages_and_tokens(ratio):
    rng = np.random.default_rng(17)
    lens = np.array([32768, 4099, 0, 3, 9001, 77], dtype=np.int32)
    B = len(lens)
    mb = (int(lens.max()) + PAGE - 1) // PAGE
    table = np.stack([rng.permutation(mb + 9)[:mb] for _ in range(B)]).astype(np.int32)
    G = 5
    budgets = O.ratio_budgets(lens, ratio)
    dev = torch.device("cuda:0")
    print(f"[case] ratio budgets {ratio}: {budgets.tolist()}", flush=True)
    # pages
    msb = int(np.ceil(np.float32(ratio) * np.float32(lens.max()))) // PAGE + 4
    scores = rng.random((B, mb)).astype(np.float32)
    desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=mb, max_sel_blocks=msb,
                        max_seq_len=int(lens.max()), num_pages=mb + 9, softmax_scale=0.1, budget_ratio=ratio)
    sel = torch.empty((B, msb), dtype=torch.int32, device=dev)
    ssl = torch.empty((B,), dtype=torch.int32, device=dev)
    vb.vegas_select_blocks(desc, torch.from_numpy(scores).to(dev), torch.from_numpy(table).to(dev),
                           torch.from_numpy(lens).to(dev), 1, sel, ssl)           # the constant budget is ignored
    torch.cuda.synchronize()
    ref_sel, ref_ssl, _ = O.select_blocks(scores, table, lens, G, 1, msb, budgets)
    assert np.array_equal(sel.cpu().numpy(), ref_sel) and np.array_equal(ssl.cpu().numpy(), ref_ssl)
    # tokens
    mst = int(budgets.max()) + 8
    tscores = rng.standard_normal((B, mb * PAGE)).astype(np.float32)
    desc_t = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=mb, max_sel_blocks=mst,
                          max_seq_len=int(lens.max()), num_pages=mb + 9, softmax_scale=0.1, budget_ratio=ratio)
    ws = torch.empty(vb.vegas_workspace_bytes(desc_t), dtype=torch.uint8, device=dev)
    selt = torch.empty((B, mst), dtype=torch.int32, device=dev)
    sslt = torch.empty((B,), dtype=torch.int32, device=dev)
    vb.vegas_select_tokens(desc_t, torch.from_numpy(tscores).to(dev), torch.from_numpy(table).to(dev),
                           torch.from_numpy(lens).to(dev), 1, selt, sslt, ws)
    torch.cuda.synchronize()
    ref_sel, ref_ssl, _ = O.select_tokens(tscores, table, lens, G, 1, mst, budgets)
    assert np.array_equal(selt.cpu().numpy(), ref_sel) and np.array_equal(sslt.cpu().numpy(), ref_ssl)


@pytest.mark.parametrize("P", [16, 1])
def test_selection_grows_with_appended_tokens(P):
    """verify/select at the old lengths, then three draft steps that each append one token: the selection is
    extended on the GPU, compared bit for bit with the oracle's, and drafted over."""
    steps = 3
    lens_old = np.array([2047, 800, 0, 1599], dtype=np.int32)             # 2047 -> 2048 starts a new 16-token page
    L = synth.make_random_case(seed=905, batch=4, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=(lens_old + steps).tolist(), logit_std=1.0, value_std=1.0, outliers=2)
    lens_old[2] = 0
    s = L.spec
    G = s.num_queries
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(3)
    mb = L.max_blocks
    if P == 16:
        scores = rng.random((s.batch, mb)).astype(np.float32)
        msb = 12
        sel, ssl, _ = O.select_blocks(scores, L.block_table, lens_old, G, 128, msb)
        kc, vc, npages = L.k_cache, L.v_cache, L.num_pages
    else:
        scores = rng.standard_normal((s.batch, mb * PAGE)).astype(np.float32)
        msb = 140
        sel, ssl, _ = O.select_tokens(scores, L.block_table, lens_old, G, 128, msb)
        kc = L.k_cache.reshape(-1, 1, s.num_kv_heads, s.head_dim)
        vc = L.v_cache.reshape(-1, 1, s.num_kv_heads, s.head_dim)
        npages = L.num_pages * PAGE
    desc = vb.make_desc(batch=s.batch, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                        max_blocks=mb, max_sel_blocks=msb, max_seq_len=min(msb * P, mb * PAGE), num_pages=npages,
                        softmax_scale=L.softmax_scale, page_size=P)
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    d_sel, d_ssl = torch.from_numpy(sel).to(dev), torch.from_numpy(ssl).to(dev)
    d_table = torch.from_numpy(L.block_table).to(dev)
    dk, dv = harness.bf16_to_device(L.k_cache, dev), harness.bf16_to_device(L.v_cache, dev)
    ref_sel, ref_ssl = sel, ssl
    for step in range(steps):
        lens_now = np.where(lens_old > 0, lens_old + step + 1, 0).astype(np.int32)
        print(f"[case] growth P={P} step={step} lens={lens_now.tolist()}", flush=True)
        vb.vegas_extend_selection(desc, d_table, torch.from_numpy(lens_now).to(dev), 1, d_sel, d_ssl)
        ref_sel, ref_ssl = O.extend_selection(ref_sel, ref_ssl, L.block_table, lens_now, 1, P)
        torch.cuda.synchronize()
        assert np.array_equal(d_sel.cpu().numpy(), ref_sel) and np.array_equal(d_ssl.cpu().numpy(), ref_ssl)
        out = torch.empty((s.batch, s.num_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
        vb.vegas_draft_attention(desc, harness.bf16_to_device(L.q_draft[step], dev), dk, dv, d_sel, d_ssl, out, ws)
        torch.cuda.synchronize()
        ref = O.draft_attention(L.q_draft[step], kc, vc, ref_sel, ref_ssl, L.softmax_scale)
        U.check_out(f"growth.P{P}.step{step}", out, ref, U.vmax_visible(L))
    assert int(ref_ssl[0]) == int(ssl[0]) + steps
