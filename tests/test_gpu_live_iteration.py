"""GPU parity of a live decoding iteration through the C ABI: verify -> select -> G x (append the drafted token's
K/V -> grow the selection -> draft), every stage of every step against the CPU oracle (Sec. 2.3: tokens are drafted
one after the other, each attending to its predecessors; Sec. 3.2, last sentence: only the prefix is sparsified,
what comes after it is kept).  The cache is compared bit for bit after every append, the selection bit for bit
after every growth step, the draft outputs within the output tolerance."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16


def bits_of(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_live(L, budget, name, token_granular=False, fused=True):
    G = L.spec.num_queries
    L = synth.with_growth(L, G)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=budget, growth=G, token_granular=token_granular,
                                       collect_rows=vb.COLLECT_FIRST_LAST if token_granular else vb.COLLECT_ALL_ROWS)
    P = 1 if token_granular else PAGE
    vs = U.vmax_visible(L)
    print(f"[case] live {name}: lens={list(map(int, L.seq_lens[:8]))} budget={budget} P={P}", flush=True)
    # the GPU runs the whole iteration as one stream of calls; the stages are then replayed one by one for comparison
    k0, v0 = dl.k_cache.clone(), dl.v_cache.clone()
    path.live_iteration(dl, fused=fused)      # fused: vegas_append_kv_extend, one launch per step instead of two
    torch.cuda.synchronize()
    # nothing the draft calls were given lay outside what their descriptor lets them see (they would clamp silently)
    err = torch.zeros(1, dtype=torch.int32, device=path.device)
    vb.vegas_debug_check_tables(path.desc_draft, vb.TABLE_SELECTION, path.sel_table, path.sel_seq_lens, err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0, f"{name}: the grown selection trips the table checker: bits {int(err.item())}"
    final_out = [path.out_draft[s].clone() for s in range(G)]
    final_sel, final_ssl = path.sel_table.cpu().numpy(), path.sel_seq_lens.cpu().numpy()
    final_k, final_lens = bits_of(dl.k_cache), dl.seq_lens_live.cpu().numpy()

    # stage by stage from the same starting state, oracle beside it
    dl.k_cache.copy_(k0)
    dl.v_cache.copy_(v0)
    dl.seq_lens_live.copy_(dl.seq_lens)
    path.verify(dl)
    path.select(dl)
    torch.cuda.synchronize()
    sel, ssl = path.sel_table.cpu().numpy(), path.sel_seq_lens.cpu().numpy()   # the GPU's own selection is carried on
    if not token_granular:
        ref_out, ref_scores = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens,
                                                 L.softmax_scale)
        U.check_out(name + ".verify", path.out_verify, ref_out, vs)
        U.check_scores(name + ".scores", path.block_scores, ref_scores)
    kc, vc, lens = L.k_cache, L.v_cache, L.seq_lens
    st = path.stream()
    row = dl.k_new[0].numel() * dl.k_new.element_size()
    for s in range(G):
        vb.vegas_append_kv(path.desc_append, dl.k_new.data_ptr() + s * row, dl.v_new.data_ptr() + s * row, 1,
                           dl.block_table, dl.seq_lens_live, dl.k_cache, dl.v_cache, stream=st)
        kc, vc, lens = O.append_kv(kc, vc, L.k_new[s], L.v_new[s], L.block_table, lens,
                                   max_seq_len=path.desc_append.max_seq_len)
        torch.cuda.synchronize()
        assert np.array_equal(dl.seq_lens_live.cpu().numpy(), lens), f"{name}: lengths after append {s}"
        assert np.array_equal(bits_of(dl.k_cache), kc) and np.array_equal(bits_of(dl.v_cache), vc), \
            f"{name}: cache after append {s}"
        vb.vegas_extend_selection(path.desc_extend, dl.block_table, dl.seq_lens_live, 1, path.sel_table,
                                  path.sel_seq_lens, stream=st)
        sel, ssl = O.extend_selection(sel, ssl, L.block_table, lens, 1, P)
        torch.cuda.synchronize()
        assert np.array_equal(path.sel_table.cpu().numpy(), sel), f"{name}: selection after step {s}"
        assert np.array_equal(path.sel_seq_lens.cpu().numpy(), ssl), f"{name}: covered length after step {s}"
        path.draft(dl, s)
        torch.cuda.synchronize()
        kview = kc.reshape(-1, P, kc.shape[2], kc.shape[3])
        vview = vc.reshape(-1, P, vc.shape[2], vc.shape[3])
        ref_d = O.draft_attention(L.q_draft[s], kview, vview, sel, ssl, L.softmax_scale)
        U.check_out(f"{name}.draft{s}", path.out_draft[s], ref_d, vs)
        # the uninterrupted run produced the same bits
        assert torch.equal(path.out_draft[s].view(torch.int16), final_out[s].view(torch.int16)), f"{name}: step {s}"
    assert np.array_equal(final_sel, sel) and np.array_equal(final_ssl, ssl)
    assert np.array_equal(final_k, kc) and np.array_equal(final_lens, lens)
    # the newest token is always among the keys of the draft that follows its append
    for b in range(L.spec.batch):
        if L.seq_lens[b] > 0:
            assert ssl[b] >= G


LIVE = [
    # name, B, Hq, Hkv, G, lens, budget
    ("crosses_a_page", 1, 32, 8, 5, [2045], 256),             # positions 2045..2049: a new 16-token page at 2048
    ("page_aligned", 1, 32, 8, 5, [4096], 512),               # the first appended token opens a page
    ("ragged_batch", 4, 32, 8, 5, [700, 2049, 31, 1600], 160),
    ("with_empty_sequence", 3, 32, 8, 3, [900, 0, 47], 64),
    ("group8_gamma6", 2, 64, 8, 7, [1500, 3001], 320),
    ("budget_covers_everything", 2, 32, 8, 5, [300, 77], 10 ** 6),
]


@pytest.mark.parametrize("fused", [True, False], ids=["one_launch", "two_calls"])
@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,budget", LIVE, ids=[c[0] for c in LIVE])
def test_live_iteration_pages(name, B, Hq, Hkv, G, lens, budget, fused):
    L = synth.make_random_case(seed=600 + len(name), batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=G,
                               seq_lens=lens, logit_std=1.5, value_std=1.0, outliers=2, outlier_logit=20.0)
    run_live(L, budget, name, fused=fused)


LIVE_TOKENS = LIVE[:4] + [
    # every token selected: the selection then grows past the longest sequence of the batch
    ("all_tokens_selected", 2, 64, 8, 6, [20, 10], 200),
    ("all_tokens_selected_one_sequence", 1, 16, 4, 5, [58], 200),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,budget", LIVE_TOKENS, ids=[c[0] for c in LIVE_TOKENS])
def test_live_iteration_tokens(name, B, Hq, Hkv, G, lens, budget):
    """The paper's own granularity: token selection from averaged logits, one-token pages, growing by one entry a step."""
    L = synth.make_random_case(seed=650 + len(name), batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=G,
                               seq_lens=lens, logit_std=1.5, value_std=1.0, outliers=2, outlier_logit=20.0)
    run_live(L, min(budget, 200), name + ".tokens", token_granular=True)


def test_live_iteration_ctx32k_full_size():
    run_live(synth.make_layer(synth.CONFIGS["ctx32k"]), synth.CONFIGS["ctx32k"].budget_tokens, "ctx32k")


def test_append_refuses_a_sequence_without_room():
    """A sequence whose table row (or the descriptor's bound) has no room for the new tokens keeps its length and
    nothing of it is written; its neighbours are appended to as usual."""
    L = synth.make_random_case(seed=41, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=2, seq_lens=[100, 160, 40],
                               max_blocks=10)
    rng = np.random.default_rng(5)
    k_new = rng.integers(0, 0x7F00, size=(3, 2, 8, 128), dtype=np.uint16)
    v_new = rng.integers(0, 0x7F00, size=(3, 2, 8, 128), dtype=np.uint16)
    table = L.block_table.copy()                        # (positions 100, 101 and 40, 41 lie in pages the rows already name)
    dev = torch.device("cuda:0")
    desc = vb.make_desc(batch=3, num_q_heads=32, num_kv_heads=8, num_queries=2, max_blocks=10, max_sel_blocks=4,
                        max_seq_len=160, num_pages=L.num_pages, softmax_scale=0.1)
    dk, dv = harness.bf16_to_device(L.k_cache, dev), harness.bf16_to_device(L.v_cache, dev)
    lens = torch.from_numpy(L.seq_lens.copy()).to(dev)
    vb.vegas_append_kv(desc, harness.bf16_to_device(k_new, dev), harness.bf16_to_device(v_new, dev), 2,
                       torch.from_numpy(table).to(dev), lens, dk, dv)
    torch.cuda.synchronize()
    kc, vc, ref_lens = O.append_kv(L.k_cache, L.v_cache, k_new, v_new, table, L.seq_lens, max_seq_len=160)
    assert list(ref_lens) == [102, 160, 42]
    assert np.array_equal(lens.cpu().numpy(), ref_lens)
    assert np.array_equal(bits_of(dk), kc) and np.array_equal(bits_of(dv), vc)


@pytest.mark.parametrize("P", [16, 1])
def test_fused_append_and_growth_leave_a_refused_sequence_alone(P):
    """vegas_append_kv_extend: a sequence without room keeps its length, its cache slots AND its selection; the
    others get exactly what the two separate calls give (the oracle's append followed by its growth step)."""
    L = synth.make_random_case(seed=43, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=2, seq_lens=[100, 160, 47],
                               max_blocks=10)
    rng = np.random.default_rng(6)
    table = L.block_table.copy()                        # position 48 of the last sequence needs a page of its own
    table[2, 3] = sorted(set(range(L.num_pages)) - set(table[table >= 0].tolist()))[0]
    k_new = rng.integers(0, 0x7F00, size=(3, 1, 8, 128), dtype=np.uint16)
    v_new = rng.integers(0, 0x7F00, size=(3, 1, 8, 128), dtype=np.uint16)
    dev = torch.device("cuda:0")
    msb = 12 if P == 16 else 170
    if P == 16:
        sel, ssl, _ = O.select_blocks(rng.random((3, 10)).astype(np.float32), table, L.seq_lens, 2, 64, msb)
    else:
        sel, ssl, _ = O.select_tokens(rng.standard_normal((3, 160)).astype(np.float32), table, L.seq_lens, 2, 64, msb)
    desc = vb.make_desc(batch=3, num_q_heads=32, num_kv_heads=8, num_queries=2, max_blocks=10, max_sel_blocks=msb,
                        max_seq_len=160, num_pages=L.num_pages, softmax_scale=0.1)
    dk, dv = harness.bf16_to_device(L.k_cache, dev), harness.bf16_to_device(L.v_cache, dev)
    lens = torch.from_numpy(L.seq_lens.copy()).to(dev)
    d_sel, d_ssl = torch.from_numpy(sel.copy()).to(dev), torch.from_numpy(ssl.copy()).to(dev)
    ref_sel, ref_ssl, ref_lens = sel, ssl, L.seq_lens
    kc, vc = L.k_cache, L.v_cache
    for step in range(2):                               # 47 -> 48 -> 49: the second step opens a 16-token page
        vb.vegas_append_kv_extend(desc, harness.bf16_to_device(k_new, dev), harness.bf16_to_device(v_new, dev), 1,
                                  torch.from_numpy(table).to(dev), lens, dk, dv, d_sel, d_ssl, P)
        torch.cuda.synchronize()
        kc, vc, new_lens = O.append_kv(kc, vc, k_new, v_new, table, ref_lens, max_seq_len=160)
        grown_sel, grown_ssl = O.extend_selection(ref_sel, ref_ssl, table, new_lens, 1, P)
        # the sequence at its bound was refused: the oracle's growth step would re-add its last position, the call must not
        grown_sel[1], grown_ssl[1] = ref_sel[1], ref_ssl[1]
        ref_sel, ref_ssl, ref_lens = grown_sel, grown_ssl, new_lens
        assert list(ref_lens) == [101 + step, 160, 48 + step]
        assert np.array_equal(lens.cpu().numpy(), ref_lens)
        assert np.array_equal(bits_of(dk), kc) and np.array_equal(bits_of(dv), vc)
        assert np.array_equal(d_sel.cpu().numpy(), ref_sel) and np.array_equal(d_ssl.cpu().numpy(), ref_ssl)
    assert int(ref_ssl[0]) == int(ssl[0]) + 2 and int(ref_ssl[1]) == int(ssl[1])
