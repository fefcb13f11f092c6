"""GPU parity of draft attention over tables of 1, 2, 4 and 8-token pages (Sec. 4: one-token pages with
the selected token indices as page indices; App. D: page sizes 1..16) against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16


def draft_small_pages(L, P, sel, ssl, step=0, chunk=0):
    """One draft call over `sel` (physical P-token page ids) through the C ABI; returns the bf16 output tensor."""
    s = L.spec
    dev = torch.device("cuda:0")
    B, msb = sel.shape
    desc = vb.make_desc(batch=B, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                        max_blocks=msb, max_sel_blocks=msb, max_seq_len=max(int(ssl.max()), 1),
                        num_pages=L.num_pages * (PAGE // P), softmax_scale=L.softmax_scale, page_size=P,
                        kv_chunk_tokens=chunk, head_dim=s.head_dim)
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    out = torch.full((B, s.num_q_heads, s.head_dim), float("nan"), dtype=torch.bfloat16, device=dev)
    vb.vegas_draft_attention(desc, harness.bf16_to_device(L.q_draft[step], dev), harness.bf16_to_device(L.k_cache, dev),
                             harness.bf16_to_device(L.v_cache, dev), torch.from_numpy(sel).to(dev),
                             torch.from_numpy(ssl).to(dev), out, ws)
    torch.cuda.synchronize()
    return out


def random_selection(L, P, rng, keep_fraction, msb_slack=3):
    """Per sequence: a random ascending subset of its P-token pages plus the last page, as physical ids
    of the pool seen with page size P; the last listed page keeps the sequence's own partial fill."""
    B = L.spec.batch
    sub = PAGE // P
    rows, lens = [], []
    for b in range(B):
        n = int(L.seq_lens[b])
        npg = (n + P - 1) // P
        if npg == 0:
            rows.append(np.zeros(0, dtype=np.int64)); lens.append(0); continue
        k = max(1, int(npg * keep_fraction))
        logical = np.sort(rng.choice(npg - 1, size=min(k - 1, npg - 1), replace=False)) if npg > 1 else np.zeros(0, int)
        logical = np.concatenate([logical, [npg - 1]]).astype(np.int64)
        phys = L.block_table[b, (logical * P) // PAGE].astype(np.int64) * sub + ((logical * P) % PAGE) // P
        rows.append(phys)
        lens.append(P * (len(logical) - 1) + (n - P * (npg - 1)))
    msb = max(len(r) for r in rows) + msb_slack
    sel = np.full((B, msb), -1, dtype=np.int32)
    for b, r in enumerate(rows):
        sel[b, :len(r)] = r
    return sel, np.array(lens, dtype=np.int32)


@pytest.mark.parametrize("P", [1, 2, 4, 8])
@pytest.mark.parametrize("sharp", [False, True], ids=["flat", "sharp"])
def test_small_page_draft_matches_oracle(P, sharp):
    L = synth.make_random_case(seed=300 + P, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[2500, 0, 333], logit_std=2.0 if sharp else 0.3, value_std=1.0,
                               outliers=3 if sharp else 0, outlier_logit=30.0)
    rng = np.random.default_rng(P)
    sel, ssl = random_selection(L, P, rng, keep_fraction=0.4)
    print(f"[case] small_pages P={P} sharp={sharp} sel_lens={ssl.tolist()}", flush=True)
    kc = L.k_cache.reshape(-1, P, L.spec.num_kv_heads, L.spec.head_dim)
    vc = L.v_cache.reshape(-1, P, L.spec.num_kv_heads, L.spec.head_dim)
    for chunk in (0, 128):                                       # the planner's chunking and many small chunks
        out = draft_small_pages(L, P, sel, ssl, step=1, chunk=chunk)
        ref = O.draft_attention(L.q_draft[1], kc, vc, sel, ssl, L.softmax_scale)
        U.check_out(f"small_pages.P{P}.chunk{chunk}", out, ref, U.vmax_visible(L))


def test_sub_pages_of_a_16_token_selection_give_the_same_bits():
    """Listing the selected 16-token pages as their P-token sub-pages feeds the small-page kernel the same tokens in
    the same order whatever P is, so the four listings (P = 1, 2, 4, 8: one kernel, four address generators) must
    agree bit for bit.  The 16-token-page call takes the 16-row kernel, whose contractions add in another order: it
    agrees with them to one unit in the last place of bf16."""
    L = synth.make_layer(synth.scaled(synth.CONFIGS["ctx4k"], seq_len=4096 + 7))
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L)
    path.iteration(dl)
    torch.cuda.synchronize()
    sel16 = path.sel_table.cpu().numpy()
    ssl = path.sel_seq_lens.cpu().numpy()
    ref16 = harness.bf16_to_host_f64(path.out_draft[2])
    s = L.spec
    dev = torch.device("cuda:0")
    k = int((sel16[0] >= 0).sum())
    bits = {}
    for P in (1, 2, 4, 8):
        sub = PAGE // P
        msb = path.max_sel_blocks * sub
        sel = np.full((1, msb), -1, dtype=np.int32)
        sel[0, :k * sub] = (sel16[0, :k, None].astype(np.int64) * sub + np.arange(sub)[None, :]).reshape(-1)
        # the planner chunks by max_seq_len: keep it equal to the 16-token call's (max_sel_blocks * 16)
        desc = vb.make_desc(batch=1, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                            max_blocks=msb, max_sel_blocks=msb, max_seq_len=path.desc_draft.max_seq_len,
                            num_pages=L.num_pages * sub, softmax_scale=L.softmax_scale, page_size=P)
        ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
        out = torch.empty((1, s.num_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
        print(f"[case] sub_pages P={P} k={k}", flush=True)
        vb.vegas_draft_attention(desc, dl.q_draft[2], dl.k_cache, dl.v_cache, torch.from_numpy(sel).to(dev),
                                 torch.from_numpy(ssl).to(dev), out, ws)
        torch.cuda.synchronize()
        bits[P] = out.view(torch.int16).cpu().numpy().copy()
        got = harness.bf16_to_host_f64(out)[0]
        ulp = np.maximum(np.abs(got), np.abs(ref16[0])) * 2.0 ** -7
        assert np.all(np.abs(got - ref16[0]) <= ulp + 1e-30), f"P={P}: more than one bf16 ulp from the 16-token call"
    for P in (1, 2, 4):
        assert np.array_equal(bits[P], bits[8]), f"P={P} and P=8 differ"


def test_small_pages_are_refused_outside_the_draft_call():
    desc = vb.make_desc(batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5, max_blocks=64, max_sel_blocks=64,
                        max_seq_len=64, num_pages=64, softmax_scale=0.1, page_size=1)
    dev = torch.device("cuda:0")
    z = torch.zeros(4096, dtype=torch.int32, device=dev)
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_select_blocks(desc, z.view(torch.float32), z, z, 16, z, z)
    assert e.value.status == vb.VEGAS_ERR_UNSUPPORTED


@pytest.mark.parametrize("P", [1, 4, 16])
def test_table5_shape_sampled_against_oracle(P):
    """The launch configuration bench.py times for the page-size sweep (App. D, Table 5: batch 16, 8192 selected
    tokens per request at random pool positions), on a smaller pool so that the host can hold it; three
    sampled requests are checked against the oracle element by element."""
    B, Hq, Hkv, D, sel_tokens = 16, 32, 8, 128, 8192
    pool_tokens = B * 16384
    rng = np.random.default_rng(55 + P)
    k_bits = synth.normal_pool_bf16(991, 0, (pool_tokens // PAGE, PAGE, Hkv, D), D ** -0.5)
    v_bits = synth.normal_pool_bf16(991, 1, (pool_tokens // PAGE, PAGE, Hkv, D), D ** -0.5)
    q_bits = synth.f32_to_bf16_bits(rng.standard_normal((B, Hq, D)).astype(np.float32) * 0.5)
    n_sel = sel_tokens // P
    ids = rng.choice(pool_tokens // P, size=B * n_sel, replace=False).astype(np.int32).reshape(B, n_sel)
    ids.sort(axis=1)
    ssl = np.full(B, sel_tokens, dtype=np.int32)
    ssl[3] = sel_tokens - P + max(1, P // 2)                     # one request ends in a partial page
    dev = torch.device("cuda:0")
    desc = vb.make_desc(batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=1, max_blocks=n_sel,
                        max_sel_blocks=n_sel, max_seq_len=sel_tokens, num_pages=pool_tokens // P,
                        softmax_scale=D ** -0.5, page_size=P)
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    out = torch.empty((B, Hq, D), dtype=torch.bfloat16, device=dev)
    print(f"[case] table5_shape P={P}", flush=True)
    vb.vegas_draft_attention(desc, harness.bf16_to_device(q_bits, dev), harness.bf16_to_device(k_bits, dev),
                             harness.bf16_to_device(v_bits, dev), torch.from_numpy(ids).to(dev),
                             torch.from_numpy(ssl).to(dev), out, ws)
    torch.cuda.synchronize()
    sample = [0, 3, 15]
    kc = k_bits.reshape(-1, P, Hkv, D)
    vc = v_bits.reshape(-1, P, Hkv, D)
    ref = O.draft_attention(q_bits[sample], kc, vc, ids[sample], ssl[sample], D ** -0.5)
    vmax = float(np.abs(O.decode_bf16(v_bits[:64])).max())
    U.check_out(f"table5_shape.P{P}", out[sample], ref, vmax)


FINISH_CASES = [
    # name, B, Hq, Hkv, D, P, lens, budget tokens
    ("hd128_pages16", 3, 32, 8, 128, 16, [4000, 0, 700], 256),
    ("hd64_pages16", 2, 32, 4, 64, 16, [2500, 37], 256),
    ("hd64_384_tokens", 2, 64, 8, 64, 16, [3000, 390], 384),
    ("three_row_blocks", 2, 80, 1, 128, 16, [1200, 5], 256),
    ("one_token_pages", 3, 16, 2, 128, 1, [900, 0, 288], 256),
    ("two_token_pages_hd64", 2, 8, 8, 64, 2, [300, 1], 256),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,D,P,lens,budget", FINISH_CASES, ids=[c[0] for c in FINISH_CASES])
def test_short_selections_need_no_merge_kernel(name, B, Hq, Hkv, D, P, lens, budget):
    """At most 256 selected tokens (384 at head dimension 64) plus two pages of slack, no chunk length passed: one
    workgroup per (sequence, KV head, row block) streams the whole selection and writes the output rows itself.
    Checked against the oracle, against the same call cut into 64-token chunks with a merge kernel, and on empty
    sequences (rows of zeros)."""
    rng = np.random.default_rng(len(name))
    L = synth.make_random_case(seed=940 + len(name), batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=2,
                               seq_lens=lens, head_dim=D, logit_std=1.5, value_std=1.0, outliers=2, outlier_logit=20.0)
    budget_pages = budget // P
    rows, sl = [], []
    for b in range(B):
        n = int(L.seq_lens[b])
        npg = (n + P - 1) // P
        if npg == 0:
            rows.append(np.zeros(0, dtype=np.int64)); sl.append(0); continue
        k = min(budget_pages, npg)
        logical = np.concatenate([np.sort(rng.choice(npg - 1, size=k - 1, replace=False)) if k > 1 else
                                  np.zeros(0, np.int64), [npg - 1]]).astype(np.int64)
        rows.append(L.block_table[b, (logical * P) // PAGE].astype(np.int64) * (PAGE // P) + ((logical * P) % PAGE) // P)
        sl.append(P * (k - 1) + (n - P * (npg - 1)))
    msb = budget_pages + 2 * (PAGE // P)                        # two 16-token pages of slack
    sel = np.full((B, msb), -1, dtype=np.int32)
    for b, r in enumerate(rows):
        sel[b, :len(r)] = r
    ssl = np.array(sl, dtype=np.int32)
    print(f"[case] merge-free draft {name} ssl={list(ssl)}", flush=True)
    s = L.spec
    desc = vb.make_desc(batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=1, max_blocks=msb, max_sel_blocks=msb,
                        max_seq_len=msb * P, num_pages=L.num_pages * (PAGE // P), softmax_scale=L.softmax_scale,
                        page_size=P, head_dim=D)
    dev = torch.device("cuda:0")
    args = (harness.bf16_to_device(L.q_draft[0], dev), harness.bf16_to_device(L.k_cache, dev),
            harness.bf16_to_device(L.v_cache, dev), torch.from_numpy(sel).to(dev), torch.from_numpy(ssl).to(dev))
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.bfloat16, device=dev)
    vb.vegas_draft_attention(desc, *args, out, ws, stages=vb.STAGE_STREAM)   # the streaming kernel alone completes the call
    torch.cuda.synchronize()
    kc = L.k_cache.reshape(-1, P, Hkv, D)
    vc = L.v_cache.reshape(-1, P, Hkv, D)
    ref = O.draft_attention(L.q_draft[0], kc, vc, sel, ssl, L.softmax_scale)
    U.check_out(name + ".merge_free", out, ref, U.vmax_visible(L))
    for b in range(B):
        if ssl[b] == 0:
            assert not out[b].float().abs().any(), "rows of an empty sequence must be zeros"
    chunked = draft_small_pages(L, P, sel, ssl, step=0, chunk=64)
    U.check_out(name + ".chunked", chunked, ref, U.vmax_visible(L))
    assert (out.float() - chunked.float()).abs().max().item() <= 2e-3 * U.vmax_visible(L)
