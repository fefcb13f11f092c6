"""GPU parity of the second attention shape, head dimension 64 (App. D: 2 KB of K+V per token; 64 query /
8 KV heads as in the paper's gpt-oss-20b runs), against the CPU oracle: the whole verify -> select -> draft
chain, both collection modes, the token-logit metric, small draft pages and local masking."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U
from tests.test_gpu_parity import run_chain
from tests.test_gpu_small_pages import draft_small_pages, random_selection
from tests.test_gpu_token_variant import check_token_scores, verify_token_scores

pytestmark = pytest.mark.gpu
PAGE = 16
D = 64

SMALL = [
    # name, B, Hq, Hkv, G, lens, kwargs
    ("one_tile", 1, 32, 8, 5, [32], {}),
    ("ragged_tail", 1, 32, 8, 5, [1000], {}),
    ("tiny", 2, 32, 8, 5, [5, 17], {}),
    ("batch_ragged_chunks", 3, 32, 8, 5, [700, 2049, 31], dict(verify_chunk=256)),
    ("group8_two_row_blocks", 2, 64, 8, 5, [1500, 640], {}),
    ("group8_chunks", 1, 64, 8, 5, [4100], dict(verify_chunk=1024)),
    ("single_query", 1, 32, 8, 1, [777], {}),
    ("mha_like", 1, 8, 8, 3, [900], {}),
    ("rows96_many_chunks", 2, 64, 8, 12, [9000, 77], dict(verify_chunk=128, draft_chunk=128)),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,kw", SMALL, ids=[c[0] for c in SMALL])
@pytest.mark.parametrize("sharp", [False, True], ids=["flat", "sharp"])
def test_small_cases_head_dim_64(name, B, Hq, Hkv, G, lens, kw, sharp):
    L = synth.make_random_case(seed=900 + len(name) + 7 * G, batch=B, num_q_heads=Hq, num_kv_heads=Hkv,
                               num_queries=G, seq_lens=lens, head_dim=D,
                               logit_std=2.0 if sharp else 0.3, value_std=1.0,
                               outliers=3 if sharp else 0, outlier_logit=30.0)
    budget = max(32, (max(lens) // 10) // PAGE * PAGE)
    run_chain(L, budget, name="hd64." + name + ("_sharp" if sharp else "_flat"), **kw)


def test_first_last_rows_head_dim_64():
    L = synth.make_random_case(seed=977, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=6,
                               seq_lens=[1234, 4000], head_dim=D, logit_std=1.0, outliers=2)
    run_chain(L, 256, collect=vb.COLLECT_FIRST_LAST, name="hd64.collect_first_last")


def test_gpt_oss_like_shape_32k_full():
    """64 query / 8 KV heads of dimension 64 at 32K context, the launch configuration bench.py times for
    --workload hd64_ctx32k."""
    L = synth.make_layer(synth.EXTRA_CONFIGS["hd64_ctx32k"])
    path, _, _ = run_chain(L, L.spec.budget_tokens, name="hd64_ctx32k")
    sel = path.sel_table.cpu().numpy()[0]
    inv = {int(p): j for j, p in enumerate(L.block_table[0])}
    ids = {inv[int(p)] for p in sel if p >= 0}
    assert set(np.unique(L.hitters[0] // PAGE)).issubset(ids)        # planted hitters are selected
    assert set(np.unique(L.sinks[0] // PAGE)).issubset(ids)


@pytest.mark.parametrize("collect", [vb.COLLECT_FIRST_LAST, vb.COLLECT_ALL_ROWS], ids=["eq3", "eq2"])
def test_token_logit_scores_head_dim_64(collect):
    L = synth.make_random_case(seed=930, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[700, 2049, 3], head_dim=D, logit_std=2.0, value_std=1.0, outliers=3,
                               outlier_logit=30.0)
    print(f"[case] hd64 token_scores collect={collect}", flush=True)
    dl, path = verify_token_scores(L, collect, 256)
    check_token_scores("hd64.token_scores", L, path, collect)
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale, 0)
    U.check_out("hd64.token_scores.out", path.out_verify, ref_out, U.vmax_visible(L))


@pytest.mark.parametrize("P", [1, 2, 4, 8])
def test_small_page_draft_head_dim_64(P):
    L = synth.make_random_case(seed=940 + P, batch=3, num_q_heads=64, num_kv_heads=8, num_queries=5,
                               seq_lens=[2500, 0, 333], head_dim=D, logit_std=2.0, value_std=1.0, outliers=3,
                               outlier_logit=30.0)
    rng = np.random.default_rng(40 + P)
    sel, ssl = random_selection(L, P, rng, keep_fraction=0.4)
    print(f"[case] hd64 small_pages P={P} sel_lens={ssl.tolist()}", flush=True)
    kc = L.k_cache.reshape(-1, P, L.spec.num_kv_heads, D)
    vc = L.v_cache.reshape(-1, P, L.spec.num_kv_heads, D)
    for chunk in (0, 128):
        out = draft_small_pages(L, P, sel, ssl, step=1, chunk=chunk)
        ref = O.draft_attention(L.q_draft[1], kc, vc, sel, ssl, L.softmax_scale)
        U.check_out(f"hd64.small_pages.P{P}.chunk{chunk}", out, ref, U.vmax_visible(L))


@pytest.mark.parametrize("name,B,Hq,G,lens,window,chunk", [
    ("w128_multi_chunk", 1, 32, 5, [5000], 128, 0),
    ("w100_ragged", 3, 32, 5, [700, 2049, 3], 100, 256),
    ("w128_group8_many_chunks", 2, 64, 5, [9000, 130], 128, 128),
], ids=["w128_multi_chunk", "w100_ragged", "w128_group8_many_chunks"])
def test_local_masking_head_dim_64(name, B, Hq, G, lens, window, chunk):
    L = synth.make_random_case(seed=960 + len(name), batch=B, num_q_heads=Hq, num_kv_heads=8, num_queries=G,
                               seq_lens=lens, head_dim=D, logit_std=1.5, value_std=1.0, outliers=2,
                               outlier_logit=20.0)
    print(f"[case] hd64 window {name} W={window}", flush=True)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=64, collect_rows=vb.COLLECT_NONE, verify_chunk=chunk,
                                       window=window)
    path.workspace.fill_(0xFF)
    path.out_verify.fill_(float("nan"))
    path.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale,
                                    0, window=window)
    U.check_out("hd64." + name, path.out_verify, ref_out, U.vmax_visible(L))


def test_other_head_dims_are_refused():
    desc = vb.make_desc(batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5, max_blocks=64, max_sel_blocks=64,
                        max_seq_len=1024, num_pages=64, softmax_scale=0.1, head_dim=96)
    assert vb.vegas_workspace_bytes(desc) == 0


@pytest.mark.parametrize("chunk", [64, 192, 256, 0])
def test_two_row_blocks_from_one_read_head_dim_64(chunk):
    L = synth.make_random_case(seed=990 + chunk, batch=3, num_q_heads=64, num_kv_heads=8, num_queries=5,
                               seq_lens=[1000, 2049 + 32, 31], head_dim=D, logit_std=2.0, value_std=1.0, outliers=3,
                               outlier_logit=30.0)
    run_chain(L, 128, verify_chunk=chunk, name=f"hd64.pair.chunk{chunk}")
