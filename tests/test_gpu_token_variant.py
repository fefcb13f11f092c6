"""GPU parity of the paper's own selection variant -- attention logits as the metric, single tokens as the
unit (Sec. 3.2 footnote, Sec. 3.3 last paragraph, Sec. 4, App. B) -- against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16

# Error bound of one token score.  The kernel contracts k_i with the sum of the collected query rows split
# into a bf16 high and low part (2^-17 per element) and accumulates 128 products per head in fp32 (128 * 2^-24);
# both are relative to sum_d |qbar_d| |k_d|.  4e-5 covers 2^-17 + 2^-17 + slack for the sum over heads.
TOKEN_SCORE_REL = 4e-5


def token_score_bound(L, collect):
    """Per token: softmax_scale / (|R| H_q) * sum_h sum_d |qbar[h, d]| |k[i, h, d]| (what the error is relative to)."""
    s = L.spec
    G, Hq, Hkv, D = s.num_queries, s.num_q_heads, s.num_kv_heads, s.head_dim
    g = Hq // Hkv
    rows = list(O.collected_rows(G, collect))
    q = O.decode_bf16(L.q_verify)
    out = np.zeros((s.batch, L.block_table.shape[1] * PAGE))
    for b in range(s.batch):
        n = int(L.seq_lens[b])
        p_len = max(n - G, 0)
        if p_len == 0:
            continue
        qbar = np.abs(q[b, rows].reshape(len(rows), Hkv, g, D).sum(axis=(0, 2)))          # [Hkv, D]
        for hk in range(Hkv):
            K = np.abs(O.gather_sequence(L.k_cache, L.block_table[b], p_len, hk))
            out[b, :p_len] += K @ qbar[hk]
        out[b] *= L.softmax_scale / (len(rows) * Hq)
    return out


def verify_token_scores(L, collect, verify_chunk=0):
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, collect_rows=collect, verify_chunk=verify_chunk,
                                       score_metric=vb.METRIC_TOKEN_LOGITS)
    path.block_scores.fill_(float("nan"))
    path.verify(dl)
    torch.cuda.synchronize()
    return dl, path


def check_token_scores(name, L, path, collect):
    ref = O.token_logit_scores(L.q_verify, L.k_cache, L.block_table, L.seq_lens, L.softmax_scale, collect)
    got = path.block_scores.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), name + ": non-finite token score"
    bound = token_score_bound(L, collect)
    err = np.abs(got - ref)
    bad = err > TOKEN_SCORE_REL * bound + 1e-12
    assert not bad.any(), f"{name}: {int(bad.sum())} token scores off, worst err/bound {float((err / np.maximum(bound, 1e-30))[bad].max()):.3e}"
    G = L.spec.num_queries
    for b in range(L.spec.batch):                                 # entries outside the prefix are written as 0
        assert np.all(got[b, max(int(L.seq_lens[b]) - G, 0):] == 0.0)
    return ref, got


CASES = [
    # name, B, Hq, Hkv, G, lens, verify_chunk
    ("basic", 1, 32, 8, 5, [3000], 0),
    ("ragged_batch", 3, 32, 8, 5, [700, 2049, 3], 256),
    ("gamma6", 1, 32, 8, 7, [5000], 512),
    ("group8_two_row_blocks", 2, 64, 8, 5, [1500, 640], 0),
    ("group8_two_row_blocks_chunk192", 2, 64, 8, 5, [1500, 640 + 45], 192),
    ("rows62_chunk64", 1, 62, 2, 2, [700], 64),
    ("group8_long_chunk_rings", 2, 64, 8, 5, [9000, 4100], 4096),
    ("single_row", 1, 32, 8, 1, [777], 0),
    ("mha_like", 1, 8, 8, 3, [900], 0),
    # row counts whose last 32-row block has no two spare rows: the query-sum rows get a row block of their own
    ("rows32_gamma7_group4", 1, 32, 8, 8, [3000], 0),              # gamma = 7 with a 4-head group (Table 1's gamma)
    ("rows32_ragged_batch", 3, 32, 8, 8, [700, 2049, 5], 256),
    ("rows64_gamma15_group4", 2, 32, 8, 16, [1500, 640], 0),
    ("rows31", 1, 31, 1, 1, [900], 0),
    ("rows63", 2, 63, 1, 1, [1300, 77], 128),
    ("rows64_group8", 1, 64, 8, 8, [2100], 512),
    ("rows96_group8", 1, 64, 8, 12, [1100], 0),
    ("rows128", 1, 64, 4, 8, [1000], 0),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,chunk", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("collect", [vb.COLLECT_FIRST_LAST, vb.COLLECT_ALL_ROWS], ids=["eq3", "eq2"])
def test_token_logit_scores(name, B, Hq, Hkv, G, lens, chunk, collect):
    L = synth.make_random_case(seed=500 + len(name) + G, batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=G,
                               seq_lens=lens, logit_std=2.0, value_std=1.0, outliers=3, outlier_logit=30.0)
    print(f"[case] token_scores {name} collect={collect}", flush=True)
    dl, path = verify_token_scores(L, collect, chunk)
    check_token_scores(name, L, path, collect)
    # the attention output of the same call is unchanged by what is collected
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale, 0)
    U.check_out(name + ".out", path.out_verify, ref_out, U.vmax_visible(L))


def test_token_logit_scores_ctx32k_full():
    L = synth.make_layer(synth.CONFIGS["ctx32k"])
    dl, path = verify_token_scores(L, vb.COLLECT_FIRST_LAST)
    ref, got = check_token_scores("ctx32k", L, path, vb.COLLECT_FIRST_LAST)
    # planted heavy hitters and sinks carry the largest averaged logits
    top = np.argsort(-got[0, :int(L.seq_lens[0]) - L.spec.num_queries])[:len(L.hitters[0]) + len(L.sinks[0])]
    assert set(map(int, L.hitters[0])).issubset(set(map(int, top)))


def test_chain_with_32_rows_per_kv_head():
    """gamma = 7 with a 4-head GQA group (32 rows per KV head), the whole token-granular chain: logit scores,
    token selection from them, drafting over the selected one-token pages."""
    L = synth.make_random_case(seed=7032, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=8, seq_lens=[2500, 900],
                               logit_std=2.0, value_std=1.0, outliers=3, outlier_logit=30.0)
    G, budget = 8, 256
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=budget, token_granular=True, collect_rows=vb.COLLECT_FIRST_LAST)
    path.iteration(dl)
    torch.cuda.synchronize()
    ref, got = check_token_scores("rows32.chain", L, path, vb.COLLECT_FIRST_LAST)
    sel, ssl = path.sel_table.cpu().numpy(), path.sel_seq_lens.cpu().numpy()
    ref_sel, ref_ssl, _ = O.select_tokens(path.block_scores.cpu().numpy(), L.block_table, L.seq_lens, G, budget,
                                          path.max_sel_blocks)
    assert np.array_equal(sel, ref_sel) and np.array_equal(ssl, ref_ssl)
    kc = L.k_cache.reshape(-1, 1, 8, 128)
    vc = L.v_cache.reshape(-1, 1, 8, 128)
    for s in range(G):
        ref_d = O.draft_attention(L.q_draft[s], kc, vc, sel, ssl, L.softmax_scale)
        U.check_out(f"rows32.chain.draft{s}", path.out_draft[s], ref_d, U.vmax_visible(L))


# ----------------------------------------------------------------------------------------------
# token selection (integer work: bit-exact on identical fp32 scores)
# ----------------------------------------------------------------------------------------------

def gpu_select_tokens(scores32, table, lens, G, budget, max_sel, budgets=None):
    dev = torch.device("cuda:0")
    B, mb = table.shape
    desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=mb, max_sel_blocks=max_sel,
                        max_seq_len=max(int(lens.max()), 1), num_pages=int(table.max()) + 1, softmax_scale=0.1)
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device=dev)
    ws.fill_(0xFF)
    sel = torch.full((B, max_sel), -7, dtype=torch.int32, device=dev)
    ssl = torch.full((B,), -7, dtype=torch.int32, device=dev)
    vb.vegas_select_tokens(desc, torch.from_numpy(scores32).to(dev), torch.from_numpy(table).to(dev),
                           torch.from_numpy(lens).to(dev), budget, sel, ssl, ws,
                           budgets=None if budgets is None else torch.from_numpy(budgets).to(dev))
    torch.cuda.synchronize()
    return sel.cpu().numpy(), ssl.cpu().numpy()


@pytest.mark.parametrize("kind", ["distinct", "ties", "logit_like"])
def test_select_tokens_bit_exact(kind):
    rng = np.random.default_rng({"distinct": 1, "ties": 2, "logit_like": 3}[kind])
    lens = np.array([20000, 4096 + 5, 0, 3, 140001, 4101, 17], dtype=np.int32)
    B = len(lens)
    mb = (int(lens.max()) + PAGE - 1) // PAGE + 3
    scores = np.zeros((B, mb * PAGE), dtype=np.float32)
    for b in range(B):
        n = int(lens[b])
        if kind == "distinct":
            scores[b, :n] = (rng.permutation(n) - n / 3.0).astype(np.float32)
        elif kind == "ties":
            scores[b, :n] = rng.integers(-3, 4, size=n).astype(np.float32) / 4.0
        else:
            x = rng.standard_normal(n).astype(np.float32) * 0.05
            x[rng.integers(0, max(n, 1), size=n // 50)] += 3.0
            scores[b, :n] = x
    scores[:, :] += 0.0
    table = np.stack([rng.permutation(mb + 11)[:mb] for _ in range(B)]).astype(np.int32)
    G = 5
    budgets = np.array([1400, 100000, 64, 1, 9800, 4100, 9], dtype=np.int32)
    max_sel = 10000
    for use_per_seq, budget in ((False, 2048), (True, 2048), (False, 7)):
        print(f"[case] select_tokens {kind} per_seq={use_per_seq} budget={budget}", flush=True)
        bud = budgets if use_per_seq else None
        sel, ssl = gpu_select_tokens(scores, table, lens, G, budget, max_sel, bud)
        ref_sel, ref_ssl, _ = O.select_tokens(scores, table, lens, G, budget, max_sel,
                                              None if bud is None else np.minimum(bud, max_sel))
        assert np.array_equal(ssl, ref_ssl)
        assert np.array_equal(sel, ref_sel)


def test_select_tokens_golden_cases():
    import json, os
    with open(os.path.join(os.path.dirname(__file__), "golden", "select_token_cases.json")) as f:
        cases = json.load(f)["cases"]
    for c in cases:
        n = c["seq_len"]
        nblk = (n + PAGE - 1) // PAGE
        scores = np.zeros((1, nblk * PAGE), dtype=np.float32)
        scores[0, :len(c["scores"])] = c["scores"]
        table = (np.arange(nblk, dtype=np.int32)[::-1] * 3 + 7)[None, :].copy()
        sel, ssl = gpu_select_tokens(scores, table, np.array([n], dtype=np.int32), c["num_queries"], c["budget"], n + 2)
        k = len(c["positions"])
        assert int(ssl[0]) == k, c["name"]
        assert list(sel[0, :k]) == [int(table[0, i // PAGE]) * PAGE + i % PAGE for i in c["positions"]], c["name"]
        assert np.all(sel[0, k:] == -1), c["name"]


# ----------------------------------------------------------------------------------------------
# the whole token-granular chain: verify (token logits) -> select tokens -> draft over one-token pages
# ----------------------------------------------------------------------------------------------

def run_token_chain(L, budget, collect=vb.COLLECT_FIRST_LAST, name="case"):
    s = L.spec
    G = s.num_queries
    dev = torch.device("cuda:0")
    dl, path = verify_token_scores(L, collect)
    ref_scores, got = check_token_scores(name, L, path, collect)
    max_sel = min(max(budget, G), int(L.seq_lens.max())) + 2
    desc_sel = vb.make_desc(batch=s.batch, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=G,
                            max_blocks=L.max_blocks, max_sel_blocks=max_sel, max_seq_len=max(int(L.seq_lens.max()), 1),
                            num_pages=L.num_pages, softmax_scale=L.softmax_scale, head_dim=s.head_dim)
    ws = torch.empty(vb.vegas_workspace_bytes(desc_sel), dtype=torch.uint8, device=dev)
    sel = torch.empty((s.batch, max_sel), dtype=torch.int32, device=dev)
    ssl = torch.empty((s.batch,), dtype=torch.int32, device=dev)
    vb.vegas_select_tokens(desc_sel, path.block_scores, dl.block_table, dl.seq_lens, budget, sel, ssl, ws)
    torch.cuda.synchronize()
    sel_h, ssl_h = sel.cpu().numpy(), ssl.cpu().numpy()
    # (1) on the GPU's own fp32 scores the selection is exactly the oracle's
    sel_same, ssl_same, _ = O.select_tokens(path.block_scores.cpu().numpy(), L.block_table, L.seq_lens, G, budget, max_sel)
    assert np.array_equal(sel_h, sel_same) and np.array_equal(ssl_h, ssl_same)
    # (2) against the selection from the oracle's float64 scores: identical outside the band the score error allows
    _, ref_ssl, ref_pos = O.select_tokens(ref_scores, L.block_table, L.seq_lens, G, budget, max_sel)
    assert np.array_equal(ssl_h, ref_ssl)
    bound = token_score_bound(L, collect)
    exact = 0
    for b in range(s.batch):
        n = int(L.seq_lens[b])
        p_len = max(n - G, 0)
        inv = {int(L.block_table[b, i // PAGE]) * PAGE + i % PAGE: i for i in range(n)}
        got_pos = np.array(sorted(inv[int(x)] for x in sel_h[b, :ssl_h[b]]), dtype=np.int64)
        assert len(set(got_pos)) == len(got_pos) == ssl_h[b]
        assert set(range(p_len, n)).issubset(set(got_pos))
        kc = int(ssl_h[b]) - (n - p_len)
        if 0 < kc < p_len:
            sc = ref_scores[b, :p_len]
            kth = np.sort(sc)[p_len - kc]
            band = 2 * TOKEN_SCORE_REL * float(bound[b, :p_len].max()) + 1e-12
            chosen = got_pos[got_pos < p_len]
            assert np.all(sc[chosen] >= kth - band), name + ": a selected token lies below the k-th score"
            must = np.nonzero(sc > kth + band)[0]
            assert set(must).issubset(set(chosen)), name + ": a token above the k-th score is missing"
        exact += int(np.array_equal(got_pos, ref_pos[b]))
    print(f"[info] {name}: {exact}/{s.batch} sequences select exactly the oracle's token set", flush=True)
    # (3) draft over the GPU's selection, one-token pages
    desc_d = vb.make_desc(batch=s.batch, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                          max_blocks=max_sel, max_sel_blocks=max_sel, max_seq_len=max(int(ssl_h.max()), 1),
                          num_pages=L.num_pages * PAGE, softmax_scale=L.softmax_scale, page_size=1, head_dim=s.head_dim)
    wsd = torch.empty(vb.vegas_workspace_bytes(desc_d), dtype=torch.uint8, device=dev)
    kc1 = L.k_cache.reshape(-1, 1, s.num_kv_heads, s.head_dim)
    vc1 = L.v_cache.reshape(-1, 1, s.num_kv_heads, s.head_dim)
    for step in (0, G - 1):
        out = torch.empty((s.batch, s.num_q_heads, s.head_dim), dtype=torch.bfloat16, device=dev)
        vb.vegas_draft_attention(desc_d, dl.q_draft[step], dl.k_cache, dl.v_cache, sel, ssl, out, wsd)
        torch.cuda.synchronize()
        ref = O.draft_attention(L.q_draft[step], kc1, vc1, sel_h, ssl_h, L.softmax_scale)
        U.check_out(f"{name}.draft{step}", out, ref, U.vmax_visible(L))


def test_token_chain_small_ragged():
    L = synth.make_random_case(seed=611, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[5000, 4, 1300], logit_std=1.5, value_std=1.0, outliers=3, outlier_logit=20.0)
    run_token_chain(L, 400, name="token_chain_ragged")


def test_token_chain_head_dim_64():
    L = synth.make_random_case(seed=612, batch=2, num_q_heads=16, num_kv_heads=4, num_queries=3, head_dim=64,
                               seq_lens=[2100, 37], logit_std=1.5, value_std=1.0, outliers=3, outlier_logit=20.0)
    run_token_chain(L, 257, collect=vb.COLLECT_ALL_ROWS, name="token_chain_hd64")


def test_token_chain_large_batch():
    """200 short sequences (some empty or shorter than the verification rows): the token variant's kernels take
    sequences as a grid dimension too."""
    rng = np.random.default_rng(4242)
    lens = [int(rng.integers(0, 301)) if rng.random() < 0.9 else int(rng.integers(0, 6)) for _ in range(200)]
    lens[0] = 300
    L = synth.make_random_case(seed=613, batch=200, num_q_heads=32, num_kv_heads=8, num_queries=5, seq_lens=lens,
                               logit_std=1.5, value_std=1.0, outliers=1, outlier_logit=20.0)
    run_token_chain(L, 40, name="token_chain_b200")


def random_token_case(i):
    """Shape i of a seeded sweep over KV heads, group sizes, rows, batch, head dimension, lengths, budgets."""
    rng = np.random.default_rng(77000 + i)
    while True:
        Hkv, g = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 8, 16]))
        G = int(rng.integers(1, min(17, 128 // g) + 1))
        if 0 < (G * g) % 32 <= 30:                       # the logit metric needs two spare rows in the last block
            break
    B, D = int(rng.integers(1, 5)), int(rng.choice([128, 64]))
    top = int(rng.choice([40, 300, 2000, 6000]))
    lens = [int(rng.integers(0, top + 1)) if rng.random() < 0.9 else int(rng.integers(0, G + 2)) for _ in range(B)]
    lens[0] = max(lens[0], G + 3)
    collect = int(rng.choice([vb.COLLECT_ALL_ROWS, vb.COLLECT_FIRST_LAST]))
    budget = int(rng.choice([1, 16, 33, 100, 257, 1000, 10 ** 6]))
    return dict(B=B, Hq=Hkv * g, Hkv=Hkv, G=G, D=D, lens=lens, collect=collect, budget=budget)


@pytest.mark.parametrize("i", range(16))
def test_token_chain_random_shapes(i):
    c = random_token_case(i)
    print(f"[case] random token shape {i}: {c}", flush=True)
    L = synth.make_random_case(seed=9000 + i, batch=c["B"], num_q_heads=c["Hq"], num_kv_heads=c["Hkv"],
                               num_queries=c["G"], seq_lens=c["lens"], head_dim=c["D"], logit_std=1.5, value_std=1.0,
                               outliers=3, outlier_logit=20.0)
    run_token_chain(L, c["budget"], collect=c["collect"], name=f"token_random{i}")


def test_token_chain_ctx32k_full():
    """The 32K workload at the paper's operating point: 7 % of the tokens (App. C), Eq. 3 rows."""
    L = synth.make_layer(synth.CONFIGS["ctx32k"])
    run_token_chain(L, int(0.07 * 32768), name="token_chain_ctx32k")


def test_token_chain_ctx128k_full():
    L = synth.make_layer(synth.CONFIGS["ctx128k_drift"])
    run_token_chain(L, int(0.07 * 131072), name="token_chain_ctx128k")


def test_token_variant_clamps_corrupt_lengths_and_page_ids():
    """As for the page variant: a negative length is an empty sequence, a huge length and garbage page ids stay
    inside the caches, the clean neighbour's token selection and draft outputs are what they are without them."""
    L = synth.make_random_case(seed=613, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[1500, 700, 900], logit_std=1.5, outliers=2, outlier_logit=20.0)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=200, token_granular=True, collect_rows=vb.COLLECT_FIRST_LAST)
    lens = dl.seq_lens.clone()
    lens[1] = -5
    lens[2] = 1 << 30
    table = dl.block_table.clone()
    gen = torch.Generator(device="cpu").manual_seed(6)
    table[2] = torch.randint(-(1 << 31), (1 << 31) - 1, (table.shape[1],), generator=gen, dtype=torch.int64).to(torch.int32).to(table.device)
    bad = harness.DeviceLayer(dl.q_verify, dl.q_draft, dl.k_cache, dl.v_cache, table, lens)
    print("[case] token variant, corrupt lengths and page ids", flush=True)
    path.iteration(bad)
    # growth of the selection with the same corrupt lengths: must complete as well
    s = L.spec
    desc_grow = vb.make_desc(batch=s.batch, num_q_heads=s.num_q_heads, num_kv_heads=s.num_kv_heads, num_queries=1,
                             max_blocks=L.max_blocks, max_sel_blocks=path.max_sel_blocks,
                             max_seq_len=min(path.max_sel_blocks, L.max_blocks * PAGE), num_pages=L.num_pages * PAGE,
                             softmax_scale=L.softmax_scale, page_size=1)
    vb.vegas_extend_selection(desc_grow, table, lens, 1, path.sel_table, path.sel_seq_lens)
    torch.cuda.synchronize()
    path.iteration(bad)
    torch.cuda.synchronize()
    G = L.spec.num_queries
    sel, ssl = path.sel_table.cpu().numpy(), path.sel_seq_lens.cpu().numpy()
    # clean sequence: its token selection from the GPU's own scores is the oracle's, and the draft over it matches
    got_scores = path.block_scores.cpu().numpy()
    ref_sel, ref_ssl, _ = O.select_tokens(got_scores[:1], L.block_table[:1], L.seq_lens[:1], G, 200, path.max_sel_blocks)
    assert np.array_equal(sel[:1], ref_sel) and np.array_equal(ssl[:1], ref_ssl)
    kc1 = L.k_cache.reshape(-1, 1, L.spec.num_kv_heads, L.spec.head_dim)
    vc1 = L.v_cache.reshape(-1, 1, L.spec.num_kv_heads, L.spec.head_dim)
    ref_d = O.draft_attention(L.q_draft[0][:1], kc1, vc1, sel[:1], ssl[:1], L.softmax_scale)
    U.check_out("token.corrupt.clean.draft0", path.out_draft[0][:1], ref_d, U.vmax_visible(L))
    assert int(ssl[1]) == 0 and bool((sel[1] == -1).all())
    assert 0 <= int(ssl[2]) <= path.max_sel_blocks
