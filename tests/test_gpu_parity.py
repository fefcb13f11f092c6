"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the
same seeded inputs.  Sizes span several tiles, several chunks and ragged tails."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import binding as vb
from paper_2602_07223_amd import harness, synth
from tests import parity_util as U

pytestmark = pytest.mark.gpu
PAGE = 16


def run_chain(L, budget, collect=vb.COLLECT_ALL_ROWS, verify_chunk=0, draft_chunk=0, name="case", vscale=None,
              log_inputs=False):
    """verify -> select -> G draft steps on the GPU, each stage compared with the oracle.
    log_inputs (the baseline configurations): prints the SHA-256 of the generated inputs and how many sequences'
    selections are exactly the oracle's set."""
    print(f"[case] {name} B={L.spec.batch} Hq={L.spec.num_q_heads} G={L.spec.num_queries} "
          f"lens={list(map(int, L.seq_lens[:8]))} budget={budget} collect={collect}", flush=True)
    if log_inputs:
        print(f"[inputs] {name} seed={L.seed} sha256={U.inputs_sha256(L)}", flush=True)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=budget, collect_rows=collect,
                                       verify_chunk=verify_chunk, draft_chunk=draft_chunk)
    G = L.spec.num_queries
    vs = U.vmax_visible(L) if vscale is None else vscale
    # stage 1: verify
    path.block_scores.fill_(float("nan"))
    path.verify(dl)
    torch.cuda.synchronize()
    ref_out, ref_scores = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens,
                                             L.softmax_scale, collect)
    U.check_out(name + ".verify.out", path.out_verify, ref_out, vs)
    U.check_scores(name + ".scores", path.block_scores, ref_scores)
    # stage 2: select (GPU scores -> GPU selection) vs oracle scores -> oracle selection
    path.select(dl)
    torch.cuda.synchronize()
    sel = path.sel_table.cpu().numpy()
    ssl = path.sel_seq_lens.cpu().numpy()
    _, ref_ssl, ref_logical = O.select_blocks(ref_scores, L.block_table, L.seq_lens, G, budget, path.max_sel_blocks)
    exact = U.check_selection(name + ".select", sel, ssl, L, ref_scores, ref_logical, G, budget)
    if log_inputs:
        print(f"[selection] {name}: exact-set match {exact} of {L.spec.batch} sequences "
              f"(the rest differ only inside the {U.TIE_BAND:g} tie band)", flush=True)
    # select on identical fp32 scores must agree bit for bit
    s32 = ref_scores.astype(np.float32)
    path.select(dl, block_scores=torch.from_numpy(s32).to(path.device))
    torch.cuda.synchronize()
    sel2, ssl2, _ = O.select_blocks(s32, L.block_table, L.seq_lens, G, budget, path.max_sel_blocks)
    assert np.array_equal(path.sel_table.cpu().numpy(), sel2), name + ": select not bit-exact"
    assert np.array_equal(path.sel_seq_lens.cpu().numpy(), ssl2), name + ": sel_seq_lens not bit-exact"
    # stage 3: draft over the GPU's own selection (restored), oracle fed the same page list
    path.select(dl)
    for s in range(G):
        path.draft(dl, s)
    torch.cuda.synchronize()
    for s in range(G):
        ref_d = O.draft_attention(L.q_draft[s], L.k_cache, L.v_cache, sel, ssl, L.softmax_scale)
        U.check_out(f"{name}.draft{s}", path.out_draft[s], ref_d, vs)
    return path, ref_out, ref_scores


SMALL = [
    # name, B, Hq, Hkv, G, lens, kwargs
    ("one_tile", 1, 32, 8, 5, [32], {}),
    ("ragged_tail", 1, 32, 8, 5, [1000], {}),
    ("tiny", 2, 32, 8, 5, [5, 17], {}),
    ("multi_chunk", 1, 32, 8, 5, [5000], dict(verify_chunk=512)),
    ("batch_ragged", 3, 32, 8, 5, [700, 2049, 31], dict(verify_chunk=256)),
    ("gamma6", 1, 32, 8, 7, [3000], {}),
    ("group8", 2, 64, 8, 5, [1500, 640], {}),
    ("group8_chunks", 1, 64, 8, 5, [4100], dict(verify_chunk=1024)),
    ("single_query", 1, 32, 8, 1, [777], {}),
    ("gamma11_g4", 1, 32, 8, 12, [2000], {}),
    ("mha_like", 1, 8, 8, 3, [900], {}),
    ("rows96", 2, 64, 8, 12, [1100, 300], {}),
    ("rows96_big_table", 2, 64, 8, 12, [2000, 77], dict(verify_chunk=128)),   # a big (rows x chunks) table in the score role
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,kw", SMALL, ids=[c[0] for c in SMALL])
@pytest.mark.parametrize("sharp", [False, True], ids=["flat", "sharp"])
def test_small_cases(name, B, Hq, Hkv, G, lens, kw, sharp):
    L = synth.make_random_case(seed=100 + len(name) + 7 * G, batch=B, num_q_heads=Hq, num_kv_heads=Hkv,
                               num_queries=G, seq_lens=lens,
                               logit_std=2.0 if sharp else 0.3, value_std=1.0,
                               outliers=3 if sharp else 0, outlier_logit=30.0)
    budget = max(32, (max(lens) // 10) // PAGE * PAGE)
    run_chain(L, budget, name=name + ("_sharp" if sharp else "_flat"), **kw)


def random_case(i):
    """Shape i of a seeded sweep over KV heads, group sizes, rows (up to 128 per KV head), batch, head dimension,
    lengths (empty, shorter than the verification rows, ragged), chunk lengths, budgets and collect modes."""
    rng = np.random.default_rng(4100 + i)
    Hkv, g = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 8, 16]))
    G = int(rng.integers(1, min(17, 128 // g) + 1))
    B, D = int(rng.integers(1, 6)), int(rng.choice([128, 64]))
    top = int(rng.choice([40, 300, 2000, 6000]))
    lens = [int(rng.integers(0, top + 1)) if rng.random() < 0.9 else int(rng.integers(0, G + 2)) for _ in range(B)]
    if max(lens) == 0:
        lens[0] = G + 3
    return dict(B=B, Hq=Hkv * g, Hkv=Hkv, G=G, D=D, lens=lens,
                collect=int(rng.choice([vb.COLLECT_ALL_ROWS, vb.COLLECT_FIRST_LAST])),
                verify_chunk=int(rng.choice([0, 0, 128, 256, 512, 1024, 2048])),
                draft_chunk=int(rng.choice([0, 0, 64, 128, 512])),
                budget=int(rng.choice([16, 32, 100, 256, 1000, 10 ** 6])), sharp=bool(rng.random() < 0.5))


@pytest.mark.parametrize("i", range(32))
def test_random_shapes(i):
    c = random_case(i)
    print(f"[case] random shape {i}: {c}", flush=True)
    L = synth.make_random_case(seed=5100 + i, batch=c["B"], num_q_heads=c["Hq"], num_kv_heads=c["Hkv"],
                               num_queries=c["G"], seq_lens=c["lens"], head_dim=c["D"],
                               logit_std=2.0 if c["sharp"] else 0.3, value_std=1.0,
                               outliers=3 if c["sharp"] else 0, outlier_logit=30.0)
    run_chain(L, c["budget"], collect=c["collect"], verify_chunk=c["verify_chunk"], draft_chunk=c["draft_chunk"],
              name=f"random{i}")


def random_batch(i):
    """Ragged batch i of a seeded sweep: 2..64 sequences (uniform, random, one long among short ones, some empty),
    no chunk length passed, so verification plans its chunks per sequence on the GPU."""
    rng = np.random.default_rng(31000 + i)
    Hkv, g = int(rng.choice([2, 4, 8])), int(rng.choice([2, 4, 8]))
    G = int(rng.integers(2, min(17, 128 // g) + 1))
    B, D = int(rng.choice([2, 3, 7, 8, 9, 16, 33, 64])), int(rng.choice([128, 64]))
    kind, top = int(rng.integers(0, 4)), int(rng.choice([600, 3000]))
    if kind == 0:
        lens = [int(rng.integers(0, top + 1)) for _ in range(B)]
    elif kind == 1:
        lens = [top] * B
    elif kind == 2:
        lens = [top * 8 if b == 0 else int(rng.integers(0, 60)) for b in range(B)]
    else:
        lens = [int(rng.integers(top // 2, top + 1)) if rng.random() < 0.7 else 0 for _ in range(B)]
    if max(lens) == 0:
        lens[0] = G + 3
    return dict(B=B, Hq=Hkv * g, Hkv=Hkv, G=G, D=D, lens=lens,
                collect=int(rng.choice([vb.COLLECT_ALL_ROWS, vb.COLLECT_FIRST_LAST])),
                budget=int(rng.choice([64, 256, 1000])))


@pytest.mark.parametrize("i", range(12))
def test_random_ragged_batches(i):
    c = random_batch(i)
    print(f"[case] random batch {i}: {c}", flush=True)
    L = synth.make_random_case(seed=12000 + i, batch=c["B"], num_q_heads=c["Hq"], num_kv_heads=c["Hkv"],
                               num_queries=c["G"], seq_lens=c["lens"], head_dim=c["D"], logit_std=1.0, value_std=1.0,
                               outliers=2, outlier_logit=30.0)
    run_chain(L, c["budget"], collect=c["collect"], name=f"random_batch{i}")


LARGE_BATCHES = [
    # name, B, Hq, Hkv, G, D, longest, budget
    ("b300_short", 300, 32, 8, 5, 128, 200, 64),
    ("b1000_tiny_hd64", 1000, 8, 2, 3, 64, 64, 32),
    ("b130_two_row_blocks", 130, 64, 8, 5, 128, 400, 128),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,D,longest,budget", LARGE_BATCHES, ids=[c[0] for c in LARGE_BATCHES])
def test_large_batches_of_short_sequences(name, B, Hq, Hkv, G, D, longest, budget):
    """Batches beyond what the per-sequence chunk plan serves (more than 64 sequences): sequences are a grid
    dimension, most workgroups own a whole short sequence, some sequences are empty or shorter than the rows."""
    rng = np.random.default_rng(77000 + B)
    lens = [int(rng.integers(0, longest + 1)) if rng.random() < 0.9 else int(rng.integers(0, G + 1)) for _ in range(B)]
    lens[0] = longest
    L = synth.make_random_case(seed=8800 + B, batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=G,
                               seq_lens=lens, head_dim=D, logit_std=1.0, value_std=1.0, outliers=1, outlier_logit=20.0)
    run_chain(L, budget, name=name)


@pytest.mark.parametrize("collect", [vb.COLLECT_FIRST_LAST, vb.COLLECT_ALL_ROWS])
def test_collect_modes(collect):
    L = synth.make_random_case(seed=77, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=6,
                               seq_lens=[1234, 4000], logit_std=1.0, outliers=2)
    run_chain(L, 256, collect=collect, name=f"collect{collect}")


def test_many_chunks_take_the_general_merge():
    """More than 64 chunks per row: the merge kernels leave their few-chunk fast paths (verification with
    and without collection, and the draft steps)."""
    L = synth.make_random_case(seed=81, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[9000, 300], logit_std=1.5, outliers=2)
    path, ref_out, _ = run_chain(L, 8800, verify_chunk=128, draft_chunk=128, name="many_chunks")
    dl = harness.DeviceLayer.upload(L)
    plain = harness.VegasPath.for_layer(L, budget_tokens=8800, collect_rows=vb.COLLECT_NONE, verify_chunk=128)
    plain.verify(dl)
    torch.cuda.synchronize()
    U.check_out("many_chunks.collect_none", plain.out_verify, ref_out, U.vmax_visible(L))


def test_collect_none_leaves_scores_untouched_and_out_correct():
    L = synth.make_random_case(seed=78, batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5, seq_lens=[2500])
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=256, collect_rows=vb.COLLECT_NONE)
    path.block_scores.fill_(-7.0)
    path.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale, 0)
    U.check_out("collect_none", path.out_verify, ref_out, U.vmax_visible(L))
    assert bool((path.block_scores == -7.0).all())


def test_baseline_config1_full():
    L = synth.make_layer(synth.CONFIGS["ctx4k"])
    run_chain(L, L.spec.budget_tokens, name="ctx4k", log_inputs=True)


def test_baseline_config2_full():
    L = synth.make_layer(synth.CONFIGS["ctx32k"])
    path, _, ref_scores = run_chain(L, L.spec.budget_tokens, name="ctx32k", log_inputs=True)
    sel = path.sel_table.cpu().numpy()[0]
    inv = {int(p): j for j, p in enumerate(L.block_table[0])}
    ids = {inv[int(p)] for p in sel if p >= 0}
    assert set(np.unique(L.hitters[0] // PAGE)).issubset(ids)        # planted hitters are selected
    assert set(np.unique(L.sinks[0] // PAGE)).issubset(ids)


def test_baseline_config3_full():
    """128K context, gamma = 6, heavy hitters drifting between verify and draft queries."""
    L = synth.make_layer(synth.CONFIGS["ctx128k_drift"])
    path, _, _ = run_chain(L, L.spec.budget_tokens, name="ctx128k_drift", log_inputs=True)
    sel = path.sel_table.cpu().numpy()[0]
    inv = {int(p): j for j, p in enumerate(L.block_table[0])}
    ids = {inv[int(p)] for p in sel if p >= 0}
    assert set(np.unique(L.hitters[0] // PAGE)).issubset(ids)        # what the verify queries saw is kept
    assert ids.__len__() == L.spec.budget_tokens // PAGE


def test_baseline_config4_full():
    """Batch 16, ragged 8K-64K contexts, 64 query heads (40 rows per KV head), shuffled pages,
    NaN poison in spare pages and in the slack of partial last pages."""
    L = synth.make_layer(synth.CONFIGS["ragged16"])
    assert len(set(int(x) % PAGE for x in L.seq_lens)) > 1            # partial last pages occur
    run_chain(L, L.spec.budget_tokens, name="ragged16", log_inputs=True)


def test_ragged_batch_one_row_block_full():
    """The ragged16 lengths with 32 query heads (20 rows per KV head): attn_split_kernel under the two-wave balanced
    plan, chunks of about 10K tokens parked whole in LDS, at the size its launch configuration is meant for."""
    L = synth.make_layer(synth.scaled(synth.CONFIGS["ragged16"], num_q_heads=32))
    run_chain(L, L.spec.budget_tokens, collect=vb.COLLECT_FIRST_LAST, name="ragged16_32heads")


@pytest.mark.parametrize("layer", range(32))
def test_baseline_config5_every_layer(layer):
    """The 32-layer stack is 32 independent single-layer calls (own seed each); every layer is checked in full,
    one at a time (generate, upload, run, oracle, compare, drop)."""
    L = synth.make_layer(synth.CONFIGS["stack32"], layer=layer)
    run_chain(L, L.spec.budget_tokens, name=f"stack32.layer{layer}", log_inputs=True)


def test_long_chunk_reloads_the_page_id_batch():
    """A chunk of 8192 tokens gives every wave 64 tiles: the 32-tile page-id batch is reloaded mid-stream."""
    L = synth.make_random_case(seed=83, batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[9000 + 7], logit_std=1.0, outliers=2)
    run_chain(L, 512, verify_chunk=8192, draft_chunk=8192, name="chunk8192")


def test_strided_cache_views():
    """The cache strides come from the descriptor: a cache that is a view into a larger allocation
    (padded token rows, an unused extra KV head) must give the same results as the packed one."""
    L = synth.make_random_case(seed=84, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[1500, 700], logit_std=1.0)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=256)
    path.iteration(dl)
    torch.cuda.synchronize()
    want = (path.out_verify.clone(), path.block_scores.clone(), path.sel_table.clone(), path.out_draft.clone())
    P, Hkv, D = L.num_pages, 8, 128
    big_k = torch.full((P, PAGE, Hkv + 1, D + 64), float("nan"), dtype=torch.bfloat16, device=path.device)
    big_v = torch.full_like(big_k, float("nan"))
    big_k[:, :, :Hkv, :D] = dl.k_cache
    big_v[:, :, :Hkv, :D] = dl.v_cache
    kview, vview = big_k[:, :, :Hkv, :D], big_v[:, :, :Hkv, :D]
    for desc in (path.desc_verify, path.desc_draft):
        desc.kv_page_stride, desc.kv_token_stride, desc.kv_head_stride = kview.stride(0), kview.stride(1), kview.stride(2)
    dl2 = harness.DeviceLayer(dl.q_verify, dl.q_draft, kview, vview, dl.block_table, dl.seq_lens)
    path.iteration(dl2)
    torch.cuda.synchronize()
    got = (path.out_verify, path.block_scores, path.sel_table, path.out_draft)
    for a, b in zip(want, got):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b)


def test_empty_and_short_sequences():
    L = synth.make_random_case(seed=79, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[0, 3, 40], spare_pages=2)
    run_chain(L, 32, name="degenerate")


def test_budget_covers_context_draft_equals_last_verify_row():
    """Cross-kernel identity: with every page selected, a draft query equal to the bonus row's query
    reproduces that verify row."""
    L = synth.make_random_case(seed=80, batch=2, num_q_heads=32, num_kv_heads=8, num_queries=4,
                               seq_lens=[1500, 333], logit_std=1.0)
    L.q_draft[0] = L.q_verify[:, -1]
    path, ref_out, _ = run_chain(L, 10 ** 6, name="full_budget")
    a = harness.bf16_to_host_f64(path.out_draft[0])
    b = harness.bf16_to_host_f64(path.out_verify[:, -1])
    assert np.abs(a - b).max() <= 2 * max(U.OUT_ATOL, U.vmax_visible(L) / 256.0)
    assert np.array_equal(path.sel_seq_lens.cpu().numpy(), L.seq_lens)


def test_results_do_not_depend_on_physical_page_ids():
    L = synth.make_random_case(seed=81, batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[3000], shuffle=False, spare_pages=0, poison=False)
    rng = np.random.default_rng(2)
    P = L.k_cache.shape[0]
    perm = rng.permutation(P)
    import copy
    L2 = copy.copy(L)
    L2.k_cache = np.empty_like(L.k_cache); L2.v_cache = np.empty_like(L.v_cache)
    L2.k_cache[perm] = L.k_cache; L2.v_cache[perm] = L.v_cache
    L2.block_table = np.where(L.block_table >= 0, perm[np.clip(L.block_table, 0, None)], -1).astype(np.int32)
    outs = []
    for X in (L, L2):
        dl = harness.DeviceLayer.upload(X)
        path = harness.VegasPath.for_layer(X, budget_tokens=320)
        path.iteration(dl)
        torch.cuda.synchronize()
        outs.append((path.out_verify.view(torch.int16).cpu().numpy().copy(), path.block_scores.cpu().numpy().copy(),
                     path.sel_table.cpu().numpy().copy(), path.out_draft.view(torch.int16).cpu().numpy().copy()))
    assert np.array_equal(outs[0][0], outs[1][0]) and np.array_equal(outs[0][1], outs[1][1])
    assert np.array_equal(outs[0][3], outs[1][3])
    assert np.array_equal(np.where(outs[0][2] >= 0, perm[np.clip(outs[0][2], 0, None)], -1), outs[1][2])


def test_run_to_run_bit_reproducible():
    L = synth.make_layer(synth.scaled(synth.CONFIGS["ctx4k"], seq_len=2048 + 9))
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L)
    snaps = []
    for _ in range(3):
        path.iteration(dl)
        torch.cuda.synchronize()
        snaps.append((path.out_verify.view(torch.int16).cpu().numpy().copy(), path.block_scores.cpu().numpy().copy(),
                      path.sel_table.cpu().numpy().copy(), path.out_draft.view(torch.int16).cpu().numpy().copy()))
    for s in snaps[1:]:
        for a, b in zip(snaps[0], s):
            assert np.array_equal(a, b)


def test_hip_graph_replays_match_eager():
    """The three calls only enqueue kernels on the caller's stream, so a whole iteration can be captured
    into a HIP graph.  Every replay (with eager work and synchronisations in between, outputs wiped before
    each) must reproduce the eager results bit for bit."""
    L = synth.make_layer(synth.scaled(synth.CONFIGS["ctx4k"], seq_len=3072 + 5))
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L)

    def snap():
        torch.cuda.synchronize()
        return (path.out_verify.view(torch.int16).cpu().numpy().copy(), path.block_scores.cpu().numpy().copy(),
                path.sel_table.cpu().numpy().copy(), path.sel_seq_lens.cpu().numpy().copy(),
                path.out_draft.view(torch.int16).cpu().numpy().copy())

    def wipe():
        path.out_verify.fill_(float("nan"))
        path.block_scores.fill_(float("nan"))
        path.sel_table.fill_(-7)
        path.sel_seq_lens.fill_(-7)
        path.out_draft.fill_(float("nan"))
        path.workspace.fill_(0xFF)

    path.iteration(dl)
    eager = snap()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path.iteration(dl)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        path.iteration(dl)
    for replay in range(4):
        wipe()
        torch.cuda.synchronize()
        graph.replay()
        got = snap()
        for a, b in zip(eager, got):
            assert np.array_equal(a, b), f"replay {replay} differs from the eager run"
        wipe()
        path.iteration(dl)                      # eager work between replays
        for a, b in zip(eager, snap()):
            assert np.array_equal(a, b)


def test_select_bit_exact_with_ties_and_budgets():
    """Integer work: many exact ties, per-sequence budgets, budgets below the forced pages and above the context."""
    rng = np.random.default_rng(5)
    B, mb = 6, 700
    lens = np.array([11200, 5000, 16, 777, 0, 9000], dtype=np.int32)
    nblk = (lens + PAGE - 1) // PAGE
    scores = np.zeros((B, mb), dtype=np.float32)
    for b in range(B):
        scores[b, :nblk[b]] = rng.integers(0, 6, size=nblk[b]).astype(np.float32) / 8.0    # heavy ties
    table = np.stack([rng.permutation(4000)[:mb] for _ in range(B)]).astype(np.int32)
    budgets = np.array([2048, 1, 64, 100000, 32, 4800], dtype=np.int32)
    G = 5
    desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=mb, max_sel_blocks=mb,
                        max_seq_len=mb * PAGE, num_pages=4000, softmax_scale=0.1)
    dev = torch.device("cuda:0")
    sel = torch.empty((B, mb), dtype=torch.int32, device=dev)
    ssl = torch.empty((B,), dtype=torch.int32, device=dev)
    for use_per_seq in (True, False):
        vb.vegas_select_blocks(desc, torch.from_numpy(scores).to(dev), torch.from_numpy(table).to(dev),
                               torch.from_numpy(lens).to(dev), 640, sel, ssl,
                               budgets=torch.from_numpy(budgets).to(dev) if use_per_seq else None)
        torch.cuda.synchronize()
        ref_sel, ref_ssl, _ = O.select_blocks(scores, table, lens, G, 640, mb, budgets if use_per_seq else None)
        assert np.array_equal(sel.cpu().numpy(), ref_sel)
        assert np.array_equal(ssl.cpu().numpy(), ref_ssl)


SCORE_KINDS = ["uniform", "all_equal", "four_values", "signed", "clustered_1_percent", "denormal", "zeros_and_inf",
               "with_nan"]


@pytest.mark.parametrize("pages", [65, 2048, 8193])
@pytest.mark.parametrize("kind", SCORE_KINDS)
def test_select_is_bit_exact_on_any_score_distribution(kind, pages):
    """Selection is integer work on the score bits: whatever the scores look like -- ties everywhere, negative
    values, scores that agree to a percent (the top two key bytes collide), denormals, zeros and infinities --
    the result on identical fp32 scores is the oracle's, bit for bit, with and without per-sequence budgets."""
    rng = np.random.default_rng(9100 + pages + len(kind))
    B, G = 3, 5
    lens = np.array([pages * PAGE - 2, (pages // 2) * PAGE + 9, 7], dtype=np.int32)
    scores = np.zeros((B, pages), dtype=np.float32)
    for b in range(B):
        if kind == "uniform":
            x = rng.random(pages)
        elif kind == "all_equal":
            x = np.full(pages, 0.25)
        elif kind == "four_values":
            x = rng.integers(0, 4, pages) * 0.125
        elif kind == "signed":
            x = rng.standard_normal(pages)
        elif kind == "clustered_1_percent":
            x = (1.0 + rng.random(pages) * 0.01) / pages
        elif kind == "denormal":
            x = rng.random(pages) * 1e-42
        elif kind == "with_nan":                          # NaN of either sign ranks below every number, -inf included
            x = rng.standard_normal(pages).astype(np.float32)
            x[rng.integers(0, pages, size=pages // 3)] = np.float32(np.nan)
            neg = rng.integers(0, pages, size=pages // 8)
            x[neg] = np.frombuffer(np.uint32(0xFFC00001).tobytes(), dtype=np.float32)[0]
            x[rng.integers(0, pages, size=4)] = -np.inf
        else:
            x = rng.random(pages) ** 8
            x[rng.integers(0, pages, size=pages // 4)] = 0.0
            x[rng.integers(0, pages, size=3)] = np.inf
        scores[b] = x.astype(np.float32)
    table = np.stack([rng.permutation(pages + 7)[:pages] for _ in range(B)]).astype(np.int32)
    dev = torch.device("cuda:0")
    for budget, budgets in ((pages, None), (100, np.array([pages * 3, 1, 100], dtype=np.int32))):
        kmax = (int(budgets.max()) if budgets is not None else budget) // PAGE + 1
        msb = min(kmax, pages) + 2
        desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=pages,
                            max_sel_blocks=msb, max_seq_len=pages * PAGE, num_pages=pages + 7, softmax_scale=0.1)
        sel = torch.empty((B, msb), dtype=torch.int32, device=dev)
        ssl = torch.empty((B,), dtype=torch.int32, device=dev)
        print(f"[case] select {kind} pages={pages} budget={budget} per_sequence={budgets is not None}", flush=True)
        vb.vegas_select_blocks(desc, torch.from_numpy(scores).to(dev), torch.from_numpy(table).to(dev),
                               torch.from_numpy(lens).to(dev), budget, sel, ssl,
                               budgets=None if budgets is None else torch.from_numpy(budgets).to(dev))
        torch.cuda.synchronize()
        ref_sel, ref_ssl, _ = O.select_blocks(scores, table, lens, G, budget, msb, budgets=budgets)
        assert np.array_equal(sel.cpu().numpy(), ref_sel)
        assert np.array_equal(ssl.cpu().numpy(), ref_ssl)


@pytest.mark.parametrize("pages", [9000, 16384, 20011, 65537])
def test_select_long_sequences(pages):
    """Page counts above what the other cases reach: keys that fill the kernel's LDS budget and, past it,
    the path that re-reads the scores; scores drawn like attention mass (a few large, most tiny, ties)."""
    rng = np.random.default_rng(pages)
    B, G = 2, 5
    lens = np.array([pages * PAGE - 3, (pages // 2) * PAGE + 1], dtype=np.int32)
    nblk = (lens + PAGE - 1) // PAGE
    scores = np.zeros((B, pages), dtype=np.float32)
    for b in range(B):
        x = rng.random(nblk[b]).astype(np.float32) ** 8
        x[rng.integers(0, nblk[b], size=nblk[b] // 4)] = np.float32(2.0 ** -14)        # many exact ties
        scores[b, :nblk[b]] = x / x.sum()
    table = np.stack([rng.permutation(pages + 50)[:pages] for _ in range(B)]).astype(np.int32)
    budget = 4096
    msb = budget // PAGE + 2
    desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=pages, max_sel_blocks=msb,
                        max_seq_len=pages * PAGE, num_pages=pages + 50, softmax_scale=0.1)
    dev = torch.device("cuda:0")
    sel = torch.empty((B, msb), dtype=torch.int32, device=dev)
    ssl = torch.empty((B,), dtype=torch.int32, device=dev)
    print(f"[case] select_long pages={pages}", flush=True)
    vb.vegas_select_blocks(desc, torch.from_numpy(scores).to(dev), torch.from_numpy(table).to(dev),
                           torch.from_numpy(lens).to(dev), budget, sel, ssl)
    torch.cuda.synchronize()
    ref_sel, ref_ssl, _ = O.select_blocks(scores, table, lens, G, budget, msb)
    assert np.array_equal(sel.cpu().numpy(), ref_sel)
    assert np.array_equal(ssl.cpu().numpy(), ref_ssl)


WINDOW_CASES = [
    # name, B, Hq, Hkv, G, lens, window, verify_chunk
    ("w128_multi_chunk", 1, 32, 8, 5, [5000], 128, 0),
    ("w100_ragged", 3, 32, 8, 5, [700, 2049, 3], 100, 256),
    ("w_wider_than_context", 1, 32, 8, 5, [900], 4096, 0),
    ("w1", 1, 32, 8, 3, [333], 1, 0),
    ("w128_group8_many_chunks", 2, 64, 8, 5, [9000, 130], 128, 128),
    ("w37_single_row", 1, 32, 8, 1, [2100], 37, 0),
]


@pytest.mark.parametrize("name,B,Hq,Hkv,G,lens,window,chunk", WINDOW_CASES, ids=[c[0] for c in WINDOW_CASES])
def test_verify_with_local_masking(name, B, Hq, Hkv, G, lens, window, chunk):
    """Banded layers (Sec. 4 names a local mask beside the causal one): the row at position pos sees
    keys pos - window + 1 .. pos; chunks and tiles before the band are skipped, so their stale partials
    (poisoned here) must never be read."""
    L = synth.make_random_case(seed=700 + len(name), batch=B, num_q_heads=Hq, num_kv_heads=Hkv, num_queries=G,
                               seq_lens=lens, logit_std=1.5, value_std=1.0, outliers=2, outlier_logit=20.0)
    print(f"[case] window {name} W={window}", flush=True)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=64, collect_rows=vb.COLLECT_NONE, verify_chunk=chunk,
                                       window=window)
    path.workspace.fill_(0xFF)                                    # NaN bit patterns in every partial
    path.out_verify.fill_(float("nan"))
    path.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale,
                                    0, window=window)
    U.check_out(name, path.out_verify, ref_out, U.vmax_visible(L))


def random_window_case(i):
    rng = np.random.default_rng(52000 + i)
    Hkv, g = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 8, 16]))
    G = int(rng.integers(1, min(17, 128 // g) + 1))
    B, D = int(rng.integers(1, 5)), int(rng.choice([128, 64]))
    top = int(rng.choice([40, 300, 2000, 9000]))
    lens = [int(rng.integers(0, top + 1)) for _ in range(B)]
    if max(lens) == 0:
        lens[0] = G + 3
    return dict(B=B, Hq=Hkv * g, Hkv=Hkv, G=G, D=D, lens=lens,
                window=int(rng.choice([1, 2, 16, 17, 37, 100, 128, 1000, 5000, 20000])),
                chunk=int(rng.choice([0, 0, 64, 128, 512, 2048])))


@pytest.mark.parametrize("i", range(16))
def test_local_masking_random_shapes(i):
    c = random_window_case(i)
    print(f"[case] random window shape {i}: {c}", flush=True)
    L = synth.make_random_case(seed=15000 + i, batch=c["B"], num_q_heads=c["Hq"], num_kv_heads=c["Hkv"],
                               num_queries=c["G"], seq_lens=c["lens"], head_dim=c["D"], logit_std=1.5, value_std=1.0,
                               outliers=2, outlier_logit=20.0)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=64, collect_rows=vb.COLLECT_NONE, verify_chunk=c["chunk"],
                                       window=c["window"])
    path.workspace.fill_(0xFF)
    path.out_verify.fill_(float("nan"))
    path.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale,
                                    0, window=c["window"])
    U.check_out(f"window_random{i}", path.out_verify, ref_out, U.vmax_visible(L))


def test_local_masking_refuses_score_collection():
    desc = vb.make_desc(batch=1, num_q_heads=32, num_kv_heads=8, num_queries=5, max_blocks=64, max_sel_blocks=64,
                        max_seq_len=1024, num_pages=64, softmax_scale=0.1, window=128)
    z = torch.zeros(1 << 19, dtype=torch.int32, device="cuda:0")
    ws = torch.empty(vb.vegas_workspace_bytes(desc), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(vb.VegasError) as e:
        vb.vegas_verify_attention(desc, z, z, z, z, z, z, z.view(torch.float32), ws)
    assert e.value.status == vb.VEGAS_ERR_UNSUPPORTED


# 33..64 rows per KV head: one workgroup serves both 32-row blocks from one read of K/V.  The chunk sizes make
# every pair run 1, 2, 3, 4, 5 and many steps (the stream's tail is peeled by hand), with odd and even tile
# counts in the last chunk; a chunk of 96 tokens holds an odd number of tiles and takes the sibling-workgroup path.
PAIR_CASES = [
    # name, Hq, Hkv, G, lens
    ("rows40", 64, 8, 5, [1000, 2049 + 32, 31]),
    ("rows33", 33, 1, 1, [777, 64]),
    ("rows64", 64, 8, 8, [1500, 640 + 17]),
    ("rows48_g16", 32, 2, 3, [905]),
]


@pytest.mark.parametrize("chunk", [64, 128, 192, 256, 320, 96, 0])
@pytest.mark.parametrize("name,Hq,Hkv,G,lens", PAIR_CASES, ids=[c[0] for c in PAIR_CASES])
def test_two_row_blocks_from_one_read(name, Hq, Hkv, G, lens, chunk):
    L = synth.make_random_case(seed=1200 + len(name) + chunk, batch=len(lens), num_q_heads=Hq, num_kv_heads=Hkv,
                               num_queries=G, seq_lens=lens, logit_std=2.0, value_std=1.0, outliers=3,
                               outlier_logit=30.0)
    collect = vb.COLLECT_FIRST_LAST if chunk in (128, 320) else vb.COLLECT_ALL_ROWS
    run_chain(L, 128, collect=collect, verify_chunk=chunk, name=f"pair.{name}.chunk{chunk}")
    dl = harness.DeviceLayer.upload(L)
    plain = harness.VegasPath.for_layer(L, budget_tokens=128, collect_rows=vb.COLLECT_NONE, verify_chunk=chunk)
    plain.workspace.fill_(0xFF)
    plain.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale, 0)
    U.check_out(f"pair.{name}.chunk{chunk}.collect_none", plain.out_verify, ref_out, U.vmax_visible(L))


@pytest.mark.parametrize("chunk,lens", [(4096, [9000, 4100]), (8192, [8192 + 77]), (2176, [6000])],
                         ids=["chunk4096", "chunk8192", "chunk2176"])
def test_long_chunks_flush_collected_values_in_rings(chunk, lens):
    """Chunks longer than the LDS ring that parks the page log-sum-exps: the ring is written out whenever it is
    full (every 2048 tokens) and once more at the end of the chunk."""
    L = synth.make_random_case(seed=1300 + chunk, batch=len(lens), num_q_heads=64, num_kv_heads=8, num_queries=5,
                               seq_lens=lens, logit_std=2.0, value_std=1.0, outliers=3, outlier_logit=30.0)
    run_chain(L, 512, verify_chunk=chunk, name=f"pair.ring.chunk{chunk}")


BALANCED_CASES = [
    # name, G, lens  (64 query / 8 KV heads: 8 G rows per KV head; no chunk length given, so the GPU plans the chunks)
    ("empty_and_tiny_members", 5, [3000, 0, 17, 900]),
    ("one_long_many_short", 5, [20000, 33, 5, 64, 2]),
    ("all_empty_but_one", 6, [0, 0, 4097, 0]),
    ("all_empty", 5, [0, 0]),
    ("sixty_four_sequences", 5, [1 + (37 * i * i + 11 * i) % 700 for i in range(64)]),
    ("equal_lengths", 8, [4096, 4096, 4096]),
]


@pytest.mark.parametrize("Hq", [64, 32, 96], ids=["two_row_blocks", "one_row_block", "three_row_blocks"])
@pytest.mark.parametrize("name,G,lens", BALANCED_CASES, ids=[c[0] for c in BALANCED_CASES])
def test_balanced_chunking_of_ragged_batches(name, G, lens, Hq):
    """Several sequences and no chunk length from the caller: the kernels give a fixed number of workgroups to the
    sequences by length (every workgroup computes the same plan from seq_lens), in every streaming kernel:
    attn_pair_kernel (two row blocks), attn_split_kernel (one) and its sibling workgroups (three)."""
    L = synth.make_random_case(seed=1400 + len(name) + Hq, batch=len(lens), num_q_heads=Hq, num_kv_heads=8, num_queries=G,
                               seq_lens=lens, logit_std=2.0, value_std=1.0, outliers=2, outlier_logit=25.0)
    run_chain(L, 256, name=f"balanced.{name}.Hq{Hq}")
    dl = harness.DeviceLayer.upload(L)
    plain = harness.VegasPath.for_layer(L, budget_tokens=256, collect_rows=vb.COLLECT_NONE)
    plain.workspace.fill_(0xFF)
    plain.verify(dl)
    torch.cuda.synchronize()
    ref_out, _ = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens, L.softmax_scale, 0)
    U.check_out(f"balanced.{name}.collect_none", plain.out_verify, ref_out, U.vmax_visible(L))


@pytest.mark.parametrize("Hq", [32, 64], ids=["one_row_block", "two_row_blocks"])
def test_loose_max_seq_len_does_not_change_results(Hq):
    """A serving engine passes its model limit as max_seq_len, far above what the batch holds: the chunk plan comes
    from seq_lens on the GPU, and the results are those of a tight bound."""
    lens = [3000, 900, 17]
    L = synth.make_random_case(seed=1500 + Hq, batch=3, num_q_heads=Hq, num_kv_heads=8, num_queries=5, seq_lens=lens,
                               logit_std=2.0, value_std=1.0, outliers=2, outlier_logit=25.0, max_blocks=4096)
    print(f"[case] loose_max_seq_len Hq={Hq}", flush=True)
    s = L.spec
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath(batch=3, num_q_heads=Hq, num_kv_heads=8, num_queries=5, max_blocks=4096,
                             max_seq_len=65536, num_pages=L.num_pages, budget_tokens=256,
                             softmax_scale=L.softmax_scale)
    path.block_scores.fill_(float("nan"))
    path.workspace.fill_(0xFF)
    path.iteration(dl)
    torch.cuda.synchronize()
    ref_out, ref_scores = O.verify_attention(L.q_verify, L.k_cache, L.v_cache, L.block_table, L.seq_lens,
                                             L.softmax_scale, vb.COLLECT_ALL_ROWS)
    vs = U.vmax_visible(L)
    U.check_out("loose.verify.out", path.out_verify, ref_out, vs)
    U.check_scores("loose.scores", path.block_scores, ref_scores)
    sel = path.sel_table.cpu().numpy()
    ssl = path.sel_seq_lens.cpu().numpy()
    _, _, ref_logical = O.select_blocks(ref_scores, L.block_table, L.seq_lens, 5, 256, path.max_sel_blocks)
    U.check_selection("loose.select", sel, ssl, L, ref_scores, ref_logical, 5, 256)
    for step in range(5):
        ref_d = O.draft_attention(L.q_draft[step], L.k_cache, L.v_cache, sel, ssl, L.softmax_scale)
        U.check_out(f"loose.draft{step}", path.out_draft[step], ref_d, vs)


def test_corrupt_lengths_and_page_ids_are_clamped():
    """The kernels clamp lengths into [0, max_seq_len] and page ids into [0, num_pages): a negative length
    behaves as an empty sequence, a huge length and a table of garbage ids give unspecified results for
    that sequence but touch nothing outside the caches, and a clean neighbour is unaffected."""
    L = synth.make_random_case(seed=91, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=5,
                               seq_lens=[1500, 700, 900], logit_std=1.0, outliers=2)
    dl = harness.DeviceLayer.upload(L)
    path = harness.VegasPath.for_layer(L, budget_tokens=256)
    lens = dl.seq_lens.clone()
    lens[1] = -5
    lens[2] = 1 << 30
    table = dl.block_table.clone()
    gen = torch.Generator(device="cpu").manual_seed(5)
    table[2] = torch.randint(-(1 << 31), (1 << 31) - 1, (table.shape[1],), generator=gen, dtype=torch.int64).to(torch.int32).to(table.device)
    bad = harness.DeviceLayer(dl.q_verify, dl.q_draft, dl.k_cache, dl.v_cache, table, lens)
    print("[case] corrupt lengths and page ids", flush=True)
    path.out_verify.fill_(float("nan"))
    path.iteration(bad)
    torch.cuda.synchronize()
    G = L.spec.num_queries
    # the clean sequence: against the oracle run on it alone
    ref_out, ref_scores = O.verify_attention(L.q_verify[:1], L.k_cache, L.v_cache, L.block_table[:1], L.seq_lens[:1],
                                             L.softmax_scale, vb.COLLECT_ALL_ROWS)
    vs = U.vmax_visible(L)
    U.check_out("corrupt.clean.verify", path.out_verify[:1], ref_out, vs)
    U.check_scores("corrupt.clean.scores", path.block_scores[:1], ref_scores)
    sel = path.sel_table.cpu().numpy()
    ssl = path.sel_seq_lens.cpu().numpy()
    for s in range(G):
        ref_d = O.draft_attention(L.q_draft[s][:1], L.k_cache, L.v_cache, sel[:1], ssl[:1], L.softmax_scale)
        U.check_out(f"corrupt.clean.draft{s}", path.out_draft[s][:1], ref_d, vs)
    # the sequence with a negative length is an empty one
    assert bool((path.out_verify[1].view(torch.int16) == 0).all())
    assert int(ssl[1]) == 0 and bool((sel[1] == -1).all())
    assert bool((path.block_scores[1] == 0).all())
    # the sequence with the huge length was cut at max_seq_len: its selection is within the row and padded
    assert 0 <= int(ssl[2]) <= path.desc_draft.max_seq_len
