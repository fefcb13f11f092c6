"""GPU parity of draft attention (Eq. 1 over the selected pages, Sec. 3.2) against the CPU oracle for every GQA
group size: groups of up to 16 heads take the 16-row kernel, larger ones the 32-row streaming kernel; both head
dimensions; page sizes 16, 1, 2 and 8; one chunk (the workgroup writes the rows itself) and many (partials and a merge kernel); selections that
end inside a page, inside a tile and exactly on one; chunks long enough that a wave reloads its page-id batch."""
import numpy as np
import pytest
import torch

from oracle import vegas_oracle as O
from paper_2602_07223_amd import synth
from tests import parity_util as U
from tests.test_gpu_small_pages import draft_small_pages, random_selection

pytestmark = pytest.mark.gpu
PAGE = 16


@pytest.mark.parametrize("P", [16, 1, 2, 8])
@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("g", [1, 2, 3, 4, 5, 7, 8, 12, 16, 32])
def test_every_group_size(g, D, P):
    """Page sizes below 16 list the same cache memory as P-token pages (Sec. 4, App. D): both kernels have an address
    generator for them."""
    Hkv = 2
    lens = [1999, 0, 512, 33, 16, 1]
    L = synth.make_random_case(seed=4400 + g + D, batch=len(lens), num_q_heads=Hkv * g, num_kv_heads=Hkv,
                               num_queries=2, seq_lens=lens, head_dim=D, logit_std=1.5, value_std=1.0, outliers=2,
                               outlier_logit=25.0)
    rng = np.random.default_rng(g)
    sel, ssl = random_selection(L, P, rng, keep_fraction=0.6)
    print(f"[case] draft groups g={g} D={D} P={P} sel_lens={ssl.tolist()}", flush=True)
    kc = L.k_cache.reshape(-1, P, Hkv, D)
    vc = L.v_cache.reshape(-1, P, Hkv, D)
    ref = O.draft_attention(L.q_draft[0], kc, vc, sel, ssl, L.softmax_scale)
    outs = []
    for chunk in (0, 128, 4096):                # the planner's chunks; one tile per wave; one chunk for everything
        out = draft_small_pages(L, P, sel, ssl, step=0, chunk=chunk)
        U.check_out(f"draft.g{g}.D{D}.P{P}.chunk{chunk}", out, ref, U.vmax_visible(L))
        outs.append(out)
    # a sequence without tokens gives rows of zeros on either path
    assert not outs[0][1].view(torch.int16).any() and not outs[2][1].view(torch.int16).any()


@pytest.mark.parametrize("D", [128, 64])
@pytest.mark.parametrize("n", [4096 + 32 * k for k in range(4)] + [4096 + 15, 4096 + 16, 4096 + 17, 4096 + 127])
def test_selection_ends_anywhere_in_a_tile(n, D):
    """The whole context selected, so the selection's length is the sequence's: every position of the end inside
    the last 128-token unit (tile boundaries, page boundaries, one token past and short of them)."""
    L = synth.make_random_case(seed=4700 + n, batch=1, num_q_heads=8, num_kv_heads=2, num_queries=2, seq_lens=[n],
                               head_dim=D, logit_std=1.0, value_std=1.0)
    sel, ssl = random_selection(L, PAGE, np.random.default_rng(1), keep_fraction=1.0)
    assert int(ssl[0]) == n
    print(f"[case] draft end n={n} D={D}", flush=True)
    ref = O.draft_attention(L.q_draft[1], L.k_cache, L.v_cache, sel, ssl, L.softmax_scale)
    for chunk in (0, 8192):                     # 8192: one workgroup, 33 tiles per wave -- the page-id batch is reloaded
        out = draft_small_pages(L, PAGE, sel, ssl, step=1, chunk=chunk)
        U.check_out(f"draft.end{n}.D{D}.chunk{chunk}", out, ref, U.vmax_visible(L))


def test_single_chunk_and_merged_chunks_agree():
    """One workgroup per (sequence, KV head) that finishes the rows itself against chunks and a merge kernel: the
    same sums in another order, so the two bf16 results differ by rounding only."""
    L = synth.make_random_case(seed=4900, batch=3, num_q_heads=32, num_kv_heads=8, num_queries=2,
                               seq_lens=[288, 100, 257], logit_std=1.0, value_std=1.0)
    sel, ssl = random_selection(L, PAGE, np.random.default_rng(5), keep_fraction=1.0)
    a = draft_small_pages(L, PAGE, sel, ssl, chunk=0)          # 288 tokens at most: no merge kernel
    b = draft_small_pages(L, PAGE, sel, ssl, chunk=128)
    ref = O.draft_attention(L.q_draft[0], L.k_cache, L.v_cache, sel, ssl, L.softmax_scale)
    U.check_out("draft.single_chunk", a, ref, U.vmax_visible(L))
    U.check_out("draft.merged_chunks", b, ref, U.vmax_visible(L))
