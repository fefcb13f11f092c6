"""The debugging aid for data-dependent input errors (vegas_debug_check_tables): lengths and page ids that the calls
would clamp silently are reported as bits of a device word.  Expected bits are worked out here from the rule."""
import numpy as np
import pytest
import torch

from paper_2602_07223_amd import binding as vb

pytestmark = pytest.mark.gpu
PAGE = 16


def expected_bits(table, lens, stride, page_size, max_seq_len, num_pages, num_queries):
    bits = 0
    for b, n in enumerate(lens):
        n = int(n)
        if n < 0 or n > max_seq_len:
            bits |= vb.CHECK_LENGTH_RANGE
        if n > stride * page_size:
            bits |= vb.CHECK_LENGTH_EXCEEDS_TABLE
        if num_queries > 0 and 0 < n < num_queries:
            bits |= vb.CHECK_SHORTER_THAN_QUERIES
        nn = min(max(n, 0), stride * page_size)
        used = table[b, :(nn + page_size - 1) // page_size]
        if ((used < 0) | (used >= num_pages)).any():
            bits |= vb.CHECK_PAGE_ID
    return bits


CASES = [
    # name, lens, corrupt (b, j, value) entries
    ("clean", [100, 160, 0, 37], []),
    ("negative_length", [100, -3, 50, 37], []),
    ("length_above_bound", [100, 161, 50, 37], []),
    ("length_above_table", [100, 1000, 50, 37], []),
    ("page_id_negative", [100, 160, 50, 37], [(1, 9, -1)]),
    ("page_id_past_pool", [100, 160, 50, 37], [(0, 0, 64)]),
    ("bad_id_in_unused_entry_is_fine", [100, 32, 50, 37], [(1, 2, 999)]),
    ("shorter_than_queries", [100, 3, 50, 37], []),
    ("several_at_once", [-1, 3, 5000, 37], [(3, 1, -7)]),
]


@pytest.mark.parametrize("name,lens,corrupt", CASES, ids=[c[0] for c in CASES])
@pytest.mark.parametrize("which", [vb.TABLE_BLOCKS, vb.TABLE_SELECTION], ids=["block_table", "selection"])
def test_check_tables_reports_what_the_rule_says(name, lens, corrupt, which):
    rng = np.random.default_rng(len(name))
    B, stride, num_pages, G = 4, 10, 64, 5
    page_size = PAGE if which == vb.TABLE_BLOCKS else 4
    table = rng.integers(0, num_pages, size=(B, stride)).astype(np.int32)
    for b, j, v in corrupt:
        table[b, j] = v
    lens = np.array(lens, dtype=np.int32)
    max_seq_len = stride * page_size
    desc = vb.make_desc(batch=B, num_q_heads=32, num_kv_heads=8, num_queries=G, max_blocks=stride, max_sel_blocks=stride,
                        max_seq_len=max_seq_len, num_pages=num_pages, softmax_scale=0.1, page_size=page_size)
    dev = torch.device("cuda:0")
    word = torch.zeros(1, dtype=torch.int32, device=dev)
    vb.vegas_debug_check_tables(desc, which, torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev), word)
    torch.cuda.synchronize()
    want = expected_bits(table, lens, stride, page_size, max_seq_len, num_pages, G if which == vb.TABLE_BLOCKS else 0)
    assert int(word.item()) == want, (name, int(word.item()), want)
    # bits accumulate: a clean second check leaves the word as it is
    clean = rng.integers(0, num_pages, size=(B, stride)).astype(np.int32)
    vb.vegas_debug_check_tables(desc, which, torch.from_numpy(clean).to(dev),
                                torch.full((B,), 40, dtype=torch.int32, device=dev), word)
    torch.cuda.synchronize()
    assert int(word.item()) == want
