"""CPU oracle for the verify -> select -> draft path of Vegas.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file; the
product path (the HIP library and its binding) never does, and this file imports nothing
from the product.  It is a plain float64 NumPy implementation of the *definitions*:

  * attention                         -- Eq. 1 (Sec. 2.1), softmax(q K^T / sqrt(d)) V
  * verification of gamma+1 tokens in one full-attention pass over the whole cache
                                      -- Sec. 2.3; masked as in Sec. 4 (criticality is taken
                                         after the causal or local mask)
  * criticality of prefix entries     -- Eq. 2 (all gamma+1 rows, all query heads) and Eq. 3
                                         (first draft row + bonus row), Sec. 3.2-3.3, with the
                                         attention *weights* as the metric (App. B) and the
                                         row/head averaging of Sec. 3.3's last paragraph
  * top-k selection                   -- the argmax of Eq. 2 / Eq. 3, here over unions of
                                         16-token KV pages; what follows the prefix stays
                                         (Sec. 3.2, last sentence): the forced tail pages
  * the paper's own selection variant -- logits as the metric (Sec. 3.2 footnote, App. B), single
                                         tokens as the unit (Sec. 4): token_logit_scores,
                                         select_tokens; drafting over them is draft_attention on
                                         the cache seen with one-token pages
  * sparse drafting                   -- Sec. 2.2 (attention over the selected entries only),
                                         realised as paged attention over the selected page
                                         list (Sec. 4, App. D)

No tiling, no online softmax, no reordering: gather the sequence's keys and values through
the page table, form the logit matrix with one matmul, mask, softmax, one more matmul.

Readings taken where the paper is silent (each is also listed in the design notes):
  * the gamma+1 verify tokens' own K/V are the last gamma+1 entries of the cache, seq_lens
    counts them, and row t (0-based) sees keys 0 .. n-G+t (bottom-right aligned causal mask);
  * a page's score is the SUM of its member tokens' weights (this makes top-k of page scores
    the exact argmax of Eq. 2 restricted to unions of pages), then the MEAN over the collected
    rows and over all query heads (so the scores of one sequence add up to 1);
  * the pages that overlap the last gamma+1 token positions are always selected and count
    towards the budget; k = min(ceil(budget/16), number of pages), raised to the number of
    forced pages if smaller; ties go to the lower logical page index;
  * a row with no visible key (only possible when seq_len < gamma+1) outputs 0 and
    contributes no weight.

Pins (tests/test_oracle_pins.py): token logit scores against scalar loops, the closed form
k_i . mean(q) and the single-head ranking identity of App. B; token selection against exhaustive
subset search for Eq. 3, numpy partition and hand-worked cases; draft attention over 1/2/4/8-token pages against library attention
over the listed tokens, closed forms for uniform weights, one-hot dominance, the
library routines torch.nn.functional.scaled_dot_product_attention and scipy.special
(softmax, logsumexp) on special cases, exhaustive subset search for the argmax of Eq. 2 on
tiny inputs, sum-to-one invariants, page-permutation invariance, budget >= context.
"""
from __future__ import annotations

from typing import Optional, Sequence, Tuple

import numpy as np

PAGE = 16

COLLECT_NONE = 0
COLLECT_ALL_ROWS = 1      # Eq. 2
COLLECT_FIRST_LAST = 2    # Eq. 3


def decode_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    b = np.asarray(bits)
    if b.dtype != np.uint16:
        raise TypeError("bf16 tensors are passed as uint16 bit patterns")
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def gather_sequence(cache_bits: np.ndarray, pages: np.ndarray, n_tokens: int, kv_head: int) -> np.ndarray:
    """Tokens 0..n_tokens-1 of one sequence for one KV head as float64 [n_tokens, D].

    Token i lives in physical page pages[i // P], slot i % P of the NHD cache
    [num_pages, P, H_kv, D] (App. D).  P is the cache's own page size: 16 on the
    verify/select path; the draft step may list pages of 1, 2, 4, 8 or 16 tokens (Sec. 4 drafts
    with one-token pages, the selected token indices serving as page indices; App. D sweeps 1..16)."""
    P = cache_bits.shape[1]
    nblk = (n_tokens + P - 1) // P
    phys = np.asarray(pages[:nblk], dtype=np.int64)
    x = cache_bits[phys, :, kv_head, :]                    # [nblk, P, D]
    x = x.reshape(nblk * P, -1)[:n_tokens]
    return decode_bf16(x)


def collected_rows(num_queries: int, collect_rows: int) -> Tuple[int, ...]:
    """Row set R of Eq. 2 (all rows) or Eq. 3 (first draft row and bonus row)."""
    if collect_rows == COLLECT_ALL_ROWS:
        return tuple(range(num_queries))
    if collect_rows == COLLECT_FIRST_LAST:
        return tuple(sorted({0, num_queries - 1}))
    return ()


def attention_weights(q_rows: np.ndarray, keys: np.ndarray, scale: float,
                      visible: np.ndarray) -> np.ndarray:
    """softmax(scale * q K^T) restricted to visible keys (Eq. 1's weights).

    q_rows [R, D], keys [n, D], visible bool [R, n].  Rows with no visible key are all 0."""
    s = (q_rows @ keys.T) * scale
    s = np.where(visible, s, -np.inf)
    m = np.max(s, axis=1, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    e = np.where(visible, np.exp(s - m), 0.0)
    z = np.sum(e, axis=1, keepdims=True)
    return np.divide(e, z, out=np.zeros_like(e), where=z > 0)


def verify_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                     block_table: np.ndarray, seq_lens: np.ndarray, scale: float,
                     collect_rows: int = COLLECT_ALL_ROWS, window: int = 0):
    """Full attention of the G = gamma+1 verify rows over the paged cache + page criticality.

    q uint16 [B, G, H_q, D]; caches uint16 [P, 16, H_kv, D]; block_table int32 [B, max_blocks];
    seq_lens int32 [B].  Returns (out float64 [B, G, H_q, D], block_scores float64 [B, max_blocks]).
    block_scores[b, j] = 1/(|R| H_q) * sum_{t in R} sum_h sum_{i in page j} w[t, h, i]; entries
    j >= ceil(n_b/16) are 0.  With COLLECT_NONE the scores are all 0.
    window > 0: local ("sliding window") masking for banded layers (Sec. 4 takes the criticality after the causal
    or the local mask): the row at position pos sees keys pos - window + 1 .. pos only."""
    B, G, Hq, D = q.shape
    Hkv = k_cache.shape[2]
    g = Hq // Hkv
    max_blocks = block_table.shape[1]
    qf = decode_bf16(q)
    out = np.zeros((B, G, Hq, D), dtype=np.float64)
    scores = np.zeros((B, max_blocks), dtype=np.float64)
    R = collected_rows(G, collect_rows)
    for b in range(B):
        n = int(seq_lens[b])
        if n <= 0:
            continue
        nblk = (n + PAGE - 1) // PAGE
        pos = np.arange(n)
        # row t of the G verify tokens sees keys 0 .. n-G+t
        last_visible = n - G + np.arange(G)
        vis_t = pos[None, :] <= last_visible[:, None]                     # [G, n]
        if window > 0:
            vis_t &= pos[None, :] > (last_visible[:, None] - window)
        for hk in range(Hkv):
            K = gather_sequence(k_cache, block_table[b], n, hk)
            V = gather_sequence(v_cache, block_table[b], n, hk)
            for j in range(g):
                h = hk * g + j
                w = attention_weights(qf[b, :, h, :], K, scale, vis_t)     # [G, n]
                out[b, :, h, :] = w @ V
                if R:
                    wr = w[list(R)].sum(axis=0)                            # [n]
                    padded = np.zeros(nblk * PAGE, dtype=np.float64)
                    padded[:n] = wr
                    scores[b, :nblk] += padded.reshape(nblk, PAGE).sum(axis=1)
        if R:
            scores[b] /= (len(R) * Hq)
    return out, scores


def forced_pages(n: int, num_queries: int) -> np.ndarray:
    """Logical pages that overlap the last num_queries token positions [n-G, n)."""
    if n <= 0:
        return np.zeros(0, dtype=np.int64)
    first = max(n - num_queries, 0) // PAGE
    last = (n - 1) // PAGE
    return np.arange(first, last + 1, dtype=np.int64)


def select_logical(scores_row: np.ndarray, n: int, num_queries: int, budget_tokens: int) -> np.ndarray:
    """Selected logical page ids (ascending) of one sequence.

    k = min(ceil(budget/16), nblk), raised to the number of forced pages; forced pages first,
    then the best remaining pages by (score descending, logical index ascending).  A NaN score is
    no criticality at all: it ranks below every number (NumPy's sort order puts NaN last)."""
    if n <= 0:
        return np.zeros(0, dtype=np.int64)
    nblk = (n + PAGE - 1) // PAGE
    F = forced_pages(n, num_queries)
    k = min((max(int(budget_tokens), 0) + PAGE - 1) // PAGE, nblk)
    k = max(k, F.size)
    rest = np.setdiff1d(np.arange(nblk, dtype=np.int64), F)
    s = np.asarray(scores_row[:nblk])[rest]
    order = np.argsort(-s, kind="stable")          # descending score; equal scores keep ascending index
    chosen = rest[order[:k - F.size]]
    return np.sort(np.concatenate([F, chosen]))


def select_blocks(block_scores: np.ndarray, block_table: np.ndarray, seq_lens: np.ndarray,
                  num_queries: int, budget_tokens: int, max_sel_blocks: int,
                  budgets: Optional[Sequence[int]] = None):
    """Top-k pages per sequence -> (sel_table int32 [B, max_sel_blocks] of PHYSICAL page ids in
    ascending logical order, -1 padded; sel_seq_lens int32 [B] = tokens covered by the selection;
    list of the logical ids per sequence)."""
    B = block_table.shape[0]
    sel_table = np.full((B, max_sel_blocks), -1, dtype=np.int32)
    sel_seq_lens = np.zeros(B, dtype=np.int32)
    logical = []
    for b in range(B):
        n = int(seq_lens[b])
        bud = int(budgets[b]) if budgets is not None else int(budget_tokens)
        ids = select_logical(block_scores[b], n, num_queries, bud)
        if ids.size > max_sel_blocks:
            raise ValueError("max_sel_blocks too small")
        logical.append(ids)
        if ids.size == 0:
            continue
        sel_table[b, :ids.size] = block_table[b, ids]
        nblk = (n + PAGE - 1) // PAGE
        tail = n - PAGE * (nblk - 1)               # tokens in the last logical page (always selected)
        sel_seq_lens[b] = PAGE * (ids.size - 1) + tail
    return sel_table, sel_seq_lens, logical


# ---------------------------------------------------------------------------------------------
# The paper's own selection variant: attention LOGITS as the metric, single tokens as the unit
# (Sec. 3.2 Eq. 2, Sec. 3.3 Eq. 3 and its last paragraph, Sec. 4, App. B)
# ---------------------------------------------------------------------------------------------

def token_logit_scores(q: np.ndarray, k_cache: np.ndarray, block_table: np.ndarray,
                       seq_lens: np.ndarray, scale: float, collect_rows: int = COLLECT_FIRST_LAST) -> np.ndarray:
    """Criticality of every PREFIX token from the verification logits.

    The prefix P of sequence b is tokens 0 .. p_b - 1 with p_b = max(n_b - G, 0): what the draft
    tokens were conditioned on, all of it visible to every verification row.  score[b, i] is the
    mean over the collected rows (all of them for Eq. 2, the first draft row and the bonus row for
    Eq. 3) and over all query heads of the scaled logit scale * q_{t,h} . k_i -- the averaging of
    Sec. 3.3's last paragraph; the top-k of these scores is the argmax of Eq. 2 / Eq. 3.
    Returns float64 [B, max_blocks * 16]; entries at and beyond p_b are 0 and mean nothing."""
    B, G, Hq, D = q.shape
    Hkv = k_cache.shape[2]
    g = Hq // Hkv
    qf = decode_bf16(q)
    R = collected_rows(G, collect_rows)
    scores = np.zeros((B, block_table.shape[1] * PAGE), dtype=np.float64)
    if not R:
        return scores
    for b in range(B):
        n = int(seq_lens[b])
        p_len = max(n - G, 0)
        if p_len == 0:
            continue
        acc = np.zeros(p_len, dtype=np.float64)
        for hk in range(Hkv):
            K = gather_sequence(k_cache, block_table[b], p_len, hk)             # [p, D]
            for j in range(g):
                h = hk * g + j
                logits = (qf[b, list(R), h, :] @ K.T) * scale                      # [|R|, p]
                acc += logits.sum(axis=0)
        scores[b, :p_len] = acc / (len(R) * Hq)
    return scores


def select_tokens_logical(scores_row: np.ndarray, n: int, num_queries: int, budget_tokens: int) -> np.ndarray:
    """Selected token positions (ascending) of one sequence.

    The last min(G, n) positions -- the tokens that are not part of the prefix -- are always kept
    (Sec. 3.2, last sentence) and count towards the budget: k = min(budget, n), raised to the
    number of kept tail tokens.  The other k - tail positions are the prefix tokens with the
    highest scores; ties go to the lower position."""
    if n <= 0:
        return np.zeros(0, dtype=np.int64)
    p_len = max(n - num_queries, 0)
    tail = np.arange(p_len, n, dtype=np.int64)
    k = min(max(int(budget_tokens), 0), n)
    k = max(k, tail.size)
    s = np.asarray(scores_row[:p_len])
    order = np.argsort(-s, kind="stable")
    chosen = order[:k - tail.size].astype(np.int64)
    return np.sort(np.concatenate([chosen, tail]))


def select_tokens(token_scores: np.ndarray, block_table: np.ndarray, seq_lens: np.ndarray,
                  num_queries: int, budget_tokens: int, max_sel_tokens: int,
                  budgets: Optional[Sequence[int]] = None):
    """Top-k tokens per sequence -> (sel_table int32 [B, max_sel_tokens]: PHYSICAL token slots
    block_table[i // 16] * 16 + i % 16 in ascending token order, i.e. page ids of the cache seen
    with one-token pages (Sec. 4), -1 padded; sel_seq_lens int32 [B] = tokens selected; list of the
    token positions per sequence)."""
    B = block_table.shape[0]
    sel_table = np.full((B, max_sel_tokens), -1, dtype=np.int32)
    sel_seq_lens = np.zeros(B, dtype=np.int32)
    logical = []
    for b in range(B):
        n = int(seq_lens[b])
        bud = int(budgets[b]) if budgets is not None else int(budget_tokens)
        ids = select_tokens_logical(token_scores[b], n, num_queries, bud)
        if ids.size > max_sel_tokens:
            raise ValueError("max_sel_tokens too small")
        logical.append(ids)
        if ids.size:
            sel_table[b, :ids.size] = block_table[b, ids // PAGE].astype(np.int64) * PAGE + ids % PAGE
            sel_seq_lens[b] = ids.size
    return sel_table, sel_seq_lens, logical


def ratio_budgets(seq_lens: np.ndarray, ratio: float) -> np.ndarray:
    """Per-sequence token budgets from a sparsity ratio (App. C): ceil(ratio * n_b), with the product
    taken in float32 so that the budget is one well-defined integer on every implementation."""
    n = np.asarray(seq_lens).astype(np.float32)
    return np.ceil(np.float32(ratio) * n).astype(np.int64)


def extend_selection(sel_table: np.ndarray, sel_seq_lens: np.ndarray, block_table: np.ndarray,
                     seq_lens_after: np.ndarray, num_new: int, page_size: int):
    """Selection after num_new freshly appended tokens per sequence were added to it (Sec. 3.2, last
    sentence: only the prefix is sparsified; later tokens are kept).  Positions
    [n' - num_new, n') join the selection: a new table entry whenever a position starts a page of the
    selection's page size (16: the physical page block_table[i // 16]; 1: the physical slot
    block_table[i // 16] * 16 + i % 16), and num_new more covered tokens.  Sequences whose row is
    full or whose selection is empty are left unchanged.  Returns new copies."""
    sel = np.array(sel_table, copy=True)
    ssl = np.array(sel_seq_lens, copy=True)
    P = int(page_size)
    for b in range(sel.shape[0]):
        if ssl[b] <= 0:
            continue
        n_new = int(seq_lens_after[b])
        count = (int(ssl[b]) + P - 1) // P
        entries = []
        for i in range(n_new - num_new, n_new):
            if i % P == 0:
                entries.append(int(block_table[b, i // PAGE]) * (PAGE // P) + (i % PAGE) // P)
        if count + len(entries) > sel.shape[1]:
            continue
        sel[b, count:count + len(entries)] = entries
        ssl[b] += num_new
    return sel, ssl


def append_kv(k_cache: np.ndarray, v_cache: np.ndarray, k_new: np.ndarray, v_new: np.ndarray,
              block_table: np.ndarray, seq_lens: np.ndarray, max_seq_len: Optional[int] = None):
    """The cache after every sequence has taken T more tokens (the drafted tokens of Sec. 2.3, whose
    K/V the draft steps that follow must see).  Token t of sequence b becomes position n_b + t: page
    block_table[b][(n_b + t) // 16], slot (n_b + t) % 16, all KV heads (the paged layout of App. D:
    [page, slot, KV head, dim]).  k_new / v_new uint16 [B, T, H_kv, D].  A sequence that would pass
    max_seq_len (default: what its table row can address) takes nothing.  Returns copies of both
    caches and the new lengths (n_b + T for the sequences that took the tokens)."""
    kc = np.array(k_cache, copy=True)
    vc = np.array(v_cache, copy=True)
    lens = np.array(seq_lens, copy=True)
    B, T = k_new.shape[0], k_new.shape[1]
    cap = block_table.shape[1] * PAGE if max_seq_len is None else min(int(max_seq_len), block_table.shape[1] * PAGE)
    for b in range(B):
        n = int(seq_lens[b])
        if n < 0 or n + T > cap:
            continue
        for t in range(T):
            i = n + t
            page = int(block_table[b, i // PAGE])
            for h in range(kc.shape[2]):
                kc[page, i % PAGE, h, :] = k_new[b, t, h, :]
                vc[page, i % PAGE, h, :] = v_new[b, t, h, :]
        lens[b] = n + T
    return kc, vc, lens


def draft_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                    sel_table: np.ndarray, sel_seq_lens: np.ndarray, scale: float) -> np.ndarray:
    """One draft query per sequence attends over exactly the tokens of the selected pages.

    q uint16 [B, H_q, D]; sel_table int32 [B, max_sel_blocks] physical page ids of the cache as it is
    passed in ([num_pages, P, H_kv, D], any page size P); sel_seq_lens[b] tokens are valid (only the
    last listed page may be partial).  No causal mask: the draft token
    is newer than everything cached.  Returns float64 [B, H_q, D]."""
    B, Hq, D = q.shape
    Hkv = k_cache.shape[2]
    g = Hq // Hkv
    qf = decode_bf16(q)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    for b in range(B):
        n = int(sel_seq_lens[b])
        if n <= 0:
            continue
        vis = np.ones((g, n), dtype=bool)
        for hk in range(Hkv):
            K = gather_sequence(k_cache, sel_table[b], n, hk)
            V = gather_sequence(v_cache, sel_table[b], n, hk)
            w = attention_weights(qf[b, hk * g:(hk + 1) * g, :], K, scale, vis)
            out[b, hk * g:(hk + 1) * g, :] = w @ V
    return out


def decoding_iteration(q_verify, q_draft, k_cache, v_cache, block_table, seq_lens, scale,
                       budget_tokens, max_sel_blocks, collect_rows=COLLECT_ALL_ROWS, budgets=None):
    """verify -> select -> one draft call per draft query slab (Sec. 2.3, Sec. 3.1)."""
    G = q_verify.shape[1]
    out_v, scores = verify_attention(q_verify, k_cache, v_cache, block_table, seq_lens, scale, collect_rows)
    sel_table, sel_seq_lens, logical = select_blocks(scores, block_table, seq_lens, G, budget_tokens,
                                                     max_sel_blocks, budgets)
    outs_d = [draft_attention(q_draft[s], k_cache, v_cache, sel_table, sel_seq_lens, scale)
              for s in range(q_draft.shape[0])]
    return out_v, scores, sel_table, sel_seq_lens, logical, outs_d
