/*
 * vegas.h -- C ABI of the MI355X (gfx950) verify -> select -> draft attention path of Vegas,
 * self-speculative decoding with verification-guided sparse attention.
 *
 * One decoding iteration of the method (Sec. 2.3, Sec. 3.1, Fig. 1b) spends its attention time in
 * three operations, which are the three calls below:
 *   1. vegas_verify_attention  full attention of the gamma+1 verification tokens over the whole
 *                              paged KV cache (Eq. 1), which as a by-product yields the criticality
 *                              of every KV page (Eq. 2 / Eq. 3, weights as the metric, App. B);
 *   2. vegas_select_blocks     top-k of those criticalities (the argmax of Eq. 2 / Eq. 3);
 *   3. vegas_draft_attention   attention of one draft token over the selected pages only, done as
 *                              paged attention whose page list is the selection (Sec. 4, App. D).
 * Around them: vegas_select_tokens (the paper's own granularity: single tokens from averaged logits, Sec. 3.3);
 * vegas_append_kv, vegas_extend_selection and vegas_append_kv_extend (the step between two draft calls of a live
 * drafting phase: Sec. 2.3, Sec. 3.2 last sentence); vegas_draft_attention_static (the draft call for callers that
 * cannot allocate device memory); vegas_init, vegas_workspace_bytes, vegas_strerror; and the vegas_debug_* entry
 * points (parts of a call for benchmarks, a table checker, a plain-read yardstick, phase stamps of profiling builds).
 *
 * Conventions shared by every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *     frees or synchronises: a call validates its arguments on the host, enqueues kernels on
 *     `hip_stream` (a hipStream_t passed as void*, NULL = the default stream) and returns.
 *   - bf16 tensors are raw 16-bit patterns.  All tensor pointers must be 16-byte aligned.
 *   - KV cache layout is "NHD" (App. D): [num_pages, page_size, num_kv_heads, head_dim] with the
 *     strides given in the descriptor (in elements; the head_dim stride is 1).  K and V are two
 *     caches with the same strides.
 *   - Query head h uses KV head h / (num_q_heads / num_kv_heads).
 *   - Return value: VEGAS_OK (0) or a negative vegas_status.  Errors that the host can detect are
 *     reported before anything is launched and leave every output untouched.  Page ids are clamped
 *     into [0, num_pages) and lengths into [0, max_seq_len] on the device, so a corrupt table or
 *     length cannot fault; results are then unspecified.
 *   - `workspace` is caller-owned device scratch of at least vegas_workspace_bytes(desc) bytes,
 *     256-byte aligned.  Its contents are meaningless between calls; calls that share a workspace
 *     must be ordered on one stream.
 *   - vegas_init() is optional but recommended once per device before the first call: it does the
 *     one-time, per-device set-up (compute-unit count, raised LDS limits of the large kernels) that
 *     the calls otherwise do lazily on first use.  A caller that captures calls into a HIP graph
 *     must either call vegas_init() first or run each call once outside capture: the lazy set-up
 *     calls hipFuncSetAttribute, which does not belong inside a capture.
 */
#ifndef VEGAS_H
#define VEGAS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum vegas_status {
  VEGAS_OK = 0,
  VEGAS_ERR_NULL = -1,        /* a required pointer is NULL */
  VEGAS_ERR_SHAPE = -2,       /* a size is non-positive or inconsistent */
  VEGAS_ERR_UNSUPPORTED = -3, /* a valid shape this build has no kernel for */
  VEGAS_ERR_ALIGN = -4,       /* pointer or stride alignment */
  VEGAS_ERR_WORKSPACE = -5,   /* workspace missing or too small */
  VEGAS_ERR_LAUNCH = -6       /* the HIP runtime refused a launch */
} vegas_status;

/* Which verification rows contribute to the page criticality. */
enum {
  VEGAS_COLLECT_NONE = 0,       /* no scores; block_scores may be NULL */
  VEGAS_COLLECT_ALL_ROWS = 1,   /* Eq. 2: all gamma+1 rows */
  VEGAS_COLLECT_FIRST_LAST = 2  /* Eq. 3: first draft row and bonus row */
};

/* The criticality vegas_verify_attention collects (vegas_desc.score_metric). */
enum {
  VEGAS_METRIC_PAGE_WEIGHTS = 0, /* per 16-token page: summed softmax weights (App. B's weight variant);
                                    block_scores is fp32 [B, max_blocks]; read by vegas_select_blocks */
  VEGAS_METRIC_TOKEN_LOGITS = 1  /* per token: averaged attention logits (the paper's default metric, Sec. 3.2
                                    footnote, Sec. 3.3 last paragraph); block_scores is fp32
                                    [B, max_blocks * 16]; read by vegas_select_tokens */
};

/* Kernels of an attention call, for the `stages` argument of the vegas_debug_*_stages calls. */
enum {
  VEGAS_STAGE_STREAM = 1,  /* the KV-streaming kernel (reads the cache, writes chunk partials) */
  VEGAS_STAGE_MERGE = 2    /* merge of the chunk partials, and the page scores for verification; a draft call
                              whose selection is short enough for one chunk per (sequence, KV head) has no such
                              kernel: its streaming kernel writes `out` itself */
};

typedef struct vegas_desc {
  int32_t batch;           /* B: sequences (at most 65535) */
  int32_t num_q_heads;     /* H_q */
  int32_t num_kv_heads;    /* H_kv, divides H_q */
  int32_t head_dim;        /* 128, or 64 (the 2 KB-per-token shape of App. D); anything else: VEGAS_ERR_UNSUPPORTED */
  int32_t page_size;       /* tokens per page: 16; vegas_draft_attention also takes 1, 2, 4, 8 */
  int32_t num_queries;     /* verify: G = gamma+1 rows per sequence; ignored by draft (1 row) */
  int32_t max_blocks;      /* row stride of block_table and block_scores */
  int32_t max_sel_blocks;  /* row stride of sel_table */
  int32_t max_seq_len;     /* upper bound on every seq_lens[b] (and sel_seq_lens[b]); sizes the
                              launch grid and the workspace; <= max_blocks*page_size for verify
                              and select, <= max_sel_blocks*page_size for draft; at most 2^30
                              (VEGAS_ERR_UNSUPPORTED above that) */
  int32_t collect_rows;    /* VEGAS_COLLECT_* */
  int32_t kv_chunk_tokens; /* tokens of one sequence handled by one workgroup (a multiple of 32); 0 = the library
                              chooses: from batch, heads and max_seq_len on the host, or, for a verification call
                              on a batch of 2..64 sequences, per sequence on the GPU from seq_lens, so that all
                              workgroups stream about the same number of tokens however loose max_seq_len is.
                              A sequence's chunks are a dimension of the launch grid: a chunk length under which
                              max_seq_len would need more than 65535 chunks (times up to four 32-row blocks where a
                              KV head carries more than 64 rows) is VEGAS_ERR_UNSUPPORTED */
  int32_t reserved;        /* must be 0 */
  float   softmax_scale;   /* Eq. 1's 1/sqrt(d) */
  int32_t score_metric;    /* VEGAS_METRIC_*: what vegas_verify_attention writes to block_scores */
  int32_t window;          /* vegas_verify_attention: > 0 = local ("sliding window") masking of a banded layer
                              (Sec. 4 names the local mask beside the causal one): the row at position pos sees keys
                              pos - window + 1 .. pos.  Such layers are not sparsified, so collect_rows must
                              be VEGAS_COLLECT_NONE.  0 = plain causal masking */
  float   budget_ratio;    /* selection calls: if > 0 and no per-sequence budgets are passed, sequence b's budget
                              is ceil(budget_ratio * seq_lens[b]) tokens (fp32 arithmetic) instead of
                              budget_tokens: a sparsity ratio adapts the budget to the context (App. C) */
  int64_t num_pages;       /* pages in each cache (device-side clamp of page ids) */
  int64_t kv_page_stride;  /* elements between pages */
  int64_t kv_token_stride; /* elements between slots of a page */
  int64_t kv_head_stride;  /* elements between KV heads of a slot */
} vegas_desc;

/* One-time set-up for the CURRENT device (hipSetDevice first): reads the device's compute-unit count
 * and raises the dynamic-LDS limit of every kernel that needs more than the default, so that no later
 * call touches a function attribute (see the conventions above for HIP graph capture).  Idempotent and
 * thread-safe; allocates nothing.  Returns VEGAS_OK, or VEGAS_ERR_LAUNCH if the HIP runtime refuses. */
int vegas_init(void);

/* Bytes of device scratch that any of the calls may need for this descriptor (the upper bound
 * max_seq_len travels in the descriptor).  Pure host function; returns 0 if the descriptor is invalid. */
size_t vegas_workspace_bytes(const vegas_desc* desc);

/*
 * Verification pass (Sec. 2.3; Eq. 1; Eq. 2 / Eq. 3 with weights, App. B).
 *   q            bf16 [B, G, H_q, D]       the gamma+1 verification tokens' queries
 *   k_cache/v_cache bf16 NHD caches; the G tokens' own K/V are already the last G entries of each
 *                sequence, and seq_lens counts them
 *   block_table  int32 [B, max_blocks]     physical page of each logical page; entries at or
 *                                          beyond ceil(seq_lens[b]/16) may be read but are never used
 *   seq_lens     int32 [B]
 *   out          bf16 [B, G, H_q, D]       row t attends to keys 0 .. seq_lens[b]-G+t (causal);
 *                                          a row with no visible key gets 0
 *   block_scores fp32 [B, max_blocks]      score[b][j] = 1/(|R| H_q) sum_{t in R} sum_h
 *                                          sum_{i in page j} w[t,h,i]; R per desc->collect_rows;
 *                                          entries j >= ceil(seq_lens[b]/16) are written as 0.
 *                                          The KV cache is read exactly once.
 */
int vegas_verify_attention(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* block_table, const int32_t* seq_lens,
                           void* out, float* block_scores,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Top-k page selection (Eq. 2's argmax over unions of pages; last sentence of Sec. 3.2 for the
 * tail; Sec. 3.3's last paragraph for "highest scores").
 *   k_b = min(ceil(budget_b/16), pages_b), raised to the number of forced pages; forced pages are
 *   those overlapping token positions [seq_lens[b]-G, seq_lens[b]); the rest are the highest
 *   scores, ties to the lower logical index.  budget_b = budgets[b] if budgets != NULL (per-sequence
 *   budgets, App. C) else budget_tokens.
 *   sel_table    int32 [B, max_sel_blocks]  PHYSICAL page ids in ascending logical order, then -1
 *   sel_seq_lens int32 [B]                  tokens covered: 16*(k_b-1) + tokens in the last page
 * Integer work: for identical fp32 scores the result is defined bit for bit.  A NaN score ranks
 * below every number (and NaNs among themselves by logical index); -0 equals +0.
 * Returns VEGAS_ERR_SHAPE if a row of sel_table cannot hold the largest k_b the call may produce:
 * max_sel_blocks < max(min(ceil(budget/16), ceil(max_seq_len/16)), pages that G positions can touch),
 * with budget = budget_tokens, or ceil(budget_ratio * max_seq_len) when the ratio is set.  The host
 * checks this only when budgets == NULL; with per-sequence budgets k_b is clamped to max_sel_blocks on
 * the device.
 */
int vegas_select_blocks(const vegas_desc* desc, const float* block_scores,
                        const int32_t* block_table, const int32_t* seq_lens,
                        int32_t budget_tokens, const int32_t* budgets,
                        int32_t* sel_table, int32_t* sel_seq_lens,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Selection of single tokens from averaged logits: the paper's own granularity and metric
 * (Sec. 3.3 Eq. 3 and its last paragraph; Sec. 4).  For each sequence b with n_b = seq_lens[b]:
 * the last min(G, n_b) tokens (those after the prefix) are always kept and count towards the
 * budget; k_b = min(budget_b, n_b), raised to the number of kept tail tokens; the other k_b - tail
 * tokens are the prefix tokens (positions < n_b - G) with the highest scores, ties to the lower
 * position.
 *   token_scores fp32 [B, max_blocks*16]    as written by vegas_verify_attention with
 *                                           score_metric = VEGAS_METRIC_TOKEN_LOGITS (only positions
 *                                           below n_b - G are read)
 *   block_table  int32 [B, max_blocks]      16-token pages, as for verification
 *   budget_tokens / budgets                 as for vegas_select_blocks (tokens)
 *   sel_table    int32 [B, max_sel_blocks]  PHYSICAL token slots block_table[i/16]*16 + i%16 in
 *                                           ascending token order, then -1: the page list of
 *                                           vegas_draft_attention with page_size = 1
 *   sel_seq_lens int32 [B]                  k_b
 * desc->page_size is 16 here (it describes block_table); desc->max_sel_blocks counts tokens.
 * Integer work: for identical fp32 scores the result is defined bit for bit (NaN ranks below every
 * number, -0 equals +0, as for vegas_select_blocks).  Five short kernels
 * (four digit-histogram passes that meet in global memory, one ordered compaction); workspace from vegas_workspace_bytes.
 * Returns VEGAS_ERR_SHAPE if max_sel_blocks < max(min(budget_tokens, max_seq_len), min(G, max_seq_len))
 * (checked when budgets == NULL; per-sequence budgets are clamped on the device).
 */
int vegas_select_tokens(const vegas_desc* desc, const float* token_scores,
                        const int32_t* block_table, const int32_t* seq_lens,
                        int32_t budget_tokens, const int32_t* budgets,
                        int32_t* sel_table, int32_t* sel_seq_lens,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The K/V write between two draft steps (Sec. 2.3: tokens are drafted one after the other, each attending to its
 * predecessors).  Every sequence takes num_new more tokens: token t of sequence b is stored at position
 * seq_lens[b] + t, i.e. in page block_table[b][(seq_lens[b] + t) / 16], slot (seq_lens[b] + t) % 16, for every KV
 * head (the cache layout of App. D with the descriptor's strides), and seq_lens[b] is advanced by num_new.
 *   k_new / v_new  bf16 [B, num_new, H_kv, D]  the new tokens' keys and values (num_new at most 4096)
 *   block_table    int32 [B, max_blocks]       must already name a page for every new position (allocating
 *                                              pages is the caller's business)
 *   seq_lens       int32 [B]                   lengths BEFORE the append on entry, AFTER it on return
 *   k_cache / v_cache                          written in place
 * A sequence for which seq_lens[b] + num_new would pass min(max_seq_len, 16 * max_blocks) takes nothing and keeps
 * its length.  Follow with vegas_extend_selection(desc, ..., num_new, ...) so that the next draft call sees the
 * new tokens (or take vegas_append_kv_extend, which does both in one launch).  One small kernel (one workgroup per sequence); no workspace.  desc->page_size is 16.
 */
int vegas_append_kv(const vegas_desc* desc, const void* k_new, const void* v_new, int32_t num_new,
                    const int32_t* block_table, int32_t* seq_lens, void* k_cache, void* v_cache, void* hip_stream);

/*
 * Growth of a selection while drafting (Sec. 3.2, last sentence: tokens after the prefix are kept).
 * Each draft step appends one token's K/V to the cache; the next draft step must see it.  Call this
 * after the caller has written the new K/V and increased seq_lens: for every sequence it adds the
 * num_new newest token positions [seq_lens[b] - num_new, seq_lens[b]) to the selection -- a new entry
 * of sel_table whenever such a position starts a page of the selection's page size, and num_new more
 * tokens in sel_seq_lens[b].
 *   desc->page_size        page size of sel_table: 16 (from vegas_select_blocks; entries are
 *                          block_table[i/16]) or 1 (from vegas_select_tokens; entries are
 *                          block_table[i/16]*16 + i%16)
 *   block_table  int32 [B, max_blocks]   16-token pages of the cache, covering the new positions
 *   seq_lens     int32 [B]               lengths AFTER the append
 *   sel_table / sel_seq_lens             updated in place; a sequence whose row of sel_table is full
 *                                        (max_sel_blocks entries) or whose selection is empty is left as is
 * Precondition: the selection ends with the sequence's last page (every selection of this library does).
 * One tiny kernel; no workspace.
 */
int vegas_extend_selection(const vegas_desc* desc, const int32_t* block_table, const int32_t* seq_lens,
                           int32_t num_new, int32_t* sel_table, int32_t* sel_seq_lens, void* hip_stream);

/*
 * vegas_append_kv followed by vegas_extend_selection in ONE launch (a draft step of a live drafting phase, Sec. 2.3
 * with Sec. 3.2's last sentence, then costs one small kernel before its draft call instead of two).  Arguments as
 * for vegas_append_kv (desc->page_size is 16: it describes the cache and block_table), plus
 *   sel_table      int32 [B, max_sel_blocks]   the selection to grow, updated in place (desc->max_sel_blocks entries
 *   sel_seq_lens   int32 [B]                   per row), under vegas_extend_selection's rules
 *   sel_page_size  page size of sel_table: 16 or 1
 * A sequence whose append is refused (no room) keeps its length AND its selection; otherwise the results are those
 * of the two calls one after the other, bit for bit.  VEGAS_ERR_UNSUPPORTED for another sel_page_size.
 */
int vegas_append_kv_extend(const vegas_desc* desc, const void* k_new, const void* v_new, int32_t num_new,
                           const int32_t* block_table, int32_t* seq_lens, void* k_cache, void* v_cache,
                           int32_t* sel_table, int32_t* sel_seq_lens, int32_t sel_page_size, void* hip_stream);

/*
 * Sparse draft attention (Sec. 2.2 last paragraph; Sec. 4: the selection is the page list).
 *   q            bf16 [B, H_q, D]           one draft token per sequence
 *   sel_table    int32 [B, max_sel_blocks]  as written by vegas_select_blocks
 *   sel_seq_lens int32 [B]
 *   out          bf16 [B, H_q, D]           softmax attention over exactly the first sel_seq_lens[b]
 *                                          token slots of the listed pages; no causal mask; 0 if
 *                                          sel_seq_lens[b] == 0
 * Page size: desc->page_size may be 1, 2, 4, 8 or 16 here (Sec. 4 drafts over one-token pages, the
 * selected token indices serving as page indices; App. D compares page sizes 1..16).  sel_table then
 * lists physical pages of the SAME cache memory seen as [num_pages, page_size, H_kv, D], with
 * kv_page_stride = page_size * kv_token_stride for a contiguous pool and num_pages counted in such
 * pages; only the last listed page of a sequence may be partial.  The other two calls return
 * VEGAS_ERR_UNSUPPORTED for page sizes other than 16.
 */
int vegas_draft_attention(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* sel_table, const int32_t* sel_seq_lens,
                          void* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * vegas_draft_attention for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but the chunk partials live in a scratch array inside the library's
 * device image (vegas_static_scratch_bytes() bytes per device, held until the process ends) instead of a
 * caller's workspace.  The call allocates nothing.
 *   - Returns VEGAS_ERR_WORKSPACE, before anything is launched, when the descriptor needs more scratch
 *     than that (compare vegas_workspace_bytes(desc), for a draft-only descriptor, with the limit).
 *   - All calls on one device share the one array: calls that may overlap in time (different streams
 *     without ordering, different threads) race on it and must be serialised by the caller.  Nothing
 *     in the array has to survive between calls and nothing in it has to start at zero.
 *   - The array's device address is looked up once per device (by vegas_init(), else by the first call
 *     on that device), with that device current.
 */
int vegas_draft_attention_static(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* sel_table, const int32_t* sel_seq_lens,
                                 void* out, void* hip_stream);

/* Size in bytes of the built-in scratch array that vegas_draft_attention_static uses. */
size_t vegas_static_scratch_bytes(void);

/*
 * Profiling aids, not part of the method: the same calls restricted to some of their kernels.
 * `stages` is a mask of VEGAS_STAGE_* bits (0 = the whole call); with anything but the whole call the
 * outputs are incomplete.  The benchmark times the KV-streaming kernel alone through these.
 */
int vegas_debug_verify_attention_stages(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                        const int32_t* block_table, const int32_t* seq_lens,
                                        void* out, float* block_scores,
                                        void* workspace, size_t workspace_bytes, void* hip_stream, int32_t stages);
int vegas_debug_draft_attention_stages(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                       const int32_t* sel_table, const int32_t* sel_seq_lens,
                                       void* out, void* workspace, size_t workspace_bytes, void* hip_stream,
                                       int32_t stages);

/*
 * Debugging aid for the data-dependent errors that the calls do not report: in normal operation a page id outside
 * the pool or a length outside its bounds is clamped on the device (no fault, unspecified results).  This call
 * checks the same inputs and ORs what it finds into a device word, which the caller clears beforehand and reads
 * back whenever it likes (the library never synchronises):
 *   VEGAS_CHECK_LENGTH_RANGE            a length is negative or above desc->max_seq_len
 *   VEGAS_CHECK_LENGTH_EXCEEDS_TABLE    a length needs more pages than a row of the table holds
 *   VEGAS_CHECK_PAGE_ID                 a page id that the length makes the calls read is outside [0, num_pages)
 *   VEGAS_CHECK_SHORTER_THAN_QUERIES    (block tables) 0 < length < num_queries: defined behaviour -- rows with no
 *                                       visible key give 0 -- but hardly what a caller meant
 * `which` says what `table` and `lens` are: VEGAS_TABLE_BLOCKS = block_table / seq_lens of verification and
 * selection (row stride max_blocks, 16-token pages), VEGAS_TABLE_SELECTION = sel_table / sel_seq_lens of a draft
 * call (row stride max_sel_blocks, pages of desc->page_size tokens, num_pages counted in such pages).
 * One small kernel, one workgroup per sequence.
 */
enum { VEGAS_TABLE_BLOCKS = 0, VEGAS_TABLE_SELECTION = 1 };
enum {
  VEGAS_CHECK_LENGTH_RANGE = 1,
  VEGAS_CHECK_LENGTH_EXCEEDS_TABLE = 2,
  VEGAS_CHECK_PAGE_ID = 4,
  VEGAS_CHECK_SHORTER_THAN_QUERIES = 8
};
int vegas_debug_check_tables(const vegas_desc* desc, int32_t which, const int32_t* table, const int32_t* lens,
                             int32_t* error_word, void* hip_stream);

/*
 * Profiling builds only (the library compiled with -DVEGAS_TIMELINE; an ordinary build returns
 * VEGAS_ERR_UNSUPPORTED and its kernels carry no such code).  Registers a device buffer into which every wave of
 * the KV-streaming kernels launched from now on stores eight 64-bit wall-clock stamps (100 MHz) when it exits:
 * [workgroup (x + grid_x * y)][wave][event], events in program order: wave entry, length known, first tile's loads
 * issued, queries in LDS, first tile done, last tile done, merge barrier passed, partial stored.  A launch that
 * needs more than `bytes` writes nothing; NULL switches the stamps off.  Process-wide, not thread-safe: a tool for
 * one profiling run (bench.py --timeline prints the per-phase table from it).
 */
int vegas_debug_set_timeline(void* buffer, size_t bytes);

/*
 * Measurement yardstick, not part of the method: one kernel that does nothing but read two device buffers of
 * bytes_each bytes (a multiple of 16; 16-byte aligned) front to back, coalesced, with `workgroups` workgroups of
 * 256 threads, each on a contiguous slice; non_temporal != 0 marks the loads as read-once, as the verification
 * pass does.  `sink` receives workgroups * 256 32-bit words (their only purpose is to keep the loads alive).
 * The benchmark times it over the same K and V caches the verification kernel streams: the rate it reaches is
 * what the memory system gives a kernel of that footprint that computes nothing.
 */
int vegas_debug_stream_read(const void* a, const void* b, size_t bytes_each, int32_t workgroups, int32_t non_temporal,
                            void* sink, void* hip_stream);

/* Static, human-readable text for a vegas_status. */
const char* vegas_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* VEGAS_H */
