// Host side of the C ABI declared in include/vegas.h: argument validation, launch planning,
// workspace carving and kernel launches.  Nothing here allocates or synchronises.
#include "../../include/vegas.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <map>
#include <mutex>
#include <set>
#include <utility>

#include "attn_finalize.hpp"
#include "attn_draft.hpp"
#include "attn_pair.hpp"
#include "attn_split.hpp"
#include "debug_kernels.hpp"
#include "kv_append.hpp"
#include "select_blocks.hpp"
#include "select_tokens.hpp"
#include "vegas_common.hpp"

namespace {

using namespace vegas;

constexpr int kDefaultCU = 256;       // MI355X compute units: assumed where no device is visible
constexpr size_t kAlign = 256;

// Compute units of the current device, asked once per device.  The launch plans aim at one or two workgroups per
// compute unit, and the workspace is sized from the same plans, so sizing and launching must see the same number:
// without a visible device (the pure-host sizing call on a machine that has none) it is the MI355X's 256.
int device_cu_count() {
  static std::mutex mu;
  static std::map<int, int> known;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return kDefaultCU;
  }
  std::lock_guard<std::mutex> lock(mu);
  const auto it = known.find(dev);
  if (it != known.end()) return it->second;
  int n = 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) {
    (void)hipGetLastError();
    n = kDefaultCU;
  }
  known[dev] = n;
  return n;
}
// longest selection a draft call streams with one workgroup per (sequence, KV head): 256 tokens at head dimension 128,
// 384 at 64 (tiles of half the bytes), each plus the two pages of slack a selection table carries
constexpr int kFinishTokens128 = 288, kFinishTokens64 = 416;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct SplitPlan {
  int R = 0, Rc = 0, NB = 0, NW = 0, chunk = 0, nsplit = 0, lse_pages = 0;   // Rc: collected rows per KV head
  bool pair = false;                 // 33..64 rows per KV head: one workgroup serves both row blocks (attn_pair_kernel)
  bool balanced = false;             // chunk lengths per sequence, computed on the GPU from the lengths (ragged batches)
  int J = 0, J2 = 0, JS = 0;         // balanced: workgroups per KV head of a one-wave and a two-wave plan; slots held
  int cap_units = 0;                 // balanced: longest chunk, in units of kTile * NW tokens
  size_t off_trash = 0;              // a word for stores that must go nowhere
  size_t off_plan = 0;               // balanced: [B] (first slot, chunk tokens)
  size_t off_part_o = 0, off_part_ml = 0, off_page_lse = 0, total = 0;
};

int check_common(const vegas_desc* d) {
  if (!d) return VEGAS_ERR_NULL;
  if (d->batch <= 0 || d->num_q_heads <= 0 || d->num_kv_heads <= 0 || d->max_blocks <= 0 ||
      d->max_seq_len <= 0 || d->num_pages <= 0)
    return VEGAS_ERR_SHAPE;
  if (d->num_q_heads % d->num_kv_heads != 0) return VEGAS_ERR_SHAPE;
  if (d->head_dim != 128 && d->head_dim != 64) return VEGAS_ERR_UNSUPPORTED;
  if (d->max_seq_len > (1 << 30)) return VEGAS_ERR_UNSUPPORTED;      // token counts and offsets are 32-bit in the kernels
  if (d->batch > 65535) return VEGAS_ERR_UNSUPPORTED;                // sequences are a grid's y or z dimension
  if (d->page_size != 1 && d->page_size != 2 && d->page_size != 4 && d->page_size != 8 && d->page_size != kPage)
    return VEGAS_ERR_UNSUPPORTED;
  if (d->kv_head_stride < d->head_dim || d->kv_token_stride < d->head_dim ||
      d->kv_page_stride < static_cast<int64_t>(d->page_size) * d->head_dim)
    return VEGAS_ERR_SHAPE;
  if ((d->kv_head_stride % 8) || (d->kv_token_stride % 8) || (d->kv_page_stride % 8)) return VEGAS_ERR_ALIGN;
  if (d->kv_chunk_tokens < 0 || (d->kv_chunk_tokens % kTile) != 0) return VEGAS_ERR_SHAPE;
  if (!(d->softmax_scale > 0.f)) return VEGAS_ERR_SHAPE;
  if (d->reserved != 0) return VEGAS_ERR_SHAPE;
  return VEGAS_OK;
}

// Verification and selection work on 16-token pages and a block table that covers max_seq_len.
int check_paged16(const vegas_desc* d) {
  if (d->page_size != kPage) return VEGAS_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(d->max_seq_len) > static_cast<int64_t>(d->max_blocks) * kPage) return VEGAS_ERR_SHAPE;
  return VEGAS_OK;
}

// Rows stacked on one KV head decide the kernel variant; the chunk size decides the grid.
// max_len bounds the lengths the call may see; small problems get small workgroups.
// collect: 0 nothing, 1 page log-sum-exps [pages x rows], 2 token sums [padded tokens] per (sequence, KV head)
// sum_block: the logit metric's two query-sum rows get a row block of their own (no spare rows in the last real one)
int plan_split(const vegas_desc* d, int rows_per_head, int max_len, int collect, int wg_per_cu, SplitPlan* pl,
               bool may_pair = false, bool may_finish = false, bool sum_block = false) {
  pl->R = rows_per_head;
  const int num_cu = device_cu_count();
  const int64_t heads = static_cast<int64_t>(d->batch) * d->num_kv_heads;
  if (rows_per_head > 128) return VEGAS_ERR_UNSUPPORTED;
  pl->NB = (rows_per_head + 31) / 32 + (sum_block ? 1 : 0);   // 32-row blocks
  pl->NW = 4;                                        // measured: 4-wave groups match or beat 8-wave groups everywhere
  // Two row blocks: one workgroup per chunk reads K/V once for both (attn_pair_kernel) when the chunk holds an even
  // number of tiles; otherwise (and for 3 or 4 blocks) sibling workgroups, one per block, share an XCD's L2.
  pl->pair = may_pair && !sum_block && pl->NB == 2;
  if (pl->pair && d->kv_chunk_tokens != 0 && d->kv_chunk_tokens % (kTile * kPairs) != 0) pl->pair = false;
  // A draft call over a short selection (may_finish): one workgroup per (sequence, KV head) streams all of it and
  // writes the output rows itself, so no merge kernel is launched.  Measured at 4K context, five draft calls per
  // iteration: 256 selected tokens (eight tiles, two per wave) 54.7 us against 59.3 us with three chunks and a merge;
  // 384 tokens 61.8 against 59.4; 512 tokens 67.2 against 59.8 -- a workgroup takes about 0.35 us per further tile,
  // with four waves or with eight, so the merge launch is the cheaper price from nine or ten tiles on.  At head
  // dimension 64 (32K context, 64 query heads): 256 tokens 66.5 against 73.0 us, 384 tokens 71.4 against 73.0,
  // 512 tokens 75.1 against 73.3.
  const bool finish = may_finish && d->kv_chunk_tokens == 0 &&
                      max_len <= (d->head_dim == 64 ? kFinishTokens64 : kFinishTokens128) &&
                      static_cast<int64_t>(d->batch) * d->num_kv_heads * pl->NB <= num_cu;
  const int unit = kTile * pl->NW;
  int chunk = d->kv_chunk_tokens;
  if (finish) chunk = (max_len + unit - 1) / unit * unit;
  if (chunk == 0) {
    // Verification: one workgroup per CU when the batch is small (at 32K context 256 equal workgroups
    // beat 512); draft calls are latency-bound and like two small workgroups per CU.  With many
    // (sequence, head) columns, shorter chunks balance ragged lengths better.
    const int64_t columns = heads * (pl->pair ? 1 : pl->NB);
    int64_t splits = static_cast<int64_t>(num_cu) * wg_per_cu / columns;
    if (splits < 1) splits = 1;
    int64_t c = (max_len + splits - 1) / splits;
    {
      // Round to whole units: up, unless a bound a little above a multiple (a selection table with two pages of
      // slack) would then double every wave's tiles -- a quarter more workgroups than planned is the better price.
      const int64_t up = (c + unit - 1) / unit * unit, down = c / unit * unit;
      c = up;
      if (down >= unit && ((max_len + down - 1) / down) * columns * 4 <= static_cast<int64_t>(num_cu) * wg_per_cu * 5) c = down;
    }
    if (pl->pair) {
      // the pair kernel likes two workgroups per CU once their chunks are long enough (one sequence of 128K tokens,
      // 40 rows: 512 chunks of 2048 tokens 115 us, 256 of 4096 132 us; at 32K tokens the finalising kernel's
      // larger table of chunks eats the gain)
      const int64_t c2 = ((max_len + 2 * splits - 1) / (2 * splits) + unit - 1) / unit * unit;
      if (wg_per_cu == 1 && c2 >= 2048) { c = c2; splits *= 2; }
    }
    // What a workgroup collects is parked in LDS until its chunk ends, so a chunk cannot be arbitrarily long.  A
    // chunk that gives every CU exactly one workgroup is taken as it is while its LDS fits (batch 4 x 64K tokens:
    // 256 chunks of 8192 tokens reach 78 % of the HBM peak, 512 chunks of 4096 tokens 75 %); otherwise chunks are
    // capped so that two workgroups fit a CU.  (The pair kernel parks nothing per chunk: any chunk length.)
    const int64_t cap = (columns >= num_cu) ? 2048 : 4096;
    const int prows = rows_per_head < 32 ? rows_per_head : 32;
    const bool fits_alone = columns * splits >= num_cu / 2 &&
                            split_lds_bytes(pl->NW, prows, collect, static_cast<int>(c), d->head_dim) <= 150 * 1024;
    if (!pl->pair && c > cap && !(wg_per_cu == 1 && fits_alone)) c = cap;
    chunk = static_cast<int>(c);
  }
  // A batch of several sequences whose lengths the host does not know (only max_seq_len, which may be loose): every
  // workgroup derives the chunk length of each sequence from seq_lens on the GPU (balanced_slot), so that a fixed
  // number of workgroups stream about the same number of tokens each.  (A host-side chunk length cuts a ragged
  // batch into unequal numbers of equal chunks: 45 % of the HBM peak on 16 sequences of 8K..64K tokens, 40 rows,
  // against 68 % with the plan; and it sizes chunks for lengths that may never occur.)
  const int64_t per_head = static_cast<int64_t>(d->num_kv_heads) * (pl->pair ? 1 : pl->NB);   // workgroups per slot
  pl->balanced = may_pair && d->kv_chunk_tokens == 0 && d->batch >= 2 && d->batch <= 64 && max_len < (1 << 24) &&
                 per_head <= num_cu;
  pl->chunk = chunk;
  pl->nsplit = (max_len + chunk - 1) / chunk;
  size_t slots = static_cast<size_t>(heads) * pl->nsplit;       // chunk partials the workspace holds
  if (pl->balanced) {
    int64_t most_chunks;                                        // of one sequence
    if (pl->pair) {
      // one launch wave (two workgroups per CU) without collection; with it, shorter chunks in two waves were
      // measured faster (16 sequences of 8K..64K tokens, 40 rows: 505 us against 515 us).  Nothing is parked.
      pl->J = pl->J2 = static_cast<int>((collect ? 4 : 2) * num_cu / per_head);
      pl->cap_units = 1 << 20;
      pl->chunk = unit;                                         // (unused: every sequence has its own)
      most_chunks = pl->J;
    } else {
      // one workgroup per CU with chunks as long as its LDS can park (16 x 36864 tokens, 20 rows: 256 chunks of
      // 18432 tokens reach 80 % of the peak, 512 of 9216 75 %, 4096-token chunks 69 %); two waves when the
      // lengths are too ragged for one
      pl->J = static_cast<int>(num_cu / per_head);
      // (slots no plan uses still cost a workgroup that works that out, at one workgroup per CU in a wave of their
      // own behind the others: a small batch, whose kernel is short, gets the one-wave plan only)
      pl->J2 = d->batch >= 8 ? 2 * pl->J : pl->J;
      const int prows = rows_per_head < 32 ? rows_per_head : 32;
      int cap = 1 << 24;
      if (collect != 0) {
        cap = unit;
        while (split_lds_bytes(pl->NW, prows, collect, cap + unit, d->head_dim) <= 150 * 1024 && cap < (1 << 24)) cap += unit;
      }
      pl->cap_units = cap / unit;
      pl->chunk = collect != 0 ? cap : unit;                    // sizes the LDS that parks a chunk's collected values
      most_chunks = (static_cast<int64_t>(max_len) + cap - 1) / cap;
      if (most_chunks < pl->J2) most_chunks = pl->J2;
    }
    if (pl->J < 1) pl->J = 1;
    if (pl->J2 < pl->J) pl->J2 = pl->J;
    // slots: a plan for J2 workgroups never takes more than max(J2, B) of them; a capped one B * most_chunks
    int64_t js = pl->J2 > d->batch ? pl->J2 : d->batch;
    const int64_t capped = static_cast<int64_t>(d->batch) * ((static_cast<int64_t>(max_len) + static_cast<int64_t>(pl->cap_units) * unit - 1) /
                                                            (static_cast<int64_t>(pl->cap_units) * unit));
    if (capped > js) js = capped;
    pl->JS = static_cast<int>(js);
    pl->nsplit = static_cast<int>(most_chunks);                 // most chunks one sequence can get
    slots = static_cast<size_t>(d->num_kv_heads) * pl->JS;   // (sibling row blocks share a slot)
  }
  pl->lse_pages = collect == 1 ? (max_len + kPage - 1) / kPage
                               : (collect == 2 ? (pl->balanced ? (max_len + unit - 1) / unit * unit : pl->nsplit * chunk) : 0);
  size_t off = 0;
  const size_t hs = static_cast<size_t>(heads);
  pl->off_part_o = off;  off += align_up(slots * pl->R * d->head_dim * sizeof(float));
  pl->off_part_ml = off; off += align_up(slots * pl->R * sizeof(float2));
  pl->off_page_lse = off;
  pl->Rc = collected_count(d->collect_rows, d->num_queries, d->num_q_heads / d->num_kv_heads);
  off += align_up(hs * static_cast<size_t>(pl->lse_pages) * (collect == 2 ? 1 : pl->Rc) * sizeof(float));
  pl->off_plan = off;
  if (pl->balanced) off += align_up(static_cast<size_t>(d->batch) * sizeof(int2));
  pl->off_trash = off;
  off += kAlign;
  pl->total = off;
  return VEGAS_OK;
}

int plan_verify(const vegas_desc* d, SplitPlan* pl) {
  if (d->num_queries <= 0) return VEGAS_ERR_SHAPE;
  if (d->collect_rows < 0 || d->collect_rows > 2) return VEGAS_ERR_SHAPE;
  const int g = d->num_q_heads / d->num_kv_heads;
  if (d->score_metric != VEGAS_METRIC_PAGE_WEIGHTS && d->score_metric != VEGAS_METRIC_TOKEN_LOGITS)
    return VEGAS_ERR_SHAPE;
  const int R = d->num_queries * g;
  const int collect = d->collect_rows == 0 ? 0 : (d->score_metric == VEGAS_METRIC_TOKEN_LOGITS ? 2 : 1);
  // The logit metric's two query-sum rows ride in spare rows of the last 32-row block of a KV head; where that block
  // has fewer than two (R = 31, 32, 63, 64, ... rows) they get a sibling row block of their own, which streams K
  // alongside the others (same XCD, served by its L2) and writes no output rows.
  const bool sum_block = collect == 2 && (R % 32 == 0 || R % 32 == 31);
  return plan_split(d, R, d->max_seq_len, collect, 1, pl, d->window == 0, false, sum_block);
}

int plan_draft(const vegas_desc* d, SplitPlan* pl) {
  const int g = d->num_q_heads / d->num_kv_heads;
  return plan_split(d, g, d->max_seq_len, 0, 2, pl, false, true);
}

// A kernel whose static + dynamic LDS passes the default 64 KB limit needs its limit raised first: once
// per (device, kernel function).  The table is keyed by the function's address because every
// instantiation of the streaming kernel has the same C++ type.
// (vegas_init raises every kernel's limit up front; this lazy path serves callers that never call it.)
int ensure_dynamic_lds(const void* kern, size_t lds) {
  if (lds <= 32 * 1024) return VEGAS_OK;
  static std::mutex mu;
  static std::set<std::pair<int, const void*>> raised;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return VEGAS_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(mu);
  const std::pair<int, const void*> key(dev, kern);
  if (raised.count(key)) return VEGAS_OK;
  hipFuncAttributes attr;
  if (hipFuncGetAttributes(&attr, kern) != hipSuccess) return VEGAS_ERR_LAUNCH;
  const int room = 160 * 1024 - static_cast<int>(attr.sharedSizeBytes);   // the CU's LDS minus the kernel's static part
  if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, room) != hipSuccess)
    return VEGAS_ERR_LAUNCH;
  raised.insert(key);
  return VEGAS_OK;
}

// Profiling builds (-DVEGAS_TIMELINE): the buffer that vegas_debug_set_timeline registered receives the phase stamps of
// the next streaming kernels (if it is large enough for the launch); ordinary builds have no such buffer.
unsigned long long* g_timeline = nullptr;
size_t g_timeline_bytes = 0;

template <typename Kern>
int launch_one(Kern kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, SplitParams sp) {
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds)) return rc;
  const size_t tl_need = static_cast<size_t>(grid.x) * grid.y * grid.z * (block.x / 64) * kTimelineEvents * sizeof(unsigned long long);
  sp.timeline = (g_timeline != nullptr && tl_need <= g_timeline_bytes) ? g_timeline : nullptr;
  hipLaunchKernelGGL(kern, grid, block, lds, st, VEGAS_SPLIT_HOT_ARGS(sp), sp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

template <bool CAUSAL, int COLLECT, int D>
int launch_split_d(const SplitPlan& pl, SplitParams sp, int batch, hipStream_t st, int page_size) {
  if constexpr (CAUSAL) {
    if (pl.pair) {                                  // both row blocks from one read of K/V
      const dim3 pgrid = pl.balanced ? dim3(pl.JS, sp.Hkv, 1) : dim3(pl.nsplit, sp.Hkv, batch);   // chunks fastest
      const size_t plds = pair_lds_bytes(pl.R, COLLECT, D);
      sp.lds_q_off = static_cast<int32_t>(plds - pair_lds_tail_bytes(D));
      sp.row_blocks = 1;
      if (plds > 160 * 1024) return VEGAS_ERR_UNSUPPORTED;
      return launch_one(attn_pair_kernel<COLLECT, D>, pgrid, dim3(kPairWaves * 64), plds, st, sp);
    }
  }
  // (KV head, row block + NB * chunk, sequence): the kernels read their indices off the grid without a division
  const dim3 grid = pl.balanced ? dim3(sp.Hkv, static_cast<unsigned>(pl.NB) * pl.JS, 1)
                                : dim3(sp.Hkv, static_cast<unsigned>(pl.NB) * pl.nsplit, batch);
  if (grid.y > 65535u) return VEGAS_ERR_UNSUPPORTED;        // more chunks per sequence than a grid dimension holds
  const int rows = pl.R < 32 ? pl.R : 32;
  const size_t lds = split_lds_bytes(pl.NW, rows, COLLECT, pl.chunk, D);
  sp.lds_q_off = static_cast<int32_t>(lds - split_lds_tail_bytes(pl.NW, D));
  sp.row_blocks = pl.NB;
  if (lds > 160 * 1024) return VEGAS_ERR_UNSUPPORTED;
  if constexpr (!CAUSAL && COLLECT == 0) {
    // one draft token, a group of at most 16 heads, 16-token pages: the kernel written for exactly that
    if (pl.R <= kDraftRows && sp.G == 1 && pl.NB == 1) {
      const dim3 dblock(kDraftWaves * 64);
      const size_t dlds = draft16_lds_bytes(pl.R, D);
      switch (page_size) {                              // (draft calls may walk a table of smaller pages)
        case 1: return launch_one(attn_draft16_kernel<D, 0>, grid, dblock, dlds, st, sp);
        case 2: return launch_one(attn_draft16_kernel<D, 1>, grid, dblock, dlds, st, sp);
        case 4: return launch_one(attn_draft16_kernel<D, 2>, grid, dblock, dlds, st, sp);
        case 8: return launch_one(attn_draft16_kernel<D, 3>, grid, dblock, dlds, st, sp);
        default: return launch_one(attn_draft16_kernel<D, 4>, grid, dblock, dlds, st, sp);
      }
    }
    switch (page_size) {                                // larger groups: the 32-row kernel, any page size
      case 1: return launch_one(attn_split_kernel<4, 2, false, 0, false, 0, false, D>, grid, dim3(256), lds, st, sp);
      case 2: return launch_one(attn_split_kernel<4, 2, false, 0, false, 1, false, D>, grid, dim3(256), lds, st, sp);
      case 4: return launch_one(attn_split_kernel<4, 2, false, 0, false, 2, false, D>, grid, dim3(256), lds, st, sp);
      case 8: return launch_one(attn_split_kernel<4, 2, false, 0, false, 3, false, D>, grid, dim3(256), lds, st, sp);
      default: break;
    }
  }
  if constexpr (CAUSAL && COLLECT == 0) {           // banded layer: local masking on top of the causal mask
    if (sp.window > 0) {
      if (pl.NB == 1) return launch_one(attn_split_kernel<4, 2, true, 0, true, 4, true, D>, grid, dim3(256), lds, st, sp);
      return launch_one(attn_split_kernel<4, 2, true, 0, false, 4, true, D>, grid, dim3(256), lds, st, sp);
    }
  }
  constexpr bool kVerify = CAUSAL;                  // the verification pass is the only causal caller
  if (kVerify && pl.NB == 1)                        // one reader per K/V line, read once: stream it
    return launch_one(attn_split_kernel<4, 2, CAUSAL, COLLECT, kVerify, 4, false, D>, grid, dim3(256), lds, st, sp);
  return launch_one(attn_split_kernel<4, 2, CAUSAL, COLLECT, false, 4, false, D>, grid, dim3(256), lds, st, sp);
}

template <bool CAUSAL, int COLLECT>
int launch_split(const SplitPlan& pl, const SplitParams& sp, int batch, hipStream_t st, int head_dim, int page_size = kPage) {
  if (head_dim == 64) return launch_split_d<CAUSAL, COLLECT, 64>(pl, sp, batch, st, page_size);
  return launch_split_d<CAUSAL, COLLECT, 128>(pl, sp, batch, st, page_size);
}

void fill_split_params(const vegas_desc* d, const SplitPlan& pl, int G, const void* q, const void* k,
                       const void* v, const int32_t* table, int table_stride, const int32_t* lens,
                       unsigned char* ws, SplitParams* sp) {
  sp->q = static_cast<const uint16_t*>(q);
  sp->k = static_cast<const uint16_t*>(k);
  sp->v = static_cast<const uint16_t*>(v);
  sp->table = table;
  sp->lens = lens;
  sp->part_o = reinterpret_cast<float*>(ws + pl.off_part_o);
  sp->part_ml = reinterpret_cast<float2*>(ws + pl.off_part_ml);
  sp->page_lse = reinterpret_cast<float*>(ws + pl.off_page_lse);
  sp->table_stride = table_stride;
  sp->G = G;
  sp->g = d->num_q_heads / d->num_kv_heads;
  sp->R = pl.R;
  sp->Hq = d->num_q_heads;
  sp->Hkv = d->num_kv_heads;
  sp->chunk_tokens = pl.chunk;
  sp->nsplit = pl.nsplit;
  sp->lse_pages = pl.lse_pages;
  sp->collect_rows = d->collect_rows;
  sp->Rc = pl.Rc;
  sp->window = 0;
  sp->out_direct = nullptr;
  sp->trash = reinterpret_cast<float*>(ws + pl.off_trash);
  sp->plan = pl.balanced ? reinterpret_cast<int2*>(ws + pl.off_plan) : nullptr;
  sp->batch = d->batch;
  sp->slots_target = pl.J;
  sp->slots_target2 = pl.J2;
  sp->chunk_cap_units = pl.cap_units;
  sp->slots_total = pl.JS;
  sp->chunk_unit = kTile * pl.NW;
  sp->max_tokens = d->max_seq_len;
  sp->page_stride = d->kv_page_stride;
  sp->token_stride = d->kv_token_stride;
  sp->head_stride = d->kv_head_stride;
  sp->num_pages = d->num_pages;
  sp->scale_log2e = d->softmax_scale * 1.4426950408889634f;
  sp->timeline = nullptr;
}

// Scratch of vegas_select_tokens: digit histograms [B, 4 passes, slices, 256].
int token_slices(const vegas_desc* d) {
  return static_cast<int>((static_cast<int64_t>(d->max_blocks) * kPage + kTokSlice - 1) / kTokSlice);
}
size_t token_select_bytes(const vegas_desc* d) {
  return align_up(static_cast<size_t>(d->batch) * 4 * token_slices(d) * 256 * sizeof(uint32_t));
}

// Largest token budget a selection call can meet when no per-sequence budgets are passed: the constant,
// or (budget_ratio > 0) the ratio applied to the longest allowed sequence, in the kernels' fp32 arithmetic.
int64_t ratio_or_constant_budget(const vegas_desc* d, int32_t budget_tokens) {
  if (d->budget_ratio > 0.f) return static_cast<int64_t>(std::ceil(d->budget_ratio * static_cast<float>(d->max_seq_len)));
  return budget_tokens;
}

int launch_combine(const vegas_desc* d, const SplitPlan& pl, const SplitParams& sp, void* out, hipStream_t st) {
  CombineParams cp;
  cp.part_o = sp.part_o;
  cp.part_ml = sp.part_ml;
  cp.lens = sp.lens;
  cp.out = static_cast<uint16_t*>(out);
  cp.G = sp.G; cp.g = sp.g; cp.R = sp.R; cp.Hq = sp.Hq; cp.Hkv = sp.Hkv;
  cp.chunk_tokens = pl.chunk; cp.nsplit = pl.nsplit; cp.max_tokens = d->max_seq_len;
  cp.window = sp.window;
  cp.D = d->head_dim;
  cp.plan = sp.plan;
  cp.slots_total = sp.slots_total;
  const dim3 grid(pl.R, sp.Hkv, d->batch);
  if (pl.nsplit <= 8)
    hipLaunchKernelGGL(attn_combine_small_kernel<8>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 12)
    hipLaunchKernelGGL(attn_combine_small_kernel<12>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 16)
    hipLaunchKernelGGL(attn_combine_small_kernel<16>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 20)
    hipLaunchKernelGGL(attn_combine_small_kernel<20>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 24)
    hipLaunchKernelGGL(attn_combine_small_kernel<24>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 32)
    hipLaunchKernelGGL(attn_combine_small_kernel<32>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 40)
    hipLaunchKernelGGL(attn_combine_small_kernel<40>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 48)
    hipLaunchKernelGGL(attn_combine_small_kernel<48>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else if (pl.nsplit <= 64)
    hipLaunchKernelGGL(attn_combine_small_kernel<64>, grid, dim3(cp.D), 0, st, VEGAS_COMBINE_HOT_ARGS(cp), cp);
  else
    hipLaunchKernelGGL(attn_combine_kernel, grid, dim3(cp.D), 0, st, cp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

// Scratch of vegas_draft_attention_static: the chunk partials of one draft call, in the library's own device image
// instead of a caller's workspace.  Every device the library runs on holds its own copy of the array at its own
// address until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address it yields (per device, asked once with that device current) is what kernels and copies get.
constexpr size_t kStaticScratchBytes = size_t(8) << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int static_scratch_address(void** out) {
  static std::mutex mu;
  static std::map<int, void*> known;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return VEGAS_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(mu);
  const auto it = known.find(dev);
  if (it != known.end()) {
    *out = it->second;
    return VEGAS_OK;
  }
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
    (void)hipGetLastError();
    return VEGAS_ERR_LAUNCH;
  }
  known[dev] = ptr;
  *out = ptr;
  return VEGAS_OK;
}

// Every kernel that is launched with dynamic LDS, for vegas_init: f(kernel address).
template <typename F>
int for_each_lds_kernel(F f) {
  int rc = VEGAS_OK;
  auto one = [&](auto kern) { if (rc == VEGAS_OK) rc = f(reinterpret_cast<const void*>(kern)); };
  auto per_dim = [&](auto dtag) {
    constexpr int D = decltype(dtag)::value;
    one(attn_split_kernel<4, 2, false, 0, false, 0, false, D>);      // draft calls, page sizes 1, 2, 4, 8, 16
    one(attn_split_kernel<4, 2, false, 0, false, 1, false, D>);
    one(attn_split_kernel<4, 2, false, 0, false, 2, false, D>);
    one(attn_split_kernel<4, 2, false, 0, false, 3, false, D>);
    one(attn_split_kernel<4, 2, false, 0, false, 4, false, D>);
    one(attn_split_kernel<4, 2, true, 0, true, 4, true, D>);         // verification of a banded layer
    one(attn_split_kernel<4, 2, true, 0, false, 4, true, D>);
    one(attn_split_kernel<4, 2, true, 0, true, 4, false, D>);        // verification: no collection / page weights / logits,
    one(attn_split_kernel<4, 2, true, 0, false, 4, false, D>);       // one reader per line or sibling row blocks
    one(attn_split_kernel<4, 2, true, 1, true, 4, false, D>);
    one(attn_split_kernel<4, 2, true, 1, false, 4, false, D>);
    one(attn_split_kernel<4, 2, true, 2, true, 4, false, D>);
    one(attn_split_kernel<4, 2, true, 2, false, 4, false, D>);
    one(attn_draft16_kernel<D, 0>);
    one(attn_draft16_kernel<D, 1>);
    one(attn_draft16_kernel<D, 2>);
    one(attn_draft16_kernel<D, 3>);
    one(attn_draft16_kernel<D, 4>);
    one(attn_pair_kernel<0, D>);
    one(attn_pair_kernel<1, D>);
    one(attn_pair_kernel<2, D>);
  };
  per_dim(std::integral_constant<int, 128>{});
  per_dim(std::integral_constant<int, 64>{});
  one(verify_finalize_kernel<16, 0>); one(verify_finalize_kernel<32, 0>);
  one(verify_finalize_kernel<64, 0>); one(verify_finalize_kernel<0, 0>);
  one(verify_finalize_kernel<16, 1>); one(verify_finalize_kernel<32, 1>);
  one(verify_finalize_kernel<64, 1>); one(verify_finalize_kernel<0, 1>);
  one(select_blocks_kernel);
  return rc;
}

}  // namespace

extern "C" {

int vegas_init(void) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return VEGAS_ERR_LAUNCH;
  }
  (void)device_cu_count();
  void* ptr = nullptr;
  if (int rc = static_scratch_address(&ptr)) return rc;
  return for_each_lds_kernel([](const void* kern) { return ensure_dynamic_lds(kern, 160 * 1024); });
}

size_t vegas_static_scratch_bytes(void) { return kStaticScratchBytes; }

size_t vegas_workspace_bytes(const vegas_desc* desc) {
  if (check_common(desc) != VEGAS_OK) return 0;
  SplitPlan pv, pd;
  size_t need = kAlign;
  if (desc->num_queries > 0 && check_paged16(desc) == VEGAS_OK && plan_verify(desc, &pv) == VEGAS_OK)
    need = pv.total > need ? pv.total : need;
  if (plan_draft(desc, &pd) == VEGAS_OK) need = pd.total > need ? pd.total : need;
  if (check_paged16(desc) == VEGAS_OK) {
    const size_t ts = token_select_bytes(desc);
    need = ts > need ? ts : need;
  }
  return need;
}

static int verify_impl(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                       const int32_t* block_table, const int32_t* seq_lens, void* out, float* block_scores,
                       void* workspace, size_t workspace_bytes, void* hip_stream, int32_t stages) {
  if (stages < 0 || stages > (VEGAS_STAGE_STREAM | VEGAS_STAGE_MERGE)) return VEGAS_ERR_SHAPE;
  int rc = check_common(desc);
  if (rc == VEGAS_OK) rc = check_paged16(desc);
  if (rc != VEGAS_OK) return rc;
  if (!q || !k_cache || !v_cache || !block_table || !seq_lens || !out) return VEGAS_ERR_NULL;
  SplitPlan pl;
  rc = plan_verify(desc, &pl);
  if (rc != VEGAS_OK) return rc;
  const bool collect = desc->collect_rows != VEGAS_COLLECT_NONE;
  const bool logits = collect && desc->score_metric == VEGAS_METRIC_TOKEN_LOGITS;
  if (collect && !block_scores) return VEGAS_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(block_table) ||
      (block_scores && !aligned16(block_scores)))
    return VEGAS_ERR_ALIGN;
  if (!workspace || workspace_bytes < pl.total) return VEGAS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return VEGAS_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);

  SplitParams sp;
  fill_split_params(desc, pl, desc->num_queries, q, k_cache, v_cache, block_table, desc->max_blocks, seq_lens, ws, &sp);
  if (desc->window < 0) return VEGAS_ERR_SHAPE;
  if (desc->window > 0 && collect) return VEGAS_ERR_UNSUPPORTED;   // banded layers are not sparsified: nothing to score
  sp.window = desc->window;
  const bool do_stream = stages == 0 || (stages & VEGAS_STAGE_STREAM);
  const bool do_merge = stages == 0 || (stages & VEGAS_STAGE_MERGE);
  if (do_stream) {
    const int hd = desc->head_dim;
    rc = !collect ? launch_split<true, 0>(pl, sp, desc->batch, st, hd)
                  : (logits ? launch_split<true, 2>(pl, sp, desc->batch, st, hd)
                            : launch_split<true, 1>(pl, sp, desc->batch, st, hd));
    if (rc != VEGAS_OK) return rc;
  }
  if (!do_merge) return VEGAS_OK;
  if (!collect) return launch_combine(desc, pl, sp, out, st);
  FinalizeParams fp;
  fp.part_o = sp.part_o;
  fp.part_ml = sp.part_ml;
  fp.page_lse = sp.page_lse;
  fp.lens = seq_lens;
  fp.out = static_cast<uint16_t*>(out);
  fp.block_scores = block_scores;
  fp.G = desc->num_queries; fp.g = sp.g; fp.R = pl.R; fp.Hq = sp.Hq; fp.Hkv = sp.Hkv;
  fp.chunk_tokens = pl.chunk; fp.nsplit = pl.nsplit; fp.max_tokens = desc->max_seq_len;
  fp.max_blocks = desc->max_blocks; fp.lse_pages = pl.lse_pages; fp.collect_rows = desc->collect_rows;
  fp.Rc = pl.Rc;
  fp.D = desc->head_dim;
  fp.plan = sp.plan;
  fp.slots_total = sp.slots_total;
  const int rows_per_wg = 256 / fp.D;                  // merge workgroups: 256 threads, D per row
  fp.nA = (sp.Hkv * pl.R + rows_per_wg - 1) / rows_per_wg;
  const int nrows = (desc->collect_rows == VEGAS_COLLECT_ALL_ROWS) ? desc->num_queries
                                                                   : (desc->num_queries > 1 ? 2 : 1);
  fp.inv_norm = 1.0f / (static_cast<float>(nrows) * static_cast<float>(desc->num_q_heads));
  // Every score workgroup (32 pages) rebuilds the row log-sum-exps from the (rows x chunks) table of
  // (max, sum) pairs; giving a workgroup more pages to amortise that was measured slower.
  const size_t hr = static_cast<size_t>(sp.Hkv) * pl.R;
  int nB = (desc->max_blocks + 31) / 32;
  size_t shm = (hr + 256 + 16 * hr) * sizeof(float);   // role B needs the most; role A fits inside
  fp.nC = 0;
  fp.tok_norm = 0.f;
  if (logits) {                                        // token sums instead of page scores: 1024 tokens per workgroup
    fp.nC = static_cast<int>((static_cast<int64_t>(desc->max_blocks) * kPage + 1023) / 1024);
    fp.tok_norm = desc->softmax_scale / (static_cast<float>(nrows) * static_cast<float>(desc->num_q_heads));
    nB = fp.nC;
    shm = 272 * sizeof(float);
  }
  if (shm > 160 * 1024) return VEGAS_ERR_UNSUPPORTED;
  const dim3 fgrid(fp.nA + nB, desc->batch);
  auto launch_finalize = [&](auto kern) -> int {
    if (int lrc = ensure_dynamic_lds(reinterpret_cast<const void*>(kern), shm)) return lrc;
    hipLaunchKernelGGL(kern, fgrid, dim3(256), shm, st, fp);
    return VEGAS_OK;
  };
  if (logits) {
    if (pl.nsplit <= 16) rc = launch_finalize(verify_finalize_kernel<16, 1>);
    else if (pl.nsplit <= 32) rc = launch_finalize(verify_finalize_kernel<32, 1>);
    else if (pl.nsplit <= 64) rc = launch_finalize(verify_finalize_kernel<64, 1>);
    else rc = launch_finalize(verify_finalize_kernel<0, 1>);
  } else {
    if (pl.nsplit <= 16) rc = launch_finalize(verify_finalize_kernel<16>);
    else if (pl.nsplit <= 32) rc = launch_finalize(verify_finalize_kernel<32>);
    else if (pl.nsplit <= 64) rc = launch_finalize(verify_finalize_kernel<64>);
    else rc = launch_finalize(verify_finalize_kernel<0>);
  }
  if (rc != VEGAS_OK) return rc;
  if (hipGetLastError() != hipSuccess) return VEGAS_ERR_LAUNCH;
  return VEGAS_OK;
}

int vegas_select_blocks(const vegas_desc* desc, const float* block_scores, const int32_t* block_table,
                        const int32_t* seq_lens, int32_t budget_tokens, const int32_t* budgets,
                        int32_t* sel_table, int32_t* sel_seq_lens, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  (void)workspace;
  (void)workspace_bytes;
  int rc = check_common(desc);
  if (rc == VEGAS_OK) rc = check_paged16(desc);
  if (rc != VEGAS_OK) return rc;
  if (!block_scores || !block_table || !seq_lens || !sel_table || !sel_seq_lens) return VEGAS_ERR_NULL;
  if (desc->num_queries <= 0 || desc->max_sel_blocks <= 0) return VEGAS_ERR_SHAPE;
  if (!budgets) {
    const int64_t bt = ratio_or_constant_budget(desc, budget_tokens);
    if (bt <= 0) return VEGAS_ERR_SHAPE;
    const int64_t max_pages = (static_cast<int64_t>(desc->max_seq_len) + kPage - 1) / kPage;
    int64_t kmax = (bt + kPage - 1) / kPage;
    const int64_t forced = (desc->num_queries + kPage - 2) / kPage + 1;   // pages G positions can touch
    if (kmax < forced) kmax = forced;
    if (kmax > max_pages) kmax = max_pages;
    if (desc->max_sel_blocks < kmax) return VEGAS_ERR_SHAPE;
  }
  SelectParams sp;
  sp.block_scores = block_scores;
  sp.block_table = block_table;
  sp.seq_lens = seq_lens;
  sp.budgets = budgets;
  sp.sel_table = sel_table;
  sp.sel_seq_lens = sel_seq_lens;
  sp.budget_tokens = budget_tokens;
  sp.G = desc->num_queries;
  sp.max_blocks = desc->max_blocks;
  sp.max_sel_blocks = desc->max_sel_blocks;
  sp.max_tokens = desc->max_seq_len;
  sp.budget_ratio = desc->budget_ratio;
  const int64_t max_pages = (static_cast<int64_t>(desc->max_seq_len) + kPage - 1) / kPage;
  sp.key_cap = static_cast<int32_t>(max_pages < kSelectKeyCap ? max_pages : kSelectKeyCap);
  const size_t shm = static_cast<size_t>(sp.key_cap) * sizeof(uint32_t);
  if (int rc = ensure_dynamic_lds(reinterpret_cast<const void*>(select_blocks_kernel), shm)) return rc;
  hipLaunchKernelGGL(select_blocks_kernel, dim3(desc->batch), dim3(kSelectThreads), shm,
                     static_cast<hipStream_t>(hip_stream), sp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

int vegas_select_tokens(const vegas_desc* desc, const float* token_scores, const int32_t* block_table,
                        const int32_t* seq_lens, int32_t budget_tokens, const int32_t* budgets,
                        int32_t* sel_table, int32_t* sel_seq_lens, void* workspace, size_t workspace_bytes,
                        void* hip_stream) {
  int rc = check_common(desc);
  if (rc == VEGAS_OK) rc = check_paged16(desc);
  if (rc != VEGAS_OK) return rc;
  if (!token_scores || !block_table || !seq_lens || !sel_table || !sel_seq_lens) return VEGAS_ERR_NULL;
  if (desc->num_queries <= 0 || desc->max_sel_blocks <= 0) return VEGAS_ERR_SHAPE;
  if (!budgets) {
    const int64_t bt = ratio_or_constant_budget(desc, budget_tokens);
    if (bt <= 0) return VEGAS_ERR_SHAPE;
    int64_t kmax = bt < desc->max_seq_len ? bt : desc->max_seq_len;
    const int64_t tail = desc->num_queries < desc->max_seq_len ? desc->num_queries : desc->max_seq_len;
    if (kmax < tail) kmax = tail;
    if (desc->max_sel_blocks < kmax) return VEGAS_ERR_SHAPE;
  }
  const size_t need = token_select_bytes(desc);
  if (!workspace || workspace_bytes < need) return VEGAS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return VEGAS_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  TokenSelectParams tp;
  tp.scores = token_scores;
  tp.block_table = block_table;
  tp.seq_lens = seq_lens;
  tp.budgets = budgets;
  tp.sel_table = sel_table;
  tp.sel_seq_lens = sel_seq_lens;
  tp.hist = reinterpret_cast<uint32_t*>(ws);
  tp.budget_tokens = budget_tokens;
  tp.G = desc->num_queries;
  tp.max_blocks = desc->max_blocks;
  tp.max_sel = desc->max_sel_blocks;
  tp.max_tokens = desc->max_seq_len;
  tp.slices = token_slices(desc);
  tp.budget_ratio = desc->budget_ratio;
  const dim3 grid(tp.slices, desc->batch);
  for (int pass = 0; pass < 4; ++pass)
    hipLaunchKernelGGL(token_select_hist, grid, dim3(kTokThreads), 0, st, tp, pass);
  hipLaunchKernelGGL(token_select_write, grid, dim3(kTokThreads), 0, st, tp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

static int append_impl(const vegas_desc* desc, const void* k_new, const void* v_new, int32_t num_new,
                       const int32_t* block_table, int32_t* seq_lens, void* k_cache, void* v_cache, int32_t* sel_table,
                       int32_t* sel_seq_lens, int32_t sel_page_size, void* hip_stream) {
  int rc = check_common(desc);
  if (rc == VEGAS_OK) rc = check_paged16(desc);
  if (rc != VEGAS_OK) return rc;
  if (!k_new || !v_new || !block_table || !seq_lens || !k_cache || !v_cache) return VEGAS_ERR_NULL;
  if (num_new <= 0 || num_new > 4096) return VEGAS_ERR_SHAPE;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_cache) || !aligned16(v_cache)) return VEGAS_ERR_ALIGN;
  AppendParams ap;
  ap.k_new = static_cast<const uint16_t*>(k_new);
  ap.v_new = static_cast<const uint16_t*>(v_new);
  ap.k_cache = static_cast<uint16_t*>(k_cache);
  ap.v_cache = static_cast<uint16_t*>(v_cache);
  ap.block_table = block_table;
  ap.seq_lens = seq_lens;
  ap.T = num_new;
  ap.Hkv = desc->num_kv_heads;
  ap.D = desc->head_dim;
  ap.max_blocks = desc->max_blocks;
  ap.max_tokens = desc->max_seq_len;
  ap.page_stride = desc->kv_page_stride;
  ap.token_stride = desc->kv_token_stride;
  ap.head_stride = desc->kv_head_stride;
  ap.num_pages = desc->num_pages;
  ap.grow.block_table = block_table;
  ap.grow.seq_lens = seq_lens;
  ap.grow.sel_table = sel_table;
  ap.grow.sel_seq_lens = sel_seq_lens;
  ap.grow.batch = desc->batch;
  ap.grow.num_new = num_new;
  ap.grow.max_blocks = desc->max_blocks;
  ap.grow.max_sel_blocks = desc->max_sel_blocks;
  ap.grow.page_size = sel_page_size;
  hipLaunchKernelGGL(append_kv_kernel, dim3(desc->batch), dim3(256), 0, static_cast<hipStream_t>(hip_stream), ap);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

int vegas_append_kv(const vegas_desc* desc, const void* k_new, const void* v_new, int32_t num_new,
                    const int32_t* block_table, int32_t* seq_lens, void* k_cache, void* v_cache, void* hip_stream) {
  return append_impl(desc, k_new, v_new, num_new, block_table, seq_lens, k_cache, v_cache, nullptr, nullptr, kPage,
                     hip_stream);
}

int vegas_append_kv_extend(const vegas_desc* desc, const void* k_new, const void* v_new, int32_t num_new,
                           const int32_t* block_table, int32_t* seq_lens, void* k_cache, void* v_cache,
                           int32_t* sel_table, int32_t* sel_seq_lens, int32_t sel_page_size, void* hip_stream) {
  if (!sel_table || !sel_seq_lens) return VEGAS_ERR_NULL;
  if (sel_page_size != kPage && sel_page_size != 1) return VEGAS_ERR_UNSUPPORTED;
  if (!desc || desc->max_sel_blocks <= 0) return desc ? VEGAS_ERR_SHAPE : VEGAS_ERR_NULL;
  return append_impl(desc, k_new, v_new, num_new, block_table, seq_lens, k_cache, v_cache, sel_table, sel_seq_lens,
                     sel_page_size, hip_stream);
}

int vegas_extend_selection(const vegas_desc* desc, const int32_t* block_table, const int32_t* seq_lens,
                           int32_t num_new, int32_t* sel_table, int32_t* sel_seq_lens, void* hip_stream) {
  int rc = check_common(desc);
  if (rc != VEGAS_OK) return rc;
  if (desc->page_size != kPage && desc->page_size != 1) return VEGAS_ERR_UNSUPPORTED;
  if (!block_table || !seq_lens || !sel_table || !sel_seq_lens) return VEGAS_ERR_NULL;
  if (num_new <= 0 || desc->max_sel_blocks <= 0) return VEGAS_ERR_SHAPE;
  ExtendParams ep;
  ep.block_table = block_table;
  ep.seq_lens = seq_lens;
  ep.sel_table = sel_table;
  ep.sel_seq_lens = sel_seq_lens;
  ep.batch = desc->batch;
  ep.num_new = num_new;
  ep.max_blocks = desc->max_blocks;
  ep.max_sel_blocks = desc->max_sel_blocks;
  ep.page_size = desc->page_size;
  hipLaunchKernelGGL(extend_selection_kernel, dim3((desc->batch + 63) / 64), dim3(64), 0,
                     static_cast<hipStream_t>(hip_stream), ep);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

static int draft_impl(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                      const int32_t* sel_table, const int32_t* sel_seq_lens, void* out, void* workspace,
                      size_t workspace_bytes, void* hip_stream, int32_t stages) {
  if (stages < 0 || stages > (VEGAS_STAGE_STREAM | VEGAS_STAGE_MERGE)) return VEGAS_ERR_SHAPE;
  int rc = check_common(desc);
  if (rc != VEGAS_OK) return rc;
  if (!q || !k_cache || !v_cache || !sel_table || !sel_seq_lens || !out) return VEGAS_ERR_NULL;
  if (desc->max_sel_blocks <= 0) return VEGAS_ERR_SHAPE;
  if (static_cast<int64_t>(desc->max_seq_len) > static_cast<int64_t>(desc->max_sel_blocks) * desc->page_size)
    return VEGAS_ERR_SHAPE;
  SplitPlan pl;
  rc = plan_draft(desc, &pl);
  if (rc != VEGAS_OK) return rc;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out) || !aligned16(sel_table))
    return VEGAS_ERR_ALIGN;
  if (!workspace || workspace_bytes < pl.total) return VEGAS_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return VEGAS_ERR_ALIGN;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  SplitParams sp;
  fill_split_params(desc, pl, 1, q, k_cache, v_cache, sel_table, desc->max_sel_blocks, sel_seq_lens, ws, &sp);
  // One chunk per (sequence, KV head): the streaming kernel finishes the rows itself and no merge kernel is launched.
  const bool direct = pl.nsplit == 1;
  if (direct) sp.out_direct = static_cast<uint16_t*>(out);
  if (stages == 0 || (stages & VEGAS_STAGE_STREAM)) {
    rc = launch_split<false, 0>(pl, sp, desc->batch, st, desc->head_dim, desc->page_size);
    if (rc != VEGAS_OK) return rc;
  }
  if (direct || (stages != 0 && !(stages & VEGAS_STAGE_MERGE))) return VEGAS_OK;
  return launch_combine(desc, pl, sp, out, st);
}

int vegas_verify_attention(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                           const int32_t* block_table, const int32_t* seq_lens, void* out, float* block_scores,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  return verify_impl(desc, q, k_cache, v_cache, block_table, seq_lens, out, block_scores, workspace, workspace_bytes,
                     hip_stream, 0);
}

int vegas_draft_attention(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* sel_table, const int32_t* sel_seq_lens, void* out, void* workspace,
                          size_t workspace_bytes, void* hip_stream) {
  return draft_impl(desc, q, k_cache, v_cache, sel_table, sel_seq_lens, out, workspace, workspace_bytes, hip_stream, 0);
}

int vegas_draft_attention_static(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                 const int32_t* sel_table, const int32_t* sel_seq_lens, void* out, void* hip_stream) {
  const int rc = check_common(desc);
  if (rc != VEGAS_OK) return rc;
  SplitPlan pl;
  if (int prc = plan_draft(desc, &pl)) return prc;
  if (pl.total > kStaticScratchBytes) return VEGAS_ERR_WORKSPACE;      // the call needs more than the built-in scratch
  void* ptr = nullptr;
  if (int src = static_scratch_address(&ptr)) return src;
  return draft_impl(desc, q, k_cache, v_cache, sel_table, sel_seq_lens, out, ptr, kStaticScratchBytes, hip_stream, 0);
}

int vegas_debug_verify_attention_stages(const vegas_desc* desc, const void* q, const void* k_cache,
                                        const void* v_cache, const int32_t* block_table, const int32_t* seq_lens,
                                        void* out, float* block_scores, void* workspace, size_t workspace_bytes,
                                        void* hip_stream, int32_t stages) {
  return verify_impl(desc, q, k_cache, v_cache, block_table, seq_lens, out, block_scores, workspace, workspace_bytes,
                     hip_stream, stages);
}

int vegas_debug_draft_attention_stages(const vegas_desc* desc, const void* q, const void* k_cache, const void* v_cache,
                                       const int32_t* sel_table, const int32_t* sel_seq_lens, void* out,
                                       void* workspace, size_t workspace_bytes, void* hip_stream, int32_t stages) {
  return draft_impl(desc, q, k_cache, v_cache, sel_table, sel_seq_lens, out, workspace, workspace_bytes, hip_stream,
                    stages);
}

int vegas_debug_stream_read(const void* a, const void* b, size_t bytes_each, int32_t workgroups, int32_t non_temporal,
                            void* sink, void* hip_stream) {
  if (!a || !b || !sink) return VEGAS_ERR_NULL;
  if (bytes_each < 16 || (bytes_each % 16) != 0 || workgroups <= 0 || workgroups > (1 << 20)) return VEGAS_ERR_SHAPE;
  if (!aligned16(a) || !aligned16(b) || !aligned16(sink)) return VEGAS_ERR_ALIGN;
  StreamReadParams rp;
  rp.a = static_cast<const u32x4*>(a);
  rp.b = static_cast<const u32x4*>(b);
  rp.vecs = bytes_each / 16;
  rp.sink = static_cast<uint32_t*>(sink);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (non_temporal) hipLaunchKernelGGL(stream_read_kernel<true>, dim3(workgroups), dim3(256), 0, st, rp);
  else hipLaunchKernelGGL(stream_read_kernel<false>, dim3(workgroups), dim3(256), 0, st, rp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

int vegas_debug_check_tables(const vegas_desc* desc, int32_t which, const int32_t* table, const int32_t* lens,
                             int32_t* error_word, void* hip_stream) {
  const int rc = check_common(desc);
  if (rc != VEGAS_OK) return rc;
  if (!table || !lens || !error_word) return VEGAS_ERR_NULL;
  if (which != VEGAS_TABLE_BLOCKS && which != VEGAS_TABLE_SELECTION) return VEGAS_ERR_SHAPE;
  CheckParams cp;
  cp.table = table;
  cp.lens = lens;
  cp.error_word = error_word;
  cp.batch = desc->batch;
  cp.max_tokens = desc->max_seq_len;
  cp.num_pages = desc->num_pages;
  if (which == VEGAS_TABLE_BLOCKS) {
    cp.stride = desc->max_blocks;
    cp.page_size = kPage;
    cp.num_queries = desc->num_queries;
  } else {
    if (desc->max_sel_blocks <= 0) return VEGAS_ERR_SHAPE;
    cp.stride = desc->max_sel_blocks;
    cp.page_size = desc->page_size;
    cp.num_queries = 0;
  }
  hipLaunchKernelGGL(check_tables_kernel, dim3(desc->batch), dim3(256), 0, static_cast<hipStream_t>(hip_stream), cp);
  return hipGetLastError() == hipSuccess ? VEGAS_OK : VEGAS_ERR_LAUNCH;
}

int vegas_debug_set_timeline(void* buffer, size_t bytes) {
#ifdef VEGAS_TIMELINE
  g_timeline = static_cast<unsigned long long*>(buffer);
  g_timeline_bytes = buffer ? bytes : 0;
  return VEGAS_OK;
#else
  (void)buffer;
  (void)bytes;
  return VEGAS_ERR_UNSUPPORTED;
#endif
}

const char* vegas_strerror(int status) {
  switch (status) {
    case VEGAS_OK: return "ok";
    case VEGAS_ERR_NULL: return "a required pointer is NULL";
    case VEGAS_ERR_SHAPE: return "a size is non-positive or inconsistent";
    case VEGAS_ERR_UNSUPPORTED:
      return "shape not supported by this build (head_dim 128 or 64; page_size 16, in draft calls also 1, 2, 4, 8; "
             "<= 128 rows per KV head; max_seq_len <= 2^30; batch <= 65535)";
    case VEGAS_ERR_ALIGN: return "pointer or stride alignment";
    case VEGAS_ERR_WORKSPACE: return "workspace missing or too small";
    case VEGAS_ERR_LAUNCH: return "the HIP runtime refused a kernel launch";
    default: return "unknown status";
  }
}

}  // extern "C"
