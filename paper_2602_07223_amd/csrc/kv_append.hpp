// Appending freshly computed K/V rows to the paged cache: the step between two draft calls.
//
// Drafting produces one token per step (Sec. 2.3); its K and V must be in the cache before the next draft step
// attends, and everything after the sparsified prefix is kept (Sec. 3.2, last sentence), so the selection grows
// with the sequence (vegas_extend_selection).  Token t of sequence b goes to position n_b + t: page
// block_table[b][(n_b + t) / 16], slot (n_b + t) % 16, every KV head (App. D's [page, slot, KV head, dim] layout
// with the descriptor's strides).  The lengths live on the device, so the kernel also advances them.
#pragma once
#include "select_blocks.hpp"
#include "vegas_common.hpp"

namespace vegas {

struct AppendParams {
  const uint16_t* k_new;    // bf16 [B, T, Hkv, D]
  const uint16_t* v_new;
  uint16_t* k_cache;
  uint16_t* v_cache;
  const int32_t* block_table;   // [B, max_blocks]
  int32_t* seq_lens;            // [B], advanced by T
  int32_t T, Hkv, D, max_blocks, max_tokens;
  int64_t page_stride, token_stride, head_stride, num_pages;
  ExtendParams grow;            // sel_table != nullptr: the selection grows by the same tokens in the same launch
};

// One workgroup per sequence.  A thread moves 16 bytes: (token, K or V, KV head, 16-byte piece of the head's row).
// The length is read by every thread before anybody advances it (a barrier separates the two).  A sequence without
// room for T more tokens (its table row, or the descriptor's bound) is left alone: nothing written, length kept.
// With a selection to grow (vegas_append_kv_extend), the sequence's first thread then does what
// extend_selection_kernel does for the advanced length -- one launch per draft step instead of two; a sequence
// whose append was refused keeps its selection as it is.
__global__ __launch_bounds__(256) void append_kv_kernel(const AppendParams p) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int n = p.seq_lens[b];
  __syncthreads();
  const int64_t cap = min(static_cast<int64_t>(p.max_blocks) * kPage, static_cast<int64_t>(p.max_tokens));
  if (n < 0 || static_cast<int64_t>(n) + p.T > cap) return;
  const int pieces = p.D / 8;                          // 16-byte pieces of one head's row
  const int per_token = 2 * p.Hkv * pieces;            // K and V
  const int32_t* table = p.block_table + static_cast<int64_t>(b) * p.max_blocks;
  for (int e = tid; e < p.T * per_token; e += 256) {
    const int t = e / per_token, r = e % per_token;
    const int which = r / (p.Hkv * pieces), hr = r % (p.Hkv * pieces);
    const int h = hr / pieces, piece = hr % pieces;
    const int pos = n + t;
    int64_t page = table[pos / kPage];
    page = page < 0 ? 0 : (page >= p.num_pages ? p.num_pages - 1 : page);   // a corrupt table cannot fault
    const int64_t src = ((static_cast<int64_t>(b) * p.T + t) * p.Hkv + h) * p.D + piece * 8;
    const int64_t dst = page * p.page_stride + static_cast<int64_t>(pos % kPage) * p.token_stride +
                        static_cast<int64_t>(h) * p.head_stride + piece * 8;
    const u32x4 v = *reinterpret_cast<const u32x4*>((which ? p.v_new : p.k_new) + src);
    *reinterpret_cast<u32x4*>((which ? p.v_cache : p.k_cache) + dst) = v;
  }
  if (tid == 0) {
    p.seq_lens[b] = n + p.T;
    if (p.grow.sel_table != nullptr) extend_selection_row(p.grow, b, n + p.T);
  }
}

}  // namespace vegas
