// Measurement aids that are not part of the method: a plain streaming read of two buffers, the yardstick the
// KV-streaming kernels are held against (what the memory system delivers to a kernel that does nothing else).
#pragma once
#include "vegas_common.hpp"

namespace vegas {

struct StreamReadParams {
  const u32x4* a;          // two buffers of `vecs` 16-byte vectors each (a K cache and a V cache, say)
  const u32x4* b;
  uint64_t vecs;
  uint32_t* sink;          // [workgroups * 256]: what keeps the loads alive
};

// Every workgroup reads one contiguous slice of each buffer: 256 threads x 16 bytes per instruction (4 KB, fully
// coalesced), eight instructions per buffer in flight per thread (64 KB per workgroup and buffer), the shape of the
// streaming kernels' K loads.  Indices past the end are clamped to the last vector (re-read, never out of bounds).
template <bool NT>
__global__ __launch_bounds__(256) void stream_read_kernel(const StreamReadParams p) {
  constexpr uint64_t kStep = 256 * 8;
  const uint64_t per_wg = (p.vecs + gridDim.x - 1) / gridDim.x;
  const uint64_t span = (per_wg + kStep - 1) / kStep * kStep;
  const uint64_t begin = static_cast<uint64_t>(blockIdx.x) * span;
  const uint64_t end = begin + span < p.vecs ? begin + span : p.vecs;
  const uint64_t last = p.vecs - 1;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (uint64_t i = begin + threadIdx.x; i < end; i += kStep) {
    u32x4 x[8], y[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint64_t j = i + 256u * u < last ? i + 256u * u : last;
      if constexpr (NT) {
        x[u] = __builtin_nontemporal_load(p.a + j);
        y[u] = __builtin_nontemporal_load(p.b + j);
      } else {
        x[u] = p.a[j];
        y[u] = p.b[j];
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= x[u] ^ y[u];
  }
  p.sink[blockIdx.x * 256 + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

// Validation of the data-dependent inputs the calls otherwise clamp silently: lengths and page ids.
struct CheckParams {
  const int32_t* table;     // [B, stride] page ids
  const int32_t* lens;      // [B]
  int32_t* error_word;      // bits are OR-ed in, never cleared
  int32_t batch, stride, page_size, max_tokens, num_queries;
  int64_t num_pages;
};
constexpr int kCheckLengthRange = 1, kCheckLengthExceedsTable = 2, kCheckPageId = 4, kCheckShorterThanQueries = 8;

// One workgroup per sequence: its length against the descriptor's bounds, and every page id the length makes the
// calls read against the pool.
__global__ __launch_bounds__(256) void check_tables_kernel(const CheckParams p) {
  const int b = blockIdx.x;
  const int n = p.lens[b];
  int bits = 0;
  if (n < 0 || n > p.max_tokens) bits |= kCheckLengthRange;
  const int64_t cap = static_cast<int64_t>(p.stride) * p.page_size;
  if (n > cap) bits |= kCheckLengthExceedsTable;
  if (p.num_queries > 0 && n > 0 && n < p.num_queries) bits |= kCheckShorterThanQueries;
  const int64_t nn = n < 0 ? 0 : (n > cap ? cap : n);
  const int pages = static_cast<int>((nn + p.page_size - 1) / p.page_size);
  const int32_t* row = p.table + static_cast<int64_t>(b) * p.stride;
  for (int j = threadIdx.x; j < pages; j += 256) {
    const int64_t id = row[j];
    if (id < 0 || id >= p.num_pages) bits |= kCheckPageId;
  }
  if (bits) atomicOr(p.error_word, bits);
}

}  // namespace vegas
