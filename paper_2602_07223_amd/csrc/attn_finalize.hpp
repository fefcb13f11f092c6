// Merge of the per-chunk partial results, and the page-criticality finalisation.
#pragma once
#include "vegas_common.hpp"

namespace vegas {

// One workgroup of 128 threads (= head dims) per (query row, KV head, sequence): merges the
// chunk partials of that row with the usual max/sum bookkeeping (all in log2 units), writes the
// bf16 output row (Eq. 1) and the row's global log2-sum-exp2.
__global__ __launch_bounds__(128) void attn_combine_kernel(const CombineParams p) {
  const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int d = threadIdx.x;
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int ns = (n + p.chunk_tokens - 1) / p.chunk_tokens;
  const int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit;
  float m = -INFINITY;
  for (int s = 0; s < ns; ++s) m = fmaxf(m, p.part_ml[(pbase + s) * p.R + r].x);
  const float m_use = (m == -INFINITY) ? 0.f : m;
  float accv = 0.f, L = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float2 ml = p.part_ml[(pbase + s) * p.R + r];
    const float w = fast_exp2(ml.x - m_use);
    L += w * ml.y;
    accv += w * p.part_o[((pbase + s) * p.R + r) * kHeadDim + d];
  }
  const float o = (L > 0.f) ? accv / L : 0.f;
  const int t = r / p.g, j = r % p.g;
  p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * kHeadDim + d] = float_to_bf16_bits(o);
  if (p.row_lse != nullptr && d == 0)
    p.row_lse[(static_cast<int64_t>(b) * p.Hkv + h) * p.R + r] = (L > 0.f) ? m_use + fast_log2(L) : -INFINITY;
}

// Page criticality (Eq. 2 / Eq. 3 with weights, averaged over rows and heads as in the last
// paragraph of Sec. 3.3): score[b][j] = inv_norm * sum_h sum_{rows in R} 2^(page_lse - row_lse).
// One wave per page: the Hkv*R values of a page are contiguous, lanes stride over them and a
// wave reduction adds them up.  Pages at or beyond the sequence's page count are written as 0.
__global__ __launch_bounds__(256) void block_score_kernel(const ScoreParams p) {
  extern __shared__ float sm_row[];           // [Hkv * R] global row lse; -inf for rows not collected
  const int b = blockIdx.y;
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int nblk = (n + kPage - 1) / kPage;
  const int HR = p.Hkv * p.R;
  for (int i = threadIdx.x; i < HR; i += blockDim.x) {
    const int t = (i % p.R) / p.g;
    const bool use = (p.collect_rows == 1) || (t == 0) || (t == p.G - 1);
    sm_row[i] = use ? p.row_lse[static_cast<int64_t>(b) * HR + i] : -INFINITY;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int j = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (j >= p.max_blocks) return;
  float s = 0.f;
  if (j < nblk) {
    const float* pl = p.page_lse + (static_cast<int64_t>(b) * p.lse_pages + j) * HR;
    for (int i = lane; i < HR; i += 64) {
      const float rl = sm_row[i];
      if (rl != -INFINITY) s += fast_exp2(pl[i] - rl);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    s *= p.inv_norm;
  }
  if (lane == 0) p.block_scores[static_cast<int64_t>(b) * p.max_blocks + j] = s;
}

}  // namespace vegas
