// Merge of the per-chunk partial results, and the page-criticality finalisation.
#pragma once
#include "vegas_common.hpp"

namespace vegas {

// One workgroup of 128 threads (= head dims) per (query row, KV head, sequence): merges the
// chunk partials of that row with the usual max/sum bookkeeping (all in log2 units), writes the
// bf16 output row (Eq. 1) and the row's global log2-sum-exp2.  The per-chunk (max, sum) pairs are
// fetched by one thread each, so the whole merge costs two dependent memory round trips.
__global__ __launch_bounds__(128) void attn_combine_kernel(const CombineParams p) {
  __shared__ float sw[128];
  __shared__ float sred[4];
  const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int ns = (n + p.chunk_tokens - 1) / p.chunk_tokens;
  const int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit;
  const float2* ml = p.part_ml + pbase * p.R + r;                 // stride R between chunks
  const float* po = p.part_o + (pbase * p.R + r) * kHeadDim + tid; // stride R*128 between chunks
  const int64_t ostride = static_cast<int64_t>(p.R) * kHeadDim;

  // pass 1: global max over chunks
  float m = -INFINITY;
  for (int s = tid; s < ns; s += 128) m = fmaxf(m, ml[static_cast<int64_t>(s) * p.R].x);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((tid & 63) == 0) sred[wave] = m;
  __syncthreads();
  m = fmaxf(sred[0], sred[1]);
  const float m_use = (m == -INFINITY) ? 0.f : m;

  // pass 2: weights of up to 128 chunks at a time, then the weighted sum of the partial rows
  float accv = 0.f, L = 0.f;
  for (int s0 = 0; s0 < ns; s0 += 128) {
    const int cnt = min(128, ns - s0);
    float wl = 0.f;
    if (tid < cnt) {
      const float2 v = ml[static_cast<int64_t>(s0 + tid) * p.R];
      const float w = fast_exp2(v.x - m_use);
      sw[tid] = w;
      wl = w * v.y;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) wl += __shfl_xor(wl, off, 64);
    if ((tid & 63) == 0) sred[2 + wave] = wl;
    __syncthreads();
    L += sred[2] + sred[3];
    int s = 0;
    for (; s + 4 <= cnt; s += 4) {
      const float x0 = po[(s0 + s) * ostride], x1 = po[(s0 + s + 1) * ostride];
      const float x2 = po[(s0 + s + 2) * ostride], x3 = po[(s0 + s + 3) * ostride];
      accv += sw[s] * x0 + sw[s + 1] * x1 + sw[s + 2] * x2 + sw[s + 3] * x3;
    }
    for (; s < cnt; ++s) accv += sw[s] * po[(s0 + s) * ostride];
    __syncthreads();
  }
  const float o = (L > 0.f) ? accv / L : 0.f;
  const int t = r / p.g, j = r % p.g;
  p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * kHeadDim + tid] = float_to_bf16_bits(o);
  if (p.row_lse != nullptr && tid == 0)
    p.row_lse[(static_cast<int64_t>(b) * p.Hkv + h) * p.R + r] = (L > 0.f) ? m_use + fast_log2(L) : -INFINITY;
}

// Page criticality (Eq. 2 / Eq. 3 with weights, averaged over rows and heads as in the last
// paragraph of Sec. 3.3): score[b][j] = inv_norm * sum_h sum_{rows in R} 2^(page_lse - row_lse).
// A workgroup of 256 threads covers 64 pages: lane = page, the 4 waves split the KV heads; a thread
// walks the R values of its (head, page) -- neighbouring lanes read neighbouring R-float pieces, so
// every fetched line is used in full -- and the waves' sums meet in LDS.  Pages at or beyond the
// sequence's page count are written as 0.
__global__ __launch_bounds__(256) void block_score_kernel(const ScoreParams p) {
  extern __shared__ float sm_row[];           // [Hkv * R] global row lse (-inf: row not collected), then [4][64] sums
  const int b = blockIdx.y;
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int nblk = (n + kPage - 1) / kPage;
  const int HR = p.Hkv * p.R;
  float* sm_sum = sm_row + HR;
  for (int i = threadIdx.x; i < HR; i += blockDim.x) {
    const int t = (i % p.R) / p.g;
    const bool use = (p.collect_rows == 1) || (t == 0) || (t == p.G - 1);
    sm_row[i] = use ? p.row_lse[static_cast<int64_t>(b) * HR + i] : -INFINITY;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + lane;
  float s = 0.f;
  if (j < nblk) {
    for (int h = wave; h < p.Hkv; h += 4) {
      const float* pl = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + j) * p.R;
      const float* rl = sm_row + h * p.R;
      for (int r = 0; r < p.R; ++r) {
        const float x = rl[r];
        if (x != -INFINITY) s += fast_exp2(pl[r] - x);
      }
    }
  }
  sm_sum[wave * 64 + lane] = s;
  __syncthreads();
  if (wave == 0 && j < p.max_blocks) {
    const float tot = (sm_sum[lane] + sm_sum[64 + lane]) + (sm_sum[128 + lane] + sm_sum[192 + lane]);
    p.block_scores[static_cast<int64_t>(b) * p.max_blocks + j] = (j < nblk) ? tot * p.inv_norm : 0.f;
  }
}

}  // namespace vegas
