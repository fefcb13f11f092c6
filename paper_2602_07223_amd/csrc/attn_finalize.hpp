// Merge of the per-chunk partial results, and the page-criticality finalisation.
#pragma once
#include "vegas_common.hpp"

namespace vegas {

// One workgroup of 128 threads (= head dims) per (query row, KV head, sequence): merges the
// chunk partials of that row with the usual max/sum bookkeeping (all in log2 units), writes the
// bf16 output row (Eq. 1).  The per-chunk (max, sum) pairs are
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
}

// Verification epilogue in ONE launch (a kernel boundary costs ~3 us on this GPU): workgroups
// [0, nA) merge the chunk partials of two query rows each (as attn_combine_kernel does) and write
// the bf16 output rows (Eq. 1); workgroups [nA, nA + nB) turn the per-(row, page) log-sum-exps of
// page_groups x 32 pages into page criticalities (Eq. 2 / Eq. 3 with weights, averaged over rows and heads as in the
// last paragraph of Sec. 3.3): score[b][j] = inv_norm * sum_h sum_{rows in R} 2^(page_lse - row_lse).
// A score workgroup derives the global row log-sum-exps itself from the chunks' (max, sum) pairs,
// so it does not depend on the merge workgroups.  Pages at or beyond the sequence's page count get 0.
__global__ __launch_bounds__(256) void verify_finalize_kernel(const FinalizeParams p) {
  extern __shared__ float smf[];              // role A: [2][128] weights + [2][4]; role B: [Hkv*R] + [8][32] + [Hkv*R][8] pairs
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int ns = (n + p.chunk_tokens - 1) / p.chunk_tokens;
  const int HR = p.Hkv * p.R;

  if (static_cast<int>(blockIdx.x) < p.nA) {
    // ---- role A: rows 2*bx and 2*bx+1 of the Hkv*R rows, 128 threads (= head dims) each
    const int sub = tid >> 7, t128 = tid & 127, wv = (tid >> 6) & 1;
    float* sw = smf + sub * 128;
    float* sred = smf + 256 + sub * 4;
    const int rr_raw = 2 * blockIdx.x + sub;
    const bool valid = rr_raw < HR;
    const int rr = valid ? rr_raw : HR - 1;
    const int h = rr / p.R, r = rr % p.R;
    const int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit;
    const float2* ml = p.part_ml + pbase * p.R + r;
    const float* po = p.part_o + (pbase * p.R + r) * kHeadDim + t128;
    const int64_t ostride = static_cast<int64_t>(p.R) * kHeadDim;
    float m = -INFINITY;
    for (int s = t128; s < ns; s += 128) m = fmaxf(m, ml[static_cast<int64_t>(s) * p.R].x);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if ((tid & 63) == 0) sred[wv] = m;
    __syncthreads();
    m = fmaxf(sred[0], sred[1]);
    const float m_use = (m == -INFINITY) ? 0.f : m;
    float accv = 0.f, L = 0.f;
    for (int s0 = 0; s0 < ns; s0 += 128) {
      const int cnt = min(128, ns - s0);
      float wl = 0.f;
      if (t128 < cnt) {
        const float2 v = ml[static_cast<int64_t>(s0 + t128) * p.R];
        const float w = fast_exp2(v.x - m_use);
        sw[t128] = w;
        wl = w * v.y;
      }
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) wl += __shfl_xor(wl, off, 64);
      if ((tid & 63) == 0) sred[2 + wv] = wl;
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
    if (valid) {
      const float o = (L > 0.f) ? accv / L : 0.f;
      const int t = r / p.g, j = r % p.g;
      p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * kHeadDim + t128] = float_to_bf16_bits(o);
    }
    return;
  }

  // ---- role B: 32 pages; thread = (page, head slot)
  const int nblk = (n + kPage - 1) / kPage;
  const int pg = tid & 31, slot = tid >> 5;
  const int jbase = (blockIdx.x - p.nA) * 32 * p.page_groups;       // page_groups x 32 pages per workgroup
  float* out_row = p.block_scores + static_cast<int64_t>(b) * p.max_blocks;
  if (jbase >= nblk) {                                             // whole workgroup past the sequence
    for (int j = jbase + tid; j < jbase + 32 * p.page_groups && j < p.max_blocks; j += 256) out_row[j] = 0.f;
    return;
  }
  float* sm_row = smf;                        // [HR] global row lse; -inf for rows that do not count
  float* sm_sum = smf + HR;                   // [8][32]
  float2* sm_pair = reinterpret_cast<float2*>(smf + HR + 256);   // [HR][8] (max, sum) of a row over 1/8 of the chunks
  // Each (row, eighth of the chunks) pair is one unit of work.  A thread first issues the (max, sum)
  // loads of four units (up to 16 independent loads), then merges them, so the whole table costs
  // about one memory round trip instead of one per chunk.
  for (int s0 = 0; s0 < ns; s0 += 32) {
    for (int u0 = tid; u0 < HR * 8; u0 += 4 * 256) {
      float2 v[4][4];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int u = u0 + 256 * a;
        const bool uv = u < HR * 8;
        const int i = uv ? (u >> 3) : 0, sg = u & 7;
        const int h = i / p.R, r = i % p.R;
        const float2* ml = p.part_ml + (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit * p.R + r;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int sidx = s0 + sg + 8 * q;
          v[a][q] = (uv && sidx < ns) ? ml[static_cast<int64_t>(sidx) * p.R] : make_float2(-INFINITY, 0.f);
        }
      }
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int u = u0 + 256 * a;
        if (u < HR * 8) {
          float2 cur = (s0 == 0) ? make_float2(-INFINITY, 0.f) : sm_pair[u];
          float m = cur.x;
#pragma unroll
          for (int q = 0; q < 4; ++q) m = fmaxf(m, v[a][q].x);
          const float mu = (m == -INFINITY) ? 0.f : m;
          float L = cur.y * fast_exp2(cur.x - mu);
#pragma unroll
          for (int q = 0; q < 4; ++q) L += v[a][q].y * fast_exp2(v[a][q].x - mu);
          sm_pair[u] = make_float2(m, L);
        }
      }
    }
  }
  __syncthreads();
  for (int i = tid; i < HR; i += 256) {
    const int t = (i % p.R) / p.g;
    const bool use = (p.collect_rows == 1) || (t == 0) || (t == p.G - 1);
    float m = -INFINITY;
#pragma unroll
    for (int q = 0; q < 8; ++q) m = fmaxf(m, sm_pair[i * 8 + q].x);
    const float m_use = (m == -INFINITY) ? 0.f : m;
    float L = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float2 v = sm_pair[i * 8 + q];
      L += fast_exp2(v.x - m_use) * v.y;
    }
    sm_row[i] = (use && L > 0.f) ? m_use + fast_log2(L) : -INFINITY;
  }
  __syncthreads();
  for (int grp = 0; grp < p.page_groups; ++grp) {
    const int j = jbase + grp * 32 + pg;
    float sc = 0.f;
    if (j < nblk) {
      for (int h = slot; h < p.Hkv; h += 8) {
        const float* pl = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + j) * p.R;
        const float* rl = sm_row + h * p.R;
        if ((p.R & 3) == 0) {
          for (int r = 0; r < p.R; r += 4) {
            const f32x4 x = *reinterpret_cast<const f32x4*>(pl + r);
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (rl[r + q] != -INFINITY) sc += fast_exp2(x[q] - rl[r + q]);
          }
        } else {
          for (int r = 0; r < p.R; ++r)
            if (rl[r] != -INFINITY) sc += fast_exp2(pl[r] - rl[r]);
        }
      }
    }
    sm_sum[slot * 32 + pg] = sc;
    __syncthreads();
    if (slot == 0 && j < p.max_blocks) {
      float tot = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) tot += sm_sum[q * 32 + pg];
      out_row[j] = (j < nblk) ? tot * p.inv_norm : 0.f;
    }
    __syncthreads();
  }
}

}  // namespace vegas
