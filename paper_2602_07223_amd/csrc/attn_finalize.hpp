// Merge of the per-chunk partial results, and the page-criticality finalisation.
#pragma once
#include "vegas_common.hpp"

namespace vegas {

// One workgroup of D threads (= head dims; 128 or 64) per (query row, KV head, sequence): merges the
// chunk partials of that row with the usual max/sum bookkeeping (all in log2 units), writes the
// bf16 output row (Eq. 1).  The per-chunk (max, sum) pairs are
// fetched by one thread each, so the whole merge costs two dependent memory round trips.
__global__ __launch_bounds__(128) void attn_combine_kernel(const CombineParams p) {
  __shared__ float sw[128];
  __shared__ float sred[4];
  const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int T = p.D;                                              // threads of this workgroup = head dims
  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const ColumnSlots cs = column_slots(p.plan, p.slots_total, b, p.Hkv, p.nsplit, p.chunk_tokens);
  const int ns = (n + cs.chunk - 1) / cs.chunk;
  const int64_t pbase = cs.off + static_cast<int64_t>(h) * cs.stride_h;
  const float2* ml = p.part_ml + pbase * p.R + r;                 // stride R between chunks
  const float* po = p.part_o + (pbase * p.R + r) * T + tid;       // stride R*D between chunks
  const int64_t ostride = static_cast<int64_t>(p.R) * T;

  const int s_lo = first_live_chunk(n, p.G, p.window, cs.chunk);   // earlier chunks were skipped (local masking)
  // pass 1: global max over chunks
  float m = -INFINITY;
  for (int s = s_lo + tid; s < ns; s += T) m = fmaxf(m, ml[static_cast<int64_t>(s) * p.R].x);
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((tid & 63) == 0) sred[wave] = m;
  __syncthreads();
  m = T > 64 ? fmaxf(sred[0], sred[1]) : sred[0];
  const float m_use = (m == -INFINITY) ? 0.f : m;

  // pass 2: weights of up to D chunks at a time, then the weighted sum of the partial rows
  float accv = 0.f, L = 0.f;
  for (int s0 = s_lo; s0 < ns; s0 += T) {
    const int cnt = min(T, ns - s0);
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
    L += T > 64 ? sred[2] + sred[3] : sred[2];
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
  p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * T + tid] = float_to_bf16_bits(o);
}

// The same merge for at most MAXS (<= 64) chunks, in ONE memory round trip: the sequence length, the
// chunks' (max, sum) pairs (lane s of every wave fetches chunk s) and the thread's element of every
// chunk's partial row are all requested before any of them is used.  Chunks at or past the end of the
// sequence were never written; their slots are loaded all the same (the workspace holds nsplit of them)
// and then discarded.  Addresses are a scalar base plus a 32-bit offset: the kernel is so short that
// 64-bit address arithmetic per load would show in its run time.
template <int MAXS>
struct RowMerge {
  f32x2 mine;        // (max, sum) of chunk `lane`
  float x[MAXS];     // this thread's head dim of every chunk's partial row
  // ml, po: the row's first chunk (wave-uniform); d: head dim of this thread
  // last: the largest chunk index whose slot may be read (slots past the row's chunks are loaded and discarded)
  __device__ __forceinline__ void issue(const float2* ml, const float* po, int d, int R, int last_slot, int D) {
    const int lane = threadIdx.x & 63;
    const unsigned char* mlb = uniform_ptr(reinterpret_cast<const unsigned char*>(ml));
    const unsigned char* pob = uniform_ptr(reinterpret_cast<const unsigned char*>(po));
    const uint32_t last = static_cast<uint32_t>(last_slot);
    mine = gload<f32x2, false>(mlb, min(static_cast<uint32_t>(lane), last) * static_cast<uint32_t>(R) * 8u);
    const uint32_t stride = static_cast<uint32_t>(R) * static_cast<uint32_t>(D) * 4u;
    const uint32_t off = static_cast<uint32_t>(d) * 4u;
#pragma unroll
    for (int s = 0; s < MAXS; ++s) x[s] = gload<float, false>(pob, off + min(static_cast<uint32_t>(s), last) * stride);
    __builtin_amdgcn_sched_barrier(0);     // every request leaves before the first use
  }
  // Output element: sum_s 2^(m_s - m) x_s / sum_s 2^(m_s - m) l_s over the first ns chunks; 0 if no key was visible.
  // Chunks before s_lo were skipped by a call with local masking and hold nothing either.
  __device__ __forceinline__ float finish(int ns, int s_lo = 0) const {
    const int lane = threadIdx.x & 63;
    const bool live = lane >= s_lo && lane < ns;
    const float ms = live ? mine[0] : -INFINITY;
    float m = ms;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    const float m_use = (m == -INFINITY) ? 0.f : m;
    const float w = fast_exp2(ms - m_use);              // 0 for lanes at or past ns
    float L = live ? w * mine[1] : 0.f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) L += __shfl_xor(L, off, 64);
    float acc = 0.f;
#pragma unroll
    for (int s = 0; s < MAXS; ++s) {
      const float ws = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), s));
      acc += (s >= s_lo && s < ns) ? ws * x[s] : 0.f;
    }
    return (L > 0.f) ? acc / L : 0.f;
  }
};

template <int MAXS>
__global__ __launch_bounds__(128) void attn_combine_small_kernel(VEGAS_COMBINE_HOT_PARAMS, const CombineParams pfull) {   // launched with D threads
  CombineParams p = pfull;                   // what the requests depend on arrives preloaded in scalar registers
  VEGAS_COMBINE_HOT_ASSIGN(p);
  const int r = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x;
  const ColumnSlots cs = column_slots(p.plan, p.slots_total, b, p.Hkv, p.nsplit, p.chunk_tokens);
  const int64_t pbase = cs.off + static_cast<int64_t>(h) * cs.stride_h;
  int n = p.lens[b];
  RowMerge<MAXS> rm;
  rm.issue(p.part_ml + pbase * p.R + r, p.part_o + (pbase * p.R + r) * p.D, tid, p.R, cs.last, p.D);
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int ns = (n + cs.chunk - 1) / cs.chunk;
  const float o = rm.finish(ns, first_live_chunk(n, p.G, p.window, cs.chunk));
  const int t = r / p.g, j = r % p.g;
  p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * p.D + tid] = float_to_bf16_bits(o);
}

// Verification epilogue in ONE launch (a kernel boundary costs ~3 us on this GPU): workgroups
// [0, nA) merge the chunk partials of two query rows each (as the combine kernels do) and write
// the bf16 output rows (Eq. 1); workgroups [nA, nA + nB) turn the per-(row, page) log-sum-exps of
// 32 pages into page criticalities (Eq. 2 / Eq. 3 with weights, averaged over rows and heads as in the
// last paragraph of Sec. 3.3): score[b][j] = inv_norm * sum_h sum_{rows in R} 2^(page_lse - row_lse).
// A score workgroup derives the global row log-sum-exps itself from the chunks' (max, sum) pairs,
// so it does not depend on the merge workgroups.  Pages at or beyond the sequence's page count get 0.
// MAXS > 0: at most MAXS chunks, the merge workgroups take the one-round-trip path; 0: any number.
// Loads are ordered so that a workgroup's dependent memory round trips are as few as possible: the
// kernel runs for a handful of microseconds and every trip is a sizeable part of that.
constexpr int kFinUnits = 6;     // (row, eighth of the chunks) units a score thread loads per batch
constexpr int kFinPre = 8;       // page log-sum-exps a score thread keeps in registers: 4 * kFinPre rows

// METRIC 1 (the paper's logit metric, token granularity) replaces the page-score role by workgroups
// [nA, nA + nC) that add the H_kv per-head token sums of 1024 tokens each: score[b][i] = tok_norm *
// sum_h partial[b][h][i] for prefix tokens i < n_b - G (Sec. 3.3, last paragraph), 0 elsewhere.
template <int MAXS, int METRIC = 0>
__global__ __launch_bounds__(256) void verify_finalize_kernel(const FinalizeParams p) {
  extern __shared__ float smf[];              // role A (general path): [256 / D][D] weights + [256 / D][4]; role B: [Hkv*R] + [8][32] + [Hkv*R][8] pairs
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int HR = p.Hkv * p.R;
  const ColumnSlots cs = column_slots(p.plan, p.slots_total, b, p.Hkv, p.nsplit, p.chunk_tokens);

  if (static_cast<int>(blockIdx.x) < p.nA) {
    // ---- role A: 256 / D consecutive rows of the Hkv*R rows, D threads (= head dims) each
    const int T = p.D;
    const int sub = tid / T, t128 = tid % T, wv = (tid >> 6) % (T >> 6);
    const int rr_raw = (256 / T) * blockIdx.x + sub;
    const bool valid = rr_raw < HR;
    const int rr = valid ? rr_raw : HR - 1;
    const int h = rr / p.R, r = rr % p.R;
    const int64_t pbase = cs.off + static_cast<int64_t>(h) * cs.stride_h;
    const float2* ml = p.part_ml + pbase * p.R + r;
    float o;
    if constexpr (MAXS > 0) {
      int n = p.lens[b];
      RowMerge<MAXS> rm;
      rm.issue(ml, p.part_o + (pbase * p.R + r) * T, t128, p.R, cs.last, T);
      n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
      o = rm.finish((n + cs.chunk - 1) / cs.chunk);
    } else {
      int n = p.lens[b];
      n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
      const int ns = (n + cs.chunk - 1) / cs.chunk;
      // The host's bound on the chunks of one sequence may be far above what this sequence has (balanced chunking
      // bounds it by all the slots of a head): with few chunks the one-round-trip merge is taken after all.
      if (ns <= 32) {
        if (ns <= 16) {
          RowMerge<16> rm;
          rm.issue(ml, p.part_o + (pbase * p.R + r) * T, t128, p.R, cs.last, T);
          o = rm.finish(ns);
        } else {
          RowMerge<32> rm;
          rm.issue(ml, p.part_o + (pbase * p.R + r) * T, t128, p.R, cs.last, T);
          o = rm.finish(ns);
        }
        if (valid) {
          const int t = r / p.g, j = r % p.g;
          p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * T + t128] = float_to_bf16_bits(o);
        }
        return;
      }
      const float* po = p.part_o + (pbase * p.R + r) * T + t128;
      float* sw = smf + sub * T;
      float* sred = smf + 256 + sub * 4;
      const int64_t ostride = static_cast<int64_t>(p.R) * T;
      float m = -INFINITY;
      for (int s = t128; s < ns; s += T) m = fmaxf(m, ml[static_cast<int64_t>(s) * p.R].x);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
      if ((tid & 63) == 0) sred[wv] = m;
      __syncthreads();
      m = T > 64 ? fmaxf(sred[0], sred[1]) : sred[0];
      const float m_use = (m == -INFINITY) ? 0.f : m;
      float accv = 0.f, L = 0.f;
      for (int s0 = 0; s0 < ns; s0 += T) {
        const int cnt = min(T, ns - s0);
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
        L += T > 64 ? sred[2] + sred[3] : sred[2];
        int s = 0;
        for (; s + 4 <= cnt; s += 4) {
          const float x0 = po[(s0 + s) * ostride], x1 = po[(s0 + s + 1) * ostride];
          const float x2 = po[(s0 + s + 2) * ostride], x3 = po[(s0 + s + 3) * ostride];
          accv += sw[s] * x0 + sw[s + 1] * x1 + sw[s + 2] * x2 + sw[s + 3] * x3;
        }
        for (; s < cnt; ++s) accv += sw[s] * po[(s0 + s) * ostride];
        __syncthreads();
      }
      o = (L > 0.f) ? accv / L : 0.f;
    }
    if (valid) {
      const int t = r / p.g, j = r % p.g;
      p.out[((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * T + t128] = float_to_bf16_bits(o);
    }
    return;
  }

  if constexpr (METRIC == 1) {
    // ---- role C: 1024 tokens; thread = 4 consecutive tokens
    const int i0 = (static_cast<int>(blockIdx.x) - p.nA) * 1024 + 4 * tid;
    const int cap = p.max_blocks * kPage;
    if (i0 >= cap) return;
    int n = p.lens[b];
    // The heads' partial sums are requested eight at a time, unconditionally (clamped), before the length is needed.
    const int iload = min(i0, p.lse_pages - 4);
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int h0 = 0; h0 < p.Hkv; h0 += 8) {
      f32x4 part[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        part[u] = *reinterpret_cast<const f32x4*>(
            p.page_lse + (static_cast<int64_t>(b) * p.Hkv + min(h0 + u, p.Hkv - 1)) * p.lse_pages + iload);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (h0 + u < p.Hkv) sum += part[u];
    }
    n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
    const int p_len = max(n - p.G, 0);
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (i0 + e < p_len) ? sum[e] * p.tok_norm : 0.f;
    *reinterpret_cast<f32x4*>(p.block_scores + static_cast<int64_t>(b) * cap + i0) = o;
    return;
  }

  // ---- role B: 32 pages; thread = (page, head slot)
  const int pg = tid & 31, slot = tid >> 5;
  const int jbase = (blockIdx.x - p.nA) * 32;
  float* out_row = p.block_scores + static_cast<int64_t>(b) * p.max_blocks;
  float* sm_row = smf;                        // [HR] global row lse; -inf for rows that do not count
  float* sm_sum = smf + HR;                   // [8][32]
  float2* sm_pair = reinterpret_cast<float2*>(smf + HR + 256);   // [HR][8] (max, sum) of a row over 1/8 of the chunks

  // Each (row, eighth of the chunks) pair is one unit of work: a thread requests the (max, sum) pairs of
  // kFinUnits units (four chunks each) at once and merges them afterwards, so the table costs about one
  // memory round trip per batch instead of one per chunk.  Slots of chunks past the sequence's end are
  // loaded too (the workspace holds nsplit of them) and dropped at the merge.
  // ns_live: chunk slots worth loading.  With balanced chunking the slots of a head are shared by all sequences and
  // one sequence owns few of them, so its count is worked out first (one more round trip, in a kernel that is
  // bound by bytes at such batch sizes); otherwise every slot up to the host's bound is requested at once.
  int ns_live = p.nsplit;
  if (p.plan) {
    int n0 = p.lens[b];
    n0 = n0 < 0 ? 0 : (n0 > p.max_tokens ? p.max_tokens : n0);
    ns_live = (n0 + cs.chunk - 1) / cs.chunk;
  }
  float2 v[kFinUnits][4];
  auto load_units = [&](int s0, int u0) {
#pragma unroll
    for (int a = 0; a < kFinUnits; ++a) {
      const int u = u0 + 256 * a;
      const int i = u < HR * 8 ? (u >> 3) : 0, sg = u & 7;
      const int h = i / p.R, r = i % p.R;
      const float2* ml = p.part_ml + (cs.off + static_cast<int64_t>(h) * cs.stride_h) * p.R + r;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int sidx = s0 + sg + 8 * q;
        v[a][q] = sidx < ns_live ? ml[static_cast<int64_t>(min(sidx, cs.last)) * p.R] : make_float2(-INFINITY, 0.f);
      }
    }
  };
  // The first batch, and (with few rows) this thread's page log-sum-exps, are
  // requested before the sequence length is needed.
  const int Rc = p.Rc;                        // collected rows per KV head: the only ones that were written
  const bool pre_ok = (Rc & 3) == 0 && Rc <= 4 * kFinPre && p.Hkv <= 8;
  f32x4 pre[kFinPre];
  const int jpre = min(jbase + pg, p.lse_pages - 1);
  if (pre_ok && slot < p.Hkv) {
    const float* pl = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + slot) * p.lse_pages + jpre) * Rc;
#pragma unroll
    for (int q = 0; q < kFinPre; ++q)
      if (4 * q < Rc) pre[q] = *reinterpret_cast<const f32x4*>(pl + 4 * q);
  }
  load_units(0, tid);

  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int ns = (n + cs.chunk - 1) / cs.chunk;
  const int nblk = (n + kPage - 1) / kPage;
  if (jbase >= nblk) {                                             // whole workgroup past the sequence
    if (tid < 32 && jbase + tid < p.max_blocks) out_row[jbase + tid] = 0.f;
    return;
  }
  bool loaded = true;
  for (int s0 = 0; s0 < ns; s0 += 32) {
    for (int u0 = tid; u0 < HR * 8; u0 += kFinUnits * 256) {
      if (!loaded) load_units(s0, u0);
      loaded = false;
#pragma unroll
      for (int a = 0; a < kFinUnits; ++a) {
        const int u = u0 + 256 * a;
        if (u < HR * 8) {
          const int sg = u & 7;
          float2 cur = (s0 == 0) ? make_float2(-INFINITY, 0.f) : sm_pair[u];
          float m = cur.x;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (s0 + sg + 8 * q >= ns) v[a][q] = make_float2(-INFINITY, 0.f);
            m = fmaxf(m, v[a][q].x);
          }
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
  for (int i = tid; i < p.Hkv * Rc; i += 256) {           // sm_row: [Hkv][Rc], the collected rows only
    const int src = (i / Rc) * p.R + collected_row(i % Rc, p.collect_rows, p.G, p.g);
    float m = -INFINITY;
#pragma unroll
    for (int q = 0; q < 8; ++q) m = fmaxf(m, sm_pair[src * 8 + q].x);
    const float m_use = (m == -INFINITY) ? 0.f : m;
    float L = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float2 pr = sm_pair[src * 8 + q];
      L += fast_exp2(pr.x - m_use) * pr.y;
    }
    sm_row[i] = (L > 0.f) ? m_use + fast_log2(L) : -INFINITY;
  }
  __syncthreads();
  {
    const int j = jbase + pg;
    float sc = 0.f;
    if (j < nblk) {
      if (pre_ok) {
        if (slot < p.Hkv) {
          const float* rl = sm_row + slot * Rc;
#pragma unroll
          for (int q = 0; q < kFinPre; ++q) {
            if (4 * q < Rc) {
#pragma unroll
              for (int e = 0; e < 4; ++e)
                if (rl[4 * q + e] != -INFINITY) sc += fast_exp2(pre[q][e] - rl[4 * q + e]);
            }
          }
        }
      } else {
        for (int h = slot; h < p.Hkv; h += 8) {
          const float* pl = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + j) * Rc;
          const float* rl = sm_row + h * Rc;
          if ((Rc & 3) == 0) {
            for (int r = 0; r < Rc; r += 4) {
              const f32x4 x = *reinterpret_cast<const f32x4*>(pl + r);
#pragma unroll
              for (int q = 0; q < 4; ++q)
                if (rl[r + q] != -INFINITY) sc += fast_exp2(x[q] - rl[r + q]);
            }
          } else {
            for (int r = 0; r < Rc; ++r)
              if (rl[r] != -INFINITY) sc += fast_exp2(pl[r] - rl[r]);
          }
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
  }
}

}  // namespace vegas
