// Top-k page selection: workgroup-wide radix select over fp32 score bit patterns, then an
// order-preserving compaction that gathers physical page ids.
//
// The argmax of Eq. 2 / Eq. 3 over unions of pages is the k pages with the largest scores.  The
// pages overlapping the last G token positions are always kept (last sentence of Sec. 3.2) and
// are a suffix of the logical page range, so the search runs over the prefix [0, f0) only.
// Everything is integer work on the score bits: the result is defined bit for bit, ties go to the
// lower logical page index.
#pragma once
#include <type_traits>

#include "vegas_common.hpp"

namespace vegas {

constexpr int kSelectThreads = 1024;
constexpr int kSelectKeyCap = 16384;   // keys kept in LDS (64 KB); longer prefixes re-read the scores
constexpr int kSelectRegRows = 8;      // prefixes of up to 8 x 1024 pages keep their keys in registers instead

// Inclusive prefix sum over the 64 lanes of a wave with DPP row shifts and row broadcasts (no LDS).
__device__ __forceinline__ uint32_t wave_prefix_sum(uint32_t x) {
  int v = static_cast<int>(x);
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return static_cast<uint32_t>(v);
}

// Order-preserving key of a score (larger float <=> larger unsigned); -0 is folded onto +0 and every NaN onto
// key 0, below -infinity: a NaN score ranks last, NaNs among themselves by index like any other tie.
__device__ __forceinline__ uint32_t score_key(float s) {
  const uint32_t u = __float_as_uint(s + 0.0f);
  const uint32_t key = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (s != s) ? 0u : key;
}

__global__ __launch_bounds__(kSelectThreads) void select_blocks_kernel(const SelectParams p) {
  extern __shared__ uint32_t skeys[];                 // [min(prefix pages, key_cap)]
  __shared__ uint32_t hist[kSelectThreads / 64][256];   // one digit histogram per wave: no cross-wave contention
  __shared__ uint32_t sh_prefix, sh_need, sh_count;
  __shared__ uint32_t wave_take[kSelectThreads / 64], wave_eq[kSelectThreads / 64];
  __shared__ uint32_t cell_eq[kSelectRegRows * (kSelectThreads / 64)], cell_gt[kSelectRegRows * (kSelectThreads / 64)];

  const int b = blockIdx.x;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  int32_t* sel = p.sel_table + static_cast<int64_t>(b) * p.max_sel_blocks;
  const int32_t* table = p.block_table + static_cast<int64_t>(b) * p.max_blocks;
  const float* scores = p.block_scores + static_cast<int64_t>(b) * p.max_blocks;

  // With at most 8192 pages per row the scores are requested before the sequence length is known (one memory
  // round trip less, and all requests in flight together): every index below max_blocks is a valid address, what
  // lies past the prefix is dropped.
  constexpr int kPre = 8;
  const bool prefetched = p.max_blocks <= kPre * kSelectThreads;
  float pre[kPre];
  if (prefetched) {
#pragma unroll
    for (int i = 0; i < kPre; ++i) pre[i] = scores[min(tid + i * kSelectThreads, p.max_blocks - 1)];
  }

  int n = p.seq_lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int nblk = (n + kPage - 1) / kPage;
  if (nblk == 0) {
    for (int i = tid; i < p.max_sel_blocks; i += kSelectThreads) sel[i] = -1;
    if (tid == 0) p.sel_seq_lens[b] = 0;
    return;
  }
  const int budget = sequence_budget(p.budgets, p.budget_ratio, p.budget_tokens, b, n);
  const int f0 = max(n - p.G, 0) / kPage;            // first forced page
  int nF = nblk - f0;                                // forced pages (1 or 2 for G <= 17)
  int k = min((budget + kPage - 1) / kPage, nblk);
  k = max(k, nF);
  k = min(k, p.max_sel_blocks);                      // device-side clamp; the host rejects this case
  nF = min(nF, k);
  const int kc = k - nF;                             // pages to take from the prefix [0, f0)
  const bool need_search = kc > 0 && kc < f0;
  const bool take_all = kc >= f0;

  // ---- the whole prefix is taken: its pages in order, nothing to search
  if (kc > 0 && take_all) {
    for (int j = tid; j < f0; j += kSelectThreads) sel[j] = table[j];
  }

  // ---- up to 8192 prefix pages: a thread keeps the keys of pages tid, tid + 1024, ... in registers for the digit
  //      passes and the compaction (no key ever goes through LDS; a wave is bound by the instructions it issues
  //      here, and this is the shortest stream).  Cell (row u, wave w) covers pages 1024 u + 64 w + lane, so cells
  //      in (u, w) order are the pages in ascending order.
  auto register_path = [&]() {
    constexpr int kRows = kSelectRegRows;
    constexpr int kWaves = kSelectThreads / 64;
    constexpr int kCells = kRows * kWaves / 64;                           // cells per lane in the scan below
    const int rows = (f0 + kSelectThreads - 1) / kSelectThreads;          // 1 .. kRows, uniform
    uint32_t key[kRows];
    int32_t page[kRows];
    {
      // (rows past the prefix are skipped by uniform branches: loops stay fully unrolled, arrays in registers)
      float v[kRows];
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        v[u] = 0.f;
        page[u] = 0;
        if (u < rows) {
          v[u] = (prefetched && u < kPre) ? pre[u < kPre ? u : 0] : scores[min(u * kSelectThreads + tid, f0 - 1)];
          page[u] = table[min(u * kSelectThreads + tid, f0 - 1)];         // coalesced, used if the page is taken
        }
      }
#pragma unroll
      for (int u = 0; u < kRows; ++u) key[u] = score_key(v[u]);
    }
    // radix select (see the general path below for the early exit)
    uint32_t prefix = 0u, mask = 0u, need = static_cast<uint32_t>(kc);
    // Scores cluster: the top byte of nearly all keys is the same, background pages often agree to a percent (two
    // bytes), tie-heavy scores in every byte -- and per-lane atomics would then collide on one LDS address.  A pass
    // whose predecessor left at least three quarters of its keys in one bin counts the lanes that share the first
    // active lane's digit with ONE atomic (the others add themselves); otherwise digits are spread and every lane
    // adds itself, which is fewer instructions.
    bool clustered = true;
    uint32_t active = static_cast<uint32_t>(f0);
#pragma unroll 1
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      uint32_t* h = hist[wave];
#pragma unroll
      for (int i = 0; i < 4; ++i) h[lane + 64 * i] = 0u;       // wave-private: ordered by the wave's own LDS stream
#pragma unroll
      for (int u = 0; u < kRows; ++u) {
        if (u >= rows) continue;
        const bool act = u * kSelectThreads + tid < f0 && (key[u] & mask) == prefix;
        const uint32_t d = (key[u] >> shift) & 255u;
        if (clustered) {
          const uint64_t am = __builtin_amdgcn_ballot_w64(act);
          const int leader = am ? __builtin_ctzll(am) : 0;
          const uint32_t dl = __builtin_amdgcn_readlane(d, leader);
          const uint64_t same = __builtin_amdgcn_ballot_w64(act && d == dl);
          if (lane == leader && am != 0ull) atomicAdd(&h[dl], static_cast<uint32_t>(__popcll(same)));
          if (act && d != dl) atomicAdd(&h[d], 1u);
        } else if (act) {
          atomicAdd(&h[d], 1u);
        }
      }
      __syncthreads();
      if (wave == 0) {
        uint32_t c[4] = {0u, 0u, 0u, 0u};                     // lane l owns bins 4l .. 4l+3
        for (int w = 0; w < kWaves; ++w) {
#pragma unroll
          for (int i = 0; i < 4; ++i) c[i] += hist[w][4 * lane + i];
        }
        const uint32_t mine = c[0] + c[1] + c[2] + c[3];
        const uint32_t incl = wave_prefix_sum(mine);
        uint32_t above = __builtin_amdgcn_readlane(incl, 63) - incl;      // keys in the bins above this lane's
#pragma unroll
        for (int i = 3; i >= 0; --i) {
          if (above < need && need <= above + c[i]) {
            sh_prefix = prefix | (static_cast<uint32_t>(4 * lane + i) << shift);
            sh_need = need - above;
            sh_count = c[i];
          }
          above += c[i];
        }
      }
      __syncthreads();
      prefix = sh_prefix;
      need = sh_need;
      mask |= 255u << shift;
      const uint32_t count = sh_count;         // keys in the chosen bin: the next pass's active keys
      if (count == need) break;                // the whole bin is taken: its lower digits do not matter
      clustered = 4u * count >= 3u * active;
      active = count;
    }
    const uint32_t T = prefix, need_eq = need, kmask = mask;
    // compaction: per cell the keys above T and the ties; one wave turns the 128 counts into tie ranks and
    // output positions; then every thread places its taken pages
    const uint64_t lt = (1ull << lane) - 1ull;
    uint64_t beq[kRows], bgt[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      beq[u] = bgt[u] = 0ull;
      if (u >= rows) continue;
      const bool valid = u * kSelectThreads + tid < f0;
      const uint32_t km = key[u] & kmask;
      beq[u] = __builtin_amdgcn_ballot_w64(valid && km == T);
      bgt[u] = __builtin_amdgcn_ballot_w64(valid && km > T);
      if (lane == 0) {
        cell_eq[u * kWaves + wave] = static_cast<uint32_t>(__popcll(beq[u]));
        cell_gt[u * kWaves + wave] = static_cast<uint32_t>(__popcll(bgt[u]));
      }
    }
    __syncthreads();
    if (wave == 0) {                                          // lane l owns cells kCells l .. kCells l + kCells - 1
      const int live = rows * kWaves;                         // cells of rows past the prefix were never written
      uint32_t e[kCells], g[kCells], esum = 0u;
#pragma unroll
      for (int c = 0; c < kCells; ++c) {
        const int cell = kCells * lane + c;
        e[c] = cell < live ? cell_eq[cell] : 0u;
        g[c] = cell < live ? cell_gt[cell] : 0u;
        esum += e[c];
      }
      uint32_t eb = wave_prefix_sum(esum) - esum, tsum = 0u;  // ties before the lane's first cell
      uint32_t t[kCells];
#pragma unroll
      for (int c = 0; c < kCells; ++c) {
        t[c] = g[c] + min(e[c], need_eq > eb ? need_eq - eb : 0u);      // pages the cell takes
        if (kCells * lane + c < live) cell_eq[kCells * lane + c] = eb;  // ties before the cell
        eb += e[c];
        tsum += t[c];
      }
      uint32_t pb = wave_prefix_sum(tsum) - tsum;
#pragma unroll
      for (int c = 0; c < kCells; ++c) {
        if (kCells * lane + c < live) cell_gt[kCells * lane + c] = pb;  // output position of the cell
        pb += t[c];
      }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      if (u >= rows) continue;
      const uint32_t eb = cell_eq[u * kWaves + wave], pb = cell_gt[u * kWaves + wave];
      const bool eq = (beq[u] >> lane) & 1ull, gt = (bgt[u] >> lane) & 1ull;
      const bool take = gt || (eq && eb + __popcll(beq[u] & lt) < need_eq);
      const uint64_t btk = __builtin_amdgcn_ballot_w64(take);
      if (take) {
        const uint32_t pos = pb + __popcll(btk & lt);
        if (pos < static_cast<uint32_t>(p.max_sel_blocks)) sel[pos] = page[u];
      }
    }
  };

  // ---- longer prefixes: keys go to LDS once (up to key_cap of them; beyond that they are recomputed from the scores)
  const bool in_regs = f0 <= kSelectRegRows * kSelectThreads;
  const bool in_lds = f0 <= p.key_cap;
  if (need_search && !in_regs && in_lds) {
    // groups of kPre independent requests (clamped, so that none sits behind a branch)
    for (int base = tid; base < f0; base += kPre * kSelectThreads) {
      float v[kPre];
#pragma unroll
      for (int i = 0; i < kPre; ++i) v[i] = scores[min(base + i * kSelectThreads, f0 - 1)];
#pragma unroll
      for (int i = 0; i < kPre; ++i)
        if (base + i * kSelectThreads < f0) skeys[base + i * kSelectThreads] = score_key(v[i]);
    }
    __syncthreads();
  }

  // The search and the compaction for prefixes of more than 8192 pages (only reached when a search is needed),
  // compiled once for keys held in LDS and once for keys recomputed from the scores (prefixes longer than the LDS
  // area): the choice is uniform for the workgroup and taken once.
  auto search_and_compact = [&](auto lds_tag) {
    constexpr bool kKeysInLds = decltype(lds_tag)::value;
    auto key_at = [&](int j) -> uint32_t {
      if constexpr (kKeysInLds) return skeys[j];
      else return score_key(scores[j]);
    };

    // ---- radix select: key of the kc-th largest prefix score, and how many of its ties to take.  The search
    //      stops as soon as the digit bin that holds the kc-th key is needed whole (distinct scores: after three
    //      passes as a rule): T then is a key PREFIX, kmask its resolved bits, and every key with that prefix is
    //      a "tie".
    uint32_t T, need_eq, kmask;
    {
      uint32_t prefix = 0u, mask = 0u, need = static_cast<uint32_t>(kc);
#pragma unroll 1
      for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        uint32_t* h = hist[wave];
#pragma unroll
        for (int i = 0; i < 4; ++i) h[lane + 64 * i] = 0u;     // wave-private: ordered by the wave's own LDS stream
        // Up to four key rows per trip (independent chains overlap; a wave is bound by instruction issue and
        // latency here).  A row whose active lanes all carry one digit -- the rule for the top byte, where scores
        // cluster -- is counted by one atomic of its first active lane; any other row adds lane by lane.
        auto count_rows = [&](int base, auto rows_tag) {
          constexpr int kR = decltype(rows_tag)::value;
          uint32_t d[kR];
          bool act[kR];
#pragma unroll
          for (int u = 0; u < kR; ++u) {
            const int j = base + u * kSelectThreads + tid;
            const uint32_t key = key_at(min(j, f0 - 1));
            act[u] = j < f0 && (key & mask) == prefix;
            d[u] = (key >> shift) & 255u;
          }
          uint64_t am[kR], same[kR];
          uint32_t dl[kR];
#pragma unroll
          for (int u = 0; u < kR; ++u) {
            am[u] = __builtin_amdgcn_ballot_w64(act[u]);
            const int leader = am[u] ? __builtin_ctzll(am[u]) : 0;
            dl[u] = __builtin_amdgcn_readlane(d[u], leader);
            same[u] = __builtin_amdgcn_ballot_w64(act[u] && d[u] == dl[u]);
          }
#pragma unroll
          for (int u = 0; u < kR; ++u) {
            if (am[u] == 0ull) continue;
            if (same[u] == am[u]) {
              if (lane == 0) atomicAdd(&h[dl[u]], static_cast<uint32_t>(__popcll(am[u])));
            } else if (act[u]) {
              atomicAdd(&h[d[u]], 1u);
            }
          }
        };
        for (int base = 0; base < f0;) {
          const int rows = (f0 - base + kSelectThreads - 1) / kSelectThreads;
          if (rows >= 4) {
            count_rows(base, std::integral_constant<int, 4>{});
            base += 4 * kSelectThreads;
          } else if (rows >= 2) {
            count_rows(base, std::integral_constant<int, 2>{});
            base += 2 * kSelectThreads;
          } else {
            count_rows(base, std::integral_constant<int, 1>{});
            base += kSelectThreads;
          }
        }
        __syncthreads();
        if (wave == 0) {
          // lane l owns bins 4l .. 4l+3; count from the top bin downwards
          uint32_t c[4] = {0u, 0u, 0u, 0u};
          for (int w = 0; w < kSelectThreads / 64; ++w) {
#pragma unroll
            for (int i = 0; i < 4; ++i) c[i] += hist[w][4 * lane + i];
          }
          const uint32_t mine = c[0] + c[1] + c[2] + c[3];
          uint32_t incl = mine;                        // sum over lanes >= lane
#pragma unroll
          for (int off = 1; off < 64; off <<= 1) {
            const uint32_t o = __shfl_down(incl, off, 64);
            if (lane + off < 64) incl += o;
          }
          uint32_t above = incl - mine;                // elements in bins above this lane's bins
#pragma unroll
          for (int i = 3; i >= 0; --i) {
            if (above < need && need <= above + c[i]) {
              sh_prefix = prefix | (static_cast<uint32_t>(4 * lane + i) << shift);
              sh_need = need - above;
              sh_count = c[i];
            }
            above += c[i];
          }
        }
        __syncthreads();
        prefix = sh_prefix;
        need = sh_need;
        mask |= 255u << shift;
        if (sh_count == need) break;         // the whole bin is taken: its lower digits do not matter
      }
      T = prefix;
      need_eq = need;
      kmask = mask;
    }

    // ---- ordered compaction of the prefix: wave w owns the contiguous pages [w*span, (w+1)*span) and walks
    //      them 64 at a time (lane = page), so page order is (wave, step, lane) and every memory access is
    //      coalesced.  Ballots count the keys above T and the ties; a 16-entry prefix over the wave totals turns
    //      the counts into global tie ranks and output positions.
    {
      constexpr int kWaves = kSelectThreads / 64;
      const int span = ((f0 + kWaves - 1) / kWaves + 63) / 64 * 64;
      const int w0 = min(wave * span, f0), w1 = min(w0 + span, f0);
      const uint64_t lt = (1ull << lane) - 1ull;
      // pass A: keys above T and ties in this wave's pages (up to four steps per trip).  A wave's takes follow
      //         from the counts: its keys above T plus as many of its ties as are still wanted.
      uint32_t eq_wave = 0u, gt_wave = 0u;
      {
        auto count_steps = [&](int base, auto steps_tag) {
          constexpr int kS = decltype(steps_tag)::value;
#pragma unroll
          for (int i = 0; i < kS; ++i) {
            const int j = base + 64 * i + lane;
            const uint32_t key = key_at(min(j, f0 - 1)) & kmask;
            eq_wave += __popcll(__builtin_amdgcn_ballot_w64(j < w1 && key == T));
            gt_wave += __popcll(__builtin_amdgcn_ballot_w64(j < w1 && key > T));
          }
        };
        int base = w0;
        for (; base + 64 * 3 < w1; base += 64 * 4) count_steps(base, std::integral_constant<int, 4>{});
        for (; base < w1; base += 64) count_steps(base, std::integral_constant<int, 1>{});
      }
      if (lane == 0) {
        wave_eq[wave] = eq_wave;
        wave_take[wave] = gt_wave;
      }
      __syncthreads();
      uint32_t eq_before = 0u, pos_run = 0u;
      for (int w = 0; w < wave; ++w) {
        const uint32_t e = wave_eq[w];
        const uint32_t wanted = need_eq > eq_before ? need_eq - eq_before : 0u;   // ties still wanted where wave w starts
        pos_run += wave_take[w] + min(e, wanted);
        eq_before += e;
      }
      // pass B: the decisions, now with positions; gather the physical page ids.  The page ids of kGather steps
      //         are requested together and unconditionally (coalesced, clamped): a request per taken page
      //         behind its decision would cost one memory round trip per step.
      constexpr int kGather = 8;
      uint32_t eq_run = eq_before;
      for (int base = w0; base < w1; base += 64 * kGather) {
        int32_t page[kGather];
#pragma unroll
        for (int i = 0; i < kGather; ++i) page[i] = table[min(base + 64 * i + lane, f0 - 1)];
#pragma unroll
        for (int i = 0; i < kGather; ++i) {
          if (base + 64 * i >= w1) break;
          const int j = base + 64 * i + lane;
          const uint32_t key = key_at(min(j, f0 - 1)) & kmask;
          const bool eq = j < w1 && key == T;
          const bool gt = j < w1 && key > T;
          const uint64_t beq = __builtin_amdgcn_ballot_w64(eq);
          const bool take = gt || (eq && eq_run + __popcll(beq & lt) < need_eq);
          eq_run += __popcll(beq);
          const uint64_t btk = __builtin_amdgcn_ballot_w64(take);
          if (take) {
            const uint32_t pos = pos_run + __popcll(btk & lt);
            if (pos < static_cast<uint32_t>(p.max_sel_blocks)) sel[pos] = page[i];
          }
          pos_run += __popcll(btk);
        }
      }
    }
  };
  if (need_search) {
    if (in_regs) register_path();
    else if (in_lds) search_and_compact(std::true_type{});
    else search_and_compact(std::false_type{});
  }

  // ---- forced tail pages, padding, covered length
  for (int i = tid; i < nF; i += kSelectThreads) sel[kc + i] = table[nblk - nF + i];
  for (int i = k + tid; i < p.max_sel_blocks; i += kSelectThreads) sel[i] = -1;
  if (tid == 0) p.sel_seq_lens[b] = kPage * (k - 1) + (n - kPage * (nblk - 1));
}

// Adds the num_new newest token positions of sequence b, whose length now is n_new, to its selection: a new table
// entry whenever a position starts a page of the selection's page size (one thread's work).
__device__ __forceinline__ void extend_selection_row(const ExtendParams& p, int b, int n_new) {
  const int covered = p.sel_seq_lens[b];
  if (covered <= 0) return;
  const int P = p.page_size;
  int32_t* sel = p.sel_table + static_cast<int64_t>(b) * p.max_sel_blocks;
  const int32_t* table = p.block_table + static_cast<int64_t>(b) * p.max_blocks;
  int count = (covered + P - 1) / P;
  int added = 0;
  for (int i = n_new - p.num_new; i < n_new; ++i) added += (i >= 0 && i % P == 0) ? 1 : 0;
  if (count + added > p.max_sel_blocks) return;            // row full: left as it is
  for (int i = n_new - p.num_new; i < n_new; ++i) {
    if (i >= 0 && i % P == 0) {
      const int page16 = min(i / kPage, p.max_blocks - 1);
      sel[count++] = table[page16] * (kPage / P) + (i % kPage) / P;
    }
  }
  p.sel_seq_lens[b] = covered + p.num_new;
}

// One thread per sequence.
__global__ void extend_selection_kernel(const ExtendParams p) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= p.batch) return;
  extend_selection_row(p, b, p.seq_lens[b]);
}

}  // namespace vegas
