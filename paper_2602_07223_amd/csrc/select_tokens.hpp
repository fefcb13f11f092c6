// Top-k selection over single tokens (the paper's own granularity: Sec. 3.3 last paragraph, Sec. 4).
//
// A sequence has up to a few hundred thousand prefix tokens, too many for one workgroup, so the
// radix select of the page version is spread over workgroups that own 4096-token slices and meet in
// per-slice digit histograms between launches (plain stores, nothing to clear, no global atomics):
//   token_select_hist x 4  pass q: every workgroup sums the slices' histograms of passes < q, derives
//                          the key prefix they fix, counts digit q of its own slice's matching keys
//                          in LDS and stores its 256 counts
//   token_select_write     derives the k-th key T the same way; the keys > T and == T in the slices
//                          before its own follow from those slices' histograms, so it knows where its
//                          output starts; then an order-preserving compaction of the slice;
//                          physical slot = table[i / 16] * 16 + i % 16
// The last min(G, n) tokens are not part of the prefix and are always kept (Sec. 3.2, last sentence).
// Integer work on the score bits: defined bit for bit, ties go to the lower position.
#pragma once
#include "select_blocks.hpp"
#include "vegas_common.hpp"

namespace vegas {

constexpr int kTokSlice = 4096;       // prefix tokens per workgroup
constexpr int kTokThreads = 1024;

struct TokenSelectParams {
  const float* scores;        // [B, max_blocks * 16]
  const int32_t* block_table; // [B, max_blocks]
  const int32_t* seq_lens;
  const int32_t* budgets;     // or nullptr
  int32_t* sel_table;         // [B, max_sel] physical token slots
  int32_t* sel_seq_lens;
  uint32_t* hist;             // [B, 4, slices, 256] digit histogram of every (pass, slice)
  int32_t budget_tokens, G, max_blocks, max_sel, max_tokens, slices;
  float budget_ratio;         // > 0: budget = ceil(ratio * seq_len) unless per-sequence budgets are given
};

// What one sequence asks for.
struct TokenPlan {
  int n, p_len, tail, k, kc;
  bool need_search, take_all;
};

__device__ __forceinline__ TokenPlan token_plan(const TokenSelectParams& p, int b) {
  TokenPlan t;
  int n = p.seq_lens[b];
  t.n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  t.p_len = max(t.n - p.G, 0);
  t.tail = t.n - t.p_len;
  const int budget = sequence_budget(p.budgets, p.budget_ratio, p.budget_tokens, b, t.n);
  int k = min(budget, t.n);
  k = max(k, t.tail);
  t.k = min(k, p.max_sel);                           // device-side clamp; the host rejects this case
  t.kc = max(t.k - t.tail, 0);
  t.need_search = t.kc > 0 && t.kc < t.p_len;
  t.take_all = t.kc >= t.p_len;
  return t;
}

// All threads: sh_tot[q][bin] = sum over the sequence's slices of histogram (pass q, bin) for q < passes,
// and, if sh_bef is given, the same sum over the slices before `upto` only.  Followed by a barrier.
__device__ __forceinline__ void token_sum_hists(const TokenSelectParams& p, int b, int passes, int nslices, int upto,
                                                uint32_t (*sh_tot)[256], uint32_t (*sh_bef)[256]) {
  const int q = threadIdx.x >> 8, bin = threadIdx.x & 255;          // 1024 threads = 4 passes x 256 bins
  if (q < passes) {
    const uint32_t* h = p.hist + ((static_cast<int64_t>(b) * 4 + q) * p.slices) * 256 + bin;
    uint32_t tot = 0u, bef = 0u;
    for (int sl0 = 0; sl0 < nslices; sl0 += 8) {          // eight independent loads in flight per round trip
      uint32_t c[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) c[u] = h[static_cast<int64_t>(min(sl0 + u, nslices - 1)) * 256];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        tot += sl0 + u < nslices ? c[u] : 0u;
        bef += sl0 + u < upto ? c[u] : 0u;
      }
    }
    sh_tot[q][bin] = tot;
    if (sh_bef) sh_bef[q][bin] = bef;
  }
  __syncthreads();
}

// Executed by ONE full wave: walks the summed histograms of passes 0 .. passes-1 and returns, in every
// lane, the key prefix they fix and how many keys are still wanted inside it.
__device__ __forceinline__ void token_prefix(const uint32_t (*sh_tot)[256], int passes, uint32_t kc,
                                             uint32_t* prefix_out, uint32_t* need_out) {
  const int lane = threadIdx.x & 63;
  uint32_t prefix = 0u, need = kc;
  for (int q = 0; q < passes; ++q) {
    const int shift = 24 - 8 * q;
    // lane l owns bins 255-4l .. 252-4l, so an inclusive prefix sum over lanes counts from the top bin down
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] = sh_tot[q][255 - 4 * lane - i];
    const uint32_t mine = c[0] + c[1] + c[2] + c[3];
    uint32_t above = wave_prefix_sum(mine) - mine;
    uint32_t found = 0u, digit = 0u, rest = 0u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (above < need && need <= above + c[i]) {
        found = 1u;
        digit = static_cast<uint32_t>(255 - 4 * lane - i);
        rest = need - above;
      }
      above += c[i];
    }
    const uint64_t who = __builtin_amdgcn_ballot_w64(found != 0u);   // exactly one lane when need <= matching keys
    const int src = who ? __builtin_ctzll(who) : 0;
    digit = __builtin_amdgcn_readlane(digit, src);
    rest = __builtin_amdgcn_readlane(rest, src);
    prefix |= digit << shift;
    need = rest;
  }
  *prefix_out = prefix;
  *need_out = need;
}

__global__ __launch_bounds__(kTokThreads) void token_select_hist(const TokenSelectParams p, int pass) {
  __shared__ uint32_t hist[kTokThreads / 64][256];
  __shared__ uint32_t sh_tot[4][256];
  __shared__ uint32_t sh_prefix;
  const int b = blockIdx.y, s = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const TokenPlan t = token_plan(p, b);
  const int base = s * kTokSlice;
  if (!t.need_search || base >= t.p_len) return;
  const int nslices = (t.p_len + kTokSlice - 1) / kTokSlice;
  // The thread's scores do not depend on the earlier passes: they are requested first (together, clamped indices,
  // none behind a branch), so their round trip overlaps the one of the slices' histograms.
  const float* scores = p.scores + static_cast<int64_t>(b) * p.max_blocks * kPage;
  float sc[kTokSlice / kTokThreads];
#pragma unroll
  for (int it = 0; it < kTokSlice / kTokThreads; ++it) sc[it] = scores[min(base + it * kTokThreads + tid, t.p_len - 1)];
  uint32_t* h = hist[wave];
#pragma unroll
  for (int i = 0; i < 4; ++i) h[lane + 64 * i] = 0u;
  token_sum_hists(p, b, pass, nslices, 0, sh_tot, nullptr);
  if (wave == 0) {
    uint32_t prefix, need;
    token_prefix(sh_tot, pass, static_cast<uint32_t>(t.kc), &prefix, &need);
    if (lane == 0) sh_prefix = prefix;
  }
  __syncthreads();
  const uint32_t prefix = sh_prefix;
  const uint32_t mask = pass == 0 ? 0u : (0xFFFFFFFFu << (32 - 8 * pass));
  const int shift = 24 - 8 * pass;
#pragma unroll
  for (int it = 0; it < kTokSlice / kTokThreads; ++it) {
    const int j = base + it * kTokThreads + tid;
    const uint32_t key = score_key(sc[it]);
    bool act = j < t.p_len && (key & mask) == prefix;
    const uint32_t d = (key >> shift) & 255u;
    // lanes that share the leader's digit are counted by one atomic; what is left after two rounds adds itself
#pragma unroll
    for (int round = 0; round < 2; ++round) {
      const uint64_t am = __builtin_amdgcn_ballot_w64(act);
      const int leader = am ? __builtin_ctzll(am) : 0;
      const uint32_t dl = __builtin_amdgcn_readlane(d, leader);
      const bool hit = act && d == dl;
      const uint64_t same = __builtin_amdgcn_ballot_w64(hit);
      if (hit && lane == leader) atomicAdd(&h[dl], static_cast<uint32_t>(__popcll(same)));
      act = act && !hit;
    }
    if (act) atomicAdd(&h[d], 1u);
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t c = 0u;
#pragma unroll
    for (int w = 0; w < kTokThreads / 64; ++w) c += hist[w][tid];
    p.hist[((static_cast<int64_t>(b) * 4 + pass) * p.slices + s) * 256 + tid] = c;
  }
}

__global__ __launch_bounds__(kTokThreads) void token_select_write(const TokenSelectParams p) {
  __shared__ uint32_t sh_tot[4][256], sh_bef[4][256];
  __shared__ uint32_t sh_T, sh_need_eq, sh_eq_before, sh_pos_before;
  __shared__ uint32_t wave_take[kTokThreads / 64], wave_eq[kTokThreads / 64];
  const int b = blockIdx.y, s = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const TokenPlan t = token_plan(p, b);
  int32_t* sel = p.sel_table + static_cast<int64_t>(b) * p.max_sel;
  const int32_t* table = p.block_table + static_cast<int64_t>(b) * p.max_blocks;
  const float* scores = p.scores + static_cast<int64_t>(b) * p.max_blocks * kPage;
  auto slot_of = [&](int i) -> int32_t { return table[i >> 4] * kPage + (i & 15); };

  // ---- the kept tail, the padding and the length: spread over the sequence's workgroups
  const int stride = gridDim.x * kTokThreads;
  for (int i = s * kTokThreads + tid; i < t.tail; i += stride)
    if (t.kc + i < p.max_sel) sel[t.kc + i] = slot_of(t.p_len + i);
  for (int i = t.k + s * kTokThreads + tid; i < p.max_sel; i += stride) sel[i] = -1;
  if (s == 0 && tid == 0) p.sel_seq_lens[b] = t.k;

  const int base = s * kTokSlice;
  if (t.kc == 0 || base >= t.p_len) return;
  // This thread's tokens (wave w owns tokens [base + 256 w, base + 256 (w + 1)), 64 per step, lane = token): their
  // scores and the table entries of their pages are requested now, unconditionally and together, so that the
  // round trip overlaps the one of the slices' histograms and no request waits behind a decision.
  constexpr int kSteps = kTokSlice / kTokThreads;
  const int w0 = base + wave * (64 * kSteps);
  uint32_t key[kSteps];
  int32_t page_of[kSteps];
  bool valid[kSteps];
#pragma unroll
  for (int st = 0; st < kSteps; ++st) {
    const int j = w0 + 64 * st + lane;
    valid[st] = j < t.p_len;
    key[st] = score_key(scores[min(j, t.p_len - 1)]);
    page_of[st] = table[min(j, t.p_len - 1) >> 4];
  }
  if (t.need_search) {
    const int nslices = (t.p_len + kTokSlice - 1) / kTokSlice;
    token_sum_hists(p, b, 4, nslices, s, sh_tot, sh_bef);
    if (wave == 0) {
      uint32_t T, need_eq;
      token_prefix(sh_tot, 4, static_cast<uint32_t>(t.kc), &T, &need_eq);
      // In the slices before this one: keys > T are, pass by pass, the keys that match T's prefix so far and
      // have a larger digit; keys == T are the last pass's count of T's low digit.
      uint32_t gt = 0u;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t digit = (T >> (24 - 8 * q)) & 255u;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t bin = static_cast<uint32_t>(4 * lane + i);
          gt += bin > digit ? sh_bef[q][bin] : 0u;
        }
      }
      gt = __builtin_amdgcn_readlane(wave_prefix_sum(gt), 63);
      const uint32_t eq_before = sh_bef[3][T & 255u];
      if (lane == 0) {
        sh_T = T;
        sh_need_eq = need_eq;
        sh_eq_before = eq_before;
        sh_pos_before = gt + min(eq_before, need_eq);        // ties are taken in order until need_eq are found
      }
    }
  }
  __syncthreads();
  const bool all = t.take_all;
  const uint32_t T = all ? 0u : sh_T, need_eq = all ? 0u : sh_need_eq;
  const uint32_t slice_eq_before = all ? 0u : sh_eq_before;
  const uint32_t slice_pos_before = all ? static_cast<uint32_t>(base) : sh_pos_before;

  // ---- ordered compaction
  const uint64_t lt = (1ull << lane) - 1ull;
  uint32_t eq_wave = 0u;
#pragma unroll
  for (int st = 0; st < kSteps; ++st) eq_wave += __popcll(__builtin_amdgcn_ballot_w64(valid[st] && !all && key[st] == T));
  if (lane == 0) wave_eq[wave] = eq_wave;
  __syncthreads();
  uint32_t eq_before = slice_eq_before;
  for (int w = 0; w < wave; ++w) eq_before += wave_eq[w];
  uint32_t take_wave = 0u, eq_run = eq_before;
  bool take[kSteps];
#pragma unroll
  for (int st = 0; st < kSteps; ++st) {
    const bool eq = valid[st] && !all && key[st] == T;
    const bool gt = valid[st] && !all && key[st] > T;
    const uint64_t beq = __builtin_amdgcn_ballot_w64(eq);
    take[st] = all ? valid[st] : (gt || (eq && eq_run + __popcll(beq & lt) < need_eq));
    eq_run += __popcll(beq);
    take_wave += __popcll(__builtin_amdgcn_ballot_w64(take[st]));
  }
  if (lane == 0) wave_take[wave] = take_wave;
  __syncthreads();
  uint32_t pos_run = slice_pos_before;
  for (int w = 0; w < wave; ++w) pos_run += wave_take[w];
#pragma unroll
  for (int st = 0; st < kSteps; ++st) {
    const uint64_t btk = __builtin_amdgcn_ballot_w64(take[st]);
    if (take[st]) {
      const uint32_t pos = pos_run + __popcll(btk & lt);
      if (pos < static_cast<uint32_t>(p.max_sel)) sel[pos] = page_of[st] * kPage + ((w0 + 64 * st + lane) & 15);
    }
    pos_run += __popcll(btk);
  }
}

}  // namespace vegas
