// Shared device-side types and helpers for the gfx950 kernels (wave64, MFMA, LDS).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vegas {

constexpr int kPage = 16;       // tokens per KV page
constexpr int kHeadDim = 128;   // the larger of the two head dimensions (128, 64) the kernels are written for
constexpr int kTile = 32;       // tokens per MFMA tile (two pages)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// Value of the lane 32 positions away (the other half of the wave).
__device__ __forceinline__ float xhalf(float x) { return __shfl_xor(x, 32, 64); }

// Orders LDS traffic between the lanes of ONE wave (a wave's LDS instructions execute in order,
// so only the compiler has to be kept from moving accesses across this point).
__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// float -> bf16 bits, round to nearest even (finite values and infinities).
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}

// Pins a wave-uniform pointer into scalar registers so that loads take the
// "scalar base + 32-bit lane offset" addressing form.
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* ptr) {
  const uint64_t v = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v));
  const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(v >> 32));
  return reinterpret_cast<const unsigned char*>((static_cast<uint64_t>(hi) << 32) | lo);
}

// Global-memory load at (wave-uniform base) + (32-bit lane offset).  STREAMING marks data that is
// read once (the verification pass over the whole cache): the non-temporal hint keeps it from
// displacing useful lines and was worth 7-12 % of the kernel time.
template <typename T, bool STREAMING>
__device__ __forceinline__ T gload(const unsigned char* sbase, uint32_t voff) {
  typedef const __attribute__((address_space(1))) T* gp;
  gp ptr = (gp)((const __attribute__((address_space(1))) unsigned char*)sbase + voff);
  if constexpr (STREAMING) return __builtin_nontemporal_load(ptr);
  else return *ptr;
}

// Arguments of the KV-streaming attention kernel (verification and draft share it).
struct SplitParams {
  const uint16_t* q;        // verify [B, G, Hq, D]; draft [B, Hq, D] (G = 1)
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* table;     // [B, table_stride] physical page of each logical page
  const int32_t* lens;      // [B] valid tokens
  float* part_o;            // [B, Hkv, nsplit, R, D] un-normalised partial outputs
  float2* part_ml;          // [B, Hkv, nsplit, R]    (running max in log2 units, partial sum)
  float* page_lse;          // [B, Hkv, lse_pages, Rc] log2-sum-exp2 of each page's scaled logits for the Rc collected
                            // rows of a KV head; or, for the logit metric, [B, Hkv, lse_pages] per-token sums of
                            // the collected rows' q . k
  int32_t table_stride;
  int32_t G, g, R, Hq, Hkv;
  int32_t chunk_tokens, nsplit, lse_pages, max_tokens;
  int32_t lds_q_off;        // byte offset of the query tile inside dynamic LDS
  int32_t row_blocks;       // ceil(R / 32): 32-row blocks of one KV head, one workgroup each
  int32_t collect_rows;     // which verification rows are collected (1: all, 2: first and last)
  int32_t Rc;               // collected rows per KV head (collected_count)
  int32_t window;           // > 0: local masking, a row at position pos sees keys pos - window + 1 .. pos (causal calls)
  uint16_t* out_direct;     // draft calls with one chunk per (sequence, KV head): the bf16 output [B, G, Hq, D], which
                            // the streaming kernel then normalises and writes itself (nullptr: partials for a merge kernel)
  float* trash;             // attn_pair_kernel: a word of the workspace that takes the stores of invalid elements
  int2* plan;               // balanced chunking (or nullptr): [B] (first partial slot, chunk tokens) per sequence,
                            // computed by every workgroup from the lengths and written here by workgroup 0
  int32_t batch;            // B (balanced chunking)
  int32_t slots_target;     // j1: workgroups per KV head (and row block) of one launch wave
  int32_t slots_target2;    // j2: of two waves (= j1 where only one plan is wanted)
  int32_t chunk_cap_units;  // longest chunk the plan may produce, in units
  int32_t slots_total;      // slots per KV head the workspace holds
  int32_t chunk_unit;       // chunk lengths are multiples of this many tokens
  int64_t page_stride, token_stride, head_stride, num_pages;
  float scale_log2e;
  unsigned long long* timeline;   // profiling builds: where the waves' phase stamps go (nullptr: nowhere)
};

// ---- per-wave phase timeline (builds with -DVEGAS_TIMELINE only: a profiling build, never the product) ----
// Every wave of a streaming kernel notes the wall clock (100 MHz, the same on all compute units) at a few fixed
// program points and stores the notes when it exits: [workgroup][wave][kTimelineEvents] 64-bit stamps in a buffer
// the caller registers with vegas_debug_set_timeline.  In ordinary builds the macros expand to nothing.
constexpr int kTimelineEvents = 8;
enum {
  kTlEntry = 0,        // first instruction of the wave
  kTlLength = 1,       // sequence length known (past the early exit)
  kTlLoadsIssued = 2,  // the first tile's K/V requests are out
  kTlQueries = 3,      // queries in LDS, workgroup past its first barrier
  kTlFirstTile = 4,    // first tile's arithmetic done
  kTlStreamed = 5,     // last tile's arithmetic done
  kTlMerged = 6,       // row maxima exchanged: past the merge's first barrier
  kTlExit = 7          // partial result stored
};
#ifdef VEGAS_TIMELINE
#define VEGAS_TL_DECL unsigned long long tl_stamps[kTimelineEvents] = {0, 0, 0, 0, 0, 0, 0, 0}
// (the empty asm statements keep the compiler from moving memory operations across a stamp)
#define VEGAS_TL(ev)                                       \
  do {                                                     \
    asm volatile("" ::: "memory");                         \
    tl_stamps[ev] = __builtin_amdgcn_s_memrealtime();      \
    asm volatile("" ::: "memory");                         \
  } while (0)
#define VEGAS_TL_FLUSH(buf, waves)                                                                              \
  do {                                                                                                          \
    if ((buf) != nullptr && (threadIdx.x & 63) == 0) {                                                          \
      const unsigned lin = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);                      \
      unsigned long long* tl_dst = (buf) + (static_cast<size_t>(lin) * (waves) + (threadIdx.x >> 6)) * kTimelineEvents; \
      for (int tl_i = 0; tl_i < kTimelineEvents; ++tl_i) tl_dst[tl_i] = tl_stamps[tl_i];                        \
    }                                                                                                           \
  } while (0)
#else
#define VEGAS_TL_DECL
#define VEGAS_TL(ev)
#define VEGAS_TL_FLUSH(buf, waves)
#endif

// Leading kernel arguments of the streaming kernels: the fields of SplitParams that the first memory requests (page
// ids, sequence length, query rows) depend on -- 14 dwords, all that can be preloaded.  Leading scalar arguments are preloaded into scalar registers when a wave starts
// (the library is built with kernel-argument preloading); the copies inside SplitParams are then not read.
#define VEGAS_SPLIT_HOT_PARAMS                                                                                     \
  const int32_t *hot_table, const int32_t *hot_lens, int2 *hot_plan, const uint16_t *hot_q, int32_t hot_table_stride, \
      int32_t hot_chunk_tokens, int32_t hot_Hkv, int32_t hot_row_blocks, int32_t hot_G, int32_t hot_Hq
#define VEGAS_SPLIT_HOT_ASSIGN(p)            \
  do {                                       \
    (p).table = hot_table;                   \
    (p).lens = hot_lens;                     \
    (p).plan = hot_plan;                     \
    (p).q = hot_q;                           \
    (p).table_stride = hot_table_stride;     \
    (p).chunk_tokens = hot_chunk_tokens;     \
    (p).Hkv = hot_Hkv;                       \
    (p).row_blocks = hot_row_blocks;         \
    (p).G = hot_G;                           \
    (p).Hq = hot_Hq;                         \
    (p).g = hot_Hq / hot_Hkv;                \
    (p).R = hot_G * (p).g;                   \
  } while (0)
#define VEGAS_SPLIT_HOT_ARGS(sp)                                                                                   \
  (sp).table, (sp).lens, (sp).plan, (sp).q, (sp).table_stride, (sp).chunk_tokens, (sp).Hkv, (sp).row_blocks, (sp).G, \
      (sp).Hq

struct CombineParams {
  const float* part_o;
  const float2* part_ml;
  const int32_t* lens;
  uint16_t* out;            // bf16 [B, G, Hq, D]
  int32_t G, g, R, Hq, Hkv, chunk_tokens, nsplit, max_tokens;
  int32_t window;           // > 0: chunks wholly before token n - G - window + 1 were skipped and hold nothing
  int32_t D;                // head dimension (128 or 64) = threads per row
  const int2* plan;         // balanced chunking (or nullptr): [B] (first partial slot, chunk tokens)
  int32_t slots_total;      // balanced chunking: partial slots per KV head
};

// Leading (preloaded) kernel arguments of the one-round-trip merge kernel: everything its requests depend on.
#define VEGAS_COMBINE_HOT_PARAMS                                                                                   \
  const float *hot_part_o, const float2 *hot_part_ml, const int32_t *hot_lens, const int2 *hot_plan, int32_t hot_R, \
      int32_t hot_Hkv, int32_t hot_nsplit, int32_t hot_chunk_tokens, int32_t hot_D, int32_t hot_slots_total
#define VEGAS_COMBINE_HOT_ASSIGN(p)          \
  do {                                       \
    (p).part_o = hot_part_o;                 \
    (p).part_ml = hot_part_ml;               \
    (p).lens = hot_lens;                     \
    (p).plan = hot_plan;                     \
    (p).R = hot_R;                           \
    (p).Hkv = hot_Hkv;                       \
    (p).nsplit = hot_nsplit;                 \
    (p).chunk_tokens = hot_chunk_tokens;     \
    (p).D = hot_D;                           \
    (p).slots_total = hot_slots_total;       \
  } while (0)
#define VEGAS_COMBINE_HOT_ARGS(cp) \
  (cp).part_o, (cp).part_ml, (cp).lens, (cp).plan, (cp).R, (cp).Hkv, (cp).nsplit, (cp).chunk_tokens, (cp).D, (cp).slots_total

// The rows of one KV head (row = t * g + j for verification token t, head j of the group) whose page log-sum-exps
// are collected: all G g rows (Eq. 2), or the g rows of the first verification token and the g rows of the bonus
// token (Eq. 3; with G <= 2 that is every row).  Only these are written and read back.
__host__ __device__ __forceinline__ int collected_count(int collect_rows, int G, int g) {
  return (collect_rows == 1 || G <= 2) ? G * g : 2 * g;
}
__device__ __forceinline__ int collected_row(int ci, int collect_rows, int G, int g) {   // ci-th collected row
  return (collect_rows == 1 || G <= 2 || ci < g) ? ci : ci + (G - 2) * g;
}

// First chunk that any row of a (windowed) verification call can see.
__device__ __forceinline__ int first_live_chunk(int n, int G, int window, int chunk_tokens) {
  if (window <= 0) return 0;
  const int lo = n - G - window + 1;
  return lo > 0 ? lo / chunk_tokens : 0;
}

// Where the chunk partials of sequence b live and how long its chunks are.  Partial slot of (KV head h, chunk s):
// off + h * stride_h + s.  Uniform chunking: every (sequence, head) column owns nsplit slots of chunk_tokens
// tokens.  Balanced chunking: the slots of one head are shared by all sequences, sequence b starts at plan[b].x
// and its chunks are plan[b].y tokens long.  `last`: the largest s that still is a slot of the workspace (loads
// of slots past a column's chunks are clamped to it and discarded).
struct ColumnSlots {
  int64_t off;
  int32_t stride_h, chunk, last;
};
__device__ __forceinline__ ColumnSlots column_slots(const int2* plan, int slots_total, int b, int Hkv, int nsplit,
                                                    int chunk_tokens) {
  ColumnSlots c;
  if (plan) {
    const int2 e = plan[b];
    c.off = e.x;
    c.stride_h = slots_total;
    c.chunk = e.y > 0 ? e.y : 1;
    c.last = slots_total - 1 - e.x;
  } else {
    c.off = static_cast<int64_t>(b) * Hkv * nsplit;
    c.stride_h = nsplit;
    c.chunk = chunk_tokens;
    c.last = nsplit - 1;
  }
  return c;
}

// Balanced chunking of a batch (B <= 64 sequences, lengths < 2^24), computed identically by every wave that
// calls it, from the lengths alone (the host does not know them).  J workgroups per KV head are given to the
// sequences so that the longest chunk is as short as possible: with C the smallest chunk length for which
// sum_b ceil(n_b / C) <= J, sequence b is cut into s_b = ceil(n_b / C) equal chunks (multiples of `unit` tokens).
// J is j1 (one launch wave of workgroups) unless the lengths are so ragged that the chunks of that plan would
// leave more than a tenth of the wave idle; then it is j2 (two waves of half-size chunks, handed out longest
// first, which evens the waves out).  No chunk is longer than cap_units * unit tokens (what a workgroup can park
// in LDS); a batch too long for J chunks of that size simply takes more slots.  Slot ranges [P_b, P_b + s_b)
// are laid out by descending chunk length, so workgroups start in that order; slot j maps to chunk j - P_b of
// the sequence whose range holds it.
struct BalancedSlot {
  int32_t b, split, chunk;      // b < 0: slot j is not used
};
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
  return x;
}
// ceil(x / d) for 0 <= x < 2^23, 1 <= d < 2^23 (a float reciprocal and one correction step instead of an integer division)
__device__ __forceinline__ uint32_t ceil_div_small(uint32_t x, uint32_t d) {
  uint32_t q = static_cast<uint32_t>(static_cast<float>(x) * __builtin_amdgcn_rcpf(static_cast<float>(d)));
  q = q * d > x ? q - 1u : q;                                   // (the estimate is off by one at most)
  q = (q + 1u) * d <= x ? q + 1u : q;                           // q = floor(x / d)
  return q * d < x ? q + 1u : q;
}
// Smallest C >= 1 (in units) with sum over lanes of ceil(nu / C) <= J; nu is this lane's length in units (< 2^18),
// total their sum, longest their maximum (the condition always holds there when J >= number of sequences, and
// nothing changes beyond it).  No plan can beat ceil(total / J), and a batch of equal lengths meets it, so the
// search starts there and widens its steps before it bisects: one evaluation for a uniform batch.
__device__ __forceinline__ uint32_t balanced_chunk_units(uint32_t nu, uint32_t total, uint32_t longest, uint32_t J) {
  auto fits = [&](uint32_t c) { return wave_sum_u32(ceil_div_small(nu, c)) <= J; };
  uint32_t lo = (total + J - 1u) / J;                           // wave-uniform from here on
  lo = lo < 1u ? 1u : lo;
  if (lo >= longest || fits(lo)) return lo < longest ? lo : longest;
  uint32_t step = (lo + 15u) / 16u, hi = lo + step;             // lo fails; find a length that fits
  while (hi < longest && !fits(hi)) { lo = hi; step *= 2u; hi = lo + step; }
  hi = hi < longest ? hi : longest;
  ++lo;                                                         // invariant: everything below lo fails, hi fits (or is the end)
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (fits(mid)) hi = mid; else lo = mid + 1u;
  }
  return lo;
}
__device__ __forceinline__ BalancedSlot balanced_slot(const int32_t* lens, int B, int max_tokens, int j1, int j2,
                                                      int cap_units, int unit, int j, int2* plan_out) {
  const int lane = threadIdx.x & 63;
  uint32_t n = 0u;
  if (lane < B) {
    const int v = lens[lane];
    n = static_cast<uint32_t>(v < 0 ? 0 : (v > max_tokens ? max_tokens : v));
  }
  const uint32_t nu = (n + unit - 1u) / unit;                   // length in units
  const uint32_t total = wave_sum_u32(nu);
  BalancedSlot r;
  r.b = -1; r.split = 0; r.chunk = unit;
  if (total == 0u) {
    if (plan_out && lane < B) plan_out[lane] = make_int2(0, unit);
    return r;
  }
  uint32_t longest = nu;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) longest = max(longest, static_cast<uint32_t>(__shfl_xor(longest, off, 64)));
  uint32_t C = balanced_chunk_units(nu, total, longest, static_cast<uint32_t>(j1));
  if (j2 > j1 && 10u * total < 9u * static_cast<uint32_t>(j1) * C)   // less than 90 % of the wave would be busy
    C = balanced_chunk_units(nu, total, longest, static_cast<uint32_t>(j2));
  C = min(C, static_cast<uint32_t>(cap_units));
  const uint32_t s = (nu + C - 1u) / C;                         // chunks of this sequence (0 if empty)
  const int chunk = s > 0u ? static_cast<int>((nu + s - 1u) / s * unit) : 0;   // equal chunks, at most C units
  int P = 0;                                                    // slots of the sequences with longer chunks
  for (int i = 0; i < B; ++i) {
    const int ci = __shfl(chunk, i, 64);
    const int si = static_cast<int>(__shfl(s, i, 64));
    P += (ci > chunk || (ci == chunk && i < lane)) ? si : 0;
  }
  if (plan_out && lane < B) plan_out[lane] = make_int2(P, chunk > 0 ? chunk : unit);
  const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < B && s > 0u && j >= P && j < P + static_cast<int>(s));
  if (hit == 0ull) return r;
  const int b = __builtin_ctzll(hit);
  r.b = b;
  r.split = j - __shfl(P, b, 64);
  r.chunk = __shfl(chunk, b, 64);
  return r;
}

struct FinalizeParams {
  const float* part_o;
  const float2* part_ml;
  const float* page_lse;
  const int32_t* lens;
  uint16_t* out;            // bf16 [B, G, Hq, D]
  float* block_scores;      // [B, max_blocks]
  int32_t G, g, R, Hq, Hkv, chunk_tokens, nsplit, max_tokens;
  int32_t max_blocks, lse_pages, collect_rows;
  int32_t Rc;               // collected rows per KV head (collected_count)
  int32_t D;                // head dimension (128 or 64)
  const int2* plan;         // balanced chunking (or nullptr): [B] (first partial slot, chunk tokens)
  int32_t slots_total;      // balanced chunking: partial slots per KV head
  int32_t nC;               // logit metric: workgroups that sum the token partials (1024 tokens each)
  float tok_norm;           // logit metric: softmax_scale / (collected rows * H_q)
  int32_t nA;               // workgroups that merge rows (two rows each); the rest score pages
  float inv_norm;
};

struct SelectParams {
  const float* block_scores;
  const int32_t* block_table;
  const int32_t* seq_lens;
  const int32_t* budgets;   // or nullptr
  int32_t* sel_table;
  int32_t* sel_seq_lens;
  int32_t budget_tokens, G, max_blocks, max_sel_blocks, max_tokens;
  int32_t key_cap;          // score keys that fit the kernel's dynamic LDS
  float budget_ratio;       // > 0: budget = ceil(ratio * seq_len) unless per-sequence budgets are given
};

// Token budget of one sequence: per-sequence value, or a sparsity ratio of its length (App. C), or the call's constant.
__device__ __forceinline__ int sequence_budget(const int32_t* budgets, float ratio, int constant, int b, int n) {
  int budget = budgets ? budgets[b] : (ratio > 0.f ? static_cast<int>(ceilf(ratio * static_cast<float>(n))) : constant);
  return budget < 0 ? 0 : budget;
}

struct ExtendParams {
  const int32_t* block_table;
  const int32_t* seq_lens;   // lengths after the append
  int32_t* sel_table;
  int32_t* sel_seq_lens;
  int32_t batch, num_new, max_blocks, max_sel_blocks, page_size;
};

}  // namespace vegas
