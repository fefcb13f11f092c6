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
  float* trash;             // attn_pair_kernel: a word of the workspace that takes the stores of invalid elements
  int2* plan;               // balanced chunking (or nullptr): [B] (first partial slot, chunk tokens) per sequence,
                            // computed by every workgroup from the lengths and written here by workgroup 0
  int32_t batch;            // B (balanced chunking)
  int32_t slots_target;     // J: partial slots (= workgroups) per KV head the lengths are apportioned to
  int32_t slots_total;      // JS = J + B: slots per KV head the workspace holds
  int32_t chunk_unit;       // chunk lengths are multiples of this many tokens
  int64_t page_stride, token_stride, head_stride, num_pages;
  float scale_log2e;
};

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

// Balanced chunking of a ragged batch (B <= 64 sequences, lengths <= 2^24), computed identically by every wave
// that calls it.  The J >= B slots of a KV head go to the sequences so that the longest chunk is as short as
// possible: with C the smallest chunk length for which sum_b ceil(n_b / C) <= J, sequence b is cut into
// s_b = ceil(n_b / C) equal chunks (rounded up to `unit` tokens), and slot j maps to chunk j - P_b of the sequence
// whose slot range [P_b, P_b + s_b) holds it.  With as many workgroups as the GPU runs at once, every workgroup then streams
// about the same number of tokens in ONE launch wave, however ragged the batch is.
struct BalancedSlot {
  int32_t b, split, chunk;      // b < 0: slot j is not used
};
__device__ __forceinline__ BalancedSlot balanced_slot(const int32_t* lens, int B, int max_tokens, int J, int unit, int j,
                                                      int2* plan_out) {
  const int lane = threadIdx.x & 63;
  uint32_t n = 0u;
  if (lane < B) {
    const int v = lens[lane];
    n = static_cast<uint32_t>(v < 0 ? 0 : (v > max_tokens ? max_tokens : v));
  }
  uint32_t N = n;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) N += __shfl_xor(N, off, 64);
  BalancedSlot r;
  r.b = -1; r.split = 0; r.chunk = unit;
  if (N == 0u) {
    if (plan_out && lane < B) plan_out[lane] = make_int2(0, unit);
    return r;
  }
  // Smallest chunk length C (in units) for which sum_b ceil(n_b / C) <= J: bisection, 18 rounds cover 2^24 tokens.
  const uint32_t nu = (n + unit - 1u) / unit;                   // length in units
  uint32_t lo = 1u, hi = nu;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) hi = max(hi, static_cast<uint32_t>(__shfl_xor(hi, off, 64)));
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    uint32_t cnt = (nu + mid - 1u) / mid;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    if (cnt <= static_cast<uint32_t>(J)) hi = mid; else lo = mid + 1u;
  }
  const uint32_t s = (nu + lo - 1u) / lo;                       // chunks of this sequence (0 if empty)
  const int chunk = s > 0u ? static_cast<int>((nu + s - 1u) / s * unit) : unit;   // equal chunks, at most C
  uint32_t incl = s;                                            // inclusive prefix sum over lanes
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t o = __shfl_up(incl, off, 64);
    if (lane >= off) incl += o;
  }
  const int P = static_cast<int>(incl - s);
  if (plan_out && lane < B) plan_out[lane] = make_int2(P, chunk);
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
