// KV-streaming attention kernel for gfx950: one pass over a chunk of one sequence's paged bf16
// K/V for one KV head, for all (query row x GQA group) rows at once.
//
// What it computes (Eq. 1 of the paper, split over the context): for the R = G*g query rows that
// share KV head h, the un-normalised partial softmax(q K^T * scale) V over the chunk's tokens,
// with the running max and sum needed to merge chunks, and -- when COLLECT -- for every
// (row, page) the log2-sum-exp2 of the page's scaled logits, from which the verification pass
// later forms the page criticality of Eq. 2 / Eq. 3 (weights as the metric, App. B) without
// reading the cache a second time.
//
// Mapping to the hardware
//   * A workgroup = NW waves working on one (sequence, KV head, chunk); wave w takes the 32-token
//     tiles w, w+NW, ... of the chunk, so the workgroup streams a contiguous range of pages.
//   * Per tile a wave issues S^T = K Q^T as 32x32x16 bf16 MFMAs (M = tokens, N = query rows,
//     K = head_dim) and O^T += V^T P^T (M = head_dim, N = query rows, K = tokens).  With this
//     orientation the softmax weights leave the first MFMA already in the lane layout the second
//     one wants as its B operand, a row's statistics live in one lane pair (lanes l and l+32),
//     and both pages of the tile sit in separate registers, so page sums need no shuffles beyond
//     one half-wave exchange.
//   * K is loaded fully coalesced (four 256-byte token rows per 1 KB instruction), staged through
//     a wave-private LDS tile (rows padded to 272 bytes against bank conflicts) and re-read in
//     MFMA operand layout.
//   * V needs no staging: tokens are the contraction index of the second MFMA, so a lane reads
//     8 bytes (4 head dims) of one token per instruction -- 32 lanes cover one 256-byte row --
//     and two byte-permutes per register pair build the operand.
//   * All query rows of the GQA group (x G verification rows) are stacked in the N dimension, so
//     every K/V byte is loaded once per workgroup and never re-read.  The queries sit in LDS
//     (padded like K) and are shared by the workgroup's waves.  More than 32 rows per KV head are
//     split into 32-row blocks handled by sibling workgroups whose ids differ by the number of KV
//     heads: ids are dealt round-robin to the 8 XCDs, so siblings share an L2 and the second
//     reader of a K/V line is served from it -- HBM still sees each byte once.
//   * Loads run one tile ahead: as soon as K(current) has been handed to LDS, K(next) goes into
//     the same registers and V(next) into a second register set, so a wave keeps a full tile
//     (16 KB) in flight for the whole duration of the math.
//   * At the end the NW waves merge their (max, sum, O) through LDS and the workgroup writes one
//     partial result.
#pragma once
#include <type_traits>

#include "vegas_common.hpp"

namespace vegas {

// Both halves of the wave get op(x, x from the other half) with one VALU lane swap.
__device__ __forceinline__ float half_max(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_sum(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Per head dimension D (128, or 64 for the 2 KB/token shape of App. D): a K/Q row is 2 D bytes, padded by 16 bytes in
// LDS so that rows spread over the banks; the cross-wave merge buffer pads its rows by 4 floats.
constexpr int row_pitch(int D) { return 2 * D + 16; }
constexpr int red_pitch(int D) { return D + 4; }

// Query rows of one KV head -> LDS [rows][D / 8 chunks of 16 B] with padded rows, by all `threads` threads of the
// workgroup.  Tile row r holds row row0 + r of the head's R = G g rows (row = t g + j) for r < valid; later rows
// are zero.  with_sums (the logit metric, Sec. 3.2 footnote / App. B): rows `valid` and `valid + 1` carry the sum of
// the collected query rows of this KV head as a bf16 high part and a bf16 low part (together good to 2^-17).
template <int D>
__device__ __forceinline__ void load_queries_to_lds(unsigned char* qlds, const SplitParams& p, int b, int h, int rows,
                                                    int row0, int valid, bool with_sums, int tid, int threads) {
  constexpr int CH = D / 8;
  constexpr int pitch = row_pitch(D);
  for (int idx = tid; idx < rows * CH; idx += threads) {
    const int row = idx / CH, chunk = idx % CH;
    u32x4 raw = {0u, 0u, 0u, 0u};
    if (row < valid) {
      const int t = (row0 + row) / p.g, j = (row0 + row) % p.g;
      raw = *reinterpret_cast<const u32x4*>(
          p.q + ((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * D + chunk * 8);
    }
    if (with_sums && row == valid) {
      // sum over the collected rows (Eq. 2: all; Eq. 3: first draft row and bonus row) in ascending row order,
      // eight requests in flight at a time
      float sum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int c0 = 0; c0 < p.Rc; c0 += 8) {
        u32x4 qv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int r = collected_row(min(c0 + u, p.Rc - 1), p.collect_rows, p.G, p.g);
          const int t = r / p.g, j = r % p.g;
          qv[u] = *reinterpret_cast<const u32x4*>(
              p.q + ((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * D + chunk * 8);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          if (c0 + u >= p.Rc) continue;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            sum[2 * e] += bf16_bits_to_float(static_cast<uint16_t>(qv[u][e] & 0xFFFFu));
            sum[2 * e + 1] += bf16_bits_to_float(static_cast<uint16_t>(qv[u][e] >> 16));
          }
        }
      }
      u32x4 hi, lo;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint16_t h0 = float_to_bf16_bits(sum[2 * e]), h1 = float_to_bf16_bits(sum[2 * e + 1]);
        const uint16_t l0 = float_to_bf16_bits(sum[2 * e] - bf16_bits_to_float(h0));
        const uint16_t l1 = float_to_bf16_bits(sum[2 * e + 1] - bf16_bits_to_float(h1));
        hi[e] = static_cast<uint32_t>(h0) | (static_cast<uint32_t>(h1) << 16);
        lo[e] = static_cast<uint32_t>(l0) | (static_cast<uint32_t>(l1) << 16);
      }
      *reinterpret_cast<u32x4*>(qlds + valid * pitch + chunk * 16) = hi;
      *reinterpret_cast<u32x4*>(qlds + (valid + 1) * pitch + chunk * 16) = lo;
      continue;
    }
    if (with_sums && row == valid + 1) continue;                             // written together with row `valid`
    *reinterpret_cast<u32x4*>(qlds + row * pitch + chunk * 16) = raw;
  }
}

// The same copy in two phases, for the kernels' common case (no sum rows): the loads leave as soon as the workgroup
// knows its sequence and head -- they depend on nothing else, so they travel together with the first page-table
// request instead of after the first K/V requests -- and reach LDS later.  QI 16-byte pieces per thread.
template <int D, int QI>
__device__ __forceinline__ void issue_query_loads(u32x4 (&raw)[QI], const SplitParams& p, int b, int h, int rows, int row0,
                                                  int valid, int tid, int threads) {
  constexpr int CH = D / 8;
  // Row r of the KV head is token t = r / g, head j = r % g of the group.  r < 128, so the quotient comes exactly
  // from one reciprocal (a hardware integer division is two dozen instructions); the address is a wave-uniform
  // 64-bit base (sequence, KV head) plus a 32-bit lane offset.
  const float rcp_g = __builtin_amdgcn_rcpf(static_cast<float>(p.g));
  const unsigned char* base = uniform_ptr(reinterpret_cast<const unsigned char*>(
      p.q + (static_cast<int64_t>(b) * p.G * p.Hq + h * p.g) * D));
#pragma unroll
  for (int i = 0; i < QI; ++i) {
    const int idx = tid + i * threads;
    const int row = idx / CH, chunk = idx % CH;
    raw[i] = u32x4{0u, 0u, 0u, 0u};
    if (idx < rows * CH && row < valid) {
      const int r = row0 + row;
      const int t = static_cast<int>((static_cast<float>(r) + 0.5f) * rcp_g), j = r - t * p.g;
      raw[i] = gload<u32x4, false>(base, static_cast<uint32_t>((t * p.Hq + j) * D + chunk * 8) * 2u);
    }
  }
}
template <int D, int QI>
__device__ __forceinline__ void store_queries_to_lds(unsigned char* qlds, const u32x4 (&raw)[QI], int rows, int tid,
                                                     int threads) {
  constexpr int CH = D / 8;
  constexpr int pitch = row_pitch(D);
#pragma unroll
  for (int i = 0; i < QI; ++i) {
    const int idx = tid + i * threads;
    if (idx < rows * CH) *reinterpret_cast<u32x4*>(qlds + (idx / CH) * pitch + (idx % CH) * 16) = raw[i];
  }
}

// NW: waves per workgroup; WPS: waves per SIMD the register budget is sized for (2 -> at most
// 256 registers per lane).  One workgroup handles up to 32 query rows of one KV head.
// NT_LOADS: K/V are read with the non-temporal hint -- right for the verification pass that streams
// the cache once with one reader per line; wrong for draft (the next draft step re-reads the same
// pages) and for row-block siblings (the second reader wants the L2 hit).
// COLLECT: 0 nothing; 1 the log-sum-exp of every (row, page) -- page criticality from softmax weights;
// 2 the paper's own metric (Sec. 3.2 footnote, App. B): per-token sums of the collected rows' LOGITS.
// A sum of logits is linear in the query, sum_r q_r . k = (sum_r q_r) . k, so the sum of the collected
// query rows of this KV head rides along as two spare rows of the query tile (a bf16 high part and a
// bf16 low part, together good to 2^-17) and the first MFMA delivers the token sums for free.  The host puts
// them in the last row block of the KV head; when that block is full (or one row short of full) the last
// row block is one that holds nothing but those two rows (Rl = 0: it streams K like its siblings, parks the
// token sums, and writes no partial output).
// PS: log2 of the tokens per page of the table the kernel walks.  4 (16-token pages) is the path
// described above; 0..3 (1, 2, 4, 8-token pages: Sec. 4 drafts with one-token pages, App. D sweeps
// 1..16) is for draft calls only: a tile then spans 32 >> PS pages, every lane looks up the page of
// its own token, and the page ids travel one tile ahead through a small per-wave LDS ring.
// LOCAL: local ("sliding window") masking of a banded layer on top of the causal mask (verification without
// collection only); a separate instantiation so that the other variants keep their register budget.
// D: head dimension.  64 halves everything that scales with it: a 16-byte K load covers 8 token rows instead of
// 4, the first contraction has 4 steps, the output has 2 blocks of 32, a V load is 4 bytes (2 head dims).
template <int NW, int WPS, bool CAUSAL, int COLLECT, bool NT_LOADS, int PS = 4, bool LOCAL = false, int D = 128>
__global__ __launch_bounds__(NW * 64, WPS) void attn_split_kernel(VEGAS_SPLIT_HOT_PARAMS, const SplitParams pfull) {
  // What the first memory requests need arrives in scalar registers with the wave (kernel-argument preloading)
  // instead of through a load of the argument block: one dependent round trip less at the head of the kernel.
  VEGAS_TL_DECL;
  VEGAS_TL(kTlEntry);
  SplitParams p = pfull;
  VEGAS_SPLIT_HOT_ASSIGN(p);
  static_assert(PS == 4 || (!CAUSAL && COLLECT == 0 && !NT_LOADS), "small pages: draft calls only");
  static_assert(!LOCAL || (CAUSAL && COLLECT == 0), "local masking: verification without collection only");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  static_assert(D == 128 || D == 64, "head dimension");
  constexpr int NB = 1;                      // one 32-row block per workgroup
  constexpr int CH = D / 8;                  // 16-byte chunks of a K/Q row
  constexpr int TPI = 64 / CH;               // token rows one K load instruction covers
  constexpr int NK = 32 / TPI;               // K load instructions per tile
  constexpr int NBLK = D / 32;               // 32-wide blocks of the output's head dimension
  constexpr int kRowPitch = row_pitch(D);
  constexpr int kRedPitch = red_pitch(D);
  using VReg = typename std::conditional<D == 128, u32x2, uint32_t>::type;   // NBLK head dims of one token
  constexpr int TP = 32 >> (PS < 4 ? PS : 0);   // pages per tile on the small-page path
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int l32 = lane & 31;
  // Grid (KV head, row block + row_blocks * chunk, sequence): the indices come without a division (a few dozen
  // instructions each at the head of a kernel whose waves are issue-bound), and linear workgroup ids stay
  // head-fastest, so the 8 KV heads of a chunk still land on the 8 XCDs and sibling row blocks share one.
  const int h = blockIdx.x;
  const int rb = p.row_blocks == 1 ? 0 : static_cast<int>(blockIdx.y) % p.row_blocks;
  int split = p.row_blocks == 1 ? static_cast<int>(blockIdx.y) : static_cast<int>(blockIdx.y) / p.row_blocks;
  int b = blockIdx.z;
  int chunk_tokens = p.chunk_tokens;
  bool planned = false;                      // balanced chunking: the partial slot is the plan's
  if constexpr (CAUSAL && PS == 4 && !LOCAL) {
    if (p.plan) {                            // balanced chunking: slot j of this head -> (sequence, chunk)
      const int j = split;
      const BalancedSlot bs = balanced_slot(p.lens, p.batch, p.max_tokens, p.slots_target, p.slots_target2,
                                            p.chunk_cap_units, p.chunk_unit, j,
                                            ((blockIdx.x | blockIdx.y) == 0 && wave == 0) ? p.plan : nullptr);
      if (bs.b < 0) return;
      b = bs.b;
      split = bs.split;
      chunk_tokens = bs.chunk;
      planned = true;
    }
  }
  const int slot_j = p.row_blocks == 1 ? static_cast<int>(blockIdx.y) : static_cast<int>(blockIdx.y) / p.row_blocks;
  const int row0 = rb * 32;                  // first query row (of this KV head) handled here
  const int Rl = max(min(32, p.R - row0), 0);   // valid rows in this block (none in a block that only carries the sum rows)

  // Physical page ids of the wave's next 32 tiles live in one register: lane (k, half) holds the id of
  // page `half` of tile tile_first + k*NW.  They are read back with readlane, so the streaming loop
  // never waits on a page-table load.  The first batch is requested before the sequence length is
  // known (one memory round trip less at the head of the kernel): indices are clamped to the table
  // row, entries past the sequence's pages are read but never used.
  const int32_t* table = p.table + static_cast<int64_t>(b) * p.table_stride;
  const int c0 = split * chunk_tokens;
  const int tile_first = c0 / kTile + wave;
  int pagevec = 0;
  auto table_entry = [&](int kbase) -> int {           // (raw: clamped into the pool by the caller)
    int page = 2 * (tile_first + (kbase + l32) * NW) + half;
    page = page < p.table_stride ? page : p.table_stride - 1;
    return table[page];
  };
  auto into_pool = [&](int raw) -> int {
    const int64_t ph = raw;
    return static_cast<int>(ph < 0 ? 0 : (ph >= p.num_pages ? p.num_pages - 1 : ph));
  };
  auto load_pagevec = [&](int kbase) { pagevec = into_pool(table_entry(kbase)); };
  // Small pages: ids of the TP pages of this wave's tile k, lane e (mod TP) -> page e of the tile.
  auto ids_entry = [&](int k) -> int {
    int page = (tile_first + k * NW) * TP + (lane & (TP - 1));
    page = page < p.table_stride ? page : p.table_stride - 1;
    return table[page];
  };
  auto load_ids = [&](int k) -> int { return into_pool(ids_entry(k)); };

  // ---- The head of the kernel is a chain of memory round trips (arguments -> table and length -> K/V), each about
  //      a microsecond after a kernel boundary, in a kernel that runs for a few; so everything that can be asked for
  //      at once is.  (1) The first page-table request and the length need only the preloaded arguments: they leave
  //      first.  (2) The rest of the argument block is pulled into registers in one go while those two are in flight
  //      (left to itself the compiler fetches it piecemeal, each piece with a wait of its own, several of them between
  //      the table's arrival and the first K/V request).  (3) The query loads follow.  (4) Only then is the table
  //      entry waited for -- pinned here, or the compiler sinks the request below the length's early exit and turns
  //      two parallel trips into two consecutive ones.
  int first_entry = 0;
  if constexpr (PS == 4) first_entry = table_entry(0);
  else first_entry = ids_entry(0);
  int n = p.lens[b];
  // Query loads leave now (they depend on the sequence and the head only).
  constexpr int QI = (32 * CH + NW * 64 - 1) / (NW * 64);
  u32x4 qraw[QI];
  if constexpr (COLLECT != 2) issue_query_loads<D, QI>(qraw, p, b, h, NB * 32, row0, Rl, tid, NW * 64);
  asm volatile("" : "+s"(p.k), "+s"(p.v), "+s"(p.page_stride), "+s"(p.token_stride), "+s"(p.head_stride),
               "+s"(p.num_pages), "+s"(p.out_direct));
  asm volatile("" : "+s"(p.max_tokens), "+s"(p.lds_q_off), "+s"(p.nsplit), "+s"(p.scale_log2e), "+s"(p.part_o),
               "+s"(p.part_ml));
  asm volatile("" : "+v"(first_entry));
  // Dynamic LDS: [K staging, NW tiles + page lse | merge buffer NW x R rows][queries][row maxima][row sums][page-id ring]
  unsigned char* qlds = smem + p.lds_q_off;
  float* sm_m = reinterpret_cast<float*>(qlds + NB * 32 * kRowPitch);
  float* sm_l = sm_m + NW * NB * 32;
  // [pages of the chunk][Rl] page log-sum-exp (COLLECT only): behind the K tiles; the merge buffer may
  // overlap it because it is flushed (and a barrier passed) before the merge starts.
  float* lse_lds = reinterpret_cast<float*>(smem + NW * 32 * kRowPitch);
  float* tok_lds = lse_lds;                  // COLLECT == 2: [2][chunk tokens] high-part and low-part token sums
  int* ids_lds = reinterpret_cast<int*>(sm_l + NW * NB * 32) + wave * 64;   // [2 tiles][32 page ids] of this wave
  // this workgroup's partial slot
  const int64_t pbase = planned ? static_cast<int64_t>(h) * p.slots_total + slot_j
                                : (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit + split;
  int ids_pending = 0;
  if constexpr (PS == 4) pagevec = into_pool(first_entry);
  else ids_pending = into_pool(first_entry);

  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  if (c0 >= n) {                             // whole workgroup: nothing to do, no partial is read
    if (p.out_direct != nullptr) {           // no merge kernel follows: the rows of an empty sequence are zeros
      for (int e = tid; e < Rl * D; e += NW * 64) {
        const int r = row0 + e / D;
        p.out_direct[((static_cast<int64_t>(b) * p.G + r / p.g) * p.Hq + h * p.g + r % p.g) * D + e % D] = 0;
      }
    }
    return;
  }
  VEGAS_TL(kTlLength);
  const int c1 = min(c0 + chunk_tokens, n);
  // Local masking: no row sees a token before lo_min; chunks and tiles wholly before it are skipped.
  const int lo_min = LOCAL ? max(n - p.G - p.window + 1, 0) : 0;
  if (LOCAL && c0 / chunk_tokens < first_live_chunk(n, p.G, p.window, chunk_tokens)) return;
  const int nblk = (n + kPage - 1) / kPage;

  // ---- per-lane constants
  const int64_t head_off = static_cast<int64_t>(h) * p.head_stride;
  const int k_tok = lane / CH;               // K load i: token TPI*i + lane/CH of the tile ...
  const int k_chunk = lane % CH;             // ... 16-byte chunk lane%CH
  unsigned char* kst = smem + wave * (32 * kRowPitch);

  // Addresses are a wave-uniform 64-bit base (scalar registers) plus a 32-bit per-lane byte offset.
  const uint32_t ts_bytes = static_cast<uint32_t>(p.token_stride) * 2u;
  const uint32_t k_lane_off = static_cast<uint32_t>(k_tok) * ts_bytes + static_cast<uint32_t>(k_chunk) * 16u;
  const uint32_t v_lane_off = static_cast<uint32_t>(4 * half) * ts_bytes + static_cast<uint32_t>(l32) * (2u * NBLK);
  const int tile_end = (c1 + kTile - 1) / kTile;
  auto page_base = [&](const uint16_t* cache, int ph) -> const unsigned char* {
    return uniform_ptr(reinterpret_cast<const unsigned char*>(cache + static_cast<int64_t>(ph) * p.page_stride + head_off));
  };
  // tile index k counts this wave's tiles: tile = tile_first + k*NW
  // Small pages: byte address of token t (0..31) of tile k for this lane's KV head, from the ring slot of that tile.
  typedef const __attribute__((address_space(1))) unsigned char* gbytes;
  auto token_addr = [&](const uint16_t* cache, int k, int t) -> gbytes {
    const int id = ids_lds[(k & 1) * 32 + (t >> (PS & 3))];
    const int tokin = t & ((1 << (PS & 3)) - 1);
    const int64_t el = static_cast<int64_t>(id) * p.page_stride + static_cast<int64_t>(tokin) * p.token_stride + head_off;
    return (gbytes)cache + el * 2;
  };
  auto issue_k = [&](int k, u32x4 (&kr)[NK]) {
    if constexpr (PS != 4) {
#pragma unroll
      for (int i = 0; i < NK; ++i) {
        typedef const __attribute__((address_space(1))) u32x4* gp;
        kr[i] = *(gp)(token_addr(p.k, k, TPI * i + k_tok) + k_chunk * 16);
      }
      return;
    }
    if ((k & 31) == 0 && k > 0) load_pagevec(k);
    const int ph0 = __builtin_amdgcn_readlane(pagevec, k & 31);
    const int ph1 = __builtin_amdgcn_readlane(pagevec, 32 + (k & 31));
    const unsigned char* kb0 = page_base(p.k, ph0);
    const unsigned char* kb1 = page_base(p.k, ph1);
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      const unsigned char* base = ((TPI * i < kPage) ? kb0 : kb1) + static_cast<uint32_t>((TPI * i) & (kPage - 1)) * ts_bytes;
      kr[i] = gload<u32x4, NT_LOADS>(base, k_lane_off);
    }
  };
  // V load (s, jj): token 16s + 8(jj/4) + 4*half + jj%4 of the tile, head dims NBLK*l32 .. NBLK*l32 + NBLK-1
  auto issue_v = [&](int k, VReg (&vr)[16]) {
    if constexpr (PS != 4) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          typedef const __attribute__((address_space(1))) VReg* gp;
          vr[s * 8 + jj] = *(gp)(token_addr(p.v, k, 16 * s + 8 * (jj >> 2) + 4 * half + (jj & 3)) + l32 * (2 * NBLK));
        }
      }
      return;
    }
    const int ph0 = __builtin_amdgcn_readlane(pagevec, k & 31);
    const int ph1 = __builtin_amdgcn_readlane(pagevec, 32 + (k & 31));
    const unsigned char* vb0 = page_base(p.v, ph0);
    const unsigned char* vb1 = page_base(p.v, ph1);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const unsigned char* base = (s ? vb1 : vb0) + static_cast<uint32_t>(8 * (jj >> 2) + (jj & 3)) * ts_bytes;
        vr[s * 8 + jj] = gload<VReg, NT_LOADS>(base, v_lane_off);
      }
    }
  };

  // ---- first tile's loads go out before anything else
  u32x4 kr[NK];
  VReg va[16], vb[16];
  if constexpr (PS != 4) {                   // tile 0's page ids enter the ring; tile 1's are requested
    if (lane < TP) ids_lds[lane] = ids_pending;
    ids_pending = load_ids(1);
    wave_lds_fence();
  }
  if (tile_first < tile_end) {
    issue_k(0, kr);
    issue_v(0, va);
  }
  VEGAS_TL(kTlLoadsIssued);

  // ---- query rows -> LDS [row][CH chunks of 16 B], padded rows; rows past R are zero
  // COLLECT == 2: the last row block carries the sum of the collected query rows in rows Rl (high part) and Rl + 1 (low part)
  const bool has_extra = COLLECT == 2 && rb == p.row_blocks - 1;
  if constexpr (COLLECT == 2) load_queries_to_lds<D>(qlds, p, b, h, NB * 32, row0, Rl, has_extra, tid, NW * 64);
  else store_queries_to_lds<D, QI>(qlds, qraw, NB * 32, tid, NW * 64);
  int limit[NB];                             // last visible token of this lane's row
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int t = (l32 < Rl) ? (row0 + l32) / p.g : 0;
    limit[nb] = CAUSAL ? (n - p.G + t) : (n - 1);
  }
  __syncthreads();
  VEGAS_TL(kTlQueries);

  // ---- running state: lane (row, half) keeps the row max m (same in both halves), its half's
  //      partial sum l, and O^T accumulators acc[nb][blk][i] = O[row][NBLK*(8(i/4) + 4half + i%4) + blk]
  float m_run[NB], l_run[NB];
  f32x16 acc[NB][NBLK];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m_run[nb] = -INFINITY;
    l_run[nb] = 0.f;
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nb][blk][i] = 0.f;
  }

  // One tile: vcur holds this tile's V, vnxt receives the next tile's.
  // (has_next is a compile-time property of the call site: a prefetch under a run-time branch would
  // make the compiler's load-counter waits assume the worst case and drain the prefetch early.)
  auto step = [&](int k, VReg (&vcur)[16], VReg (&vnxt)[16], auto has_next_tag) {
    constexpr bool has_next = decltype(has_next_tag)::value;
    const int cur = tile_first + k * NW;
    const int tok0 = cur * kTile;
    // K: registers -> LDS tile [32 tokens][CH chunks of 16 B]; then refill the registers
#pragma unroll
    for (int i = 0; i < NK; ++i) {
      *reinterpret_cast<u32x4*>(kst + (TPI * i + k_tok) * kRowPitch + k_chunk * 16) = kr[i];
    }
    if (has_next) {
      if constexpr (PS != 4) {               // next tile's ids -> ring; the ids after that -> on their way
        if (lane < TP) ids_lds[((k + 1) & 1) * 32 + lane] = ids_pending;
        ids_pending = load_ids(k + 2);
        wave_lds_fence();
      }
      issue_k(k + 1, kr);
      issue_v(k + 1, vnxt);
    }
    wave_lds_fence();
    f32x16 st[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[nb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const int off = l32 * kRowPitch + half * 16 + kk * 32;
      const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kst + off));
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        const bf16x8 qb =
            __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qlds + nb * 32 * kRowPitch + off));
        st[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb, st[nb], 0, 0, 0);
      }
    }
    wave_lds_fence();

    if constexpr (COLLECT == 2) {
      // Columns Rl and Rl + 1 of S^T hold k_i . (high part) and k_i . (low part) for the tile's 32 tokens:
      // those two lanes (of each half) park them; register i covers token 8(i/4) + 4 half + i%4.
      if (has_extra && (l32 == Rl || l32 == Rl + 1)) {
        float* dst = tok_lds + (l32 - Rl) * chunk_tokens + (tok0 - c0) + 4 * half;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *reinterpret_cast<f32x4*>(dst + 8 * i4) =
              f32x4{st[0][4 * i4], st[0][4 * i4 + 1], st[0][4 * i4 + 2], st[0][4 * i4 + 3]};
      }
    }

    const bool tail = (tok0 + kTile > n) || (CAUSAL && (tok0 + kTile - 1 > n - p.G)) ||
                      (LOCAL && (tok0 < n - p.window || tok0 + kTile > c1));   // tiles the largest lower bound cuts into
    bf16x8 pb[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      if (tail) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = tok0 + 8 * (i >> 2) + 4 * half + (i & 3);
          // (the local variant may step on a tile past its chunk, see below: nothing there is visible)
          if (tok > limit[nb] || (LOCAL && (tok <= limit[nb] - p.window || tok >= c1))) st[nb][i] = -INFINITY;
        }
      }
      float tmax = st[nb][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, st[nb][i]);
      tmax = half_max(tmax) * p.scale_log2e;               // scale > 0: max commutes with scaling
      const float m_new = fmaxf(m_run[nb], tmax);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2(m_run[nb] - m_use);
      float pr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) pr[i] = fast_exp2(__builtin_fmaf(st[nb][i], p.scale_log2e, -m_use));
      float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { ps0 += pr[i]; ps1 += pr[8 + i]; }
      if constexpr (!CAUSAL && COLLECT == 0) {
        // Draft calls: the row sum adds the weights as the second contraction sees them (rounded to bf16), so that
        // numerator and denominator of Eq. 1 carry the same rounding errors; they cancel where one key dominates.
        // (Verification keeps the unrounded sums: the page scores are formed from them.)
        float rs = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) rs += static_cast<float>(static_cast<__bf16>(pr[i]));
        l_run[nb] = l_run[nb] * alpha + rs;
      } else {
        l_run[nb] = l_run[nb] * alpha + (ps0 + ps1);
      }
      float m_run_before[NB];
      m_run_before[nb] = m_run[nb];
      m_run[nb] = m_new;
      if (COLLECT == 1) {
        const float f0 = half_sum(ps0);
        const float f1 = half_sum(ps1);
        const int page = cur * 2 + half;                 // parked in LDS, written out in bulk at the end
        if (l32 < Rl && page < nblk) lse_lds[(page - c0 / kPage) * Rl + l32] = m_use + fast_log2(half ? f1 : f0);
      }
      // (nothing to rescale where the row had seen no key yet: its sums are still zero)
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f && m_run_before[nb] != -INFINITY) != 0) {
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[nb][blk][i] *= alpha;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) pb[nb][s2][jj] = static_cast<__bf16>(pr[s2 * 8 + jj]);
    }

    if (tok0 + kTile > n) {                  // slots past the end may hold anything: feed zeros
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
          const int tok = tok0 + 16 * s2 + 8 * (jj >> 2) + 4 * half + (jj & 3);
          if (tok >= n) vcur[s2 * 8 + jj] = VReg{};
        }
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
      for (int blk = 0; blk < NBLK; ++blk) {
        u32x4 raw;
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) {
          unsigned lo, hi;                     // the dword that holds head dim blk of two consecutive tokens
          if constexpr (D == 128) {
            lo = (blk < 2) ? vcur[s2 * 8 + 2 * pp][0] : vcur[s2 * 8 + 2 * pp][1];
            hi = (blk < 2) ? vcur[s2 * 8 + 2 * pp + 1][0] : vcur[s2 * 8 + 2 * pp + 1][1];
          } else {
            lo = vcur[s2 * 8 + 2 * pp];
            hi = vcur[s2 * 8 + 2 * pp + 1];
          }
          raw[pp] = __builtin_amdgcn_perm(hi, lo, (blk & 1) ? 0x07060302u : 0x05040100u);
        }
        const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[nb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[nb][s2], acc[nb][blk], 0, 0, 0);
      }
    }
#ifdef VEGAS_TIMELINE
    if (tl_stamps[kTlFirstTile] == 0) VEGAS_TL(kTlFirstTile);
#endif
  };

  // ---- stream the chunk's tiles
  if (tile_first < tile_end) {
    const int ntiles = (tile_end - tile_first + NW - 1) / NW;      // this wave's tiles
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int k = 0;
    if constexpr (LOCAL) {                   // this wave's first tile that reaches lo_min
      const int first_tile = lo_min / kTile;
      if (first_tile > tile_first) k = (first_tile - tile_first + NW - 1) / NW;
      if (k > 0 && k < ntiles) {             // the preloaded tile 0 is not the first one: fetch the right one
        if (k >= 32) load_pagevec(k & ~31);
        issue_k(k, kr);
        issue_v(k, va);
      }
    }
    if constexpr (LOCAL) {
      // (Local masking may leave this wave without a tile.)  This variant always steps two tiles at a time, the last
      // one possibly past the chunk's end, where every token is masked out: one loop shape less keeps it inside its
      // register budget.
      if (k < ntiles) {
        const int stop = k + ((ntiles - k + 1) & ~1);
        for (; k + 2 < stop; k += 2) {
          step(k, va, vb, yes{});
          step(k + 1, vb, va, yes{});
        }
        step(k, va, vb, yes{});
        step(k + 1, vb, va, no{});
      }
    } else {
      while (k + 2 < ntiles) {
        step(k, va, vb, yes{});
        step(k + 1, vb, va, yes{});
        k += 2;
      }
      if (k + 1 < ntiles) {
        step(k, va, vb, yes{});
        step(k + 1, vb, va, no{});
      } else {
        step(k, va, vb, no{});
      }
    }
  }

  // ---- merge the NW waves: exchange row maxima, rescale, park the valid rows of every wave's
  //      accumulators in LDS as [wave][row][d], then all threads add across waves and write the
  //      workgroup's partial result with consecutive threads on consecutive addresses.
  VEGAS_TL(kTlStreamed);
  if (half == 0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) sm_m[wave * (NB * 32) + nb * 32 + l32] = m_run[nb];
  }
  __syncthreads();                                       // also: every wave is done with its K tile
  VEGAS_TL(kTlMerged);
  if constexpr (COLLECT == 2) {
    // The chunk's token sums (high + low part) leave in one coalesced write; positions at or past the
    // end of the sequence are never read.
    if (has_extra) {
      float* dst = p.page_lse + (static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + c0;
      for (int e = tid; e < c1 - c0; e += NW * 64) dst[e] = tok_lds[e] + tok_lds[chunk_tokens + e];
    }
    __syncthreads();
  }
  if (COLLECT == 1) {
    // One contiguous, coalesced write of the chunk's page log-sum-exps (a store per tile inside the
    // streaming loop costs ~14 % of the kernel: small scattered writes disturb the read stream).
    const int pg0 = c0 / kPage;
    const int npg = min(nblk, (c1 + kPage - 1) / kPage) - pg0;
    float* dst = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + pg0) * p.Rc;
    if (Rl == p.R && p.Rc == p.R && (Rl & 3) == 0) {         // 16 bytes per thread and trip (rows of 4 k floats stay aligned)
      const f32x4* src4 = reinterpret_cast<const f32x4*>(lse_lds);
      f32x4* dst4 = reinterpret_cast<f32x4*>(dst);
#pragma unroll 2
      for (int e = tid; e < npg * (Rl >> 2); e += NW * 64) dst4[e] = src4[e];
    } else if (Rl == p.R && p.Rc == p.R) {
      for (int e = tid; e < npg * Rl; e += NW * 64) dst[e] = lse_lds[e];
    } else {                                 // only the collected rows, and of those the ones in this row block
      for (int e = tid; e < npg * p.Rc; e += NW * 64) {
        const int r = collected_row(e % p.Rc, p.collect_rows, p.G, p.g) - row0;
        if (r >= 0 && r < Rl) dst[e] = lse_lds[(e / p.Rc) * Rl + r];
      }
    }
    __syncthreads();
  }
  float* red = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int row = nb * 32 + l32;
    float mw = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mw = fmaxf(mw, sm_m[w * (NB * 32) + row]);
    const float m_use = (mw == -INFINITY) ? 0.f : mw;
    const float sc = fast_exp2(m_run[nb] - m_use);
    const float lsum = half_sum(l_run[nb] * sc);
    if (half == 0) sm_l[wave * (NB * 32) + row] = lsum;
    if (row < Rl) {
      float* dst = red + (wave * Rl + row) * kRedPitch;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int d0 = NBLK * (8 * (i >> 2) + 4 * half + (i & 3));
        if constexpr (D == 128) {
          *reinterpret_cast<f32x4*>(dst + d0) =
              f32x4{acc[nb][0][i] * sc, acc[nb][1][i] * sc, acc[nb][2][i] * sc, acc[nb][3][i] * sc};
        } else {
          *reinterpret_cast<f32x2*>(dst + d0) = f32x2{acc[nb][0][i] * sc, acc[nb][1][i] * sc};
        }
      }
    }
  }
  __syncthreads();
  // The workgroup's rows: every thread adds the waves' copies of four neighbouring head dims (16-byte LDS reads, all
  // of a thread's reads issued before the first is used) -- the tail of a kernel this short is worth its microsecond.
  constexpr int V4 = D / 4;
  constexpr int kSumTrips = (32 * V4 + NW * 64 - 1) / (NW * 64);
  f32x4 sums[kSumTrips];
  const int sum_trips = (Rl * V4 + NW * 64 - 1) / (NW * 64);       // (few rows: the later trips have nothing to do)
#pragma unroll
  for (int it = 0; it < kSumTrips; ++it) {
    if (it < sum_trips) {
      const int e = min(tid + it * NW * 64, Rl * V4 - 1);
      const float* src = red + (e / V4) * kRedPitch + 4 * (e % V4);
      f32x4 acc4 = *reinterpret_cast<const f32x4*>(src);
#pragma unroll
      for (int w = 1; w < NW; ++w) acc4 += *reinterpret_cast<const f32x4*>(src + w * Rl * kRedPitch);
      sums[it] = acc4;
    }
  }
  if (p.out_direct != nullptr) {
    // The only chunk of its (sequence, KV head): the workgroup's sums are the whole result, so it divides by the
    // softmax denominator and writes the bf16 rows itself (Eq. 1); no partials, no merge kernel.
    const float rcp_g = __builtin_amdgcn_rcpf(static_cast<float>(p.g));     // (row / g without an integer division)
    uint16_t* const out_base = p.out_direct + (static_cast<int64_t>(b) * p.G * p.Hq + h * p.g) * D;
#pragma unroll
    for (int it = 0; it < kSumTrips; ++it) {
      const int e = tid + it * NW * 64;
      if (e < Rl * V4) {
        const int row = e / V4, d = 4 * (e % V4);
        float lw = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) lw += sm_l[w * (NB * 32) + row];
        const int r = row0 + row;
        const int rt = static_cast<int>((static_cast<float>(r) + 0.5f) * rcp_g), rj = r - rt * p.g;
        const float inv = lw > 0.f ? 1.0f / lw : 0.f;       // (a row with no visible key: zeros)
        u32x2 packed;
        packed[0] = static_cast<uint32_t>(float_to_bf16_bits(sums[it][0] * inv)) |
                    (static_cast<uint32_t>(float_to_bf16_bits(sums[it][1] * inv)) << 16);
        packed[1] = static_cast<uint32_t>(float_to_bf16_bits(sums[it][2] * inv)) |
                    (static_cast<uint32_t>(float_to_bf16_bits(sums[it][3] * inv)) << 16);
        *reinterpret_cast<u32x2*>(out_base + (rt * p.Hq + rj) * D + d) = packed;
      }
    }
    VEGAS_TL(kTlExit);
    VEGAS_TL_FLUSH(p.timeline, NW);
    return;
  }
  float* po = p.part_o + (pbase * p.R + row0) * D;
#pragma unroll
  for (int it = 0; it < kSumTrips; ++it) {
    const int e = tid + it * NW * 64;
    if (e < Rl * V4) *reinterpret_cast<f32x4*>(po + 4 * e) = sums[it];
  }
  if (tid < Rl) {
    float mw = -INFINITY, lw = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      mw = fmaxf(mw, sm_m[w * (NB * 32) + tid]);
      lw += sm_l[w * (NB * 32) + tid];
    }
    p.part_ml[pbase * p.R + row0 + tid] = make_float2(mw, lw);
  }
  VEGAS_TL(kTlExit);
  VEGAS_TL_FLUSH(p.timeline, NW);
}

// Dynamic LDS bytes of attn_split_kernel<NW, ...> when a workgroup holds up to `rows` (<= 32) valid rows.
inline size_t split_lds_tail_bytes(int NW, int D = 128) {
  return static_cast<size_t>(32) * row_pitch(D) + 2 * static_cast<size_t>(NW) * 32 * sizeof(float) +
         static_cast<size_t>(NW) * 64 * sizeof(int);                 // queries, row maxima and sums, page-id ring
}
// collect 1: the chunk's page log-sum-exps (chunk pages x rows floats) sit right behind the K tiles;
// collect 2: the chunk's token sums, high and low part (2 x chunk tokens floats).
inline size_t split_lds_bytes(int NW, int rows, int collect = 0, int chunk_tokens = 0, int D = 128) {
  size_t park = 0;
  if (collect == 1) park = static_cast<size_t>(chunk_tokens / kPage) * rows * sizeof(float);
  if (collect == 2) park = 2 * static_cast<size_t>(chunk_tokens) * sizeof(float);
  size_t stage = static_cast<size_t>(NW) * 32 * row_pitch(D) + park;
  const size_t red = static_cast<size_t>(NW) * rows * red_pitch(D) * sizeof(float);
  if (red > stage) stage = red;
  stage = (stage + 15) / 16 * 16;
  return stage + split_lds_tail_bytes(NW, D);
}

}  // namespace vegas
