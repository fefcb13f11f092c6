// KV-streaming verification kernel for 33..64 query rows per KV head (two 32-row blocks), gfx950.
//
// Same arithmetic and the same partial-result layout as attn_split_kernel (Eq. 1 split over the context, page
// log-sum-exps for Eq. 2 / Eq. 3, or the token sums of the logit metric), but the two row blocks are served from
// ONE read of K and V.  Sibling workgroups that each load the whole stream (the other way to serve two row blocks)
// hold the same bytes twice in their registers, so only half of what a CU has in flight is new to the memory
// system and the stream turns latency-bound.  Here instead:
//   * a workgroup of 4 waves is two PAIRS; pair p takes the 32-token tiles p, p+2, ... of the chunk;
//   * within a pair, wave `role` (0 or 1) owns row block `role` AND loads page `role` of every tile (16 tokens:
//     4 KB of K, 4 KB of V), two tiles ahead, into registers -- so a wave still keeps 16 KB in flight, all of it
//     bytes nobody else requests, and the non-temporal hint applies (one reader per line);
//   * both waves drop their page into the pair's K and V tiles in LDS, the workgroup meets at a barrier, and both
//     read the whole tile from there: K as the A operand of S^T = K Q^T, V as the A operand of O^T += V^T P^T
//     (8-byte reads in the same token/lane pattern the register path uses), then a second barrier frees the tile.
// What a step collects (the page log-sum-exps of its four pages for the collected rows, or the token sums of its 64 tokens) meets in a few
// hundred bytes of LDS and leaves right after the step's closing barrier in ONE store per thread, so a chunk may be
// arbitrarily long.  That store is unconditional and issued after the step's loads: invalid elements go to a
// scratch word instead of being branched around, because a store under a run-time branch would make the
// compiler's load-counter waits assume the worst and stall every step on the loads it has just issued (the
// counter covers loads and stores in issue order).  A bulk flush of a longer LDS ring every 2048 tokens was
// measured 15 % slower: the whole GPU drained its loads behind a synchronised burst of stores.
// Every pair runs the same number of steps (a pair whose last tile lies past the chunk works on a fully masked
// tile; that only happens in a sequence's last chunk because a full chunk holds an even number of tiles), and
// every load is unconditional with clamped page ids, so the barriers are uniform and the load counter waits exact.
#pragma once
#include <type_traits>

#include "attn_split.hpp"
#include "vegas_common.hpp"

namespace vegas {

constexpr int kPairWaves = 4;    // two pairs
constexpr int kPairs = 2;

template <int COLLECT, int D>
__global__ __launch_bounds__(kPairWaves * 64, 2) void attn_pair_kernel(VEGAS_SPLIT_HOT_PARAMS, const SplitParams pfull) {
  VEGAS_TL_DECL;                             // (profiling builds: per-wave phase stamps, see vegas_common.hpp)
  VEGAS_TL(kTlEntry);
  SplitParams p = pfull;                     // (see attn_split_kernel: the preloaded arguments)
  VEGAS_SPLIT_HOT_ASSIGN(p);
  static_assert(D == 128 || D == 64, "head dimension");
  // Dynamic LDS: [pair][K tile | V tile][page lse or token sums | merge buffer (aliases everything before)]
  //              [queries, 64 rows][row maxima][row sums]
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NW = kPairWaves, NP = kPairs;
  constexpr int CH = D / 8;                  // 16-byte chunks of a K/Q row
  constexpr int TPI = 64 / CH;               // token rows one K load instruction covers
  constexpr int NKH = kPage / TPI;           // K load instructions per page
  constexpr int NBLK = D / 32;               // 32-wide blocks of the output's head dimension
  constexpr int kRowPitch = row_pitch(D);
  constexpr int kRedPitch = red_pitch(D);
  constexpr int kTileBytes = 32 * kRowPitch;
  using VReg = typename std::conditional<D == 128, u32x2, uint32_t>::type;   // NBLK head dims of one token
  unsigned char* qlds = smem + p.lds_q_off;
  float* sm_m = reinterpret_cast<float*>(qlds + 64 * kRowPitch);
  float* sm_l = sm_m + NP * 64;
  float* lse_lds = reinterpret_cast<float*>(smem + NP * 2 * kTileBytes);   // COLLECT 1: [4 pages of the step][R]
  float* tok_lds = lse_lds;                                                // COLLECT 2: [2][64 tokens of the step]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int pr = wave >> 1, role = wave & 1;
  const int half = lane >> 5;
  const int l32 = lane & 31;
  // Grid (chunk, KV head, sequence): workgroup ids go round-robin to the XCDs, so with chunks fastest every XCD works
  // on all KV heads (measured 3.5 % faster for this kernel than one XCD per head; the other streaming kernels, which
  // are shorter, keep heads fastest).
  const int h = blockIdx.y;
  int split = blockIdx.x;
  int b = blockIdx.z;
  int chunk_tokens = p.chunk_tokens;
  int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit + split;   // this workgroup's partial slot
  if (p.plan) {                              // balanced chunking: slot j of this head -> (sequence, chunk)
    const int j = split;
    const BalancedSlot bs = balanced_slot(p.lens, p.batch, p.max_tokens, p.slots_target, p.slots_target2,
                                          p.chunk_cap_units, p.chunk_unit, j,
                                          ((blockIdx.x | blockIdx.y) == 0 && wave == 0) ? p.plan : nullptr);
    if (bs.b < 0) return;
    b = bs.b;
    split = bs.split;
    chunk_tokens = bs.chunk;
    pbase = static_cast<int64_t>(h) * p.slots_total + j;
  }
  const int row0 = 32 * role;                // first query row (of this KV head) of this wave's block
  const int Rl = min(32, p.R - row0);        // valid rows in it (R > 32)

  // Page ids of this wave's page of the pair's next 64 tiles, one per lane, read back with readlane.  Requested
  // before the sequence length is known; indices are clamped to the table row and ids to the pool.
  const int32_t* table = p.table + static_cast<int64_t>(b) * p.table_stride;
  const int c0 = split * chunk_tokens;
  const int tile0 = c0 / kTile;
  int pagevec = 0;
  auto load_pagevec = [&](int kbase) {
    int page = 2 * (tile0 + pr + (kbase + lane) * NP) + role;
    page = page < p.table_stride ? page : p.table_stride - 1;
    int64_t ph = table[page];
    ph = ph < 0 ? 0 : (ph >= p.num_pages ? p.num_pages - 1 : ph);
    pagevec = static_cast<int>(ph);
  };
  load_pagevec(0);

  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  if (c0 >= n) return;                       // whole workgroup: nothing to do, no partial is read
  VEGAS_TL(kTlLength);
  const int c1 = min(c0 + chunk_tokens, n);
  const int nblk = (n + kPage - 1) / kPage;
  const int tile_end = (c1 + kTile - 1) / kTile;
  // Steps of every pair, rounded up to an even number: the streaming loop below works on two register sets in turn,
  // and one loop shape (pairs of steps, the last pair without loads) keeps the kernel inside its register budget.  A
  // chunk that is a multiple of four tiles has an even count by itself; otherwise (the ragged end of a sequence, a
  // caller's chunk length) the extra step sees a tile past the chunk's end, which is masked out like any other token
  // the rows may not see.
  const int T = ((tile_end - tile0 + NP - 1) / NP + 1) & ~1;

  // ---- per-lane constants
  const int64_t head_off = static_cast<int64_t>(h) * p.head_stride;
  const int k_tok = lane / CH;               // K load i: token TPI*i + lane/CH of the page ...
  const int k_chunk = lane % CH;             // ... 16-byte chunk lane%CH
  unsigned char* kt = smem + pr * (2 * kTileBytes);
  unsigned char* vt = kt + kTileBytes;
  const uint32_t ts_bytes = static_cast<uint32_t>(p.token_stride) * 2u;
  const uint32_t k_lane_off = static_cast<uint32_t>(k_tok) * ts_bytes + static_cast<uint32_t>(k_chunk) * 16u;
  const uint32_t v_lane_off = static_cast<uint32_t>(4 * half) * ts_bytes + static_cast<uint32_t>(l32) * (2u * NBLK);
  auto page_base = [&](const uint16_t* cache, int ph) -> const unsigned char* {
    return uniform_ptr(reinterpret_cast<const unsigned char*>(cache + static_cast<int64_t>(ph) * p.page_stride + head_off));
  };
  // Loads of this wave's page of the pair's tile k: K rows TPI*i + lane/CH; V load jj: token
  // 8(jj/4) + 4*half + jj%4 of the page, head dims NBLK*l32 .. NBLK*l32 + NBLK-1.
  auto issue = [&](int k, u32x4 (&kr)[NKH], VReg (&vr)[8]) {
    if ((k & 63) == 0 && k > 0) load_pagevec(k);
    const int ph = __builtin_amdgcn_readlane(pagevec, k & 63);
    const unsigned char* kb = page_base(p.k, ph);
    const unsigned char* vb = page_base(p.v, ph);
#pragma unroll
    for (int i = 0; i < NKH; ++i) kr[i] = gload<u32x4, true>(kb + static_cast<uint32_t>(TPI * i) * ts_bytes, k_lane_off);
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      vr[jj] = gload<VReg, true>(vb + static_cast<uint32_t>(8 * (jj >> 2) + (jj & 3)) * ts_bytes, v_lane_off);
  };

  // ---- the first two tiles' loads go out before anything else (tile 1 may be a masked one: still a valid address)
  u32x4 kr0[NKH], kr1[NKH];
  VReg vr0[8], vr1[8];
  issue(0, kr0, vr0);
  issue(1, kr1, vr1);
  VEGAS_TL(kTlLoadsIssued);

  // ---- query rows -> LDS [64 rows][CH chunks of 16 B], padded rows; rows past R are zero.
  // COLLECT == 2: rows R (high part) and R + 1 (low part) carry the sum of the collected query rows.
  load_queries_to_lds<D>(qlds, p, b, h, 64, 0, p.R, COLLECT == 2, tid, NW * 64);
  VEGAS_TL(kTlQueries);                      // (queries written; the first step's barrier publishes them)
  const int xr = p.R - row0;                 // COLLECT 2: column of the high-part sum row inside block 1
  const bool has_extra = COLLECT == 2 && role == 1;
  // last visible token of this lane's row: the causal bound, and nothing past this workgroup's chunk
  const int limit = min(n - p.G + ((l32 < Rl) ? (row0 + l32) / p.g : 0), c1 - 1);
  // (the first barrier of the first step also publishes the queries)

  // ---- collection: the element of a step's collected values this thread stores (elements repeat when there are
  //      fewer than threads: the same value goes to the same address twice), and where step 0's copy goes
  // (Threads beyond the step's element count have nothing to store: their store goes to the workgroup's scratch word
  //  too.  Repeating elements instead -- the same value to the same address from a second thread -- costs real write
  //  requests: a step's values then leave in 256 stores instead of 160, or of 64.)
  int col_elem = 0, col_page = 0;
  float* const trash = p.trash + ((blockIdx.x + 8 * blockIdx.y) & 63);        // one of 64 words: workgroups do not all share one
  float* col_dst = trash;
  bool col_active = false;
  if constexpr (COLLECT == 1) {
    col_active = tid < 4 * p.Rc;
    const int e = tid % (4 * p.Rc);            // [page of the step][collected row]
    col_page = e / p.Rc;
    col_elem = col_page * p.R + collected_row(e % p.Rc, p.collect_rows, p.G, p.g);   // where it sits in LDS
    col_dst = p.page_lse + ((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + c0 / kPage) * p.Rc + e;
  }
  if constexpr (COLLECT == 2) {
    col_active = tid < kTile * NP;
    col_elem = tid % (kTile * NP);             // token of the step
    col_dst = p.page_lse + (static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + c0 + col_elem;
  }

  // ---- running state: lane (row, half) keeps the row max m (same in both halves), its half's partial sum l,
  //      and O^T accumulators acc[blk][i] = O[row][NBLK*(8(i/4) + 4half + i%4) + blk]
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 acc[NBLK];
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[blk][i] = 0.f;

  // One step of the pair: krs/vrs hold this wave's page of tile k and are refilled with tile k + 2.
  auto step = [&](int k, u32x4 (&krs)[NKH], VReg (&vrs)[8], auto load_tag) {
    constexpr bool load_next = decltype(load_tag)::value;
    const int cur = tile0 + pr + k * NP;
    const int tok0 = cur * kTile;
    // this wave's page -> the pair's K and V tiles
#pragma unroll
    for (int i = 0; i < NKH; ++i)
      *reinterpret_cast<u32x4*>(kt + (kPage * role + TPI * i + k_tok) * kRowPitch + k_chunk * 16) = krs[i];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      *reinterpret_cast<VReg*>(vt + (kPage * role + 8 * (jj >> 2) + 4 * half + (jj & 3)) * kRowPitch + l32 * (2 * NBLK)) = vrs[jj];
    if (load_next) issue(k + 2, krs, vrs);
    __syncthreads();                         // both pages of the tile are in LDS

    f32x16 st;
#pragma unroll
    for (int i = 0; i < 16; ++i) st[i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < D / 16; ++kk) {
      const int off = l32 * kRowPitch + half * 16 + kk * 32;
      const bf16x8 a = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(kt + off));
      const bf16x8 qb = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qlds + row0 * kRowPitch + off));
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qb, st, 0, 0, 0);
    }

    if constexpr (COLLECT == 2) {
      // Columns xr and xr + 1 of block 1's S^T hold k_i . (high part) and k_i . (low part) for the tile's tokens.
      if (has_extra && (l32 == xr || l32 == xr + 1)) {
        float* dst = tok_lds + (l32 - xr) * (kTile * NP) + pr * kTile + 4 * half;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
          *reinterpret_cast<f32x4*>(dst + 8 * i4) = f32x4{st[4 * i4], st[4 * i4 + 1], st[4 * i4 + 2], st[4 * i4 + 3]};
      }
    }

    const bool tail = (tok0 + kTile > c1) || (tok0 + kTile - 1 > n - p.G);
    if (tail) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int tok = tok0 + 8 * (i >> 2) + 4 * half + (i & 3);
        if (tok > limit) st[i] = -INFINITY;
      }
    }
    float tmax = st[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, st[i]);
    tmax = half_max(tmax) * p.scale_log2e;               // scale > 0: max commutes with scaling
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    float pw[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) pw[i] = fast_exp2(__builtin_fmaf(st[i], p.scale_log2e, -m_use));
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { ps0 += pw[i]; ps1 += pw[8 + i]; }
    l_run = l_run * alpha + (ps0 + ps1);
    const float m_before = m_run;
    m_run = m_new;
    if (COLLECT == 1) {
      const float f0 = half_sum(ps0);
      const float f1 = half_sum(ps1);                    // page 2 pr + half of the step
      if (l32 < Rl) lse_lds[(2 * pr + half) * p.R + row0 + l32] = m_use + fast_log2(half ? f1 : f0);
    }
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f && m_before != -INFINITY) != 0) {   // (no key seen yet: sums still zero)
#pragma unroll
      for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[blk][i] *= alpha;
    }
    bf16x8 pb[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) pb[s2][jj] = static_cast<__bf16>(pw[s2 * 8 + jj]);

    const bool past_end = tok0 + kTile > n;              // slots past the end may hold anything: feed zeros
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      VReg vcur[8];
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const int tl = 16 * s2 + 8 * (jj >> 2) + 4 * half + (jj & 3);
        vcur[jj] = *reinterpret_cast<const VReg*>(vt + tl * kRowPitch + l32 * (2 * NBLK));
        if (past_end && tok0 + tl >= n) vcur[jj] = VReg{};
      }
#pragma unroll
      for (int blk = 0; blk < NBLK; ++blk) {
        u32x4 raw;
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) {
          unsigned lo, hi;                     // the dword that holds head dim blk of two consecutive tokens
          if constexpr (D == 128) {
            lo = (blk < 2) ? vcur[2 * pp][0] : vcur[2 * pp][1];
            hi = (blk < 2) ? vcur[2 * pp + 1][0] : vcur[2 * pp + 1][1];
          } else {
            lo = vcur[2 * pp];
            hi = vcur[2 * pp + 1];
          }
          raw[pp] = __builtin_amdgcn_perm(hi, lo, (blk & 1) ? 0x07060302u : 0x05040100u);
        }
        acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, raw), pb[s2], acc[blk], 0, 0, 0);
      }
    }
    __syncthreads();                         // everybody is done with the tile: the next step may overwrite it
    // What the step collected leaves now (nobody writes the LDS values again before the next step's first barrier,
    // which no wave passes before every wave has read its element here).
    if constexpr (COLLECT == 1) {
      const bool ok = col_active && c0 / kPage + 4 * k + col_page < min(nblk, (c1 + kPage - 1) / kPage);
      float* dst = ok ? col_dst + static_cast<int64_t>(k) * (4 * p.Rc) : trash;
      *dst = lse_lds[col_elem];
    }
    if constexpr (COLLECT == 2) {
      const bool ok = col_active && c0 + (kTile * NP) * k + col_elem < c1;
      float* dst = ok ? col_dst + k * (kTile * NP) : trash;
      *dst = tok_lds[col_elem] + tok_lds[kTile * NP + col_elem];
    }
#ifdef VEGAS_TIMELINE
    if (tl_stamps[kTlFirstTile] == 0) VEGAS_TL(kTlFirstTile);
#endif
  };

  // ---- stream the chunk: T steps (even), the two register sets in turn; the last two steps issue no loads
  {
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int k = 0;
    for (; k + 2 < T; k += 2) {
      step(k, kr0, vr0, yes{});
      step(k + 1, kr1, vr1, yes{});
    }
    step(k, kr0, vr0, no{});
    step(k + 1, kr1, vr1, no{});
  }

  // ---- merge the two pairs, one row block after the other (the merge buffer aliases the tiles and the parked
  //      values): row maxima meet in LDS, every wave rescales, the waves of the block park their rows as
  //      [pair][row][d], all threads add the pairs and write the block's rows of the workgroup's partial.
  VEGAS_TL(kTlStreamed);
  if (half == 0) sm_m[pr * 64 + row0 + l32] = m_run;
  __syncthreads();                           // also: the collected values have been read out of LDS
  VEGAS_TL(kTlMerged);
  const float mw = fmaxf(sm_m[row0 + l32], sm_m[64 + row0 + l32]);
  const float m_fin = (mw == -INFINITY) ? 0.f : mw;
  const float sc = fast_exp2(m_run - m_fin);
  const float lsum = half_sum(l_run * sc);
  if (half == 0) sm_l[pr * 64 + row0 + l32] = lsum;
  float* red = reinterpret_cast<float*>(smem);
#pragma unroll 1
  for (int blk_rows = 0; blk_rows < 2; ++blk_rows) {
    const int rows = min(32, p.R - 32 * blk_rows);       // valid rows of this block
    if (role == blk_rows && l32 < rows) {
      float* dst = red + (pr * rows + l32) * kRedPitch;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int d0 = NBLK * (8 * (i >> 2) + 4 * half + (i & 3));
        if constexpr (D == 128) {
          *reinterpret_cast<f32x4*>(dst + d0) = f32x4{acc[0][i] * sc, acc[1][i] * sc, acc[2][i] * sc, acc[3][i] * sc};
        } else {
          *reinterpret_cast<f32x2*>(dst + d0) = f32x2{acc[0][i] * sc, acc[1][i] * sc};
        }
      }
    }
    __syncthreads();
    float* po = p.part_o + (pbase * p.R + 32 * blk_rows) * D;
    for (int e = tid; e < rows * D; e += NW * 64) {
      const int row = e / D, d = e % D;
      po[e] = red[row * kRedPitch + d] + red[(rows + row) * kRedPitch + d];
    }
    __syncthreads();
  }
  if (tid < p.R) {
    const float m2 = fmaxf(sm_m[tid], sm_m[64 + tid]);
    p.part_ml[pbase * p.R + tid] = make_float2(m2, sm_l[tid] + sm_l[64 + tid]);
  }
  VEGAS_TL(kTlExit);
  VEGAS_TL_FLUSH(p.timeline, NW);
}

// Dynamic LDS bytes of attn_pair_kernel for R rows per KV head.
inline size_t pair_lds_tail_bytes(int D) {
  return static_cast<size_t>(64) * row_pitch(D) + 2 * static_cast<size_t>(kPairs) * 64 * sizeof(float);   // queries, row maxima and sums
}
inline size_t pair_lds_bytes(int R, int collect, int D) {
  size_t park = 0;                                                         // what one step collects
  if (collect == 1) park = static_cast<size_t>(4) * R * sizeof(float);
  if (collect == 2) park = 2 * static_cast<size_t>(kTile * kPairs) * sizeof(float);
  size_t stage = static_cast<size_t>(kPairs) * 2 * 32 * row_pitch(D) + park;
  const size_t red = static_cast<size_t>(kPairs) * 32 * red_pitch(D) * sizeof(float);
  if (red > stage) stage = red;
  stage = (stage + 15) / 16 * 16;
  return stage + pair_lds_tail_bytes(D);
}

}  // namespace vegas
