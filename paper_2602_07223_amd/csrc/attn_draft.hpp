// Draft-attention streaming kernel for up to 16 query rows per KV head (one draft token, GQA groups of up to 16
// heads), gfx950; 16-token pages, or the 1, 2, 4, 8-token pages of Sec. 4 / App. D through a template argument.
//
// Same arithmetic, chunking, partial-result layout and merge kernels as attn_split_kernel (Eq. 1 over the selected
// pages of Sec. 3.2, split over the selection), but shaped for a call that is a few microseconds long and whose
// waves are bound by what they have to issue: a draft call stacks g (typically 4 or 8) rows on a KV head, so a
// 32-row MFMA tile is seven eighths padding, and the time goes into instructions around the contractions.
//   * 16x16x32 bf16 MFMAs: S^T = K Q^T per page (M = the page's 16 tokens, N = 16 query rows, K = 32 head dims per
//     instruction) and O^T += V^T P^T per 16 head dims (M = head dims, N = rows, K = the tile's 32 tokens): half the
//     matrix-core time of the 32-row tile, 8 logits and 32 (D = 128) accumulators per lane instead of 16 and 64.
//   * K needs no LDS: lane (token i, dim group kg) loads the 16 bytes K[i][32 kk + 8 kg ..] straight into the A
//     operand's register layout (four lanes read 64 consecutive bytes of a token row).
//   * Q needs no LDS and no barrier: lane (row n, kg) loads Q[n][32 kk + 8 kg ..] into the B operand's layout once.
//   * The softmax weights leave the first MFMA as P[token 4 kg + r of page pg][row n] in lane (n, kg): taking the
//     second contraction's index as k = 8 kg + e <-> (page e / 4, token 4 kg + e % 4) makes {P of page 0, P of page 1}
//     the B operand as it stands, and V is loaded to match: lane (m, kg) reads 16 bytes (D / 16 head dims from
//     (D / 16) m on) of those eight tokens; one byte-permute per register pair builds each A operand, and output
//     block blk then holds head dims (D / 16) m' + blk.
//   * A row's running maximum is shared by the four lanes (n, 0..3): two lane-swap instructions per reduction.
// Loads run one tile ahead as in attn_split_kernel (K back into its registers once the first contraction has
// consumed them, V into a second register set); the four waves merge through LDS and write one partial, or the
// finished bf16 rows when the workgroup's chunk is the whole selection.
#pragma once
#include <type_traits>

#include "attn_split.hpp"
#include "vegas_common.hpp"

namespace vegas {

// Reductions over the four lanes l % 16 + {0, 16, 32, 48}; every lane gets the result.
__device__ __forceinline__ float quad_rows_max(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return half_max(fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1])));
}
__device__ __forceinline__ float quad_rows_sum(float x) {
  const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return half_sum(__uint_as_float(r[0]) + __uint_as_float(r[1]));
}

constexpr int kDraftWaves = 4;
constexpr int kDraftRows = 16;     // query rows (of one KV head) a workgroup can take

// Dynamic LDS of attn_draft16_kernel for R (<= 16) rows: the waves' rows for the merge, their row maxima and sums.
inline size_t draft16_lds_bytes(int R, int D) {
  return static_cast<size_t>(kDraftWaves) * R * red_pitch(D) * sizeof(float) +
         2 * static_cast<size_t>(kDraftWaves) * kDraftRows * sizeof(float);
}

// PS: log2 of the tokens per page of the selection table (4: 16-token pages; 0..3: the 1, 2, 4, 8-token pages of
// Sec. 4 / App. D).  With small pages a tile spans 32 >> PS pages: their ids are loaded one tile ahead into one
// register (lane e <-> page e of the tile), every lane fetches the id of each of its tokens with a lane permute and
// forms a 64-bit address of its own; everything after the loads is the 16-token code.
template <int D, int PS = 4>
__global__ __launch_bounds__(kDraftWaves * 64, 2) void attn_draft16_kernel(VEGAS_SPLIT_HOT_PARAMS, const SplitParams pfull) {
  VEGAS_TL_DECL;
  VEGAS_TL(kTlEntry);
  SplitParams p = pfull;                     // (see attn_split_kernel: the preloaded arguments)
  VEGAS_SPLIT_HOT_ASSIGN(p);
  static_assert(D == 128 || D == 64, "head dimension");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int NW = kDraftWaves;
  constexpr int KK = D / 32;                 // steps of the first contraction = K loads per page
  constexpr int NBLK = D / 16;               // 16-wide blocks of the output = head dims one V load covers
  constexpr int kRedPitch = red_pitch(D);
  using VReg = typename std::conditional<D == 128, u32x4, u32x2>::type;      // NBLK head dims of one token
  constexpr int TP = 32 >> (PS < 4 ? PS : 0);   // pages per tile on the small-page path
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = lane >> 5;
  const int l32 = lane & 31;
  const int l16 = lane & 15;                 // token of a page (K), query row (Q, S^T, O^T), head-dim group (V)
  const int kg = lane >> 4;                  // which 8 of a contraction step's 32 indices
  const int h = blockIdx.x;                  // grid (KV head, chunk, sequence)
  const int split = blockIdx.y;
  const int b = blockIdx.z;
  const int Rl = p.R;                        // rows of this KV head: one draft token, g heads (G = 1)

  // Physical page ids of the wave's next 32 tiles in one register, lane (k, half) <-> page `half` of tile
  // tile_first + k NW, requested before the length is known (see attn_split_kernel).
  const int32_t* table = p.table + static_cast<int64_t>(b) * p.table_stride;
  const int c0 = split * p.chunk_tokens;
  const int tile_first = c0 / kTile + wave;
  int pagevec = 0;
  auto table_entry = [&](int kbase) -> int {
    int page = 2 * (tile_first + (kbase + l32) * NW) + half;
    page = page < p.table_stride ? page : p.table_stride - 1;
    return table[page];
  };
  auto into_pool = [&](int raw) -> int {
    const int64_t ph = raw;
    return static_cast<int>(ph < 0 ? 0 : (ph >= p.num_pages ? p.num_pages - 1 : ph));
  };
  auto load_pagevec = [&](int kbase) { pagevec = into_pool(table_entry(kbase)); };
  // Small pages: ids of the TP pages of this wave's tile k, lane e (mod TP) <-> page e of the tile.
  auto ids_entry = [&](int k) -> int {
    int page = (tile_first + k * NW) * TP + (lane & (TP - 1));
    page = page < p.table_stride ? page : p.table_stride - 1;
    return table[page];
  };

  // ---- one round trip for everything the preloaded arguments can address: table entry, length, query rows; the
  //      rest of the argument block is pulled in one go meanwhile (see attn_split_kernel)
  int first_entry = PS == 4 ? table_entry(0) : ids_entry(0);
  int n = p.lens[b];
  u32x4 qreg[KK];
  {
    const unsigned char* qbase = uniform_ptr(reinterpret_cast<const unsigned char*>(
        p.q + (static_cast<int64_t>(b) * p.Hq + h * p.g) * D));
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      qreg[kk] = u32x4{0u, 0u, 0u, 0u};      // rows past the group's heads: zeros
      if (l16 < Rl) qreg[kk] = gload<u32x4, false>(qbase, static_cast<uint32_t>(l16 * D + 32 * kk + 8 * kg) * 2u);
    }
  }
  asm volatile("" : "+s"(p.k), "+s"(p.v), "+s"(p.page_stride), "+s"(p.token_stride), "+s"(p.head_stride),
               "+s"(p.num_pages), "+s"(p.out_direct));
  asm volatile("" : "+s"(p.max_tokens), "+s"(p.nsplit), "+s"(p.scale_log2e), "+s"(p.part_o), "+s"(p.part_ml));
  asm volatile("" : "+v"(first_entry));
  float* red = reinterpret_cast<float*>(smem);                     // [wave][row][D] (padded rows)
  float* sm_m = red + NW * Rl * kRedPitch;                         // [wave][16] row maxima
  float* sm_l = sm_m + NW * kDraftRows;                            // [wave][16] row sums
  const int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit + split;   // this workgroup's partial slot
  // (when the workgroup finishes the rows itself: G = 1, so the group's rows are consecutive)
  auto out_rows = [&]() -> uint16_t* { return p.out_direct + (static_cast<int64_t>(b) * p.Hq + h * p.g) * D; };
  int ids_cur = 0, ids_pending = 0;          // small pages: ids of the tile whose loads go out next; of the one after
  if constexpr (PS == 4) pagevec = into_pool(first_entry);
  else ids_cur = into_pool(first_entry);

  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  if (c0 >= n) {                             // nothing to do, no partial is read
    if (p.out_direct != nullptr) {           // no merge kernel follows: the rows of an empty sequence are zeros
      uint16_t* rows = out_rows();
      for (int e = tid; e < Rl * D; e += NW * 64) rows[e] = 0;
    }
    return;
  }
  VEGAS_TL(kTlLength);
  const int c1 = min(c0 + p.chunk_tokens, n);
  const int tile_end = (c1 + kTile - 1) / kTile;

  const int64_t head_off = static_cast<int64_t>(h) * p.head_stride;
  const uint32_t ts_bytes = static_cast<uint32_t>(p.token_stride) * 2u;
  const uint32_t k_lane_off = static_cast<uint32_t>(l16) * ts_bytes + static_cast<uint32_t>(kg) * 16u;
  const uint32_t v_lane_off = static_cast<uint32_t>(4 * kg) * ts_bytes + static_cast<uint32_t>(l16) * (2u * NBLK);
  auto page_base = [&](const uint16_t* cache, int ph) -> const unsigned char* {
    return uniform_ptr(reinterpret_cast<const unsigned char*>(cache + static_cast<int64_t>(ph) * p.page_stride + head_off));
  };
  // Small pages: byte address of token t (0..31, a per-lane value) of the tile whose page ids are in ids_cur.
  typedef const __attribute__((address_space(1))) unsigned char* gbytes;
  auto token_addr = [&](const uint16_t* cache, int t) -> gbytes {
    const int id = __shfl(ids_cur, t >> (PS & 3), 64);
    const int tokin = t & ((1 << (PS & 3)) - 1);
    const int64_t el = static_cast<int64_t>(id) * p.page_stride + static_cast<int64_t>(tokin) * p.token_stride + head_off;
    return (gbytes)cache + el * 2;
  };
  // K load (pg, kk): token l16 of page pg, head dims 32 kk + 8 kg .. + 7
  auto issue_k = [&](int k, u32x4 (&kr)[2][KK]) {
    if constexpr (PS != 4) {
      typedef const __attribute__((address_space(1))) u32x4* gp;
#pragma unroll
      for (int pg = 0; pg < 2; ++pg) {
        const gbytes row = token_addr(p.k, 16 * pg + l16) + kg * 16;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) kr[pg][kk] = *(gp)(row + kk * 64);
      }
      return;
    }
    if ((k & 31) == 0 && k > 0) load_pagevec(k);
    const unsigned char* kb0 = page_base(p.k, __builtin_amdgcn_readlane(pagevec, k & 31));
    const unsigned char* kb1 = page_base(p.k, __builtin_amdgcn_readlane(pagevec, 32 + (k & 31)));
#pragma unroll
    for (int pg = 0; pg < 2; ++pg)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) kr[pg][kk] = gload<u32x4, false>((pg ? kb1 : kb0) + kk * 64, k_lane_off);
  };
  // V load e: token 4 kg + e % 4 of page e / 4, head dims NBLK l16 .. + NBLK - 1
  auto issue_v = [&](int k, VReg (&vr)[8]) {
    if constexpr (PS != 4) {
      typedef const __attribute__((address_space(1))) VReg* gp;
#pragma unroll
      for (int e = 0; e < 8; ++e) vr[e] = *(gp)(token_addr(p.v, 16 * (e >> 2) + 4 * kg + (e & 3)) + l16 * (2 * NBLK));
      return;
    }
    const unsigned char* vb0 = page_base(p.v, __builtin_amdgcn_readlane(pagevec, k & 31));
    const unsigned char* vb1 = page_base(p.v, __builtin_amdgcn_readlane(pagevec, 32 + (k & 31)));
#pragma unroll
    for (int e = 0; e < 8; ++e)
      vr[e] = gload<VReg, false>((e < 4 ? vb0 : vb1) + static_cast<uint32_t>(e & 3) * ts_bytes, v_lane_off);
  };

  u32x4 kr[2][KK];
  VReg va[8], vb[8];
  if constexpr (PS != 4) ids_pending = into_pool(ids_entry(1));     // (requested before tile 0's loads: it is back first)
  if (tile_first < tile_end) {
    issue_k(0, kr);
    issue_v(0, va);
  }
  VEGAS_TL(kTlLoadsIssued);
  VEGAS_TL(kTlQueries);

  // ---- running state of lane (row n, kg): the row maximum (the same in the row's four lanes), this lane's share
  //      of the row sum, and acc[blk][r] = O[n][NBLK (4 kg + r) + blk]
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 acc[NBLK];
#pragma unroll
  for (int blk = 0; blk < NBLK; ++blk) acc[blk] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto step = [&](int k, VReg (&vcur)[8], VReg (&vnxt)[8], auto has_next_tag) {
    constexpr bool has_next = decltype(has_next_tag)::value;
    const int tok0 = (tile_first + k * NW) * kTile;
    f32x4 st[2] = {f32x4{0.f, 0.f, 0.f, 0.f}, f32x4{0.f, 0.f, 0.f, 0.f}};     // st[pg][r]: token 4 kg + r of page pg, row l16
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
#pragma unroll
      for (int pg = 0; pg < 2; ++pg)
        st[pg] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kr[pg][kk]),
                                                         __builtin_bit_cast(bf16x8, qreg[kk]), st[pg], 0, 0, 0);
    if (has_next) {
      if constexpr (PS != 4) {               // the next tile's ids are here (requested a tile ago); ask for the ones after
        ids_cur = ids_pending;
        ids_pending = into_pool(ids_entry(k + 2));
      }
      issue_k(k + 1, kr);
      issue_v(k + 1, vnxt);
    }
    const bool tail = tok0 + kTile > n;      // (chunks are whole tiles: only the sequence's end cuts into one)
    if (tail) {
#pragma unroll
      for (int pg = 0; pg < 2; ++pg)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (tok0 + 16 * pg + 4 * kg + r >= n) st[pg][r] = -INFINITY;
    }
    float tmax = fmaxf(fmaxf(fmaxf(st[0][0], st[0][1]), fmaxf(st[0][2], st[0][3])),
                       fmaxf(fmaxf(st[1][0], st[1][1]), fmaxf(st[1][2], st[1][3])));
    tmax = quad_rows_max(tmax) * p.scale_log2e;           // scale > 0: max commutes with scaling
    const float m_new = fmaxf(m_run, tmax);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    float pw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) pw[i] = fast_exp2(__builtin_fmaf(st[i >> 2][i & 3], p.scale_log2e, -m_use));
    // The row sum adds the weights as the second contraction sees them, i.e. rounded to bf16: numerator and
    // denominator of Eq. 1 then carry the same rounding errors, which cancel where one key dominates (the output
    // is a convex combination of V rows again) and do no harm elsewhere.
    bf16x8 pb;
    float pr[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      pb[i] = static_cast<__bf16>(pw[i]);
      pr[i] = static_cast<float>(pb[i]);
    }
    l_run = l_run * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7]));
    const float m_before = m_run;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f && m_before != -INFINITY) != 0) {   // (no key seen yet: sums still zero)
#pragma unroll
      for (int blk = 0; blk < NBLK; ++blk) acc[blk] *= alpha;
    }
    if (tail) {                              // slots past the end may hold anything: feed zeros
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (tok0 + 16 * (e >> 2) + 4 * kg + (e & 3) >= n) vcur[e] = VReg{};
    }
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
      u32x4 raw;
#pragma unroll
      for (int j = 0; j < 4; ++j)              // head dim blk of this lane's group, tokens 2 j and 2 j + 1 of its eight
        raw[j] = __builtin_amdgcn_perm(vcur[2 * j + 1][blk >> 1], vcur[2 * j][blk >> 1],
                                       (blk & 1) ? 0x07060302u : 0x05040100u);
      acc[blk] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, raw), pb, acc[blk], 0, 0, 0);
    }
#ifdef VEGAS_TIMELINE
    if (tl_stamps[kTlFirstTile] == 0) VEGAS_TL(kTlFirstTile);
#endif
  };

  // ---- stream the chunk's tiles (the last one peeled: prefetches are unconditional, load-counter waits exact)
  if (tile_first < tile_end) {
    const int ntiles = (tile_end - tile_first + NW - 1) / NW;      // this wave's tiles
    using yes = std::integral_constant<bool, true>;
    using no = std::integral_constant<bool, false>;
    int k = 0;
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

  // ---- merge the waves: row maxima meet in LDS, every wave rescales and parks its rows as [wave][row][d], all
  //      threads add the waves' copies and write the workgroup's partial (or the finished rows)
  VEGAS_TL(kTlStreamed);
  if (kg == 0) sm_m[wave * kDraftRows + l16] = m_run;
  __syncthreads();
  VEGAS_TL(kTlMerged);
  {
    float mw = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mw = fmaxf(mw, sm_m[w * kDraftRows + l16]);
    const float m_fin = (mw == -INFINITY) ? 0.f : mw;
    const float sc = fast_exp2(m_run - m_fin);
    const float lsum = quad_rows_sum(l_run * sc);
    if (kg == 0) sm_l[wave * kDraftRows + l16] = lsum;
    if (l16 < Rl) {
      float* dst = red + (wave * Rl + l16) * kRedPitch;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int d0 = NBLK * (4 * kg + r);
        *reinterpret_cast<f32x4*>(dst + d0) = f32x4{acc[0][r] * sc, acc[1][r] * sc, acc[2][r] * sc, acc[3][r] * sc};
        if constexpr (D == 128)
          *reinterpret_cast<f32x4*>(dst + d0 + 4) = f32x4{acc[4][r] * sc, acc[5][r] * sc, acc[6][r] * sc, acc[7][r] * sc};
      }
    }
  }
  __syncthreads();
  constexpr int V4 = D / 4;
  constexpr int kSumTrips = (kDraftRows * V4 + NW * 64 - 1) / (NW * 64);
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
    // The only chunk of its (sequence, KV head): divide by the softmax denominator and write the bf16 rows (Eq. 1).
    uint16_t* const rows = out_rows();
#pragma unroll
    for (int it = 0; it < kSumTrips; ++it) {
      const int e = tid + it * NW * 64;
      if (e < Rl * V4) {
        const int row = e / V4;
        float lw = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) lw += sm_l[w * kDraftRows + row];
        const float inv = lw > 0.f ? 1.0f / lw : 0.f;       // (a row with no visible key: zeros)
        u32x2 packed;
        packed[0] = static_cast<uint32_t>(float_to_bf16_bits(sums[it][0] * inv)) |
                    (static_cast<uint32_t>(float_to_bf16_bits(sums[it][1] * inv)) << 16);
        packed[1] = static_cast<uint32_t>(float_to_bf16_bits(sums[it][2] * inv)) |
                    (static_cast<uint32_t>(float_to_bf16_bits(sums[it][3] * inv)) << 16);
        *reinterpret_cast<u32x2*>(rows + 4 * e) = packed;
      }
    }
    VEGAS_TL(kTlExit);
    VEGAS_TL_FLUSH(p.timeline, NW);
    return;
  }
  float* po = p.part_o + pbase * p.R * D;
#pragma unroll
  for (int it = 0; it < kSumTrips; ++it) {
    const int e = tid + it * NW * 64;
    if (e < Rl * V4) *reinterpret_cast<f32x4*>(po + 4 * e) = sums[it];
  }
  if (tid < Rl) {
    float mw = -INFINITY, lw = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      mw = fmaxf(mw, sm_m[w * kDraftRows + tid]);
      lw += sm_l[w * kDraftRows + tid];
    }
    p.part_ml[pbase * p.R + tid] = make_float2(mw, lw);
  }
  VEGAS_TL(kTlExit);
  VEGAS_TL_FLUSH(p.timeline, NW);
}

}  // namespace vegas
