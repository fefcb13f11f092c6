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
//     a wave-private, XOR-swizzled 8 KB LDS tile and re-read in MFMA operand layout.
//   * V needs no staging: tokens are the contraction index of the second MFMA, so a lane reads
//     8 bytes (4 head dims) of one token per instruction -- 32 lanes cover one 256-byte row --
//     and two byte-permutes per register pair build the operand.
//   * All query rows of the GQA group (x G verification rows) are stacked in the N dimension, so
//     every K/V byte is loaded once per workgroup and never re-read.
//   * Loads for tile i+1 are in flight (in registers) while tile i is computed.
//   * At the end the NW waves merge their (max, sum, O) through LDS and the workgroup writes one
//     partial result.
#pragma once
#include "vegas_common.hpp"

namespace vegas {

struct TileRegs {
  u32x4 k[8];    // K: load i covers tokens 4i .. 4i+3 of the tile (16 lanes x 16 B per token)
  u32x2 v[16];   // V: [s*8 + jj] = 4 head dims of token 16s + 8(jj/4) + 4*half + jj%4
};

template <int NB, int NW, bool CAUSAL, bool COLLECT>
__global__ __launch_bounds__(NW * 64) void attn_split_kernel(const SplitParams p) {
  // K staging (NW x 8 KB), reused for the cross-wave merge of the output accumulators.
  __shared__ __attribute__((aligned(16))) unsigned char smem[NW * 8192];
  __shared__ float sm_m[NW][NB * 32];
  __shared__ float sm_l[NW][NB * 32];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int half = lane >> 5;
  const int l32 = lane & 31;
  const int h = blockIdx.x % p.Hkv;
  const int split = blockIdx.x / p.Hkv;
  const int b = blockIdx.y;

  int n = p.lens[b];
  n = n < 0 ? 0 : (n > p.max_tokens ? p.max_tokens : n);
  const int c0 = split * p.chunk_tokens;
  if (c0 >= n) return;                       // whole workgroup: nothing to do, no partial is read
  const int c1 = min(c0 + p.chunk_tokens, n);
  const int nblk = (n + kPage - 1) / kPage;
  const int32_t* table = p.table + static_cast<int64_t>(b) * p.table_stride;

  // ---- query rows -> B operand of S^T = K Q^T: lane (row = l32, half) holds q[row][16kk+8half .. +8]
  bf16x8 qreg[NB][8];
  int limit[NB];                             // last visible token of this lane's row
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int row = nb * 32 + l32;
    const bool valid = row < p.R;
    const int t = valid ? row / p.g : 0;
    const int j = valid ? row % p.g : 0;
    const uint16_t* qp = p.q + ((static_cast<int64_t>(b) * p.G + t) * p.Hq + h * p.g + j) * kHeadDim + half * 8;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      u32x4 raw = {0u, 0u, 0u, 0u};
      if (valid) raw = *reinterpret_cast<const u32x4*>(qp + kk * 16);
      qreg[nb][kk] = __builtin_bit_cast(bf16x8, raw);
    }
    limit[nb] = CAUSAL ? (n - p.G + t) : (n - 1);
  }

  // ---- per-lane constant offsets
  const int64_t head_off = static_cast<int64_t>(h) * p.head_stride;
  // K load i: token 4i + lane/16 of the tile, 16-byte chunk lane%16
  const int k_tok = lane >> 4;
  const int k_chunk = lane & 15;
  // V load (s, jj): token 16s + 8(jj/4) + 4*half + jj%4, head dims 4*l32 .. 4*l32+3
  unsigned char* kst = smem + wave * 8192;

  auto issue = [&](int tile, TileRegs& r) {
    const int pg0 = tile * 2;
    const int pg1 = (pg0 + 1 < nblk) ? pg0 + 1 : pg0;          // a missing second page aliases the first
    int64_t ph0 = table[pg0];
    int64_t ph1 = table[pg1];
    ph0 = ph0 < 0 ? 0 : (ph0 >= p.num_pages ? p.num_pages - 1 : ph0);
    ph1 = ph1 < 0 ? 0 : (ph1 >= p.num_pages ? p.num_pages - 1 : ph1);
    const uint16_t* kb0 = p.k + ph0 * p.page_stride + head_off;
    const uint16_t* kb1 = p.k + ph1 * p.page_stride + head_off;
    const uint16_t* vb0 = p.v + ph0 * p.page_stride + head_off;
    const uint16_t* vb1 = p.v + ph1 * p.page_stride + head_off;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int slot = (4 * i + k_tok) & 15;
      const uint16_t* base = (i < 4) ? kb0 : kb1;
      r.k[i] = *reinterpret_cast<const u32x4*>(base + slot * p.token_stride + k_chunk * 8);
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const uint16_t* base = s ? vb1 : vb0;
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const int slot = 8 * (jj >> 2) + 4 * half + (jj & 3);
        r.v[s * 8 + jj] = *reinterpret_cast<const u32x2*>(base + slot * p.token_stride + l32 * 4);
      }
    }
  };

  // ---- running state: lane (row, half) keeps max m (shared by both halves), its half's partial sum l,
  //      and O^T accumulators acc[nb][blk][i] = O[row][d = 4*(8(i/4) + 4half + i%4) + blk]
  float m_run[NB], l_run[NB];
  f32x16 acc[NB][4];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    m_run[nb] = -INFINITY;
    l_run[nb] = 0.f;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nb][blk][i] = 0.f;
  }

  auto compute = [&](int tile, TileRegs& r) {
    const int tok0 = tile * kTile;
    // K: registers -> swizzled LDS tile [32 tokens][16 chunks of 16 B]
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int tok = 4 * i + k_tok;
      *reinterpret_cast<u32x4*>(kst + tok * 256 + ((k_chunk ^ (tok & 15)) << 4)) = r.k[i];
    }
    wave_lds_fence();
    f32x16 st[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int i = 0; i < 16; ++i) st[nb][i] = 0.f;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int chunk = 2 * kk + half;
      const u32x4 raw = *reinterpret_cast<const u32x4*>(kst + l32 * 256 + ((chunk ^ (l32 & 15)) << 4));
      const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
        st[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[nb][kk], st[nb], 0, 0, 0);
    }
    wave_lds_fence();

    const bool tail = (tok0 + kTile > n) || (CAUSAL && (tok0 + kTile - 1 > n - p.G));
    bf16x8 pb[NB][2];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      float s[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) s[i] = st[nb][i] * p.scale_log2e;
      if (tail) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int tok = tok0 + 8 * (i >> 2) + 4 * half + (i & 3);
          if (tok > limit[nb]) s[i] = -INFINITY;
        }
      }
      float tmax = s[0];
#pragma unroll
      for (int i = 1; i < 16; ++i) tmax = fmaxf(tmax, s[i]);
      tmax = fmaxf(tmax, xhalf(tmax));
      const float m_new = fmaxf(m_run[nb], tmax);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = fast_exp2(m_run[nb] - m_use);
      float pr[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) pr[i] = fast_exp2(s[i] - m_use);
      float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) { ps0 += pr[i]; ps1 += pr[8 + i]; }
      l_run[nb] = l_run[nb] * alpha + (ps0 + ps1);
      m_run[nb] = m_new;
      if (COLLECT) {
        const float f0 = ps0 + xhalf(ps0);
        const float f1 = ps1 + xhalf(ps1);
        const int row = nb * 32 + l32;
        const int page = tile * 2 + half;
        if (row < p.R && page < nblk) {
          const float lse = m_use + fast_log2(half ? f1 : f0);
          p.page_lse[((static_cast<int64_t>(b) * p.Hkv + h) * p.lse_pages + page) * p.R + row] = lse;
        }
      }
      if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
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
          if (tok >= n) r.v[s2 * 8 + jj] = u32x2{0u, 0u};
        }
    }
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        u32x4 raw;
#pragma unroll
        for (int pp = 0; pp < 4; ++pp) {
          const u32x2 ev = r.v[s2 * 8 + 2 * pp];
          const u32x2 od = r.v[s2 * 8 + 2 * pp + 1];
          const unsigned lo = (blk < 2) ? ev[0] : ev[1];
          const unsigned hi = (blk < 2) ? od[0] : od[1];
          raw[pp] = __builtin_amdgcn_perm(hi, lo, (blk & 1) ? 0x07060302u : 0x05040100u);
        }
        const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
          acc[nb][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[nb][s2], acc[nb][blk], 0, 0, 0);
      }
    }
  };

  // ---- stream the chunk's tiles, next tile's loads in flight during the current tile's math
  {
    TileRegs ra, rb;
    int tile = c0 / kTile + wave;
    const int tile_end = (c1 + kTile - 1) / kTile;
    if (tile < tile_end) {
      issue(tile, ra);
      while (true) {
        int nxt = tile + NW;
        if (nxt < tile_end) issue(nxt, rb);
        compute(tile, ra);
        if (nxt >= tile_end) break;
        tile = nxt;
        nxt = tile + NW;
        if (nxt < tile_end) issue(nxt, ra);
        compute(tile, rb);
        if (nxt >= tile_end) break;
        tile = nxt;
      }
    }
  }

  // ---- merge the NW waves
  if (half == 0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) sm_m[wave][nb * 32 + l32] = m_run[nb];
  }
  __syncthreads();
  float m_wg[NB];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    float mw = -INFINITY;
#pragma unroll
    for (int w = 0; w < NW; ++w) mw = fmaxf(mw, sm_m[w][nb * 32 + l32]);
    m_wg[nb] = mw;
    const float m_use = (mw == -INFINITY) ? 0.f : mw;
    const float sc = fast_exp2(m_run[nb] - m_use);
    float lsum = l_run[nb] * sc;
    lsum += xhalf(lsum);
    if (half == 0) sm_l[wave][nb * 32 + l32] = lsum;
#pragma unroll
    for (int blk = 0; blk < 4; ++blk)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nb][blk][i] *= sc;
  }
  f32x4* red = reinterpret_cast<f32x4*>(smem);          // [slot][16 quads][64 lanes] per row block
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int stride = NW / 2; stride >= 1; stride >>= 1) {
      __syncthreads();
      if (wave >= stride && wave < 2 * stride) {
        f32x4* dst = red + (wave - stride) * 16 * 64;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
          for (int qd = 0; qd < 4; ++qd)
            dst[(blk * 4 + qd) * 64 + lane] = f32x4{acc[nb][blk][4 * qd], acc[nb][blk][4 * qd + 1],
                                                    acc[nb][blk][4 * qd + 2], acc[nb][blk][4 * qd + 3]};
      }
      __syncthreads();
      if (wave < stride) {
        const f32x4* src = red + wave * 16 * 64;
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            const f32x4 x = src[(blk * 4 + qd) * 64 + lane];
            acc[nb][blk][4 * qd] += x[0];
            acc[nb][blk][4 * qd + 1] += x[1];
            acc[nb][blk][4 * qd + 2] += x[2];
            acc[nb][blk][4 * qd + 3] += x[3];
          }
      }
    }
  }
  if (NW == 1) __syncthreads();

  if (wave == 0) {
    const int64_t pbase = (static_cast<int64_t>(b) * p.Hkv + h) * p.nsplit + split;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      const int row = nb * 32 + l32;
      if (row < p.R) {
        float* po = p.part_o + (pbase * p.R + row) * kHeadDim;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int d0 = 4 * (8 * (i >> 2) + 4 * half + (i & 3));
          *reinterpret_cast<f32x4*>(po + d0) =
              f32x4{acc[nb][0][i], acc[nb][1][i], acc[nb][2][i], acc[nb][3][i]};
        }
        if (half == 0) {
          float lw = 0.f;
#pragma unroll
          for (int w = 0; w < NW; ++w) lw += sm_l[w][row];
          p.part_ml[pbase * p.R + row] = make_float2(m_wg[nb], lw);
        }
      }
    }
  }
}

}  // namespace vegas
