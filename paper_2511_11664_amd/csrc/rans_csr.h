// rans_csr.h -- modified CSR, encode side (Sec. 3.1 "Modified CSR Encoding"): compaction, row counts
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

#include "rans_quant.h"

namespace {

// ------------------------------------------------------------------ kernels: modified CSR

__device__ __forceinline__ void load16(const uint8_t *p, uint64_t e0, uint64_t n, bool aligned, uint8_t out[16]) {
  if (aligned && e0 + 16 <= n) {
    uint4 w = *(const uint4 *)(p + e0);
    uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int k = 0; k < 16; k++) out[k] = (uint8_t)(ww[k >> 2] >> (8 * (k & 3)));
  } else {
#pragma unroll
    for (int k = 0; k < 16; k++) out[k] = (e0 + k < n) ? p[e0 + k] : (uint8_t)0;
  }
}

// The same 16 symbols as four words (symbol k in byte k % 4 of word k / 4).
__device__ __forceinline__ void load16w(const uint8_t *p, uint64_t e0, uint64_t n, bool aligned, uint32_t out[4]) {
  if (aligned && e0 + 16 <= n) {
    const uint4 w = *(const uint4 *)(p + e0);
    out[0] = w.x; out[1] = w.y; out[2] = w.z; out[3] = w.w;
  } else {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      uint32_t t = 0;
#pragma unroll
      for (int q = 0; q < 4; q++) t |= (e0 + 4 * j + q < n ? (uint32_t)p[e0 + 4 * j + q] : 0u) << (8 * q);
      out[j] = t;
    }
  }
}
// Bit k of the result is set when symbol k of the 16 (four words) is not zero: bit 7 of every nonzero byte by
// word arithmetic, moved down to a 0/1 byte, and the four bytes of a word gathered by a dot product with the bit
// weights (two words share one accumulator; a 32-bit multiply, the other way to gather, runs at a quarter of the rate).
__device__ __forceinline__ uint32_t nonzero_mask16(const uint32_t (&w)[4]) {
  auto ones = [](uint32_t x) { return ((((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u) >> 7; };
  const uint32_t lo = __builtin_amdgcn_udot4(ones(w[1]), 0x80402010u, __builtin_amdgcn_udot4(ones(w[0]), 0x08040201u, 0u, false), false);
  const uint32_t hi = __builtin_amdgcn_udot4(ones(w[3]), 0x80402010u, __builtin_amdgcn_udot4(ones(w[2]), 0x08040201u, 0u, false), false);
  return lo | (hi << 8);
}

// Rows of KK columns with KK dividing 16 lie inside a lane's 16 symbols: their counts r (Sec. 3.1, the
// non-cumulative row counts) are the population counts of KK-bit fields of the lane's nonzero mask.  The lane
// stores them (consecutive lanes, consecutive rows: one store of up to 16 bytes each) and counts them in an LDS
// histogram of eight counters per value, one per lane residue.
template <uint32_t KK>
__device__ __forceinline__ void rows_inside_lane(uint32_t mask, uint64_t e0, uint32_t n, uint16_t *r, uint32_t *s_r,
                                                 uint32_t lane_rep) {
  constexpr uint32_t NF = 16 / KK;
  const uint32_t row0 = (uint32_t)(e0 / KK);
  uint32_t v[NF];
#pragma unroll
  for (uint32_t f = 0; f < NF; f++) v[f] = (uint32_t)__popc((mask >> (f * KK)) & ((1u << KK) - 1u));
  const bool full = e0 + 16 <= n;  // n is a multiple of KK: otherwise whole rows are missing at the end
  if (full) {
    if constexpr (NF == 1) {
      r[row0] = (uint16_t)v[0];
    } else {
      uint32_t w[NF / 2];
#pragma unroll
      for (uint32_t q = 0; q < NF / 2; q++) w[q] = v[2 * q] | (v[2 * q + 1] << 16);
      if constexpr (NF == 2) *(uint32_t *)(r + row0) = w[0];
      else if constexpr (NF == 4) *(uint2 *)(r + row0) = make_uint2(w[0], w[1]);
      else if constexpr (NF == 8) *(uint4 *)(r + row0) = make_uint4(w[0], w[1], w[2], w[3]);
      else {
        *(uint4 *)(r + row0) = make_uint4(w[0], w[1], w[2], w[3]);
        *(uint4 *)(r + row0 + 8) = make_uint4(w[4], w[5], w[6], w[7]);
      }
    }
  }
#pragma unroll
  for (uint32_t f = 0; f < NF; f++) {
    if (full || e0 + f * KK < n) {
      if (!full) r[row0 + f] = (uint16_t)v[f];
      atomicAdd(&s_r[v[f] + lane_rep * (KK + 1)], 1u);
    }
  }
}

// Stream compaction of the nonzero symbols in flat (= row-major) order: v gets the
// values, c the column indices, row_end[i] the number of nonzeros up to and
// including row i.  Column indices are histogrammed into cnt on the way.
// A work-group takes tiles_per_wg consecutive tiles: a tile's nonzeros are compacted in LDS first
// and leave with consecutive lanes on consecutive entries (that loop also counts their columns in an LDS
// histogram: every lane has work at every step there), and the column histogram is added to a
// global one once at the end (few work-groups: same-address global atomics are what costs here).
// k_quant_hist has counted the nonzeros of every tile (blk_nnz) and of every group of tiles_per_grp
// tiles (grp_nnz); the place of the work-group's first tile in v and c is the sum over the groups
// and then the tiles before it, and every further tile follows the one before.
// A lane takes 16 consecutive symbols as four words, derives the mask of its nonzero ones with a few word
// operations and then visits only the set bits (about a third of the symbols of a post-ReLU tensor; a wave
// runs as many steps as its fullest lane has nonzeros, nine or ten of 16; the step is kept to a dozen vector
// instructions, which is what bounds the walk).  Row ends come from the mask
// afterwards: symbol p ends a row when the lane's first column plus p + 1 is a multiple of K.
// SHORT_ROWS (few columns): eight counters per column, see below.
template <bool LDS_HIST, bool SHORT_ROWS = false>
__global__ __launch_bounds__(kWG) void k_csr_compact(const uint8_t *sym, uint32_t n, int aligned, uint32_t K,
                                                     const uint32_t *blk_nnz, const uint32_t *grp_nnz,
                                                     uint32_t tiles_per_grp, uint8_t *v, uint16_t *c,
                                                     uint32_t *row_end, uint32_t *cnt, uint32_t A, uint32_t n_tiles,
                                                     uint32_t tiles_per_wg, uint32_t n_rep, int rows_in_lane,
                                                     uint16_t *r, uint32_t N, CtlRef ctl) {
  extern __shared__ uint32_t hist[];
  // rows_in_lane: 1 (K divides 16), 3 (any other K < 16) or 2 (K divides the tile of 4096 symbols, 64 <= K, so that
  // every tile starts a row and holds at most 64 of them): the row counts, their histogram and l_D come from this
  // kernel, and neither the row ends nor k_csr_rows are needed.  2: the lane that holds a row's last symbol leaves the number of the
  // tile's nonzeros up to there in LDS, and after the tile's barrier a thread per row takes the difference.
  __shared__ uint32_t s_r[17 * 8];
  __shared__ uint32_t s_rowend[64];
  if (threadIdx.x < 17 * 8) s_r[threadIdx.x] = 0;  // ordered before its use by the barriers of the first tile
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint64_t sh64[kWG / 64];
  __shared__ uint32_t s_vc[kCsrTile];  // value | column << 8 of the tile's nonzeros, in order (one LDS write each)
  if (LDS_HIST) {
    for (uint32_t a = threadIdx.x; a < ((A + 15u) & ~15u); a += kWG) hist[a] = 0;
  }
  // few columns (the host selects SHORT_ROWS for K <= 32 with 8 K <= A, so the counters fit): eight counters per
  // column, one per lane residue and K slots apart - a wave's 64 consecutive nonzeros meet only K distinct columns
  const uint32_t rep_off = SHORT_ROWS ? (threadIdx.x & 7u) * K : 0u;
  const uint32_t t0 = blockIdx.x * tiles_per_wg;  // < n_tiles by the size of the grid
  const uint32_t t1 = t0 + tiles_per_wg < n_tiles ? t0 + tiles_per_wg : n_tiles;
  uint32_t w[4];
  load16w(sym, (uint64_t)t0 * kCsrTile + threadIdx.x * 16, n, aligned, w);
  uint32_t base;
  {
    const uint32_t g0 = t0 / tiles_per_grp;
    uint64_t part = 0;
    for (uint32_t u0 = threadIdx.x; u0 < g0; u0 += 8 * kWG) {
      uint32_t x8[8];
#pragma unroll
      for (int k = 0; k < 8; k++) x8[k] = u0 + k * kWG < g0 ? grp_nnz[u0 + k * kWG] : 0u;
#pragma unroll
      for (int k = 0; k < 8; k++) part += x8[k];
    }
    for (uint32_t t = g0 * tiles_per_grp + threadIdx.x; t < t0; t += kWG) part += blk_nnz[t];
    base = (uint32_t)block_sum64<kWG>(part, sh64);
  }
  // (x * inv16) >> 16 = x / K for the x < 32 that occur when K < 16
  const uint32_t inv16 = 65536u / K + 1u;
  // Row and column of the lane's first symbol, and the first row of the tile: one division before the loop, then
  // from tile to tile by the quotient and remainder of the tile size (a 64-bit division per lane and tile cost
  // as many instructions as a third of the walk).
  const uint32_t tile_q = kCsrTile / K, tile_r = kCsrTile % K;
  uint32_t row0, col0, tile_row0;
  {
    const uint64_t e_first = (uint64_t)t0 * kCsrTile + threadIdx.x * 16;
    row0 = (uint32_t)(e_first / K);
    col0 = (uint32_t)(e_first - (uint64_t)row0 * K);
    tile_row0 = (uint32_t)((uint64_t)t0 * kCsrTile / K);  // of use where K divides the tile
  }
  for (uint32_t tile = t0; tile < t1; tile++) {
    const uint64_t e0 = (uint64_t)tile * kCsrTile + threadIdx.x * 16;
    uint32_t nw[4];  // the next tile's symbols are on their way while this one is placed
    if (tile + 1 < t1) load16w(sym, e0 + kCsrTile, n, aligned, nw);
    // symbols past the end of the tensor read as zero
    const uint32_t mask = nonzero_mask16(w);
    uint32_t tot;
    const uint32_t loc0 = block_excl_scan<kWG>((uint32_t)__popc(mask), sh, &tot);  // also orders the hist zeroing and the staging reuse
    if (e0 < n) {
      // the walk, once for each way of wrapping the column (decided outside the loop: K is uniform)
      auto walk = [&](auto wide_rows) {
        uint32_t loc = loc0;
        for (uint32_t mk = mask; mk; mk &= mk - 1u) {
          const uint32_t k = (uint32_t)__ffs((int)mk) - 1u;
          // byte k of the lane's 16: a byte permute of each half (selector byte 0 = k mod 8, the others give
          // zero), and the half that holds it
          const uint32_t sel = 0x0c0c0c00u | (k & 7u);
          const uint32_t val = k < 8 ? __builtin_amdgcn_perm(w[1], w[0], sel) : __builtin_amdgcn_perm(w[3], w[2], sel);
          uint32_t col = col0 + k;
          if (decltype(wide_rows)::value == 2) col &= K - 1u;             // K a power of two
          else if (decltype(wide_rows)::value == 1) col -= col >= K ? K : 0u;  // K >= 16: at most one wrap
          else col -= K * ((col * inv16) >> 16);
          s_vc[loc++] = val | (col << 8);
        }
      };
      if ((K & (K - 1u)) == 0) walk(std::integral_constant<int, 2>{});
      else if (K >= 16) walk(std::integral_constant<int, 1>{});
      else walk(std::integral_constant<int, 0>{});
      if (rows_in_lane == 3) {
        // short rows that straddle lanes (K < 16, not a divisor of 16): the lane takes the rows that start inside
        // its 16 symbols and looks at the nonzero flags of the 16 symbols behind them for the ends
        uint32_t ext[4];
        load16w(sym, e0 + 16, n, aligned, ext);
        const uint32_t m32 = mask | (nonzero_mask16(ext) << 16);
        const uint32_t lr = threadIdx.x & 7u;
        uint32_t row = row0 + (col0 ? 1u : 0u);
        for (uint32_t p = col0 ? K - col0 : 0u; p < 16 && e0 + p < n; p += K, row++) {
          const uint32_t rj = (uint32_t)__popc((m32 >> p) & ((1u << K) - 1u));
          r[row] = (uint16_t)rj;
          atomicAdd(&s_r[rj + lr * (K + 1)], 1u);
        }
      } else if (rows_in_lane == 2) {  // uniform; one row end per lane at most
        const uint32_t p = K - 1 - col0;
        if (p < 16) s_rowend[row0 - tile_row0] = loc0 + (uint32_t)__popc(mask & ((2u << p) - 1u));
      } else if (rows_in_lane) {
        const uint32_t lr = threadIdx.x & 7u;
        if (K == 4) rows_inside_lane<4>(mask, e0, n, r, s_r, lr);
        else if (K == 2) rows_inside_lane<2>(mask, e0, n, r, s_r, lr);
        else if (K == 8) rows_inside_lane<8>(mask, e0, n, r, s_r, lr);
        else if (K == 16) rows_inside_lane<16>(mask, e0, n, r, s_r, lr);
        else rows_inside_lane<1>(mask, e0, n, r, s_r, lr);
      } else {
        uint32_t row = row0;
        for (uint32_t p = K - 1 - col0; p < 16 && e0 + p < n; p += K)
          row_end[row++] = base + loc0 + (uint32_t)__popc(mask & ((2u << p) - 1u));
      }
    }
    __syncthreads();
    if (rows_in_lane == 2) {
      const uint32_t row = tile_row0 + threadIdx.x;
      if (threadIdx.x < kCsrTile / K && row < N) {
        const uint32_t rj = s_rowend[threadIdx.x] - (threadIdx.x ? s_rowend[threadIdx.x - 1] : 0u);
        r[row] = (uint16_t)rj;
        atomicAdd(&hist[rj], 1u);  // the same alphabet as the columns: one histogram for all of D
      }
    }
    // the tile's nonzeros to their place, and their columns into the histogram: here every lane has work at
    // every step (in the walk a wave runs as long as its fullest lane)
    for (uint32_t i = threadIdx.x; i < tot; i += kWG) {
      const uint32_t vc = s_vc[i], col = vc >> 8;
      v[base + i] = (uint8_t)vc;
      c[base + i] = (uint16_t)col;
      if (LDS_HIST) atomicAdd(&hist[SHORT_ROWS ? col + rep_off : col], 1u);
      else atomicAdd(&cnt[col], 1u);
    }
    base += tot;
    row0 += tile_q;
    col0 += tile_r;
    if (col0 >= K) {
      col0 -= K;
      row0++;
    }
    tile_row0 += tile_q;  // exact where it is used (K divides the tile)
    if (tile + 1 < t1) {
#pragma unroll
      for (int k = 0; k < 4; k++) w[k] = nw[k];
    }
    __syncthreads();  // staging and scan scratch are reused by the next tile
  }
  if (rows_in_lane) {
    __syncthreads();
    uint32_t *dst_r = cnt + (n_rep ? (size_t)(1 + blockIdx.x % n_rep) * A : 0);
    if (rows_in_lane != 2 && threadIdx.x <= K) {
      uint32_t t = 0;
#pragma unroll
      for (uint32_t q = 0; q < 8; q++) t += s_r[threadIdx.x + q * (K + 1)];
      if (t) atomicAdd(&dst_r[threadIdx.x], t);
    }
    if (t1 == n_tiles && threadIdx.x == 0) {  // the work-group with the last tile knows the number of nonzeros
      ctl->nnz = base;
      ctl->len_d = 2ull * base + N;
    }
  }
  if (LDS_HIST) {
    // into one of the partial histograms: a thousand work-groups adding to the same few hundred addresses
    // would keep the kernel busy long after its last tile
    uint32_t *dst = cnt + (n_rep ? (size_t)(1 + blockIdx.x % n_rep) * A : 0);
    for (uint32_t a = threadIdx.x; a < (SHORT_ROWS ? K : A); a += kWG) {
      uint32_t t = 0;
      if (SHORT_ROWS) {
#pragma unroll
        for (uint32_t k = 0; k < 8; k++) t += hist[a + k * K];
      } else {
        t = hist[a];
      }
      if (t) atomicAdd(&dst[a], t);
    }
  }
}

// r[i] = row_end[i] - row_end[i-1] (the NON-cumulative row count), histogrammed.  Work-groups stride
// over the rows and add their histogram to the global one once.
// REP (short rows, 8 (K + 1) <= A): a row count is one of K + 1 values, which a wave's lanes would all add to
// the same few LDS addresses; every value gets eight counters, one per lane residue, K + 1 slots apart.
template <bool LDS_HIST, bool REP = false>
__global__ __launch_bounds__(kWG) void k_csr_rows(const uint32_t *row_end, uint32_t N, uint16_t *r, uint32_t *cnt,
                                                  uint32_t A, CtlRef ctl, uint32_t n_cols, uint32_t n_rep) {
  extern __shared__ uint32_t hist[];
  if (LDS_HIST) {
    for (uint32_t a = threadIdx.x; a < A; a += kWG) hist[a] = 0;
    __syncthreads();
  }
  const uint32_t n_val = n_cols + 1;  // REP: distinct row counts
  const uint32_t rep_off = REP ? (threadIdx.x & 7u) * n_val : 0u;
  // a lane takes four consecutive rows: one 16-byte load of their ends, one 8-byte store of their counts;
  // the loads of four such quads are in flight together
  const uint32_t n_quads = (N + 3) / 4;
  constexpr int kU = 4;
  auto load_quad = [&](uint32_t q, uint32_t (&e)[5]) {
    const uint32_t i = 4 * q;
    e[0] = i ? row_end[i - 1] : 0;
    if (i + 4 <= N) {
      const uint4 w = *(const uint4 *)(row_end + i);
      e[1] = w.x; e[2] = w.y; e[3] = w.z; e[4] = w.w;
    } else {
#pragma unroll
      for (int k = 0; k < 4; k++) e[k + 1] = i + k < N ? row_end[i + k] : e[k];
    }
  };
  auto do_quad = [&](uint32_t q, const uint32_t (&e)[5]) {
    const uint32_t i = 4 * q;
    uint32_t rr[4];
#pragma unroll
    for (int k = 0; k < 4; k++) rr[k] = e[k + 1] - e[k];
    if (i + 4 <= N) {
      *(uint2 *)(r + i) = make_uint2(rr[0] | (rr[1] << 16), rr[2] | (rr[3] << 16));
    } else {
#pragma unroll
      for (int k = 0; k < 4; k++)
        if (i + k < N) r[i + k] = (uint16_t)rr[k];
    }
#pragma unroll
    for (int k = 0; k < 4; k++) {
      if (i + k < N) {
        if (LDS_HIST) atomicAdd(&hist[rr[k] + rep_off], 1u);
        else atomicAdd(&cnt[rr[k]], 1u);
      }
    }
    if (i + 4 >= N) {  // the quad with the last row (ends behind it repeat the last row's)
      const uint32_t e1 = e[4];
      ctl->nnz = e1;
      ctl->len_d = 2ull * e1 + N;
    }
  };
  for (uint32_t q0 = blockIdx.x * (kWG * kU) + threadIdx.x; q0 < n_quads; q0 += gridDim.x * (kWG * kU)) {
    uint32_t e[kU][5];
#pragma unroll
    for (int u = 0; u < kU; u++)
      if (q0 + u * kWG < n_quads) load_quad(q0 + u * kWG, e[u]);
#pragma unroll
    for (int u = 0; u < kU; u++)
      if (q0 + u * kWG < n_quads) do_quad(q0 + u * kWG, e[u]);
  }
  // The partial histograms (one of n_rep, by work-group) are summed by the kernel that builds the table, which
  // starts after this one has ended.
  if (LDS_HIST) {
    __syncthreads();
    uint32_t *dst = cnt + (n_rep ? (size_t)(1 + blockIdx.x % n_rep) * A : 0);
    for (uint32_t a = threadIdx.x; a < (REP ? n_val : A); a += kWG) {
      uint32_t t = 0;
      if (REP) {
#pragma unroll
        for (uint32_t k = 0; k < 8; k++) t += hist[a + k * n_val];
      } else {
        t = hist[a];
      }
      if (t) atomicAdd(&dst[a], t);
    }
  }
}

}  // namespace
