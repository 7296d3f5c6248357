// rans_reshape.h -- reshape search (Sec. 3.2, Algorithm 1)
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

#include "rans_common.h"

namespace {

// ------------------------------------------------------------------ kernels: reshape search (Sec. 3.2)

// The quantised tensor is fixed over all reshapes [N, K]: so are the nonzero values v and their
// number.  Only the histograms of the column indices (position mod K) and of the row counts change.
// One pass turns the tensor into a zero mask (16 positions per entry), the number of nonzeros
// before each entry inside its tile, the tile totals and the histogram of v; everything else is
// computed from those.
constexpr uint32_t kRsTile = kWG * 16;
struct RsCands {
  uint32_t n;
  uint16_t K[RANS_RESHAPE_MAX_CAND];
};
struct RsOffsets {  // first bin of each candidate's row-count histogram; entry n = total
  uint32_t hr[RANS_RESHAPE_MAX_CAND + 1];
  // first work-group of each candidate in the grid of k_rs_rows (shares in proportion to the number of rows, so
  // that the candidates with the shortest rows do not run on alone at the end); entry n = the grid
  uint32_t wg0[RANS_RESHAPE_MAX_CAND + 1];
};
// Candidates are grouped so that the members of a group have a common multiple L of at most kRsLcmMax: one
// histogram of the nonzero positions modulo L then serves every member, whose own column histogram
// (positions modulo K) is that one folded K-periodically.
constexpr uint32_t kRsLcmMax = 32768;  // LDS words of k_rs_cols
struct RsGroups {
  uint32_t n;
  uint32_t L[RANS_RESHAPE_MAX_CAND];        // residues of group g: a multiple of every K in it, at least 16
  uint32_t off[RANS_RESHAPE_MAX_CAND + 1];  // first word of its histogram in hl; entry n = total
  uint8_t of[RANS_RESHAPE_MAX_CAND];        // group of candidate k
};

__global__ __launch_bounds__(kWG) void k_rs_mask(const uint8_t *sym, uint32_t n, int aligned, uint32_t n_tiles,
                                                 uint16_t *mask16, uint16_t *lp, uint32_t *tile_cnt, uint32_t *hv,
                                                 uint32_t q_bits, uint32_t *bad_flag) {
  __shared__ uint32_t sh[kWG / 64];
  // eight counters per value, one per lane residue: activations have a few very frequent values, and a wave's
  // additions to one LDS address are performed one after the other
  __shared__ uint32_t h[256 * 8];
  for (uint32_t i = threadIdx.x; i < 256 * 8; i += kWG) h[i] = 0;
  const uint32_t rep = threadIdx.x & 7u;
  __syncthreads();
  uint8_t b[16];
  if (blockIdx.x < n_tiles) load16(sym, (uint64_t)blockIdx.x * kRsTile + threadIdx.x * 16, n, aligned, b);
  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const uint64_t e0 = (uint64_t)tile * kRsTile + threadIdx.x * 16;
    uint8_t nb[16];  // the next tile's symbols are on their way while this one is looked at
    const bool more = tile + gridDim.x < n_tiles;
    if (more) load16(sym, e0 + (uint64_t)gridDim.x * kRsTile, n, aligned, nb);
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < 16; k++) {
      if (b[k]) {
        m |= 1u << k;
        if (b[k] >> q_bits) atomicOr(bad_flag, 1u);  // not a symbol of this bit width
        atomicAdd(&h[b[k] * 8u + rep], 1u);
      }
    }
    uint32_t tot;
    const uint32_t ex = block_excl_scan<kWG>(__popc(m), sh, &tot);
    if (e0 < n) {
      mask16[e0 >> 4] = (uint16_t)m;
      lp[e0 >> 4] = (uint16_t)ex;
    }
    if (threadIdx.x == 0) tile_cnt[tile] = tot;
    if (more) {
#pragma unroll
      for (int k = 0; k < 16; k++) b[k] = nb[k];
    }
    __syncthreads();
  }
  uint32_t t = 0;  // kWG == 256: a thread per value
#pragma unroll
  for (int r = 0; r < 8; r++) t += h[threadIdx.x * 8 + r];
  if (t) atomicAdd(&hv[threadIdx.x], t);
}

// zeroes the histograms of a call (runs before k_rs_mask, which adds to hv)
__global__ void k_rs_zero(uint32_t *p, uint32_t words) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gridDim.x * blockDim.x) p[i] = 0;
}

// Histogram of the nonzero positions modulo L (one group of candidates; see RsGroups), in LDS and then added
// to hl.  A thread takes eight consecutive mask entries (128 positions) with one load and walks their set bits.
__global__ __launch_bounds__(kWG) void k_rs_cols(const uint16_t *mask16, uint32_t n_entries, uint32_t L, uint32_t *hl) {
  extern __shared__ uint32_t h_l[];
  for (uint32_t i = threadIdx.x; i < L; i += kWG) h_l[i] = 0;
  __syncthreads();
  const uint32_t n_oct = (n_entries + 7) / 8;
  const uint32_t stride = gridDim.x * kWG;
  const uint32_t step = (uint32_t)(((uint64_t)stride * 128) % L);  // positions between a thread's octets, modulo L
  uint32_t c = (uint32_t)(((uint64_t)(blockIdx.x * kWG + threadIdx.x) * 128) % L);
  for (uint32_t o = blockIdx.x * kWG + threadIdx.x; o < n_oct; o += stride) {
    uint32_t w[4];
    if (8 * o + 8 <= n_entries) {  // the mask array starts 256-byte aligned
      const uint4 q = *(const uint4 *)(mask16 + 8 * (size_t)o);
      w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const uint32_t e = 8 * o + 2 * j;
        w[j] = (e < n_entries ? mask16[e] : 0u) | ((e + 1 < n_entries ? (uint32_t)mask16[e + 1] : 0u) << 16);
      }
    }
    uint32_t cj = c;  // residue of the first position of the word at hand
#pragma unroll
    for (int j = 0; j < 4; j++) {
      uint32_t m = w[j];
      while (m) {
        const uint32_t bit = (uint32_t)__ffs((int)m) - 1u;
        m &= m - 1u;
        uint32_t pos = cj + bit;  // < 2 L as L >= 32
        pos = pos >= L ? pos - L : pos;
        atomicAdd(&h_l[pos], 1u);
      }
      cj += 32;
      cj = cj >= L ? cj - L : cj;
    }
    c += step;
    c = c >= L ? c - L : c;
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < L; i += kWG) {
    const uint32_t t = h_l[i];
    if (t) atomicAdd(&hl[i], t);
  }
}

// Row-count histograms of the candidates K = 2, 4, 8, 16 (those of them in the domain: hr_at[i] is the first bin of
// K = 2 << i, ~0 for none), straight from the zero mask: such rows are K-bit fields of a mask word, and their
// counts are population counts of the fields - taken for all fields of a 32-position word at once, with word
// operations for K = 2 and 4 (how many fields hold 1, 2, ... set bits) and per field for K = 8 and 16.  These
// candidates have the most rows; k_rs_rows, which looks up two prefix counts per row, is left with the others.
struct RsPow2 {
  uint32_t hr_at[4];
};
__global__ __launch_bounds__(kWG) void k_rs_rows_pow2(const uint16_t *mask16, uint32_t n_entries, uint32_t n, RsPow2 at,
                                                      uint32_t *hr) {
  __shared__ uint32_t s_h[4][17 * 8];  // eight counters per value, one per lane residue
  for (uint32_t i = threadIdx.x; i < 4 * 17 * 8; i += kWG) (&s_h[0][0])[i] = 0;
  __syncthreads();
  const uint32_t rp = threadIdx.x & 7u;
  const uint32_t n_oct = (n_entries + 7) / 8;
  uint32_t c2[3] = {0, 0, 0}, c4[5] = {0, 0, 0, 0, 0};
  for (uint32_t o = blockIdx.x * kWG + threadIdx.x; o < n_oct; o += gridDim.x * kWG) {
    uint32_t w[4];
    if (8 * o + 8 <= n_entries) {
      const uint4 q = *(const uint4 *)(mask16 + 8 * (size_t)o);
      w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
    } else {
#pragma unroll
      for (int j = 0; j < 4; j++) {
        const uint32_t e = 8 * o + 2 * j;
        w[j] = (e < n_entries ? mask16[e] : 0u) | ((e + 1 < n_entries ? (uint32_t)mask16[e + 1] : 0u) << 16);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const uint64_t p0 = ((uint64_t)o * 4 + j) * 32;  // first position of the word
      const uint32_t m = w[j];
      if (p0 + 32 <= n) {  // all of the word's rows exist (n is a multiple of every K here)
        if (at.hr_at[0] != ~0u) {
          const uint32_t x = m & 0x55555555u, y = (m >> 1) & 0x55555555u;
          const uint32_t two = (uint32_t)__popc(x & y), one = (uint32_t)__popc(x ^ y);
          c2[2] += two; c2[1] += one; c2[0] += 16u - two - one;
        }
        uint32_t t = m - ((m >> 1) & 0x55555555u);
        t = (t & 0x33333333u) + ((t >> 2) & 0x33333333u);  // eight fields of four bits: their population counts (0 .. 4)
        if (at.hr_at[1] != ~0u) {
          uint32_t rest = 8;
#pragma unroll
          for (uint32_t v = 1; v <= 4; v++) {
            const uint32_t z = t ^ (v * 0x11111111u);
            const uint32_t ne = (z | (z >> 1) | (z >> 2)) & 0x11111111u;  // bit 3 of a field is never set
            const uint32_t eq = 8u - (uint32_t)__popc(ne);
            c4[v] += eq;
            rest -= eq;
          }
          c4[0] += rest;
        }
        if (at.hr_at[2] != ~0u) {
          const uint32_t b = (t + (t >> 4)) & 0x0f0f0f0fu;  // four fields of eight bits
#pragma unroll
          for (int f = 0; f < 4; f++) atomicAdd(&s_h[2][((b >> (8 * f)) & 0xffu) * 8 + rp], 1u);
        }
        if (at.hr_at[3] != ~0u) {
          atomicAdd(&s_h[3][(uint32_t)__popc(m & 0xffffu) * 8 + rp], 1u);
          atomicAdd(&s_h[3][(uint32_t)__popc(m >> 16) * 8 + rp], 1u);
        }
      } else if (p0 < n) {  // the word with the end of the tensor: row by row
#pragma unroll
        for (uint32_t i = 0; i < 4; i++) {
          if (at.hr_at[i] == ~0u) continue;
          const uint32_t K = 2u << i;
          for (uint32_t q = 0; q < 32 && p0 + q < n; q += K)
            atomicAdd(&s_h[i][(uint32_t)__popc((m >> q) & ((1u << K) - 1u)) * 8 + rp], 1u);
        }
      }
    }
  }
#pragma unroll
  for (uint32_t v = 0; v < 3; v++)
    if (c2[v]) atomicAdd(&s_h[0][v * 8 + rp], c2[v]);
#pragma unroll
  for (uint32_t v = 0; v < 5; v++)
    if (c4[v]) atomicAdd(&s_h[1][v * 8 + rp], c4[v]);
  __syncthreads();
  if (threadIdx.x < 4 * 17) {
    const uint32_t i = threadIdx.x / 17, v = threadIdx.x % 17;
    if (at.hr_at[i] != ~0u && v <= (2u << i)) {
      uint32_t t = 0;
#pragma unroll
      for (int q = 0; q < 8; q++) t += s_h[i][v * 8 + q];
      if (t) atomicAdd(&hr[at.hr_at[i] + v], t);
    }
  }
}

// nonzeros before position g (g <= n)
__device__ __forceinline__ uint32_t rs_prefix(uint32_t g, uint32_t n, uint32_t nnz, const uint16_t *mask16,
                                              const uint16_t *lp, const uint32_t *tile_off) {
  if (g >= n) return nnz;
  const uint32_t e = g >> 4;
  return tile_off[g / kRsTile] + lp[e] + __popc((uint32_t)mask16[e] & ((1u << (g & 15)) - 1u));
}

// Histogram of the row counts r of one candidate (the work-group's, see RsOffsets): r[i] = prefix((i + 1) K) - prefix(i K).  A wave
// takes 63 consecutive rows: lane l looks up the prefix at the start of row l of them (lane 63: the end of the
// last), and a row's count is the neighbouring lane's prefix minus the lane's own - one look-up per row.
__global__ __launch_bounds__(kWG) void k_rs_rows(const uint16_t *mask16, const uint16_t *lp, const uint32_t *tile_off,
                                                 uint32_t n, uint32_t n_tiles, RsCands cands, RsOffsets offs,
                                                 uint32_t *hr) {
  __shared__ uint32_t h[257];
  const uint32_t *hr_off = offs.hr;
  uint32_t k = 0;
  while (k + 1 < cands.n && offs.wg0[k + 1] <= blockIdx.x) k++;  // uniform; at most a hundred steps
  const uint32_t K = cands.K[k];
  const uint32_t bx = blockIdx.x - offs.wg0[k], gx = offs.wg0[k + 1] - offs.wg0[k];
  const uint32_t nnz = tile_off[n_tiles];
  uint32_t *out = hr + hr_off[k];
  if (K == 1) {  // the row counts are the zero mask itself
    if (bx == 0 && threadIdx.x == 0) {
      out[0] = n - nnz;
      out[1] = nnz;
    }
    return;
  }
  for (uint32_t i = threadIdx.x; i <= K; i += kWG) h[i] = 0;
  __syncthreads();
  const uint32_t N = n / K;
  const uint32_t lane = threadIdx.x & 63;
  if (K < 16) {
    // Short rows that are not aligned fields of a mask word (K = 7, 14, ...): a row's count is the population
    // count of K bits of a 32-bit window over two mask entries.  A wave's additions to the few bins of such a
    // histogram are performed one after the other in LDS, so every lane counts in registers instead - one byte
    // per value in two 64-bit words - and the wave adds its lanes' bytes up every 255 rows at the latest.
    uint64_t pk0 = 0, pk1 = 0;
    auto flush = [&]() {
      for (uint32_t v = 0; v <= K; v++) {  // uniform
        const uint32_t mine = (uint32_t)((v < 8 ? pk0 : pk1) >> (8 * (v & 7u))) & 0xffu;
        const uint32_t tot = wave_incl_sum_scan(mine);
        if (lane == 63 && tot) atomicAdd(&h[v], tot);
      }
      pk0 = pk1 = 0;
    };
    const uint32_t n_entries = (n + 15) / 16;
    const uint32_t stride = gx * kWG;
    const uint32_t n_it = (N + stride - 1) / stride;  // the same for every thread
    for (uint32_t it = 0; it < n_it; it++) {
      const uint32_t i = bx * kWG + threadIdx.x + it * stride;
      if (i < N) {
        const uint32_t g = i * K, e = g >> 4;  // i K < n <= 2^30
        const uint32_t win = (uint32_t)mask16[e] | (e + 1 < n_entries ? (uint32_t)mask16[e + 1] << 16 : 0u);
        const uint32_t r = (uint32_t)__popc((win >> (g & 15u)) & ((1u << K) - 1u));
        if (r < 8) pk0 += 1ull << (8 * r);
        else pk1 += 1ull << (8 * (r - 8));
      }
      if ((it & 255u) == 254u) flush();
    }
    flush();
    __syncthreads();
    for (uint32_t i = threadIdx.x; i <= K; i += kWG) {
      const uint32_t t = h[i];
      if (t) atomicAdd(&out[i], t);
    }
    return;
  }
  const uint32_t waves = gx * (kWG / 64);
  // four groups of 63 rows per step, their look-ups in flight together
  constexpr uint32_t kU = 4;
  for (uint32_t i0 = (bx * (kWG / 64) + (threadIdx.x >> 6)) * 63; i0 < N; i0 += kU * waves * 63) {
    uint32_t a[kU];
#pragma unroll
    for (uint32_t u = 0; u < kU; u++) {
      const uint32_t i = i0 + u * waves * 63 + lane;  // i K stays below 2^32 (n <= 2^30, K <= 2^8) when i <= N
      a[u] = rs_prefix(i <= N ? i * K : n, n, nnz, mask16, lp, tile_off);
    }
#pragma unroll
    for (uint32_t u = 0; u < kU; u++) {
      const uint32_t i = i0 + u * waves * 63 + lane;
      const uint32_t b = (uint32_t)__shfl_down((int)a[u], 1);
      if (lane < 63 && i < N) atomicAdd(&h[b - a[u]], 1u);
    }
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i <= K; i += kWG) {
    const uint32_t t = h[i];
    if (t) atomicAdd(&out[i], t);
  }
}

// Costs and the walk of Algorithm 1.  One work-group per candidate sums its entropy terms in binary64
// (a fixed tree: lanes, then waves); the work-group that finishes last walks the candidates from the
// largest N down.  costs[] and the ticket live in the zeroed part of the workspace.
__global__ __launch_bounds__(kWG) void k_rs_cost(RsCands cands, uint32_t n, uint32_t n_tiles, uint32_t q_bits,
                                                 const uint32_t *tile_off, const uint32_t *hv, const uint32_t *hl,
                                                 const uint32_t *hr, RsOffsets offs, RsGroups grps,
                                                 const uint32_t *bad_flag, double *costs, uint32_t *ticket,
                                                 rans_reshape_result *res) {
  __shared__ double s_part[kWG / 64];
  __shared__ uint32_t s_ticket;
  __shared__ uint32_t s_col[256];  // this candidate's column histogram (K <= 2^8)
  const uint32_t *hr_off = offs.hr;
  const uint32_t k = blockIdx.x;
  const uint32_t nnz = tile_off[n_tiles];
  {
    const uint32_t K = cands.K[k], N = n / K;
    // the group's histogram of positions modulo L, folded K-periodically (K divides L)
    s_col[threadIdx.x] = 0;  // kWG == 256
    __syncthreads();
    {
      const uint32_t g = grps.of[k], L = grps.L[g];
      const uint32_t *hg = hl + grps.off[g];
      for (uint32_t i0 = threadIdx.x; i0 < L; i0 += 8 * kWG) {  // a thread's eight loads in flight together
        uint32_t t[8];
#pragma unroll
        for (int u = 0; u < 8; u++) t[u] = i0 + u * kWG < L ? hg[i0 + u * kWG] : 0u;
#pragma unroll
        for (int u = 0; u < 8; u++)
          if (t[u]) atomicAdd(&s_col[(i0 + u * kWG) % K], t[u]);
      }
    }
    __syncthreads();
    const uint32_t two_q = 1u << q_bits;
    const uint32_t A = K + 1 > two_q ? K + 1 : two_q;
    const uint64_t len = 2ull * nnz + N;
    double h = 0.0;
    for (uint32_t a = threadIdx.x; a < A; a += kWG) {
      uint64_t c = 0;
      if (a < two_q) c += hv[a];
      if (a < K) c += s_col[a];
      if (a <= K) c += hr[hr_off[k] + a];
      if (c) {
        const double p = (double)c / (double)len;
        h -= p * log2(p);
      }
    }
    const uint64_t bits = wave_incl_scan64((uint64_t)__double_as_longlong(h), [](uint64_t x, uint64_t y) {
      return (uint64_t)__double_as_longlong(__longlong_as_double((long long)x) + __longlong_as_double((long long)y));
    });
    if ((threadIdx.x & 63) == 63) s_part[threadIdx.x >> 6] = __longlong_as_double((long long)bits);
    __syncthreads();
    if (threadIdx.x == 0) {
      double H = 0.0;
      for (int w = 0; w < kWG / 64; w++) H += s_part[w];
      // device-scope store, then the ticket: the last work-group reads every cost with device-scope loads
      __hip_atomic_store(costs + k, (double)len * H, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_ticket = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
  }
  if (s_ticket != gridDim.x - 1 || threadIdx.x != 0) return;
  __atomic_thread_fence(__ATOMIC_ACQUIRE);
  double best = INFINITY, prev = INFINITY;
  uint64_t n_tilde = n;
  uint32_t evaluated = 0;
  bool walking = true;
  for (uint32_t i = 0; i < cands.n; i++) {
    const double cost = __hip_atomic_load(costs + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    res->cand_rows[i] = n / cands.K[i];
    res->cand_cost[i] = cost;
    if (walking) {
      evaluated++;
      if (cost < best) {
        best = cost;
        n_tilde = n / cands.K[i];
      }
      if (cost > prev) walking = false;  // stop after this one
      prev = cost;
    }
  }
  if (*bad_flag) {  // a symbol outside {0 .. 2^Q - 1}: no meaningful result
    best = __longlong_as_double(0x7ff8000000000000ll);
    n_tilde = n;
    evaluated = 0;
  }
  res->rows = n_tilde;
  res->cols = n / n_tilde;
  res->cost_bits = best;
  res->n_evaluated = evaluated;
  res->n_candidates = cands.n;
}

// an empty domain: rows = T, cols = 1, cost +inf
__global__ void k_rs_empty(uint32_t n, const uint32_t *bad_flag, rans_reshape_result *res) {
  res->rows = n;
  res->cols = 1;
  res->cost_bits = *bad_flag ? __longlong_as_double(0x7ff8000000000000ll) : INFINITY;
  res->n_evaluated = 0;
  res->n_candidates = 0;
}

}  // namespace
