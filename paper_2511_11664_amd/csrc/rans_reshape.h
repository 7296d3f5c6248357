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
struct RsOffsets {  // first bin of each candidate's column / row-count histogram; entry n = total
  uint32_t hc[RANS_RESHAPE_MAX_CAND + 1], hr[RANS_RESHAPE_MAX_CAND + 1];
};

__global__ __launch_bounds__(kWG) void k_rs_mask(const uint8_t *sym, uint32_t n, int aligned, uint32_t n_tiles,
                                                 uint16_t *mask16, uint16_t *lp, uint32_t *tile_cnt, uint32_t *hv,
                                                 uint32_t q_bits, uint32_t *bad_flag) {
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;  // kWG == 256
  __syncthreads();
  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const uint64_t e0 = (uint64_t)tile * kRsTile + threadIdx.x * 16;
    uint8_t b[16];
    load16(sym, e0, n, aligned, b);
    uint32_t m = 0;
#pragma unroll
    for (int k = 0; k < 16; k++) {
      if (b[k]) {
        m |= 1u << k;
        if (b[k] >> q_bits) atomicOr(bad_flag, 1u);  // not a symbol of this bit width
        atomicAdd(&h[b[k]], 1u);
      }
    }
    uint32_t tot;
    const uint32_t ex = block_excl_scan<kWG>(__popc(m), sh, &tot);
    if (e0 < n) {
      mask16[e0 >> 4] = (uint16_t)m;
      lp[e0 >> 4] = (uint16_t)ex;
    }
    if (threadIdx.x == 0) tile_cnt[tile] = tot;
    __syncthreads();
  }
  const uint32_t t = h[threadIdx.x];
  if (t) atomicAdd(&hv[threadIdx.x], t);
}

// zeroes the histograms of a call (runs before k_rs_mask, which adds to hv)
__global__ void k_rs_zero(uint32_t *p, uint32_t words) {
  for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gridDim.x * blockDim.x) p[i] = 0;
}

// Histograms of c = position mod K over the nonzero positions, for the candidates [k0, k1): their bins
// sit one after the other in LDS (at most kRsColBins in total) and in hc (at hc_off[k]).
constexpr uint32_t kRsColBins = 8192;
__global__ __launch_bounds__(kWG) void k_rs_cols(const uint16_t *mask16, uint32_t n_entries, RsCands cands, uint32_t k0,
                                                 uint32_t k1, RsOffsets offs, uint32_t *hc) {
  __shared__ uint32_t h[kRsColBins];
  const uint32_t *hc_off = offs.hc;
  const uint32_t base0 = hc_off[k0], bins = hc_off[k1] - base0;
  for (uint32_t i = threadIdx.x; i < bins; i += kWG) h[i] = 0;
  __syncthreads();
  for (uint32_t e = blockIdx.x * kWG + threadIdx.x; e < n_entries; e += gridDim.x * kWG) {
    const uint32_t m = mask16[e];
    if (!m) continue;
    const uint32_t g0 = e * 16;  // n <= 2^30: fits
    for (uint32_t k = k0; k < k1; k++) {
      const uint32_t K = cands.K[k];
      uint32_t *hk = h + (hc_off[k] - base0);
      uint32_t c = g0 % K;
#pragma unroll
      for (int bit = 0; bit < 16; bit++) {
        if (m & (1u << bit)) atomicAdd(&hk[c], 1u);
        c = c + 1 == K ? 0 : c + 1;
      }
    }
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < bins; i += kWG) {
    const uint32_t t = h[i];
    if (t) atomicAdd(&hc[base0 + i], t);
  }
}

// nonzeros before position g (g <= n)
__device__ __forceinline__ uint32_t rs_prefix(uint32_t g, uint32_t n, uint32_t nnz, const uint16_t *mask16,
                                              const uint16_t *lp, const uint32_t *tile_off) {
  if (g >= n) return nnz;
  const uint32_t e = g >> 4;
  return tile_off[g / kRsTile] + lp[e] + __popc((uint32_t)mask16[e] & ((1u << (g & 15)) - 1u));
}

// Histogram of the row counts r for candidate blockIdx.y: r[i] = prefix((i + 1) K) - prefix(i K).
__global__ __launch_bounds__(kWG) void k_rs_rows(const uint16_t *mask16, const uint16_t *lp, const uint32_t *tile_off,
                                                 uint32_t n, uint32_t n_tiles, RsCands cands, RsOffsets offs,
                                                 uint32_t *hr) {
  __shared__ uint32_t h[257];
  const uint32_t *hr_off = offs.hr;
  const uint32_t k = blockIdx.y, K = cands.K[k];
  const uint32_t nnz = tile_off[n_tiles];
  uint32_t *out = hr + hr_off[k];
  if (K == 1) {  // the row counts are the zero mask itself
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      out[0] = n - nnz;
      out[1] = nnz;
    }
    return;
  }
  for (uint32_t i = threadIdx.x; i <= K; i += kWG) h[i] = 0;
  __syncthreads();
  const uint32_t N = n / K;
  for (uint32_t i = blockIdx.x * kWG + threadIdx.x; i < N; i += gridDim.x * kWG) {
    const uint32_t a = rs_prefix(i * K, n, nnz, mask16, lp, tile_off);
    const uint32_t b = rs_prefix(i * K + K, n, nnz, mask16, lp, tile_off);
    atomicAdd(&h[b - a], 1u);
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
                                                 const uint32_t *tile_off, const uint32_t *hv, const uint32_t *hc,
                                                 const uint32_t *hr, RsOffsets offs, const uint32_t *bad_flag,
                                                 double *costs, uint32_t *ticket, rans_reshape_result *res) {
  __shared__ double s_part[kWG / 64];
  __shared__ uint32_t s_ticket;
  const uint32_t *hc_off = offs.hc, *hr_off = offs.hr;
  const uint32_t k = blockIdx.x;
  const uint32_t nnz = tile_off[n_tiles];
  {
    const uint32_t K = cands.K[k], N = n / K;
    const uint32_t two_q = 1u << q_bits;
    const uint32_t A = K + 1 > two_q ? K + 1 : two_q;
    const uint64_t len = 2ull * nnz + N;
    double h = 0.0;
    for (uint32_t a = threadIdx.x; a < A; a += kWG) {
      uint64_t c = 0;
      if (a < two_q) c += hv[a];
      if (a < K) c += hc[hc_off[k] + a];
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
