// rans_quant.h -- Eq. 6 (extrema, quantise + histogram) and the frequency table (normalisation, encoder tables, header)
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

#include "rans_common.h"

namespace {

// ------------------------------------------------------------------ kernels: set-up

// ------------------------------------------------------------------ kernels: Eq. 6

// Start-of-call bookkeeping (done by one work-group of the first kernel of a call): reset the control
// block, clear the histogram and the encoder's per-chunk / per-work-group word counters.
__device__ void reset_call_state(const CtlRef &ctl, uint32_t *cnt, uint32_t A, uint32_t *chunk_words, uint32_t nc) {
  if (threadIdx.x == 0) {
    ctl->last_seq = ctl.seq;
    // A call captured into a graph keeps its number on every replay: an error that the previous replay recorded
    // is not this one's.  (Nothing else of this call has run yet: the kernel that gets here is its first, and
    // no other work-group of it touches the status.)
    if ((uint32_t)(*(volatile unsigned long long *)&ctl.p->status >> 32) == ctl.seq)
      *(volatile unsigned long long *)&ctl.p->status = 0;
    ctl->len_d = 0;
    ctl->payload_off = ctl->dir_off = ctl->total_bytes = 0;
    ctl->nnz = 0;
    ctl->n_chunks = 0;
    ctl->hist_done = 0;
  }
  for (uint32_t a = threadIdx.x; a < A; a += blockDim.x) cnt[a] = 0;
  for (uint32_t k = threadIdx.x; k <= nc; k += blockDim.x) chunk_words[k] = 0;
  __syncthreads();
}

// Partial extrema of one work-group of k_minmax.
struct MinMaxPart {
  float mn, mx;
  uint32_t bad, pad;
};

// Global extrema, first stage.  Each lane keeps a running min / max over 16-byte
// vector loads (four independent loads in flight per lane), the wave folds them
// with cross-lane shuffles, the work-group through LDS, and one lane writes the
// group's partial result.  No atomics: thousands of same-address atomics cost more
// than reading the tensor.
template <typename T, bool VEC>
__global__ __launch_bounds__(kWG) void k_minmax(const T *x, uint32_t n, MinMaxPart *part, CtlRef ctl, uint32_t *cnt,
                                                uint32_t A, uint32_t *chunk_words, uint32_t nc) {
  if (blockIdx.x == 0) reset_call_state(ctl, cnt, A, chunk_words, nc);  // nothing in this kernel uses that state
  constexpr int V = VEC ? (int)(16 / sizeof(T)) : 1;
  constexpr int U = 4;
  float mn = INFINITY, mx = -INFINITY;
  uint32_t bad = 0;
  auto take = [&](float v) {
    bad |= ((__float_as_uint(v) & 0x7fffffffu) >= 0x7f800000u);
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  };
  auto take_vec = [&](uint32_t i) {
    if constexpr (!VEC) {
      if constexpr (sizeof(T) == 4) take(((const float *)x)[i]);
      else take(half_bits_to_float(((const uint16_t *)x)[i]));
    }
  };
  const uint32_t nvec = n / V;
  const uint32_t stride = gridDim.x * blockDim.x;
  uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
  if constexpr (VEC) {
    for (; (uint64_t)i + (uint64_t)(U - 1) * stride < nvec; i += U * stride) {
      uint4 q[U];
#pragma unroll
      for (int u = 0; u < U; u++) q[u] = ((const uint4 *)x)[i + u * stride];
#pragma unroll
      for (int u = 0; u < U; u++) {
        uint32_t w[4] = {q[u].x, q[u].y, q[u].z, q[u].w};
#pragma unroll
        for (int k = 0; k < 4; k++) {
          if constexpr (sizeof(T) == 4) {
            take(__uint_as_float(w[k]));
          } else {
            take(half_bits_to_float((uint16_t)(w[k] & 0xffffu)));
            take(half_bits_to_float((uint16_t)(w[k] >> 16)));
          }
        }
      }
    }
    for (; i < nvec; i += stride) {
      uint4 q = ((const uint4 *)x)[i];
      uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int k = 0; k < 4; k++) {
        if constexpr (sizeof(T) == 4) {
          take(__uint_as_float(w[k]));
        } else {
          take(half_bits_to_float((uint16_t)(w[k] & 0xffffu)));
          take(half_bits_to_float((uint16_t)(w[k] >> 16)));
        }
      }
    }
    uint32_t t = nvec * V + blockIdx.x * blockDim.x + threadIdx.x;  // ragged tail, fewer than V elements
    if (t < n) {
      if constexpr (sizeof(T) == 4) take(((const float *)x)[t]);
      else take(half_bits_to_float(((const uint16_t *)x)[t]));
    }
  } else {
    for (; i < nvec; i += stride) take_vec(i);
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, d));
    mx = fmaxf(mx, __shfl_xor(mx, d));
    bad |= __shfl_xor(bad, d);
  }
  __shared__ float s_mn[kWG / 64], s_mx[kWG / 64];
  __shared__ uint32_t s_bad[kWG / 64];
  if ((threadIdx.x & 63) == 0) {
    s_mn[threadIdx.x >> 6] = mn;
    s_mx[threadIdx.x >> 6] = mx;
    s_bad[threadIdx.x >> 6] = bad;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < kWG / 64; w++) {
      mn = fminf(mn, s_mn[w]);
      mx = fmaxf(mx, s_mx[w]);
      bad |= s_bad[w];
    }
    part[blockIdx.x] = MinMaxPart{mn, mx, bad, 0u};
  }
}

// Second stage of the extrema, then scale and zero point (Eq. 6), by a whole work-group of NT lanes:
// every lane returns the same values.  `bad` reports non-finite input or an overflowing range; the
// values are NaN then.
template <int NT>
__device__ rans_qinfo qinfo_from_parts(const MinMaxPart *part, uint32_t n_part, uint32_t q_bits, bool *bad_out) {
  float mn = INFINITY, mx = -INFINITY;
  uint32_t bad = 0;
  for (uint32_t i = threadIdx.x; i < n_part; i += NT) {
    MinMaxPart q = part[i];
    mn = fminf(mn, q.mn);
    mx = fmaxf(mx, q.mx);
    bad |= q.bad;
  }
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, d));
    mx = fmaxf(mx, __shfl_xor(mx, d));
    bad |= __shfl_xor(bad, d);
  }
  __shared__ float s_mn[NT / 64], s_mx[NT / 64];
  __shared__ uint32_t s_bad[NT / 64];
  if ((threadIdx.x & 63) == 0) {
    s_mn[threadIdx.x >> 6] = mn;
    s_mx[threadIdx.x >> 6] = mx;
    s_bad[threadIdx.x >> 6] = bad;
  }
  __syncthreads();
  mn = s_mn[0];
  mx = s_mx[0];
  bad = s_bad[0];
  for (int w = 1; w < NT / 64; w++) {
    mn = fminf(mn, s_mn[w]);
    mx = fmaxf(mx, s_mx[w]);
    bad |= s_bad[w];
  }
  if (n_part == 0) mn = mx = 0.0f;  // empty tensor
  mn = mn + 0.0f;                    // -0.0 becomes +0.0
  mx = mx + 0.0f;
  float range = mx - mn;
  float levels = (float)((1u << q_bits) - 1u);
  float s = range / levels;
  float zf = eq6_zero_point(mn, s);
  const bool is_bad = bad || !(fabsf(range) < INFINITY);
  if (is_bad) mn = mx = s = zf = __uint_as_float(0x7fc00000u);
  *bad_out = is_bad;
  return rans_qinfo{mn, mx, s, zf};
}

__device__ void publish_qinfo(const CtlRef &ctl, const rans_qinfo &q, bool bad, rans_qinfo *out) {
  if (bad) set_status(ctl, RANS_ERR_NONFINITE);
  ctl->x_min = q.x_min;
  ctl->x_max = q.x_max;
  ctl->scale = q.scale;
  ctl->zero_point = q.zero_point;
  if (out) *out = q;
}

// The same as a kernel of one work-group, with the start-of-call bookkeeping (empty tensors: no other
// kernel runs before it).
__global__ __launch_bounds__(kBig) void k_qinfo(CtlRef ctl, const MinMaxPart *part, uint32_t n_part, uint32_t q_bits,
                                                rans_qinfo *out, uint32_t *cnt, uint32_t A, uint32_t *chunk_words,
                                                uint32_t nc) {
  reset_call_state(ctl, cnt, A, chunk_words, nc);
  bool bad;
  const rans_qinfo q = qinfo_from_parts<kBig>(part, n_part, q_bits, &bad);
  if (threadIdx.x == 0) publish_qinfo(ctl, q, bad, out);
}

// Copies caller-provided extrema into the control block (rans_encode path) and
// recomputes s, z from them with the arithmetic of k_qinfo.
__global__ __launch_bounds__(kBig) void k_qinfo_from_user(CtlRef ctl, const rans_qinfo *in, uint32_t q_bits,
                                                          uint32_t *cnt, uint32_t A, uint32_t *chunk_words,
                                                          uint32_t nc) {
  reset_call_state(ctl, cnt, A, chunk_words, nc);
  if (threadIdx.x != 0) return;
  float mn = in->x_min, mx = in->x_max;
  float range = mx - mn;
  bool bad = !(fabsf(mn) < INFINITY) || !(fabsf(mx) < INFINITY) || !(fabsf(range) < INFINITY) || mn > mx;
  if (bad) set_status(ctl, RANS_ERR_NONFINITE);
  float levels = (float)((1u << q_bits) - 1u);
  float s = range / levels;
  float zf = eq6_zero_point(mn, s);
  ctl->x_min = mn + 0.0f;
  ctl->x_max = mx + 0.0f;
  ctl->scale = s;
  ctl->zero_point = zf;
}

// ------------------------------------------------------------------ kernels: frequency table

__device__ __forceinline__ void st32(uint8_t *p, uint32_t v) { *(uint32_t *)p = v; }
__device__ __forceinline__ uint32_t ld32(const uint8_t *p) { return *(const uint32_t *)p; }
__device__ __forceinline__ uint64_t ld64(const uint8_t *p) { return (uint64_t)ld32(p) | ((uint64_t)ld32(p + 4) << 32); }

// One work-group: counts -> f with sum 2^M (largest-count symbol absorbs a surplus,
// largest-f symbols pay a deficit, lowest index on ties), F = exclusive cumulative
// sum, encoder table {reciprocal, f | F << 16}, container header and table.
struct NormArgs {
  const uint32_t *cnt;      // histogram of D; n_rep partial histograms of A words each follow it (their sum counts)
  uint32_t n_rep;
  const uint32_t *lds_cnt;  // the folded counts in LDS, when the calling kernel has put them there (set inside it)
  uint32_t *fq;
  uint2 *enc_tab;
  uint4 *enc_tab4;
  uint32_t A;
  rans_params p;
  uint64_t n_elems;
  int dense;
  uint8_t *out;
  uint64_t cap;
  // The extrema, when the kernel that builds the table has computed them itself (set inside that kernel;
  // the control block's copy was then written by another of its work-groups and is not read).
  int mm_given;
  float x_min, x_max;
  // Set by a kernel in which every work-group builds the table for itself (the encoder): only the first one
  // writes the container's header and table and the control block's geometry; the others keep what they
  // compute to themselves.  0: the caller is the table's only builder and writes everything.
  int quiet;
  int entry_checked;  // the caller has looked at the call's status already (set inside the calling kernel)
  // Set by a kernel whose whole work-group makes the table entries (emit_entries) after one wave has normalised:
  // the wave then only leaves {f, F} of symbol a in fF[2 a] (the first half of the symbol's 16-byte table slot).
  uint2 *fF;
};
// What the table build leaves in the registers of the wave or work-group that ran it.
struct NormResult {
  uint32_t ok;  // 0: an error has been recorded, nothing below is valid
  uint32_t exact;
  uint32_t n_chunks;
  uint64_t len_d, dir_off, payload_off;
};
// Count of symbol a: the histogram's entry plus those of the partial histograms behind it.  Plain loads: the
// histogram was completed by kernels that ended before the one that reads it began.
__device__ __forceinline__ uint32_t hist_count(const NormArgs &na, uint32_t a) {
  if (na.lds_cnt) return na.lds_cnt[a];
  uint32_t c = na.cnt[a];
  for (uint32_t k = 1; k <= na.n_rep; k++) c += na.cnt[(size_t)k * na.A + a];
  return c;
}
// Container header (fixed part) and the geometry the later kernels read from the control block.
__device__ __forceinline__ void write_header(const CtlRef &ctl, const NormArgs &na, uint64_t len_d, uint64_t n_chunks, uint64_t dir_off,
                             uint64_t payload_off) {
  const rans_params &p = na.p;
  uint8_t *out = na.out;
  ctl->n_chunks = (uint32_t)n_chunks;
  ctl->dir_off = dir_off;
  ctl->payload_off = payload_off;
  st32(out + 0, 0x31464952u);  // "RIF1"
  st32(out + 4, 1u | (p.mode << 16) | (p.in_dtype << 24));
  st32(out + 8, p.q_bits | (p.freq_bits << 8));
  st32(out + 12, (uint32_t)na.n_elems);    st32(out + 16, (uint32_t)(na.n_elems >> 32));
  st32(out + 20, (uint32_t)p.rows);        st32(out + 24, (uint32_t)(p.rows >> 32));
  st32(out + 28, (uint32_t)p.cols);        st32(out + 32, (uint32_t)(p.cols >> 32));
  st32(out + 36, (uint32_t)len_d);         st32(out + 40, (uint32_t)(len_d >> 32));
  st32(out + 44, na.A);
  st32(out + 48, p.n_streams);
  st32(out + 52, p.chunk_syms);
  st32(out + 56, (uint32_t)n_chunks);
  st32(out + 60, __float_as_uint(na.mm_given ? na.x_min : ctl->x_min));
  st32(out + 64, __float_as_uint(na.mm_given ? na.x_max : ctl->x_max));
  for (uint32_t o = 68; o < kHdrBytes; o += 4) st32(out + o, 0u);
}

// floor(n / d) for n < 2^48 and 1 <= d < 2^32 when that quotient is below 2^17, without an integer or
// binary64 division (each a long dependent instruction sequence here).  The binary32 estimate n * (1 / d)
// carries a relative error below 2^-21 (two conversions, a reciprocal good to one unit in the last place, a
// product), that is less than 1/16 absolute for such quotients, so its truncation is the quotient or one
// off; the exact remainder then says which.
__device__ __forceinline__ uint32_t div_small_quot(uint64_t n, uint32_t d) {
  const float nf = __builtin_fmaf((float)(uint32_t)(n >> 32), 4294967296.0f, (float)(uint32_t)n);
  uint32_t q = (uint32_t)(nf * __builtin_amdgcn_rcpf((float)d));
  const int64_t r = (int64_t)n - (int64_t)((uint64_t)q * d);
  q = r < 0 ? q - 1 : (r >= (int64_t)d ? q + 1 : q);
  return q;
}
// floor(2^(32+k) / d) for 2^k <= d < 2^(k+1), d < 2^16: long division in base 2^16, whose two digits
// are quotients of the kind above (the first lies in (2^15, 2^16], the second below 2^16).
__device__ __forceinline__ uint64_t div_pow2_by(uint32_t k, uint32_t d) {
  const uint32_t n1 = 1u << (16 + k);
  const uint32_t q1 = div_small_quot(n1, d);
  const uint32_t r1 = n1 - q1 * d;  // < d
  const uint32_t q2 = div_small_quot((uint64_t)r1 << 16, d);
  return ((uint64_t)q1 << 16) + q2;
}

// Checks the two routines above against integer division (see rans_selftest_divide).
__global__ void k_selftest_clear(uint32_t *mismatches) { *mismatches = 0; }
__global__ __launch_bounds__(kWG) void k_selftest_divide(uint32_t *mismatches, uint64_t n_random) {
  const uint64_t i = (uint64_t)blockIdx.x * kWG + threadIdx.x;
  uint32_t bad = 0;
  if (i >= 1 && i < 65536) {
    const uint32_t d = (uint32_t)i, k = 31u - (uint32_t)__clz((int)d);
    bad += div_pow2_by(k, d) != (1ull << (32 + k)) / d;
  }
  for (uint64_t t = i; t < n_random; t += (uint64_t)gridDim.x * kWG) {
    // a divisor of 1 .. 32 bits, a quotient below 2^17 and a remainder, from a mixing function of t
    uint64_t h = (t + 1) * 0x9e3779b97f4a7c15ull;
    h ^= h >> 29; h *= 0xbf58476d1ce4e5b9ull; h ^= h >> 32;
    const uint32_t bits = 1 + (uint32_t)(h % 32);
    uint64_t h2 = h * 0x94d049bb133111ebull; h2 ^= h2 >> 31;
    uint32_t d = (uint32_t)(h2 >> 32) >> (32 - bits);
    d = d ? d : 1u;
    const uint32_t q = (uint32_t)(h2 & 0x1ffffu);
    uint64_t h3 = h2 * 0xd6e8feb86659fd93ull; h3 ^= h3 >> 32;
    const uint32_t r = t % 3 == 0 ? 0u : (t % 3 == 1 ? d - 1 : (uint32_t)(h3 % d));  // both ends of the remainder's range
    const uint64_t n = (uint64_t)q * d + r;
    if (n < (1ull << 48)) bad += div_small_quot(n, d) != q;
  }
  if (bad) atomicAdd(mismatches, bad);
}

// Everything stored per symbol: f in the container, the encoder's two table entries.  div(k, d) returns
// floor(2^(32+k) / d) for 2^k <= d < 2^(k+1), d < 2^16.  Returns whether the division-free entry is inexact.
//
// Division-free entry {lim1, mx, Fx | sh << 16, 2^M - f}: the coder renormalises when s > lim1 and
// then takes q = mulhi(s, mx) >> sh for floor(s / f) in Eq. 2.  At that point s <= lim1 =
// f * 2^(32-M) - 1.  With 2^k <= f < 2^(k+1), mx = floor(2^(32+k) / f) + 1 and e = mx * f - 2^(32+k),
// q is exact for every s with s * e < 2^(32+k); the entry is marked inexact otherwise (possible only
// for f > 2^(M-1)).  Powers of two take mx = 2^31, sh = k - 1.  f = 1 cannot have its multiplier
// 2^32: it takes mx = 2^32 - 1, which gives q = s - 1 (s >= 1 there), and the missing 2^M - f is
// added to Fx instead.  f = 0 (absent symbol) is never looked up.
//
// The one division is made for every symbol, whatever its case, and the cases select afterwards: the
// divisions of a lane's symbols are then independent instruction streams that overlap, where branches
// around them would run them one after the other.  The fallback entry's floor(2^32 / f) is the same
// quotient shifted down by k (floors of successive integer divisions compose).
template <class Div>
__device__ __forceinline__ int emit_entries(const NormArgs &na, uint32_t a, uint32_t f, uint32_t F, Div div,
                                            bool store = true) {
  const uint32_t M = na.p.freq_bits, total = 1u << M;
  const uint32_t fd = f ? f : 1u;
  const uint32_t k = 31u - (uint32_t)__clz((int)fd);
  const uint64_t two = 1ull << (32 + k);
  const uint64_t quo = div(k, fd);  // 2^32 for a power of two, else below 2^32 (f > 2^k)
  // floor(2^32 / f) for f >= 2, 2^32 - 1 for f = 1: with it mulhi(s, m) is floor(s / f) or one less
  const uint32_t m = f <= 1 ? 0xffffffffu : (uint32_t)(quo >> k);
  const uint32_t cmpl = total - f;
  const uint32_t lim1 = (f << (32 - M)) - 1u;
  const bool pow2 = (f & (f - 1)) == 0;  // also f = 0, 1
  const uint64_t mq = quo + 1;
  const uint64_t e = mq * fd - two;
  const int inexact = !pow2 && (uint64_t)lim1 * e >= two;
  uint32_t mx = pow2 ? 0x80000000u : (uint32_t)mq, sh = pow2 ? k - 1 : k, Fx = F;
  if (f == 1) {
    mx = 0xffffffffu;
    sh = 0;
    Fx = F + cmpl;
  } else if (f == 0) {
    mx = 0;
    sh = 0;
  }
  if (store) {  // a symbol of the alphabet (the caller may pass lanes beyond it, with f = 0)
    na.enc_tab[a] = make_uint2(m, f | (F << 16));
    if (!na.quiet) *(uint16_t *)(na.out + kHdrBytes + 2ull * a) = (uint16_t)f;
    na.enc_tab4[a] = make_uint4(lim1, mx, Fx | (sh << 16), cmpl);
  }
  return store && inexact;
}

__device__ void normalize_body(const CtlRef &ctl, const NormArgs &na) {
  uint32_t *fq = na.fq;
  uint2 *enc_tab = na.enc_tab;
  uint4 *enc_tab4 = na.enc_tab4;
  const uint32_t A = na.A;
  const rans_params &p = na.p;
  const uint64_t n_elems = na.n_elems;
  const int dense = na.dense;
  uint8_t *out = na.out;
  const uint64_t cap = na.cap;
  __shared__ uint64_t sh64[kBig / 64];
  __shared__ uint32_t sh32[kBig / 64];
  __shared__ int64_t s_d;
  const uint32_t M = p.freq_bits, total = 1u << M;
  if (group_has_status(ctl)) return;
  uint64_t len_loc = 0, present_loc = 0;
  for (uint32_t a = threadIdx.x; a < A; a += kBig) {
    uint32_t c = hist_count(na, a);
    len_loc += c;
    present_loc += c != 0;
  }
  const uint64_t len = block_sum64<kBig>(len_loc, sh64);
  const uint64_t present = block_sum64<kBig>(present_loc, sh64);
  // l_D as the rest of the call knows it: the tensor's size (DENSE), or what the row-count kernel derived from
  // the row ends.  A histogram that does not add up to it becomes an error, never a wrong table.
  const uint64_t len_d = dense ? n_elems : ctl->len_d;
  if (dense && threadIdx.x == 0) ctl->len_d = len_d;
  if (present > total || len != len_d) {
    if (threadIdx.x == 0) set_status(ctl, len != len_d ? RANS_ERR_HIP : RANS_ERR_ALPHABET);
    return;
  }
  // first estimate and its sum
  uint64_t sum_loc = 0, best_cnt = 0;
  for (uint32_t a = threadIdx.x; a < A; a += kBig) {
    uint32_t c = hist_count(na, a);
    uint32_t f = 0;
    if (c) {
      const uint32_t q = div_small_quot((uint64_t)c * total + len / 2, (uint32_t)len);  // at most 2^M
      f = q < 1 ? 1u : q;
      uint64_t key = ((uint64_t)c << 32) | (0xffffffffu - a);  // max count, lowest index
      best_cnt = key > best_cnt ? key : best_cnt;
    }
    fq[a] = f;
    sum_loc += f;
  }
  const uint64_t sum = block_sum64<kBig>(sum_loc, sh64);
  const uint64_t best = block_max64<kBig>(best_cnt, sh64);
  int64_t d = (int64_t)total - (int64_t)sum;
  if (len && d > 0) {
    if (threadIdx.x == 0) fq[0xffffffffu - (uint32_t)best] += (uint32_t)d;
    d = 0;
  }
  __syncthreads();
  while (d < 0) {  // uniform loop: d is identical in every thread
    uint64_t kb = 0;
    for (uint32_t a = threadIdx.x; a < A; a += kBig) {
      uint64_t key = ((uint64_t)fq[a] << 32) | (0xffffffffu - a);
      kb = key > kb ? key : kb;
    }
    kb = block_max64<kBig>(kb, sh64);
    uint32_t a_star = 0xffffffffu - (uint32_t)kb;
    int64_t take = (int64_t)(kb >> 32) - 1;
    if (take > -d) take = -d;
    if (threadIdx.x == 0) {
      fq[a_star] -= (uint32_t)take;
      s_d = d + take;
    }
    __syncthreads();
    d = s_d;
    __syncthreads();
  }
  // container geometry
  const uint64_t n_chunks = len_d == 0 ? 0 : (p.chunk_syms == 0 ? 1 : (len_d + p.chunk_syms - 1) / p.chunk_syms);
  const uint64_t table_off = kHdrBytes;
  const uint64_t dir_off = table_off + (((uint64_t)A * 2 + 7) & ~7ull);
  const uint64_t payload_off = dir_off + 8 * (n_chunks + 1);
  if (payload_off > cap) {
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CAPACITY);
    return;
  }
  if (threadIdx.x == 0) write_header(ctl, na, len_d, n_chunks, dir_off, payload_off);
  // cumulative sum, encoder table, stored table
  uint32_t carry = 0;
  int inexact = 0;
  for (uint32_t base = 0; base < A; base += kBig) {
    uint32_t a = base + threadIdx.x;
    uint32_t f = a < A ? fq[a] : 0, tot;
    uint32_t F = carry + block_excl_scan<kBig>(f, sh32, &tot);
    if (a < A) {
      inexact |= emit_entries(na, a, f, F, [](uint32_t k, uint32_t d) { return div_pow2_by(k, d); });
    }
    carry += tot;
    __syncthreads();
  }
  inexact = __syncthreads_or(inexact);
  if (threadIdx.x == 0) ctl->enc_exact = inexact ? 0u : 1u;
  for (uint64_t o = table_off + 2ull * A + 2 * threadIdx.x; o < dir_off; o += 2 * kBig) *(uint16_t *)(out + o) = 0;
}

// The same as normalize_body for alphabets of up to 64 PER symbols, by ONE wave without a barrier: lane l
// owns the symbols PER l .. PER l + PER - 1, sums and maxima are wave scans.  Called by the first wave of a
// work-group (of the encoder, where every work-group builds the table for itself, or of k_normalize).  About
// a thousand instructions of one wave; sharing the symbols out over the four waves of an encoder work-group
// was measured and is no faster, since the barriers and the four-fold instruction issue eat the gain.
constexpr uint32_t kNormWaveA = 512;
template <int PER>
__device__ __forceinline__ NormResult normalize_wave_per(const CtlRef &ctl, const NormArgs &na) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t A = na.A;
  const rans_params &p = na.p;
  const uint32_t M = p.freq_bits, total = 1u << M;
  NormResult res{};
  if (!na.entry_checked && __ballot(status_at_entry(ctl) != 0) != 0) return res;  // one decision for the wave
  auto total64 = [](uint64_t v) { return lane63_64(wave_incl_scan64(v, [](uint64_t a, uint64_t b) { return a + b; })); };
  auto max64 = [](uint64_t v) { return lane63_64(wave_incl_scan64(v, [](uint64_t a, uint64_t b) { return a > b ? a : b; })); };
  uint32_t c[PER];
#pragma unroll
  for (int q = 0; q < PER; q++) {
    const uint32_t a = PER * lane + q;
    c[q] = a < A ? hist_count(na, a) : 0;
  }
  uint64_t lp = 0;  // l_D in the low 40 bits, the number of present symbols above
#pragma unroll
  for (int q = 0; q < PER; q++) lp += (uint64_t)c[q] + ((uint64_t)(c[q] != 0) << 40);
  lp = total64(lp);
  const uint64_t len = lp & ((1ull << 40) - 1), present = lp >> 40;
  // l_D as the rest of the call knows it: the tensor's size (DENSE), or - CSR mode - what the row-count kernel
  // derived from the row ends.  A histogram that does not add up to it becomes an error, never a wrong table.
  const uint64_t len_d = na.dense ? na.n_elems : ctl->len_d;
  if (na.dense && !na.quiet && lane == 0) ctl->len_d = len_d;
  if (present > total || len != len_d) {
    if (lane == 0) set_status(ctl, len != len_d ? RANS_ERR_HIP : RANS_ERR_ALPHABET);
    return res;
  }
  // first estimate, its sum, the symbol with the largest count
  uint32_t f[PER];
  uint64_t sum = 0, best = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) {
    // the division is made for absent symbols too (and for an empty D, by 1): see emit_entries on branches
    const uint32_t e = div_small_quot((uint64_t)c[q] * total + len / 2, len ? (uint32_t)len : 1u);  // at most 2^M
    f[q] = c[q] ? (e < 1 ? 1u : e) : 0u;
    const uint64_t key = ((uint64_t)c[q] << 32) | (0xffffffffu - (PER * lane + q));  // max count, lowest index
    best = c[q] && key > best ? key : best;
    sum += f[q];
  }
  sum = total64(sum);
  best = max64(best);
  int64_t d = (int64_t)total - (int64_t)sum;
  auto adjust = [&](uint32_t a_star, int64_t by) {  // f[a_star] += by, in the lane that owns it
#pragma unroll
    for (int q = 0; q < PER; q++)
      if (PER * lane + q == a_star) f[q] = (uint32_t)((int64_t)f[q] + by);
  };
  if (len && d > 0) {
    adjust(0xffffffffu - (uint32_t)best, d);
    d = 0;
  }
  while (d < 0) {  // uniform: d is identical in every lane
    uint64_t kb = 0;
#pragma unroll
    for (int q = 0; q < PER; q++) {
      const uint64_t key = ((uint64_t)f[q] << 32) | (0xffffffffu - (PER * lane + q));
      kb = PER * lane + q < A && key > kb ? key : kb;
    }
    kb = max64(kb);
    int64_t take = (int64_t)(kb >> 32) - 1;
    if (take > -d) take = -d;
    adjust(0xffffffffu - (uint32_t)kb, -take);
    d += take;
  }
  // container geometry
  // l_D < 2^32 (at most 3 * 2^30): a 32-bit division, far shorter than the 64-bit one
  uint64_t n_chunks = len_d == 0 ? 0 : 1;
  if (len_d && p.chunk_syms) {
    const uint32_t qc = (uint32_t)len_d / p.chunk_syms;
    n_chunks = qc + ((uint32_t)len_d - qc * p.chunk_syms != 0);
  }
  const uint64_t table_off = kHdrBytes;
  const uint64_t dir_off = table_off + (((uint64_t)A * 2 + 7) & ~7ull);
  const uint64_t payload_off = dir_off + 8 * (n_chunks + 1);
  if (payload_off > na.cap) {
    if (lane == 0) set_status(ctl, RANS_ERR_CAPACITY);
    return res;
  }
  if (!na.quiet && lane == 0) write_header(ctl, na, len_d, n_chunks, dir_off, payload_off);
  // cumulative sum, encoder tables, stored table
  uint32_t mine = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) mine += f[q];
  uint32_t F = wave_incl_sum_scan(mine) - mine;
  if (na.fF) {  // the entries are made by the caller's whole work-group
#pragma unroll
    for (int q = 0; q < PER; q++) {
      const uint32_t a = PER * lane + q;
      if (a < A) na.fF[2 * a] = make_uint2(f[q], F);
      F += f[q];
    }
    if (!na.quiet)
      for (uint64_t o = table_off + 2ull * A + 2 * lane; o < dir_off; o += 2 * 64) *(uint16_t *)(na.out + o) = 0;
    res.ok = 1;
    res.n_chunks = (uint32_t)n_chunks;
    res.len_d = len_d;
    res.dir_off = dir_off;
    res.payload_off = payload_off;
    return res;
  }
  int inexact = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) {
    const uint32_t a = PER * lane + q;
    inexact |= emit_entries(na, a, f[q], F, [](uint32_t k, uint32_t d) { return div_pow2_by(k, d); }, a < A);
    F += f[q];
  }
  const bool any_inexact = __ballot(inexact) != 0;
  if (!na.quiet) {
    if (lane == 0) ctl->enc_exact = any_inexact ? 0u : 1u;
    for (uint64_t o = table_off + 2ull * A + 2 * lane; o < dir_off; o += 2 * 64) *(uint16_t *)(na.out + o) = 0;
  }
  res.ok = 1;
  res.exact = any_inexact ? 0u : 1u;
  res.n_chunks = (uint32_t)n_chunks;
  res.len_d = len_d;
  res.dir_off = dir_off;
  res.payload_off = payload_off;
  return res;
}

__device__ __forceinline__ NormResult normalize_wave(const CtlRef &ctl, const NormArgs &na) {
  // as few symbols per lane as the alphabet allows (CSR with K = 2^Q has 2^Q + 1 symbols)
  if (na.A <= 256) return normalize_wave_per<4>(ctl, na);
  if (na.A <= 320) return normalize_wave_per<5>(ctl, na);
  if (na.A <= 384) return normalize_wave_per<6>(ctl, na);
  return normalize_wave_per<8>(ctl, na);
}

__global__ __launch_bounds__(kBig) void k_normalize(CtlRef ctl, NormArgs na) {
  if (na.A <= kNormWaveA) {
    if (threadIdx.x < 64) normalize_wave(ctl, na);
  } else {
    normalize_body(ctl, na);
  }
}

// Quantise a tile and histogram its symbols.  T = float / __half: Eq. 6 per
// element, symbols written packed; T = uint8_t: symbols are the input (histogram
// only).  The LDS histogram is replicated 8 ways (bin * 8 + lane % 8) so that the
// few hot symbols of an activation tensor do not serialise the whole wave on one
// LDS address.
constexpr int kHistRep = 8;
constexpr int kQIter = 4;
constexpr int QNT = 1024;                // lanes per work-group of the quantise / histogram kernel
constexpr uint32_t kQuantBlocks = 256;   // its work-groups (persistent over tiles): few of them, because each one ends
                                         // with a burst of same-address atomics on the global histogram
constexpr uint32_t kQuantBlocksCsr = 512;  // CSR mode, where every tile ends with two barriers for its nonzero counts:
                                           // two work-groups per compute unit overlap them (c2: 30.4 -> 28.3 us; the
                                           // dense kernel is 4 us slower on c5a with 512)

template <typename T, bool VEC, int NT, bool CSR>
__global__ __launch_bounds__(NT) void k_quant_hist(const T *x, uint32_t n, CtlRef ctl, uint32_t q_bits,
                                                    uint8_t *sym, uint32_t *cnt, int skip_zero_bin,
                                                    const MinMaxPart *part, uint32_t n_part, rans_qinfo *qout,
                                                    uint32_t *blk_nnz, uint32_t *grp_nnz) {
  constexpr bool IS_SYM = sizeof(T) == 1;
  constexpr int V = VEC ? (int)(16 / sizeof(T)) : 1;
  __shared__ uint32_t h[256 * kHistRep];
  for (int i = threadIdx.x; i < 256 * kHistRep; i += NT) h[i] = 0;
  // Eq. 6's parameters: from the partial extrema (every work-group reduces them itself and gets the
  // same values; the first one records them), or from the control block when there are none
  rans_qinfo qi;
  if (part) {
    bool bad;
    qi = qinfo_from_parts<NT>(part, n_part, q_bits, &bad);
    if (blockIdx.x == 0 && threadIdx.x == 0) publish_qinfo(ctl, qi, bad, qout);
  } else {
    qi = rans_qinfo{ctl->x_min, ctl->x_max, ctl->scale, ctl->zero_point};
  }
  __syncthreads();
  // s == 0 (constant tensor): quantise with s = 1, z = 0 and a top level of 0, which maps everything
  // to symbol 0 without a branch in the loop
  const bool degenerate = !IS_SYM && !(qi.scale != 0.0f);
  const float s = degenerate ? 1.0f : qi.scale, zf = degenerate ? 0.0f : qi.zero_point;
  const float levels = degenerate ? 0.0f : (float)((1u << q_bits) - 1u);
  const float amax = fmaxf(fabsf(qi.x_min), fabsf(qi.x_max));
  const bool fast = s >= 0x1p-30f && s <= 0x1p30f && amax <= 0x1p30f;  // uniform; see FastDiv
  FastDiv fd;
  fd.init(s);
  const uint32_t rep = threadIdx.x & (kHistRep - 1);
  const uint32_t tile = NT * V * kQIter;
  // CSR: the nonzeros of each tile of kCsrTile symbols are counted on the way.  A work-group's tile of
  // NT * V * kQIter elements is V such tiles and a wave's symbols of one step lie in one of them: the lanes'
  // counts are summed with a wave scan, the last lane adds the sum to the tile's LDS counter, and after the
  // work-group's tile the counters go out with plain stores (every tile is counted by exactly one work-group).
  __shared__ uint32_t s_nz[16];
  static_assert(V <= 16, "one LDS counter per tile of kCsrTile symbols");
  if (CSR && threadIdx.x < 16) s_nz[threadIdx.x] = 0;  // ordered by the barrier below
  uint32_t lane_nz = 0;
  auto bump = [&](uint32_t a) {
    atomicAdd(&h[a * kHistRep + rep], 1u);
    if constexpr (CSR) lane_nz += a != 0;
  };
  auto run = [&](auto fast_tag) {
  constexpr bool FAST = decltype(fast_tag)::value;
  auto q = [&](float v) -> uint32_t {
    const float t = FAST ? fd.div(v) : v / s;
    const float r = rintf(t + zf);
    return (uint32_t)__builtin_amdgcn_fmed3f(r, 0.0f, levels);
  };
  // a work-group walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... and flushes its histogram once
  for (uint64_t base = (uint64_t)blockIdx.x * tile; base < n; base += (uint64_t)gridDim.x * tile) {
#pragma unroll
  for (int it = 0; it < kQIter; it++) {
    uint64_t e0 = base + ((uint64_t)it * NT + threadIdx.x) * V;
    if (!CSR && e0 >= n) break;
    if (e0 < n) {
    if (VEC && e0 + V <= n) {
      if constexpr (IS_SYM) {
        uint4 w = *(const uint4 *)((const uint8_t *)x + e0);
        uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int k = 0; k < 4; k++) {
          bump(ww[k] & 0xffu); bump((ww[k] >> 8) & 0xffu); bump((ww[k] >> 16) & 0xffu); bump(ww[k] >> 24);
        }
      } else if constexpr (sizeof(T) == 4) {
        float4 f = *(const float4 *)((const float *)x + e0);
        uint32_t a0 = q(f.x), a1 = q(f.y), a2 = q(f.z), a3 = q(f.w);
        bump(a0); bump(a1); bump(a2); bump(a3);
        *(uint32_t *)(sym + e0) = a0 | (a1 << 8) | (a2 << 16) | (a3 << 24);
      } else {
        uint4 w = *(const uint4 *)((const uint16_t *)x + e0);
        uint32_t ww[4] = {w.x, w.y, w.z, w.w};
        uint32_t a[8];
#pragma unroll
        for (int k = 0; k < 4; k++) {
          a[2 * k] = q(half_bits_to_float((uint16_t)(ww[k] & 0xffffu)));
          a[2 * k + 1] = q(half_bits_to_float((uint16_t)(ww[k] >> 16)));
        }
#pragma unroll
        for (int k = 0; k < 8; k++) bump(a[k]);
        uint2 o;
        o.x = a[0] | (a[1] << 8) | (a[2] << 16) | (a[3] << 24);
        o.y = a[4] | (a[5] << 8) | (a[6] << 16) | (a[7] << 24);
        *(uint2 *)(sym + e0) = o;
      }
    } else {  // scalar path: unaligned buffers, or the last partial vector
      for (int k = 0; k < V && e0 + k < n; k++) {
        uint32_t a;
        if constexpr (IS_SYM) a = ((const uint8_t *)x)[e0 + k];
        else if constexpr (sizeof(T) == 4) a = q(((const float *)x)[e0 + k]);
        else a = q(half_bits_to_float(((const uint16_t *)x)[e0 + k]));
        bump(a);
        if constexpr (!IS_SYM) sym[e0 + k] = (uint8_t)a;
      }
    }
    }  // e0 < n
    if constexpr (CSR) {  // every lane of the wave is here; lane 0 holds the wave's lowest element
      const uint32_t wave_nz = wave_incl_sum_scan(lane_nz);
      lane_nz = 0;
      const uint32_t slot = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((e0 - base) / kCsrTile));
      if ((threadIdx.x & 63) == 63 && wave_nz) atomicAdd(&s_nz[slot], wave_nz);
    }
  }
  if constexpr (CSR) {
    __syncthreads();
    if (threadIdx.x < 64) {  // the first wave; V <= 16 of its lanes hold a tile each
      const bool mine = threadIdx.x < V;
      const uint64_t t_idx = base / kCsrTile + threadIdx.x;
      const uint32_t c_t = mine ? s_nz[threadIdx.x] : 0u;
      const uint32_t upto = wave_incl_sum_scan(c_t);
      if (mine) {
        s_nz[threadIdx.x] = 0;
        if (t_idx * kCsrTile < n) blk_nnz[t_idx] = c_t;
      }
      // and the nonzeros of the whole group of V tiles, which spares k_csr_compact most of its additions
      if (threadIdx.x == 63) grp_nnz[base / tile] = upto;
    }
    __syncthreads();
  }
  }
  };  // run
  if (fast) run(std::true_type{});
  else run(std::false_type{});
  __syncthreads();
  // The counts go to the global histogram with additions that return nothing: the kernel that reads them
  // starts after this one has ended, which is all the ordering the histogram needs.
  for (int a = threadIdx.x; a < 256; a += NT) {
    uint32_t t = 0;
#pragma unroll
    for (int r = 0; r < kHistRep; r++) t += h[a * kHistRep + r];
    if (!t) continue;
    if (a >= (1 << q_bits)) set_status(ctl, RANS_ERR_ARG);  // caller-provided symbol outside {0..2^Q-1}
    else if (!(skip_zero_bin && a == 0)) atomicAdd(&cnt[a], t);
  }
}

}  // namespace
