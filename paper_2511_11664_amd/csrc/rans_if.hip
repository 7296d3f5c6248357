// rans_if.hip -- HIP kernels (gfx950) and the C ABI of include/rans_if.h.
//
// Pipeline (paper Sec. 3.1, Fig. 1(c)):  min/max -> quantise (Eq. 6) + histogram ->
// [modified CSR: count, scan, compact (v, c), row counts r] -> normalise to 2^M ->
// interleaved rANS encode (Eq. 2) -> container.   Decoding runs the inverse
// (Eq. 3-4, cumulative sum of r, scatter, dequantise).
//
// Everything is integer / binary32 work bound by HBM traffic and plain VALU + LDS
// throughput; nothing is a dense contraction, so there is no MFMA code here.
//
// Compile: hipcc -O3 --offload-arch=gfx950 -ffp-contract=off (no fast-math): the
// quantiser's x / s must be the correctly rounded binary32 quotient and no product
// and sum may be fused, or symbols would differ from a CPU evaluation of Eq. 6.

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_ext.h>

#include <cmath>
#include <cstring>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <vector>

#include "rans_if.h"

namespace {

constexpr uint32_t kL = 1u << 16;       // lower bound of the coder state interval [2^16, 2^32)
constexpr int kWG = 256;                // threads per work-group of the streaming kernels
constexpr int kBig = 1024;              // threads of the single-work-group kernels
constexpr uint32_t kHdrBytes = 128;
constexpr uint32_t kLdsHistMaxA = 8192; // alphabets up to this size keep histograms / tables in LDS
constexpr uint64_t kMaxElems = 1ull << 30;
constexpr uint32_t kFusedGatherMax = 16384;  // encoder work-groups up to which the encoder places its words itself
constexpr uint32_t kMaxParts = 1024;    // work-groups (partial results) of the min/max kernel

// ------------------------------------------------------------------ workspace

// Control block at the start of the workspace (device side).
struct Ctl {
  // {status, status_seq} form one 64-bit word: the first data-dependent error of call number
  // status_seq.  An entry of another call number counts as "no error", so nothing has to reset the
  // word when a call starts (and a kernel's work-groups need not wait for such a reset).
  int32_t status;
  uint32_t status_seq;
  uint32_t last_seq;                     // number of the latest call enqueued on this workspace
  uint32_t enc_exact;                    // every entry of the division-free encoder table is exact (see k_normalize)
  float x_min, x_max, scale, zero_point; // Eq. 6
  uint64_t len_d;                        // l_D of Eq. 7
  uint64_t payload_off, dir_off;         // container section offsets
  uint64_t total_bytes;
  uint32_t nnz, n_chunks;
  uint32_t hist_done;                    // work-groups of the histogram kernel that have added their counts
  uint32_t pad[45];
};
static_assert(sizeof(Ctl) == 256, "control block is 256 bytes");

// What kernels receive: the control block and the number of the call they belong to.
struct CtlRef {
  Ctl *p;
  uint32_t seq;
  __host__ __device__ Ctl *operator->() const { return p; }
  __host__ __device__ explicit operator bool() const { return p != nullptr; }
};

struct Layout {
  // common
  size_t ctl;
  // encode side
  size_t mm_part, cnt, fq, enc_tab, enc_tab4, sym, v, c, r, row_end, st, nw, chunk_words, scratch;
  // decode side (overlays the encode side from `sym` on)
  size_t dec_lut, dec_tab, dec_F, D, row_off;
  size_t total;
  uint32_t A, nc_max, capw, n_blk;
  uint32_t cnt_rep;  // partial histograms behind the histogram of D (CSR mode with an LDS-sized alphabet), else 0
  uint32_t n_pub;  // work-groups of the encoder when it also places its words (0: separate gather kernel)
  uint64_t len_max, chunk_len_max;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline uint32_t alphabet_of(const rans_params &p) {
  uint32_t a = 1u << p.q_bits;
  if (p.mode == RANS_MODE_CSR && p.cols + 1 > a) a = (uint32_t)(p.cols + 1);
  return a;
}

inline uint64_t n_chunks_of(uint64_t len, uint32_t cs) {
  if (len == 0) return 0;
  if (cs == 0) return 1;
  return (len + cs - 1) / cs;
}

int check_params(const rans_params *p, uint64_t n) {
  if (!p) return RANS_ERR_ARG;
  if (p->q_bits < 1 || p->q_bits > 8 || p->freq_bits < 1 || p->freq_bits > 15) return RANS_ERR_ARG;
  if (p->mode > RANS_MODE_CSR || p->in_dtype > RANS_F16) return RANS_ERR_ARG;
  if (p->n_streams < 1 || p->n_streams > 65536) return RANS_ERR_ARG;
  if (n > kMaxElems) return RANS_ERR_ARG;
  if (p->cols < 1) return RANS_ERR_SHAPE;
  if (p->rows != n / p->cols || p->rows * p->cols != n) return RANS_ERR_SHAPE;
  if (p->chunk_syms % p->n_streams != 0) return RANS_ERR_SHAPE;
  if (p->mode == RANS_MODE_CSR && p->cols + 1 > 65536) return RANS_ERR_ALPHABET;
  return RANS_OK;
}

constexpr uint32_t kCntRep = 8;  // partial histograms the CSR kernels spread their same-address additions over
constexpr uint32_t kCsrTile = kWG * 16;  // elements per tile in the CSR count / compact kernels
constexpr uint32_t kDenseTileCells = 16384; // symbols per tile of the CSR-to-dense kernel (one row if a row is larger)
constexpr uint32_t kCompactBlocks = 2048;  // work-groups of the compact kernel (persistent over tiles)

Layout make_layout(const rans_params &p, uint64_t n) {
  Layout L{};
  L.A = alphabet_of(p);
  L.len_max = p.mode == RANS_MODE_CSR ? 2 * n + p.rows : n;
  L.nc_max = (uint32_t)n_chunks_of(L.len_max, p.chunk_syms);
  L.chunk_len_max = p.chunk_syms ? p.chunk_syms : L.len_max;
  uint64_t per_stream = (L.chunk_len_max + p.n_streams - 1) / p.n_streams;
  L.capw = (uint32_t)align_up((size_t)per_stream, 8);  // 16-byte blocks
  L.n_blk = (uint32_t)((n + kCsrTile - 1) / kCsrTile);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  L.ctl = take(sizeof(Ctl));
  L.mm_part = take(kMaxParts * 16);
  L.cnt_rep = (p.mode == RANS_MODE_CSR && L.A <= kLdsHistMaxA) ? kCntRep : 0;
  L.cnt = take((size_t)L.A * 4 * (1 + L.cnt_rep));
  L.fq = take((size_t)L.A * 4);
  L.enc_tab = take((size_t)L.A * 8);
  L.enc_tab4 = take((size_t)L.A * 16);
  size_t overlay = o;
  L.sym = take(n);
  if (p.mode == RANS_MODE_CSR) {
    L.v = take(n);
    L.c = take(n * 2);
    L.r = take(p.rows * 2);
    L.row_end = take(p.rows * 4);
  }
  size_t n_sc = (size_t)L.nc_max * p.n_streams;
  L.st = take(n_sc * 4);
  L.nw = take(n_sc * 4);
  {
    const uint64_t wgs = (uint64_t)L.nc_max * ((p.n_streams + kWG - 1) / kWG);
    L.n_pub = (wgs > 0 && wgs <= kFusedGatherMax) ? (uint32_t)wgs : 0;
  }
  if (p.mode != RANS_MODE_CSR) L.n_blk = 0;
  // per-chunk word counts, the encoder's published totals, the nonzeros per CSR tile: all zeroed when a call starts
  L.chunk_words = take(((size_t)L.nc_max + 1 + L.n_pub + L.n_blk) * 4);
  // word blocks of the encoder, per work-group (kWG streams, absent ones included): see k_encode
  L.scratch = take((size_t)L.nc_max * ((p.n_streams + kWG - 1) / kWG) * kWG * L.capw * 2);
  size_t enc_end = o;
  o = overlay;
  L.dec_lut = take(((size_t)2 << p.freq_bits));
  L.dec_tab = take((size_t)L.A * 4);
  L.dec_F = take(((size_t)L.A + 1) * 4);
  if (p.mode == RANS_MODE_CSR) {
    L.D = take(L.len_max * 2);
    L.row_off = take((p.rows + 1) * 4);
  }
  size_t dec_end = o;
  L.total = enc_end > dec_end ? enc_end : dec_end;
  return L;
}

size_t stream_bound(const rans_params &p, const Layout &L) {
  size_t b = kHdrBytes + align_up((size_t)L.A * 2, 8) + 8 * ((size_t)L.nc_max + 1);
  b += (size_t)L.nc_max * (8 * (size_t)p.n_streams + 4) + 2 * (size_t)L.len_max;
  return b;
}

// ------------------------------------------------------------------ device helpers

// Status of the call ctl.seq (0 = no error so far).
__device__ __forceinline__ int get_status(const CtlRef &ctl) {
  const unsigned long long v = *(volatile const unsigned long long *)&ctl.p->status;
  return (uint32_t)(v >> 32) == ctl.seq ? (int)(uint32_t)v : 0;
}
// Records `code` as the error of call ctl.seq unless that call already has one.
__device__ __forceinline__ void set_status(const CtlRef &ctl, int code) {
  unsigned long long *w = (unsigned long long *)&ctl.p->status;
  unsigned long long old = *(volatile unsigned long long *)w;
  for (int tries = 0; tries < 64; tries++) {  // other writers only ever store an error of this call: one retry suffices
    if ((uint32_t)(old >> 32) == ctl.seq && (uint32_t)old != 0) return;
    const unsigned long long want = ((unsigned long long)ctl.seq << 32) | (uint32_t)code;
    const unsigned long long prev = atomicCAS(w, old, want);
    if (prev == old) return;
    old = prev;
  }
}

__device__ __forceinline__ uint32_t f2key(float v) {
  uint32_t b = __float_as_uint(v);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key2f(uint32_t k) {
  uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(b);
}

// Wave-wide inclusive scans with data-parallel-primitive moves (shifts inside rows of 16 lanes, then the
// last lane of a row broadcast into the rows above): six register-to-register steps instead of six trips
// through the LDS crossbar.  A lane without a source receives 0, the identity of + and of the unsigned max.
#define RANS_DPP_STEPS(X, OP)                                                          \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x111, 0xf, 0xf, false)); /* row_shr:1 */ \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x112, 0xf, 0xf, false)); /* row_shr:2 */ \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x114, 0xf, 0xf, false)); /* row_shr:4 */ \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x118, 0xf, 0xf, false)); /* row_shr:8 */ \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x142, 0xa, 0xf, false)); /* row_bcast:15 into rows 1, 3 */ \
  X = OP(X, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)X, 0x143, 0xc, 0xf, false)); /* row_bcast:31 into rows 2, 3 */
__device__ __forceinline__ uint32_t op_add32(uint32_t a, uint32_t b) { return a + b; }
__device__ __forceinline__ uint32_t op_max32(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t wave_incl_sum_scan(uint32_t x) {
  RANS_DPP_STEPS(x, op_add32)
  return x;
}
__device__ __forceinline__ uint32_t wave_incl_max_scan(uint32_t x) {
  RANS_DPP_STEPS(x, op_max32)
  return x;
}
#undef RANS_DPP_STEPS
// the same moves on both halves of a 64-bit value
template <class Op>
__device__ __forceinline__ uint64_t wave_incl_scan64(uint64_t x, Op op) {
  auto mv = [](uint64_t v, auto ctrl, auto rows) -> uint64_t {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, decltype(ctrl)::value, decltype(rows)::value, 0xf, false);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), decltype(ctrl)::value, decltype(rows)::value, 0xf, false);
    return ((uint64_t)hi << 32) | lo;
  };
  using std::integral_constant;
  x = op(x, mv(x, integral_constant<int, 0x111>{}, integral_constant<int, 0xf>{}));
  x = op(x, mv(x, integral_constant<int, 0x112>{}, integral_constant<int, 0xf>{}));
  x = op(x, mv(x, integral_constant<int, 0x114>{}, integral_constant<int, 0xf>{}));
  x = op(x, mv(x, integral_constant<int, 0x118>{}, integral_constant<int, 0xf>{}));
  x = op(x, mv(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xa>{}));
  x = op(x, mv(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xc>{}));
  return x;
}
__device__ __forceinline__ uint64_t lane63_64(uint64_t v) {  // the value lane 63 holds, in every lane
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)v, 63);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), 63);
  return ((uint64_t)hi << 32) | lo;
}

// Work-group barrier that orders LDS accesses only: outstanding global loads and stores stay in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Sum / max over a work-group of NT threads; every thread receives the result.
template <int NT>
__device__ uint64_t block_sum64(uint64_t v, uint64_t *sh /* NT/64 entries */) {
  v = lane63_64(wave_incl_scan64(v, [](uint64_t a, uint64_t b) { return a + b; }));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  uint64_t t = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; w++) t += sh[w];
  return t;
}
template <int NT>
__device__ uint64_t block_max64(uint64_t v, uint64_t *sh) {
  v = lane63_64(wave_incl_scan64(v, [](uint64_t a, uint64_t b) { return a > b ? a : b; }));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  uint64_t t = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; w++) t = sh[w] > t ? sh[w] : t;
  return t;
}

// Exclusive prefix sum over a work-group of NT threads; *total receives the sum.
template <int NT>
__device__ uint32_t block_excl_scan(uint32_t v, uint32_t *sh /* NT/64 entries */, uint32_t *total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_sum_scan(v);
  __syncthreads();
  if (lane == 63) sh[w] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NT / 64; i++) {
    uint32_t s = sh[i];
    if (i < w) base += s;
    tot += s;
  }
  *total = tot;
  return base + inc - v;
}

__device__ __forceinline__ float half_bits_to_float(uint16_t h) {
  return __half2float(__ushort_as_half(h));
}

// Eq. 6 for one element, in binary32: correctly rounded quotient, one addition,
// round half to even, clamp to [0, 2^Q - 1].
__device__ __forceinline__ uint32_t quant1(float x, float s, float zf, float levels) {
  float t = x / s;
  float u = t + zf;
  float r = rintf(u);
  r = fminf(fmaxf(r, 0.0f), levels);
  return (uint32_t)r;
}

// The same with the divisor-only part of the division hoisted out of the loop.
// The correctly rounded binary32 quotient is computed on this target as
//   r1 = refined reciprocal of s;  q0 = x r1;  q1 = q0 + (x - s q0) r1;  q = q1 + (x - s q1) r1
// (fused operations), wrapped in operand scaling and special-case fix-ups that only
// act when an operand is zero / denormal / non-finite or the exponents are far apart.
// With s and every |x| inside [2^-30, 2^30] (or x = 0) none of them acts and the five
// per-element operations below give the same bits; for |x| below that range the
// quotient is far below 1/2 and cannot change the rounded sum with z.
struct FastDiv {
  float s, r1;
  __device__ __forceinline__ void init(float s_) {
    s = s_;
    const float r0 = __builtin_amdgcn_rcpf(s_);
    const float e0 = __builtin_fmaf(-s_, r0, 1.0f);
    r1 = __builtin_fmaf(e0, r0, r0);
  }
  __device__ __forceinline__ float div(float x) const {
    const float q0 = x * r1;
    const float e1 = __builtin_fmaf(-s, q0, x);
    const float q1 = __builtin_fmaf(e1, r1, q0);
    const float e2 = __builtin_fmaf(-s, q1, x);
    return __builtin_fmaf(e2, r1, q1);
  }
};

// Eq. 6: z = round_half_even(-x_min / s), kept as an integer-valued float.  The
// result is built so that a zero is always +0.0: the backend may turn 0 - x into a
// sign flip, which would make z = -0.0 for x_min = +0.0.
__device__ __forceinline__ float eq6_zero_point(float x_min, float s) {
  if (!(s != 0.0f)) return 0.0f;
  float zf = rintf((0.0f - x_min) / s);
  uint32_t b = __float_as_uint(zf);
  return __uint_as_float(b == 0x80000000u ? 0u : b);
}

// ------------------------------------------------------------------ kernels: set-up

// ------------------------------------------------------------------ kernels: Eq. 6

// Start-of-call bookkeeping (done by one work-group of the first kernel of a call): reset the control
// block, clear the histogram and the encoder's per-chunk / per-work-group word counters.
__device__ void reset_call_state(const CtlRef &ctl, uint32_t *cnt, uint32_t A, uint32_t *chunk_words, uint32_t nc) {
  if (threadIdx.x == 0) {
    ctl->last_seq = ctl.seq;
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
};
// Count of symbol a: the histogram's entry plus those of the partial histograms behind it.
__device__ __forceinline__ uint32_t hist_count(const NormArgs &na, uint32_t a) {
  if (na.lds_cnt) return na.lds_cnt[a];
  uint32_t c = __hip_atomic_load(na.cnt + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (uint32_t k = 1; k <= na.n_rep; k++)
    c += __hip_atomic_load(na.cnt + (size_t)k * na.A + a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return c;
}
// Container header (fixed part) and the geometry the later kernels read from the control block.
__device__ void write_header(const CtlRef &ctl, const NormArgs &na, uint64_t len_d, uint64_t n_chunks, uint64_t dir_off,
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

// Everything stored per symbol: f in the container, the encoder's two table entries.  m_floor is
// floor(2^32 / f) (any value for f <= 1), div(two) returns floor(two / f) for two = 2^(32+k).  Returns
// whether the division-free entry is inexact.
//
// Division-free entry {lim1, mx, Fx | sh << 16, 2^M - f}: the coder renormalises when s > lim1 and
// then takes q = mulhi(s, mx) >> sh for floor(s / f) in Eq. 2.  At that point s <= lim1 =
// f * 2^(32-M) - 1.  With 2^k <= f < 2^(k+1), mx = floor(2^(32+k) / f) + 1 and e = mx * f - 2^(32+k),
// q is exact for every s with s * e < 2^(32+k); the entry is marked inexact otherwise (possible only
// for f > 2^(M-1)).  Powers of two take mx = 2^31, sh = k - 1.  f = 1 cannot have its multiplier
// 2^32: it takes mx = 2^32 - 1, which gives q = s - 1 (s >= 1 there), and the missing 2^M - f is
// added to Fx instead.  f = 0 (absent symbol) is never looked up.
template <class Div>
__device__ __forceinline__ int emit_entries(const NormArgs &na, uint32_t a, uint32_t f, uint32_t F, uint32_t m_floor,
                                            Div div) {
  const uint32_t M = na.p.freq_bits, total = 1u << M;
  int inexact = 0;
  // floor(2^32 / f) for f >= 2, 2^32 - 1 for f = 1: with it mulhi(s, m) is floor(s / f) or one less
  const uint32_t m = f <= 1 ? 0xffffffffu : m_floor;
  na.enc_tab[a] = make_uint2(m, f | (F << 16));
  *(uint16_t *)(na.out + kHdrBytes + 2ull * a) = (uint16_t)f;
  const uint32_t cmpl = total - f;
  uint32_t lim1 = (f << (32 - M)) - 1u, mx = 0, sh = 0, Fx = F;
  if (f == 1) {
    mx = 0xffffffffu;
    Fx = F + cmpl;
  } else if (f > 1) {
    const uint32_t k = 31u - (uint32_t)__clz((int)f);
    if ((f & (f - 1)) == 0) {
      mx = 0x80000000u;
      sh = k - 1;
    } else {
      const uint64_t two = 1ull << (32 + k);
      const uint64_t mq = div(two) + 1;  // < 2^32 because f > 2^k
      const uint64_t e = mq * f - two;
      if ((uint64_t)lim1 * e >= two) inexact = 1;
      mx = (uint32_t)mq;
      sh = k;
    }
  }
  na.enc_tab4[a] = make_uint4(lim1, mx, Fx | (sh << 16), cmpl);
  return inexact;
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
  if (get_status(ctl) != 0) return;  // uniform: written by an earlier kernel
  uint64_t len_loc = 0, present_loc = 0;
  for (uint32_t a = threadIdx.x; a < A; a += kBig) {
    uint32_t c = hist_count(na, a);
    len_loc += c;
    present_loc += c != 0;
  }
  const uint64_t len = block_sum64<kBig>(len_loc, sh64);
  const uint64_t present = block_sum64<kBig>(present_loc, sh64);
  if (dense) {
    if (threadIdx.x == 0) ctl->len_d = len;
  }
  const uint64_t len_d = dense ? len : ctl->len_d;
  if (present > total || len != len_d) {  // the second cannot happen; kept as a guard
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_ALPHABET);
    return;
  }
  // first estimate and its sum
  uint64_t sum_loc = 0, best_cnt = 0;
  for (uint32_t a = threadIdx.x; a < A; a += kBig) {
    uint32_t c = hist_count(na, a);
    uint32_t f = 0;
    if (c) {
      uint64_t q = ((uint64_t)c * total + len / 2) / len;
      f = q < 1 ? 1u : (uint32_t)q;
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
      inexact |= emit_entries(na, a, f, F, (uint32_t)(0x100000000ull / (f ? f : 1)), [&](uint64_t two) { return two / f; });
    }
    carry += tot;
    __syncthreads();
  }
  inexact = __syncthreads_or(inexact);
  if (threadIdx.x == 0) ctl->enc_exact = inexact ? 0u : 1u;
  for (uint64_t o = table_off + 2ull * A + 2 * threadIdx.x; o < dir_off; o += 2 * kBig) *(uint16_t *)(out + o) = 0;
}

// floor(a / b) for 0 <= a < 2^52, 1 <= b < 2^32 through one binary64 division instead of the much
// longer 64-bit integer division.  Both operands are exact in binary64.  If b divides a the division is
// exact.  Otherwise a / b lies at least 1 / b away from the integers next to it, and the correctly
// rounded quotient differs from a / b by at most (a / b) * 2^-53 < 1 / b (because a < 2^53), so it
// stays strictly between the same two integers and its floor is the floor of a / b.
__device__ __forceinline__ uint64_t floor_div_f64(uint64_t a, uint32_t b) {
  return (uint64_t)((double)a / (double)b);
}

// The same as normalize_body for alphabets of up to 64 PER symbols, by ONE wave without a barrier: lane l
// owns the symbols PER l .. PER l + PER - 1, sums and maxima are wave scans.  Called by the first wave of a
// work-group; the single work-group version spends most of its time in barriers between 16 waves.
constexpr uint32_t kNormWaveA = 512;
template <int PER>
__device__ void normalize_wave_per(const CtlRef &ctl, const NormArgs &na) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t A = na.A;
  const rans_params &p = na.p;
  const uint32_t M = p.freq_bits, total = 1u << M;
  if (get_status(ctl) != 0) return;  // uniform: written by an earlier kernel
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
  if (na.dense && lane == 0) ctl->len_d = len;
  // CSR mode: len_d was stored with a device-scope atomic by a work-group of the kernel this may run in
  const uint64_t len_d = na.dense ? len : __hip_atomic_load(&ctl->len_d, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (present > total || len != len_d) {  // the second cannot happen; kept as a guard
    if (lane == 0) set_status(ctl, RANS_ERR_ALPHABET);
    return;
  }
  // first estimate, its sum, the symbol with the largest count
  uint32_t f[PER];
  uint64_t sum = 0, best = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) {
    f[q] = 0;
    if (c[q]) {
      const uint64_t e = floor_div_f64((uint64_t)c[q] * total + len / 2, (uint32_t)len);  // < 2^46 over < 2^32
      f[q] = e < 1 ? 1u : (uint32_t)e;
      const uint64_t key = ((uint64_t)c[q] << 32) | (0xffffffffu - (PER * lane + q));  // max count, lowest index
      best = key > best ? key : best;
    }
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
  const uint64_t n_chunks = len_d == 0 ? 0 : (p.chunk_syms == 0 ? 1 : (len_d + p.chunk_syms - 1) / p.chunk_syms);
  const uint64_t table_off = kHdrBytes;
  const uint64_t dir_off = table_off + (((uint64_t)A * 2 + 7) & ~7ull);
  const uint64_t payload_off = dir_off + 8 * (n_chunks + 1);
  if (payload_off > na.cap) {
    if (lane == 0) set_status(ctl, RANS_ERR_CAPACITY);
    return;
  }
  if (lane == 0) write_header(ctl, na, len_d, n_chunks, dir_off, payload_off);
  // cumulative sum, encoder tables, stored table
  uint32_t mine = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) mine += f[q];
  uint32_t F = wave_incl_sum_scan(mine) - mine;
  int inexact = 0;
#pragma unroll
  for (int q = 0; q < PER; q++) {
    const uint32_t a = PER * lane + q;
    if (a < A) {
      const uint32_t fa = f[q];
      inexact |= emit_entries(na, a, fa, F, (uint32_t)floor_div_f64(0x100000000ull, fa ? fa : 1),
                              [&](uint64_t two) { return floor_div_f64(two, fa); });  // two <= 2^46, fa < 2^16
    }
    F += f[q];
  }
  const bool any_inexact = __ballot(inexact) != 0;
  if (lane == 0) ctl->enc_exact = any_inexact ? 0u : 1u;
  for (uint64_t o = table_off + 2ull * A + 2 * lane; o < dir_off; o += 2 * 64) *(uint16_t *)(na.out + o) = 0;
}

__device__ void normalize_wave(const CtlRef &ctl, const NormArgs &na) {
  if (na.A <= 256) normalize_wave_per<4>(ctl, na);
  else normalize_wave_per<8>(ctl, na);
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

template <typename T, bool VEC, int NT, bool CSR>
__global__ __launch_bounds__(NT) void k_quant_hist(const T *x, uint32_t n, CtlRef ctl, uint32_t q_bits,
                                                    uint8_t *sym, uint32_t *cnt, int skip_zero_bin,
                                                    const MinMaxPart *part, uint32_t n_part, rans_qinfo *qout,
                                                    int fold_norm, NormArgs na, uint32_t *blk_nnz) {
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
    if (threadIdx.x < V) {
      const uint64_t t_idx = base / kCsrTile + threadIdx.x;
      const uint32_t c_t = s_nz[threadIdx.x];
      s_nz[threadIdx.x] = 0;
      if (t_idx * kCsrTile < n) blk_nnz[t_idx] = c_t;
    }
    __syncthreads();
  }
  }
  };  // run
  if (fast) run(std::true_type{});
  else run(std::false_type{});
  __syncthreads();
  uint32_t seen = 0;
  for (int a = threadIdx.x; a < 256; a += NT) {
    uint32_t t = 0;
#pragma unroll
    for (int r = 0; r < kHistRep; r++) t += h[a * kHistRep + r];
    if (!t) continue;
    if (a >= (1 << q_bits)) set_status(ctl, RANS_ERR_ARG);  // caller-provided symbol outside {0..2^Q-1}
    else if (!(skip_zero_bin && a == 0)) {
      // with the table build folded in, the additions return their old value: a returned value is the only
      // proof that an addition has been performed before the work-group takes its ticket (one without a
      // result is acknowledged earlier than that)
      if (fold_norm) seen |= atomicAdd(&cnt[a], t);
      else atomicAdd(&cnt[a], t);
    }
  }
  if (!fold_norm) return;
  if (seen == 0xffffffffu) set_status(ctl, RANS_ERR_HIP);  // cannot happen (counts are below 2^31); keeps the values in use
  // The work-group that adds its counts last also builds the frequency table (saves a launch).  The
  // additions above are device-scope atomics that return a value; the barrier waits for the values, so
  // this work-group's additions have been performed when it takes its ticket.  The last one reads the
  // histogram with device-scope atomic loads, so no cache has to be written back or invalidated in between.
  __shared__ uint32_t s_ticket;
  __syncthreads();
  if (threadIdx.x == 0) s_ticket = __hip_atomic_fetch_add(&ctl->hist_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_ticket != gridDim.x - 1) return;
  if (part) {  // every work-group has computed the extrema itself
    na.mm_given = 1;
    na.x_min = qi.x_min;
    na.x_max = qi.x_max;
  }
  if (na.A <= kNormWaveA) {
    if (threadIdx.x < 64) normalize_wave(ctl, na);
  } else if constexpr (NT == kBig) {
    normalize_body(ctl, na);
  }
}

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

// In-place exclusive scan of a u32 array by one work-group; the total goes to a[n].
__global__ __launch_bounds__(kBig) void k_scan_u32(uint32_t *a, uint32_t n) {
  __shared__ uint32_t sh[kBig / 64];
  uint32_t carry = 0;
  for (uint32_t base = 0; base < n; base += kBig) {
    uint32_t i = base + threadIdx.x;
    uint32_t v = i < n ? a[i] : 0, tot;
    uint32_t ex = block_excl_scan<kBig>(v, sh, &tot);
    if (i < n) a[i] = carry + ex;
    carry += tot;
    __syncthreads();
  }
  if (threadIdx.x == 0) a[n] = carry;
}

// Stream compaction of the nonzero symbols in flat (= row-major) order: v gets the
// values, c the column indices, row_end[i] the number of nonzeros up to and
// including row i.  Column indices are histogrammed into cnt on the way.
// A work-group walks tiles blockIdx.x, blockIdx.x + gridDim.x, ...: a tile's nonzeros are
// compacted in LDS first and leave with consecutive lanes on consecutive entries, and the
// column histogram is added to the global one once at the end (few work-groups: same-address
// global atomics are what costs here).  blk_nnz[t] is the number of nonzeros of tile t (counted by
// k_quant_hist); a tile's place in v and c is the sum over the tiles before it, which the work-group
// adds up itself.
template <bool LDS_HIST>
__global__ __launch_bounds__(kWG) void k_csr_compact(const uint8_t *sym, uint32_t n, int aligned, uint32_t K,
                                                     const uint32_t *blk_nnz, uint8_t *v, uint16_t *c,
                                                     uint32_t *row_end, uint32_t *cnt, uint32_t A, uint32_t n_tiles,
                                                     uint32_t n_rep) {
  extern __shared__ uint32_t hist[];
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint64_t sh64[kWG / 64];
  __shared__ uint8_t s_v[kCsrTile];
  __shared__ uint16_t s_c[kCsrTile];
  if (LDS_HIST) {
    for (uint32_t a = threadIdx.x; a < A; a += kWG) hist[a] = 0;
  }
  // where the work-group's tile starts in v and c: the nonzeros of all tiles before it (k_quant_hist has
  // counted them), kept up to date from tile to tile with the counts of the tiles in between
  uint32_t base;
  {
    uint64_t part = 0;
    for (uint32_t u0 = threadIdx.x; u0 < blockIdx.x; u0 += 4 * kWG) {
      uint32_t x4[4];
#pragma unroll
      for (int k = 0; k < 4; k++) x4[k] = u0 + k * kWG < blockIdx.x ? blk_nnz[u0 + k * kWG] : 0u;
#pragma unroll
      for (int k = 0; k < 4; k++) part += x4[k];
    }
    base = (uint32_t)block_sum64<kWG>(part, sh64);
  }
  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const uint64_t e0 = (uint64_t)tile * kCsrTile + threadIdx.x * 16;
    uint8_t b[16];
    load16(sym, e0, n, aligned, b);
    uint32_t cth = 0;
#pragma unroll
    for (int k = 0; k < 16; k++) cth += b[k] != 0;
    uint32_t tot;
    uint32_t loc = block_excl_scan<kWG>(cth, sh, &tot);  // also orders the hist zeroing and the staging reuse
    if (e0 < n) {
      uint32_t row = (uint32_t)(e0 / K), col = (uint32_t)(e0 - (uint64_t)row * K);
#pragma unroll
      for (int k = 0; k < 16; k++) {
        if (e0 + k < n) {
          if (b[k]) {
            s_v[loc] = b[k];
            s_c[loc] = (uint16_t)col;
            loc++;
            if (LDS_HIST) atomicAdd(&hist[col], 1u);
            else atomicAdd(&cnt[col], 1u);
          }
          if (++col == K) {
            row_end[row] = base + loc;
            col = 0;
            row++;
          }
        }
      }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < tot; i += kWG) {
      v[base + i] = s_v[i];
      c[base + i] = s_c[i];
    }
    if (tile + gridDim.x < n_tiles) {  // uniform
      uint64_t skip = 0;
      for (uint32_t u0 = tile + threadIdx.x; u0 < tile + gridDim.x; u0 += 4 * kWG) {
        uint32_t x4[4];
#pragma unroll
        for (int k = 0; k < 4; k++) x4[k] = u0 + k * kWG < tile + gridDim.x ? blk_nnz[u0 + k * kWG] : 0u;
#pragma unroll
        for (int k = 0; k < 4; k++) skip += x4[k];
      }
      base += (uint32_t)block_sum64<kWG>(skip, sh64);
    }
    __syncthreads();  // staging and scan scratch are reused by the next tile
  }
  if (LDS_HIST) {
    // into one of the partial histograms: a thousand work-groups adding to the same few hundred addresses
    // would keep the kernel busy long after its last tile
    uint32_t *dst = cnt + (n_rep ? (size_t)(1 + blockIdx.x % n_rep) * A : 0);
    for (uint32_t a = threadIdx.x; a < A; a += kWG) {
      uint32_t t = hist[a];
      if (t) atomicAdd(&dst[a], t);
    }
  }
}

// r[i] = row_end[i] - row_end[i-1] (the NON-cumulative row count), histogrammed.  Work-groups stride
// over the rows and add their histogram to the global one once.
template <bool LDS_HIST>
__global__ __launch_bounds__(kWG) void k_csr_rows(const uint32_t *row_end, uint32_t N, uint16_t *r, uint32_t *cnt,
                                                  uint32_t A, CtlRef ctl, int fold_norm, NormArgs na) {
  extern __shared__ uint32_t hist[];
  if (LDS_HIST) {
    for (uint32_t a = threadIdx.x; a < A; a += kWG) hist[a] = 0;
    __syncthreads();
  }
  uint32_t seen = 0;
  for (uint32_t i = blockIdx.x * kWG + threadIdx.x; i < N; i += gridDim.x * kWG) {
    uint32_t e1 = row_end[i], e0 = i ? row_end[i - 1] : 0;
    uint32_t ri = e1 - e0;
    r[i] = (uint16_t)ri;
    if (LDS_HIST) atomicAdd(&hist[ri], 1u);
    else atomicAdd(&cnt[ri], 1u);
    if (i == N - 1) {
      ctl->nnz = e1;
      // an exchange, for its returned value (see below): l_D has to be in place before this work-group's ticket
      seen |= (uint32_t)__hip_atomic_exchange(&ctl->len_d, 2ull * e1 + N, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  const bool hand_over = fold_norm || na.n_rep;  // the last work-group reads what the others added
  if (LDS_HIST) {
    __syncthreads();
    uint32_t *dst = cnt + (na.n_rep ? (size_t)(1 + blockIdx.x % na.n_rep) * A : 0);
    for (uint32_t a = threadIdx.x; a < A; a += kWG) {
      uint32_t t = hist[a];
      // before a hand-over the additions return their old value: a returned value is the only proof that an
      // addition has been performed before the work-group takes its ticket
      if (t) {
        if (hand_over) seen |= atomicAdd(&dst[a], t);
        else atomicAdd(&dst[a], t);
      }
    }
  }
  if (!hand_over) return;
  if (seen == 0xffffffffu) set_status(ctl, RANS_ERR_HIP);  // cannot happen (counts are below 2^31); keeps the values in use
  // D's histogram is complete once every work-group has added its row counts: the last one to do so folds
  // the partial histograms and, if asked to, builds the frequency table (the same hand-over as at the end of
  // k_quant_hist).  It also reads len_d, which the work-group holding the last row exchanged in before the
  // barrier ahead of its ticket.
  __shared__ uint32_t s_ticket;
  __shared__ uint32_t s_cnt[kNormWaveA];
  __syncthreads();
  if (threadIdx.x == 0) s_ticket = __hip_atomic_fetch_add(&ctl->hist_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_ticket != gridDim.x - 1) return;
  if (na.n_rep) {  // all loads of a lane in flight together
    for (uint32_t a0 = threadIdx.x; a0 < A; a0 += kWG) {
      uint32_t part_c[kCntRep + 1];
#pragma unroll
      for (uint32_t k = 0; k <= kCntRep; k++)
        part_c[k] = k <= na.n_rep ? __hip_atomic_load(cnt + (size_t)k * A + a0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
      uint32_t sum = 0;
#pragma unroll
      for (uint32_t k = 0; k <= kCntRep; k++) sum += part_c[k];
      if (!fold_norm) cnt[a0] = sum;  // for k_normalize
      if (a0 < kNormWaveA) s_cnt[a0] = sum;
    }
    lds_barrier();
    na.n_rep = 0;
    if (A <= kNormWaveA) na.lds_cnt = s_cnt;
  }
  if (fold_norm && threadIdx.x < 64) normalize_wave(ctl, na);
}

// ------------------------------------------------------------------ kernels: rANS encode

// Symbol sources for the coder.  fetch<SPL>(i) returns the SPL consecutive symbols
// D[i..i+SPL) packed into one register, get(raw, q) unpacks symbol q.
struct SrcDense {
  const uint8_t *sym;
  static constexpr int kMaxSpl = 4;
  __device__ __forceinline__ void init(const CtlRef &) {}
  __device__ __forceinline__ const uint8_t *bytes() const { return sym; }  // D as a plain byte array
  // the parts of a CSR source (not meaningful here; they keep the coder's code generic)
  __device__ __forceinline__ uint64_t nnz_of() const { return 0; }
  __device__ __forceinline__ const uint8_t *v_ptr() const { return nullptr; }
  __device__ __forceinline__ const uint16_t *c_ptr() const { return nullptr; }
  __device__ __forceinline__ const uint16_t *r_ptr() const { return nullptr; }
  __device__ __forceinline__ uint32_t operator()(uint64_t i) const { return sym[i]; }
  template <int SPL>
  __device__ __forceinline__ uint32_t fetch(uint64_t i) const {
    if constexpr (SPL == 4) return *(const uint32_t *)(sym + i);
    else if constexpr (SPL == 2) return *(const uint16_t *)(sym + i);
    else return sym[i];
  }
  __device__ __forceinline__ static uint32_t get(uint32_t raw, int q) { return (raw >> (8 * q)) & 0xffu; }
};
// D = v (+) c (+) r (Eq. 7) without materialising the concatenation.
struct SrcCsr {
  const uint8_t *v;
  const uint16_t *c, *r;
  uint64_t nnz;
  static constexpr int kMaxSpl = 2;
  __device__ __forceinline__ void init(const CtlRef &ctl) { nnz = ctl->nnz; }
  __device__ __forceinline__ const uint8_t *bytes() const { return nullptr; }  // D is not one byte array
  __device__ __forceinline__ uint64_t nnz_of() const { return nnz; }
  __device__ __forceinline__ const uint8_t *v_ptr() const { return v; }
  __device__ __forceinline__ const uint16_t *c_ptr() const { return c; }
  __device__ __forceinline__ const uint16_t *r_ptr() const { return r; }
  __device__ __forceinline__ uint32_t operator()(uint64_t i) const {
    if (i < nnz) return v[i];
    if (i < 2 * nnz) return c[i - nnz];
    return r[i - 2 * nnz];
  }
  template <int SPL>
  __device__ __forceinline__ uint32_t fetch(uint64_t i) const {
    uint32_t raw = (*this)(i);
    if constexpr (SPL == 2) raw |= (*this)(i + 1) << 16;
    return raw;
  }
  __device__ __forceinline__ static uint32_t get(uint32_t raw, int q) { return (raw >> (16 * q)) & 0xffffu; }
};

constexpr int kStageRows = 32;         // rows per tile of the encoder's symbol staging (dense source)
constexpr int kStageRows2 = 16;        // the same for the CSR source (16-bit entries)
constexpr uint32_t kRingStride = 40;  // bytes between the word rings of adjacent streams: 16 slots + padding against bank conflicts
constexpr uint32_t kEncTab16MaxA = 1024;  // CSR alphabets up to this size use the 16-byte table entries
constexpr int kEncAhead = 8;  // rows of symbols fetched ahead of the coder; also the flush period of the word ring

// Encoder table entry as the coder uses it.
struct EncEntry {
  uint32_t m, f, F, cmpl;  // floor(2^32/f) (2^32-1 for f = 1), f, F, 2^M - f
};

// Table modes: 0 = {m, f | F << 16} read from global memory (very large alphabets),
// 1 = the same staged in LDS, 2 = 16-byte entries staged in LDS (small alphabets: one LDS read, no
// unpacking arithmetic): the division-free form {lim1, mx, Fx | sh << 16, 2^M - f} when every entry of it
// is exact, else {m, f, F, 2^M - f}.
template <int TAB>
__device__ __forceinline__ EncEntry load_entry(const uint2 *g_tab, const uint32_t *l_tab, uint32_t x, uint32_t totalM) {
  EncEntry e;
  if constexpr (TAB == 2) {
    uint4 q = ((const uint4 *)l_tab)[x];
    e.m = q.x; e.f = q.y; e.F = q.z; e.cmpl = q.w;
  } else {
    uint2 q = TAB == 1 ? ((const uint2 *)l_tab)[x] : g_tab[x];
    e.m = q.x; e.f = q.y & 0xffffu; e.F = q.y >> 16; e.cmpl = totalM - e.f;
  }
  return e;
}

// Interleaved rANS encoder (Eq. 2 with 16-bit renormalisation).  One work-group codes kWG * SPL
// streams of one chunk (only SPL = 1 is instantiated: the hardware interleaves waves better than the
// compiler interleaves several streams inside a lane).
//
// Symbols are taken last to first in batches of kEncAhead rows, fetched a batch ahead (dense source:
// through a per-wave LDS stage filled with 16-byte loads a whole tile ahead), table entries looked up
// three rows ahead.  The per-row arithmetic is branch-free (selects only) so that it stays one basic
// block.  floor(s / f) of Eq. 2 is a multiply-high and a shift with the per-symbol multiplier that
// k_normalize proved exact (table form 2, when every entry is exact), else a multiply-high with
// floor(2^32 / f) plus one correction step.
//
// Emitted words wait in a 16-slot LDS area per stream, filled from the top: the low half of the state
// is written to the next slot on every step and the slot pointer moves only when the renormalisation
// fires, so a slot keeps being rewritten until it is really used.  After every kEncAhead rows (a
// wave-uniform point) a stream with 8 or more waiting words moves its 8 oldest as one 16-byte block to
// scratch in global memory (block-major per work-group: lanes that flush the same block number write
// adjacent memory); inside a block ascending address = descending word number, the decoder's order.
//
// FUSE: the work-group also moves its streams' words to their place in the container (what k_gather
// does otherwise).  It publishes its word total, waits until every work-group with a lower index has
// published its own (those were dispatched earlier and never wait for a higher index, so the wait ends;
// it is bounded all the same and turns into RANS_ERR_HIP if the bound is hit), and derives the chunk's
// byte offset and its own position inside the chunk from those totals.
constexpr int kSpinMax = 1 << 18;
constexpr uint32_t kEncTileBytes = 16384;  // LDS tile of the fused placement (overlays ring and table)
__device__ __forceinline__ uint32_t wait_published(const uint32_t *pub, uint32_t i, const CtlRef &ctl) {
  for (int spins = 0; spins < kSpinMax; spins++) {
    const uint32_t v = __hip_atomic_load(pub + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v) return v;
    if ((spins & 255) == 255 && get_status(ctl) != 0) return 0;
    __builtin_amdgcn_s_sleep(4);
  }
  return 0;
}

template <class Src, int SPL, int TAB, bool MUL24, bool FUSE>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(4))) void k_encode(Src src, const uint2 *g_tab, const uint4 *g_tab4, uint32_t A, uint32_t M,
                                                uint32_t S,
                                                uint32_t cs, CtlRef ctl, uint16_t *scratch, uint32_t capw,
                                                uint32_t *st_out, uint32_t *nw_out, uint32_t *chunk_words,
                                                uint32_t groups, uint32_t *wg_pub, uint8_t *out, uint64_t cap,
                                                uint64_t *d_stream_bytes, int wide) {
  extern __shared__ __align__(16) uint32_t l_mem[];  // the only LDS of this kernel, so the ring starts at offset 0
  // every exit publishes a total (0 words), or the work-groups behind this one would wait for it
  auto bail = [&]() {
    if (FUSE && threadIdx.x == 0) __hip_atomic_store(wg_pub + blockIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  };
  if (get_status(ctl) != 0) {
    if (FUSE && blockIdx.x == 0 && threadIdx.x == 0 && d_stream_bytes) *d_stream_bytes = 0;
    bail();
    return;
  }
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  const uint32_t nc = ctl->n_chunks;
  if (k >= nc) {
    if (FUSE && nc == 0 && blockIdx.x == 0 && threadIdx.x == 0) {  // empty D: only the directory's single entry
      uint8_t *dir0 = out + ctl->dir_off;
      st32(dir0, 0u);
      st32(dir0 + 4, 0u);
      ctl->total_bytes = ctl->payload_off;
      if (d_stream_bytes) *d_stream_bytes = ctl->payload_off;
    }
    bail();
    return;
  }
  src.init(ctl);
  const uint32_t sh_lim = 32 - M, totalM = 1u << M;
  // LDS: [ring][table].  The ring comes first (LDS address 0) so that a slot address is the lane's
  // fixed base plus twice the slot number.
  constexpr uint32_t G = kWG * SPL;  // streams per work-group
  constexpr uint32_t kRingBytes = kRingStride * G;
  uint32_t *l_tab = l_mem + kRingBytes / 4;
  uint32_t *sh = l_tab + (TAB == 2 ? A * 4 : (TAB == 1 ? A * 2 : 0));  // 4 + 8 words for the final reductions
  // TAB == 2 has two forms of the table: the division-free one when every entry of it is exact for
  // this frequency table (the common case), else {floor(2^32/f), f, F, 2^M - f} with a correction step.
  const bool exact = TAB == 2 && ctl->enc_exact != 0;
  if (TAB == 1) {
    for (uint32_t a = threadIdx.x; a < A; a += kWG) ((uint2 *)l_tab)[a] = g_tab[a];
  } else if (TAB == 2) {
    if (exact) {
      for (uint32_t a = threadIdx.x; a < A; a += kWG) ((uint4 *)l_tab)[a] = g_tab4[a];
    } else {
      for (uint32_t a = threadIdx.x; a < A; a += kWG) {
        uint2 q = g_tab[a];
        ((uint4 *)l_tab)[a] = make_uint4(q.x, q.y & 0xffffu, q.y >> 16, totalM - (q.y & 0xffffu));
      }
    }
  }
  if (TAB != 0) __syncthreads();
  const uint64_t len = ctl->len_d;
  const uint64_t chunk_len = cs ? cs : len;
  const uint64_t base = (uint64_t)k * chunk_len;
  const uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
  const uint32_t j0 = (g * kWG + threadIdx.x) * SPL;
  const bool live = j0 < S;  // S is a multiple of SPL: a lane's streams are all live or all absent
  // Emitted words wait in a 16-slot LDS area per stream, filled from its top slot downwards: `wp` is the
  // LDS address of the slot of the next word.  Once 8 or more words wait, the 8 oldest (the upper half:
  // ascending address = descending word number, the order the decoder reads) leave as one 16-byte block
  // and the lower half moves up.
  uint32_t s[SPL], wp[SPL];
  // Scratch holds the work-group's 16-byte blocks block-major: block b of the stream in column c at
  // ((b * G + c) * 8) words from the work-group's base, so that the lanes of a wave that flush the
  // same block number write adjacent memory.
  uint16_t *gp[SPL];    // where the stream's next 16-byte block goes
  uint32_t colb[SPL];   // LDS address of the stream's area; areas are kRingStride bytes apart (conflict-free)
#pragma unroll
  for (int i = 0; i < SPL; i++) {
    s[i] = kL;
    gp[i] = scratch + (uint64_t)blockIdx.x * (kWG * SPL) * capw + (i * kWG + threadIdx.x) * 8;
    colb[i] = kRingStride * (i * kWG + threadIdx.x);
    wp[i] = colb[i] + 30;
  }
  // the areas start at LDS address 0, so that `wp` is a plain LDS address
  typedef __attribute__((address_space(3))) uint16_t lds_u16;
  typedef __attribute__((address_space(3))) uint64_t lds_u64;
  if ((uint32_t)(uintptr_t)(lds_u16 *)l_mem != 0) {  // cannot happen without static LDS; the slot arithmetic relies on it
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_HIP);
    bail();
    return;
  }
  auto flush = [&](int i) {
    if (wp[i] < colb[i] + 16) {  // 8 or more words wait
      lds_u64 *r = (lds_u64 *)(uintptr_t)colb[i];
      const uint64_t lo0 = r[0], lo1 = r[1], hi0 = r[2], hi1 = r[3];
      *(uint4 *)gp[i] = make_uint4((uint32_t)hi0, (uint32_t)(hi0 >> 32), (uint32_t)hi1, (uint32_t)(hi1 >> 32));
      gp[i] += kWG * SPL * 8;
      r[2] = lo0;
      r[3] = lo1;
      wp[i] += 16;
    }
  };
  // The coding loop, for one of the two table forms (an entry is {m, f, F, cmpl} with the meaning of
  // that form: EXACT {mx, lim1, Fx | sh << 16, 2^M - f}, else {floor(2^32/f), f, F, 2^M - f}).
  auto run = [&](auto exact_tag, auto wide_tag) {
    constexpr bool EXACT = decltype(exact_tag)::value;
    constexpr int WIDE_KIND = decltype(wide_tag)::value;  // 0: direct loads, 1: dense bytes through LDS, 2: CSR segments through LDS
    constexpr bool WIDE = WIDE_KIND == 1;
    // Eq. 2 for the lane's SPL streams, phase by phase across the streams so that the
    // independent chains interleave; selects only, no branches.
    auto row = [&](const EncEntry (&e)[SPL]) {
      bool c[SPL];
      uint32_t q[SPL];
#pragma unroll
      for (int i = 0; i < SPL; i++)  // too large for this symbol: emit 16 bits
        c[i] = EXACT ? s[i] > e[i].f : (s[i] >> sh_lim) >= e[i].f;
#pragma unroll
      for (int i = 0; i < SPL; i++) *(lds_u16 *)(uintptr_t)wp[i] = (uint16_t)s[i];  // speculative: the slot counts only if c
#pragma unroll
      for (int i = 0; i < SPL; i++) {
        s[i] = c[i] ? s[i] >> 16 : s[i];
        wp[i] = c[i] ? wp[i] - 2 : wp[i];
      }
#pragma unroll
      for (int i = 0; i < SPL; i++) q[i] = __umulhi(s[i], e[i].m);
      if constexpr (EXACT) {
#pragma unroll
        for (int i = 0; i < SPL; i++) q[i] >>= e[i].F >> 16;
#pragma unroll
        for (int i = 0; i < SPL; i++)
          s[i] = (MUL24 ? __umul24(q[i], e[i].cmpl) + s[i] : q[i] * e[i].cmpl + s[i]) + (e[i].F & 0xffffu);
      } else {
        uint32_t rem[SPL];
#pragma unroll
        for (int i = 0; i < SPL; i++) rem[i] = s[i] - (MUL24 ? __umul24(q[i], e[i].f) : q[i] * e[i].f);
#pragma unroll
        for (int i = 0; i < SPL; i++) q[i] += rem[i] >= e[i].f ? 1u : 0u;
#pragma unroll
        for (int i = 0; i < SPL; i++) s[i] = s[i] + e[i].F + (MUL24 ? __umul24(q[i], e[i].cmpl) : q[i] * e[i].cmpl);
      }
    };
    auto entry = [&](uint32_t x) -> EncEntry {
      if constexpr (EXACT) {
        const uint4 q = ((const uint4 *)l_tab)[x];
        return EncEntry{q.y, q.x, q.z, q.w};
      } else {
        return load_entry<TAB>(g_tab, l_tab, x, totalM);
      }
    };
    auto lookup = [&](EncEntry (&e)[SPL], uint32_t raw) {
#pragma unroll
      for (int i = 0; i < SPL; i++) e[i] = entry(Src::get(raw, i));
    };
    const uint64_t rows_full = n_here / S;
    const uint32_t rem_row = (uint32_t)(n_here - rows_full * S);
    EncEntry ea[SPL];
    if (rem_row) {  // ragged last row: only streams j < rem_row have a symbol there
#pragma unroll
      for (int i = 0; i < SPL; i++) {
        // an absent stream gets a neutral entry, which leaves the state untouched
        ea[i] = EXACT ? EncEntry{0u, 0xffffffffu, 0u, 0u} : EncEntry{0u, totalM, 0u, 0u};
        if (j0 + i < rem_row) ea[i] = entry(src(base + rows_full * S + j0 + i));
      }
      row(ea);
    }
    // rows beyond a multiple of kEncAhead, one at a time
    uint64_t t = rows_full;
    for (uint32_t r = (uint32_t)(rows_full % kEncAhead); r > 0; r--, t--) {
      lookup(ea, src.template fetch<SPL>(base + (t - 1) * S + j0));
      row(ea);
    }
    // at most 1 + 7 words staged so far; from here on every batch ends with a flush, which keeps a
    // stream's staged words below 8 at the start of a batch and below 16 (the ring size) inside it
#pragma unroll
    for (int i = 0; i < SPL; i++) flush(i);
    // full batches of kEncAhead rows: rows fetched one batch ahead, table entries one row ahead,
    // alternating between two register sets
    uint32_t cur[kEncAhead], nxt[kEncAhead];
    // Table entries are looked up kLook rows ahead of their use (an LDS read takes longer than the
    // arithmetic of a row), in a rotation of kLook + 1 register sets.
    constexpr int kLook = 3;
    EncEntry E[kLook + 1][SPL];
    auto prime = [&]() {  // entries of the first kLook rows of nxt[]
#pragma unroll
      for (int u = 0; u < kLook; u++) lookup(E[u], nxt[u]);
    };
    auto batch = [&]() {  // codes the rows in cur[]; leaves the entries of nxt[0 .. kLook-1] in E[0 .. kLook-1]
#pragma unroll
      for (int u = 0; u < kEncAhead; u++) {
        // past the end of the batch this looks up rows of the next batch; when there is none, nxt[]
        // still holds old, valid symbols and the entries are simply not used
        lookup(E[(u + kLook) % (kLook + 1)], u + kLook < kEncAhead ? cur[(u + kLook) % kEncAhead] : nxt[(u + kLook) % kEncAhead]);
        row(E[u % (kLook + 1)]);
      }
#pragma unroll
      for (int i = 0; i < SPL; i++) flush(i);
    };
    if constexpr (WIDE) {
      // Symbols through LDS: single-byte loads keep too few bytes in flight to cover the memory latency.
      // A wave owns a 64-byte column of the chunk's rows.  It fetches kStageRows rows of it at a time
      // with 16-byte loads (lane L: row L/4 and row 16 + L/4 of the tile, bytes 16 (L%4) ..), a whole tile
      // ahead of the coder, and parks them in a private LDS area that holds two tiles, row r in line
      // r mod 64; the coder reads its byte of each row from there.  No other wave touches the area.
      static_assert(!WIDE || (SPL == 1 && kEncAhead == 8 && kStageRows == 32), "tile arithmetic below");
      const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
      uint8_t *stg = (uint8_t *)(sh + 16) + wv * (2 * kStageRows * 64);
      const uint8_t *colp = src.bytes() + base + (j0 - lane) + 16 * (lane & 3);  // the lane's 16 bytes of row 0
      uint4 pend[2];
      auto request = [&](uint64_t t_lo, uint64_t t_top) {  // rows t_lo .. t_lo+31 (below t_top) of the column
#pragma unroll
        for (int h = 0; h < 2; h++) {
          const uint64_t r = t_lo + 16 * h + (lane >> 2);
          pend[h] = make_uint4(0, 0, 0, 0);
          if (r < t_top) pend[h] = *(const uint4 *)(colp + r * S);
        }
      };
      auto park = [&](uint64_t t_lo) {
#pragma unroll
        for (int h = 0; h < 2; h++)
          *(uint4 *)(stg + (((uint32_t)t_lo + 16 * h) & 63u) * 64 + 16 * lane) = pend[h];
      };
      auto read_rows = [&](uint32_t *dst, uint64_t t_hi) {  // rows t_hi-1 .. t_hi-8; t_hi is a multiple of 8
        const uint8_t *b = stg + (((uint32_t)t_hi - 8) & 63u) * 64 + lane;
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) dst[u] = b[(kEncAhead - 1 - u) * 64];
      };
      if (t) {
        const uint64_t t_lo = (t - 1) & ~(uint64_t)(kStageRows - 1);
        request(t_lo, t);
        park(t_lo);
        if (t_lo) request(t_lo - kStageRows, t_lo);
        read_rows(nxt, t);
        prime();
      }
      while (t) {
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) cur[u] = nxt[u];
        t -= kEncAhead;
        if (t) {
          if ((t & (kStageRows - 1)) == 0) {  // the next rows belong to the tile below: it has arrived by now
            park(t - kStageRows);
            if (t > kStageRows) request(t - 2 * kStageRows, t - kStageRows);
          }
          read_rows(nxt, t);
        }
        batch();
      }
    } else if constexpr (WIDE_KIND == 2) {
      // The same for D = v (+) c (+) r (Eq. 7), staged as 16-bit entries.  A wave owns 64 streams; a tile is
      // kStageRows2 rows of them, lane L fetches the 16 entries 16 (L % 4) .. of row L / 4: one 16-byte load
      // where they all lie in v, two where they all lie in c or in r (2-byte aligned: where c starts inside D
      // depends on the number of nonzeros), entry by entry where they straddle two parts or the end of D.
      static_assert(WIDE_KIND != 2 || (SPL == 1 && kEncAhead == 8 && kStageRows2 == 16), "tile arithmetic below");
      const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
      // 16-byte aligned whatever the size of the table before it
      uint8_t *stg = (uint8_t *)(((uintptr_t)(sh + 16) + 15) & ~(uintptr_t)15) + wv * (2 * kStageRows2 * 128);
      const uint64_t nnz = src.nnz_of();
      const uint64_t col_i = base + (j0 - lane) + 16 * (lane & 3);  // D index of the lane's 16 entries in row 0
      uint4 pend[2];
      auto request = [&](uint64_t t_lo, uint64_t t_top) {  // rows t_lo .. t_lo+15 (below t_top) of the column
        const uint64_t r = t_lo + (lane >> 2);
        pend[0] = pend[1] = make_uint4(0, 0, 0, 0);
        if (r < t_top) {
          const uint64_t i = col_i + r * S;
          if (i + 16 <= nnz) {  // values: bytes, widened when they are parked
            pend[0] = *(const uint4 *)(src.v_ptr() + i);
          } else if (i >= nnz && (i + 16 <= 2 * nnz || (i >= 2 * nnz && i + 16 <= len))) {
            const uint16_t *q = i < 2 * nnz ? src.c_ptr() + (i - nnz) : src.r_ptr() + (i - 2 * nnz);
            __builtin_memcpy(&pend[0], q, 16);
            __builtin_memcpy(&pend[1], q + 8, 16);
          } else {
            uint32_t w[8];
#pragma unroll
            for (int k = 0; k < 8; k++) {
              const uint32_t lo = i + 2 * k < len ? src(i + 2 * k) : 0u, hi = i + 2 * k + 1 < len ? src(i + 2 * k + 1) : 0u;
              w[k] = lo | (hi << 16);
            }
            pend[0] = make_uint4(w[0], w[1], w[2], w[3]);
            pend[1] = make_uint4(w[4], w[5], w[6], w[7]);
          }
        }
      };
      auto park = [&](uint64_t t_lo, uint64_t t_top) {
        const uint64_t r = t_lo + (lane >> 2);
        const uint64_t i = col_i + r * S;
        uint4 a = pend[0], b = pend[1];
        if (r < t_top && i + 16 <= nnz) {  // 16 bytes -> 16 16-bit entries
          const uint32_t ww[4] = {pend[0].x, pend[0].y, pend[0].z, pend[0].w};
          uint32_t e[8];
#pragma unroll
          for (int k = 0; k < 8; k++) {
            const uint32_t two = ww[k >> 1] >> (16 * (k & 1));
            e[k] = (two & 0xffu) | ((two & 0xff00u) << 8);
          }
          a = make_uint4(e[0], e[1], e[2], e[3]);
          b = make_uint4(e[4], e[5], e[6], e[7]);
        }
        uint4 *line = (uint4 *)(stg + (((uint32_t)t_lo + (lane >> 2)) & 31u) * 128 + 32 * (lane & 3));
        line[0] = a;
        line[1] = b;
      };
      auto read_rows = [&](uint32_t *dst, uint64_t t_hi) {  // rows t_hi-1 .. t_hi-8; t_hi is a multiple of 8
        const uint8_t *b = stg + (((uint32_t)t_hi - 8) & 31u) * 128 + 2 * lane;
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) dst[u] = *(const uint16_t *)(b + (kEncAhead - 1 - u) * 128);
      };
      uint64_t t_req_top = 0;  // upper row bound of the tile in flight (park needs it to tell how it was fetched)
      if (t) {
        const uint64_t t_lo = (t - 1) & ~(uint64_t)(kStageRows2 - 1);
        request(t_lo, t);
        park(t_lo, t);
        if (t_lo) {
          request(t_lo - kStageRows2, t_lo);
          t_req_top = t_lo;
        }
        read_rows(nxt, t);
        prime();
      }
      while (t) {
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) cur[u] = nxt[u];
        t -= kEncAhead;
        if (t) {
          if ((t & (kStageRows2 - 1)) == 0) {  // the next rows belong to the tile below: it has arrived by now
            park(t - kStageRows2, t_req_top);
            if (t > kStageRows2) {
              request(t - 2 * kStageRows2, t - kStageRows2);
              t_req_top = t - kStageRows2;
            }
          }
          read_rows(nxt, t);
        }
        batch();
      }
    } else {
      auto fetch_rows = [&](uint32_t *dst, uint64_t t_hi) {  // rows t_hi-1 .. t_hi-kEncAhead
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) dst[u] = src.template fetch<SPL>(base + (t_hi - 1 - u) * S + j0);
      };
      if (t) {
        fetch_rows(nxt, t);
        prime();
      }
      while (t) {
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) cur[u] = nxt[u];
        t -= kEncAhead;
        if (t) fetch_rows(nxt, t);
        batch();
      }
    }
  };
  if (live) {
    if constexpr (std::is_same<Src, SrcDense>::value && SPL == 1) {
      if (wide) {
        if (exact) run(std::true_type{}, std::integral_constant<int, 1>{});
        else run(std::false_type{}, std::integral_constant<int, 1>{});
      } else {
        if (exact) run(std::true_type{}, std::integral_constant<int, 0>{});
        else run(std::false_type{}, std::integral_constant<int, 0>{});
      }
    } else if constexpr (std::is_same<Src, SrcCsr>::value && SPL == 1) {
      if (wide) {
        if (exact) run(std::true_type{}, std::integral_constant<int, 2>{});
        else run(std::false_type{}, std::integral_constant<int, 2>{});
      } else {
        if (exact) run(std::true_type{}, std::integral_constant<int, 0>{});
        else run(std::false_type{}, std::integral_constant<int, 0>{});
      }
    } else {
      if (exact) run(std::true_type{}, std::integral_constant<int, 0>{});
      else run(std::false_type{}, std::integral_constant<int, 0>{});
    }
  }
  uint32_t nw[SPL];
#pragma unroll
  for (int i = 0; i < SPL; i++) {
    const uint16_t *g0 = scratch + (uint64_t)blockIdx.x * (kWG * SPL) * capw + (i * kWG + threadIdx.x) * 8;
    const uint32_t n_rem = (colb[i] + 30 - wp[i]) >> 1;  // fewer than 8
    nw[i] = live ? (uint32_t)((gp[i] - g0) / (kWG * SPL)) + n_rem : 0;
    if (live) {
      // the remaining words sit at the top of the area's upper half: it leaves as one more block, whose
      // first 8 - n_rem words are not part of the stream
      if (n_rem) {
        const lds_u64 *r = (const lds_u64 *)(uintptr_t)colb[i];
        const uint64_t hi0 = r[2], hi1 = r[3];
        *(uint4 *)gp[i] = make_uint4((uint32_t)hi0, (uint32_t)(hi0 >> 32), (uint32_t)hi1, (uint32_t)(hi1 >> 32));
      }
      if (!FUSE) {
        st_out[(uint64_t)k * S + j0 + i] = s[i];
        nw_out[(uint64_t)k * S + j0 + i] = nw[i];
      }
    }
  }
  uint32_t mine = 0;
#pragma unroll
  for (int i = 0; i < SPL; i++) mine += nw[i];
  uint32_t tot;
  const uint32_t ex = block_excl_scan<kWG>(mine, sh, &tot);
  if (!FUSE) {
    if (threadIdx.x == 0 && tot) atomicAdd(&chunk_words[k], tot);
    return;
  }
  if constexpr (FUSE) {
    static_assert(!FUSE || SPL == 1, "the fused placement assumes one stream per lane");
    if (threadIdx.x == 0) __hip_atomic_store(wg_pub + blockIdx.x, tot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // The lane's own words come back from scratch in the aligned 16-byte blocks written above (block 0
    // is the lowest one; it starts with `skip` words that are not part of the stream).
    constexpr int kInFlight = 4;
    const uint32_t nw1 = live ? nw[0] : 0;
    // block bi of the stream in read order (bi = 0: the newest, partial one) is block nb - 1 - bi as written
    const uint16_t *g0 = scratch + (uint64_t)blockIdx.x * kWG * capw + threadIdx.x * 8;
    const uint32_t nb = (nw1 + 7) / 8, skip = nb * 8 - nw1;
    // totals of the work-groups before this one: whole chunks give the chunk's byte offset, the groups
    // of this chunk before g give the position inside the chunk
    uint64_t off_loc = 0, pre_loc = 0;
    uint32_t failed = 0;
    for (uint32_t c = threadIdx.x; c < k; c += kWG) {
      uint64_t words = 0;
      for (uint32_t g2 = 0; g2 < groups; g2++) {
        const uint32_t v = wait_published(wg_pub, c * groups + g2, ctl);
        failed |= v == 0;
        words += v - 1;
      }
      off_loc += (8ull * S + 2 * words + 3) & ~3ull;
    }
    for (uint32_t g2 = threadIdx.x; g2 < g; g2 += kWG) {
      const uint32_t v = wait_published(wg_pub, k * groups + g2, ctl);
      failed |= v == 0;
      pre_loc += v - 1;
    }
    uint64_t *sh64 = (uint64_t *)(sh + 4);
    const uint64_t off = block_sum64<kWG>(off_loc, sh64);
    const uint64_t pre = block_sum64<kWG>(pre_loc, sh64);
    const uint64_t any_failed = block_sum64<kWG>(failed, sh64);
    if (any_failed) {  // uniform: a wait ran into its bound, or another work-group reported an error
      if (threadIdx.x == 0) {
        if (get_status(ctl) == 0) set_status(ctl, RANS_ERR_HIP);
        if (k == nc - 1 && g == groups - 1 && d_stream_bytes) *d_stream_bytes = 0;
      }
      return;
    }
    uint8_t *dir = out + ctl->dir_off;
    const uint64_t my_end = ctl->payload_off + off + 8ull * S + 2 * (pre + tot);  // end of this group's words
    const bool last_group = g == groups - 1;
    const uint64_t chunk_end = (my_end + 3) & ~3ull;  // meaningful for the chunk's last group
    const bool fits = (last_group ? chunk_end : my_end) <= cap;
    if (threadIdx.x == 0) {
      if (g == 0) {
        st32(dir + 8ull * k, (uint32_t)off);
        st32(dir + 8ull * k + 4, (uint32_t)(off >> 32));
      }
      if (k == nc - 1 && last_group) {
        const uint64_t pay = chunk_end - ctl->payload_off;
        st32(dir + 8ull * nc, (uint32_t)pay);
        st32(dir + 8ull * nc + 4, (uint32_t)(pay >> 32));
        ctl->total_bytes = chunk_end;
        if (d_stream_bytes) *d_stream_bytes = fits ? chunk_end : 0;
      }
      if (!fits) set_status(ctl, RANS_ERR_CAPACITY);
    }
    if (!fits) return;  // uniform
    uint8_t *ck = out + ctl->payload_off + off;
    const uint32_t j = j0;
    if (live) {
      st32(ck + 4ull * j, s[0]);
      st32(ck + 4ull * S + 4ull * j, nw1);
    }
    // words: registers / scratch -> LDS tile -> container.  A lane stages its own stream's words in LDS
    // at their position in the chunk; the work-group then writes the staged tile out in aligned
    // 16-byte vectors (single words only at the two ends of its range).  The tile reuses the ring and
    // the table, which are no longer needed.  Tile positions are shifted by the destination's offset
    // inside a 16-byte vector, so LDS vectors and output vectors coincide.
    uint16_t *tile = (uint16_t *)l_mem;
    constexpr uint32_t kTile = kEncTileBytes / 2;
    uint16_t *dst = (uint16_t *)(ck + 8ull * S) + pre;
    const uint32_t shift = (uint32_t)(((uintptr_t)dst >> 1) & 7);
    uint16_t *vbase = dst - shift;  // 16-byte aligned; tile word p' (over all tiles) goes to vbase[p']
    const uint32_t exs = ex + shift;
    lds_barrier();  // everyone is done with the ring, the table and the reduction scratch
    for (uint32_t t0 = 0; t0 < shift + tot; t0 += kTile) {
      const uint32_t lo = exs > t0 ? exs : t0;
      const uint32_t hi = exs + nw1 < t0 + kTile ? exs + nw1 : t0 + kTile;
      auto stage = [&](const uint4 &q, uint32_t bi) {
        const uint32_t w0 = bi * 8 - skip;  // read-order number of the block's first word (wraps in block 0)
        const uint32_t pos0 = exs + w0;
        if (bi * 8 >= skip && pos0 >= lo && pos0 + 8 <= hi) {
          // the whole block belongs to the stream and to this tile: one 16-byte LDS store at a 2-byte
          // aligned address (the target allows unaligned LDS access)
          __builtin_memcpy(tile + (pos0 - t0), &q, 16);
        } else {
          const uint32_t ww[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int i = 0; i < 8; i++) {
            const uint32_t pos = pos0 + i;
            if (w0 + i < nw1 && pos >= lo && pos < hi) tile[pos - t0] = (uint16_t)(ww[i >> 1] >> (16 * (i & 1)));
          }
        }
      };
      if (lo < hi) {
        const uint32_t b_lo = (lo - exs + skip) / 8, b_hi = (hi - 1 - exs + skip) / 8;
        for (uint32_t b0 = b_lo; b0 <= b_hi; b0 += kInFlight) {
          uint4 q[kInFlight];
#pragma unroll
          for (int u = 0; u < kInFlight; u++)
            if (b0 + u <= b_hi) q[u] = *(const uint4 *)(g0 + (uint64_t)(nb - 1 - (b0 + u)) * (kWG * 8));
#pragma unroll
          for (int u = 0; u < kInFlight; u++)
            if (b0 + u <= b_hi) stage(q[u], b0 + u);
        }
      }
      lds_barrier();
      const uint32_t a = t0 == 0 ? shift : 0;                                      // first valid tile word
      const uint32_t e = shift + tot - t0 < kTile ? shift + tot - t0 : kTile;      // end of the valid tile words
      const uint32_t head_end = a ? (e < 8u ? e : 8u) : 0;
      const uint32_t v_lo = a ? 1 : 0, v_hi = e / 8;
      const uint32_t tail_beg = v_hi >= v_lo ? 8 * v_hi : e;
      for (uint32_t v = v_lo + threadIdx.x; v < v_hi; v += kWG) ((uint4 *)(vbase + t0))[v] = ((const uint4 *)tile)[v];
      if (threadIdx.x < 8) {
        const uint32_t h = a + threadIdx.x, t = tail_beg + threadIdx.x;
        if (h < head_end) vbase[t0 + h] = tile[h];
        if (t < e) vbase[t0 + t] = tile[t];
      }
      lds_barrier();
    }
    if (last_group && live && j == S - 1 && ((pre + tot) & 1)) dst[tot] = 0;  // pad the chunk to 4 bytes
  }
}

// Chunk sizes -> directory (byte offsets from the payload start), total size.
__global__ __launch_bounds__(kBig) void k_chunk_scan(CtlRef ctl, uint32_t *chunk_words, uint32_t S, uint8_t *out,
                                                     uint64_t cap, uint64_t *d_stream_bytes) {
  __shared__ uint64_t sh64[kBig / 64];
  if (get_status(ctl) != 0) {
    if (threadIdx.x == 0 && d_stream_bytes) *d_stream_bytes = 0;
    return;
  }
  const uint32_t nc = ctl->n_chunks;
  uint8_t *dir = out + ctl->dir_off;
  uint64_t carry = 0;
  for (uint32_t base = 0; base < nc; base += kBig) {
    uint32_t k = base + threadIdx.x;
    uint64_t sz = 0;
    if (k < nc) sz = (8ull * S + 2ull * chunk_words[k] + 3) & ~3ull;
    // inclusive scan over the work-group in 64 bits
    uint64_t inc = sz;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      uint32_t lo = __shfl_up((uint32_t)inc, d), hi = __shfl_up((uint32_t)(inc >> 32), d);
      if (lane >= d) inc += ((uint64_t)hi << 32) | lo;
    }
    __syncthreads();
    if (lane == 63) sh64[w] = inc;
    __syncthreads();
    uint64_t pre = 0, tot = 0;
    for (int i = 0; i < kBig / 64; i++) {
      if (i < w) pre += sh64[i];
      tot += sh64[i];
    }
    if (k < nc) {
      uint64_t off = carry + pre + inc - sz;
      st32(dir + 8ull * k, (uint32_t)off);
      st32(dir + 8ull * k + 4, (uint32_t)(off >> 32));
    }
    carry += tot;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    st32(dir + 8ull * nc, (uint32_t)carry);
    st32(dir + 8ull * nc + 4, (uint32_t)(carry >> 32));
    uint64_t total = ctl->payload_off + carry;
    ctl->total_bytes = total;
    if (total > cap) {
      set_status(ctl, RANS_ERR_CAPACITY);
      total = 0;
    }
    if (d_stream_bytes) *d_stream_bytes = total;
  }
}

// Moves each stream's words from its scratch region to its place in the chunk and
// writes the chunk header (final states, word counts).  A lane reads its own
// stream's words in the aligned 16-byte blocks the encoder wrote, stages them in
// LDS at their scanned position, and the work-group writes the staged tile out with
// consecutive lanes on consecutive words.
//
// FUSED_SCAN: the chunk's byte offset is computed here by summing the sizes of the
// chunks before it (cheap for up to a few thousand chunks), and the work-groups with
// g == 0 write the directory; otherwise k_chunk_scan has written the directory.
constexpr uint32_t kGatherTile = 8192;     // words per LDS tile
constexpr uint32_t kFusedScanMax = 4096;   // chunks up to which the gather kernel scans the sizes itself
template <bool FUSED_SCAN>
__global__ __launch_bounds__(kWG) void k_gather(CtlRef ctl, const uint16_t *scratch, uint32_t capw, const uint32_t *st,
                                                const uint32_t *nw_arr, const uint32_t *chunk_words, uint32_t S,
                                                uint32_t groups, uint8_t *out, uint64_t cap,
                                                uint64_t *d_stream_bytes) {
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint64_t sh64[kWG / 64];
  __shared__ uint16_t tile[kGatherTile];
  if (get_status(ctl) != 0) {
    if (FUSED_SCAN && blockIdx.x == 0 && threadIdx.x == 0 && d_stream_bytes) *d_stream_bytes = 0;
    return;
  }
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  const uint32_t nc = ctl->n_chunks;
  if (FUSED_SCAN && nc == 0 && blockIdx.x == 0) {  // empty D: only the directory's single entry
    if (threadIdx.x == 0) {
      uint8_t *dir0 = out + ctl->dir_off;
      st32(dir0, 0u);
      st32(dir0 + 4, 0u);
      ctl->total_bytes = ctl->payload_off;
      if (d_stream_bytes) *d_stream_bytes = ctl->payload_off;
    }
    return;
  }
  if (k >= nc) return;
  uint8_t *dir = out + ctl->dir_off;
  uint64_t off;
  if (FUSED_SCAN) {
    uint64_t loc = 0;
    for (uint32_t i = threadIdx.x; i < k; i += kWG) loc += (8ull * S + 2ull * chunk_words[i] + 3) & ~3ull;
    off = block_sum64<kWG>(loc, sh64);
    const uint64_t my_size = (8ull * S + 2ull * chunk_words[k] + 3) & ~3ull;
    const uint64_t end_abs = ctl->payload_off + off + my_size;
    const bool fits = end_abs <= cap;
    if (g == 0 && threadIdx.x == 0) {
      st32(dir + 8ull * k, (uint32_t)off);
      st32(dir + 8ull * k + 4, (uint32_t)(off >> 32));
      if (k == nc - 1) {
        st32(dir + 8ull * nc, (uint32_t)(off + my_size));
        st32(dir + 8ull * nc + 4, (uint32_t)((off + my_size) >> 32));
        ctl->total_bytes = end_abs;
        if (d_stream_bytes) *d_stream_bytes = fits ? end_abs : 0;
      }
    }
    if (!fits) {  // uniform: this chunk would end past the buffer
      if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CAPACITY);
      return;
    }
  } else {
    off = ld64(dir + 8ull * k);
  }
  uint8_t *ck = out + ctl->payload_off + off;
  const uint32_t *nwk = nw_arr + (uint64_t)k * S;
  // words of the streams that precede this group inside the chunk
  uint64_t pre_loc = 0;
  for (uint32_t i = threadIdx.x; i < g * kWG; i += kWG) pre_loc += nwk[i];
  const uint64_t pre = block_sum64<kWG>(pre_loc, sh64);
  const uint32_t j = g * kWG + threadIdx.x;
  const uint32_t nw = j < S ? nwk[j] : 0;
  uint32_t tot;
  const uint32_t ex = block_excl_scan<kWG>(nw, sh, &tot);
  if (j < S) {
    st32(ck + 4ull * j, st[(uint64_t)k * S + j]);
    st32(ck + 4ull * S + 4ull * j, nw);
  }
  // block bi of the stream in read order (bi = 0: the newest, partial one) is block nb - 1 - bi as written
  const uint16_t *g0 = scratch + (uint64_t)blockIdx.x * kWG * capw + threadIdx.x * 8;
  const uint32_t nb = (nw + 7) / 8;                                    // aligned 8-word blocks that hold the words
  const uint32_t skip = nb * 8 - nw;                                   // words of the lowest block before the first one
  uint16_t *dst = (uint16_t *)(ck + 8ull * S) + pre;                   // first word of this group
  for (uint32_t t0 = 0; t0 < tot; t0 += kGatherTile) {
    // word w of this stream (in read order) has group position ex + w and sits in block (w + skip) / 8
    const uint32_t lo = ex > t0 ? ex : t0;
    const uint32_t hi = ex + nw < t0 + kGatherTile ? ex + nw : t0 + kGatherTile;
    if (lo < hi) {
      const uint32_t b_lo = (lo - ex + skip) / 8, b_hi = (hi - 1 - ex + skip) / 8;
      for (uint32_t bi = b_lo; bi <= b_hi; bi++) {
        const uint4 q = *(const uint4 *)(g0 + (uint64_t)(nb - 1 - bi) * (kWG * 8));
        const uint32_t ww[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int i = 0; i < 8; i++) {
          const uint32_t pos = ex + bi * 8 + i - skip;  // wraps below ex for the skipped words: fails the test
          if (bi * 8 + i >= skip && pos >= lo && pos < hi) tile[pos - t0] = (uint16_t)(ww[i >> 1] >> (16 * (i & 1)));
        }
      }
    }
    __syncthreads();
    const uint32_t cnt = tot - t0 < kGatherTile ? tot - t0 : kGatherTile;
    for (uint32_t i = threadIdx.x; i < cnt; i += kWG) dst[t0 + i] = tile[i];
    __syncthreads();
  }
  if (j == S - 1 && ((pre + tot) & 1)) dst[tot] = 0;  // pad the chunk to 4 bytes
}

// ------------------------------------------------------------------ kernels: decode

// One work-group: validate the header against the expected geometry, rebuild F,
// the slot -> symbol table (Eq. 3) and the decoder table f | F << 16, recompute
// s and z from the stored extrema.
__global__ __launch_bounds__(kBig) void k_dec_prepare(const uint8_t *in, uint64_t bytes, CtlRef ctl, rans_header h,
                                                      uint16_t *lut, uint32_t *tab, uint32_t *Farr,
                                                      rans_qinfo *qout) {
  __shared__ uint32_t sh32[kBig / 64];
  __shared__ int s_ok;
  const uint32_t A = h.alphabet, M = h.p.freq_bits, total = 1u << M;
  const uint64_t table_off = kHdrBytes;
  const uint64_t dir_off = table_off + (((uint64_t)A * 2 + 7) & ~7ull);
  const uint64_t payload_off = dir_off + 8 * ((uint64_t)h.n_chunks + 1);
  if (threadIdx.x == 0) {
    bool ok = bytes >= payload_off;
    ok = ok && ld32(in) == 0x31464952u;
    ok = ok && ld32(in + 4) == (1u | (h.p.mode << 16) | (h.p.in_dtype << 24));
    ok = ok && ld32(in + 8) == (h.p.q_bits | (M << 8));
    ok = ok && ld64(in + 12) == h.n_elems && ld64(in + 20) == h.p.rows && ld64(in + 28) == h.p.cols;
    ok = ok && ld64(in + 36) == h.len_d && ld32(in + 44) == A && ld32(in + 48) == h.p.n_streams;
    ok = ok && ld32(in + 52) == h.p.chunk_syms && ld32(in + 56) == h.n_chunks;
    ok = ok && ld32(in + 60) == __float_as_uint(h.x_min) && ld32(in + 64) == __float_as_uint(h.x_max);
    if (ok)
      for (uint32_t o = 68; o < kHdrBytes; o += 4) ok = ok && ld32(in + o) == 0;
    if (ok) {
      ok = ok && ld64(in + dir_off) == 0 && ld64(in + dir_off + 8ull * h.n_chunks) == bytes - payload_off;
    }
    s_ok = ok;
    ctl->last_seq = ctl.seq;
    if (!ok) set_status(ctl, RANS_ERR_CORRUPT);
    ctl->len_d = h.len_d;
    ctl->n_chunks = h.n_chunks;
    ctl->dir_off = dir_off;
    ctl->payload_off = payload_off;
    ctl->nnz = h.p.mode == RANS_MODE_CSR ? (uint32_t)((h.len_d - h.p.rows) / 2) : 0;
    // Eq. 6 parameters from the stored extrema, same arithmetic as on the encoding side
    float mn = h.x_min, mx = h.x_max;
    float range = mx - mn;
    float s = range / (float)((1u << h.p.q_bits) - 1u);
    float zf = eq6_zero_point(mn, s);
    ctl->x_min = mn;
    ctl->x_max = mx;
    ctl->scale = s;
    ctl->zero_point = zf;
    if (qout) {
      qout->x_min = mn;
      qout->x_max = mx;
      qout->scale = s;
      qout->zero_point = zf;
    }
  }
  __syncthreads();
  if (!s_ok) return;
  // F and the decoder table; marks for the slot table
  for (uint32_t sl = threadIdx.x; sl < total; sl += kBig) lut[sl] = 0;
  __syncthreads();
  uint32_t carry = 0;
  bool pad_ok = true;
  for (uint32_t base = 0; base < A; base += kBig) {
    uint32_t a = base + threadIdx.x;
    uint32_t f = a < A ? *(const uint16_t *)(in + table_off + 2ull * a) : 0, tot;
    uint32_t F = carry + block_excl_scan<kBig>(f, sh32, &tot);
    if (a < A) {
      tab[a] = f | (F << 16);
      Farr[a] = F;
      if (f && F < total) lut[F] = (uint16_t)a;  // symbols with f > 0 start at distinct slots
    }
    carry += tot;
    __syncthreads();
  }
  for (uint64_t o = table_off + 2ull * A + 2 * threadIdx.x; o < dir_off; o += 2 * kBig)
    pad_ok = pad_ok && *(const uint16_t *)(in + o) == 0;
  if (!pad_ok) set_status(ctl, RANS_ERR_CORRUPT);
  if (carry != (h.len_d ? total : 0u)) {
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  if (threadIdx.x == 0) Farr[A] = carry;
  __syncthreads();
  // slot table = running maximum of the marks: each thread owns a contiguous range of slots
  const uint32_t per = (total + kBig - 1) / kBig;
  const uint32_t s0 = threadIdx.x * per;
  uint32_t loc = 0;
  for (uint32_t i = 0; i < per && s0 + i < total; i++) {
    uint32_t m = lut[s0 + i];
    loc = m > loc ? m : loc;
  }
  // exclusive running maximum across threads
  uint32_t inc = loc;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    uint32_t o = __shfl_up(inc, d);
    if (lane >= d) inc = o > inc ? o : inc;
  }
  uint32_t prev = __shfl_up(inc, 1);
  if (lane == 0) prev = 0;
  __syncthreads();
  if (lane == 63) sh32[w] = inc;
  __syncthreads();
  uint32_t run = 0;
  for (int i = 0; i < w; i++) run = sh32[i] > run ? sh32[i] : run;
  run = prev > run ? prev : run;
  for (uint32_t i = 0; i < per && s0 + i < total; i++) {
    uint32_t m = lut[s0 + i];
    run = m > run ? m : run;
    lut[s0 + i] = (uint16_t)run;
  }
}

struct SinkSym {
  uint8_t *out;
  __device__ __forceinline__ void init(const CtlRef &) {}
  __device__ __forceinline__ void put(uint64_t i, uint32_t x) const { out[i] = (uint8_t)x; }
};
struct SinkU16 {
  uint16_t *out;
  __device__ __forceinline__ void init(const CtlRef &) {}
  __device__ __forceinline__ void put(uint64_t i, uint32_t x) const { out[i] = (uint16_t)x; }
};
// Inverse of Eq. 6 fused into the decoder: x = s * (xhat - z).
template <typename OutT>
struct SinkFloat {
  OutT *out;
  float s, zf, x_min;
  __device__ __forceinline__ void init(const CtlRef &ctl) {
    s = ctl->scale;
    zf = ctl->zero_point;
    x_min = ctl->x_min;
  }
  __device__ __forceinline__ void put(uint64_t i, uint32_t x) const {
    float y = s == 0.0f ? x_min : s * ((float)x - zf);
    if constexpr (sizeof(OutT) == 4) out[i] = y;
    else out[i] = __float2half_rn(y);
  }
};

// One lane per stream: slot = s mod 2^M, symbol from the slot table (Eq. 3), state
// update (Eq. 4), refill of one 16-bit word when the state drops below 2^16.  All
// sizes and offsets taken from the container are checked before use.
template <class Sink, bool LDS_TAB>
__global__ __launch_bounds__(kWG) void k_decode(const uint8_t *in, uint64_t bytes, CtlRef ctl, const uint16_t *g_lut,
                                                const uint32_t *g_tab, uint32_t A, uint32_t M, uint32_t S,
                                                uint32_t cs, uint32_t groups, Sink sink) {
  extern __shared__ __align__(16) uint32_t l_mem[];
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint64_t sh64[kWG / 64];
  if (get_status(ctl) != 0) return;
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  const uint32_t nc = ctl->n_chunks;
  if (k >= nc) return;
  sink.init(ctl);
  const uint32_t total = 1u << M;
  uint32_t *l_tab = l_mem;
  uint16_t *l_lut = (uint16_t *)(l_mem + A);
  if (LDS_TAB) {
    for (uint32_t a = threadIdx.x; a < A; a += kWG) l_tab[a] = g_tab[a];
    for (uint32_t i = threadIdx.x; i < total / 2; i += kWG) ((uint32_t *)l_lut)[i] = ((const uint32_t *)g_lut)[i];
    __syncthreads();
  }
  const uint32_t *tab = LDS_TAB ? l_tab : g_tab;
  const uint16_t *lut = LDS_TAB ? l_lut : g_lut;

  const uint64_t payload_off = ctl->payload_off;
  const uint64_t payload_bytes = bytes - payload_off;
  const uint8_t *dir = in + ctl->dir_off;
  const uint64_t o0 = ld64(dir + 8ull * k), o1 = ld64(dir + 8ull * k + 8);
  if (o0 > o1 || o1 > payload_bytes || o1 - o0 < 8ull * S || (o0 & 3)) {
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  const uint8_t *ck = in + payload_off + o0;
  const uint64_t ck_bytes = o1 - o0;
  const uint64_t len = ctl->len_d;
  const uint64_t chunk_len = cs ? cs : len;
  const uint64_t base = (uint64_t)k * chunk_len;
  const uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
  const uint32_t *nwk = (const uint32_t *)(ck + 4ull * S);
  uint64_t pre_loc = 0;
  for (uint32_t i = threadIdx.x; i < g * kWG; i += kWG) pre_loc += nwk[i];
  const uint64_t pre = block_sum64<kWG>(pre_loc, sh64);
  const uint32_t j = g * kWG + threadIdx.x;
  const bool live = j < S;
  const uint64_t n_j = (live && n_here > j) ? (n_here - j + S - 1) / S : 0;
  uint32_t nw = live ? nwk[j] : 0;
  bool bad = false;
  if (nw > n_j) {
    bad = true;
    nw = 0;
  }
  uint32_t tot;
  const uint32_t ex = block_excl_scan<kWG>(nw, sh, &tot);
  const uint64_t w0 = pre + ex;  // index of this stream's first word inside the chunk
  if (8ull * S + 2 * (w0 + nw) > ck_bytes) {
    bad = true;
    nw = 0;
  }
  if (live) {
    const uint16_t *wp = (const uint16_t *)(ck + 8ull * S) + w0;
    uint32_t s = ((const uint32_t *)ck)[j];
    uint32_t used = 0;
    const uint32_t mask = total - 1;
    for (uint64_t t = 0; t < n_j; t++) {
      bad |= s < kL;
      uint32_t slot = s & mask;
      uint32_t x = lut[slot];
      uint32_t e = tab[x];
      s = (e & 0xffffu) * (s >> M) + slot - (e >> 16);
      if (s < kL) {
        uint32_t w = 0;
        if (used < nw) w = wp[used++];
        else bad = true;
        s = (s << 16) | w;
      }
      sink.put(base + j + t * S, x);
    }
    bad |= (s != kL) || (used != nw);
    if (j == S - 1) {  // chunk size must be exactly header + words, padded to 4 bytes with zeros
      uint64_t end = 8ull * S + 2 * (w0 + nw);
      if (((end + 3) & ~3ull) != ck_bytes) bad = true;
      else if (end != ck_bytes && *(const uint16_t *)(ck + end) != 0) bad = true;
    }
  }
  if (bad) set_status(ctl, RANS_ERR_CORRUPT);
}

// ---- fast decoder: tables rebuilt per work-group in LDS, word stream read through an LDS window ----

// The 128-byte header the caller expects, as 32 little-endian words.
struct HdrImage {
  uint32_t w[32];
};

// First wave of work-group 0 of the fast decoder: compare the header and the ends of the
// directory with what the host expects, check the zero padding after the frequency table,
// publish the geometry and the quantiser parameters (Eq. 6, recomputed from the stored extrema
// with the encoder's arithmetic).  The other work-groups do not wait for this: they take the
// geometry from the kernel arguments and report what they find themselves.
__device__ void dec_check_header(const uint8_t *in, uint64_t bytes, const CtlRef &ctl, const HdrImage &img,
                                 const rans_header &h, rans_qinfo *qout) {
  const uint32_t lane = threadIdx.x;  // called by threads 0..63
  const uint32_t A = h.alphabet;
  const uint64_t table_off = kHdrBytes;
  const uint64_t dir_off = table_off + (((uint64_t)A * 2 + 7) & ~7ull);
  const uint64_t payload_off = dir_off + 8 * ((uint64_t)h.n_chunks + 1);
  bool ok = true;
  if (lane < 32) ok = ld32(in + 4 * lane) == img.w[lane];
  if (lane == 32) ok = ld64(in + dir_off) == 0;
  if (lane == 33) ok = ld64(in + dir_off + 8ull * h.n_chunks) == bytes - payload_off;
  for (uint64_t o = table_off + 2ull * A + 2 * lane; o < dir_off; o += 128) ok = ok && *(const uint16_t *)(in + o) == 0;
  const bool all_ok = __ballot(!ok) == 0;
  if (lane != 0) return;
  ctl->last_seq = ctl.seq;
  if (!all_ok) set_status(ctl, RANS_ERR_CORRUPT);
  ctl->len_d = h.len_d;
  ctl->n_chunks = h.n_chunks;
  ctl->dir_off = dir_off;
  ctl->payload_off = payload_off;
  ctl->nnz = h.p.mode == RANS_MODE_CSR ? (uint32_t)((h.len_d - h.p.rows) / 2) : 0;
  const float mn = h.x_min, mx = h.x_max;
  const float sc = (mx - mn) / (float)((1u << h.p.q_bits) - 1u);
  const float zf = eq6_zero_point(mn, sc);
  ctl->x_min = mn;
  ctl->x_max = mx;
  ctl->scale = sc;
  ctl->zero_point = zf;
  if (qout) {
    qout->x_min = mn;
    qout->x_max = mx;
    qout->scale = sc;
    qout->zero_point = zf;
  }
}

// The same as a kernel of its own, for a container without chunks (nothing else to launch).
__global__ __launch_bounds__(64) void k_dec_begin(const uint8_t *in, uint64_t bytes, CtlRef ctl, HdrImage img,
                                                  rans_header h, rans_qinfo *qout) {
  dec_check_header(in, bytes, ctl, img, h, qout);
}

// Output side of the fast decoder.  bits(x) is evaluated once per symbol value when
// the tables are built; put() stores the precomputed bits.
struct FSinkSym {
  uint8_t *out;
  __device__ __forceinline__ uint32_t bits(uint32_t x, float, float, float) const { return x; }
  // byte_off is a byte offset from a wave-uniform base: the store can take the base from scalar
  // registers; non-temporal because the output is streamed once and must not evict the coded words
  __device__ __forceinline__ static void put(uint8_t *base, uint32_t byte_off, uint32_t b) {
    __builtin_nontemporal_store((uint8_t)b, base + byte_off);
  }
};
struct FSinkU16 {
  uint16_t *out;
  __device__ __forceinline__ uint32_t bits(uint32_t x, float, float, float) const { return x; }
  __device__ __forceinline__ static void put(uint16_t *base, uint32_t byte_off, uint32_t b) {
    __builtin_nontemporal_store((uint16_t)b, (uint16_t *)((uint8_t *)base + byte_off));
  }
};
// Inverse of Eq. 6 fused into the decoder: x = s * (xhat - z), one value per symbol.
template <typename OutT>
struct FSinkFloat {
  OutT *out;
  __device__ __forceinline__ uint32_t bits(uint32_t x, float sc, float zf, float x_min) const {
    const float y = sc == 0.0f ? x_min : sc * ((float)x - zf);
    if constexpr (sizeof(OutT) == 4) return __float_as_uint(y);
    else return (uint32_t)__half_as_ushort(__float2half_rn(y));
  }
  __device__ __forceinline__ static void put(OutT *base, uint32_t byte_off, uint32_t b) {
    if constexpr (sizeof(OutT) == 4) __builtin_nontemporal_store(b, (uint32_t *)((uint8_t *)base + byte_off));
    else __builtin_nontemporal_store((uint16_t)b, (uint16_t *)((uint8_t *)base + byte_off));
  }
};


// 16 bytes of the container at a 16-byte aligned offset; bytes past the end read as zero.
__device__ __forceinline__ uint4 load_block16(const uint8_t *in, uint64_t bytes, uint64_t off) {
  if (off + 16 <= bytes) return *(const uint4 *)(in + off);
  uint32_t w[4] = {0, 0, 0, 0};
  for (int q = 0; q < 8; q++)
    if (off + 2 * q + 2 <= bytes) w[q >> 1] |= (uint32_t) * (const uint16_t *)(in + off + 2 * q) << (16 * (q & 1));
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Interleaved rANS decoder (Eq. 3-4), one stream per lane.
//
// Every work-group rebuilds the tables in LDS from the stored frequencies: F by a
// block scan, {f | F << 16, output bits} per symbol, and the slot -> symbol table
// (Eq. 3) by marking each present symbol's first slot and taking a running maximum.
//
// A stream's words are read through a 16-word window in LDS ([row][stream] layout):
// the lane loads 16-byte aligned blocks of its segment from global memory and the
// coder consumes single words from the window, keeping the next word in a register.
// Refills happen at wave-uniform points, every four steps: the block fetched at one
// check is written to LDS at the next, and a block is requested as soon as the
// reader has entered the block before it.  A stream consumes at most one word per
// step and a block holds eight, so the words are always there in time, while the
// global loads have at least four steps to complete.
//
// Everything taken from the container is checked before use; loads never leave the
// buffer, and the final state / word count of every stream is verified.
//
// WIDE: instead of the two dependent lookups slot -> symbol -> {f, F, output}, one 8-byte entry per slot
// {f | (slot - F) << 16, output bits} (a 2^M x 8 B table): one LDS access on the state's dependency chain.
// The byte-per-slot table, the per-symbol table and the scan scratch are then only needed while the tables
// are built; they live at tmp_off, which may alias the window (not yet in use at that time).
template <class Sink, typename LutT, bool MUL24, int NT, bool WIDE>
__global__ __launch_bounds__(NT) void k_decode_fast(const uint8_t *in, uint64_t bytes, CtlRef ctl, uint32_t A,
                                                     uint32_t M, uint32_t S, uint32_t cs, uint32_t groups,
                                                     uint64_t len, uint64_t dir_off, uint64_t payload_off,
                                                     float x_min, float x_max, uint32_t q_bits, uint32_t tmp_off,
                                                     HdrImage img, rans_header hdr, rans_qinfo *qout, Sink sink) {
  extern __shared__ __align__(16) uint32_t l_mem[];
  constexpr uint32_t kWinRowBytes = 2 * NT;          // one 16-bit word per stream
  constexpr uint32_t kWinBytes = 16 * kWinRowBytes;   // 16-word window per stream
  constexpr uint32_t NW = NT / 64;                    // waves per work-group
  // this is the first kernel of the call: no status to look at yet; work-group 0 checks the header
  if (blockIdx.x == 0 && threadIdx.x < 64) dec_check_header(in, bytes, ctl, img, hdr, qout);
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  const uint32_t total = 1u << M, mask = total - 1;
  // LDS: [window][lut][misc: 48 words][tab: A x 8 B], or WIDE: [window][wide table] and
  // [lut][misc][tab] at tmp_off.  The window and the table the coder reads sit at constant offsets, so
  // their addresses need no base arithmetic.
  LutT *lut = (LutT *)(l_mem + (WIDE ? tmp_off : kWinBytes) / 4);
  uint32_t *misc = (uint32_t *)lut + ((total * (uint32_t)sizeof(LutT) + 15) / 16) * 4;
  uint64_t *misc64 = (uint64_t *)(misc + 16);
  uint2 *tab = (uint2 *)(misc + 48);
  uint2 *wide = (uint2 *)(l_mem + kWinBytes / 4);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // ---- global loads of the stream set-up first: their latency overlaps the table build below
  const uint32_t f_first = threadIdx.x < A ? *(const uint16_t *)(in + kHdrBytes + 2ull * threadIdx.x) : 0;
  const uint64_t payload_bytes = bytes - payload_off;
  const uint8_t *dir = in + dir_off;
  const uint64_t o0 = ld64(dir + 8ull * k), o1 = ld64(dir + 8ull * k + 8);
  if (o0 > o1 || o1 > payload_bytes || o1 - o0 < 8ull * S || (o0 & 3)) {
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  const uint64_t ck_off = payload_off + o0;  // chunk start, from the start of the container
  const uint8_t *ck = in + ck_off;
  const uint64_t ck_bytes = o1 - o0;
  const uint64_t chunk_len = cs ? cs : len;
  const uint64_t base = (uint64_t)k * chunk_len;
  const uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
  const uint32_t *nwk = (const uint32_t *)(ck + 4ull * S);
  uint64_t pre_loc = 0;
  for (uint32_t i = threadIdx.x; i < g * NT; i += NT) pre_loc += nwk[i];
  const uint32_t j = g * NT + threadIdx.x;
  const bool live = j < S;
  const uint32_t nw_stored = live ? nwk[j] : 0;
  const uint32_t s_stored = live ? ((const uint32_t *)ck)[j] : kL;

  // ---- this work-group's streams
  const uint64_t pre = block_sum64<NT>(pre_loc, misc64);
  const uint64_t rows_full = n_here / S;
  const uint32_t rem_row = (uint32_t)(n_here - rows_full * S);
  const uint64_t n_j = live ? rows_full + (j < rem_row ? 1 : 0) : 0;
  uint32_t nw = nw_stored;
  bool bad = false;
  if (nw > n_j) {
    bad = true;
    nw = 0;
  }
  uint32_t tot;
  const uint32_t ex = block_excl_scan<NT>(nw, misc, &tot);
  const uint64_t w0 = pre + ex;  // index of this stream's first word inside the chunk
  if (8ull * S + 2 * (w0 + nw) > ck_bytes) {
    bad = true;
    nw = 0;
  }
  // where the stream's words are; its first two 16-byte blocks are requested now, so that their latency
  // overlaps the table build
  const uint64_t B0 = ck_off + 8ull * S + 2 * w0;  // first byte of the stream's words
  const uint64_t blk_base = B0 & ~15ull;           // 16-byte blocks are counted from here
  const uint8_t *sp = in + blk_base;
  const uint32_t pos0 = (uint32_t)(B0 & 15) >> 1;
  const uint32_t end16 = (uint32_t)(B0 - blk_base) + 2 * nw;  // stream end, in bytes from blk_base
  // bytes of the container from blk_base on (saturated): loads stay below this
  const uint64_t room = bytes > blk_base ? bytes - blk_base : 0;
  const uint32_t lim16 = room > 0xffffffffull ? 0xffffffffu : (uint32_t)room;
  auto load_block = [&](uint32_t off16) -> uint4 {  // 16 bytes at sp + off16; bytes past the end read as zero
    if (off16 <= lim16 && lim16 - off16 >= 16) return *(const uint4 *)(sp + off16);
    uint32_t w[4] = {0, 0, 0, 0};
    for (uint32_t q = 0; q < 8; q++)
      if ((uint64_t)off16 + 2 * q + 2 <= lim16) w[q >> 1] |= (uint32_t) * (const uint16_t *)(sp + off16 + 2 * q) << (16 * (q & 1));
    return make_uint4(w[0], w[1], w[2], w[3]);
  };
  uint4 q_first[2] = {make_uint4(0, 0, 0, 0), make_uint4(0, 0, 0, 0)};
  if (live) {
    q_first[0] = load_block(0);
    if (16 < end16) q_first[1] = load_block(16);
  }

  // ---- tables
  const float sc = (x_max - x_min) / (float)((1u << q_bits) - 1u);
  const float zf = eq6_zero_point(x_min, sc);
  for (uint32_t i = threadIdx.x; i < (total * sizeof(LutT) + 3) / 4; i += NT) ((uint32_t *)lut)[i] = 0;
  uint32_t carry = 0;
  for (uint32_t a0 = 0; a0 < A; a0 += NT) {  // also orders the zeroing above before the marks below
    const uint32_t a = a0 + threadIdx.x;
    const uint32_t f = a0 == 0 ? f_first : (a < A ? *(const uint16_t *)(in + kHdrBytes + 2ull * a) : 0);
    uint32_t tot;
    const uint32_t F = carry + block_excl_scan<NT>(f, misc, &tot);
    if (a < A) {
      tab[a] = make_uint2(f | (F << 16), sink.bits(a, sc, zf, x_min));
      if (f && F < total) lut[F] = (LutT)a;  // present symbols start at distinct slots
    }
    carry += tot;
  }
  if (carry != total) {  // uniform; an empty D never reaches this kernel
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  __syncthreads();
  {  // running maximum of the marks: each wave owns a contiguous share of the slots
    constexpr uint32_t V = 4 / sizeof(LutT);  // slots per 32-bit word
    constexpr uint32_t kIt = 4;               // words of a lane handled together (their scans do not depend on each other)
    const uint32_t per_wave = ((total + NW * 64 * V - 1) / (NW * 64 * V)) * 64 * V;
    const uint32_t lo = wave * per_wave;
    if (lo < total) {
      const uint32_t hi = lo + per_wave < total ? lo + per_wave : total;
      // symbol that owns slot lo: the largest a with F[a] <= lo
      uint32_t a_lo = 0, a_hi = A;
      while (a_hi - a_lo > 1) {
        const uint32_t mid = (a_lo + a_hi) >> 1;
        if ((tab[mid].x >> 16) <= lo) a_lo = mid;
        else a_hi = mid;
      }
      uint32_t run = a_lo;
      for (uint32_t b0 = lo; b0 < hi; b0 += 64 * V * kIt) {
        uint32_t e[kIt][V], inc[kIt];
#pragma unroll
        for (uint32_t it = 0; it < kIt; it++) {
          const uint32_t idx = b0 + it * 64 * V + lane * V;
          const uint32_t w = idx < hi ? ((const uint32_t *)lut)[idx / V] : 0;
#pragma unroll
          for (uint32_t q = 0; q < V; q++) e[it][q] = (w >> (8 * sizeof(LutT) * q)) & (sizeof(LutT) == 1 ? 0xffu : 0xffffu);
#pragma unroll
          for (uint32_t q = 1; q < V; q++) e[it][q] = e[it][q] > e[it][q - 1] ? e[it][q] : e[it][q - 1];
          inc[it] = wave_incl_max_scan(e[it][V - 1]);
        }
#pragma unroll
        for (uint32_t it = 0; it < kIt; it++) {
          const uint32_t idx = b0 + it * 64 * V + lane * V;
          // largest mark before this lane's word: the lane below's inclusive maximum, or the running one
          uint32_t prev = (uint32_t)__builtin_amdgcn_update_dpp((int)run, (int)inc[it], 0x138, 0xf, 0xf, false);  // wave_shr:1
          prev = prev > run ? prev : run;
          uint32_t sy[V];
#pragma unroll
          for (uint32_t q = 0; q < V; q++) sy[q] = e[it][q] > prev ? e[it][q] : prev;
          if (idx < hi) {
            if (WIDE) {  // straight to the slot table the coder reads
              uint2 te[V];
#pragma unroll
              for (uint32_t q = 0; q < V; q++) te[q] = tab[sy[q]];
#pragma unroll
              for (uint32_t q = 0; q < V; q++)
                if (idx + q < total) wide[idx + q] = make_uint2((te[q].x & 0xffffu) | ((idx + q - (te[q].x >> 16)) << 16), te[q].y);
            } else {
              uint32_t w = 0;
#pragma unroll
              for (uint32_t q = 0; q < V; q++) w |= sy[q] << (8 * sizeof(LutT) * q);
              ((uint32_t *)lut)[idx / V] = w;
            }
          }
          const uint32_t last = (uint32_t)__builtin_amdgcn_readlane((int)inc[it], 63);
          run = last > run ? last : run;
        }
      }
    }
  }
  __syncthreads();
  if (WIDE) __syncthreads();  // the scan scratch above may alias the window that is filled below
  if (live) {
    typedef __attribute__((address_space(3))) uint16_t lds_u16;
    constexpr uint32_t RB = kWinRowBytes, LOG_RB = NT == 1024 ? 11 : 9;
    // column of this stream inside a window row; lanes l and l+32 share a 32-bit bank word, so the two
    // halves of a wave never collide.  The window starts at LDS address 0 (this kernel has no static LDS).
    if ((uint32_t)(uintptr_t)(lds_u16 *)l_mem != 0) {  // cannot happen without static LDS; the slot arithmetic relies on it
      set_status(ctl, RANS_ERR_HIP);
      return;
    }
    const uint32_t lane_col = ((uint32_t)lane & 31u) * 2 + ((uint32_t)lane >> 5);
    const uint32_t colb = 2 * ((uint32_t)wave * 64 + lane_col);
    auto wread = [&](uint32_t rd_scaled) -> uint32_t {  // word whose number times RB is rd_scaled
      return *(lds_u16 *)(uintptr_t)((rd_scaled & (kWinBytes - 1)) | colb);
    };
    auto store_block = [&](uint32_t b, const uint4 &q) {  // block b -> rows 8(b&1) .. 8(b&1)+7
      lds_u16 *row0 = (lds_u16 *)(uintptr_t)(((b & 1u) * 8 * RB) | colb);
      const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
      for (int i = 0; i < 8; i++) row0[i * (RB / 2)] = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
    };
    // the first two blocks, requested before the table build
    store_block(0, q_first[0]);
    if (16 < end16) store_block(1, q_first[1]);
    uint32_t ldb = 2;              // next block to request
    uint32_t rd9 = pos0 * RB;      // RB times the number of the next unread word (counted from blk_base)
    uint32_t pend_b = 0;
    bool pending = false;
    uint4 pend_q = make_uint4(0, 0, 0, 0);
    uint32_t wnext = wread(rd9);
    uint32_t s = s_stored;
    uint32_t smin = s;
    auto *ob = sink.out + base + (uint64_t)g * NT;  // uniform base of this work-group's outputs
    constexpr uint32_t kOutElem = sizeof(*sink.out);
    uint32_t oi = threadIdx.x * kOutElem;           // byte offset of this stream's next output
    const uint32_t oi_step = S * kOutElem;
    // table addresses as plain LDS offsets (the window starts at 0, the slot table right after it)
    typedef __attribute__((address_space(3))) LutT lds_lut;
    typedef __attribute__((address_space(3))) uint64_t lds_u64;
    const uint32_t tab_off = (uint32_t)(uintptr_t)(lds_u64 *)tab;
    // Called every 8 steps (a step consumes at most one word).  The window holds blocks cur and cur + 1,
    // cur the block of the next unread word.  A block is requested two blocks ahead and moved into the
    // window once the block whose rows it takes (two blocks back) is read up.  Reading a block takes at
    // least 8 steps, so each block sees a call while it is being read: block b is requested during
    // block b - 2 at the latest and stored during block b - 1.
    auto refill = [&]() {
      const uint32_t cur = rd9 >> (LOG_RB + 3);
      if (pending && pend_b <= cur + 1) {
        store_block(pend_b, pend_q);
        pending = false;
      }
      if (!pending && ldb <= cur + 2 && ldb * 16 < end16) {
        pend_q = load_block(ldb * 16);
        pend_b = ldb;
        pending = true;
        ldb++;
      }
    };
    auto step = [&]() {
      const uint32_t slot = s & mask;
      uint2 e;
      uint32_t bias;  // slot - F
      if constexpr (WIDE) {
        const uint64_t e64 = *(lds_u64 *)(uintptr_t)(kWinBytes + slot * 8);
        e = make_uint2((uint32_t)e64, (uint32_t)(e64 >> 32));
        bias = e.x >> 16;
      } else {
        const uint32_t x = *(lds_lut *)(uintptr_t)(kWinBytes + slot * (uint32_t)sizeof(LutT));
        const uint64_t e64 = *(lds_u64 *)(uintptr_t)(tab_off + x * 8);
        e = make_uint2((uint32_t)e64, (uint32_t)(e64 >> 32));
        bias = slot - (e.x >> 16);
      }
      // f < 2^16 always; s >> M < 2^24 only when M >= 8
      s = (MUL24 ? __umul24(e.x & 0xffffu, s >> M) : (e.x & 0xffffu) * (s >> M)) + bias;
      sink.put(ob, oi, e.y);
      oi += oi_step;
      if (s < kL) {
        s = (s << 16) | wnext;
        rd9 += RB;
        wnext = wread(rd9);
      }
      smin = s < smin ? s : smin;
    };
    uint64_t t = 0;
    for (; t + 8 <= rows_full; t += 8) {
      refill();
#pragma unroll
      for (int u = 0; u < 8; u++) step();
    }
    if (t < rows_full || j < rem_row) {
      refill();
      for (; t < rows_full; t++) step();
      if (j < rem_row) step();
    }
    const uint32_t rd = rd9 >> LOG_RB;
    bad |= smin < kL || s != kL || rd - pos0 != nw;
    if (j == S - 1) {  // chunk size must be exactly header + words, padded to 4 bytes with zeros
      const uint64_t end = 8ull * S + 2 * (w0 + nw);
      if (((end + 3) & ~3ull) != ck_bytes) bad = true;
      else if (end != ck_bytes && *(const uint16_t *)(ck + end) != 0) bad = true;
    }
  }
  if (bad) set_status(ctl, RANS_ERR_CORRUPT);
}

// Decoder side of the modified CSR (Sec. 3.1: the cumulative sum of r is taken at decode time, then v is
// scattered).  Rows are cut into tiles of `tile_rows` rows; k_row_part sums r over each tile (and checks
// r[i] <= K), a single-work-group scan turns the sums into the index of each tile's first nonzero, and
// k_csr_to_dense rebuilds one tile per work-group in LDS and writes it out in the output type.
__global__ __launch_bounds__(kWG) void k_row_part(const uint16_t *r, uint32_t N, uint32_t K, uint32_t tile_rows,
                                                  uint32_t *part, CtlRef ctl) {
  __shared__ uint64_t sh64[kWG / 64];
  if (get_status(ctl) != 0) return;
  const uint32_t i0 = blockIdx.x * tile_rows;
  const uint32_t i1 = i0 + tile_rows < N ? i0 + tile_rows : N;
  uint64_t loc = 0;
  bool bad = false;
  for (uint32_t i = i0 + threadIdx.x; i < i1; i += kWG) {
    const uint32_t v = r[i];
    bad |= v > K;
    loc += v;
  }
  const uint64_t tot = block_sum64<kWG>(loc, sh64);
  if (bad || tot > 0xffffffffull) set_status(ctl, RANS_ERR_CORRUPT);
  if (threadIdx.x == 0) part[blockIdx.x] = (uint32_t)tot;
}

// One tile of rows: row offsets by a local scan of r, the tile zeroed in LDS, every nonzero of the tile
// placed (its row found by bisection of the local offsets) and checked (1 <= v < 2^Q, c < K, c strictly
// increasing inside a row), then the tile written out: as symbols, or dequantised (x = s (xhat - z)).
// D holds v, c, r as 16-bit symbols; part[] the exclusive scan of the tile sums, part[n_tiles] = their total.
template <typename OutT>
__global__ __launch_bounds__(kWG) void k_csr_to_dense(const uint16_t *D, const uint32_t *part, uint32_t N, uint32_t K,
                                                      uint32_t tile_rows, uint32_t q_bits, OutT *out, CtlRef ctl) {
  extern __shared__ __align__(16) uint32_t l_mem[];
  __shared__ uint32_t sh[kWG / 64];
  if (get_status(ctl) != 0) return;
  const uint32_t nnz = ctl->nnz;
  const uint32_t i0 = blockIdx.x * tile_rows;
  const uint32_t rows = i0 + tile_rows < N ? tile_rows : N - i0;
  uint32_t *roff = l_mem;                                          // rows + 1 local offsets
  uint8_t *dense = (uint8_t *)(l_mem + ((rows + 1 + 3) & ~3u));   // rows * K symbols
  const uint32_t base = part[blockIdx.x];
  const uint32_t n_tiles = gridDim.x;
  if (blockIdx.x == n_tiles - 1 && part[n_tiles] != nnz) {  // sum of r must be the number of nonzeros
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  const uint16_t *r = D + 2ull * nnz + i0;
  uint32_t carry = 0;
  for (uint32_t b0 = 0; b0 < rows; b0 += kWG) {
    const uint32_t i = b0 + threadIdx.x;
    const uint32_t v = i < rows ? r[i] : 0;
    uint32_t tot;
    const uint32_t ex = block_excl_scan<kWG>(v, sh, &tot);
    if (i < rows) roff[i] = carry + ex;
    carry += tot;
    __syncthreads();
  }
  if (threadIdx.x == 0) roff[rows] = carry;
  const uint32_t cells = rows * K;
  for (uint32_t i = threadIdx.x; i < (cells + 3) / 4; i += kWG) ((uint32_t *)dense)[i] = 0;
  __syncthreads();
  const uint32_t cnt_here = carry;
  if ((uint64_t)base + cnt_here > nnz) {  // uniform: the offsets would run past the stored nonzeros
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  bool bad = false;
  // A lane takes runs of eight consecutive nonzeros (their values and column indices come with one 16-byte
  // load each, 2-byte aligned: where c starts inside D depends on the number of nonzeros), two runs per step
  // with all loads issued first.  The row of a run's first nonzero is found by bisection of the local offsets,
  // the rows of the others by walking on from there.
  constexpr int kU = 2;
  const uint16_t *Dv = D + base, *Dc = D + (uint64_t)nnz + base;
  for (uint32_t m0 = 0; 8 * m0 < cnt_here; m0 += kWG * kU) {
    uint32_t vw[kU][4], cw[kU][4], cp[kU];
#pragma unroll
    for (int u = 0; u < kU; u++) {
      const uint32_t j = 8 * (m0 + u * kWG + threadIdx.x);
      cp[u] = 0;
#pragma unroll
      for (int k = 0; k < 4; k++) vw[u][k] = cw[u][k] = 0;
      if (j + 8 <= cnt_here) {
        __builtin_memcpy(vw[u], Dv + j, 16);
        __builtin_memcpy(cw[u], Dc + j, 16);
      } else {
#pragma unroll
        for (int k = 0; k < 8; k++) {
          if (j + k < cnt_here) {
            vw[u][k >> 1] |= (uint32_t)Dv[j + k] << (16 * (k & 1));
            cw[u][k >> 1] |= (uint32_t)Dc[j + k] << (16 * (k & 1));
          }
        }
      }
      if (j && j < cnt_here) cp[u] = Dc[j - 1];
    }
#pragma unroll
    for (int u = 0; u < kU; u++) {
      const uint32_t j0 = 8 * (m0 + u * kWG + threadIdx.x);
      if (j0 < cnt_here) {
        uint32_t lo = 0, hi = rows;  // largest local row with roff[row] <= j0 (roff[rows] = cnt_here > j0)
        while (hi - lo > 1) {
          const uint32_t mid = (lo + hi) >> 1;
          if (roff[mid] <= j0) lo = mid;
          else hi = mid;
        }
        uint32_t row = lo, row_beg = roff[lo], row_end = roff[lo + 1], prev_c = cp[u];
#pragma unroll
        for (int k = 0; k < 8; k++) {
          const uint32_t j = j0 + k;
          if (j < cnt_here) {
            while (j >= row_end) {  // ends: row_end of the last row is cnt_here > j
              row++;
              row_beg = row_end;
              row_end = roff[row + 1];
            }
            const uint32_t vv = (vw[u][k >> 1] >> (16 * (k & 1))) & 0xffffu, cc = (cw[u][k >> 1] >> (16 * (k & 1))) & 0xffffu;
            bool b = vv == 0 || vv >= (1u << q_bits) || cc >= K;
            if (j > row_beg && prev_c >= cc) b = true;
            if (b) bad = true;
            else dense[row * K + cc] = (uint8_t)vv;
            prev_c = cc;
          }
        }
      }
    }
  }
  if (bad) set_status(ctl, RANS_ERR_CORRUPT);
  __syncthreads();
  const float s = ctl->scale, zf = ctl->zero_point, x_min = ctl->x_min;
  OutT *o = out + (uint64_t)i0 * K;
  auto conv = [&](uint32_t sym) -> OutT {
    if constexpr (sizeof(OutT) == 1) {
      return (OutT)sym;
    } else {
      const float y = s == 0.0f ? x_min : s * ((float)sym - zf);
      if constexpr (sizeof(OutT) == 4) return y;
      else return __float2half_rn(y);
    }
  };
  // four cells per lane and step when the tile starts on a 4-cell boundary of a 16-byte aligned output
  const bool vec4 = (((uint64_t)i0 * K) & 3) == 0 && ((uintptr_t)out & 15) == 0;
  const uint32_t cells4 = vec4 ? cells / 4 : 0;
  for (uint32_t q = threadIdx.x; q < cells4; q += kWG) {
    const uint32_t w = ((const uint32_t *)dense)[q];
    struct alignas(4 * sizeof(OutT)) Quad { OutT a, b, c, d; };
    ((Quad *)o)[q] = Quad{conv(w & 0xffu), conv((w >> 8) & 0xffu), conv((w >> 16) & 0xffu), conv(w >> 24)};
  }
  for (uint32_t i = cells4 * 4 + threadIdx.x; i < cells; i += kWG) o[i] = conv(dense[i]);
}

// Inverse of Eq. 6 over a symbol array.  VEC: sixteen symbols per lane and step (both arrays 16-byte
// aligned); the tail and unaligned arrays go one symbol at a time.
template <typename OutT, bool VEC>
__global__ __launch_bounds__(kWG) void k_dequant(const uint8_t *sym, uint64_t n, const rans_qinfo *qi, CtlRef ctl,
                                                 OutT *out) {
  if (ctl && get_status(ctl) != 0) return;
  const float s = qi->scale, zf = qi->zero_point, x_min = qi->x_min;
  auto conv = [&](uint32_t a) -> OutT {
    const float y = s == 0.0f ? x_min : s * ((float)a - zf);
    if constexpr (sizeof(OutT) == 4) return y;
    else return __float2half_rn(y);
  };
  const uint64_t tid = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (uint64_t)gridDim.x * blockDim.x;
  uint64_t done = 0;
  if constexpr (VEC) {
    struct alignas(4 * sizeof(OutT)) Quad { OutT a, b, c, d; };
    const uint64_t nv = n / 16;
    for (uint64_t i = tid; i < nv; i += stride) {
      const uint4 w = ((const uint4 *)sym)[i];
      const uint32_t ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int k = 0; k < 4; k++)
        ((Quad *)out)[4 * i + k] = Quad{conv(ww[k] & 0xffu), conv((ww[k] >> 8) & 0xffu), conv((ww[k] >> 16) & 0xffu), conv(ww[k] >> 24)};
    }
    done = nv * 16;
  }
  for (uint64_t i = done + tid; i < n; i += stride) out[i] = conv(sym[i]);
}

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

// ------------------------------------------------------------------ instrumentation

// Optional per-kernel timing for benchmarks: when a kernel's bit is set in the
// mask, each of its launches is bracketed by a pair of HIP events recorded on the
// launch stream.  Off by default; the normal path records nothing.
enum KernelId {
  KID_MINMAX = 0, KID_QINFO, KID_QUANT_HIST, KID_SCAN, KID_CSR_COMPACT, KID_CSR_ROWS,
  KID_NORMALIZE, KID_ENCODE, KID_CHUNK_SCAN, KID_GATHER, KID_DEC_PREPARE, KID_DECODE, KID_ROW_SCAN,
  KID_CSR_EXPAND, KID_DEQUANT, KID_COUNT
};
const char *const kKernelNames[KID_COUNT] = {
    "k_minmax", "k_qinfo", "k_quant_hist", "k_scan_u32", "k_csr_compact", "k_csr_rows",
    "k_normalize", "k_encode", "k_chunk_scan", "k_gather", "k_dec_prepare", "k_decode", "k_row_part",
    "k_csr_to_dense", "k_dequant"};

struct ProfRecord {
  int kid;
  hipEvent_t a, b;
};
struct Profiler {
  uint64_t mask = 0;
  uint32_t every = 1;                 // bracket every n-th launch of an enabled kernel
  uint32_t seen[32] = {0};            // launches seen per kernel id since the last enable
  std::vector<ProfRecord> recs;   // records in use
  std::vector<ProfRecord> pool;   // event pairs ready for reuse
  std::mutex mu;
};
Profiler g_prof;

// Takes an event pair for launch `kid` if that launch is to be timed.
inline bool prof_take(int kid, ProfRecord *r) {
  if (!((g_prof.mask >> kid) & 1)) return false;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  if (g_prof.seen[kid]++ % g_prof.every != 0) return false;
  if (!g_prof.pool.empty()) {
    *r = g_prof.pool.back();
    g_prof.pool.pop_back();
  } else if (hipEventCreate(&r->a) != hipSuccess || hipEventCreate(&r->b) != hipSuccess) {
    return false;
  }
  r->kid = kid;
  return true;
}
inline void prof_keep(const ProfRecord &r) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.recs.push_back(r);
}

// ------------------------------------------------------------------ host side

// Kernel launch; a timed launch hands its event pair to the runtime, which stamps
// them with the begin and end of the kernel's execution on the device (the same
// interval a kernel trace reports), the stream is always the 5th macro argument.
#define PROF_LAUNCH(KID, KERNEL, GRID, BLOCK, LDS, STREAM, ...)                                \
  do {                                                                                         \
    ProfRecord prof_rec_{-1, nullptr, nullptr};                                                \
    if (prof_take(KID, &prof_rec_)) {                                                          \
      hipExtLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, STREAM, prof_rec_.a, prof_rec_.b, 0,     \
                            __VA_ARGS__);                                                      \
      prof_keep(prof_rec_);                                                                    \
    } else {                                                                                   \
      hipLaunchKernelGGL(KERNEL, GRID, BLOCK, LDS, STREAM, __VA_ARGS__);                       \
    }                                                                                          \
  } while (0)

#define LAUNCH_CHECK()                                  \
  do {                                                  \
    if (hipGetLastError() != hipSuccess) return RANS_ERR_HIP; \
  } while (0)

inline bool aligned_to(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

// Call numbers: process-wide, never 0 (a zeroed control block then never matches a call).
std::atomic<uint32_t> g_call_seq{0};
inline uint32_t next_seq() {
  uint32_t v = ++g_call_seq;
  if (v == 0) v = ++g_call_seq;
  return v;
}

inline uint32_t grid_for(uint64_t n, uint32_t per_block, uint32_t cap) {
  uint64_t g = (n + per_block - 1) / per_block;
  if (g < 1) g = 1;
  return (uint32_t)(g > cap ? cap : g);
}

// Index of the last of the counters behind L.chunk_words that a call starts from zero, and the tile counts among them.
inline uint32_t counter_words(const Layout &L) { return L.nc_max + L.n_pub + L.n_blk; }
inline uint32_t *tile_counts_of(const Layout &L, uint8_t *ws) {
  return L.n_blk ? (uint32_t *)(ws + L.chunk_words) + L.nc_max + 1 + L.n_pub : nullptr;
}

NormArgs norm_args(const rans_params &p, const Layout &L, uint8_t *ws, uint64_t n, uint8_t *d_stream, size_t cap) {
  return NormArgs{(const uint32_t *)(ws + L.cnt), L.cnt_rep, nullptr, (uint32_t *)(ws + L.fq), (uint2 *)(ws + L.enc_tab),
                  (uint4 *)(ws + L.enc_tab4), L.A, p, n, p.mode == RANS_MODE_CSR ? 0 : 1, d_stream, (uint64_t)cap};
}

// Extrema, Eq. 6, symbols and their histogram.  With `na` (dense mode, a container follows) the
// histogram kernel also builds the frequency table and the container header.
int launch_quantize(const void *d_x, uint64_t n, const rans_params &p, const Layout &L, uint8_t *ws, uint8_t *d_sym,
                    rans_qinfo *d_qinfo, hipStream_t st, uint32_t seq, const NormArgs *na) {
  const CtlRef ctl{(Ctl *)(ws + L.ctl), seq};
  uint32_t *cnt = (uint32_t *)(ws + L.cnt);
  uint32_t *cw_ = (uint32_t *)(ws + L.chunk_words);
  const uint32_t ncz_ = counter_words(L);
  const bool f16 = p.in_dtype == RANS_F16;
  const bool vec = aligned_to(d_x, 16) && aligned_to(d_sym, 8);
  const uint32_t V = vec ? (f16 ? 8 : 4) : 1;
  MinMaxPart *part = (MinMaxPart *)(ws + L.mm_part);
  uint32_t n_part = 0;
  if (n) {
    uint32_t g = n_part = grid_for(n, kWG * V * 4, kMaxParts);
    if (f16) {
      if (vec) PROF_LAUNCH(KID_MINMAX, (k_minmax<__half, true>), dim3(g), dim3(kWG), 0, st, (const __half *)d_x, (uint32_t)n, part, ctl, cnt, L.A * (1 + L.cnt_rep), cw_, ncz_);
      else PROF_LAUNCH(KID_MINMAX, (k_minmax<__half, false>), dim3(g), dim3(kWG), 0, st, (const __half *)d_x, (uint32_t)n, part, ctl, cnt, L.A * (1 + L.cnt_rep), cw_, ncz_);
    } else {
      if (vec) PROF_LAUNCH(KID_MINMAX, (k_minmax<float, true>), dim3(g), dim3(kWG), 0, st, (const float *)d_x, (uint32_t)n, part, ctl, cnt, L.A * (1 + L.cnt_rep), cw_, ncz_);
      else PROF_LAUNCH(KID_MINMAX, (k_minmax<float, false>), dim3(g), dim3(kWG), 0, st, (const float *)d_x, (uint32_t)n, part, ctl, cnt, L.A * (1 + L.cnt_rep), cw_, ncz_);
    }
    LAUNCH_CHECK();
  }
  if (!n) {  // empty tensor: only the bookkeeping and the (zero) quantiser parameters
    PROF_LAUNCH(KID_QINFO, k_qinfo, dim3(1), dim3(kBig), 0, st, ctl, part, n_part, p.q_bits, d_qinfo, cnt, L.A * (1 + L.cnt_rep), cw_, ncz_);
    LAUNCH_CHECK();
  }
  if (n) {
    uint32_t g = grid_for(n, QNT * V * kQIter, kQuantBlocks);
    int skip0 = p.mode == RANS_MODE_CSR;
    const int fold = na != nullptr;
    const NormArgs nav = na ? *na : NormArgs{};
    auto launch_qh = [&](auto csr_tag) {
      constexpr bool CSRV = decltype(csr_tag)::value;
      if (f16) {
        if (vec) PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<__half, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const __half *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, fold, nav, tile_counts_of(L, ws));
        else PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<__half, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const __half *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, fold, nav, tile_counts_of(L, ws));
      } else {
        if (vec) PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<float, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const float *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, fold, nav, tile_counts_of(L, ws));
        else PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<float, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const float *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, fold, nav, tile_counts_of(L, ws));
      }
    };
    if (skip0) launch_qh(std::true_type{});
    else launch_qh(std::false_type{});
    LAUNCH_CHECK();
  }
  return RANS_OK;
}

// Everything after the symbol histogram: CSR, table, coder, container.
int launch_encode_tail(const uint8_t *d_sym, uint64_t n, const rans_params &p, const Layout &L, uint8_t *ws,
                       uint8_t *d_stream, size_t cap, uint64_t *d_stream_bytes, hipStream_t st, uint32_t seq,
                       bool table_done) {
  const CtlRef ctl{(Ctl *)(ws + L.ctl), seq};
  uint32_t *cnt = (uint32_t *)(ws + L.cnt);
  const bool csr = p.mode == RANS_MODE_CSR;
  const uint32_t A = L.A, S = p.n_streams;
  const bool lds_hist = A <= kLdsHistMaxA;
  if (csr) {
    const int al = aligned_to(d_sym, 16);
    const uint32_t *blk = tile_counts_of(L, ws);  // counted by k_quant_hist
    uint32_t *row_end = (uint32_t *)(ws + L.row_end);
    if (n) {
      const uint32_t g_compact = L.n_blk < kCompactBlocks ? L.n_blk : kCompactBlocks;
      if (lds_hist)
        PROF_LAUNCH(KID_CSR_COMPACT, (k_csr_compact<true>), dim3(g_compact), dim3(kWG), A * 4, st, d_sym, (uint32_t)n, al,
                           (uint32_t)p.cols, blk, ws + L.v, (uint16_t *)(ws + L.c), row_end, cnt, A, L.n_blk, L.cnt_rep);
      else
        PROF_LAUNCH(KID_CSR_COMPACT, (k_csr_compact<false>), dim3(g_compact), dim3(kWG), 0, st, d_sym, (uint32_t)n, al,
                           (uint32_t)p.cols, blk, ws + L.v, (uint16_t *)(ws + L.c), row_end, cnt, A, L.n_blk, L.cnt_rep);
      LAUNCH_CHECK();
      uint32_t N = (uint32_t)p.rows;
      uint32_t g = (N + kWG - 1) / kWG;
      // few work-groups: each ends with additions to the same few addresses and a ticket; more only when a
      // lane would otherwise walk very many rows
      const uint32_t g_cap = N > (1u << 20) ? 512u : 128u;
      g = g > g_cap ? g_cap : g;
      const int fold = A <= kNormWaveA;  // one wave of the last work-group can build the table
      const NormArgs na = norm_args(p, L, ws, n, d_stream, cap);
      if (lds_hist)
        PROF_LAUNCH(KID_CSR_ROWS, (k_csr_rows<true>), dim3(g), dim3(kWG), A * 4, st, row_end, N, (uint16_t *)(ws + L.r), cnt, A, ctl, fold, na);
      else
        PROF_LAUNCH(KID_CSR_ROWS, (k_csr_rows<false>), dim3(g), dim3(kWG), 0, st, row_end, N, (uint16_t *)(ws + L.r), cnt, A, ctl, fold, na);
      LAUNCH_CHECK();
      table_done = fold != 0;
    }
  }
  if (!table_done) {  // else the histogram kernel has built the table
    NormArgs na_k = norm_args(p, L, ws, n, d_stream, cap);
    if (csr && n) na_k.n_rep = 0;  // k_csr_rows has folded the partial histograms
    PROF_LAUNCH(KID_NORMALIZE, k_normalize, dim3(1), dim3(kBig), 0, st, ctl, na_k);
    LAUNCH_CHECK();
  }
  const uint32_t groups = (S + kWG - 1) / kWG;
  const bool fused_gather = L.n_pub != 0;  // the encoder places its words itself: no k_chunk_scan / k_gather
  if (L.nc_max) {
    uint16_t *scratch = (uint16_t *)(ws + L.scratch);
    uint32_t *st_arr = (uint32_t *)(ws + L.st), *nw_arr = (uint32_t *)(ws + L.nw);
    uint32_t *cw = (uint32_t *)(ws + L.chunk_words);
    const uint2 *tab = (const uint2 *)(ws + L.enc_tab);
    const uint4 *tab4 = (const uint4 *)(ws + L.enc_tab4);
    const bool lds_tab = lds_hist;
    const bool mul24 = p.freq_bits >= 8;  // then floor(s/f) < 2^24 and both products fit the 24-bit multiplier
#define ENC_LAUNCH2(SRCT, SPLV, TABV, M24, FUSEV)                                                                 \
  PROF_LAUNCH(KID_ENCODE, (k_encode<SRCT, SPLV, TABV, M24, FUSEV>), dim3(L.nc_max * groups_e), dim3(kWG), lds_e, st, \
              src, tab, tab4, A, p.freq_bits, S, p.chunk_syms, ctl, scratch, L.capw, st_arr, nw_arr, cw, groups_e,      \
              cw + L.nc_max + 1, d_stream, (uint64_t)cap, d_stream_bytes, wide_e)
#define ENC_LAUNCH(SRCT, SPLV, TABV)                                                                              \
  do {                                                                                                            \
    const uint32_t groups_e = (S + kWG * SPLV - 1) / (kWG * SPLV);                                                \
    size_t lds_e = (TABV == 2 ? A * 16 : (TABV == 1 ? A * 8 : 0)) + kRingStride * kWG * SPLV + 64;                         \
    const int wide_e = SPLV == 1 && S % 64 == 0 && (csr || aligned_to(d_sym, 16));                                \
    if (wide_e) lds_e += csr ? (kWG / 64) * 2 * kStageRows2 * 128 + 16 : (kWG / 64) * 2 * kStageRows * 64;        \
    if (fused_gather && lds_e < kEncTileBytes) lds_e = kEncTileBytes;                                             \
    if (mul24) {                                                                                                  \
      if (fused_gather) ENC_LAUNCH2(SRCT, SPLV, TABV, true, true);                                                \
      else ENC_LAUNCH2(SRCT, SPLV, TABV, true, false);                                                            \
    } else {                                                                                                      \
      if (fused_gather) ENC_LAUNCH2(SRCT, SPLV, TABV, false, true);                                               \
      else ENC_LAUNCH2(SRCT, SPLV, TABV, false, false);                                                           \
    }                                                                                                             \
  } while (0)
    // One stream per lane: the hardware interleaves waves better than the compiler interleaves
    // several streams inside a lane, and the stream count rarely exceeds what the chip can hold.
    if (csr) {
      SrcCsr src{ws + L.v, (const uint16_t *)(ws + L.c), (const uint16_t *)(ws + L.r), 0};
      if (A <= kEncTab16MaxA) ENC_LAUNCH(SrcCsr, 1, 2);
      else if (lds_tab) ENC_LAUNCH(SrcCsr, 1, 1);
      else ENC_LAUNCH(SrcCsr, 1, 0);
    } else {
      SrcDense src{d_sym};
      ENC_LAUNCH(SrcDense, 1, 2);
    }
#undef ENC_LAUNCH
#undef ENC_LAUNCH2
    LAUNCH_CHECK();
  }
  if (fused_gather) return RANS_OK;
  const bool fused_scan = L.nc_max <= kFusedScanMax;
  if (!fused_scan) {
    PROF_LAUNCH(KID_CHUNK_SCAN, k_chunk_scan, dim3(1), dim3(kBig), 0, st, ctl, (uint32_t *)(ws + L.chunk_words), S,
                d_stream, (uint64_t)cap, d_stream_bytes);
    LAUNCH_CHECK();
  }
  {
    const uint32_t gg = L.nc_max ? L.nc_max * groups : 1;  // an empty D still needs its one directory entry
    if (fused_scan)
      PROF_LAUNCH(KID_GATHER, (k_gather<true>), dim3(gg), dim3(kWG), 0, st, ctl, (const uint16_t *)(ws + L.scratch),
                  L.capw, (const uint32_t *)(ws + L.st), (const uint32_t *)(ws + L.nw),
                  (const uint32_t *)(ws + L.chunk_words), S, groups, d_stream, (uint64_t)cap, d_stream_bytes);
    else
      PROF_LAUNCH(KID_GATHER, (k_gather<false>), dim3(gg), dim3(kWG), 0, st, ctl, (const uint16_t *)(ws + L.scratch),
                  L.capw, (const uint32_t *)(ws + L.st), (const uint32_t *)(ws + L.nw),
                  (const uint32_t *)(ws + L.chunk_words), S, groups, d_stream, (uint64_t)cap, d_stream_bytes);
    LAUNCH_CHECK();
  }
  return RANS_OK;
}

int check_common(const rans_params *p, uint64_t n, const void *d_ws, size_t ws_bytes, Layout *L) {
  int rc = check_params(p, n);
  if (rc) return rc;
  if (!d_ws || !aligned_to(d_ws, 256)) return RANS_ERR_ARG;
  *L = make_layout(*p, n);
  if (ws_bytes < L->total) return RANS_ERR_WORKSPACE;
  if ((uint64_t)L->nc_max * ((p->n_streams + kWG - 1) / kWG) > 0x7fffffffull) return RANS_ERR_ARG;
  return RANS_OK;
}

int header_from_bytes(const uint8_t *b, size_t nb, rans_header *h) {
  if (!b || !h) return RANS_ERR_ARG;
  if (nb < kHdrBytes) return RANS_ERR_CORRUPT;
  auto g16 = [&](size_t o) { return (uint32_t)b[o] | ((uint32_t)b[o + 1] << 8); };
  auto g32 = [&](size_t o) { return g16(o) | (g16(o + 2) << 16); };
  auto g64 = [&](size_t o) { return (uint64_t)g32(o) | ((uint64_t)g32(o + 4) << 32); };
  if (g32(0) != 0x31464952u || g16(4) != 1) return RANS_ERR_CORRUPT;
  memset(h, 0, sizeof(*h));
  h->p.mode = b[6];
  h->p.in_dtype = b[7];
  h->p.q_bits = b[8];
  h->p.freq_bits = b[9];
  if (g16(10) != 0) return RANS_ERR_CORRUPT;
  h->n_elems = g64(12);
  h->p.rows = g64(20);
  h->p.cols = g64(28);
  h->len_d = g64(36);
  h->alphabet = g32(44);
  h->p.n_streams = g32(48);
  h->p.chunk_syms = g32(52);
  h->n_chunks = g32(56);
  uint32_t u = g32(60);
  memcpy(&h->x_min, &u, 4);
  u = g32(64);
  memcpy(&h->x_max, &u, 4);
  for (size_t i = 68; i < kHdrBytes; i++)
    if (b[i]) return RANS_ERR_CORRUPT;
  return RANS_OK;
}

int validate_header(const rans_header *h) {
  if (h->n_elems > kMaxElems || h->p.rows > kMaxElems || h->p.cols > kMaxElems) return RANS_ERR_CORRUPT;
  if (check_params(&h->p, h->n_elems) != RANS_OK) return RANS_ERR_CORRUPT;
  if (!std::isfinite(h->x_min) || !std::isfinite(h->x_max) || h->x_min > h->x_max) return RANS_ERR_CORRUPT;
  if (h->alphabet != alphabet_of(h->p)) return RANS_ERR_CORRUPT;
  if (h->p.mode == RANS_MODE_DENSE) {
    if (h->len_d != h->n_elems) return RANS_ERR_CORRUPT;
  } else {
    if (h->len_d < h->p.rows || (h->len_d - h->p.rows) % 2 != 0) return RANS_ERR_CORRUPT;
    if ((h->len_d - h->p.rows) / 2 > h->n_elems) return RANS_ERR_CORRUPT;
  }
  if ((uint64_t)h->n_chunks != n_chunks_of(h->len_d, h->p.chunk_syms)) return RANS_ERR_CORRUPT;
  return RANS_OK;
}

// Shared body of rans_decode / rans_decompress.  out_kind: 0 symbols, 1 fp32, 2 fp16.
int decode_common(const uint8_t *d_stream, size_t stream_bytes, const rans_header *h_hdr, int out_kind, void *d_out,
                  uint64_t out_cap, rans_qinfo *d_qinfo, void *d_ws, size_t ws_bytes, hipStream_t st) {
  if (!d_stream || !aligned_to(d_stream, 16)) return RANS_ERR_ARG;
  rans_header h;
  if (h_hdr) {
    h = *h_hdr;
  } else {
    if (stream_bytes < kHdrBytes) return RANS_ERR_CORRUPT;
    uint8_t hb[kHdrBytes];
    if (hipMemcpyAsync(hb, d_stream, kHdrBytes, hipMemcpyDeviceToHost, st) != hipSuccess) return RANS_ERR_HIP;
    if (hipStreamSynchronize(st) != hipSuccess) return RANS_ERR_HIP;
    int rc = header_from_bytes(hb, kHdrBytes, &h);
    if (rc) return rc;
  }
  int rc = validate_header(&h);
  if (rc) return rc;
  const uint64_t n = h.n_elems;
  if (n > out_cap) return RANS_ERR_CAPACITY;
  if (n && !d_out) return RANS_ERR_ARG;
  Layout L;
  rc = check_common(&h.p, n, d_ws, ws_bytes, &L);
  if (rc) return rc;
  const uint32_t A = L.A, M = h.p.freq_bits, S = h.p.n_streams;
  const uint64_t payload_off = kHdrBytes + align_up((size_t)A * 2, 8) + 8 * ((uint64_t)h.n_chunks + 1);
  if (stream_bytes < payload_off) return RANS_ERR_CORRUPT;
  uint8_t *ws = (uint8_t *)d_ws;
  const uint32_t seq = next_seq();
  const CtlRef ctl{(Ctl *)(ws + L.ctl), seq};
  const uint32_t groups = (S + kWG - 1) / kWG;
  const bool csr = h.p.mode == RANS_MODE_CSR;
  const size_t lut_elem = A <= 256 ? 1 : 2;
  // work-group size of the fast decoder: 1024 lanes share one set of tables when a chunk has that many streams
  const uint32_t nt = S > 512 ? 1024u : 256u;
  const uint32_t groups_f = (S + nt - 1) / nt;
  const size_t win_b = 32 * (size_t)nt;
  const size_t tmp_b = align_up((size_t)lut_elem << M, 16) + 192 + (size_t)A * 8;  // [lut][misc][tab]
  const size_t lds_two = win_b + tmp_b;
  // wide table: 8 bytes per slot after the window; the build-time tables alias the window if they fit there
  const size_t wide_b = (size_t)8 << M;
  const bool tmp_alias = tmp_b <= win_b;
  const size_t lds_wide = win_b + wide_b + (tmp_alias ? 0 : tmp_b);
  const uint32_t tmp_off = (uint32_t)(tmp_alias ? 0 : win_b + wide_b);
  const size_t kLdsMax = 160 * 1024;
  // worth it when the table is shared by enough lanes: always up to 2^13 slots, at 2^14 only for 1024-lane groups
  const bool use_wide = lds_wide <= kLdsMax && (M <= 13 || nt == 1024);
  const size_t lds_fast = use_wide ? lds_wide : lds_two;
  // the fast decoder indexes a chunk's outputs and words with 32-bit offsets
  const bool small_chunk = L.chunk_len_max < (1ull << 29) && L.capw < (1u << 20);
  if (lds_fast <= kLdsMax && small_chunk) {
    // fast path: one small kernel for the header, one decode kernel that builds its tables in LDS
    HdrImage img;
    memset(&img, 0, sizeof(img));
    img.w[0] = 0x31464952u;
    img.w[1] = 1u | (h.p.mode << 16) | (h.p.in_dtype << 24);
    img.w[2] = h.p.q_bits | (M << 8);
    uint8_t *ib = (uint8_t *)img.w;
    memcpy(ib + 12, &h.n_elems, 8);
    memcpy(ib + 20, &h.p.rows, 8);
    memcpy(ib + 28, &h.p.cols, 8);
    memcpy(ib + 36, &h.len_d, 8);
    memcpy(ib + 44, &A, 4);
    memcpy(ib + 48, &h.p.n_streams, 4);
    memcpy(ib + 52, &h.p.chunk_syms, 4);
    memcpy(ib + 56, &h.n_chunks, 4);
    memcpy(ib + 60, &h.x_min, 4);
    memcpy(ib + 64, &h.x_max, 4);
    if (!h.n_chunks) {
      PROF_LAUNCH(KID_DEC_PREPARE, k_dec_begin, dim3(1), dim3(64), 0, st, d_stream, (uint64_t)stream_bytes, ctl, img, h,
                  d_qinfo);
      LAUNCH_CHECK();
    }
    if (h.n_chunks) {
      const dim3 grid(h.n_chunks * groups_f), blk(nt);
      const uint64_t dir_off = kHdrBytes + align_up((size_t)A * 2, 8);
#define FDEC_ARGS                                                                                            \
  d_stream, (uint64_t)stream_bytes, ctl, A, M, S, h.p.chunk_syms, groups_f, h.len_d, dir_off, payload_off, h.x_min, \
      h.x_max, h.p.q_bits, tmp_off, img, h, d_qinfo
#define FDEC_ONE(SINKT, LUTT, MULV, NTV, WIDEV, sinkv)                                                              \
  do {                                                                                                             \
    auto kfn = k_decode_fast<SINKT, LUTT, MULV, NTV, WIDEV>;                                                       \
    /* once per instantiation: allow dynamic LDS beyond the default 64 KB */                                       \
    static const hipError_t attr_rc =                                                                              \
        hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);          \
    if (lds_fast > 64 * 1024 && attr_rc != hipSuccess) return RANS_ERR_HIP;                                        \
    PROF_LAUNCH(KID_DECODE, kfn, grid, blk, lds_fast, st, FDEC_ARGS, sinkv);                                       \
  } while (0)
#define FDEC_LAUNCH(SINKT, LUTT, sinkv)                                                                            \
  do {                                                                                                             \
    if (use_wide) {                                                                                                \
      if (M >= 8 && nt == 1024) FDEC_ONE(SINKT, LUTT, true, 1024, true, sinkv);                                    \
      else if (M >= 8) FDEC_ONE(SINKT, LUTT, true, 256, true, sinkv);                                              \
      else if (nt == 1024) FDEC_ONE(SINKT, LUTT, false, 1024, true, sinkv);                                        \
      else FDEC_ONE(SINKT, LUTT, false, 256, true, sinkv);                                                         \
    } else {                                                                                                       \
      if (M >= 8 && nt == 1024) FDEC_ONE(SINKT, LUTT, true, 1024, false, sinkv);                                   \
      else if (M >= 8) FDEC_ONE(SINKT, LUTT, true, 256, false, sinkv);                                             \
      else if (nt == 1024) FDEC_ONE(SINKT, LUTT, false, 1024, false, sinkv);                                       \
      else FDEC_ONE(SINKT, LUTT, false, 256, false, sinkv);                                                        \
    }                                                                                                              \
  } while (0)
      if (csr) {
        FSinkU16 sk{(uint16_t *)(ws + L.D)};
        if (lut_elem == 1) FDEC_LAUNCH(FSinkU16, uint8_t, sk);
        else FDEC_LAUNCH(FSinkU16, uint16_t, sk);
      } else if (out_kind == 0) {
        FSinkSym sk{(uint8_t *)d_out};
        FDEC_LAUNCH(FSinkSym, uint8_t, sk);
      } else if (out_kind == 1) {
        FSinkFloat<float> sk{(float *)d_out};
        FDEC_LAUNCH(FSinkFloat<float>, uint8_t, sk);
      } else {
        FSinkFloat<__half> sk{(__half *)d_out};
        FDEC_LAUNCH(FSinkFloat<__half>, uint8_t, sk);
      }
#undef FDEC_LAUNCH
#undef FDEC_ONE
#undef FDEC_ARGS
      LAUNCH_CHECK();
    }
  } else {
  // generic path for tables that do not fit LDS: tables built once in global memory
  uint16_t *lut = (uint16_t *)(ws + L.dec_lut);
  uint32_t *tab = (uint32_t *)(ws + L.dec_tab);
  PROF_LAUNCH(KID_DEC_PREPARE, k_dec_prepare, dim3(1), dim3(kBig), 0, st, d_stream, (uint64_t)stream_bytes, ctl, h, lut, tab,
                     (uint32_t *)(ws + L.dec_F), d_qinfo);
  LAUNCH_CHECK();
  const size_t lds = (size_t)A * 4 + ((size_t)2 << M);
  const bool lds_tab = lds <= 48 * 1024;
  if (h.n_chunks) {
    dim3 grid(h.n_chunks * groups), blk(kWG);
#define DEC_LAUNCH(SINKT, sinkv)                                                                                   \
  do {                                                                                                             \
    if (lds_tab)                                                                                                   \
      PROF_LAUNCH(KID_DECODE, (k_decode<SINKT, true>), grid, blk, lds, st, d_stream, (uint64_t)stream_bytes, ctl, lut,   \
                         tab, A, M, S, h.p.chunk_syms, groups, sinkv);                                             \
    else                                                                                                           \
      PROF_LAUNCH(KID_DECODE, (k_decode<SINKT, false>), grid, blk, 0, st, d_stream, (uint64_t)stream_bytes, ctl, lut,    \
                         tab, A, M, S, h.p.chunk_syms, groups, sinkv);                                             \
  } while (0)
    if (csr) {
      SinkU16 sk{(uint16_t *)(ws + L.D)};
      DEC_LAUNCH(SinkU16, sk);
    } else if (out_kind == 0) {
      SinkSym sk{(uint8_t *)d_out};
      DEC_LAUNCH(SinkSym, sk);
    } else if (out_kind == 1) {
      SinkFloat<float> sk{(float *)d_out, 0, 0, 0};
      DEC_LAUNCH(SinkFloat<float>, sk);
    } else {
      SinkFloat<__half> sk{(__half *)d_out, 0, 0, 0};
      DEC_LAUNCH(SinkFloat<__half>, sk);
    }
#undef DEC_LAUNCH
    LAUNCH_CHECK();
  }
  }
  if (csr && n) {
    const uint32_t N = (uint32_t)h.p.rows, K = (uint32_t)h.p.cols;
    const uint64_t nnz = (h.len_d - N) / 2;
    const uint16_t *D = (const uint16_t *)(ws + L.D);
    // tile of rows per work-group: up to 16K cells, fewer for small tensors (so that there are about a thousand
    // tiles), at least one row (a row has at most 65535 cells)
    uint64_t cells = n / 1024;
    cells = cells < 2048 ? 2048 : (cells > kDenseTileCells ? kDenseTileCells : cells);
    uint32_t tile_rows = (uint32_t)(cells / K);
    tile_rows = tile_rows < 1 ? 1 : (tile_rows > 4096 ? 4096 : tile_rows);
    if (tile_rows >= 4) tile_rows &= ~3u;  // then every tile starts on a 4-cell boundary (vector stores)
    const uint32_t n_tiles = (N + tile_rows - 1) / tile_rows;
    uint32_t *part = (uint32_t *)(ws + L.row_off);  // n_tiles + 1 entries (n_tiles <= N)
    PROF_LAUNCH(KID_ROW_SCAN, k_row_part, dim3(n_tiles), dim3(kWG), 0, st, D + 2 * nnz, N, K, tile_rows, part, ctl);
    LAUNCH_CHECK();
    PROF_LAUNCH(KID_SCAN, k_scan_u32, dim3(1), dim3(kBig), 0, st, part, n_tiles);
    LAUNCH_CHECK();
    const size_t lds = (((size_t)tile_rows + 1 + 3) & ~(size_t)3) * 4 + (((size_t)tile_rows * K + 3) & ~(size_t)3);
    if (lds > 64 * 1024) {  // a single long row: allow dynamic LDS beyond the default 64 KB (once per instantiation)
      static const hipError_t a0 = hipFuncSetAttribute((const void *)k_csr_to_dense<uint8_t>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      static const hipError_t a1 = hipFuncSetAttribute((const void *)k_csr_to_dense<float>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      static const hipError_t a2 = hipFuncSetAttribute((const void *)k_csr_to_dense<__half>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      if (a0 != hipSuccess || a1 != hipSuccess || a2 != hipSuccess) return RANS_ERR_HIP;
    }
    if (out_kind == 0)
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<uint8_t>), dim3(n_tiles), dim3(kWG), lds, st, D, part, N, K, tile_rows,
                  h.p.q_bits, (uint8_t *)d_out, ctl);
    else if (out_kind == 1)
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<float>), dim3(n_tiles), dim3(kWG), lds, st, D, part, N, K, tile_rows,
                  h.p.q_bits, (float *)d_out, ctl);
    else
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<__half>), dim3(n_tiles), dim3(kWG), lds, st, D, part, N, K, tile_rows,
                  h.p.q_bits, (__half *)d_out, ctl);
    LAUNCH_CHECK();
  }
  return RANS_OK;
}


// ---- reshape search: host side

struct RsPlan {
  RsCands cands;
  RsOffsets offs;
  uint32_t n_entries, n_tiles;
  size_t mask16, lp, tile_cnt, zero0, hv, hc, hr, bad, costs, ticket, total;  // byte offsets in the workspace
  uint32_t zero_words;
  bool too_many;
};

uint64_t isqrt_u64(uint64_t t) {
  uint64_t r = (uint64_t)sqrt((double)t);
  while (r * r > t) r--;
  while ((r + 1) * (r + 1) <= t) r++;
  return r;
}

// Domain of Algorithm 1 in walk order (N descending = K ascending): K | T, K <= 2^Q, T/K > sqrt(T).
RsPlan rs_plan(uint64_t n, uint32_t q_bits) {
  RsPlan P{};
  const uint64_t two_q = 1ull << q_bits;
  const uint64_t n_sq = isqrt_u64(n) + 1, n_q = (n + two_q - 1) / two_q;
  const uint64_t n_min = n_sq > n_q ? n_sq : n_q;
  for (uint64_t K = 1; K <= two_q && K <= n; K++) {
    if (n % K) continue;
    if (n / K < n_min) break;
    if (P.cands.n == RANS_RESHAPE_MAX_CAND) {
      P.too_many = true;
      break;
    }
    P.cands.K[P.cands.n++] = (uint16_t)K;
  }
  uint32_t oc = 0, orr = 0;
  for (uint32_t k = 0; k < P.cands.n; k++) {
    P.offs.hc[k] = oc;
    P.offs.hr[k] = orr;
    oc += P.cands.K[k];
    orr += P.cands.K[k] + 1u;
  }
  P.offs.hc[P.cands.n] = oc;
  P.offs.hr[P.cands.n] = orr;
  P.n_entries = (uint32_t)((n + 15) / 16);
  P.n_tiles = (uint32_t)((n + kRsTile - 1) / kRsTile);
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align_up(o + bytes, 256);
    return at;
  };
  P.mask16 = take((size_t)P.n_entries * 2);
  P.lp = take((size_t)P.n_entries * 2);
  P.tile_cnt = take(((size_t)P.n_tiles + 1) * 4);
  P.zero0 = o;
  P.hv = take(256 * 4);
  P.hc = take((size_t)oc * 4 + 4);
  P.hr = take((size_t)orr * 4 + 4);
  P.bad = take(4);
  P.costs = take(RANS_RESHAPE_MAX_CAND * 8);
  P.ticket = take(4);
  P.zero_words = (uint32_t)((o - P.zero0) / 4);
  P.total = o;
  return P;
}

int launch_search_reshape(const uint8_t *d_sym, uint64_t n, uint32_t q_bits, rans_reshape_result *d_res, uint8_t *ws,
                          const RsPlan &P, hipStream_t st) {
  uint16_t *mask16 = (uint16_t *)(ws + P.mask16), *lp = (uint16_t *)(ws + P.lp);
  uint32_t *tile_cnt = (uint32_t *)(ws + P.tile_cnt);
  uint32_t *hv = (uint32_t *)(ws + P.hv), *hc = (uint32_t *)(ws + P.hc), *hr = (uint32_t *)(ws + P.hr);
  uint32_t *bad = (uint32_t *)(ws + P.bad);
  hipLaunchKernelGGL(k_rs_zero, dim3(8), dim3(256), 0, st, (uint32_t *)(ws + P.zero0), P.zero_words);
  LAUNCH_CHECK();
  hipLaunchKernelGGL(k_rs_mask, dim3(P.n_tiles < 1024 ? P.n_tiles : 1024), dim3(kWG), 0, st, d_sym, (uint32_t)n,
                     (int)aligned_to(d_sym, 16), P.n_tiles, mask16, lp, tile_cnt, hv, q_bits, bad);
  LAUNCH_CHECK();
  hipLaunchKernelGGL(k_scan_u32, dim3(1), dim3(kBig), 0, st, tile_cnt, P.n_tiles);
  LAUNCH_CHECK();
  const uint32_t g_e = grid_for(P.n_entries, kWG, 1024);
  for (uint32_t k0 = 0; k0 < P.cands.n;) {  // groups of candidates whose column bins fit in LDS together
    uint32_t k1 = k0 + 1;
    while (k1 < P.cands.n && P.offs.hc[k1 + 1] - P.offs.hc[k0] <= kRsColBins) k1++;
    hipLaunchKernelGGL(k_rs_cols, dim3(g_e), dim3(kWG), 0, st, mask16, P.n_entries, P.cands, k0, k1, P.offs, hc);
    LAUNCH_CHECK();
    k0 = k1;
  }
  if (P.cands.n) {
    hipLaunchKernelGGL(k_rs_rows, dim3(grid_for(n, kWG, 512), P.cands.n), dim3(kWG), 0, st, mask16, lp, tile_cnt,
                       (uint32_t)n, P.n_tiles, P.cands, P.offs, hr);
    LAUNCH_CHECK();
  }
  if (P.cands.n)
    hipLaunchKernelGGL(k_rs_cost, dim3(P.cands.n), dim3(kWG), 0, st, P.cands, (uint32_t)n, P.n_tiles, q_bits, tile_cnt, hv, hc,
                       hr, P.offs, bad, (double *)(ws + P.costs), (uint32_t *)(ws + P.ticket), d_res);
  else
    hipLaunchKernelGGL(k_rs_empty, dim3(1), dim3(1), 0, st, (uint32_t)n, bad, d_res);
  LAUNCH_CHECK();
  return RANS_OK;
}

}  // namespace

// ------------------------------------------------------------------ C ABI

extern "C" {

int rans_workspace_bytes(const rans_params *p, uint64_t n_elems, size_t *ws_bytes, size_t *max_stream_bytes) {
  int rc = check_params(p, n_elems);
  if (rc) return rc;
  Layout L = make_layout(*p, n_elems);
  if (ws_bytes) *ws_bytes = L.total;
  if (max_stream_bytes) *max_stream_bytes = stream_bound(*p, L);
  return RANS_OK;
}

int rans_quantize(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_sym, rans_qinfo *d_qinfo,
                  void *d_ws, size_t ws_bytes, void *stream) {
  Layout L;
  int rc = check_common(p, n_elems, d_ws, ws_bytes, &L);
  if (rc) return rc;
  if (!d_qinfo || (n_elems && (!d_x || !d_sym))) return RANS_ERR_ARG;
  if (!aligned_to(d_x, p->in_dtype == RANS_F16 ? 2 : 4) || !aligned_to(d_qinfo, 4)) return RANS_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  uint8_t *ws = (uint8_t *)d_ws;
  return launch_quantize(d_x, n_elems, *p, L, ws, d_sym, d_qinfo, st, next_seq(), nullptr);
}

int rans_encode(const uint8_t *d_sym, uint64_t n_elems, const rans_params *p, const rans_qinfo *d_qinfo,
                uint8_t *d_stream, size_t stream_cap, uint64_t *d_stream_bytes, void *d_ws, size_t ws_bytes,
                void *stream) {
  Layout L;
  int rc = check_common(p, n_elems, d_ws, ws_bytes, &L);
  if (rc) return rc;
  if (!d_qinfo || !d_stream || !d_stream_bytes || (n_elems && !d_sym)) return RANS_ERR_ARG;
  if (!aligned_to(d_stream, 16) || !aligned_to(d_stream_bytes, 8) || !aligned_to(d_qinfo, 4)) return RANS_ERR_ARG;
  if (stream_cap < kHdrBytes) return RANS_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)stream;
  uint8_t *ws = (uint8_t *)d_ws;
  const uint32_t seq = next_seq();
  const CtlRef ctl{(Ctl *)(ws + L.ctl), seq};
  PROF_LAUNCH(KID_QINFO, k_qinfo_from_user, dim3(1), dim3(kBig), 0, st, ctl, d_qinfo, p->q_bits,
              (uint32_t *)(ws + L.cnt), L.A * (1 + L.cnt_rep), (uint32_t *)(ws + L.chunk_words), counter_words(L));
  LAUNCH_CHECK();
  if (n_elems) {
    const bool vec = aligned_to(d_sym, 16);
    const uint32_t g = grid_for(n_elems, QNT * (vec ? 16 : 1) * kQIter, kQuantBlocks);
    const int skip0 = p->mode == RANS_MODE_CSR;
    const int fold = !skip0;  // dense: the histogram is complete after this kernel, which then builds the table
    const NormArgs na = norm_args(*p, L, ws, n_elems, d_stream, stream_cap);
    auto launch_qh = [&](auto csr_tag) {
      constexpr bool CSRV = decltype(csr_tag)::value;
      if (vec)
        PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<uint8_t, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, d_sym, (uint32_t)n_elems, ctl, p->q_bits, (uint8_t *)nullptr, (uint32_t *)(ws + L.cnt), skip0, (const MinMaxPart *)nullptr, 0u, (rans_qinfo *)nullptr, fold, na, tile_counts_of(L, ws));
      else
        PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<uint8_t, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, d_sym, (uint32_t)n_elems, ctl, p->q_bits, (uint8_t *)nullptr, (uint32_t *)(ws + L.cnt), skip0, (const MinMaxPart *)nullptr, 0u, (rans_qinfo *)nullptr, fold, na, tile_counts_of(L, ws));
    };
    if (skip0) launch_qh(std::true_type{});
    else launch_qh(std::false_type{});
    LAUNCH_CHECK();
  }
  return launch_encode_tail(d_sym, n_elems, *p, L, ws, d_stream, stream_cap, d_stream_bytes, st, seq,
                            n_elems && p->mode != RANS_MODE_CSR);
}

int rans_compress(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream, size_t stream_cap,
                  uint64_t *d_stream_bytes, void *d_ws, size_t ws_bytes, void *stream) {
  Layout L;
  int rc = check_common(p, n_elems, d_ws, ws_bytes, &L);
  if (rc) return rc;
  if (!d_stream || !d_stream_bytes || (n_elems && !d_x)) return RANS_ERR_ARG;
  if (!aligned_to(d_x, p->in_dtype == RANS_F16 ? 2 : 4)) return RANS_ERR_ARG;
  if (!aligned_to(d_stream, 16) || !aligned_to(d_stream_bytes, 8)) return RANS_ERR_ARG;
  if (stream_cap < kHdrBytes) return RANS_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)stream;
  uint8_t *ws = (uint8_t *)d_ws;
  const uint32_t seq = next_seq();
  const bool fold = n_elems && p->mode != RANS_MODE_CSR;  // dense: the histogram kernel also builds the table
  const NormArgs na = norm_args(*p, L, ws, n_elems, d_stream, stream_cap);
  rc = launch_quantize(d_x, n_elems, *p, L, ws, ws + L.sym, nullptr, st, seq, fold ? &na : nullptr);
  if (rc) return rc;
  return launch_encode_tail(ws + L.sym, n_elems, *p, L, ws, d_stream, stream_cap, d_stream_bytes, st, seq, fold);
}

int rans_decode(const uint8_t *d_stream, size_t stream_bytes, const rans_header *h_hdr, uint8_t *d_sym,
                uint64_t sym_cap, rans_qinfo *d_qinfo, void *d_ws, size_t ws_bytes, void *stream) {
  if (d_qinfo && !aligned_to(d_qinfo, 4)) return RANS_ERR_ARG;
  return decode_common(d_stream, stream_bytes, h_hdr, 0, d_sym, sym_cap, d_qinfo, d_ws, ws_bytes, (hipStream_t)stream);
}

int rans_decompress(const uint8_t *d_stream, size_t stream_bytes, const rans_header *h_hdr, uint32_t out_dtype,
                    void *d_x_out, uint64_t elem_cap, void *d_ws, size_t ws_bytes, void *stream) {
  if (out_dtype > RANS_F16) return RANS_ERR_ARG;
  if (!aligned_to(d_x_out, out_dtype == RANS_F16 ? 2 : 4)) return RANS_ERR_ARG;
  return decode_common(d_stream, stream_bytes, h_hdr, out_dtype == RANS_F16 ? 2 : 1, d_x_out, elem_cap, nullptr, d_ws,
                       ws_bytes, (hipStream_t)stream);
}

int rans_dequantize(const uint8_t *d_sym, uint64_t n_elems, const rans_qinfo *d_qinfo, uint32_t out_dtype,
                    void *d_x_out, void *stream) {
  if (!d_qinfo || out_dtype > RANS_F16 || n_elems > kMaxElems) return RANS_ERR_ARG;
  if (n_elems && (!d_sym || !d_x_out)) return RANS_ERR_ARG;
  if (!aligned_to(d_x_out, out_dtype == RANS_F16 ? 2 : 4) || !aligned_to(d_qinfo, 4)) return RANS_ERR_ARG;
  if (!n_elems) return RANS_OK;
  hipStream_t st = (hipStream_t)stream;
  const bool vec = aligned_to(d_sym, 16) && aligned_to(d_x_out, 16);
  const uint32_t g = grid_for(n_elems, kWG * 16, 8192);
  const CtlRef no_ctl{nullptr, 0};
  if (out_dtype == RANS_F32) {
    if (vec) PROF_LAUNCH(KID_DEQUANT, (k_dequant<float, true>), dim3(g), dim3(kWG), 0, st, d_sym, n_elems, d_qinfo, no_ctl, (float *)d_x_out);
    else PROF_LAUNCH(KID_DEQUANT, (k_dequant<float, false>), dim3(g), dim3(kWG), 0, st, d_sym, n_elems, d_qinfo, no_ctl, (float *)d_x_out);
  } else {
    if (vec) PROF_LAUNCH(KID_DEQUANT, (k_dequant<__half, true>), dim3(g), dim3(kWG), 0, st, d_sym, n_elems, d_qinfo, no_ctl, (__half *)d_x_out);
    else PROF_LAUNCH(KID_DEQUANT, (k_dequant<__half, false>), dim3(g), dim3(kWG), 0, st, d_sym, n_elems, d_qinfo, no_ctl, (__half *)d_x_out);
  }
  LAUNCH_CHECK();
  return RANS_OK;
}

int rans_peek_header(const void *h_bytes, size_t n_bytes, rans_header *out) {
  int rc = header_from_bytes((const uint8_t *)h_bytes, n_bytes, out);
  if (rc) return rc;
  return validate_header(out);
}

int rans_search_workspace_bytes(uint64_t n_elems, uint32_t q_bits, size_t *ws_bytes) {
  if (!ws_bytes || n_elems == 0 || n_elems > kMaxElems || q_bits < 1 || q_bits > 8) return RANS_ERR_ARG;
  const RsPlan P = rs_plan(n_elems, q_bits);
  if (P.too_many) return RANS_ERR_ARG;
  *ws_bytes = P.total;
  return RANS_OK;
}

int rans_search_reshape(const uint8_t *d_sym, uint64_t n_elems, uint32_t q_bits, rans_reshape_result *d_result,
                        void *d_ws, size_t ws_bytes, void *stream) {
  if (!d_sym || !d_result || !d_ws || n_elems == 0 || n_elems > kMaxElems || q_bits < 1 || q_bits > 8) return RANS_ERR_ARG;
  if (!aligned_to(d_ws, 256) || !aligned_to(d_result, 8)) return RANS_ERR_ARG;
  const RsPlan P = rs_plan(n_elems, q_bits);
  if (P.too_many) return RANS_ERR_ARG;
  if (ws_bytes < P.total) return RANS_ERR_WORKSPACE;
  return launch_search_reshape(d_sym, n_elems, q_bits, d_result, (uint8_t *)d_ws, P, (hipStream_t)stream);
}

int rans_last_status(const void *d_ws, void *stream) {
  if (!d_ws) return RANS_ERR_ARG;
  uint32_t w[3] = {0, 0, 0};  // status, status_seq, last_seq
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(w, d_ws, sizeof(w), hipMemcpyDeviceToHost, st) != hipSuccess) return RANS_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return RANS_ERR_HIP;
  return w[1] == w[2] ? (int32_t)w[0] : RANS_OK;  // an error of an older call is not this call's
}

int rans_profile_enable(uint64_t kernel_mask, uint32_t every) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  g_prof.mask = kernel_mask;
  g_prof.every = every ? every : 1;
  for (auto &c : g_prof.seen) c = 0;
  return RANS_OK;
}

int rans_profile_reset(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (auto &r : g_prof.recs) g_prof.pool.push_back(r);
  g_prof.recs.clear();
  return RANS_OK;
}

const char *rans_profile_kernel_name(int kernel_id) {
  return (kernel_id >= 0 && kernel_id < KID_COUNT) ? kKernelNames[kernel_id] : nullptr;
}

int rans_profile_read(int kernel_id, double *total_ms, uint64_t *count) {
  if (kernel_id < 0 || kernel_id >= KID_COUNT || !total_ms || !count) return RANS_ERR_ARG;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  double tot = 0;
  uint64_t n = 0;
  for (auto &r : g_prof.recs) {
    if (r.kid != kernel_id) continue;
    if (hipEventSynchronize(r.b) != hipSuccess) return RANS_ERR_HIP;
    float ms = 0;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return RANS_ERR_HIP;
    tot += ms;
    n++;
  }
  *total_ms = tot;
  *count = n;
  return RANS_OK;
}

const char *rans_strerror(int code) {
  switch (code) {
    case RANS_OK: return "ok";
    case RANS_ERR_ARG: return "invalid argument";
    case RANS_ERR_SHAPE: return "rows*cols != n_elems, or chunk_syms not a multiple of n_streams";
    case RANS_ERR_ALPHABET: return "more distinct symbols than 2^freq_bits, or CSR with cols > 65535";
    case RANS_ERR_CAPACITY: return "output buffer too small";
    case RANS_ERR_WORKSPACE: return "workspace too small";
    case RANS_ERR_NONFINITE: return "non-finite value in the tensor";
    case RANS_ERR_CORRUPT: return "corrupt container";
    case RANS_ERR_HIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

}  // extern "C"
