// rans_common.h -- constants, workspace layout, device helpers shared by all kernels
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

namespace {


constexpr uint32_t kL = 1u << 16;       // lower bound of the coder state interval [2^16, 2^32)
constexpr int kWG = 256;                // threads per work-group of the streaming kernels
constexpr int kBig = 1024;              // threads of the single-work-group kernels
constexpr uint32_t kHdrBytes = 128;
constexpr uint32_t kLdsHistMaxA = 8192; // alphabets up to this size keep histograms / tables in LDS
constexpr uint64_t kMaxElems = 1ull << 30;
constexpr uint32_t kFusedGatherMax = 16384;  // encoder work-groups up to which the encoder places its words itself
constexpr uint32_t kMaxParts = 512;     // work-groups (partial results) of the min/max kernel: two per compute unit read fastest

// ------------------------------------------------------------------ workspace

// Control block at the start of the workspace (device side).
struct Ctl {
  // {status, status_seq} form one 64-bit word: the first data-dependent error of call number
  // status_seq.  An entry of another call number counts as "no error", so nothing has to reset the
  // word when a call starts (and a kernel's work-groups need not wait for such a reset).
  int32_t status;
  uint32_t status_seq;
  uint32_t last_seq;                     // number of the latest call enqueued on this workspace
  uint32_t enc_exact;                    // every entry of the division-free encoder table is exact (see emit_entries)
  float x_min, x_max, scale, zero_point; // Eq. 6
  uint64_t len_d;                        // l_D of Eq. 7
  uint64_t payload_off, dir_off;         // container section offsets
  uint64_t total_bytes;
  uint32_t nnz, n_chunks;
  uint32_t hist_done;                    // not used (kept for the layout)
  uint32_t pad0;
  // First data-dependent error of ANY call on this workspace since the host last read it (rans_last_status):
  // kStickyTag in the upper 48 bits, minus the error code in the lower 16 (0 = none).  A word without the tag
  // is a workspace that has never recorded an error (fresh memory), so nothing has to initialise it.
  unsigned long long sticky;
  uint32_t pad[42];
};
static_assert(sizeof(Ctl) == 256, "control block is 256 bytes");
static_assert(offsetof(Ctl, sticky) == 80, "rans_last_status reads the sticky word at this offset");
constexpr unsigned long long kStickyTag = 0x52414e535354ull;  // "RANSST"

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
  // the counters behind `chunk_words` (32-bit words; everything before tc_off is zeroed when a call starts, and so
  // are the n_blk tile counts there): [0, nc_max] words per chunk, then n_pub published work-group totals, then -
  // at the even index acc_off - one 64-bit counter per chunk (fused placement only), then at tc_off the nonzeros
  // per CSR tile and per group of tiles
  uint32_t acc_off, tc_off;
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
  L.acc_off = (L.nc_max + 1 + L.n_pub + 1) & ~1u;
  L.tc_off = L.acc_off + (L.n_pub ? 2 * L.nc_max : 0);
  L.chunk_words = take(((size_t)L.tc_off + 2 * (size_t)L.n_blk) * 4);
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
// The same at the start of a kernel, where the errors of interest are those of the kernels before it: they
// ended before this one began, so an ordinary cached load sees them, and it returns several times sooner than
// the load above, which goes past the caches.
__device__ __forceinline__ int status_at_entry(const CtlRef &ctl) {
  const unsigned long long v = *(const unsigned long long *)&ctl.p->status;  // {status, status_seq}
  return (uint32_t)(v >> 32) == ctl.seq ? (int)(uint32_t)v : 0;
}
// Records `code` as the error of call ctl.seq unless that call already has one, and as the workspace's
// sticky error unless an earlier one is still waiting to be read.
__device__ __forceinline__ void set_status(const CtlRef &ctl, int code) {
  {
    unsigned long long *sw = &ctl.p->sticky;
    unsigned long long old = *(volatile unsigned long long *)sw;
    const unsigned long long want = (kStickyTag << 16) | (unsigned long long)(uint16_t)(-code);
    for (int tries = 0; tries < 64; tries++) {
      if ((old >> 16) == kStickyTag && (old & 0xffffu) != 0) break;  // an earlier error stays
      const unsigned long long prev = atomicCAS(sw, old, want);
      if (prev == old) break;
      old = prev;
    }
  }
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

// The status at entry as ONE value for a whole work-group (every thread must call it).  Another work-group
// of the running kernel may record an error at any moment; lanes that each read the word themselves could
// then disagree, and the ones that carry on would meet barriers and LDS slots the others never reach.
__device__ __forceinline__ bool group_has_status(const CtlRef &ctl) {
  return __syncthreads_or(status_at_entry(ctl) != 0) != 0;
}

// The same through an LDS word of the caller's (for kernels whose LDS layout must not gain a static variable,
// which the reduction above may bring in).  The word is free again when the function returns.
__device__ __forceinline__ bool group_has_status(const CtlRef &ctl, uint32_t *lds_word) {
  if (threadIdx.x == 0) *lds_word = status_at_entry(ctl) != 0;
  __syncthreads();
  const bool any = *lds_word != 0;
  __syncthreads();
  return any;
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
__device__ __forceinline__ uint64_t block_sum64(uint64_t v, uint64_t *sh /* NT/64 entries */) {
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
__device__ __forceinline__ uint64_t block_max64(uint64_t v, uint64_t *sh) {
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
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *sh /* NT/64 entries */, uint32_t *total) {
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

}  // namespace
