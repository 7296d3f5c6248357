// rans_decode.h -- rANS decoder (Eq. 3-4), CSR expand, dequantise
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

#include "rans_common.h"

namespace {

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
  if (group_has_status(ctl)) return;
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
  static constexpr bool kNarrow = true;  // the output value has at most 16 bits
  __device__ __forceinline__ uint32_t bits(uint32_t x, float, float, float) const { return x; }
  // byte_off is a byte offset from a wave-uniform base: the store can take the base from scalar
  // registers; non-temporal because the output is streamed once and must not evict the coded words
  __device__ __forceinline__ static void put(uint8_t *base, uint32_t byte_off, uint32_t b) {
    __builtin_nontemporal_store((uint8_t)b, base + byte_off);
  }
};
struct FSinkU16 {
  uint16_t *out;
  static constexpr bool kNarrow = true;
  __device__ __forceinline__ uint32_t bits(uint32_t x, float, float, float) const { return x; }
  __device__ __forceinline__ static void put(uint16_t *base, uint32_t byte_off, uint32_t b) {
    __builtin_nontemporal_store((uint16_t)b, (uint16_t *)((uint8_t *)base + byte_off));
  }
};
// Inverse of Eq. 6 fused into the decoder: x = s * (xhat - z), one value per symbol.
template <typename OutT>
struct FSinkFloat {
  OutT *out;
  static constexpr bool kNarrow = sizeof(OutT) <= 2;
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
// A stream's words are read through a 16-word window in LDS (one 32-byte line per
// stream): the lane loads 16-byte aligned blocks of its segment from global memory,
// a block goes into its half of the line with one 16-byte store, and the coder consumes
// single words from the line, keeping the next word in a register.  Refills happen at
// wave-uniform points, every eight steps: the block fetched at one check is written to
// LDS at a later one, and a block is requested as soon as the reader has entered the
// block before it.  A stream consumes at most one word per step and a block holds
// eight, so the words are always there in time, while the global loads have at least
// eight steps to complete.
//
// Everything taken from the container is checked before use; loads never leave the
// buffer, and the final state / word count of every stream is verified.
//
// WIDE: instead of the two dependent lookups slot -> symbol -> {f, F, output}, one 8-byte entry per slot
// {f | (slot - F) << 16, output bits} - or, for outputs of at most 16 bits, {f, output | (slot - F) << 16}, which
// saves the unpacking of f - (a 2^M x 8 B table): one LDS access on the state's dependency chain.
// The byte-per-slot table, the per-symbol table and the scan scratch are then only needed while the tables
// are built; they live at tmp_off, which may alias the window (not yet in use at that time).
template <class Sink, typename LutT, bool MUL24, int NT, bool WIDE>
__global__ __launch_bounds__(NT) void k_decode_fast(const uint8_t *in, uint64_t bytes, CtlRef ctl, uint32_t A,
                                                     uint32_t M, uint32_t S, uint32_t cs, uint32_t groups,
                                                     uint64_t len, uint64_t dir_off, uint64_t payload_off,
                                                     float x_min, float x_max, uint32_t q_bits, uint32_t tmp_off,
                                                     uint32_t misc_off, HdrImage img, rans_header hdr,
                                                     rans_qinfo *qout, Sink sink) {
  extern __shared__ __align__(16) uint32_t l_mem[];
  constexpr uint32_t kWinBytes = 32 * NT;             // 16-word window per stream, one 32-byte line each
  constexpr uint32_t NW = NT / 64;                    // waves per work-group
  // this is the first kernel of the call: no status to look at yet; work-group 0 checks the header
  if (blockIdx.x == 0 && threadIdx.x < 64) dec_check_header(in, bytes, ctl, img, hdr, qout);
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  const uint32_t total = 1u << M, mask = total - 1;
  // LDS: [window][lut][misc: 48 words][tab: A x 8 B], or WIDE: [window][wide table], [lut] at tmp_off and
  // [misc][tab] behind it or, with misc_off != 0, there (the tables of the build may lie over the window, which
  // is filled after the build).  The window and the table the coder reads sit at constant offsets, so their
  // addresses need no base arithmetic.
  LutT *lut = (LutT *)(l_mem + (WIDE ? tmp_off : kWinBytes) / 4);
  uint32_t *misc = (WIDE && misc_off) ? l_mem + misc_off / 4
                                      : (uint32_t *)lut + ((total * (uint32_t)sizeof(LutT) + 15) / 16) * 4;
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
                if (idx + q < total) {
                  const uint32_t fq = te[q].x & 0xffffu, bq = idx + q - (te[q].x >> 16);  // f, slot - F
                  wide[idx + q] = Sink::kNarrow ? make_uint2(fq, (te[q].y & 0xffffu) | (bq << 16)) : make_uint2(fq | (bq << 16), te[q].y);
                }
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
    // A stream's 16-word window is one 32-byte line of LDS: a block of eight words arrives with ONE 16-byte
    // store (the refill code is issued for the whole wave whenever any lane needs it, so its length counts
    // on every call), single words are read at 2 (n mod 16) inside the line.  rd9 is twice the number of the
    // next unread word.  The window starts at LDS address 0 (this kernel has no static LDS).
    constexpr uint32_t RB = 2, LOG_RB = 1;
    if ((uint32_t)(uintptr_t)(lds_u16 *)l_mem != 0) {  // cannot happen without static LDS; the slot arithmetic relies on it
      set_status(ctl, RANS_ERR_HIP);
      return;
    }
    const uint32_t colb = 32 * ((uint32_t)wave * 64 + (uint32_t)lane);
    auto wread = [&](uint32_t rd_scaled) -> uint32_t {  // word whose number times 2 is rd_scaled
      return *(lds_u16 *)(uintptr_t)((rd_scaled & 31u) | colb);
    };
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) u32x4 lds_u128;
    auto store_block = [&](uint32_t b, const uint4 &q) {  // block b -> words 8 (b & 1) .. 8 (b & 1) + 7 of the line
      *(lds_u128 *)(uintptr_t)(((b & 1u) * 16) | colb) = u32x4{q.x, q.y, q.z, q.w};
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
    // The state is at least 2^16 before every symbol if it is at the start: a step leaves f (s >> M) + (slot - F)
    // with f >= 1 (every slot of a table that sums to 2^M belongs to a present symbol) and s >> M >= 1, that is at
    // least 1, and a value below 2^16 is then shifted up by 16 bits.  So only the stored state needs the check.
    const bool s_low = s < kL;
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
      uint32_t fx;    // f
      if constexpr (WIDE) {
        const uint64_t e64 = *(lds_u64 *)(uintptr_t)(kWinBytes + slot * 8);
        e = make_uint2((uint32_t)e64, (uint32_t)(e64 >> 32));
        if constexpr (Sink::kNarrow) {  // {f, output | (slot - F) << 16}: f needs no unpacking, the store takes the low bits
          fx = e.x;
          bias = e.y >> 16;
        } else {
          fx = e.x & 0xffffu;
          bias = e.x >> 16;
        }
      } else {
        const uint32_t x = *(lds_lut *)(uintptr_t)(kWinBytes + slot * (uint32_t)sizeof(LutT));
        const uint64_t e64 = *(lds_u64 *)(uintptr_t)(tab_off + x * 8);
        e = make_uint2((uint32_t)e64, (uint32_t)(e64 >> 32));
        bias = slot - (e.x >> 16);
        fx = e.x & 0xffffu;
      }
      // f < 2^16 always; s >> M < 2^24 only when M >= 8
      s = (MUL24 ? __umul24(fx, s >> M) : fx * (s >> M)) + bias;
      sink.put(ob, oi, e.y);
      oi += oi_step;
      if (s < kL) {
        s = (s << 16) | wnext;
        rd9 += RB;
        wnext = wread(rd9);
      }
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
    bad |= s_low || s != kL || rd - pos0 != nw;
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
// r[i] <= K); the index of a tile's first nonzero is the sum of the tile sums before it, which the tile's
// work-group adds up itself (a single-work-group scan kernel does it when there are thousands of tiles), and
// k_csr_to_dense rebuilds one tile per work-group in LDS and writes it out in the output type.
__global__ __launch_bounds__(kWG) void k_row_part(const uint16_t *r, uint32_t N, uint32_t K, uint32_t tile_rows,
                                                  uint32_t n_tiles, uint32_t *part, CtlRef ctl) {
  // A wave per tile (a tile has at most 4096 rows): no barrier and no LDS, and a quarter of the work-groups.
  // The status word is read first and looked at after the counts: the two trips to memory overlap (r lies inside
  // D whatever an earlier kernel has found).
  const bool failed = status_at_entry(ctl) != 0;
  const uint32_t lane = threadIdx.x & 63u, tile = blockIdx.x * (kWG / 64) + (threadIdx.x >> 6);
  if (tile >= n_tiles) return;  // whole waves
  const uint32_t i0 = tile * tile_rows;
  const uint32_t i1 = i0 + tile_rows < N ? i0 + tile_rows : N;
  uint32_t loc = 0;  // at most 4096 counts below 2^16
  bool bad = false;
  // eight counts per lane and step (one 16-byte load, 2-byte aligned: r starts behind v and c), the tail one by one
  const uint32_t n8 = (i1 - i0) / 8;
  for (uint32_t q0 = lane; q0 < n8; q0 += 64 * 4) {  // four loads in flight
    uint32_t w[4][4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
#pragma unroll
      for (int k = 0; k < 4; k++) w[u][k] = 0;
      if (q0 + 64 * u < n8) __builtin_memcpy(w[u], r + i0 + 8 * (q0 + 64 * u), 16);
    }
#pragma unroll
    for (int u = 0; u < 4; u++) {
#pragma unroll
      for (int k = 0; k < 4; k++) {
        const uint32_t a = w[u][k] & 0xffffu, b = w[u][k] >> 16;
        bad |= a > K || b > K;
        loc += a + b;
      }
    }
  }
  for (uint32_t i = i0 + 8 * n8 + lane; i < i1; i += 64) {
    const uint32_t v = r[i];
    bad |= v > K;
    loc += v;
  }
  if (__ballot(failed) != 0) return;  // one decision for the wave
  const uint32_t tot = wave_incl_sum_scan(loc);
  if (bad) set_status(ctl, RANS_ERR_CORRUPT);
  if (lane == 63) part[tile] = tot;
}

// LDS of one tile of k_csr_to_dense, in bytes from the start of the dynamic allocation (the host sizes the
// launch with the same figures): the tile's non-empty rows in order, one bit per nonzero of the tile (set where
// a row begins), the number of set bits before each 32-bit word of that map, and the tile itself.
struct ExpandLds {
  uint32_t nerow, heads, wrank, dense, total;
};
__host__ __device__ inline ExpandLds expand_lds(uint32_t tile_rows, uint32_t K) {
  const uint32_t cells = tile_rows * K;                 // at most 65535 (checked by the host)
  const uint32_t nw = ((cells + 31) / 32 + 7) & ~7u;  // words of the map, a multiple of eight
  ExpandLds l;
  l.nerow = 0;
  l.heads = (2 * tile_rows + 15) & ~15u;
  l.wrank = l.heads + 4 * nw;
  l.dense = l.wrank + 2 * nw;
  l.total = l.dense + ((cells + 3) & ~3u);
  return l;
}

// One tile of rows, rebuilt in LDS and written out as symbols or dequantised (x = s (xhat - z)).
// D holds v, c, r as 16-bit symbols; part[] the exclusive scan of the tile sums with part[n_tiles] = their total
// (`scanned`), or - with few enough tiles that every work-group can add up the sums before its own - the tile
// sums themselves, which spares the scan kernel.  nnz is the number of nonzeros the header implies.
//
// The tile's nonzeros are j = 0 .. cnt-1 (cnt = sum of the tile's r).  A scan of r gives every non-empty row the
// index of its first nonzero and its rank among the non-empty rows; the row writes its number to nerow[rank] and
// sets bit j_first of `heads`.  The row of nonzero j is then nerow[(set bits of heads at or below j) - 1]: a
// lane that takes eight consecutive nonzeros needs the count of set bits before its byte of the map (wrank of the
// word plus a population count) and eight independent LDS reads - no search through row offsets and no walk from
// row to row, whose dependent LDS reads dominated an earlier form of this kernel.
// Checked here: 1 <= v < 2^Q, c < K, c strictly increasing inside a row (a nonzero that is not the first of its
// row must have a larger column than its predecessor), the tile sums against nnz.  r[i] <= K was checked by
// k_row_part, which is what keeps a tile's sum below 2^16.
// The loads of r, of the tile sums and - once the tile's first nonzero is known - of the first 16 kWG values and
// column indices are all issued before the scans that say how many of them the tile really has (reads past the
// tile's own nonzeros stay inside v and c: they are bounded by nnz).
template <typename OutT>
__global__ __launch_bounds__(kWG) void k_csr_to_dense(const uint16_t *D, const uint32_t *part, int scanned, uint32_t N,
                                                      uint32_t K, uint32_t tile_rows, uint32_t q_bits, uint32_t nnz,
                                                      OutT *out, CtlRef ctl) {
  extern __shared__ __align__(16) uint32_t l_mem[];
  __shared__ uint32_t sh[kWG / 64];
  __shared__ uint64_t sh64[kWG / 64];
  // Work-groups are handed to the compute units in the order of their numbers, and (almost) all of them are on
  // the chip at once.  The earlier ones of a unit get the higher wave priority: they reach their stores sooner,
  // so that writing starts while the later ones still place their nonzeros.
  {
    const uint32_t turn = blockIdx.x >> 9;  // two work-groups per unit and level, with 256 units
    if (turn == 0) __builtin_amdgcn_s_setprio(3);
    else if (turn == 1) __builtin_amdgcn_s_setprio(2);
    else if (turn == 2) __builtin_amdgcn_s_setprio(1);
  }
  const ExpandLds lay = expand_lds(tile_rows, K);
  uint16_t *nerow = (uint16_t *)((uint8_t *)l_mem + lay.nerow);
  uint32_t *heads = (uint32_t *)((uint8_t *)l_mem + lay.heads);
  uint16_t *wrank = (uint16_t *)((uint8_t *)l_mem + lay.wrank);
  uint8_t *dense = (uint8_t *)l_mem + lay.dense;
  const uint32_t i0 = blockIdx.x * tile_rows;  // below N: the grid has ceil(N / tile_rows) work-groups
  const uint32_t rows = i0 + tile_rows < N ? tile_rows : N - i0;
  const uint32_t cells = rows * K;
  const uint32_t n_tiles = gridDim.x;
  // the counts of the tile's rows: one per lane, or (more than kWG rows: at most 16 kWG, by the host's choice of
  // tile) sixteen consecutive ones per lane, two to a word
  constexpr int kRpt = 16;
  const uint16_t *r = D + 2ull * nnz + i0;
  const bool one_row = rows <= kWG;
  const uint32_t t0 = threadIdx.x * kRpt;
  uint32_t rw[kRpt / 2];
#pragma unroll
  for (int k = 0; k < kRpt / 2; k++) rw[k] = 0;
  if (one_row) {
    if (threadIdx.x < rows) rw[0] = r[threadIdx.x];
  } else if (t0 + kRpt <= rows) {
    __builtin_memcpy(rw, r + t0, 2 * kRpt);  // 2-byte aligned: r starts behind v and c
  } else {
#pragma unroll
    for (int k = 0; k < kRpt; k++)
      if (t0 + k < rows) rw[k >> 1] |= (uint32_t)r[t0 + k] << (16 * (k & 1));
  }
  // the map and the tile start at zero
  for (uint32_t i = threadIdx.x; i < (lay.wrank - lay.heads) / 4; i += kWG) heads[i] = 0;
  for (uint32_t i = threadIdx.x; i < (cells + 3) / 4; i += kWG) ((uint32_t *)dense)[i] = 0;
  uint64_t base64, total;
  if (scanned) {
    base64 = part[blockIdx.x];
    total = part[n_tiles];
  } else {
    uint64_t loc = 0;
    for (uint32_t u0 = threadIdx.x; u0 < blockIdx.x; u0 += 4 * kWG) {
      uint32_t x4[4];
#pragma unroll
      for (int k = 0; k < 4; k++) x4[k] = u0 + k * kWG < blockIdx.x ? part[u0 + k * kWG] : 0u;
#pragma unroll
      for (int k = 0; k < 4; k++) loc += x4[k];
    }
    base64 = loc;
    total = part[blockIdx.x];
  }
  if (group_has_status(ctl)) return;
  if (!scanned) {
    base64 = block_sum64<kWG>(base64, sh64);
    total += base64;  // of interest in the last work-group only
  }
  if ((blockIdx.x == n_tiles - 1 && total != nnz) || base64 > nnz) {  // sum of r must be the number of nonzeros
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  const uint32_t base = (uint32_t)base64;
  const uint32_t cap = nnz - base;  // nonzeros stored from the tile's first one on
  // A lane takes runs of eight consecutive nonzeros (their values and column indices come with one 16-byte
  // load each, 2-byte aligned: where c starts inside D depends on the number of nonzeros), two runs per step.
  // The first step's loads go out now.
  constexpr int kU = 2;
  const uint16_t *Dv = D + base, *Dc = D + (uint64_t)nnz + base;
  uint32_t vw[kU][4], cw[kU][4], cp[kU];
#pragma unroll
  for (int u = 0; u < kU; u++) {
    const uint32_t j = 8 * (u * kWG + threadIdx.x);
    cp[u] = 0;
#pragma unroll
    for (int k = 0; k < 4; k++) vw[u][k] = cw[u][k] = 0;
    if (j < cells && j + 8 <= cap) {
      __builtin_memcpy(vw[u], Dv + j, 16);
      __builtin_memcpy(cw[u], Dc + j, 16);
    }
    if (j && j < cells && j < cap) cp[u] = Dc[j - 1];
  }
  // scan of the counts, packed: nonzeros in the low half, non-empty rows in the high half (a tile has at most
  // 65535 cells, so neither sum leaves its half)
  uint32_t carry = 0;
  if (one_row) {
    const uint32_t v = rw[0];
    const uint32_t ex = block_excl_scan<kWG>(v | (v ? 0x10000u : 0u), sh, &carry);
    if (v) {
      nerow[ex >> 16] = (uint16_t)threadIdx.x;
      atomicOr(&heads[(ex & 0xffffu) >> 5], 1u << (ex & 31));
    }
  } else {
    uint32_t loc[kRpt], sum = 0;
#pragma unroll
    for (int k = 0; k < kRpt; k++) {
      const uint32_t v = (rw[k >> 1] >> (16 * (k & 1))) & 0xffffu;
      loc[k] = sum;
      sum += v | (v ? 0x10000u : 0u);
    }
    const uint32_t ex = block_excl_scan<kWG>(sum, sh, &carry);
    // consecutive rows mostly begin inside the same word of the map: one atomic per word
    uint32_t cur = 0, acc = 0;
#pragma unroll
    for (int k = 0; k < kRpt; k++) {
      const uint32_t v = (rw[k >> 1] >> (16 * (k & 1))) & 0xffffu;
      if (v) {
        const uint32_t q = ex + loc[k], wd = (q & 0xffffu) >> 5;
        nerow[q >> 16] = (uint16_t)(t0 + k);
        if (wd != cur) {
          if (acc) atomicOr(&heads[cur], acc);
          cur = wd;
          acc = 0;
        }
        acc |= 1u << (q & 31);
      }
    }
    if (acc) atomicOr(&heads[cur], acc);
  }
  const uint32_t cnt_here = carry & 0xffffu;
  if (cnt_here > cap) {  // uniform: the tile's nonzeros would run past the stored ones
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_CORRUPT);
    return;
  }
  __syncthreads();
  {
    // set bits of the map before each of its words: eight words per lane, one scan over the lanes
    const uint32_t nw = (cnt_here + 31) >> 5, w0 = threadIdx.x * 8;
    uint32_t pc[8], sum = 0;
#pragma unroll
    for (int k = 0; k < 8; k++) pc[k] = 0;
    if (w0 < nw) {
      const uint4 a = *(const uint4 *)(heads + w0), b = *(const uint4 *)(heads + w0 + 4);
      const uint32_t hw[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
      for (int k = 0; k < 8; k++) {
        pc[k] = sum;
        sum += __popc(hw[k]);
      }
    }
    uint32_t tot;
    const uint32_t ex = block_excl_scan<kWG>(sum, sh, &tot);
    if (w0 < nw)
      *(uint4 *)(wrank + w0) = make_uint4((ex + pc[0]) | ((ex + pc[1]) << 16), (ex + pc[2]) | ((ex + pc[3]) << 16),
                                          (ex + pc[4]) | ((ex + pc[5]) << 16), (ex + pc[6]) | ((ex + pc[7]) << 16));
  }
  __syncthreads();
  bool bad = false;
  for (uint32_t m0 = 0; 8 * m0 < cnt_here; m0 += kWG * kU) {
#pragma unroll
    for (int u = 0; u < kU; u++) {
      const uint32_t j = 8 * (m0 + u * kWG + threadIdx.x);
      if (m0) {  // later steps (a tile with more than 16 kWG nonzeros) load here
        cp[u] = 0;
#pragma unroll
        for (int k = 0; k < 4; k++) vw[u][k] = cw[u][k] = 0;
        if (j < cnt_here && j + 8 <= cap) {
          __builtin_memcpy(vw[u], Dv + j, 16);
          __builtin_memcpy(cw[u], Dc + j, 16);
        }
        if (j < cnt_here) cp[u] = Dc[j - 1];
      }
      if (j < cnt_here && j + 8 > cap) {  // the last few nonzeros of all: one by one
#pragma unroll
        for (int k = 0; k < 8; k++) {
          if (j + k < cnt_here) {
            vw[u][k >> 1] |= (uint32_t)Dv[j + k] << (16 * (k & 1));
            cw[u][k >> 1] |= (uint32_t)Dc[j + k] << (16 * (k & 1));
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kU; u++) {
      const uint32_t j0 = 8 * (m0 + u * kWG + threadIdx.x);
      if (j0 < cnt_here) {
        const uint32_t word = heads[j0 >> 5], sft = j0 & 31;
        const uint32_t first8 = (word >> sft) & 0xffu;
        uint32_t rank = wrank[j0 >> 5] + __popc(word & ((1u << sft) - 1u));  // rows begun before j0
        uint32_t prev_c = cp[u];
#pragma unroll
        for (int k = 0; k < 8; k++) {
          if (j0 + k < cnt_here) {
            const bool head = (first8 >> k) & 1u;
            rank += head;
            // rank >= 1: the tile's first nonzero begins a row (the guard only keeps the read inside nerow)
            const uint32_t row = nerow[(rank ? rank : 1u) - 1u];
            const uint32_t vv = (vw[u][k >> 1] >> (16 * (k & 1))) & 0xffffu, cc = (cw[u][k >> 1] >> (16 * (k & 1))) & 0xffffu;
            bool b = vv == 0 || vv >= (1u << q_bits) || cc >= K || row >= rows;
            if (!head && prev_c >= cc) b = true;
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
  if (ctl && group_has_status(ctl)) return;
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

}  // namespace
