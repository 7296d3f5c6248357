// rans_encode.h -- interleaved rANS encoder (Eq. 2) and the placement of its words in the container
//
// Part of the one translation unit rans_if.hip (included there, in this order); not a stand-alone header.
#pragma once

#include "rans_csr.h"

namespace {

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
  if (group_has_status(ctl, l_mem)) {  // through the dynamic LDS: this kernel must not have static LDS (see below)
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
  if (group_has_status(ctl)) {
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
  if (group_has_status(ctl)) {
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

}  // namespace
