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

constexpr int kStageRows = 16;         // rows per register tile of the encoder's symbol staging (dense source); LDS holds as many per wave
constexpr int kStageRows2 = 16;        // the same for the CSR source (16-bit entries)
constexpr uint32_t kEncTab16MaxA = 1024;  // CSR alphabets up to this size use the 16-byte table entries
constexpr int kEncAhead = 8;  // rows of symbols fetched ahead of the coder; also the period of the word area's overflow check
constexpr uint32_t kEncGuard = 16;     // unused LDS bytes below the first stream's word area

// Words a stream can keep in LDS: rw slots of 16 bits in an area of 2 rw + 4 bytes.  rw is a multiple of 16, so
// the distance between the areas of adjacent streams is an odd number of 32-bit words and the lanes of a wave
// that write the same slot number hit 64 different banks.
__host__ __device__ inline uint32_t enc_area_stride(uint32_t rw) { return 2 * rw + 4; }

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

// Interleaved rANS encoder (Eq. 2 with 16-bit renormalisation).  One work-group codes kWG streams of one
// chunk, one stream per lane (the hardware interleaves waves better than the compiler interleaves several
// streams inside a lane).
//
// Symbols are taken last to first in batches of kEncAhead rows, fetched ahead of the coder (through a
// per-wave LDS stage filled with 16-byte loads two tiles ahead), table entries looked up three rows ahead.
// The per-row arithmetic is branch-free (selects only) so that it stays one basic block.  floor(s / f) of
// Eq. 2 is a multiply-high and a shift with the per-symbol multiplier that the table build proved exact (table
// form 2, when every entry is exact), else a multiply-high with floor(2^32 / f) plus one correction step.
//
// Emitted words stay in LDS: every stream has an area of rw 16-bit slots, filled from its top slot downwards
// (ascending address = descending word number, the order the decoder reads).  The low half of the state is
// written to the next slot on every step and the slot pointer moves only when the renormalisation fires, so a
// slot keeps being rewritten until it is really used.  Most streams of a chunk fit their area.  One that
// does not - checked after every kEncAhead rows, a wave-uniform point - moves its complete 8-word blocks,
// oldest first, as 16-byte blocks to scratch in global memory (block-major per work-group: lanes that spill
// the same block number write adjacent memory) and its few remaining words to the top of the area.
//
// FUSE: the work-group also moves its streams' words to their place in the container (what k_gather does
// otherwise).  It adds its word total to its chunk's counter and publishes it for the later groups of the
// chunk, waits until every earlier chunk is complete and every earlier group of its own chunk has published
// (those work-groups were dispatched earlier and never wait for a higher index, so the wait ends; it is bounded
// all the same and turns into RANS_ERR_HIP if the bound is hit), and derives the chunk's byte offset and its
// own position inside the chunk from those totals: one load per chunk instead of one per work-group, all of
// a lane's loads independent of each other.  Its words then go straight from the areas to their place in the
// container (eight lanes per stream, 16-byte pieces to addresses that are only 2-byte aligned, a tail of 4-, 2-
// and 1-word stores), and the blocks of the streams that spilled from scratch, 16 bytes at a time.
// Without FUSE everything is spilled to scratch at the end, in the block format k_gather reads.
constexpr int kSpinMax = 1 << 18;
constexpr uint64_t kChunkWordsMask = (1ull << 40) - 1;  // chunk counter: words below, finished groups above
__device__ __forceinline__ uint32_t wait_published(const uint32_t *pub, uint32_t i, const CtlRef &ctl) {
  for (int spins = 0; spins < kSpinMax; spins++) {
    const uint32_t v = __hip_atomic_load(pub + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (v) return v;
    if ((spins & 255) == 255 && get_status(ctl) != 0) return 0;
    __builtin_amdgcn_s_sleep(4);
  }
  return 0;
}
// Words of chunk c once all of its `groups` work-groups have added theirs; ~0 if the wait gives up.
__device__ __forceinline__ uint64_t wait_chunk(const unsigned long long *acc, uint32_t c, uint32_t groups, const CtlRef &ctl) {
  for (int spins = 0; spins < kSpinMax; spins++) {
    const unsigned long long v = __hip_atomic_load(acc + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((uint32_t)(v >> 40) == groups) return v & kChunkWordsMask;
    if ((spins & 255) == 255 && get_status(ctl) != 0) return ~0ull;
    __builtin_amdgcn_s_sleep(4);
  }
  return ~0ull;
}

// Sixteen bytes at an address that is only 2-byte aligned, moved to or from registers in one access.
struct __attribute__((packed, aligned(2))) Block16 { uint32_t x, y, z, w; };

template <class Src, int TAB, bool MUL24, bool FUSE>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu(4))) void k_encode(
    Src src, const uint2 *g_tab, const uint4 *g_tab4, uint32_t A, uint32_t M, uint32_t S, uint32_t cs, CtlRef ctl,
    uint16_t *scratch, uint32_t capw, uint32_t *st_out, uint32_t *nw_out, uint32_t *chunk_words, uint32_t groups,
    uint32_t *wg_pub, unsigned long long *chunk_acc, uint8_t *out, uint64_t cap, uint64_t *d_stream_bytes, int wide,
    uint32_t rw, uint32_t wgs_per_class, uint32_t n_classes, int build_tab, NormArgs na) {
  extern __shared__ __align__(16) uint32_t l_mem[];  // the only LDS of this kernel, so the word areas start at offset kEncGuard
  const uint32_t k = blockIdx.x / groups, g = blockIdx.x % groups;
  // every exit publishes a total (0 words), or the work-groups behind this one would wait for it
  auto bail = [&]() {
    if (FUSE && threadIdx.x == 0) {
      __hip_atomic_store(wg_pub + blockIdx.x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(chunk_acc + k, 1ull << 40, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  if (group_has_status(ctl, l_mem)) {  // through the dynamic LDS: this kernel must not have static LDS (see below)
    if (FUSE && blockIdx.x == 0 && threadIdx.x == 0 && d_stream_bytes) *d_stream_bytes = 0;
    bail();
    return;
  }
  // The grid is sized for the longest D the tensor could have (in CSR mode the host does not know the number of
  // nonzeros): a work-group whose chunk does not exist leaves before the table build, not after it.  l_D is
  // known here - the CSR kernels stored it - and with it the number of chunks.
  // (A dense grid has exactly one work-group per part of a chunk: nothing to leave, and no load to wait for.)
  if (!std::is_same<Src, SrcDense>::value) {
    const uint64_t len_pre = ctl->len_d;
    uint32_t nc_pre = len_pre ? 1u : 0u;
    if (len_pre && cs) {
      const uint32_t qc = (uint32_t)len_pre / cs;  // l_D < 2^32
      nc_pre = qc + ((uint32_t)len_pre - qc * cs != 0);
    }
    if (k >= nc_pre && blockIdx.x != 0) {  // the first work-group stays: it writes the header whatever l_D is
      bail();
      return;
    }
  }
  const uint32_t sh_lim = 32 - M, totalM = 1u << M;
  // LDS: [guard][word areas][table][reduction scratch][symbol stage].  The areas come first so that a slot
  // address is the lane's fixed base plus twice the slot number; what follows them is reused as the tile of
  // the fused placement once the coding is over.
  const uint32_t stride = enc_area_stride(rw);
  const uint32_t areas_end = kEncGuard + stride * kWG;  // a multiple of 16
  uint32_t *l_tab = l_mem + areas_end / 4;
  uint32_t *sh = l_tab + (TAB == 2 ? A * 4 : (TAB == 1 ? A * 2 : 0));  // 4 + 8 words for the final reductions
  // Frequency table (Sec. 3.2's normalisation) and container geometry.  build_tab (alphabets that one wave
  // can normalise): D's histogram is complete, because the kernels that counted have ended, and every
  // work-group derives the same table from it for itself, straight into its LDS.  That is about three
  // microseconds of one wave per work-group; a hand-over from the last counting work-group, or a launch of
  // its own for the table, costs the call as much or more and needs ordering between work-groups that this
  // does not.  The first work-group also writes the header and the table of the container.  Otherwise
  // k_normalize has left tables and geometry in memory.
  uint32_t nc, exact_tab;
  uint64_t len, dir_off, payload_off;
  if (TAB == 2 && build_tab) {
    uint2 *const l_tab8 = (uint2 *)(sh + 16);  // {floor(2^32/f), f | F << 16}: in the stage, which is free until the coding
    uint32_t *const l_cnt = (uint32_t *)(l_tab8 + A);
    {  // the counts, partial histograms summed, with all of a lane's loads in flight together
      constexpr uint32_t kParts = kCntRep + 1;  // n_rep is 0 or kCntRep
      for (uint32_t a = threadIdx.x; a < A; a += kWG) {
        uint32_t c[kParts];
#pragma unroll
        for (uint32_t q = 0; q < kParts; q++) c[q] = q <= na.n_rep ? na.cnt[(size_t)q * A + a] : 0u;
        uint32_t t = 0;
#pragma unroll
        for (uint32_t q = 0; q < kParts; q++) t += c[q];
        l_cnt[a] = t;
      }
      __syncthreads();
    }
    if constexpr (std::is_same<Src, SrcDense>::value) {
      // While the first wave builds the table the others touch the lines that the coder asks for first (the
      // last 32 rows of the chunk, which is coded from its end), so that they come from the cache by then.
      // A wave's 64-byte column shares its 128-byte lines with the neighbouring wave's.
      if (wide && threadIdx.x >= 64) {
        const uint64_t cl = cs ? cs : na.n_elems, b0 = (uint64_t)k * cl;
        if (b0 < na.n_elems) {
          const uint64_t nh = na.n_elems - b0 < cl ? na.n_elems - b0 : cl, rows = nh / S;
          const uint32_t ln = threadIdx.x & 63;
          const uint8_t *colp = src.bytes() + b0 + (g * kWG + (threadIdx.x - ln)) + 16 * (ln & 3);
          uint32_t acc = 0;
#pragma unroll
          for (uint32_t u = 1; u <= 2; u++)
            if (rows >= 16 * u) acc ^= *(const uint32_t *)(colp + (rows - 16 * u + (ln >> 2)) * S);
          if (acc == 0x9e3779b9u && wide == 0x7fffffff) l_mem[1] = acc;  // never true: keeps the loads
        }
      }
    }
    NormArgs nl = na;  // a copy in registers: the argument itself cannot be changed in place
    nl.lds_cnt = l_cnt;
    nl.enc_tab = l_tab8;
    nl.enc_tab4 = (uint4 *)l_tab;
    nl.quiet = blockIdx.x != 0;
    nl.entry_checked = 1;
    // Alphabets above 256 symbols (CSR): the wave would make five to eight symbols' entries per lane, so it stops at
    // the frequencies and the whole work-group makes the entries, a lane per symbol (c2 as CSR: 2 us less).  With
    // a byte alphabet the wave does it all: the second step's barriers and its instructions on all sixteen waves
    // of a compute unit cost more than they save there (c5a: 0.8 us more).
    const bool split = A > 256;
    nl.fF = split ? (uint2 *)l_tab : nullptr;
    if (threadIdx.x < 64) {  // frequencies and their running sums: one wave
      const NormResult r = normalize_wave(ctl, nl);
      if (threadIdx.x == 0) {
        sh[0] = r.ok; sh[1] = split ? 0u : (r.exact ? 0u : 1u); sh[2] = r.n_chunks;
        *(uint64_t *)(sh + 4) = r.len_d; *(uint64_t *)(sh + 6) = r.dir_off; *(uint64_t *)(sh + 8) = r.payload_off;
      }
    }
    __syncthreads();
    const uint32_t ok = sh[0];
    nc = sh[2];
    len = *(const uint64_t *)(sh + 4); dir_off = *(const uint64_t *)(sh + 6); payload_off = *(const uint64_t *)(sh + 8);
    if (!ok) {
      if (FUSE && blockIdx.x == 0 && threadIdx.x == 0 && d_stream_bytes) *d_stream_bytes = 0;
      bail();
      return;
    }
    if (split) {  // the table entries: every lane its symbol's (a division each), which overwrite {f, F} in the slot
      int inexact = 0;
      for (uint32_t a = threadIdx.x; a < A; a += kWG) {
        const uint2 e = nl.fF[2 * a];
        inexact |= emit_entries(nl, a, e.x, e.y, [](uint32_t kk, uint32_t d) { return div_pow2_by(kk, d); });
      }
      if (inexact) atomicOr(&sh[1], 1u);
      __syncthreads();
      if (blockIdx.x == 0 && threadIdx.x == 0) ctl->enc_exact = sh[1] == 0;
    }
    exact_tab = sh[1] == 0;
    if (!exact_tab) {
      for (uint32_t a = threadIdx.x; a < A; a += kWG) {
        const uint2 q = l_tab8[a];
        ((uint4 *)l_tab)[a] = make_uint4(q.x, q.y & 0xffffu, q.y >> 16, totalM - (q.y & 0xffffu));
      }
    }
    __syncthreads();  // the table is complete; sh and the stage may be written again
  } else {
    nc = ctl->n_chunks; len = ctl->len_d; dir_off = ctl->dir_off; payload_off = ctl->payload_off;
    exact_tab = TAB == 2 && ctl->enc_exact != 0;
    // TAB == 2 has two forms of the table: the division-free one when every entry of it is exact for
    // this frequency table (the common case), else {floor(2^32/f), f, F, 2^M - f} with a correction step.
    if (TAB == 1) {
      for (uint32_t a = threadIdx.x; a < A; a += kWG) ((uint2 *)l_tab)[a] = g_tab[a];
    } else if (TAB == 2) {
      if (exact_tab) {
        for (uint32_t a = threadIdx.x; a < A; a += kWG) ((uint4 *)l_tab)[a] = g_tab4[a];
      } else {
        for (uint32_t a = threadIdx.x; a < A; a += kWG) {
          uint2 q = g_tab[a];
          ((uint4 *)l_tab)[a] = make_uint4(q.x, q.y & 0xffffu, q.y >> 16, totalM - (q.y & 0xffffu));
        }
      }
    }
    if (TAB != 0) __syncthreads();
  }
  const bool exact = exact_tab != 0;
  if (k >= nc) {
    if (FUSE && nc == 0 && blockIdx.x == 0 && threadIdx.x == 0) {  // empty D: only the directory's single entry
      uint8_t *dir0 = out + dir_off;
      st32(dir0, 0u);
      st32(dir0 + 4, 0u);
      ctl->total_bytes = payload_off;
      if (d_stream_bytes) *d_stream_bytes = payload_off;
    }
    bail();
    return;
  }
  src.init(ctl);
  const uint64_t chunk_len = cs ? cs : len;
  const uint64_t base = (uint64_t)k * chunk_len;
  const uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
  const uint32_t j0 = g * kWG + threadIdx.x;
  const bool live = j0 < S;
  // the areas are addressed as plain LDS addresses
  typedef __attribute__((address_space(3))) uint16_t lds_u16;
  typedef __attribute__((address_space(3))) uint32_t lds_u32;
  if ((uint32_t)(uintptr_t)(lds_u16 *)l_mem != 0) {  // cannot happen without static LDS; the slot arithmetic relies on it
    if (threadIdx.x == 0) set_status(ctl, RANS_ERR_HIP);
    bail();
    return;
  }
  uint32_t s = kL;
  const uint32_t colb = kEncGuard + stride * threadIdx.x;  // the lane's area: slots colb, colb + 2, ..., top - 2
  const uint32_t top = colb + 2 * rw;
  uint32_t wp = top - 2;                                   // LDS address of the slot of the next word
  // Scratch holds the work-group's spilled 16-byte blocks block-major: block b of the stream in column c at
  // ((b * kWG + c) * 8) words from the work-group's base.
  uint16_t *const g0 = scratch + (uint64_t)blockIdx.x * kWG * capw + threadIdx.x * 8;
  uint16_t *gp = g0;  // where the stream's next spilled block goes
  auto words_in_area = [&]() { return (top - 2 - wp) >> 1; };
  // Moves the area's complete 8-word blocks (oldest first: from the top) to scratch and what is left, fewer
  // than 8 words, to the top of the area.  `all`: the remainder goes out too, as one more block whose first
  // 8 - r words are not part of the stream (the format k_gather reads).
  auto spill = [&](bool all) {
    const uint32_t n_used = words_in_area();
    const uint32_t nblk = n_used >> 3, r = n_used & 7;
    for (uint32_t b = 0; b < nblk; b++) {
      const lds_u32 *q = (const lds_u32 *)(uintptr_t)(top - 16 * (b + 1));
      *(uint4 *)gp = make_uint4(q[0], q[1], q[2], q[3]);
      gp += kWG * 8;
    }
    if (r && nblk) {  // the remaining words sit at the bottom end of what was used: up to the top
      for (uint32_t i = 0; i < r; i++)
        *(lds_u16 *)(uintptr_t)(top - 2 * r + 2 * i) = *(const lds_u16 *)(uintptr_t)(wp + 2 + 2 * i);
    }
    wp = top - 2 - 2 * r;
    if (all && r) {
      const lds_u32 *q = (const lds_u32 *)(uintptr_t)(top - 16);
      *(uint4 *)gp = make_uint4(q[0], q[1], q[2], q[3]);
      gp += kWG * 8;
    }
  };
  // after every batch: a stream with fewer than kEncAhead free slots left makes room
  auto make_room = [&]() {
    if (wp < colb + 2 * (kEncAhead - 1)) spill(false);
  };
  // The hardware issues a compute unit's oldest waves first: of several work-groups on a unit the first finishes
  // well before the last, which then runs alone and cannot fill the unit; and a work-group that polls for the
  // others' totals while its neighbours still code delays every vector load of the unit that is issued behind
  // the poll, i.e. their symbols.  Work-groups are placed round robin, so blockIdx.x / wgs_per_class tells the
  // work-groups of a unit apart.  With four of them per unit and long streams each takes every wave priority in
  // turn, sixteen rows at a time, and all finish at about the same time.  Otherwise (two or three per unit, or
  // streams of fewer than 128 rows, where the priorities did not even the progress out) an early one instead
  // sleeps before its first poll, without a single load, for about as long as the later ones still need: a
  // share of its own coding time per work-group behind it - an estimate that only decides when the polling
  // starts, not what is computed.  (Measured on c5a, 256 rows: 48 us with the sleep, 45 us with the priorities;
  // c2 DENSE, 98 rows: 24.5 us with the sleep, 30 us with the priorities.)
  const uint32_t prio_class = n_classes > 1 ? blockIdx.x / wgs_per_class : 0;  // < n_classes by the host's choice
  const bool prio_rotate = n_classes == 4 && chunk_len / S >= 128;
  const bool timed_wait = n_classes > 1 && !prio_rotate;
  const unsigned long long t_begin = (FUSE && timed_wait) ? wall_clock64() : 0ull;
  auto rotate_prio = [&](uint64_t t) {
    if (prio_rotate) {
      const uint32_t pr = (prio_class + ((uint32_t)t >> 4)) & 3u;
      if (pr == 0) __builtin_amdgcn_s_setprio(0);
      else if (pr == 1) __builtin_amdgcn_s_setprio(1);
      else if (pr == 2) __builtin_amdgcn_s_setprio(2);
      else __builtin_amdgcn_s_setprio(3);
    }
  };
  // The coding loop, for one of the two table forms (an entry is {m, f, F, cmpl} with the meaning of
  // that form: EXACT {mx, lim1, Fx | sh << 16, 2^M - f}, else {floor(2^32/f), f, F, 2^M - f}).
  auto run = [&](auto exact_tag, auto wide_tag) {
    constexpr bool EXACT = decltype(exact_tag)::value;
    constexpr int WIDE_KIND = decltype(wide_tag)::value;  // 0: direct loads, 1: dense bytes through LDS, 2: CSR segments through LDS
    constexpr bool WIDE = WIDE_KIND == 1;
    // Eq. 2; selects only, no branches.
    auto row = [&](const EncEntry &e) {
      const bool c = EXACT ? s > e.f : (s >> sh_lim) >= e.f;  // too large for this symbol: emit 16 bits
      *(lds_u16 *)(uintptr_t)wp = (uint16_t)s;                // speculative: the slot counts only if c
      s = c ? s >> 16 : s;
      wp = c ? wp - 2 : wp;
      uint32_t q = __umulhi(s, e.m);
      if constexpr (EXACT) {
        q >>= e.F >> 16;
        s = (MUL24 ? __umul24(q, e.cmpl) + s : q * e.cmpl + s) + (e.F & 0xffffu);
      } else {
        const uint32_t rem = s - (MUL24 ? __umul24(q, e.f) : q * e.f);
        q += rem >= e.f ? 1u : 0u;
        s = s + e.F + (MUL24 ? __umul24(q, e.cmpl) : q * e.cmpl);
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
    const uint64_t rows_full = n_here / S;
    const uint32_t rem_row = (uint32_t)(n_here - rows_full * S);
    if (rem_row) {  // ragged last row: only streams j < rem_row have a symbol there
      // an absent stream gets a neutral entry, which leaves the state untouched
      EncEntry ea = EXACT ? EncEntry{0u, 0xffffffffu, 0u, 0u} : EncEntry{0u, totalM, 0u, 0u};
      if (j0 < rem_row) ea = entry(src(base + rows_full * S + j0));
      row(ea);
    }
    // rows beyond a multiple of kEncAhead, one at a time
    uint64_t t = rows_full;
    for (uint32_t r = (uint32_t)(rows_full % kEncAhead); r > 0; r--, t--) row(entry(src(base + (t - 1) * S + j0)));
    // at most 1 + 7 words so far (rw >= 16): from here on every batch ends with make_room(), which keeps at least
    // kEncAhead slots free at the start of a batch
    make_room();
    // full batches of kEncAhead rows: rows fetched one batch ahead, table entries kLook rows ahead of their use
    // (an LDS read takes longer than the arithmetic of a row), in a rotation of kLook + 1 register sets
    uint32_t cur[kEncAhead], nxt[kEncAhead];
    constexpr int kLook = 3;
    EncEntry E[kLook + 1];
    auto prime = [&]() {  // entries of the first kLook rows of nxt[]
#pragma unroll
      for (int u = 0; u < kLook; u++) E[u] = entry(nxt[u]);
    };
    auto batch = [&]() {  // codes the rows in cur[]; leaves the entries of nxt[0 .. kLook-1] in E[0 .. kLook-1]
#pragma unroll
      for (int u = 0; u < kEncAhead; u++) {
        // past the end of the batch this looks up rows of the next batch; when there is none, nxt[]
        // still holds old, valid symbols and the entries are simply not used
        E[(u + kLook) % (kLook + 1)] = entry(u + kLook < kEncAhead ? cur[(u + kLook) % kEncAhead] : nxt[(u + kLook) % kEncAhead]);
        row(E[u % (kLook + 1)]);
      }
      make_room();
    };
    if constexpr (WIDE) {
      // Symbols through LDS: single-byte loads keep too few bytes in flight to cover the memory latency.
      // A wave owns a 64-byte column of the chunk's rows.  It fetches 16 rows of it at a time with 16-byte loads
      // (lane L: row L / 4 of the tile, bytes 16 (L % 4) ..; tiles start at multiples of 16 rows) and keeps two such
      // tiles waiting in registers, so a request has 24 to 32 rows of coding to arrive.  LDS holds two slots of
      // 8 rows per wave: before a batch, the half tile with its rows is parked in the slot the batch before the
      // last one has read up (a half tile is what 32 lanes hold, and lane L's 16 bytes go to byte 16 L of the
      // two slots taken as one area: rows 0-7 of a tile to slot 0, rows 8-15 to slot 1).  No other wave touches the area.
      static_assert(!WIDE || (kEncAhead == 8 && kStageRows == 16), "tile arithmetic below");
      const uint32_t lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
      uint8_t *stg = (uint8_t *)(sh + 16) + wv * (kStageRows * 64);
      const uint8_t *colp = src.bytes() + base + (j0 - lane) + 16 * (lane & 3);  // the lane's 16 bytes of row 0
      auto request = [&](uint64_t t_lo, uint64_t t_top) -> uint4 {  // rows t_lo .. t_lo+15 (below t_top) of the column
        const uint64_t r = t_lo + (lane >> 2);
        return r < t_top ? *(const uint4 *)(colp + r * S) : make_uint4(0, 0, 0, 0);
      };
      auto park_half = [&](const uint4 &q, uint32_t upper) {  // rows 8 upper .. 8 upper + 7 of the tile in q
        if ((lane >> 5) == upper) *(uint4 *)(stg + 16 * lane) = q;
      };
      auto read_rows = [&](uint32_t *dst, uint64_t t_hi) {  // rows t_hi-1 .. t_hi-8; t_hi is a multiple of 8
        const uint8_t *b = stg + (((uint32_t)t_hi - 8) & 8u) * 64 + lane;
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) dst[u] = b[(kEncAhead - 1 - u) * 64];
      };
      // pend[0]: the tile the next batch lies in (or the one below, once it is parked whole); pend[i]: i tiles below
      constexpr int kPend = 2;
      uint4 pend[kPend];
#pragma unroll
      for (int i = 0; i < kPend; i++) pend[i] = make_uint4(0, 0, 0, 0);
      auto advance = [&](uint64_t lowest_lo_plus16) {  // pend[0] is used up: the others move up, a new tile is requested below them
#pragma unroll
        for (int i = 0; i + 1 < kPend; i++) pend[i] = pend[i + 1];
        pend[kPend - 1] = make_uint4(0, 0, 0, 0);
        if (lowest_lo_plus16 >= kStageRows) pend[kPend - 1] = request(lowest_lo_plus16 - kStageRows, lowest_lo_plus16);
      };
      if (t) {
        const uint64_t t_lo = (t - 1) & ~(uint64_t)(kStageRows - 1);
        pend[0] = request(t_lo, t);
#pragma unroll
        for (int i = 1; i < kPend; i++)
          if (t_lo >= (uint64_t)i * kStageRows) pend[i] = request(t_lo - (uint64_t)i * kStageRows, t_lo - (uint64_t)(i - 1) * kStageRows);
        if ((t & 15) == 8) {  // the first batch is the tile's lower half, its upper half lies past the end
          park_half(pend[0], 0);
          advance(t_lo >= (uint64_t)(kPend - 1) * kStageRows ? t_lo - (uint64_t)(kPend - 1) * kStageRows : 0);
        } else {
          park_half(pend[0], 1);
        }
        read_rows(nxt, t);
        prime();
      }
      while (t) {
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) cur[u] = nxt[u];
        t -= kEncAhead;
        rotate_prio(t);
        if (t) {  // the next batch is rows t-8 .. t-1
          if ((t & 15) == 0) {
            park_half(pend[0], 1);  // upper half of the tile below the one just finished
          } else {
            park_half(pend[0], 0);  // lower half of the same tile; with it the tile is parked whole
            // pend[0] was the tile [t-8, t+8); the lowest pending one is kPend - 1 tiles below it
            const uint64_t low = t - 8;  // start of the used-up tile
            advance(low >= (uint64_t)(kPend - 1) * kStageRows ? low - (uint64_t)(kPend - 1) * kStageRows : 0);
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
      static_assert(WIDE_KIND != 2 || (kEncAhead == 8 && kStageRows2 == 16), "tile arithmetic below");
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
            const Block16 b0 = *(const Block16 *)q, b1 = *(const Block16 *)(q + 8);
            pend[0] = make_uint4(b0.x, b0.y, b0.z, b0.w);
            pend[1] = make_uint4(b1.x, b1.y, b1.z, b1.w);
          } else {
            uint32_t w[8];
#pragma unroll
            for (int kk = 0; kk < 8; kk++) {
              const uint32_t lo = i + 2 * kk < len ? src(i + 2 * kk) : 0u, hi = i + 2 * kk + 1 < len ? src(i + 2 * kk + 1) : 0u;
              w[kk] = lo | (hi << 16);
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
          for (int kk = 0; kk < 8; kk++) {
            const uint32_t two = ww[kk >> 1] >> (16 * (kk & 1));
            e[kk] = (two & 0xffu) | ((two & 0xff00u) << 8);
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
        rotate_prio(t);
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
        for (int u = 0; u < kEncAhead; u++) dst[u] = src(base + (t_hi - 1 - u) * S + j0);
      };
      if (t) {
        fetch_rows(nxt, t);
        prime();
      }
      while (t) {
#pragma unroll
        for (int u = 0; u < kEncAhead; u++) cur[u] = nxt[u];
        t -= kEncAhead;
        rotate_prio(t);
        if (t) fetch_rows(nxt, t);
        batch();
      }
    }
  };
  if (live) {
    if constexpr (std::is_same<Src, SrcDense>::value) {
      if (wide) {
        if (exact) run(std::true_type{}, std::integral_constant<int, 1>{});
        else run(std::false_type{}, std::integral_constant<int, 1>{});
      } else {
        if (exact) run(std::true_type{}, std::integral_constant<int, 0>{});
        else run(std::false_type{}, std::integral_constant<int, 0>{});
      }
    } else {
      if (wide) {
        if (exact) run(std::true_type{}, std::integral_constant<int, 2>{});
        else run(std::false_type{}, std::integral_constant<int, 2>{});
      } else {
        if (exact) run(std::true_type{}, std::integral_constant<int, 0>{});
        else run(std::false_type{}, std::integral_constant<int, 0>{});
      }
    }
  }
  if (prio_rotate) __builtin_amdgcn_s_setprio(0);
  if (!FUSE && live) spill(true);  // k_gather finds every word in scratch
  const uint32_t n_lds = (FUSE && live) ? words_in_area() : 0;                     // words still in the area
  const uint32_t nbg = live ? (uint32_t)((gp - g0) / (kWG * 8)) : 0;               // blocks in scratch
  // without FUSE the last block may be partial: spill(true) has left wp at the top minus the r words it holds
  const uint32_t nw = !live ? 0 : (FUSE ? 8 * nbg + n_lds : ((top - 2 - wp) >> 1 ? 8 * (nbg - 1) + ((top - 2 - wp) >> 1) : 8 * nbg));
  if (!FUSE && live) {
    st_out[(uint64_t)k * S + j0] = s;
    nw_out[(uint64_t)k * S + j0] = nw;
  }
  uint32_t tot;
  const uint32_t ex = block_excl_scan<kWG>(nw, sh, &tot);
  if (!FUSE) {
    if (threadIdx.x == 0 && tot) atomicAdd(&chunk_words[k], tot);
    return;
  }
  if constexpr (FUSE) {
    if (threadIdx.x == 0) {
      __hip_atomic_store(wg_pub + blockIdx.x, tot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_fetch_add(chunk_acc + k, (1ull << 40) | tot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // The spilled blocks of the whole work-group, taken as one list in stream order and, inside a stream, in
    // read order (the last written first): thread i moves blocks i, i + kWG, ...  Their owners and places come
    // from three small tables in LDS (the stage is no longer needed).  Every thread requests its first kPre
    // blocks now, so that they arrive while the work-group waits for the totals of the others.
    uint32_t *t_bex = sh + 16, *t_dst = t_bex + kWG, *t_nbg = t_dst + kWG;
    uint32_t n_spilled;
    const uint32_t bex = block_excl_scan<kWG>(nbg, sh, &n_spilled);
    constexpr int kPre = 2;
    uint4 pre_q[kPre];
    uint32_t pre_dst[kPre];  // word offset from the work-group's first word; ~0: no block
    auto owner_of = [&](uint32_t i) {  // the last stream whose first block is at or before i
      uint32_t lo = 0, hi = kWG;
      while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (t_bex[mid] <= i) lo = mid;
        else hi = mid;
      }
      return lo;
    };
    auto block_src = [&](uint32_t i, uint32_t *dst_off) -> const uint4 * {
      const uint32_t o = owner_of(i), bi = i - t_bex[o];
      *dst_off = t_dst[o] + 8 * bi;
      return (const uint4 *)(scratch + (uint64_t)blockIdx.x * kWG * capw + ((uint64_t)(t_nbg[o] - 1 - bi) * kWG + o) * 8);
    };
    if (n_spilled) {  // uniform
      t_bex[threadIdx.x] = bex;
      t_dst[threadIdx.x] = ex + n_lds;
      t_nbg[threadIdx.x] = nbg;
      lds_barrier();
#pragma unroll
      for (int u = 0; u < kPre; u++) {
        const uint32_t i = threadIdx.x + u * kWG;
        pre_dst[u] = ~0u;
        if (i < n_spilled) pre_q[u] = *block_src(i, &pre_dst[u]);
      }
    }
    if (timed_wait && threadIdx.x < 64) {  // the sleep before the first poll (see above)
      const unsigned long long now = wall_clock64();
      const unsigned long long until = now + ((now - t_begin) * (n_classes - 1 - prio_class) * 12) / 100;
      while (wall_clock64() < until) __builtin_amdgcn_s_sleep(32);
    }
    // Totals of what lies before this work-group's words: every earlier chunk (its size gives the chunk's
    // byte offset) and the earlier groups of this chunk (the position inside the chunk).  The first wave
    // collects them - a lane's loads are independent of each other - and hands the sums over through LDS.
    uint64_t *sh64 = (uint64_t *)(sh + 4);  // [0] chunk offset, [1] words before this group, [2] a wait failed
    const uint32_t lane = threadIdx.x & 63;
    if (threadIdx.x < 64) {
      uint64_t off_loc = 0, pre_loc = 0, failed = 0;
      for (uint32_t c = lane; c < k; c += 64) {
        const uint64_t words = wait_chunk(chunk_acc, c, groups, ctl);
        failed |= words == ~0ull;
        off_loc += (8ull * S + 2 * words + 3) & ~3ull;
      }
      for (uint32_t g2 = lane; g2 < g; g2 += 64) {
        const uint32_t v = wait_published(wg_pub, k * groups + g2, ctl);
        failed |= v == 0;
        pre_loc += v - 1;
      }
      auto add64 = [](uint64_t x, uint64_t y) { return x + y; };
      off_loc = lane63_64(wave_incl_scan64(off_loc, add64));
      pre_loc = lane63_64(wave_incl_scan64(pre_loc, add64));
      failed = lane63_64(wave_incl_scan64(failed, add64));
      if (lane == 0) {
        sh64[0] = off_loc;
        sh64[1] = pre_loc;
        sh64[2] = failed;
      }
    }
    __syncthreads();
    const uint64_t off = sh64[0], pre = sh64[1];
    if (sh64[2]) {  // uniform: a wait ran into its bound, or another work-group reported an error
      if (threadIdx.x == 0) {
        if (get_status(ctl) == 0) set_status(ctl, RANS_ERR_HIP);
        if (k == nc - 1 && g == groups - 1 && d_stream_bytes) *d_stream_bytes = 0;
      }
      return;
    }
    uint8_t *dir = out + dir_off;
    const uint64_t my_end = payload_off + off + 8ull * S + 2 * (pre + tot);  // end of this group's words
    const bool last_group = g == groups - 1;
    const uint64_t chunk_end = (my_end + 3) & ~3ull;  // meaningful for the chunk's last group
    const bool fits = (last_group ? chunk_end : my_end) <= cap;
    if (threadIdx.x == 0) {
      if (g == 0) {
        st32(dir + 8ull * k, (uint32_t)off);
        st32(dir + 8ull * k + 4, (uint32_t)(off >> 32));
      }
      if (k == nc - 1 && last_group) {
        const uint64_t pay = chunk_end - payload_off;
        st32(dir + 8ull * nc, (uint32_t)pay);
        st32(dir + 8ull * nc + 4, (uint32_t)(pay >> 32));
        ctl->total_bytes = chunk_end;
        if (d_stream_bytes) *d_stream_bytes = fits ? chunk_end : 0;
      }
      if (!fits) set_status(ctl, RANS_ERR_CAPACITY);
    }
    if (!fits) return;  // uniform
    uint8_t *ck = out + payload_off + off;
    if (live) {
      st32(ck + 4ull * j0, s);
      st32(ck + 4ull * S + 4ull * j0, nw);
    }
    // Words.  In read order a stream's words are the area's, lowest address first, then its spilled blocks, the
    // last written first.  The areas: eight lanes share a stream, each moving eight of its words (and eight more
    // 64 words on, where an area holds that many) as one 16-byte piece - both ends are only 2-byte aligned, which the target allows - so a
    // wave moves eight streams per step and their pieces are adjacent in the container.
    uint16_t *dst = (uint16_t *)(ck + 8ull * S) + pre;  // first word of this group
    for (uint32_t L0 = 0; L0 < 64; L0 += 8) {
      const int from = (int)(L0 + (lane >> 3));
      const uint32_t nL = (uint32_t)__shfl((int)n_lds, from), eL = (uint32_t)__shfl((int)ex, from);
      const uint32_t aL = (uint32_t)__shfl((int)wp, from) + 2;
      for (uint32_t w0 = 8 * (lane & 7); w0 < nL; w0 += 64) {
        const uint16_t *sp = (const uint16_t *)l_mem + (aL >> 1) + w0;
        uint16_t *dp = dst + eL + w0;
        if (w0 + 8 <= nL) {
          uint4 q;
          __builtin_memcpy(&q, sp, 16);
          __builtin_memcpy(dp, &q, 16);
        } else {  // the stream's last piece, 1 to 7 words: four, two, one
          const uint32_t rem = nL - w0;
          uint32_t o = 0;
          if (rem & 4) {
            uint2 q;
            __builtin_memcpy(&q, sp, 8);
            __builtin_memcpy(dp, &q, 8);
            o = 4;
          }
          if (rem & 2) {
            uint32_t q;
            __builtin_memcpy(&q, sp + o, 4);
            __builtin_memcpy(dp + o, &q, 4);
            o += 2;
          }
          if (rem & 1) dp[o] = sp[o];
        }
      }
    }
    // a spilled block to its place: 16 bytes to a 2-byte aligned address
    auto put_block = [&](const uint4 &q, uint32_t dst_off) { *(Block16 *)(dst + dst_off) = Block16{q.x, q.y, q.z, q.w}; };
    if (n_spilled) {
#pragma unroll
      for (int u = 0; u < kPre; u++)
        if (pre_dst[u] != ~0u) put_block(pre_q[u], pre_dst[u]);
      for (uint32_t i0 = threadIdx.x + kPre * kWG; i0 < n_spilled; i0 += 4 * kWG) {  // the rest, four in flight per thread
        uint4 q[4];
        uint32_t d_off[4];
#pragma unroll
        for (int u = 0; u < 4; u++) {
          d_off[u] = ~0u;
          if (i0 + u * kWG < n_spilled) q[u] = *block_src(i0 + u * kWG, &d_off[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; u++)
          if (d_off[u] != ~0u) put_block(q[u], d_off[u]);
      }
    }
    if (last_group && live && j0 == S - 1 && ((pre + tot) & 1)) dst[tot] = 0;  // pad the chunk to 4 bytes
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
