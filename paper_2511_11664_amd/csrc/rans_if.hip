// rans_if.hip -- HIP kernels (gfx950) and the C ABI of include/rans_if.h.
//
// One translation unit: the kernels live in the rans_*.h files next to this one (common helpers, Eq. 6 and the
// frequency table, modified CSR, encoder, decoder, reshape search); this file holds the per-kernel timing aid,
// the host side (launch sequences, workspace checks) and the extern "C" entry points.
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
#include <cstddef>
#include <cstring>
#include <atomic>
#include <mutex>
#include <type_traits>
#include <vector>

#include "rans_if.h"

#include "rans_common.h"
#include "rans_quant.h"
#include "rans_csr.h"
#include "rans_encode.h"
#include "rans_decode.h"
#include "rans_reshape.h"

// Workspace of rans_compress_noalloc (declared in rans_if.h): device memory that belongs to the library, so
// that callers which cannot allocate need not bring a workspace.  The rest of this file never uses the name
// except to look its device address up (static_ws_of_current_device).
static __device__ __align__(256) uint8_t static_ws[RANS_NOALLOC_WS_BYTES];

namespace {

// ------------------------------------------------------------------ instrumentation

// Optional per-kernel timing for benchmarks: when a kernel's bit is set in the
// mask, each of its launches is bracketed by a pair of HIP events recorded on the
// launch stream.  Off by default; the normal path records nothing.
enum KernelId {
  KID_MINMAX = 0, KID_QINFO, KID_QUANT_HIST, KID_SCAN, KID_CSR_COMPACT, KID_CSR_ROWS,
  KID_NORMALIZE, KID_ENCODE, KID_CHUNK_SCAN, KID_GATHER, KID_DEC_PREPARE, KID_DECODE, KID_ROW_SCAN,
  KID_CSR_EXPAND, KID_DEQUANT, KID_RS_MASK, KID_RS_COLS, KID_RS_ROWS, KID_RS_COST, KID_RS_ROWS_POW2, KID_COUNT
};
const char *const kKernelNames[KID_COUNT] = {
    "k_minmax", "k_qinfo", "k_quant_hist", "k_scan_u32", "k_csr_compact", "k_csr_rows",
    "k_normalize", "k_encode", "k_chunk_scan", "k_gather", "k_dec_prepare", "k_decode", "k_row_part",
    "k_csr_to_dense", "k_dequant", "k_rs_mask", "k_rs_cols", "k_rs_rows", "k_rs_cost", "k_rs_rows_pow2"};

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

// Compute units of the current device (0 if the query fails); asked once per device.
inline uint32_t compute_units() {
  static std::atomic<int> cached[64];
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int v = cached[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 0;
    cached[dev].store(v, std::memory_order_relaxed);
  }
  return (uint32_t)v;
}

constexpr uint32_t kDecWideGroupMinChunks = 192;
constexpr uint32_t kExpandOwnSumMaxTiles = 4096;
constexpr uint32_t kShortRowCols = 32;  // rows up to this length: k_csr_compact derives its row ends from a mask

inline uint32_t grid_for(uint64_t n, uint32_t per_block, uint32_t cap) {
  uint64_t g = (n + per_block - 1) / per_block;
  if (g < 1) g = 1;
  return (uint32_t)(g > cap ? cap : g);
}

// Index of the last of the counters behind L.chunk_words that a call starts from zero, and the tile counts among them.
inline uint32_t counter_words(const Layout &L) { return L.tc_off + L.n_blk - 1; }
inline uint32_t *tile_counts_of(const Layout &L, uint8_t *ws) {
  return L.n_blk ? (uint32_t *)(ws + L.chunk_words) + L.tc_off : nullptr;
}

inline uint32_t *grp_counts_of(const Layout &L, uint8_t *ws) {  // nonzeros per group of tiles (one work-group step of k_quant_hist)
  return L.n_blk ? tile_counts_of(L, ws) + L.n_blk : nullptr;
}

NormArgs norm_args(const rans_params &p, const Layout &L, uint8_t *ws, uint64_t n, uint8_t *d_stream, size_t cap) {
  return NormArgs{(const uint32_t *)(ws + L.cnt), L.cnt_rep, nullptr, (uint32_t *)(ws + L.fq), (uint2 *)(ws + L.enc_tab),
                  (uint4 *)(ws + L.enc_tab4), L.A, p, n, p.mode == RANS_MODE_CSR ? 0 : 1, d_stream, (uint64_t)cap};
}

// Extrema, Eq. 6, symbols and their histogram.
int launch_quantize(const void *d_x, uint64_t n, const rans_params &p, const Layout &L, uint8_t *ws, uint8_t *d_sym,
                    rans_qinfo *d_qinfo, hipStream_t st, uint32_t seq, uint32_t *tiles_per_grp = nullptr) {
  const CtlRef ctl{(Ctl *)(ws + L.ctl), seq};
  uint32_t *cnt = (uint32_t *)(ws + L.cnt);
  uint32_t *cw_ = (uint32_t *)(ws + L.chunk_words);
  const uint32_t ncz_ = counter_words(L);
  const bool f16 = p.in_dtype == RANS_F16;
  const bool vec = aligned_to(d_x, 16) && aligned_to(d_sym, 8);
  const uint32_t V = vec ? (f16 ? 8 : 4) : 1;
  static_assert(QNT * kQIter == kCsrTile, "a work-group step of k_quant_hist is V tiles of the CSR kernels");
  if (tiles_per_grp) *tiles_per_grp = V;
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
    int skip0 = p.mode == RANS_MODE_CSR;
    uint32_t g = grid_for(n, QNT * V * kQIter, skip0 ? kQuantBlocksCsr : kQuantBlocks);
    auto launch_qh = [&](auto csr_tag) {
      constexpr bool CSRV = decltype(csr_tag)::value;
      if (f16) {
        if (vec) PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<__half, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const __half *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, tile_counts_of(L, ws), grp_counts_of(L, ws));
        else PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<__half, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const __half *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, tile_counts_of(L, ws), grp_counts_of(L, ws));
      } else {
        if (vec) PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<float, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const float *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, tile_counts_of(L, ws), grp_counts_of(L, ws));
        else PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<float, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, (const float *)d_x, (uint32_t)n, ctl, p.q_bits, d_sym, cnt, skip0, part, n_part, d_qinfo, tile_counts_of(L, ws), grp_counts_of(L, ws));
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
                       uint32_t tiles_per_grp) {
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
      const uint32_t tpw = (L.n_blk + kCompactBlocks - 1) / kCompactBlocks;  // consecutive tiles per work-group
      const uint32_t g_compact = (L.n_blk + tpw - 1) / tpw;
      const uint32_t *grp = grp_counts_of(L, ws);
      // rows that lie inside a lane's 16 symbols: the compaction also produces the row counts (see rows_inside_lane)
      // or inside a tile whose every start is a row start (the LDS column histogram in its plain layout also takes
      // the row counts then): see k_csr_compact
      const bool short_rows = lds_hist && p.cols <= kShortRowCols && 8ull * p.cols <= A;
      const int rows_in_lane = (p.cols <= 16 && 16 % p.cols == 0) ? 1
                               : p.cols < 16 ? 3
                               : (lds_hist && !short_rows && p.cols >= 64 && kCsrTile % p.cols == 0) ? 2 : 0;
      if (lds_hist && p.cols <= kShortRowCols && 8ull * p.cols <= A)
        PROF_LAUNCH(KID_CSR_COMPACT, (k_csr_compact<true, true>), dim3(g_compact), dim3(kWG), ((A + 15u) & ~15u) * 4, st, d_sym, (uint32_t)n, al,
                           (uint32_t)p.cols, blk, grp, tiles_per_grp, ws + L.v, (uint16_t *)(ws + L.c), row_end, cnt, A, L.n_blk, tpw, L.cnt_rep, rows_in_lane, (uint16_t *)(ws + L.r), (uint32_t)p.rows, ctl);
      else if (lds_hist)
        PROF_LAUNCH(KID_CSR_COMPACT, (k_csr_compact<true>), dim3(g_compact), dim3(kWG), ((A + 15u) & ~15u) * 4, st, d_sym, (uint32_t)n, al,
                           (uint32_t)p.cols, blk, grp, tiles_per_grp, ws + L.v, (uint16_t *)(ws + L.c), row_end, cnt, A, L.n_blk, tpw, L.cnt_rep, rows_in_lane, (uint16_t *)(ws + L.r), (uint32_t)p.rows, ctl);
      else
        PROF_LAUNCH(KID_CSR_COMPACT, (k_csr_compact<false>), dim3(g_compact), dim3(kWG), 0, st, d_sym, (uint32_t)n, al,
                           (uint32_t)p.cols, blk, grp, tiles_per_grp, ws + L.v, (uint16_t *)(ws + L.c), row_end, cnt, A, L.n_blk, tpw, L.cnt_rep, rows_in_lane, (uint16_t *)(ws + L.r), (uint32_t)p.rows, ctl);
      LAUNCH_CHECK();
      if (!rows_in_lane) {
      uint32_t N = (uint32_t)p.rows;
      uint32_t g = (N + 16 * kWG - 1) / (16 * kWG);  // a lane takes 16 rows per step
      // few work-groups: each ends with additions to the same few addresses
      const uint32_t g_cap = N > (1u << 20) ? 256u : 128u;
      g = g > g_cap ? g_cap : g;
      if (lds_hist && 8ull * (p.cols + 1) <= A)  // short rows: eight counters per row count
        PROF_LAUNCH(KID_CSR_ROWS, (k_csr_rows<true, true>), dim3(g), dim3(kWG), A * 4, st, row_end, N, (uint16_t *)(ws + L.r), cnt, A, ctl, (uint32_t)p.cols, L.cnt_rep);
      else if (lds_hist)
        PROF_LAUNCH(KID_CSR_ROWS, (k_csr_rows<true>), dim3(g), dim3(kWG), A * 4, st, row_end, N, (uint16_t *)(ws + L.r), cnt, A, ctl, (uint32_t)p.cols, L.cnt_rep);
      else
        PROF_LAUNCH(KID_CSR_ROWS, (k_csr_rows<false>), dim3(g), dim3(kWG), 0, st, row_end, N, (uint16_t *)(ws + L.r), cnt, A, ctl, (uint32_t)p.cols, L.cnt_rep);
      LAUNCH_CHECK();
      }
    }
  }
  // D's histogram is complete here (the kernels that counted end before the next one starts).  Alphabets
  // that one wave can normalise: every work-group of the encoder builds the table for itself; otherwise, and
  // when there is nothing to encode, a kernel of its own does.
  NormArgs na_k = norm_args(p, L, ws, n, d_stream, cap);
  if (!(csr && n)) na_k.n_rep = 0;  // only k_csr_rows spreads its counts over partial histograms
  const int enc_builds = A <= kNormWaveA && L.nc_max != 0;
  if (!enc_builds) {
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
#define ENC_LAUNCH2(SRCT, TABV, M24, FUSEV)                                                                        \
  do {                                                                                                              \
    auto kfn = k_encode<SRCT, TABV, M24, FUSEV>;                                                                    \
    /* once per instantiation: allow dynamic LDS beyond the default 64 KB (large alphabets) */                     \
    static const hipError_t attr_rc =                                                                               \
        hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);             \
    if (lds_e > 64 * 1024 && attr_rc != hipSuccess) return RANS_ERR_HIP;                                            \
    PROF_LAUNCH(KID_ENCODE, kfn, dim3(n_wg_e), dim3(kWG), lds_e, st, src, tab, tab4, A, p.freq_bits, S,             \
                p.chunk_syms, ctl, scratch, L.capw, st_arr, nw_arr, cw, groups, cw + L.nc_max + 1,                  \
                (unsigned long long *)(cw + L.acc_off), d_stream, (uint64_t)cap, d_stream_bytes, wide_e, rw_e,      \
                wgs_per_class_e, n_classes_e, (TABV == 2 && enc_builds) ? 1 : 0, na_k);                             \
  } while (0)
#define ENC_LAUNCH(SRCT, TABV)                                                                                      \
  do {                                                                                                              \
    const int wide_e = S % 64 == 0 && (csr || aligned_to(d_sym, 16));                                               \
    /* LDS behind the word areas: table, reduction scratch, then the symbol stage, which the placement reuses   */ \
    /* for three tables of kWG words                                                                             */ \
    size_t stage_e = wide_e ? (csr ? (kWG / 64) * 2 * kStageRows2 * 128 + 16 : (kWG / 64) * kStageRows * 64) : 0;   \
    if (stage_e < 3 * kWG * 4) stage_e = 3 * kWG * 4;                                                               \
    if (enc_builds && stage_e < A * 12) stage_e = A * 12; /* counts and the table's other form, while it is built */ \
    const size_t rest_e = (TABV == 2 ? A * 16 : (TABV == 1 ? A * 8 : 0)) + 64 + stage_e;                            \
    /* slots per stream: what a stream can need (capw), as far as the LDS goes when every work-group of the grid */ \
    /* (up to four per compute unit) is to be resident at once                                                  */ \
    const uint32_t n_wg_e = L.nc_max * groups;                                                                      \
    const uint32_t n_cu_e = compute_units();                                                                        \
    uint32_t want_cu_e = n_cu_e ? (n_wg_e + n_cu_e - 1) / n_cu_e : 4;                                               \
    want_cu_e = want_cu_e < 1 ? 1 : (want_cu_e > 4 ? 4 : want_cu_e);                                                \
    const size_t budget_e = (160 * 1024) / want_cu_e;                                                               \
    uint32_t rw_e = L.capw < 16 ? 16 : (L.capw > 252 ? 252 : (L.capw + 3) & ~3u);                                   \
    while (rw_e > 16 && kEncGuard + enc_area_stride(rw_e) * kWG + rest_e > budget_e) rw_e -= 4;                     \
    const size_t lds_e = kEncGuard + enc_area_stride(rw_e) * kWG + rest_e;                                          \
    /* work-groups per compute unit when the whole grid is resident at once (see the kernel on wave priorities) */ \
    size_t per_cu_e = (160 * 1024) / lds_e;                                                                         \
    per_cu_e = per_cu_e > 8 ? 8 : per_cu_e;                                                                         \
    const bool resident_e = n_cu_e && per_cu_e && n_wg_e <= n_cu_e * per_cu_e;                                      \
    const uint32_t wgs_per_class_e = resident_e ? n_cu_e : n_wg_e;                                                  \
    uint32_t n_classes_e = resident_e ? (n_wg_e + n_cu_e - 1) / n_cu_e : 1;                                         \
    if (n_classes_e > 4) n_classes_e = 1; /* there are four wave priorities */                                      \
    if (mul24) {                                                                                                    \
      if (fused_gather) ENC_LAUNCH2(SRCT, TABV, true, true);                                                        \
      else ENC_LAUNCH2(SRCT, TABV, true, false);                                                                    \
    } else {                                                                                                        \
      if (fused_gather) ENC_LAUNCH2(SRCT, TABV, false, true);                                                       \
      else ENC_LAUNCH2(SRCT, TABV, false, false);                                                                   \
    }                                                                                                               \
  } while (0)
    if (csr) {
      SrcCsr src{ws + L.v, (const uint16_t *)(ws + L.c), (const uint16_t *)(ws + L.r), 0};
      if (A <= kEncTab16MaxA) ENC_LAUNCH(SrcCsr, 2);
      else if (lds_tab) ENC_LAUNCH(SrcCsr, 1);
      else ENC_LAUNCH(SrcCsr, 0);
    } else {
      SrcDense src{d_sym};
      ENC_LAUNCH(SrcDense, 2);
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
  // ... and there are enough chunks to give every CU one; with fewer, smaller groups spread a chunk over more CUs
  // (two of 512 lanes where the per-slot table takes most of a CU's LDS and each group has to build its own)
  const uint32_t nt = S <= 512 ? 256u : (h.n_chunks >= kDecWideGroupMinChunks ? 1024u : (M >= 14 ? 512u : 256u));
  const uint32_t groups_f = (S + nt - 1) / nt;
  const size_t win_b = 32 * (size_t)nt;
  const size_t tmp_b = align_up((size_t)lut_elem << M, 16) + 192 + (size_t)A * 8;  // [lut][misc][tab]
  const size_t lds_two = win_b + tmp_b;
  // wide table: 8 bytes per slot after the window; the build-time tables alias the window if they fit there
  const size_t wide_b = (size_t)8 << M;
  // (or only the slot -> symbol table does, and the rest follows the wide table)
  const size_t lut_b = align_up((size_t)lut_elem << M, 16);
  const bool tmp_alias = tmp_b <= win_b;
  const bool lut_alias = !tmp_alias && lut_b <= win_b;
  const size_t lds_wide = win_b + wide_b + (tmp_alias ? 0 : (lut_alias ? tmp_b - lut_b : tmp_b));
  const uint32_t tmp_off = (uint32_t)((tmp_alias || lut_alias) ? 0 : win_b + wide_b);
  const uint32_t misc_off = (uint32_t)(lut_alias ? win_b + wide_b : 0);
  const size_t kLdsMax = 160 * 1024;
  // worth it when the table is shared by enough lanes: always up to 2^13 slots, at 2^14 only for 1024-lane groups
  const bool use_wide = lds_wide <= kLdsMax && (M <= 13 || nt >= 512);
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
      h.x_max, h.p.q_bits, tmp_off, misc_off, img, h, d_qinfo
#define FDEC_ONE(SINKT, LUTT, MULV, NTV, WIDEV, sinkv)                                                              \
  do {                                                                                                             \
    auto kfn = k_decode_fast<SINKT, LUTT, MULV, NTV, WIDEV>;                                                       \
    /* once per instantiation: allow dynamic LDS beyond the default 64 KB */                                       \
    static const hipError_t attr_rc =                                                                              \
        hipFuncSetAttribute((const void *)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsMax);          \
    if (lds_fast > 64 * 1024 && attr_rc != hipSuccess) return RANS_ERR_HIP;                                        \
    PROF_LAUNCH(KID_DECODE, kfn, grid, blk, lds_fast, st, FDEC_ARGS, sinkv);                                       \
  } while (0)
#define FDEC_NT(SINKT, LUTT, MULV, WIDEV, sinkv)                                                                   \
  do {                                                                                                             \
    if (nt == 1024) FDEC_ONE(SINKT, LUTT, MULV, 1024, WIDEV, sinkv);                                               \
    else if (nt == 512) FDEC_ONE(SINKT, LUTT, MULV, 512, WIDEV, sinkv);                                            \
    else FDEC_ONE(SINKT, LUTT, MULV, 256, WIDEV, sinkv);                                                           \
  } while (0)
#define FDEC_LAUNCH(SINKT, LUTT, sinkv)                                                                            \
  do {                                                                                                             \
    if (use_wide) {                                                                                                \
      if (M >= 8) FDEC_NT(SINKT, LUTT, true, true, sinkv);                                                         \
      else FDEC_NT(SINKT, LUTT, false, true, sinkv);                                                               \
    } else {                                                                                                       \
      if (M >= 8) FDEC_NT(SINKT, LUTT, true, false, sinkv);                                                        \
      else FDEC_NT(SINKT, LUTT, false, false, sinkv);                                                              \
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
#undef FDEC_NT
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
    auto rows_of = [&](uint64_t c) {
      uint32_t tr = (uint32_t)(c / K);
      tr = tr < 1 ? 1 : (tr > 4096 ? 4096 : tr);
      if (tr >= 4) tr &= ~3u;  // then every tile starts on a 4-cell boundary (vector stores)
      return tr;
    };
    auto lds_of = [&](uint32_t tr) { return (size_t)expand_lds(tr, K).total; };
    uint32_t tile_rows = rows_of(cells);
    if (cells == kDenseTileCells) {
      // Large tensors.  The kernel is fastest with every tile on the chip at once (256 CUs; a CU holds eight
      // work-groups of this size, fewer if their LDS does not fit) and the tiles spread evenly: its time follows
      // the most loaded CU, which has m = ceil(tiles / 256) tiles.  For every m that tile sizes from half to 9/8
      // of the nominal one allow, the smallest tile with that m is a candidate.  The cost is m tiles (each with a
      // fixed part worth about 2048 cells), with a surcharge of the share of the tiles that does not fit the chip
      // at once, and another eighth beyond 2048 tiles (the row-sum kernel then needs a second turn as well).
      // Tiles of which fewer than seven fit a CU are taken only if there is no other: measured, the loss of
      // resident waves costs more than the larger tile saves.
      const uint32_t lo = rows_of(kDenseTileCells / 2), hi = rows_of(kDenseTileCells + kDenseTileCells / 8);
      const uint32_t unit = (K & 3) == 0 ? 1 : 4;  // keeps every tile's first cell on a 4-cell boundary
      bool found = false;
      for (int pass = 0; pass < 2 && !found; pass++) {
        const uint64_t min_per_cu = pass ? 1 : 7;
        uint64_t best_cost = ~0ull;
        for (uint64_t m = ((uint64_t)N + 256ull * hi - 1) / (256ull * hi); m <= 64; m++) {
          uint64_t tr = ((uint64_t)N + 256 * m - 1) / (256 * m);
          tr = (tr + unit - 1) / unit * unit;
          if (tr < lo) break;
          if (tr > hi || tr * K > 65535) continue;
          const uint64_t nt = (N + tr - 1) / tr;
          uint64_t per_cu = (160 * 1024) / (lds_of((uint32_t)tr) + 256);
          per_cu = per_cu > 8 ? 8 : per_cu;
          if (per_cu < min_per_cu) continue;
          uint64_t cost = m * (tr * K + 2048) * 64;
          if (nt > 256 * per_cu) cost += cost * (nt - 256 * per_cu) / nt;
          if (nt > 2048) cost += cost / 8;
          if (cost < best_cost) {
            best_cost = cost;
            tile_rows = (uint32_t)tr;
            found = true;
          }
        }
      }
    }
    const uint32_t n_tiles = (N + tile_rows - 1) / tile_rows;
    uint32_t *part = (uint32_t *)(ws + L.row_off);  // n_tiles + 1 entries (n_tiles <= N)
    PROF_LAUNCH(KID_ROW_SCAN, k_row_part, dim3((n_tiles + kWG / 64 - 1) / (kWG / 64)), dim3(kWG), 0, st, D + 2 * nnz, N, K, tile_rows,
                n_tiles, part, ctl);
    LAUNCH_CHECK();
    // up to a few thousand tiles every work-group of the expand kernel adds up the sums before its own
    const int scanned = n_tiles > kExpandOwnSumMaxTiles;
    if (scanned) {
      PROF_LAUNCH(KID_SCAN, k_scan_u32, dim3(1), dim3(kBig), 0, st, part, n_tiles);
      LAUNCH_CHECK();
    }
    const size_t lds = lds_of(tile_rows);
    if (lds > 64 * 1024) {  // a single long row: allow dynamic LDS beyond the default 64 KB (once per instantiation)
      static const hipError_t a0 = hipFuncSetAttribute((const void *)k_csr_to_dense<uint8_t>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      static const hipError_t a1 = hipFuncSetAttribute((const void *)k_csr_to_dense<float>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      static const hipError_t a2 = hipFuncSetAttribute((const void *)k_csr_to_dense<__half>, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
      if (a0 != hipSuccess || a1 != hipSuccess || a2 != hipSuccess) return RANS_ERR_HIP;
    }
    if (out_kind == 0)
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<uint8_t>), dim3(n_tiles), dim3(kWG), lds, st, D, part, scanned, N, K, tile_rows,
                  h.p.q_bits, (uint32_t)nnz, (uint8_t *)d_out, ctl);
    else if (out_kind == 1)
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<float>), dim3(n_tiles), dim3(kWG), lds, st, D, part, scanned, N, K, tile_rows,
                  h.p.q_bits, (uint32_t)nnz, (float *)d_out, ctl);
    else
      PROF_LAUNCH(KID_CSR_EXPAND, (k_csr_to_dense<__half>), dim3(n_tiles), dim3(kWG), lds, st, D, part, scanned, N, K, tile_rows,
                  h.p.q_bits, (uint32_t)nnz, (__half *)d_out, ctl);
    LAUNCH_CHECK();
  }
  return RANS_OK;
}


// Shared body of rans_compress and rans_compress_noalloc.
int compress_impl(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream, size_t stream_cap,
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
  uint32_t tpg = 1;
  rc = launch_quantize(d_x, n_elems, *p, L, ws, ws + L.sym, nullptr, st, seq, &tpg);
  if (rc) return rc;
  return launch_encode_tail(ws + L.sym, n_elems, *p, L, ws, d_stream, stream_cap, d_stream_bytes, st, seq, tpg);
}

// ---- the workspace of rans_compress_noalloc: a device array of the library itself
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  In host code the array's name is only a handle for the look-up below; what kernels, copies and the
// status read take is the device address that look-up returns, kept per device.
constexpr size_t kStaticWsBytes = RANS_NOALLOC_WS_BYTES;
constexpr int kStaticWsMaxDevices = 64;
struct StaticWs {
  std::mutex mu;
  void *ptr[kStaticWsMaxDevices] = {nullptr};
};
StaticWs g_static_ws;

int static_ws_of_current_device(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return RANS_ERR_HIP;
  if (dev < 0 || dev >= kStaticWsMaxDevices) return RANS_ERR_ARG;
  std::lock_guard<std::mutex> lk(g_static_ws.mu);
  if (!g_static_ws.ptr[dev]) {  // once per device, with that device current
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(static_ws)) != hipSuccess || !p) return RANS_ERR_HIP;
    if (!aligned_to(p, 256)) return RANS_ERR_HIP;
    g_static_ws.ptr[dev] = p;
  }
  *out = g_static_ws.ptr[dev];
  return RANS_OK;
}

// ---- reshape search: host side

struct RsPlan {
  RsCands cands;
  RsOffsets offs;
  RsGroups grps;
  RsPow2 pow2;    // candidates whose row counts k_rs_rows_pow2 takes from the mask
  bool any_pow2;
  uint32_t n_entries, n_tiles;
  size_t mask16, lp, tile_cnt, zero0, hv, hl, hr, bad, costs, ticket, total;  // byte offsets in the workspace
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
  uint32_t orr = 0;
  for (uint32_t k = 0; k < P.cands.n; k++) {
    P.offs.hr[k] = orr;
    orr += P.cands.K[k] + 1u;
  }
  P.offs.hr[P.cands.n] = orr;
  {  // work-groups of k_rs_rows: about kRowsGrid in all, shared out by the number of rows (K = 1 needs one)
    constexpr uint64_t kRowsGrid = 4096;
    // K = 1 has a closed form and K = 2, 4, 8, 16 a kernel of their own: no rows for k_rs_rows
    auto rows_of = [&](uint32_t K) -> uint64_t { return (K == 1 || K == 2 || K == 4 || K == 8 || K == 16) ? 0 : n / K; };
    for (uint32_t i = 0; i < 4; i++) P.pow2.hr_at[i] = ~0u;
    for (uint32_t k = 0; k < P.cands.n; k++)
      for (uint32_t i = 0; i < 4; i++)
        if (P.cands.K[k] == (2u << i)) {
          P.pow2.hr_at[i] = P.offs.hr[k];
          P.any_pow2 = true;
        }
    uint64_t rows_all = 0;
    for (uint32_t k = 0; k < P.cands.n; k++) rows_all += rows_of(P.cands.K[k]);
    uint32_t w = 0;
    for (uint32_t k = 0; k < P.cands.n; k++) {
      P.offs.wg0[k] = w;
      const uint64_t rows = rows_of(P.cands.K[k]);
      const uint64_t need = (rows + 4 * 63 - 1) / (4 * 63);  // work-groups that have a row at all
      uint64_t share = rows_all ? (rows * kRowsGrid + rows_all - 1) / rows_all : 1;
      share = share > need ? need : share;
      w += (uint32_t)((share < 1 && (rows || P.cands.K[k] == 1)) ? 1 : share);  // K = 1 keeps one work-group for its closed form
    }
    P.offs.wg0[P.cands.n] = w;
  }
  // groups of consecutive candidates with a common multiple of at most kRsLcmMax (see RsGroups)
  uint32_t ol = 0;
  {
    auto gcd = [](uint32_t a, uint32_t b) {
      while (b) {
        const uint32_t t = a % b;
        a = b;
        b = t;
      }
      return a;
    };
    uint32_t cur = 0;  // common multiple of the open group, 0: none open
    for (uint32_t k = 0; k < P.cands.n; k++) {
      const uint32_t K = P.cands.K[k];
      const uint64_t l2 = cur ? (uint64_t)cur / gcd(cur, K) * K : 0;
      if (cur && l2 <= kRsLcmMax) {
        cur = (uint32_t)l2;
      } else {
        if (cur) P.grps.n++;
        cur = K;
      }
      P.grps.of[k] = (uint8_t)P.grps.n;
      P.grps.L[P.grps.n] = cur;
    }
    if (cur) P.grps.n++;
    for (uint32_t g = 0; g < P.grps.n; g++) {
      uint32_t &L = P.grps.L[g];
      if (L < 32) L *= (32 + L - 1) / L;  // the kernel's wrap-around assumes at least 32 residues
      P.grps.off[g] = ol;
      ol += L;
    }
    P.grps.off[P.grps.n] = ol;
  }
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
  P.hl = take((size_t)ol * 4 + 4);
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
  uint32_t *hv = (uint32_t *)(ws + P.hv), *hl = (uint32_t *)(ws + P.hl), *hr = (uint32_t *)(ws + P.hr);
  uint32_t *bad = (uint32_t *)(ws + P.bad);
  hipLaunchKernelGGL(k_rs_zero, dim3(8), dim3(256), 0, st, (uint32_t *)(ws + P.zero0), P.zero_words);
  LAUNCH_CHECK();
  PROF_LAUNCH(KID_RS_MASK, k_rs_mask, dim3(P.n_tiles < 512 ? P.n_tiles : 512), dim3(kWG), 0, st, d_sym, (uint32_t)n,
              (int)aligned_to(d_sym, 16), P.n_tiles, mask16, lp, tile_cnt, hv, q_bits, bad);
  LAUNCH_CHECK();
  PROF_LAUNCH(KID_SCAN, k_scan_u32, dim3(1), dim3(kBig), 0, st, tile_cnt, P.n_tiles);
  LAUNCH_CHECK();
  {
    static const hipError_t attr_rc = hipFuncSetAttribute((const void *)k_rs_cols, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                          kRsLcmMax * 4);
    if (attr_rc != hipSuccess) return RANS_ERR_HIP;
    const uint32_t n_cu = compute_units();
    const uint32_t g_e = grid_for((P.n_entries + 7) / 8, kWG, n_cu ? n_cu : 256);  // one work-group per compute unit
    for (uint32_t g = 0; g < P.grps.n; g++) {
      PROF_LAUNCH(KID_RS_COLS, k_rs_cols, dim3(g_e), dim3(kWG), P.grps.L[g] * 4, st, mask16, P.n_entries, P.grps.L[g],
                  hl + P.grps.off[g]);
      LAUNCH_CHECK();
    }
  }
  if (P.any_pow2) {
    const uint32_t n_cu = compute_units();
    PROF_LAUNCH(KID_RS_ROWS_POW2, k_rs_rows_pow2, dim3(grid_for((P.n_entries + 7) / 8, kWG, n_cu ? n_cu : 256)), dim3(kWG), 0, st,
                mask16, P.n_entries, (uint32_t)n, P.pow2, hr);
    LAUNCH_CHECK();
  }
  if (P.cands.n && P.offs.wg0[P.cands.n]) {
    PROF_LAUNCH(KID_RS_ROWS, k_rs_rows, dim3(P.offs.wg0[P.cands.n]), dim3(kWG), 0, st, mask16, lp, tile_cnt,
                (uint32_t)n, P.n_tiles, P.cands, P.offs, hr);
    LAUNCH_CHECK();
  }
  if (P.cands.n)
    PROF_LAUNCH(KID_RS_COST, k_rs_cost, dim3(P.cands.n), dim3(kWG), 0, st, P.cands, (uint32_t)n, P.n_tiles, q_bits, tile_cnt, hv, hl,
                hr, P.offs, P.grps, bad, (double *)(ws + P.costs), (uint32_t *)(ws + P.ticket), d_res);
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
    const int skip0 = p->mode == RANS_MODE_CSR;
    const uint32_t g = grid_for(n_elems, QNT * (vec ? 16 : 1) * kQIter, skip0 ? kQuantBlocksCsr : kQuantBlocks);
    auto launch_qh = [&](auto csr_tag) {
      constexpr bool CSRV = decltype(csr_tag)::value;
      if (vec)
        PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<uint8_t, true, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, d_sym, (uint32_t)n_elems, ctl, p->q_bits, (uint8_t *)nullptr, (uint32_t *)(ws + L.cnt), skip0, (const MinMaxPart *)nullptr, 0u, (rans_qinfo *)nullptr, tile_counts_of(L, ws), grp_counts_of(L, ws));
      else
        PROF_LAUNCH(KID_QUANT_HIST, (k_quant_hist<uint8_t, false, QNT, CSRV>), dim3(g), dim3(QNT), 0, st, d_sym, (uint32_t)n_elems, ctl, p->q_bits, (uint8_t *)nullptr, (uint32_t *)(ws + L.cnt), skip0, (const MinMaxPart *)nullptr, 0u, (rans_qinfo *)nullptr, tile_counts_of(L, ws), grp_counts_of(L, ws));
    };
    if (skip0) launch_qh(std::true_type{});
    else launch_qh(std::false_type{});
    LAUNCH_CHECK();
  }
  return launch_encode_tail(d_sym, n_elems, *p, L, ws, d_stream, stream_cap, d_stream_bytes, st, seq,
                            aligned_to(d_sym, 16) ? 16u : 1u);
}

int rans_compress(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream, size_t stream_cap,
                  uint64_t *d_stream_bytes, void *d_ws, size_t ws_bytes, void *stream) {
  return compress_impl(d_x, n_elems, p, d_stream, stream_cap, d_stream_bytes, d_ws, ws_bytes, stream);
}

int rans_compress_noalloc(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream,
                          size_t stream_cap, uint64_t *d_stream_bytes, void **d_ws_used, void *stream) {
  int rc = check_params(p, n_elems);
  if (rc) return rc;
  if (make_layout(*p, n_elems).total > kStaticWsBytes) return RANS_ERR_WORKSPACE;  // beyond the stated maximum
  void *ws = nullptr;
  rc = static_ws_of_current_device(&ws);
  if (rc) return rc;
  if (d_ws_used) *d_ws_used = ws;
  return compress_impl(d_x, n_elems, p, d_stream, stream_cap, d_stream_bytes, ws, kStaticWsBytes, stream);
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

int rans_selftest_divide(uint32_t *d_mismatches, uint64_t n_random, void *stream) {
  if (!d_mismatches || !aligned_to(d_mismatches, 4)) return RANS_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  hipLaunchKernelGGL(k_selftest_clear, dim3(1), dim3(1), 0, st, d_mismatches);
  LAUNCH_CHECK();
  uint64_t g = (n_random + kWG - 1) / kWG;
  g = g < 256 ? 256 : (g > 4096 ? 4096 : g);  // at least the 65536 divisors of the first check
  hipLaunchKernelGGL(k_selftest_divide, dim3((uint32_t)g), dim3(kWG), 0, st, d_mismatches, n_random);
  LAUNCH_CHECK();
  return RANS_OK;
}

int rans_last_status(void *d_ws, void *stream) {
  if (!d_ws) return RANS_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  unsigned long long w = 0;  // the control block's sticky word
  uint8_t *at = (uint8_t *)d_ws + offsetof(Ctl, sticky);
  if (hipMemcpyAsync(&w, at, sizeof(w), hipMemcpyDeviceToHost, st) != hipSuccess) return RANS_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return RANS_ERR_HIP;
  // without the tag the workspace has never recorded an error
  if ((w >> 16) != kStickyTag || (w & 0xffffu) == 0) return RANS_OK;
  // reading clears it (stream-ordered; the source is copied before the call returns)
  static const unsigned long long cleared = kStickyTag << 16;
  if (hipMemcpyAsync(at, &cleared, sizeof(cleared), hipMemcpyHostToDevice, st) != hipSuccess) return RANS_ERR_HIP;
  if (hipStreamSynchronize(st) != hipSuccess) return RANS_ERR_HIP;
  return -(int)(uint32_t)(w & 0xffffu);
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
