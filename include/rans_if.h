/*
 * rans_if.h -- C ABI of the MI355X rANS intermediate-feature codec.
 *
 * The library implements the compression pipeline of the paper's Sec. 3.1
 * (Fig. 1(c)): reshape (Eq. 5) -> asymmetric integer quantisation (Eq. 6) ->
 * modified CSR (v, c, r) -> concatenation D = v (+) c (+) r (Eq. 7) -> one
 * frequency table -> rANS (Sec. 2.1, Eq. 2-4), and its inverse.  Everything
 * runs in HIP kernels on one gfx950 device; there is no CPU fallback.
 *
 * Conventions
 *   - Pointers named d_* are DEVICE pointers owned by the caller; h_* are host
 *     pointers.  The entry points with a workspace argument allocate and free
 *     nothing: scratch lives in the caller's workspace d_ws, whose size
 *     rans_workspace_bytes() returns.  d_ws must be 256-byte aligned, d_stream
 *     16-byte aligned, tensors aligned to their element size.  A workspace
 *     needs no initialisation and may be reused by any sequence of calls, one
 *     at a time.  Host-side state of the library: a process-wide call counter
 *     (calls are numbered so that a kernel can tell its own call's status
 *     from an older one's) and, only while rans_profile_enable() is on, the
 *     event pairs of the timing aid.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All work is enqueued on it; calls return without synchronising unless
 *     stated otherwise.
 *   - Return value: RANS_OK or a negative RANS_ERR_*.  Errors that depend only
 *     on the arguments are detected on the host before any launch.  Errors
 *     that depend on the data (non-finite input, too many distinct symbols,
 *     a caller-provided symbol outside {0..2^Q-1}, output capacity, corrupt
 *     container) are recorded in the workspace; the kernels of that call then
 *     stop producing output, and rans_last_status() reports the first error
 *     recorded by ANY call on the workspace since the status was last read.
 *     RANS_ERR_HIP as a recorded status means an internal check failed: a
 *     histogram that does not add up to the number of symbols, or the
 *     encoder's bounded wait for the work-groups before it ran out (possible
 *     when the GPU is time-sliced between processes); the output of that call
 *     is invalid and the call can simply be repeated.  No call aborts or throws.
 *   - Limits: n_elems <= 2^30; 1 <= Q <= 8; 1 <= M <= 15; 1 <= S <= 65536;
 *     CSR mode needs cols <= 65535.
 *   - Stream capture: every entry point that takes a `stream`, except
 *     rans_last_status and rans_decode / rans_decompress without a header
 *     hint (these read a few bytes back and synchronise), only enqueues
 *     kernels and may be captured into a HIP graph.  A replay writes the same
 *     bytes as the eager call.  Every replay starts like a fresh call; an
 *     error that a replay records stays in the workspace until
 *     rans_last_status() has read it.
 */
#ifndef RANS_IF_H
#define RANS_IF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RANS_OK = 0,
  RANS_ERR_ARG = -1,       /* null/misaligned pointer, parameter out of range           */
  RANS_ERR_SHAPE = -2,     /* rows*cols != n_elems, chunk_syms not a multiple of S      */
  RANS_ERR_ALPHABET = -3,  /* more distinct symbols than 2^M, or CSR with cols > 65535  */
  RANS_ERR_CAPACITY = -4,  /* output buffer too small                                   */
  RANS_ERR_WORKSPACE = -5, /* ws_bytes smaller than rans_workspace_bytes() reports      */
  RANS_ERR_NONFINITE = -6, /* NaN/Inf in the tensor, or x_max - x_min overflows         */
  RANS_ERR_CORRUPT = -7,   /* container fails validation                                */
  RANS_ERR_HIP = -8        /* a HIP runtime call failed                                 */
};

enum { RANS_MODE_DENSE = 0, RANS_MODE_CSR = 1 };
enum { RANS_F32 = 0, RANS_F16 = 1 };

/* The paper's statement of the problem: bit width Q (Eq. 6), coding precision
 * n (Eq. 2-4, called M here), reshape N x K (Eq. 5).  mode selects what is
 * coded: the paper's D = v (+) c (+) r (CSR), or the quantised tensor itself
 * (DENSE, for activations without exact zeros).  n_streams / chunk_syms shape
 * the parallel coder: D is cut into chunks of chunk_syms symbols, and inside a
 * chunk symbol i belongs to stream i mod n_streams; every stream is an
 * independent rANS coder sharing the one frequency table. */
typedef struct {
  uint32_t q_bits;     /* Q, 1..8                                          */
  uint32_t freq_bits;  /* M, 1..15                                         */
  uint64_t rows, cols; /* N, K with rows * cols == n_elems, cols >= 1      */
  uint32_t mode;       /* RANS_MODE_*                                      */
  uint32_t n_streams;  /* S >= 1                                           */
  uint32_t chunk_syms; /* multiple of S; 0 = all of D in one chunk         */
  uint32_t in_dtype;   /* RANS_F32 / RANS_F16: element type of the tensor  */
} rans_params;

/* Eq. 6: extrema, scale s and zero point z (an integer-valued float). */
typedef struct {
  float x_min, x_max, scale, zero_point;
} rans_qinfo;

/* Fixed part of a container, as rans_peek_header() reads it. */
typedef struct {
  rans_params p;
  uint64_t n_elems;  /* T                                    */
  uint64_t len_d;    /* number of coded symbols, l_D of Eq. 7 */
  uint32_t alphabet; /* max(2^Q, K+1) in CSR mode, else 2^Q  */
  uint32_t n_chunks;
  float x_min, x_max;
} rans_header;

/* Size of the workspace every entry point below needs for these parameters,
 * and an upper bound of the container size (either output may be NULL). Host only. */
int rans_workspace_bytes(const rans_params *p, uint64_t n_elems, size_t *ws_bytes,
                         size_t *max_stream_bytes);

/* Eq. 6 over the whole tensor: global min/max, scale, zero point, then
 * xhat = clamp(round_half_even(x / s + z), 0, 2^Q - 1) in binary32 without FMA.
 * d_x: n_elems elements of p->in_dtype.  d_sym: n_elems bytes out.
 * d_qinfo: one rans_qinfo out (device).  A constant tensor gives s = 0 and all
 * symbols 0.  Data errors: RANS_ERR_NONFINITE. */
int rans_quantize(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_sym,
                  rans_qinfo *d_qinfo, void *d_ws, size_t ws_bytes, void *stream);

/* Sec. 3.1 "Modified CSR Encoding", "Concatenation and rANS Encoding", and
 * Sec. 2.1 Eq. 2 with renormalisation: symbols -> container.
 * d_sym: n_elems quantised symbols (< 2^Q).  d_qinfo: the extrema that go into
 * the header (device).  d_stream / stream_cap: output buffer; the number of
 * bytes written goes to *d_stream_bytes (device, 8-byte aligned; 0 on a data
 * error).  Data errors: RANS_ERR_ALPHABET, RANS_ERR_CAPACITY, RANS_ERR_ARG (a
 * symbol >= 2^Q), RANS_ERR_NONFINITE (extrema in d_qinfo), RANS_ERR_HIP (see above). */
int rans_encode(const uint8_t *d_sym, uint64_t n_elems, const rans_params *p,
                const rans_qinfo *d_qinfo, uint8_t *d_stream, size_t stream_cap,
                uint64_t *d_stream_bytes, void *d_ws, size_t ws_bytes, void *stream);

/* Sec. 2.1 Eq. 3-4 and the decoder side of the modified CSR (cumulative sum of
 * r, scatter of v): container -> symbols.
 * h_hdr: the container's header as rans_peek_header() returned it; it sizes the
 * launches and is checked against the bytes on the device.  If NULL the library
 * copies the 128-byte header to the host itself, which SYNCHRONISES the stream.
 * d_sym / sym_cap: n_elems symbols out.  d_qinfo: nullable, receives the
 * quantiser parameters recomputed from the header.  Every field, table, offset
 * and final coder state is validated; nothing is read or written out of bounds
 * for any input bytes.  Data errors: RANS_ERR_CORRUPT. */
int rans_decode(const uint8_t *d_stream, size_t stream_bytes, const rans_header *h_hdr,
                uint8_t *d_sym, uint64_t sym_cap, rans_qinfo *d_qinfo, void *d_ws,
                size_t ws_bytes, void *stream);

/* Inverse of Eq. 6: x = s * (xhat - z), one subtraction and one multiplication
 * in binary32 without FMA; out_dtype RANS_F16 narrows with round-half-even.
 * s = 0 (constant tensor) yields x_min everywhere. */
int rans_dequantize(const uint8_t *d_sym, uint64_t n_elems, const rans_qinfo *d_qinfo,
                    uint32_t out_dtype, void *d_x_out, void *stream);

/* Fig. 1(c) end to end: tensor -> container.  Same bytes as rans_quantize
 * followed by rans_encode. */
int rans_compress(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream,
                  size_t stream_cap, uint64_t *d_stream_bytes, void *d_ws, size_t ws_bytes,
                  void *stream);

/* rans_compress for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch memory is an array of
 * RANS_NOALLOC_WS_BYTES bytes inside the library's own device image (every GPU the library runs on holds
 * its copy until the process ends); the call allocates and frees nothing.  Same container bytes as rans_compress.
 * Parameters whose workspace (rans_workspace_bytes) exceeds RANS_NOALLOC_WS_BYTES: RANS_ERR_WORKSPACE, nothing
 * is launched.  *d_ws_used (host pointer, nullable) receives the device address of the array, for
 * rans_last_status(); a data error also shows as *d_stream_bytes == 0.  All calls on one GPU share the one
 * array: calls that overlap in time on the same GPU (two streams, two threads) race and must be serialised
 * by the caller.  Everything a call needs to start from zero it clears itself; a recorded error stays until
 * rans_last_status() reads it.  The first call on a device looks the array's address up (a host-side step,
 * not a kernel: make that call outside stream capture). */
#define RANS_NOALLOC_WS_BYTES (32u << 20)
int rans_compress_noalloc(const void *d_x, uint64_t n_elems, const rans_params *p, uint8_t *d_stream,
                          size_t stream_cap, uint64_t *d_stream_bytes, void **d_ws_used, void *stream);

/* container -> tensor of out_dtype (elem_cap elements available at d_x_out).
 * Same values as rans_decode followed by rans_dequantize. */
int rans_decompress(const uint8_t *d_stream, size_t stream_bytes, const rans_header *h_hdr,
                    uint32_t out_dtype, void *d_x_out, uint64_t elem_cap, void *d_ws,
                    size_t ws_bytes, void *stream);

/* Sec. 3.2, Algorithm 1: approximate search for the reshape N~ of the modified CSR.  The cost of a
 * reshape [N, K = T/N] is the size proxy of Eq. 8 with alpha_enc = alpha_dec = 0,
 * T_tot(N) = l_D * H(p(N)) in bits, H the entropy of the one histogram over D = v (+) c (+) r (Eq. 7),
 * in binary64.  The domain is N > sqrt(T), T/N <= 2^Q, N | T; the walk goes from N = T downwards,
 * keeps the cheapest N and stops after the first N that costs more than the one before it.
 * d_sym: the n_elems quantised symbols (< 2^Q).  *d_result (device, 8-byte aligned) receives the
 * result; the costs of ALL reshapes of the domain are computed (cand_* in walk order, the first
 * n_evaluated of them are the ones the walk looks at).  An empty domain gives rows = T, cols = 1,
 * cost_bits = +inf.  More than RANS_RESHAPE_MAX_CAND reshapes in the domain: RANS_ERR_ARG.
 * Workspace: rans_search_workspace_bytes(). */
#define RANS_RESHAPE_MAX_CAND 128
typedef struct {
  uint64_t rows, cols;   /* N~, T / N~ */
  double cost_bits;      /* T_tot(N~) */
  uint32_t n_evaluated;  /* reshapes the walk evaluated before it stopped */
  uint32_t n_candidates; /* reshapes in the domain */
  uint64_t cand_rows[RANS_RESHAPE_MAX_CAND];
  double cand_cost[RANS_RESHAPE_MAX_CAND];
} rans_reshape_result;
int rans_search_workspace_bytes(uint64_t n_elems, uint32_t q_bits, size_t *ws_bytes);
int rans_search_reshape(const uint8_t *d_sym, uint64_t n_elems, uint32_t q_bits,
                        rans_reshape_result *d_result, void *d_ws, size_t ws_bytes, void *stream);

/* Parse the fixed 128-byte header on the host.  h_bytes: at least 128 bytes.
 * RANS_ERR_CORRUPT if the fields are not a valid header. */
int rans_peek_header(const void *h_bytes, size_t n_bytes, rans_header *out);

/* First data-dependent error that any call on this workspace has recorded since
 * the previous rans_last_status() on it (RANS_OK if none): a failed call is not
 * hidden by later successful ones.  Reading clears the record.  Synchronises
 * `stream`, on which the calls to be covered must have been enqueued. */
int rans_last_status(void *d_ws, void *stream);

const char *rans_strerror(int code);

/* Diagnostic (not part of the paper's method): runs, on the device, the two
 * division routines with which the frequency-table kernels replace integer
 * division (Sec. 3.2's normalisation and the encoder's reciprocal multipliers of
 * Eq. 2) against the integer division they stand for: floor(2^(32+k) / d) for
 * every d in 1 .. 65535 with 2^k <= d < 2^(k+1), and floor(n / d) for n_random
 * pseudo-random pairs with a quotient below 2^17.  *d_mismatches (device, 4
 * bytes, written by the call) receives the number of disagreements: 0 on a
 * correct build.  Enqueued on `stream`. */
int rans_selftest_divide(uint32_t *d_mismatches, uint64_t n_random, void *stream);

/* Measurement aid for benchmarks (not part of the paper's method): per-kernel
 * launch durations.  rans_profile_enable(mask) makes every later launch of the
 * kernels whose bit (1 << kernel_id) is set record a pair of HIP events on its
 * launch stream (only every `every`-th launch of each kernel, to keep the cost
 * of the event packets out of a timed region; 0 or 1 = every launch); mask 0
 * switches it off (the default: nothing is recorded).
 * rans_profile_read() waits for the recorded events of one kernel and returns
 * their summed elapsed time and their number; rans_profile_reset() forgets all
 * records.  rans_profile_kernel_name() maps ids 0..n-1 to kernel names and
 * returns NULL past the end.  Host only; the event pairs are created on demand. */
int rans_profile_enable(uint64_t kernel_mask, uint32_t every);
int rans_profile_reset(void);
int rans_profile_read(int kernel_id, double *total_ms, uint64_t *count);
const char *rans_profile_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif
