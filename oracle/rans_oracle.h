/*
 * rans_oracle.h -- CPU oracle for the rANS intermediate-feature codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded C
 * implementation of what the codec computes, written from the paper
 * (Sec. 2.1 "Brief Introduction to rANS", Sec. 3.1 "rANS-based Compression
 * Pipeline", Sec. 3.2 Algorithm 1 for the reshape search).  It exists so that tests, the smoke check and the benchmark's
 * cpu_baseline leg can compare the GPU library against it.  Nothing in the
 * product path may include, link or call it, and it shares no code with the
 * GPU library.
 *
 * Every function states the passage it follows.  Where the paper gives no
 * procedure (frequency normalisation, word size of the renormalisation,
 * stream interleaving, container bytes) the function implements this build's
 * format definition; those parts are marked "format definition".
 *
 * Parity pins (see tests/test_oracle_*.py): quantisation invariants and
 * closed-form values, the hand-computed two-symbol example of Eq. 2 / Eq. 4,
 * exact round trip, a big-integer coder written directly from Eq. 2-4,
 * the histogram of D against an independent count,
 * exhaustive brute force over tiny alphabets, CSR brute force, size against
 * the entropy bound of Eq. 1; the reshape cost against an independent numpy /
 * scipy construction, a closed form for K = 1 and a planted column structure,
 * the search against a re-walk of Algorithm 1's rules over those costs.
 * Parity unpinned by the paper (format
 * definitions of this build, checked only for self-consistency): container
 * byte layout, normalisation tie-break rule, chunk/stream assignment.
 */
#ifndef RANS_ORACLE_H
#define RANS_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  ORC_OK = 0,
  ORC_ERR_ARG = -1,       /* null pointer, Q/M/S/dtype/mode out of range      */
  ORC_ERR_SHAPE = -2,     /* rows*cols != T, chunk_syms not a multiple of S   */
  ORC_ERR_ALPHABET = -3,  /* more present symbols than 2^M, or K+1 > 65536    */
  ORC_ERR_CAPACITY = -4,  /* output buffer too small                          */
  ORC_ERR_NONFINITE = -6, /* NaN/Inf in the input, or max-min overflows       */
  ORC_ERR_CORRUPT = -7    /* container fails validation                       */
};

enum { ORC_MODE_DENSE = 0, ORC_MODE_CSR = 1 };
enum { ORC_F32 = 0, ORC_F16 = 1 };

typedef struct {
  uint32_t q_bits;     /* Q of Eq. 6, 1..8                                   */
  uint32_t freq_bits;  /* n of Eq. 2-4 (called M here), 1..15                */
  uint64_t rows, cols; /* N, K of Eq. 5                                      */
  uint32_t mode;       /* ORC_MODE_*                                         */
  uint32_t n_streams;  /* S interleaved coders per chunk                     */
  uint32_t chunk_syms; /* symbols per chunk, multiple of S; 0 = one chunk    */
  uint32_t in_dtype;   /* ORC_F32 / ORC_F16                                  */
} orc_params;

typedef struct {
  float x_min, x_max, scale, zero_point;
} orc_qinfo;

/* fp16 <-> fp32 by the IEEE-754 binary16 definition. */
float orc_half_to_float(uint16_t h);
uint16_t orc_float_to_half(float x);

/* Eq. 6: global extrema of the (widened) tensor. */
int orc_minmax(const void *x, uint64_t n_elems, uint32_t dtype, float *x_min, float *x_max);
/* Eq. 6: scale s and zero point z from the extrema. */
int orc_qinfo_from_minmax(float x_min, float x_max, uint32_t q_bits, orc_qinfo *qi);
/* Eq. 6: one element. */
uint8_t orc_quantize_one(float x, const orc_qinfo *qi, uint32_t q_bits);
/* Eq. 6 over a tensor: extrema, scale, zero point, symbols. */
int orc_quantize(const void *x, uint64_t n_elems, uint32_t dtype, uint32_t q_bits, uint8_t *sym,
                 orc_qinfo *qi);
/* Inverse of Eq. 6 (format definition; the paper prints no formula). */
float orc_dequantize_one(uint8_t sym, const orc_qinfo *qi);
int orc_dequantize(const uint8_t *sym, uint64_t n_elems, const orc_qinfo *qi, uint32_t out_dtype,
                   void *x_out);

/* Sec. 3.1 "Modified CSR Encoding": v, c (nnz each) and non-cumulative r (N).
 * v, c must hold rows*cols entries, r rows entries. */
int orc_csr(const uint8_t *xhat, uint64_t rows, uint64_t cols, uint16_t *v, uint16_t *c,
            uint16_t *r, uint64_t *nnz);
/* Decoder side of the same paragraph: cumulative sum of r, scatter of v. */
int orc_csr_expand(const uint16_t *v, const uint16_t *c, const uint16_t *r, uint64_t nnz,
                   uint64_t rows, uint64_t cols, uint32_t q_bits, uint8_t *xhat);

/* Sec. 3.1 "Concatenation and rANS Encoding": alphabet size of D. */
uint32_t orc_alphabet(uint32_t mode, uint32_t q_bits, uint64_t cols);
/* Same paragraph: one frequency vector over the whole of D. */
void orc_histogram(const uint16_t *D, uint64_t len, uint32_t A, uint64_t *cnt);
/* Format definition: counts -> f with sum 2^M; F = exclusive cumulative sum (A+1 entries). */
int orc_normalize(const uint64_t *cnt, uint32_t A, uint32_t M, uint16_t *f, uint32_t *F);

/* Eq. 2 with 16-bit renormalisation: one encoder step.  Returns 1 and sets
 * *word if a word was emitted before the update. */
int orc_rans_encode_step(uint32_t *state, uint32_t fx, uint32_t Fx, uint32_t M, uint16_t *word);
/* Eq. 3-4: one decoder step without the refill; returns the slot. */
uint32_t orc_rans_decode_step(uint32_t *state, uint32_t fx, uint32_t Fx, uint32_t M);

/* One coder (format definition for the word size and order): symbols
 * D[first + t*stride], t < n, taken last to first from state 2^16; words come
 * back in decoder read order.  words must hold n entries. */
int orc_encode_stream(const uint16_t *D, uint64_t first, uint64_t stride, uint64_t n,
                      const uint16_t *f, const uint32_t *F, uint32_t M, uint16_t *words,
                      uint64_t *n_words, uint32_t *final_state);
/* Its inverse, with validation (final state 2^16, all words consumed). */
int orc_decode_stream(uint32_t state, const uint16_t *words, uint64_t n_words, const uint16_t *f,
                      const uint32_t *F, uint32_t A, uint32_t M, uint16_t *D, uint64_t first,
                      uint64_t stride, uint64_t n);

/* Encode D (len symbols) into a container.  Returns ORC_OK and *out_bytes. */
int orc_encode_container(const uint16_t *D, uint64_t len, const orc_params *p, uint64_t n_elems,
                         float x_min, float x_max, uint8_t *out, size_t out_cap,
                         size_t *out_bytes);
/* The pieces orc_encode_container is made of (also called, chunk by chunk from several threads, by the
 * all-cores timing driver rans_oracle_mt.cpp): fixed header and frequency table; one chunk's states, word
 * counts and words into a buffer of its own (out_cap bytes; *chunk_bytes includes the padding to 4 bytes). */
int orc_write_header_and_table(const orc_params *p, uint64_t n_elems, uint64_t len, float x_min, float x_max,
                               const uint16_t *f, uint8_t *out, size_t out_cap, size_t *dir_off,
                               size_t *payload_off);
int orc_encode_chunk(const uint16_t *D, uint64_t base, uint64_t n_here, uint32_t S, const uint16_t *f,
                     const uint32_t *F, uint32_t M, uint8_t *out, size_t out_cap, size_t *chunk_bytes);
/* Upper bound of the container size for len symbols. */
size_t orc_container_bound(uint64_t len, const orc_params *p, uint64_t n_elems);

typedef struct {
  orc_params p;
  uint64_t n_elems, len_D;
  uint32_t A, n_chunks;
  float x_min, x_max;
  size_t table_off, dir_off, payload_off;
} orc_header;

/* Parse and validate the fixed header only. */
int orc_parse_header(const uint8_t *buf, size_t bytes, orc_header *h);
/* The pieces orc_decode_container is made of: the stored table (validated), one chunk. */
int orc_read_table(const uint8_t *buf, size_t bytes, const orc_header *h, uint16_t *f, uint32_t *F);
int orc_decode_chunk(const uint8_t *buf, size_t bytes, const orc_header *h, uint32_t k, const uint16_t *f,
                     const uint32_t *F, uint16_t *D);
/* Decode a container to D (cap >= len_D), validating everything. */
int orc_decode_container(const uint8_t *buf, size_t bytes, uint16_t *D, uint64_t D_cap,
                         orc_header *h);

/* Sec. 3.2, Eq. 8 with alpha_enc = alpha_dec = 0 (as Algorithm 1 sets them): the size proxy
 * T_tot(N) = l_D * H(p(N)) in bits for the reshape [N, T/N] of the quantised tensor: D and its
 * histogram as orc_csr / orc_histogram give them, H = -sum p log2 p with p = count / l_D, all in
 * binary64, symbols summed in ascending order.  N must divide T and T/N must be at most 65535. */
int orc_reshape_cost(const uint8_t *xhat, uint64_t T, uint64_t N, uint32_t q_bits, double *cost_bits,
                     uint64_t *len_D);
/* Algorithm 1.  Domain: the reshapes [N, K = T/N] with K | T, K <= 2^Q and N > sqrt(T) (the algorithm's
 * N_min = max(floor(sqrt T) + 1, ceil(T / 2^Q)) <= N <= T), in the order of descending N.  Every reshape of the
 * domain is costed with orc_reshape_cost; the reshapes are then looked at in that order up to and including the
 * first one that costs more than its predecessor, and the cheapest one looked at wins (the earliest on equal
 * cost).  cand_N / cand_cost (nullable, cand_cap entries) receive the reshapes looked at and their costs,
 * *n_cand their number.  Empty domain: *N_best = T, *best_cost = +inf, *n_cand = 0. */
int orc_search_reshape(const uint8_t *xhat, uint64_t T, uint32_t q_bits, uint64_t *N_best, double *best_cost,
                       uint64_t *cand_N, double *cand_cost, uint32_t cand_cap, uint32_t *n_cand);

/* Whole path: tensor -> container, container -> symbols / floats. */
int orc_compress(const void *x, uint64_t n_elems, const orc_params *p, uint8_t *out,
                 size_t out_cap, size_t *out_bytes, uint8_t *sym_out /* nullable, T */);
int orc_decompress(const uint8_t *buf, size_t bytes, uint8_t *sym /* T */, uint64_t sym_cap,
                   orc_qinfo *qi, uint32_t out_dtype, void *x_out /* nullable */);

#ifdef __cplusplus
}
#endif
#endif
