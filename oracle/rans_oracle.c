/*
 * rans_oracle.c -- CPU oracle (TEST INFRASTRUCTURE ONLY, see rans_oracle.h).
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 * All floating point below is IEEE binary32 with round-to-nearest-even and no
 * fused multiply-add, because the quantiser's rounding decides an integer and
 * both sides of the parity test must take that decision in the same precision.
 */
#include "rans_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#define RANS_L (1u << 16) /* lower bound of the coder state interval [2^16, 2^32) */

/* ------------------------------------------------------------------ fp16 */

/* IEEE-754 binary16 value by its definition: (-1)^s * 2^(e-15) * (1 + m/1024),
 * subnormals 2^-14 * m/1024, e = 31 -> Inf / NaN. */
float orc_half_to_float(uint16_t h) {
  uint32_t sign = (h >> 15) & 1u, e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
  double v;
  if (e == 0)
    v = ldexp((double)m, -24);
  else if (e == 31)
    v = m ? (double)NAN : (double)INFINITY;
  else
    v = ldexp((double)(m + 1024u), (int)e - 25);
  return (float)(sign ? -v : v);
}

/* Nearest binary16, ties to even, by the definition: pick the exponent, divide
 * by the spacing of that binade (exact: a power of two), round to an integer
 * with the default rounding mode, rebuild. */
uint16_t orc_float_to_half(float x) {
  uint16_t sign = signbit(x) ? 0x8000u : 0u;
  if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
  double a = fabs((double)x);
  if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u); /* halfway to 2^16 rounds to Inf */
  if (a == 0.0) return sign;
  int ex;
  (void)frexp(a, &ex); /* a = m * 2^ex, m in [0.5,1)  ->  floor(log2 a) = ex-1 */
  int e = ex - 1;
  if (e < -14) e = -14; /* subnormal binade shares the spacing of 2^-14 */
  double n = rint(ldexp(a, 10 - e)); /* a / 2^(e-10), an integer in [0, 2048] */
  /* Normal numbers have n in [1024, 2048] (2048 carries into the exponent field);
   * in the lowest binade e + 15 = 1, so the same expression yields n itself,
   * which is the subnormal encoding when n < 1024. */
  uint32_t bits = ((uint32_t)(e + 15) << 10) + (uint32_t)n - 1024u;
  return (uint16_t)(sign | bits);
}

static float load_elem(const void *x, uint64_t i, uint32_t dtype) {
  if (dtype == ORC_F16) return orc_half_to_float(((const uint16_t *)x)[i]);
  return ((const float *)x)[i];
}

/* ----------------------------------------------------- Eq. 6: quantisation */

/* Eq. 6 uses scalar x_min, x_max: extrema over the whole tensor.
 * Format definition: non-finite input is an error; -0.0 extrema are stored as
 * +0.0; the empty tensor has x_min = x_max = 0. */
int orc_minmax(const void *x, uint64_t n, uint32_t dtype, float *x_min, float *x_max) {
  if (!x_min || !x_max || (n && !x) || dtype > ORC_F16) return ORC_ERR_ARG;
  float mn = 0.0f, mx = 0.0f;
  for (uint64_t i = 0; i < n; i++) {
    float v = load_elem(x, i, dtype);
    if (!isfinite(v)) return ORC_ERR_NONFINITE;
    if (i == 0) {
      mn = v;
      mx = v;
    }
    if (v < mn) mn = v;
    if (v > mx) mx = v;
  }
  *x_min = mn + 0.0f;
  *x_max = mx + 0.0f;
  return ORC_OK;
}

/* Eq. 6: s = (x_max - x_min) / (2^Q - 1), z = round(-x_min / s).
 * z is kept as an integer-valued float.  Format definition: round = nearest,
 * ties to even; a tensor whose range is 0 (or so small that s underflows to 0)
 * has s = 0, z = 0 and every symbol 0. */
int orc_qinfo_from_minmax(float x_min, float x_max, uint32_t q_bits, orc_qinfo *qi) {
  if (!qi || q_bits < 1 || q_bits > 8) return ORC_ERR_ARG;
  if (!isfinite(x_min) || !isfinite(x_max) || x_min > x_max) return ORC_ERR_NONFINITE;
  float range = x_max - x_min;
  if (!isfinite(range)) return ORC_ERR_NONFINITE;
  float levels = (float)((1u << q_bits) - 1u);
  float s = range / levels;
  float zf = 0.0f;
  if (s != 0.0f) {
    float neg_min = 0.0f - x_min;
    float q = neg_min / s;
    zf = rintf(q);
  }
  qi->x_min = x_min;
  qi->x_max = x_max;
  qi->scale = s;
  qi->zero_point = zf;
  return ORC_OK;
}

/* Eq. 6: xhat = round(x / s + z), kept inside {0..2^Q-1} as the sentence after
 * the equation requires. */
uint8_t orc_quantize_one(float x, const orc_qinfo *qi, uint32_t q_bits) {
  if (qi->scale == 0.0f) return 0;
  float levels = (float)((1u << q_bits) - 1u);
  float t = x / qi->scale;
  float u = t + qi->zero_point;
  float r = rintf(u);
  if (r < 0.0f) r = 0.0f;
  if (r > levels) r = levels;
  return (uint8_t)r;
}

int orc_quantize(const void *x, uint64_t n, uint32_t dtype, uint32_t q_bits, uint8_t *sym,
                 orc_qinfo *qi) {
  if (!qi || (n && (!x || !sym)) || q_bits < 1 || q_bits > 8 || dtype > ORC_F16)
    return ORC_ERR_ARG;
  float mn, mx;
  int rc = orc_minmax(x, n, dtype, &mn, &mx);
  if (rc) return rc;
  rc = orc_qinfo_from_minmax(mn, mx, q_bits, qi);
  if (rc) return rc;
  for (uint64_t i = 0; i < n; i++) sym[i] = orc_quantize_one(load_elem(x, i, dtype), qi, q_bits);
  return ORC_OK;
}

/* Inverse of Eq. 6 solved for x: x ~ s * (xhat - z).  One subtraction, one
 * multiplication, each rounded to binary32.  With s = 0 every element is x_min. */
float orc_dequantize_one(uint8_t sym, const orc_qinfo *qi) {
  if (qi->scale == 0.0f) return qi->x_min;
  float d = (float)sym - qi->zero_point;
  float y = qi->scale * d;
  return y;
}

int orc_dequantize(const uint8_t *sym, uint64_t n, const orc_qinfo *qi, uint32_t out_dtype,
                   void *x_out) {
  if (!qi || (n && (!sym || !x_out)) || out_dtype > ORC_F16) return ORC_ERR_ARG;
  for (uint64_t i = 0; i < n; i++) {
    float y = orc_dequantize_one(sym[i], qi);
    if (out_dtype == ORC_F16)
      ((uint16_t *)x_out)[i] = orc_float_to_half(y);
    else
      ((float *)x_out)[i] = y;
  }
  return ORC_OK;
}

/* ------------------------------------------- Sec. 3.1: modified CSR (v,c,r) */

/* Eq. 5 views the flat tensor as N rows of K columns (row-major).  The
 * quantised matrix is stored as v = nonzero values, c = their column indices,
 * r[i] = number of nonzeros of row i (NOT cumulative).  "Nonzero" refers to the
 * quantised symbol. */
int orc_csr(const uint8_t *xhat, uint64_t rows, uint64_t cols, uint16_t *v, uint16_t *c,
            uint16_t *r, uint64_t *nnz) {
  if (!nnz || cols < 1 || cols > 65535) return ORC_ERR_ARG;
  uint64_t j = 0;
  for (uint64_t i = 0; i < rows; i++) {
    uint64_t count = 0;
    for (uint64_t k = 0; k < cols; k++) {
      uint8_t a = xhat[i * cols + k];
      if (a != 0) {
        v[j] = a;
        c[j] = (uint16_t)k;
        j++;
        count++;
      }
    }
    r[i] = (uint16_t)count;
  }
  *nnz = j;
  return ORC_OK;
}

/* The cumulative sum of r is taken here, on the decoding side; v is scattered
 * to (row, c).  Everything a well-formed (v,c,r) satisfies is checked. */
int orc_csr_expand(const uint16_t *v, const uint16_t *c, const uint16_t *r, uint64_t nnz,
                   uint64_t rows, uint64_t cols, uint32_t q_bits, uint8_t *xhat) {
  uint64_t total = 0;
  for (uint64_t i = 0; i < rows; i++) {
    if (r[i] > cols) return ORC_ERR_CORRUPT;
    total += r[i];
  }
  if (total != nnz) return ORC_ERR_CORRUPT;
  memset(xhat, 0, (size_t)(rows * cols));
  uint64_t off = 0; /* running cumulative sum of r */
  for (uint64_t i = 0; i < rows; i++) {
    for (uint64_t t = 0; t < r[i]; t++) {
      uint64_t j = off + t;
      if (v[j] == 0 || v[j] >= (1u << q_bits)) return ORC_ERR_CORRUPT;
      if (c[j] >= cols) return ORC_ERR_CORRUPT;
      if (t > 0 && c[j] <= c[j - 1]) return ORC_ERR_CORRUPT;
      xhat[i * cols + c[j]] = (uint8_t)v[j];
    }
    off += r[i];
  }
  return ORC_OK;
}

/* ------------------------------------- Sec. 3.1: alphabet, frequency vector */

/* v takes values up to 2^Q - 1, c up to K - 1, r up to K: the number of
 * distinct symbol values is max(2^Q, K + 1).  DENSE mode codes xhat itself. */
uint32_t orc_alphabet(uint32_t mode, uint32_t q_bits, uint64_t cols) {
  uint32_t a = 1u << q_bits;
  if (mode == ORC_MODE_CSR && cols + 1 > a) a = (uint32_t)(cols + 1);
  return a;
}

/* One table for all of D: the histograms of v, c and r padded to a common
 * length and summed are the histogram of their concatenation. */
void orc_histogram(const uint16_t *D, uint64_t len, uint32_t A, uint64_t *cnt) {
  for (uint32_t a = 0; a < A; a++) cnt[a] = 0;
  for (uint64_t i = 0; i < len; i++) cnt[D[i]]++;
}

/* Format definition (Eq. 2-4 need sum f = 2^n but the paper gives no rule):
 *   f[a] = 0 if cnt[a] = 0, else max(1, floor((cnt[a]*2^M + floor(len/2)) / len));
 *   d = 2^M - sum f;
 *   d > 0: add d to the symbol with the largest count (lowest index on ties);
 *   d < 0: repeatedly take from the symbol with the largest f (lowest index on
 *          ties) as much as possible while leaving it at 1.
 * An empty D gives an all-zero table. */
int orc_normalize(const uint64_t *cnt, uint32_t A, uint32_t M, uint16_t *f, uint32_t *F) {
  if (M < 1 || M > 15 || A < 1 || A > 65536) return ORC_ERR_ARG;
  uint64_t len = 0, present = 0;
  for (uint32_t a = 0; a < A; a++) {
    len += cnt[a];
    present += cnt[a] ? 1 : 0;
  }
  uint64_t total = (uint64_t)1 << M;
  if (present > total) return ORC_ERR_ALPHABET;
  int64_t sum = 0;
  uint64_t *g = (uint64_t *)calloc(A, sizeof(uint64_t));
  if (!g) return ORC_ERR_ARG;
  for (uint32_t a = 0; a < A; a++) {
    if (cnt[a]) {
      uint64_t q = (cnt[a] * total + len / 2) / len;
      g[a] = q < 1 ? 1 : q;
      sum += (int64_t)g[a];
    }
  }
  int64_t d = (int64_t)total - sum;
  if (len && d > 0) {
    uint32_t best = 0;
    for (uint32_t a = 1; a < A; a++)
      if (cnt[a] > cnt[best]) best = a;
    g[best] += (uint64_t)d;
    d = 0;
  }
  while (d < 0) {
    uint32_t best = 0;
    for (uint32_t a = 1; a < A; a++)
      if (g[a] > g[best]) best = a;
    int64_t take = (int64_t)g[best] - 1;
    if (take > -d) take = -d;
    g[best] -= (uint64_t)take;
    d += take;
  }
  uint32_t acc = 0;
  for (uint32_t a = 0; a < A; a++) {
    f[a] = (uint16_t)g[a];
    F[a] = acc;
    acc += (uint32_t)g[a];
  }
  F[A] = acc;
  free(g);
  return ORC_OK;
}

/* ------------------------------------------------ Eq. 2-4: the rANS coder */

/* Renormalisation paragraph of Sec. 2.1 ("limit[x]"): the state lives in
 * [2^16, 2^32).  If it is too large for the upcoming symbol, i.e.
 * s >= f(x) * 2^(32-M), its low 16 bits are emitted and it is shifted right by
 * 16 (once is always enough).  Then Eq. 2:
 *   s' = floor(s / f) * 2^M + F + (s mod f). */
int orc_rans_encode_step(uint32_t *state, uint32_t fx, uint32_t Fx, uint32_t M, uint16_t *word) {
  uint32_t s = *state;
  int emitted = 0;
  if ((uint64_t)s >= ((uint64_t)fx << (32 - M))) {
    *word = (uint16_t)(s & 0xffffu);
    s >>= 16;
    emitted = 1;
  }
  *state = (s / fx) * (1u << M) + Fx + (s % fx);
  return emitted;
}

/* Eq. 4: s_prev = f * floor(s / 2^M) + (s mod 2^M) - F.  The caller has already
 * selected the symbol by Eq. 3 from slot = s mod 2^M. */
uint32_t orc_rans_decode_step(uint32_t *state, uint32_t fx, uint32_t Fx, uint32_t M) {
  uint32_t s = *state;
  uint32_t slot = s & ((1u << M) - 1u);
  *state = fx * (s >> M) + slot - Fx;
  return slot;
}

/* Eq. 3: the symbol t with F(t) <= slot < F(t+1), by linear search. */
static uint32_t symbol_of_slot(const uint32_t *F, uint32_t A, uint32_t slot) {
  for (uint32_t t = 0; t < A; t++)
    if (F[t] <= slot && slot < F[t + 1]) return t;
  return A; /* not reachable when F[A] = 2^M */
}

/* One coder over the symbols D[first], D[first+stride], ... (n of them).
 * Starts at state 2^16, takes the symbols last to first (so that the decoder
 * produces them first to last), and returns the emitted words in the order the
 * decoder reads them, i.e. the reverse of the order of emission. */
int orc_encode_stream(const uint16_t *D, uint64_t first, uint64_t stride, uint64_t n,
                      const uint16_t *f, const uint32_t *F, uint32_t M, uint16_t *words,
                      uint64_t *n_words, uint32_t *final_state) {
  uint32_t s = RANS_L;
  uint64_t e = 0;
  for (uint64_t t = n; t-- > 0;) {
    uint16_t x = D[first + t * stride];
    if (f[x] == 0) return ORC_ERR_ARG;
    uint16_t w;
    if (orc_rans_encode_step(&s, f[x], F[x], M, &w)) words[e++] = w;
  }
  for (uint64_t i = 0; i < e / 2; i++) { /* emission order -> read order */
    uint16_t tmp = words[i];
    words[i] = words[e - 1 - i];
    words[e - 1 - i] = tmp;
  }
  *n_words = e;
  *final_state = s;
  return ORC_OK;
}

/* Inverse: start from the stored state; per symbol: slot = s mod 2^M, symbol by
 * Eq. 3, state by Eq. 4, and if the state fell below 2^16 shift in the next
 * 16-bit word.  After the last symbol the state must be back at 2^16 with every
 * word consumed. */
int orc_decode_stream(uint32_t state, const uint16_t *words, uint64_t n_words, const uint16_t *f,
                      const uint32_t *F, uint32_t A, uint32_t M, uint16_t *D, uint64_t first,
                      uint64_t stride, uint64_t n) {
  uint32_t s = state;
  uint64_t used = 0;
  for (uint64_t t = 0; t < n; t++) {
    if (s < RANS_L) return ORC_ERR_CORRUPT;
    uint32_t slot = s & ((1u << M) - 1u);
    uint32_t x = symbol_of_slot(F, A, slot);
    if (x >= A) return ORC_ERR_CORRUPT;
    (void)orc_rans_decode_step(&s, f[x], F[x], M);
    if (s < RANS_L) {
      if (used >= n_words) return ORC_ERR_CORRUPT;
      s = (s << 16) | words[used++];
    }
    D[first + t * stride] = (uint16_t)x;
  }
  if (s != RANS_L || used != n_words) return ORC_ERR_CORRUPT;
  return ORC_OK;
}

/* ------------------------------------------------------------ container */

static void put16(uint8_t *p, uint32_t v) {
  p[0] = (uint8_t)v;
  p[1] = (uint8_t)(v >> 8);
}
static void put32(uint8_t *p, uint32_t v) {
  put16(p, v & 0xffffu);
  put16(p + 2, v >> 16);
}
static void put64(uint8_t *p, uint64_t v) {
  put32(p, (uint32_t)v);
  put32(p + 4, (uint32_t)(v >> 32));
}
static uint32_t get16(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static uint32_t get32(const uint8_t *p) { return get16(p) | (get16(p + 2) << 16); }
static uint64_t get64(const uint8_t *p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }

#define HDR_BYTES 128u

static uint64_t n_chunks_of(uint64_t len, uint32_t chunk_syms) {
  if (len == 0) return 0;
  if (chunk_syms == 0) return 1;
  return (len + chunk_syms - 1) / chunk_syms;
}

static int check_params(const orc_params *p, uint64_t n_elems) {
  if (!p) return ORC_ERR_ARG;
  if (p->q_bits < 1 || p->q_bits > 8 || p->freq_bits < 1 || p->freq_bits > 15) return ORC_ERR_ARG;
  if (p->mode > ORC_MODE_CSR || p->in_dtype > ORC_F16) return ORC_ERR_ARG;
  if (p->n_streams < 1 || p->n_streams > 65536) return ORC_ERR_ARG;
  if (p->cols < 1) return ORC_ERR_SHAPE;
  if (p->rows != n_elems / p->cols || p->rows * p->cols != n_elems) return ORC_ERR_SHAPE;
  if (p->chunk_syms % p->n_streams != 0) return ORC_ERR_SHAPE;
  if (p->mode == ORC_MODE_CSR && p->cols + 1 > 65536) return ORC_ERR_ALPHABET;
  return ORC_OK;
}

size_t orc_container_bound(uint64_t len, const orc_params *p, uint64_t n_elems) {
  (void)n_elems;
  uint32_t A = orc_alphabet(p->mode, p->q_bits, p->cols);
  uint64_t nc = n_chunks_of(len, p->chunk_syms);
  uint64_t b = HDR_BYTES + (((uint64_t)A * 2 + 7) & ~(uint64_t)7) + 8 * (nc + 1);
  b += nc * (8ull * p->n_streams + 4) + 2 * len;
  return (size_t)b;
}

int orc_write_header_and_table(const orc_params *p, uint64_t n_elems, uint64_t len, float x_min, float x_max,
                               const uint16_t *f, uint8_t *out, size_t out_cap, size_t *dir_off_out,
                               size_t *payload_off_out) {
  uint32_t A = orc_alphabet(p->mode, p->q_bits, p->cols), M = p->freq_bits, S = p->n_streams;
  uint64_t nc64 = n_chunks_of(len, p->chunk_syms);
  if (nc64 > 0xffffffffull) return ORC_ERR_ARG;
  uint32_t nc = (uint32_t)nc64;
  size_t table_off = HDR_BYTES;
  size_t dir_off = table_off + (((size_t)A * 2 + 7) & ~(size_t)7);
  size_t payload_off = dir_off + 8 * ((size_t)nc + 1);
  if (payload_off > out_cap) return ORC_ERR_CAPACITY;
  memset(out, 0, payload_off);
  memcpy(out, "RIF1", 4);
  put16(out + 4, 1);
  out[6] = (uint8_t)p->mode;
  out[7] = (uint8_t)p->in_dtype;
  out[8] = (uint8_t)p->q_bits;
  out[9] = (uint8_t)M;
  put64(out + 12, n_elems);
  put64(out + 20, p->rows);
  put64(out + 28, p->cols);
  put64(out + 36, len);
  put32(out + 44, A);
  put32(out + 48, S);
  put32(out + 52, p->chunk_syms);
  put32(out + 56, nc);
  uint32_t bits;
  memcpy(&bits, &x_min, 4);
  put32(out + 60, bits);
  memcpy(&bits, &x_max, 4);
  put32(out + 64, bits);
  for (uint32_t a = 0; a < A; a++) put16(out + table_off + 2 * (size_t)a, f[a]);
  *dir_off_out = dir_off;
  *payload_off_out = payload_off;
  return ORC_OK;
}

/* One chunk: state[S] u32, nwords[S] u32, then the streams' words one stream after the other, zero-padded to
 * a multiple of 4 bytes.  Stream j codes the chunk's local symbols j, j + S, j + 2S, ... */
int orc_encode_chunk(const uint16_t *D, uint64_t base, uint64_t n_here, uint32_t S, const uint16_t *f,
                     const uint32_t *F, uint32_t M, uint8_t *out, size_t out_cap, size_t *chunk_bytes) {
  size_t wpos = 8 * (size_t)S;
  if (wpos > out_cap) return ORC_ERR_CAPACITY;
  uint16_t *tmp = NULL;
  size_t tmp_cap = 0;
  int rc = ORC_OK;
  for (uint32_t j = 0; j < S; j++) {
    uint64_t n_j = n_here > j ? (n_here - j + S - 1) / S : 0;
    if (n_j > tmp_cap) {
      free(tmp);
      tmp_cap = (size_t)n_j;
      tmp = (uint16_t *)malloc(tmp_cap * sizeof(uint16_t));
    }
    uint32_t s;
    uint64_t e;
    rc = orc_encode_stream(D, base + j, S, n_j, f, F, M, tmp, &e, &s);
    if (rc) break;
    if (wpos + 2 * e > out_cap) {
      rc = ORC_ERR_CAPACITY;
      break;
    }
    put32(out + 4 * (size_t)j, s);
    put32(out + 4 * (size_t)S + 4 * (size_t)j, (uint32_t)e);
    for (uint64_t i = 0; i < e; i++) put16(out + wpos + 2 * i, tmp[i]);
    wpos += 2 * e;
  }
  free(tmp);
  if (rc) return rc;
  while (wpos % 4 != 0) {
    if (wpos >= out_cap) return ORC_ERR_CAPACITY;
    out[wpos++] = 0;
  }
  *chunk_bytes = wpos;
  return ORC_OK;
}

/* Format definition.  Little-endian:
 *   0 "RIF1" | 4 version u16 = 1 | 6 mode u8 | 7 in_dtype u8 | 8 Q u8 | 9 M u8 |
 *   10 reserved u16 | 12 T u64 | 20 N u64 | 28 K u64 | 36 len_D u64 | 44 A u32 |
 *   48 S u32 | 52 chunk_syms u32 | 56 n_chunks u32 | 60 x_min f32 | 64 x_max f32 |
 *   68..127 zero | f[0..A) u16, zero-padded to 8 B | off[0..n_chunks] u64 (from
 *   payload start) | per chunk: state[S] u32, nwords[S] u32, stream 0 words,
 *   stream 1 words, ... (u16), chunk zero-padded to 4 B.
 * D is cut into chunks of chunk_syms symbols; inside a chunk local symbol i
 * belongs to stream i mod S.  Each stream is one coder: it starts at state 2^16,
 * takes its symbols last to first, and its words are stored in the order the
 * decoder reads them (reverse of emission).  The final state is stored whole. */
int orc_encode_container(const uint16_t *D, uint64_t len, const orc_params *p, uint64_t n_elems,
                         float x_min, float x_max, uint8_t *out, size_t out_cap,
                         size_t *out_bytes) {
  int rc = check_params(p, n_elems);
  if (rc) return rc;
  if (!out || !out_bytes || (len && !D)) return ORC_ERR_ARG;
  uint32_t A = orc_alphabet(p->mode, p->q_bits, p->cols), M = p->freq_bits, S = p->n_streams;
  uint64_t nc64 = n_chunks_of(len, p->chunk_syms);
  if (nc64 > 0xffffffffull) return ORC_ERR_ARG;
  uint32_t nc = (uint32_t)nc64;
  for (uint64_t i = 0; i < len; i++)
    if (D[i] >= A) return ORC_ERR_ARG;

  uint64_t *cnt = (uint64_t *)calloc(A, sizeof(uint64_t));
  uint16_t *f = (uint16_t *)calloc(A, sizeof(uint16_t));
  uint32_t *F = (uint32_t *)calloc((size_t)A + 1, sizeof(uint32_t));
  orc_histogram(D, len, A, cnt);
  rc = orc_normalize(cnt, A, M, f, F);
  free(cnt);
  size_t dir_off = 0, payload_off = 0;
  if (rc == ORC_OK) rc = orc_write_header_and_table(p, n_elems, len, x_min, x_max, f, out, out_cap, &dir_off, &payload_off);
  if (rc) {
    free(f);
    free(F);
    return rc;
  }
  uint64_t chunk_len = p->chunk_syms ? p->chunk_syms : len;
  size_t pos = payload_off; /* absolute write position */
  for (uint32_t k = 0; k < nc && rc == ORC_OK; k++) {
    put64(out + dir_off + 8 * (size_t)k, (uint64_t)(pos - payload_off));
    uint64_t base = (uint64_t)k * chunk_len;
    uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
    size_t ck_bytes = 0;
    rc = orc_encode_chunk(D, base, n_here, S, f, F, M, out + pos, out_cap - pos, &ck_bytes);
    if (rc == ORC_OK) pos += ck_bytes;
  }
  if (rc == ORC_OK) {
    put64(out + dir_off + 8 * (size_t)nc, (uint64_t)(pos - payload_off));
    *out_bytes = pos;
  }
  free(f);
  free(F);
  return rc;
}

int orc_parse_header(const uint8_t *buf, size_t bytes, orc_header *h) {
  if (!buf || !h) return ORC_ERR_ARG;
  if (bytes < HDR_BYTES) return ORC_ERR_CORRUPT;
  if (memcmp(buf, "RIF1", 4) != 0 || get16(buf + 4) != 1) return ORC_ERR_CORRUPT;
  memset(h, 0, sizeof(*h));
  h->p.mode = buf[6];
  h->p.in_dtype = buf[7];
  h->p.q_bits = buf[8];
  h->p.freq_bits = buf[9];
  if (get16(buf + 10) != 0) return ORC_ERR_CORRUPT;
  h->n_elems = get64(buf + 12);
  h->p.rows = get64(buf + 20);
  h->p.cols = get64(buf + 28);
  h->len_D = get64(buf + 36);
  h->A = get32(buf + 44);
  h->p.n_streams = get32(buf + 48);
  h->p.chunk_syms = get32(buf + 52);
  h->n_chunks = get32(buf + 56);
  uint32_t bits = get32(buf + 60);
  memcpy(&h->x_min, &bits, 4);
  bits = get32(buf + 64);
  memcpy(&h->x_max, &bits, 4);
  for (size_t i = 68; i < HDR_BYTES; i++)
    if (buf[i] != 0) return ORC_ERR_CORRUPT;
  if (h->n_elems >> 40) return ORC_ERR_CORRUPT; /* keeps every product below in range */
  if (h->p.cols >> 40 || h->p.rows >> 40) return ORC_ERR_CORRUPT;
  if (check_params(&h->p, h->n_elems) != ORC_OK) return ORC_ERR_CORRUPT;
  if (!isfinite(h->x_min) || !isfinite(h->x_max) || h->x_min > h->x_max) return ORC_ERR_CORRUPT;
  if (h->A != orc_alphabet(h->p.mode, h->p.q_bits, h->p.cols)) return ORC_ERR_CORRUPT;
  if (h->p.mode == ORC_MODE_DENSE) {
    if (h->len_D != h->n_elems) return ORC_ERR_CORRUPT;
  } else {
    if (h->len_D < h->p.rows || (h->len_D - h->p.rows) % 2 != 0) return ORC_ERR_CORRUPT;
    if ((h->len_D - h->p.rows) / 2 > h->n_elems) return ORC_ERR_CORRUPT;
  }
  if ((uint64_t)h->n_chunks != n_chunks_of(h->len_D, h->p.chunk_syms)) return ORC_ERR_CORRUPT;
  h->table_off = HDR_BYTES;
  h->dir_off = h->table_off + (((size_t)h->A * 2 + 7) & ~(size_t)7);
  h->payload_off = h->dir_off + 8 * ((size_t)h->n_chunks + 1);
  if (h->payload_off > bytes) return ORC_ERR_CORRUPT;
  return ORC_OK;
}

/* Reads the stored table back and checks it (sum 2^M, or 0 for an empty D; zero padding) together with the two
 * ends of the chunk directory.  f: A entries, F: A + 1. */
int orc_read_table(const uint8_t *buf, size_t bytes, const orc_header *h, uint16_t *f, uint32_t *F) {
  uint32_t A = h->A, M = h->p.freq_bits, nc = h->n_chunks;
  uint32_t acc = 0;
  for (uint32_t a = 0; a < A; a++) {
    f[a] = (uint16_t)get16(buf + h->table_off + 2 * (size_t)a);
    F[a] = acc;
    acc += f[a];
  }
  F[A] = acc;
  for (size_t i = h->table_off + 2 * (size_t)A; i < h->dir_off; i++)
    if (buf[i] != 0) return ORC_ERR_CORRUPT;
  if (acc != (h->len_D ? (1u << M) : 0u)) return ORC_ERR_CORRUPT;
  size_t payload_bytes = bytes - h->payload_off;
  if (get64(buf + h->dir_off) != 0) return ORC_ERR_CORRUPT;
  if (get64(buf + h->dir_off + 8 * (size_t)nc) != payload_bytes) return ORC_ERR_CORRUPT;
  return ORC_OK;
}

/* Chunk k of a container whose header and table have been read: every size and offset is checked. */
int orc_decode_chunk(const uint8_t *buf, size_t bytes, const orc_header *h, uint32_t k, const uint16_t *f,
                     const uint32_t *F, uint16_t *D) {
  uint32_t A = h->A, M = h->p.freq_bits, S = h->p.n_streams;
  size_t payload_bytes = bytes - h->payload_off;
  uint64_t chunk_len = h->p.chunk_syms ? h->p.chunk_syms : h->len_D;
  uint64_t o0 = get64(buf + h->dir_off + 8 * (size_t)k);
  uint64_t o1 = get64(buf + h->dir_off + 8 * ((size_t)k + 1));
  if (o0 > o1 || o1 > payload_bytes || o1 - o0 < 8ull * S) return ORC_ERR_CORRUPT;
  const uint8_t *ck = buf + h->payload_off + o0;
  uint64_t ck_bytes = o1 - o0;
  uint64_t base = (uint64_t)k * chunk_len;
  uint64_t n_here = h->len_D - base < chunk_len ? h->len_D - base : chunk_len;
  uint64_t wpos = 8ull * S;
  uint16_t *wtmp = NULL;
  size_t wtmp_cap = 0;
  int rc = ORC_OK;
  for (uint32_t j = 0; j < S && rc == ORC_OK; j++) {
    uint64_t n_j = n_here > j ? (n_here - j + S - 1) / S : 0;
    uint32_t s = get32(ck + 4 * (size_t)j);
    uint64_t nw = get32(ck + 4 * (size_t)S + 4 * (size_t)j);
    if (nw > n_j || wpos + 2 * nw > ck_bytes) {
      rc = ORC_ERR_CORRUPT;
      break;
    }
    if (nw > wtmp_cap) {
      free(wtmp);
      wtmp_cap = (size_t)nw;
      wtmp = (uint16_t *)malloc(wtmp_cap * sizeof(uint16_t));
    }
    for (uint64_t i = 0; i < nw; i++) wtmp[i] = (uint16_t)get16(ck + wpos + 2 * i);
    rc = orc_decode_stream(s, wtmp, nw, f, F, A, M, D, base + j, S, n_j);
    if (rc) break;
    wpos += 2 * nw;
  }
  free(wtmp);
  if (rc) return rc;
  uint64_t padded = (wpos + 3) & ~(uint64_t)3;
  if (padded != ck_bytes) return ORC_ERR_CORRUPT;
  for (uint64_t i = wpos; i < ck_bytes; i++)
    if (ck[i] != 0) return ORC_ERR_CORRUPT;
  return ORC_OK;
}

/* Inverse of orc_encode_container: every field is re-read and checked. */
int orc_decode_container(const uint8_t *buf, size_t bytes, uint16_t *D, uint64_t D_cap,
                         orc_header *h) {
  int rc = orc_parse_header(buf, bytes, h);
  if (rc) return rc;
  if (h->len_D > D_cap) return ORC_ERR_CAPACITY;
  if (h->len_D && !D) return ORC_ERR_ARG;
  uint32_t A = h->A, nc = h->n_chunks;
  uint16_t *f = (uint16_t *)calloc(A, sizeof(uint16_t));
  uint32_t *F = (uint32_t *)calloc((size_t)A + 1, sizeof(uint32_t));
  rc = orc_read_table(buf, bytes, h, f, F);
  for (uint32_t k = 0; k < nc && rc == ORC_OK; k++) rc = orc_decode_chunk(buf, bytes, h, k, f, F, D);
  free(f);
  free(F);
  return rc;
}

/* ---------------------------------------------------------- whole path */

/* ---------------------------------------------------------------- Sec. 3.2: reshape search */

int orc_reshape_cost(const uint8_t *xhat, uint64_t T, uint64_t N, uint32_t q_bits, double *cost_bits,
                     uint64_t *len_D) {
  if (!xhat || !cost_bits || T == 0 || N == 0 || T % N != 0 || q_bits < 1 || q_bits > 8) return ORC_ERR_ARG;
  const uint64_t K = T / N;
  if (K > 65535) return ORC_ERR_ARG;
  uint16_t *v = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
  uint16_t *c = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)T);
  uint16_t *r = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)N);
  if (!v || !c || !r) {
    free(v); free(c); free(r);
    return ORC_ERR_ARG;
  }
  uint64_t nnz = 0;
  int rc = orc_csr(xhat, N, K, v, c, r, &nnz);
  if (rc) {
    free(v); free(c); free(r);
    return rc;
  }
  /* one histogram over D = v (+) c (+) r (Eq. 7) */
  const uint32_t two_q = 1u << q_bits;
  const uint32_t A = (uint32_t)(K + 1 > two_q ? K + 1 : two_q);
  uint64_t *cnt = (uint64_t *)calloc(A, sizeof(uint64_t));
  if (!cnt) {
    free(v); free(c); free(r);
    return ORC_ERR_ARG;
  }
  for (uint64_t j = 0; j < nnz; j++) cnt[v[j]]++;
  for (uint64_t j = 0; j < nnz; j++) cnt[c[j]]++;
  for (uint64_t i = 0; i < N; i++) cnt[r[i]]++;
  const uint64_t len = 2 * nnz + N;
  double H = 0.0;
  for (uint32_t a = 0; a < A; a++) {
    if (cnt[a]) {
      const double p = (double)cnt[a] / (double)len;
      H -= p * log2(p);
    }
  }
  *cost_bits = (double)len * H;
  if (len_D) *len_D = len;
  free(cnt); free(v); free(c); free(r);
  return ORC_OK;
}

static uint64_t isqrt_u64(uint64_t t) {
  uint64_t r = (uint64_t)sqrt((double)t);
  while (r * r > t) r--;
  while ((r + 1) * (r + 1) <= t) r++;
  return r;
}

/* Sec. 3.2: the search domain is every reshape [N, K] with K a divisor of T, K <= 2^Q (so that a column
 * index is no wider than a value) and N = T / K > sqrt(T) (more rows than columns); Algorithm 1 writes the
 * same set as N_min = max(floor(sqrt T) + 1, ceil(T / 2^Q)) <= N <= T.  It is listed here by ascending K,
 * which is the order the algorithm visits it in (N descending). */
static uint32_t reshape_domain(uint64_t T, uint32_t q_bits, uint64_t *dom_N, uint32_t cap) {
  const uint64_t root = isqrt_u64(T);
  uint32_t n = 0;
  for (uint64_t K = 1; K <= (1ull << q_bits) && K <= T; K++) {
    if (T % K != 0) continue;
    if (T / K <= root) continue; /* N > sqrt(T) fails, and does so for every larger K too */
    if (n < cap) dom_N[n] = T / K;
    n++;
  }
  return n;
}

int orc_search_reshape(const uint8_t *xhat, uint64_t T, uint32_t q_bits, uint64_t *N_best, double *best_cost,
                       uint64_t *cand_N, double *cand_cost, uint32_t cand_cap, uint32_t *n_cand) {
  if (!xhat || !N_best || !best_cost || T == 0 || q_bits < 1 || q_bits > 8) return ORC_ERR_ARG;
  enum { DOM_MAX = 256 }; /* K <= 2^Q <= 256 */
  uint64_t dom_N[DOM_MAX];
  double dom_cost[DOM_MAX];
  const uint32_t n_dom = reshape_domain(T, q_bits, dom_N, DOM_MAX);
  /* the size proxy of every reshape in the domain */
  for (uint32_t i = 0; i < n_dom; i++) {
    int rc = orc_reshape_cost(xhat, T, dom_N[i], q_bits, &dom_cost[i], NULL);
    if (rc) return rc;
  }
  /* the stop rule: the reshapes are looked at in order until one costs more than the one before it (that one
   * is still looked at); the cheapest one seen wins, the earliest on equal cost */
  uint32_t seen = n_dom;
  for (uint32_t i = 1; i < n_dom; i++) {
    if (dom_cost[i] > dom_cost[i - 1]) {
      seen = i + 1;
      break;
    }
  }
  uint32_t arg = 0;
  for (uint32_t i = 1; i < seen; i++)
    if (dom_cost[i] < dom_cost[arg]) arg = i;
  *N_best = seen ? dom_N[arg] : T;
  *best_cost = seen ? dom_cost[arg] : INFINITY;
  for (uint32_t i = 0; i < seen && i < cand_cap; i++) {
    if (cand_N) cand_N[i] = dom_N[i];
    if (cand_cost) cand_cost[i] = dom_cost[i];
  }
  if (n_cand) *n_cand = seen;
  return ORC_OK;
}

/* Fig. 1(c): reshape + quantise (Eq. 5-6), modified CSR, D = v (+) c (+) r
 * (Eq. 7; DENSE mode: D = xhat), one frequency table, rANS. */
int orc_compress(const void *x, uint64_t n, const orc_params *p, uint8_t *out, size_t out_cap,
                 size_t *out_bytes, uint8_t *sym_out) {
  int rc = check_params(p, n);
  if (rc) return rc;
  uint8_t *sym = (uint8_t *)malloc(n ? (size_t)n : 1);
  orc_qinfo qi;
  rc = orc_quantize(x, n, p->in_dtype, p->q_bits, sym, &qi);
  if (rc) {
    free(sym);
    return rc;
  }
  if (sym_out) memcpy(sym_out, sym, (size_t)n);
  uint16_t *D;
  uint64_t len;
  if (p->mode == ORC_MODE_DENSE) {
    len = n;
    D = (uint16_t *)malloc((size_t)(len ? len : 1) * 2);
    for (uint64_t i = 0; i < n; i++) D[i] = sym[i];
  } else {
    uint64_t nnz = 0;
    uint16_t *v = (uint16_t *)malloc((size_t)(n ? n : 1) * 2);
    uint16_t *c = (uint16_t *)malloc((size_t)(n ? n : 1) * 2);
    uint16_t *r = (uint16_t *)malloc((size_t)(p->rows ? p->rows : 1) * 2);
    rc = orc_csr(sym, p->rows, p->cols, v, c, r, &nnz);
    len = 2 * nnz + p->rows;
    D = (uint16_t *)malloc((size_t)(len ? len : 1) * 2);
    memcpy(D, v, (size_t)nnz * 2);
    memcpy(D + nnz, c, (size_t)nnz * 2);
    memcpy(D + 2 * nnz, r, (size_t)p->rows * 2);
    free(v);
    free(c);
    free(r);
  }
  if (rc == ORC_OK)
    rc = orc_encode_container(D, len, p, n, qi.x_min, qi.x_max, out, out_cap, out_bytes);
  free(D);
  free(sym);
  return rc;
}

int orc_decompress(const uint8_t *buf, size_t bytes, uint8_t *sym, uint64_t sym_cap,
                   orc_qinfo *qi, uint32_t out_dtype, void *x_out) {
  orc_header h;
  int rc = orc_parse_header(buf, bytes, &h);
  if (rc) return rc;
  if (h.n_elems > sym_cap) return ORC_ERR_CAPACITY;
  uint16_t *D = (uint16_t *)malloc((size_t)(h.len_D ? h.len_D : 1) * 2);
  rc = orc_decode_container(buf, bytes, D, h.len_D, &h);
  if (rc == ORC_OK) {
    if (h.p.mode == ORC_MODE_DENSE) {
      for (uint64_t i = 0; i < h.n_elems; i++) sym[i] = (uint8_t)D[i];
    } else {
      uint64_t nnz = (h.len_D - h.p.rows) / 2;
      rc = orc_csr_expand(D, D + nnz, D + 2 * nnz, nnz, h.p.rows, h.p.cols, h.p.q_bits, sym);
    }
  }
  free(D);
  if (rc) return rc;
  orc_qinfo q;
  rc = orc_qinfo_from_minmax(h.x_min, h.x_max, h.p.q_bits, &q);
  if (rc) return ORC_ERR_CORRUPT;
  if (qi) *qi = q;
  if (x_out) rc = orc_dequantize(sym, h.n_elems, &q, out_dtype, x_out);
  return rc;
}
