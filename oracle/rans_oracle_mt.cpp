// rans_oracle_mt.cpp -- all-cores TIMING driver of the CPU oracle (TEST INFRASTRUCTURE ONLY).
//
// The oracle itself (rans_oracle.c) is single-threaded on purpose.  This file adds nothing to what is
// computed: it cuts the same work into independent pieces and hands each piece to the oracle's own routines
// on a std::thread -- slices of the tensor for the extrema, Eq. 6 and the dequantisation, blocks of rows for
// the modified CSR (Sec. 3.1), slices of D for the histogram (partial counts are added), and chunks of D for
// the coder (chunks are independent coders by the container's definition).  The bytes it produces are the
// oracle's bytes (tests/test_oracle_mt.py compares them); the benchmark times it next to the single-thread
// oracle as the "all host cores" figure.  Only tests and bench.py's cpu_baseline leg may load it.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "rans_oracle.h"

namespace {

// fn(lo, hi, t) over [0, n) cut into n_threads contiguous ranges whose bounds are multiples of `grain`
template <class Fn>
void parallel_ranges(uint64_t n, uint64_t grain, unsigned n_threads, Fn fn) {
  if (n_threads < 1) n_threads = 1;
  const uint64_t units = (n + grain - 1) / grain;
  const uint64_t per = (units + n_threads - 1) / n_threads;
  std::vector<std::thread> th;
  for (unsigned t = 0; t < n_threads; t++) {
    const uint64_t lo = std::min<uint64_t>(n, (uint64_t)t * per * grain), hi = std::min<uint64_t>(n, (uint64_t)(t + 1) * per * grain);
    th.emplace_back([=] { fn(lo, hi, t); });
  }
  for (auto &x : th) x.join();
}

// items 0..n-1 handed out one at a time (chunks differ in cost)
template <class Fn>
void parallel_items(uint32_t n, unsigned n_threads, Fn fn) {
  if (n_threads < 1) n_threads = 1;
  std::vector<std::thread> th;
  for (unsigned t = 0; t < n_threads; t++)
    th.emplace_back([=] {
      for (uint32_t i = t; i < n; i += n_threads) fn(i);
    });
  for (auto &x : th) x.join();
}

const void *elem_ptr(const void *x, uint64_t i, uint32_t dtype) {
  return (const uint8_t *)x + i * (dtype == ORC_F16 ? 2 : 4);
}

}  // namespace

extern "C" {

// Same container as orc_compress (rans_oracle.c), computed by n_threads threads.
int orc_mt_compress(const void *x, uint64_t n, const orc_params *p, uint8_t *out, size_t out_cap, size_t *out_bytes,
                    unsigned n_threads) {
  if (!p || !out || !out_bytes || (n && !x)) return ORC_ERR_ARG;
  if (p->cols < 1 || p->rows * p->cols != n || p->n_streams < 1 || p->chunk_syms % p->n_streams != 0) return ORC_ERR_SHAPE;
  const unsigned nt = n_threads ? n_threads : 1;
  // extrema (Eq. 6): per slice, then folded; the first slice's values start the fold as in orc_minmax
  std::vector<float> mn(nt, 0.0f), mx(nt, 0.0f);
  std::vector<int> rcs(nt, ORC_OK), used(nt, 0);
  parallel_ranges(n, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned t) {
    if (lo < hi) {
      used[t] = 1;
      rcs[t] = orc_minmax(elem_ptr(x, lo, p->in_dtype), hi - lo, p->in_dtype, &mn[t], &mx[t]);
    }
  });
  float x_min = 0.0f, x_max = 0.0f;
  bool first = true;
  for (unsigned t = 0; t < nt; t++) {
    if (rcs[t]) return rcs[t];
    if (!used[t]) continue;
    if (first || mn[t] < x_min) x_min = mn[t];
    if (first || mx[t] > x_max) x_max = mx[t];
    first = false;
  }
  orc_qinfo qi;
  int rc = orc_qinfo_from_minmax(x_min, x_max, p->q_bits, &qi);
  if (rc) return rc;
  // symbols (Eq. 6), element by element
  std::vector<uint8_t> sym(n ? n : 1);
  parallel_ranges(n, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned) {
    for (uint64_t i = lo; i < hi; i++) {
      float v = p->in_dtype == ORC_F16 ? orc_half_to_float(((const uint16_t *)x)[i]) : ((const float *)x)[i];
      sym[i] = orc_quantize_one(v, &qi, p->q_bits);
    }
  });
  // D (Eq. 7)
  std::vector<uint16_t> D;
  uint64_t len = 0;
  if (p->mode == ORC_MODE_DENSE) {
    len = n;
    D.resize(len ? len : 1);
    parallel_ranges(n, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned) {
      for (uint64_t i = lo; i < hi; i++) D[i] = sym[i];
    });
  } else {
    // blocks of rows through orc_csr, their v and c parts concatenated in row order
    std::vector<std::vector<uint16_t>> vs(nt), cs(nt);
    std::vector<uint16_t> r(p->rows ? p->rows : 1);
    std::vector<uint64_t> nz(nt, 0);
    parallel_ranges(p->rows, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned t) {
      const uint64_t cells = (hi - lo) * p->cols;
      vs[t].resize(cells ? cells : 1);
      cs[t].resize(cells ? cells : 1);
      if (lo < hi) rcs[t] = orc_csr(sym.data() + lo * p->cols, hi - lo, p->cols, vs[t].data(), cs[t].data(), r.data() + lo, &nz[t]);
    });
    uint64_t nnz = 0;
    for (unsigned t = 0; t < nt; t++) {
      if (rcs[t]) return rcs[t];
      nnz += nz[t];
    }
    len = 2 * nnz + p->rows;
    D.resize(len ? len : 1);
    uint64_t at = 0;
    for (unsigned t = 0; t < nt; t++) {
      std::memcpy(D.data() + at, vs[t].data(), nz[t] * 2);
      std::memcpy(D.data() + nnz + at, cs[t].data(), nz[t] * 2);
      at += nz[t];
    }
    std::memcpy(D.data() + 2 * nnz, r.data(), p->rows * 2);
  }
  // one frequency vector over D: partial histograms of slices, added
  const uint32_t A = orc_alphabet(p->mode, p->q_bits, p->cols), M = p->freq_bits, S = p->n_streams;
  std::vector<std::vector<uint64_t>> parts(nt, std::vector<uint64_t>(A, 0));
  parallel_ranges(len, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned t) { orc_histogram(D.data() + lo, hi - lo, A, parts[t].data()); });
  std::vector<uint64_t> cnt(A, 0);
  for (unsigned t = 0; t < nt; t++)
    for (uint32_t a = 0; a < A; a++) cnt[a] += parts[t][a];
  std::vector<uint16_t> f(A);
  std::vector<uint32_t> F((size_t)A + 1);
  rc = orc_normalize(cnt.data(), A, M, f.data(), F.data());
  if (rc) return rc;
  size_t dir_off = 0, payload_off = 0;
  rc = orc_write_header_and_table(p, n, len, qi.x_min, qi.x_max, f.data(), out, out_cap, &dir_off, &payload_off);
  if (rc) return rc;
  // chunks: each coded into a buffer of its own, then laid out one after the other
  const uint64_t chunk_len = p->chunk_syms ? p->chunk_syms : len;
  const uint32_t nc = len == 0 ? 0 : (uint32_t)((len + chunk_len - 1) / chunk_len);
  std::vector<std::vector<uint8_t>> bufs(nc);
  std::vector<size_t> sizes(nc, 0);
  std::vector<int> crc(nc, ORC_OK);
  parallel_items(nc, nt, [&](uint32_t k) {
    const uint64_t base = (uint64_t)k * chunk_len;
    const uint64_t n_here = len - base < chunk_len ? len - base : chunk_len;
    bufs[k].resize(8 * (size_t)S + 2 * n_here + 4);
    crc[k] = orc_encode_chunk(D.data(), base, n_here, S, f.data(), F.data(), M, bufs[k].data(), bufs[k].size(), &sizes[k]);
  });
  auto put64 = [&](size_t o, uint64_t v) {
    for (int b = 0; b < 8; b++) out[o + b] = (uint8_t)(v >> (8 * b));
  };
  size_t pos = payload_off;
  for (uint32_t k = 0; k < nc; k++) {
    if (crc[k]) return crc[k];
    if (pos + sizes[k] > out_cap) return ORC_ERR_CAPACITY;
    put64(dir_off + 8 * (size_t)k, pos - payload_off);
    pos += sizes[k];
  }
  put64(dir_off + 8 * (size_t)nc, pos - payload_off);
  std::vector<size_t> starts(nc);
  {
    size_t q = payload_off;
    for (uint32_t k = 0; k < nc; k++) {
      starts[k] = q;
      q += sizes[k];
    }
  }
  parallel_items(nc, nt, [&](uint32_t k) { std::memcpy(out + starts[k], bufs[k].data(), sizes[k]); });
  *out_bytes = pos;
  return ORC_OK;
}

// Same outputs as orc_decompress, computed by n_threads threads.
int orc_mt_decompress(const uint8_t *buf, size_t bytes, uint8_t *sym, uint64_t sym_cap, uint32_t out_dtype, void *x_out,
                      unsigned n_threads) {
  const unsigned nt = n_threads ? n_threads : 1;
  orc_header h;
  int rc = orc_parse_header(buf, bytes, &h);
  if (rc) return rc;
  if (h.n_elems > sym_cap) return ORC_ERR_CAPACITY;
  std::vector<uint16_t> f(h.A);
  std::vector<uint32_t> F((size_t)h.A + 1);
  rc = orc_read_table(buf, bytes, &h, f.data(), F.data());
  if (rc) return rc;
  std::vector<uint16_t> D(h.len_D ? h.len_D : 1);
  std::vector<int> crc(h.n_chunks ? h.n_chunks : 1, ORC_OK);
  parallel_items(h.n_chunks, nt, [&](uint32_t k) { crc[k] = orc_decode_chunk(buf, bytes, &h, k, f.data(), F.data(), D.data()); });
  for (uint32_t k = 0; k < h.n_chunks; k++)
    if (crc[k]) return crc[k];
  if (h.p.mode == ORC_MODE_DENSE) {
    parallel_ranges(h.n_elems, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned) {
      for (uint64_t i = lo; i < hi; i++) sym[i] = (uint8_t)D[i];
    });
  } else {
    // blocks of rows: a block's first nonzero is the sum of the row counts before it (the cumulative sum of r
    // is taken here, on the decoding side); orc_csr_expand checks each block's own total
    const uint64_t nnz = (h.len_D - h.p.rows) / 2, N = h.p.rows, K = h.p.cols;
    const uint16_t *r = D.data() + 2 * nnz;
    for (uint64_t i = 0; i < N; i++)
      if (r[i] > K) return ORC_ERR_CORRUPT;
    std::vector<uint64_t> lo_of(nt + 1, 0), first(nt + 1, 0);
    const uint64_t per = (N + nt - 1) / nt;
    for (unsigned t = 0; t <= nt; t++) lo_of[t] = std::min<uint64_t>(N, (uint64_t)t * per);
    for (unsigned t = 0; t < nt; t++) {
      uint64_t s = 0;
      for (uint64_t i = lo_of[t]; i < lo_of[t + 1]; i++) s += r[i];
      first[t + 1] = first[t] + s;
    }
    if (first[nt] != nnz) return ORC_ERR_CORRUPT;
    std::vector<int> erc(nt, ORC_OK);
    std::vector<std::thread> th;
    for (unsigned t = 0; t < nt; t++)
      th.emplace_back([&, t] {
        const uint64_t lo = lo_of[t], hi = lo_of[t + 1];
        if (lo < hi)
          erc[t] = orc_csr_expand(D.data() + first[t], D.data() + nnz + first[t], r + lo, first[t + 1] - first[t], hi - lo, K,
                                  h.p.q_bits, sym + lo * K);
      });
    for (auto &x : th) x.join();
    for (unsigned t = 0; t < nt; t++)
      if (erc[t]) return erc[t];
  }
  orc_qinfo q;
  rc = orc_qinfo_from_minmax(h.x_min, h.x_max, h.p.q_bits, &q);
  if (rc) return ORC_ERR_CORRUPT;
  if (x_out) {
    const size_t eb = out_dtype == ORC_F16 ? 2 : 4;
    std::vector<int> drc(nt, ORC_OK);
    parallel_ranges(h.n_elems, 1, nt, [&](uint64_t lo, uint64_t hi, unsigned t) {
      if (lo < hi) drc[t] = orc_dequantize(sym + lo, hi - lo, &q, out_dtype, (uint8_t *)x_out + lo * eb);
    });
    for (unsigned t = 0; t < nt; t++)
      if (drc[t]) return drc[t];
  }
  return ORC_OK;
}

}  // extern "C"
