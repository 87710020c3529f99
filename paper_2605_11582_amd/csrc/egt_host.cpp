// Host side of the SparseGemv library: shape rules, N:4 magnitude pruning, the
// group-wise INT4 quantiser and the 2bit-CSR encoder / decoder (Sec. 3.2 and
// Sec. 3.3 "Sparse Index Structure" of the paper).  Plain C++, no GPU calls.
#include "egt.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>

namespace {

// ---------------------------------------------------------------- binary16
inline double half_to_double(uint16_t h) {
  const int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0) v = std::ldexp((double)m, -24);
  else if (e == 31) v = m ? NAN : INFINITY;
  else v = std::ldexp((double)(m + 1024), e - 25);
  return sign ? -v : v;
}

// One rounding, nearest-even, straight from binary64 (never through binary32).
inline uint16_t double_to_half(double v) {
  const uint16_t sign = std::signbit(v) ? 0x8000u : 0u;
  if (std::isnan(v)) return sign | 0x7E00u;
  double a = std::fabs(v);
  if (a >= 65520.0) return sign | 0x7C00u;          // rounds to infinity
  if (a < std::ldexp(1.0, -14)) {                    // subnormal range: units of 2^-24
    const double q = std::nearbyint(std::ldexp(a, 24));
    return sign | (uint16_t)q;                       // q == 1024 is the smallest normal
  }
  int e;
  std::frexp(a, &e);                                 // a = f * 2^e, f in [0.5, 1)
  e -= 1;                                            // a in [2^e, 2^(e+1))
  double q = std::nearbyint(std::ldexp(a, 10 - e));  // in [1024, 2048]
  if (q >= 2048.0) { q = 1024.0; e += 1; }
  return sign | (uint16_t)(((e + 15) << 10) + ((int)q - 1024));
}

inline bool half_is_finite(uint16_t h) { return ((h >> 10) & 31) != 31; }

// ---------------------------------------------------------------- threading
template <class F>
void parallel_rows(int rows, F &&body) {
  unsigned hw = std::thread::hardware_concurrency();
  int nt = (int)std::min<unsigned>(hw ? hw : 1u, 16u);
  nt = std::max(1, std::min(nt, rows / 64));
  if (nt <= 1) { body(0, rows); return; }
  std::vector<std::thread> th;
  const int chunk = (rows + nt - 1) / nt;
  for (int t = 0; t < nt; ++t) {
    const int r0 = t * chunk, r1 = std::min(rows, r0 + chunk);
    if (r0 >= r1) break;
    th.emplace_back([&body, r0, r1] { body(r0, r1); });
  }
  for (auto &x : th) x.join();
}

// INT4 values in either nibble order
inline bool is_int4(int val_kind) { return val_kind == EGT_VAL_INT4 || val_kind == EGT_VAL_INT4_PAIRED; }
// Where the code of global slot t lives: byte and shift.  Canonical order: slot j of a word
// of eight slots in nibble j.  Paired order: in nibble (j >> 1) + 4 (j & 1), i.e. the
// nibbles of a word hold the slots 0, 2, 4, 6, 1, 3, 5, 7.
inline int64_t nibble_byte(int64_t t, int val_kind, int &shift) {
  const int j = (int)(t & 7);
  const int pos = val_kind == EGT_VAL_INT4_PAIRED ? (j >> 1) + 4 * (j & 1) : j;
  shift = 4 * (pos & 1);
  return (t >> 3) * 4 + (pos >> 1);
}

// ---------------------------------------------------------------- shape rules
egt_status check_shape(int rows, int cols, int n_keep, int group, int val_kind) {
  if (rows < 0 || cols < 0) return EGT_ERR_SHAPE;
  if (cols % 32 != 0) return EGT_ERR_SHAPE;
  if (n_keep < 1 || n_keep > 4) return EGT_ERR_SHAPE;
  if (is_int4(val_kind)) {
    if (group <= 0 || group % 4 != 0 || cols % group != 0) return EGT_ERR_SHAPE;
  } else if (val_kind == EGT_VAL_FP16) {
    if (group != 0) return EGT_ERR_SHAPE;
  } else {
    return EGT_ERR_SHAPE;
  }
  const uint64_t slots = (uint64_t)rows * (uint64_t)n_keep * (uint64_t)(cols / 4);
  if (slots >= (1ull << 32)) return EGT_ERR_SHAPE;   // row_ptr is uint32
  return EGT_OK;
}

// Shape rules of a matrix whose rows keep row_n_keep[r] (1..4) entries per 4-group each;
// `slots`: the total number of slots.
egt_status check_rows(int rows, int cols, const int32_t *row_n_keep, int group, int val_kind, uint64_t &slots) {
  const egt_status st = check_shape(rows, cols, 1, group, val_kind);
  if (st != EGT_OK) return st;
  slots = 0;
  for (int r = 0; r < rows; ++r) {
    if (row_n_keep[r] < 1 || row_n_keep[r] > 4) return EGT_ERR_SHAPE;
    slots += (uint64_t)row_n_keep[r] * (uint64_t)(cols / 4);
  }
  if (slots >= (1ull << 32)) return EGT_ERR_SHAPE;
  return EGT_OK;
}

void fill_sizes(int rows, int cols, uint64_t slots, int group, int val_kind, size_t bytes[4]) {
  bytes[0] = sizeof(uint32_t) * ((size_t)rows + 1);
  bytes[1] = is_int4(val_kind) ? (size_t)(slots / 2) : (size_t)(slots * 2);
  bytes[2] = (size_t)(slots / 8) * sizeof(uint16_t);
  bytes[3] = is_int4(val_kind) ? sizeof(uint16_t) * 2 * (size_t)rows * (size_t)(cols / group) : 0;
}

egt_status pack_rows(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm, int rows, int cols,
                     int n_keep, const int32_t *row_n_keep, int group, int val_kind, const int32_t *row_group,
                     egt_2bitcsr *out);

// Scale and zero point of one group from the extrema of its kept values.
struct QParam { uint16_t s_bits; double s; int z; };
inline QParam make_qparam(double vmin, double vmax) {
  const double xmin = std::min(0.0, vmin), xmax = std::max(0.0, vmax);
  uint16_t sb = double_to_half((xmax - xmin) / 15.0);
  if ((sb & 0x7FFF) == 0) sb = 0x3C00;               // s == 0 -> 1.0
  const double s = half_to_double(sb);
  double z = std::nearbyint(-xmin / s);
  z = std::min(15.0, std::max(0.0, z));
  return {sb, s, (int)z};
}
inline int make_code(double v, const QParam &p) {
  double q = std::nearbyint(v / p.s) + (double)p.z;
  q = std::min(15.0, std::max(0.0, q));
  return (int)q;
}

// Chosen in-group offsets of one 4-group: the kept ones plus, if fewer than n,
// the smallest unused offsets.  Returns a 4-bit set, or -1 when over-full.
inline int choose4(const uint8_t *m, int n) {
  int set = 0, cnt = 0;
  for (int j = 0; j < 4; ++j) if (m[j]) { set |= 1 << j; ++cnt; }
  if (cnt > n) return -1;
  for (int j = 0; j < 4 && cnt < n; ++j) if (!(set >> j & 1)) { set |= 1 << j; ++cnt; }
  return set;
}

}  // namespace

extern "C" {

const char *egt_status_str(egt_status status) {
  switch (status) {
    case EGT_OK: return "ok";
    case EGT_ERR_NULL: return "null pointer";
    case EGT_ERR_SHAPE: return "bad shape";
    case EGT_ERR_MASK: return "mask keeps more than n_keep entries in a 4-group";
    case EGT_ERR_NONFINITE: return "non-finite kept weight";
    case EGT_ERR_BUFFER: return "inconsistent buffer contents";
    case EGT_ERR_UNSUPPORTED: return "unsupported configuration";
    case EGT_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

egt_status egt_2bitcsr_sizes(int rows, int cols, int n_keep, int group, int val_kind,
                             size_t bytes[4]) {
  if (!bytes) return EGT_ERR_NULL;
  const egt_status st = check_shape(rows, cols, n_keep, group, val_kind);
  if (st != EGT_OK) return st;
  const size_t slots = (size_t)rows * (size_t)n_keep * (size_t)(cols / 4);
  bytes[0] = 4 * ((size_t)rows + 1);
  bytes[1] = is_int4(val_kind) ? slots / 2 : slots * 2;
  bytes[2] = 2 * (slots / 8);
  bytes[3] = is_int4(val_kind) ? 4 * (size_t)rows * (size_t)(cols / group) : 0;
  return EGT_OK;
}

egt_status egt_prune_n4(const uint16_t *w, int64_t ldw, int rows, int cols, int n_keep,
                        uint8_t *mask, int64_t ldm) {
  if (!w || !mask) return EGT_ERR_NULL;
  if (rows < 0 || cols < 0 || cols % 4 != 0 || n_keep < 1 || n_keep > 4 || ldw < cols || ldm < cols)
    return EGT_ERR_SHAPE;
  parallel_rows(rows, [=](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      const uint16_t *wr = w + (int64_t)r * ldw;
      uint8_t *mr = mask + (int64_t)r * ldm;
      for (int c = 0; c < cols; c += 4) {
        // |w| ordering of finite binary16 numbers = ordering of the low 15 bits
        int mag[4];
        for (int j = 0; j < 4; ++j) mag[j] = wr[c + j] & 0x7FFF;
        for (int j = 0; j < 4; ++j) {
          int beats = 0;
          for (int i = 0; i < 4; ++i) {
            if (i == j) continue;
            beats += i < j ? (mag[i] >= mag[j]) : (mag[i] > mag[j]);
          }
          mr[c + j] = beats < n_keep ? 1 : 0;
        }
      }
    }
  });
  return EGT_OK;
}

egt_status egt_prune_n4_importance(const uint16_t *w, int64_t ldw, const float *act_norm,
                                   const float *grad_abs, int64_t ldg, int rows, int cols,
                                   int n_keep, uint8_t *mask, int64_t ldm) {
  if (!w || !act_norm || !mask) return EGT_ERR_NULL;
  if (rows < 0 || cols < 0 || cols % 4 != 0 || n_keep < 1 || n_keep > 4 || ldw < cols || ldm < cols ||
      (grad_abs && ldg < cols))
    return EGT_ERR_SHAPE;
  for (int c = 0; c < cols; ++c)
    if (!(act_norm[c] >= 0.0f) || std::isinf(act_norm[c])) return EGT_ERR_NONFINITE;
  std::atomic<int> err(EGT_OK);
  parallel_rows(rows, [&](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      for (int c = 0; c < cols; ++c) {
        if ((w[(int64_t)r * ldw + c] & 0x7C00) == 0x7C00) err.store(EGT_ERR_NONFINITE);
        if (grad_abs) {
          const float gv = grad_abs[(int64_t)r * ldg + c];
          if (!(gv >= 0.0f) || std::isinf(gv)) err.store(EGT_ERR_NONFINITE);
        }
      }
    }
  });
  if (err.load() != EGT_OK) return (egt_status)err.load();
  parallel_rows(rows, [=](int r0, int r1) {
#pragma clang fp contract(off)
    for (int r = r0; r < r1; ++r) {
      const uint16_t *wr = w + (int64_t)r * ldw;
      uint8_t *mr = mask + (int64_t)r * ldm;
      for (int c = 0; c < cols; c += 4) {
        double score[4];
        for (int j = 0; j < 4; ++j) {
          const double a = std::fabs(half_to_double(wr[c + j]));
          const double p1 = a * (double)act_norm[c + j];
          const double p2 = grad_abs ? a * (double)grad_abs[(int64_t)r * ldg + c + j] : 0.0;
          score[j] = p1 + p2;
        }
        for (int j = 0; j < 4; ++j) {
          int beats = 0;
          for (int i = 0; i < 4; ++i) {
            if (i == j) continue;
            beats += i < j ? (score[i] >= score[j]) : (score[i] > score[j]);
          }
          mr[c + j] = beats < n_keep ? 1 : 0;
        }
      }
    }
  });
  return EGT_OK;
}

egt_status egt_pack_2bitcsr(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                            int rows, int cols, int n_keep, int group, int val_kind,
                            egt_2bitcsr *out) {
  return pack_rows(w, ldw, mask, ldm, rows, cols, n_keep, nullptr, group, val_kind, nullptr, out);
}

egt_status egt_pack_2bitcsr_rowgroups(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                                      int rows, int cols, int n_keep, int group, int val_kind,
                                      const int32_t *row_group, egt_2bitcsr *out) {
  return pack_rows(w, ldw, mask, ldm, rows, cols, n_keep, nullptr, group, val_kind, row_group, out);
}

egt_status egt_pack_2bitcsr_rows(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                                 int rows, int cols, const int32_t *row_n_keep, int group, int val_kind,
                                 egt_2bitcsr *out) {
  if (!row_n_keep) return EGT_ERR_NULL;
  return pack_rows(w, ldw, mask, ldm, rows, cols, 0, row_n_keep, group, val_kind, nullptr, out);
}

egt_status egt_2bitcsr_sizes_rows(int rows, int cols, const int32_t *row_n_keep, int group, int val_kind,
                                  size_t bytes[4]) {
  if (!bytes || !row_n_keep) return EGT_ERR_NULL;
  uint64_t slots = 0;
  const egt_status st = check_rows(rows, cols, row_n_keep, group, val_kind, slots);
  if (st != EGT_OK) return st;
  fill_sizes(rows, cols, slots, group, val_kind, bytes);
  return EGT_OK;
}

}  // extern "C"

namespace {

// The encoder.  row_n_keep == nullptr: n_keep entries per 4-group in every row; else row r
// keeps row_n_keep[r] (rows of different lengths, row_ptr a true prefix sum, n_keep = 0
// in the view).
egt_status pack_rows(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm, int rows, int cols,
                     int n_keep, const int32_t *row_n_keep, int group, int val_kind, const int32_t *row_group,
                     egt_2bitcsr *out) {
  if (!w || !mask || !out) return EGT_ERR_NULL;
  uint64_t total_slots = 0;
  egt_status st = row_n_keep ? check_rows(rows, cols, row_n_keep, group, val_kind, total_slots)
                             : check_shape(rows, cols, n_keep, group, val_kind);
  if (st != EGT_OK) return st;
  auto n_of = [=](int r) { return row_n_keep ? (int)row_n_keep[r] : n_keep; };
  if (ldw < cols || ldm < cols) return EGT_ERR_SHAPE;
  if (!out->row_ptr || !out->values || !out->idx) return EGT_ERR_NULL;
  if (is_int4(val_kind) && !out->qparams) return EGT_ERR_NULL;
  if (row_group) {
    if (!is_int4(val_kind)) return EGT_ERR_SHAPE;
    for (int r = 0; r < rows; ++r)
      if (row_group[r] <= 0 || row_group[r] % group != 0 || cols % row_group[r] != 0) return EGT_ERR_SHAPE;
  }

  // pass 1: validate everything before a single output byte is written.  The error reported
  // is that of the first offending 4-group in row-major order, whatever the thread timing; a
  // group that is both over-full and holds a non-finite kept weight reports the mask.
  std::atomic<int64_t> first(INT64_MAX);             // (index of the 4-group in the matrix) * 8 + code
  const int64_t gpr = cols / 4;
  parallel_rows(rows, [&](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      if ((int64_t)r * gpr * 8 > first.load(std::memory_order_relaxed)) break;
      const uint16_t *wr = w + (int64_t)r * ldw;
      const uint8_t *mr = mask + (int64_t)r * ldm;
      const int n_row = n_of(r);
      for (int c = 0; c < cols; c += 4) {
        int cnt = 0;
        bool nonfinite = false;
        for (int j = 0; j < 4; ++j) {
          if (!mr[c + j]) continue;
          ++cnt;
          nonfinite |= !half_is_finite(wr[c + j]);
        }
        if (cnt <= n_row && !nonfinite) continue;
        const int64_t key = ((int64_t)r * gpr + (c >> 2)) * 8 + (cnt > n_row ? EGT_ERR_MASK : EGT_ERR_NONFINITE);
        int64_t seen = first.load();
        while (key < seen && !first.compare_exchange_weak(seen, key)) {}
        r = r1;                                         // later rows of this range cannot come first
        break;
      }
    }
  });
  if (first.load() != INT64_MAX) return (egt_status)(first.load() & 7);

  const int G = is_int4(val_kind) ? cols / group : 0;
  // first slot of every row (uniform rows: r * S)
  for (int64_t r = 0, t = 0; r <= rows; ++r) {
    out->row_ptr[r] = (uint32_t)t;
    if (r < rows) t += (int64_t)n_of((int)r) * (cols / 4);
  }
  uint8_t *vals8 = (uint8_t *)out->values;
  uint16_t *vals16 = (uint16_t *)out->values;
  uint32_t *row_ptr = out->row_ptr;
  uint16_t *idx = out->idx, *qparams = out->qparams;

  parallel_rows(rows, [=](int r0, int r1) {
    std::vector<QParam> qp((size_t)std::max(G, 1));
    for (int r = r0; r < r1; ++r) {
      const uint16_t *wr = w + (int64_t)r * ldw;
      const uint8_t *mr = mask + (int64_t)r * ldm;
      const int n_row = n_of(r);
      if (is_int4(val_kind)) {
        // the row's own group size; its parameters are stored once per `group` columns
        const int gr = row_group ? row_group[r] : group, rep = gr / group;
        for (int g0 = 0; g0 < G; g0 += rep) {
          double vmin = INFINITY, vmax = -INFINITY;
          for (int c = g0 * group; c < g0 * group + gr; ++c) {
            if (!mr[c]) continue;
            const double v = half_to_double(wr[c]);
            vmin = std::min(vmin, v);
            vmax = std::max(vmax, v);
          }
          if (vmin > vmax) { vmin = 0.0; vmax = 0.0; }          // nothing kept
          const QParam p = make_qparam(vmin, vmax);
          for (int g = g0; g < g0 + rep; ++g) {
            qp[g] = p;
            uint16_t *o = qparams + ((int64_t)r * G + g) * 2;
            o[0] = p.s_bits;
            o[1] = double_to_half((double)p.z);
          }
        }
      }
      int64_t t = (int64_t)row_ptr[r];                            // global slot id
      uint32_t word = 0;
      for (int c = 0; c < cols; c += 4) {
        const int set = choose4(mr + c, n_row);
        for (int j = 0; j < 4; ++j) {
          if (!(set >> j & 1)) continue;
          word |= (uint32_t)j << (2 * (t & 7));
          const bool kept = mr[c + j] != 0;
          if (val_kind == EGT_VAL_FP16) {
            vals16[t] = kept ? wr[c + j] : (uint16_t)0;
          } else {
            const QParam &p = qp[(c + j) / group];
            const int q = kept ? make_code(half_to_double(wr[c + j]), p) : p.z;
            // (a row is a whole number of 4-byte words and no other row shares them: the
            //  first nibble of a byte sets it, the second is or-ed in)
            int shift;
            const int64_t b = nibble_byte(t, val_kind, shift);
            vals8[b] = shift ? (uint8_t)(vals8[b] | (q << 4)) : (uint8_t)q;
          }
          if ((t & 7) == 7) { idx[t >> 3] = (uint16_t)word; word = 0; }
          ++t;
        }
      }
    }
  });
  out->rows = rows; out->cols = cols; out->n_keep = row_n_keep ? 0 : n_keep;
  out->group_size = group; out->val_kind = val_kind;
  out->total_slots = row_ptr[rows];
  return EGT_OK;
}

}  // namespace

extern "C" {

egt_status egt_unpack_2bitcsr(const egt_2bitcsr *in, uint16_t *w_dense, int64_t ldw,
                              uint8_t *mask, int64_t ldm) {
  if (!in) return EGT_ERR_NULL;
  const int rows = in->rows, cols = in->cols, group = in->group_size;
  const bool mixed = in->n_keep == 0;                  // rows of different lengths
  egt_status st = check_shape(rows, cols, mixed ? 1 : in->n_keep, group, in->val_kind);
  if (st != EGT_OK) return st;
  if (!in->row_ptr || !in->values || !in->idx) return EGT_ERR_NULL;
  if (is_int4(in->val_kind) && !in->qparams) return EGT_ERR_NULL;
  if ((w_dense && ldw < cols) || (mask && ldm < cols)) return EGT_ERR_SHAPE;
  // row_ptr: the uniform progression, or a running sum of whole rows that ends at total_slots
  const int64_t quarter = cols / 4;
  std::vector<int> n_row((size_t)rows);
  for (int r = 0; r < rows; ++r) {
    const int64_t len = (int64_t)in->row_ptr[r + 1] - (int64_t)in->row_ptr[r];
    if (mixed) {
      if (quarter == 0 || len % quarter != 0 || len / quarter < 1 || len / quarter > 4) return EGT_ERR_BUFFER;
      n_row[r] = (int)(len / quarter);
    } else {
      if (in->row_ptr[r] != (uint32_t)((int64_t)r * in->n_keep * quarter) || len != in->n_keep * quarter) return EGT_ERR_BUFFER;
      n_row[r] = in->n_keep;
    }
  }
  if (rows > 0 && in->row_ptr[0] != 0) return EGT_ERR_BUFFER;
  if (mixed && in->row_ptr[rows] != in->total_slots) return EGT_ERR_BUFFER;
  // offsets of a 4-group must ascend strictly
  std::atomic<int> err(EGT_OK);
  const uint16_t *idx = in->idx;
  const uint32_t *row_ptr = in->row_ptr;
  parallel_rows(rows, [&](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      int64_t t = (int64_t)row_ptr[r];
      for (int c = 0; c < cols; c += 4) {
        int prev = -1;
        for (int k = 0; k < n_row[r]; ++k, ++t) {
          const int off = (idx[t >> 3] >> (2 * (t & 7))) & 3;
          if (off <= prev) err.store(EGT_ERR_BUFFER);
          prev = off;
        }
      }
    }
  });
  if (err.load() != EGT_OK) return (egt_status)err.load();

  const uint8_t *vals8 = (const uint8_t *)in->values;
  const uint16_t *vals16 = (const uint16_t *)in->values;
  const uint16_t *qparams = in->qparams;
  const int val_kind = in->val_kind;
  const int G = is_int4(val_kind) ? cols / group : 0;
  const int *nr = n_row.data();
  parallel_rows(rows, [=](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      if (w_dense) std::memset(w_dense + (int64_t)r * ldw, 0, sizeof(uint16_t) * (size_t)cols);
      if (mask) std::memset(mask + (int64_t)r * ldm, 0, (size_t)cols);
      int64_t t = (int64_t)row_ptr[r];
      for (int c = 0; c < cols; c += 4) {
        for (int k = 0; k < nr[r]; ++k, ++t) {
          const int col = c + ((idx[t >> 3] >> (2 * (t & 7))) & 3);
          if (mask) mask[(int64_t)r * ldm + col] = 1;
          if (!w_dense) continue;
          uint16_t bits;
          if (val_kind == EGT_VAL_FP16) {
            bits = vals16[t];
          } else {
            int shift;
            const int64_t b = nibble_byte(t, val_kind, shift);
            const int q = (vals8[b] >> shift) & 15;
            const uint16_t *p = qparams + ((int64_t)r * G + col / group) * 2;
            bits = double_to_half(half_to_double(p[0]) * ((double)q - half_to_double(p[1])));
          }
          w_dense[(int64_t)r * ldw + col] = bits;
        }
      }
    }
  });
  return EGT_OK;
}

egt_status egt_quant_int4(const uint16_t *w, int64_t ldw, int rows, int cols, int group,
                          uint8_t *q, uint16_t *qparams) {
  if (!w || !q || !qparams) return EGT_ERR_NULL;
  if (rows < 0 || cols < 0 || group <= 0 || group % 4 != 0 || cols % group != 0 || ldw < cols)
    return EGT_ERR_SHAPE;
  std::atomic<int> err(EGT_OK);
  parallel_rows(rows, [&](int r0, int r1) {
    for (int r = r0; r < r1; ++r)
      for (int c = 0; c < cols; ++c)
        if (!half_is_finite(w[(int64_t)r * ldw + c])) err.store(EGT_ERR_NONFINITE);
  });
  if (err.load() != EGT_OK) return (egt_status)err.load();
  const int G = cols / group;
  parallel_rows(rows, [=](int r0, int r1) {
    for (int r = r0; r < r1; ++r) {
      const uint16_t *wr = w + (int64_t)r * ldw;
      for (int g = 0; g < G; ++g) {
        double vmin = INFINITY, vmax = -INFINITY;
        for (int c = g * group; c < (g + 1) * group; ++c) {
          const double v = half_to_double(wr[c]);
          vmin = std::min(vmin, v);
          vmax = std::max(vmax, v);
        }
        const QParam p = make_qparam(vmin, vmax);
        uint16_t *o = qparams + ((int64_t)r * G + g) * 2;
        o[0] = p.s_bits;
        o[1] = double_to_half((double)p.z);
        for (int c = g * group; c < (g + 1) * group; c += 2) {
          const int q0 = make_code(half_to_double(wr[c]), p);
          const int q1 = make_code(half_to_double(wr[c + 1]), p);
          q[(int64_t)r * (cols / 2) + c / 2] = (uint8_t)(q0 | (q1 << 4));
        }
      }
    }
  });
  return EGT_OK;
}

egt_status egt_fit_verify_cost(const int *m, const double *t, int n, double *a, double *b) {
  if (!m || !t || !a || !b) return EGT_ERR_NULL;
  if (n < 2) return EGT_ERR_SHAPE;
  double sm = 0, st = 0, smm = 0, smt = 0;
  for (int i = 0; i < n; ++i) {
    if (m[i] < 1 || !std::isfinite(t[i])) return EGT_ERR_SHAPE;
    sm += m[i]; st += t[i]; smm += (double)m[i] * m[i]; smt += (double)m[i] * t[i];
  }
  const double den = n * smm - sm * sm;
  if (den == 0.0) return EGT_ERR_SHAPE;               // all M equal: no slope
  *b = (n * smt - sm * st) / den;
  *a = (st - *b * sm) / n;
  return EGT_OK;
}

egt_status egt_trigger_depth(double t_ar, double a, double b, const int *cand, const int *remaining,
                             int depth, int *best, double *benefit) {
  if (!cand || !remaining || !best || !benefit) return EGT_ERR_NULL;
  if (depth < 1) return EGT_ERR_SHAPE;
  int arg = -1;
  double top = 0.0;
  for (int d = 0; d < depth; ++d) {
    if (cand[d] < 0 || remaining[d] < 0) return EGT_ERR_SHAPE;
    const double gain = remaining[d] * t_ar - (a + b * cand[d]);
    if (gain > top) { top = gain; arg = d; }          // first depth wins among equal gains
  }
  *best = arg;
  *benefit = top;
  return EGT_OK;
}

}  // extern "C"
