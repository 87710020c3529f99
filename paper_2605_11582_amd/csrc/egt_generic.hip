// Generic (any n_keep, any group size, any K % 32 == 0, rows of different lengths) kernels
// of the SparseGemv library.  They follow the format slot by slot with scalar FP32
// arithmetic and serve every shape the tuned kernels do not cover.  One wavefront per matrix
// row; lanes stride over the row's index words.
#include "egt_device.h"

namespace egt {

// One wave per row, MT activation rows per pass (blockIdx.y selects the M-chunk).
// RAGGED: rows of different lengths (n_keep == 0 in the view).  The row's extent comes from
// row_ptr[r] and row_ptr[r + 1]; it is followed only if it is a whole row of 1..4 entries per
// 4-group that starts on an index word and ends inside `total_slots`, the extent of values
// and idx the caller vouches for.  Otherwise the row is never read and reports NaN.
template <int VAL_KIND, int MT, bool RAGGED>
__global__ __launch_bounds__(256) void k_sparse_generic(
    const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
    const uint16_t *__restrict__ idx, const uint16_t *__restrict__ qparams, int rows, int cols,
    int n_keep, uint32_t total_slots, int group, int paired, const __half *__restrict__ X, int64_t ldx,
    __half *__restrict__ Y, int64_t ldy, int M) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int m0 = blockIdx.y * MT;
  const uint32_t quarter = (uint32_t)(cols >> 2);
  uint32_t S = (uint32_t)n_keep * quarter;
  const uint32_t t_row = row_ptr[r];
  bool ok;
  if (RAGGED) {
    const uint32_t t_end = row_ptr[r + 1];
    S = t_end - t_row;
    n_keep = quarter ? (int)(S / quarter) : 1;
    ok = t_end >= t_row && t_end <= total_slots && (t_row & 7u) == 0 && n_keep >= 1 && n_keep <= 4 &&
         (uint32_t)n_keep * quarter == S;
    if (quarter == 0) ok = t_end == t_row;
  } else {
    // uniform rows: anything but the progression r*S is reported as NaN, never followed
    ok = t_row == (uint32_t)r * S;
  }
  float acc[MT];
#pragma unroll
  for (int m = 0; m < MT; ++m) acc[m] = 0.f;
  const int G = VAL_KIND == EGT_VAL_INT4 ? cols / group : 0;
  if (ok) {
    for (uint32_t w = lane; w < (S >> 3); w += 64) {
      const uint32_t t0 = t_row + 8 * w;
      const uint32_t iw = idx[t0 >> 3];
      uint32_t nib = 0;
      uint4 hv = {0, 0, 0, 0};
      if (VAL_KIND == EGT_VAL_INT4) nib = *(const uint32_t *)(values + (t0 >> 1));
      else hv = *(const uint4 *)(values + 2ull * t0);
      const uint32_t hw[4] = {hv.x, hv.y, hv.z, hv.w};
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const uint32_t j = 8 * w + k;                       // slot inside the row
        const int col = 4 * (int)(j / (uint32_t)n_keep) + (int)((iw >> (2 * k)) & 3u);
        float wv;
        if (VAL_KIND == EGT_VAL_INT4) {
          // paired nibble order: slot k of the word sits in nibble (k >> 1) + 4 (k & 1)
          const int q = (nib >> (paired ? 4 * ((k >> 1) + 4 * (k & 1)) : 4 * k)) & 15;
          const uint16_t *p = qparams + ((size_t)r * G + col / group) * 2;
          wv = __half2float(__ushort_as_half(p[0])) * ((float)q - __half2float(__ushort_as_half(p[1])));
        } else {
          wv = __half2float(__ushort_as_half((uint16_t)(hw[k >> 1] >> (16 * (k & 1)))));
        }
#pragma unroll
        for (int m = 0; m < MT; ++m)
          if (m0 + m < M) acc[m] = fmaf(wv, __half2float(X[(int64_t)(m0 + m) * ldx + col]), acc[m]);
      }
    }
  }
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    float v = acc[m];
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    if (lane == 0 && m0 + m < M)
      Y[(int64_t)(m0 + m) * ldy + r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
  }
}

// floor(j / d) for 1 <= d and j * d < 2^32 by a multiplication: inv = ceil(2^32 / d), and
// d = 1 (whose reciprocal does not fit) passes j through.
__device__ __forceinline__ uint32_t div_by(uint32_t j, uint32_t d, uint32_t inv) {
  return d == 1 ? j : __umulhi(j, inv);
}

// Where column c of x sits in LDS, in halves.  A lane reads the columns of eight consecutive slots
// (8, 16 or 32 columns apart from its neighbour's), which unswizzled puts every 4th to 16th lane
// on one bank; folding bits 7..10 of the column into bits 1..4 spreads them over all banks and
// keeps each pair of halves together.
__device__ __forceinline__ uint32_t x_swizzle(uint32_t c) { return c ^ (((c >> 7) & 15u) << 1); }

// What one lane requests for one word of eight slots: the index word, the codes or FP16 values,
// and the {scale, zero} pairs of the quantisation groups of its first and of its last slot.
struct SlotWord {
  uint32_t iw, nib, p_first, p_last;
  uint4 hv;
};

// One lane's share of one row's dot product with x, for the M = 1 kernel below.  N (kept entries
// per 4 columns of this row) is a compile-time constant, so the 4-group of slot k of word w is
// (8 w + k) / N with one division per word at most (N = 3; the others shift), and TWO says
// that no word of eight slots reaches into more than two quantisation groups ((N + 6) / N <=
// group / 4), so that the two {scale, zero} pairs requested with the index and value words
// cover every slot; ONE that every word lies inside one group (8 / N divides group / 4), where
// the pair is applied once per word: s (sum q x - z sum x).  With neither, each slot requests
// its own pair.  A lane requests U words (64 words apart) before it uses the first.
enum { Q_EACH = 0, Q_TWO = 1, Q_ONE = 2 };
template <int VAL_KIND, int N, int QMODE, bool X_IN_LDS, int U = 1>
__device__ __forceinline__ float row_dot(const uint8_t *__restrict__ values, const uint16_t *__restrict__ idx,
                                         const uint32_t *__restrict__ qrow, uint32_t t_row, uint32_t words,
                                         uint32_t g4, uint32_t inv_g4, int lane,
                                         const __half *__restrict__ xv) {
  constexpr bool INT4 = VAL_KIND != EGT_VAL_FP16, paired = VAL_KIND == EGT_VAL_INT4_PAIRED;
  constexpr bool TWO = QMODE == Q_TWO, ONE = QMODE == Q_ONE;
  float acc = 0.f;
  for (uint32_t w0 = lane; w0 < words; w0 += 64 * U) {
    SlotWord in[U];
    uint32_t c4_first[U], rem_first[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t w = w0 + 64 * u;
      in[u] = SlotWord{0, 0, 0, 0, {0, 0, 0, 0}};
      c4_first[u] = N == 3 ? __umulhi(8 * w, 0x55555556u) : 8 * w / N;      // 4-group of the word's first slot
      rem_first[u] = N == 3 ? 8 * w - 3 * c4_first[u] : 0;                  // (8 w is a multiple of 1, 2 and 4)
      if (w < words) {
        const uint32_t t0 = t_row + 8 * w;
        in[u].iw = idx[t0 >> 3];
        if (INT4) {
          in[u].nib = *(const uint32_t *)(values + (t0 >> 1));
          if (ONE) in[u].p_first = qrow[div_by(c4_first[u], g4, inv_g4)];
          if (TWO) {
            // (v * 11) >> 5 = v / 3 for v < 16
            const uint32_t c4_7 = c4_first[u] + (N == 3 ? ((rem_first[u] + 7) * 11u) >> 5 : 7u / N);
            in[u].p_first = qrow[div_by(c4_first[u], g4, inv_g4)];
            in[u].p_last = qrow[div_by(c4_7, g4, inv_g4)];
          }
        } else {
          in[u].hv = *(const uint4 *)(values + 2ull * t0);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (w0 + 64 * u >= words) break;
      const uint32_t c4_0 = c4_first[u], rem = rem_first[u], iw = in[u].iw, nib = in[u].nib;
      // first 4-group past the first slot's quantisation group
      const uint32_t b_first = TWO ? (div_by(c4_0, g4, inv_g4) + 1) * g4 : 0;
      const float s_first = __half2float(__ushort_as_half((uint16_t)(in[u].p_first & 0xFFFFu)));
      const float z_first = __half2float(__ushort_as_half((uint16_t)(in[u].p_first >> 16)));
      const float s_last = __half2float(__ushort_as_half((uint16_t)(in[u].p_last & 0xFFFFu)));
      const float z_last = __half2float(__ushort_as_half((uint16_t)(in[u].p_last >> 16)));
      const uint32_t hw[4] = {in[u].hv.x, in[u].hv.y, in[u].hv.z, in[u].hv.w};
      float sum_qx = 0.f, sum_x = 0.f;
#pragma unroll
      for (int k = 0; k < 8; ++k) {
        const uint32_t c4 = c4_0 + (N == 3 ? ((rem + k) * 11u) >> 5 : (uint32_t)k / N);
        const uint32_t col_plain = 4 * c4 + ((iw >> (2 * k)) & 3u);
        // (for N = 1, 2, 4 a word's columns share bits 7 and up, so one shift serves its eight slots)
        const uint32_t col = !X_IN_LDS ? col_plain : N == 3 ? x_swizzle(col_plain) : col_plain ^ (((c4_0 >> 5) & 15u) << 1);
        float wv;
        if (INT4 && ONE) {
          const int q = (nib >> (paired ? 4 * ((k >> 1) + 4 * (k & 1)) : 4 * k)) & 15;
          const float xk = __half2float(xv[col]);
          sum_qx = fmaf((float)q, xk, sum_qx);
          sum_x += xk;
          continue;
        }
        if (INT4) {
          const int q = (nib >> (paired ? 4 * ((k >> 1) + 4 * (k & 1)) : 4 * k)) & 15;
          float sc, zp;
          if (TWO) {
            sc = c4 < b_first ? s_first : s_last;
            zp = c4 < b_first ? z_first : z_last;
          } else {
            const uint32_t p = qrow[div_by(c4, g4, inv_g4)];
            sc = __half2float(__ushort_as_half((uint16_t)(p & 0xFFFFu)));
            zp = __half2float(__ushort_as_half((uint16_t)(p >> 16)));
          }
          wv = sc * ((float)q - zp);
        } else {
          wv = __half2float(__ushort_as_half((uint16_t)(hw[k >> 1] >> (16 * (k & 1)))));
        }
        acc = fmaf(wv, __half2float(xv[col]), acc);
      }
      if (INT4 && ONE) acc = fmaf(s_first, sum_qx - z_first * sum_x, acc);
    }
  }
  return acc;
}

// M = 1 form of the kernel above: x is staged in LDS once per workgroup (when it fits), so
// that the gather by decoded column is an LDS read instead of a dependent global load, and
// the {scale, zero} pairs - whose addresses depend on the slot's position only, never on its
// index bits - are requested together with the index and value words.  Sixteen waves per
// workgroup each take several rows, so x is staged a few hundred times per launch, not once
// per four rows.
template <int VAL_KIND, bool RAGGED, bool X_IN_LDS>
__global__ __launch_bounds__(1024, 8) void k_sparse_generic_m1(
    const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
    const uint16_t *__restrict__ idx, const uint16_t *__restrict__ qparams, int rows, int cols,
    int n_uniform, uint32_t total_slots, int group, const __half *__restrict__ x,
    __half *__restrict__ y) {
  extern __shared__ __align__(16) uint8_t xs[];
  constexpr bool INT4 = VAL_KIND != EGT_VAL_FP16;
  if (X_IN_LDS) {
    for (int p = threadIdx.x; p < (cols >> 2); p += blockDim.x) {       // cols % 4 == 0
      const uint2 v = ((const uint2 *)x)[p];
      *(uint32_t *)(xs + 2 * x_swizzle(4 * p)) = v.x;
      *(uint32_t *)(xs + 2 * x_swizzle(4 * p + 2)) = v.y;
    }
    __syncthreads();
  }
  const __half *xv = X_IN_LDS ? (const __half *)xs : x;
  const int lane = threadIdx.x & 63, wpb = blockDim.x >> 6;
  const uint32_t quarter = (uint32_t)(cols >> 2);
  const uint32_t g4 = INT4 ? (uint32_t)(group >> 2) : 1u;        // 4-groups per quantisation group
  const uint32_t inv_g4 = (uint32_t)((0x100000000ull + g4 - 1) / g4);
  // rows are dealt to the workgroups in turn (wave v of workgroup b takes rows b + gridDim.x * (v + 16 i)),
  // so that the rows past one per resident wave spread over all compute units
  for (int r = (int)((threadIdx.x >> 6) * gridDim.x + blockIdx.x); r < rows; r += (int)gridDim.x * wpb) {
    int n_keep = n_uniform;
    uint32_t S = (uint32_t)n_keep * quarter;
    const uint32_t t_row = row_ptr[r];
    bool ok;
    if (RAGGED) {
      const uint32_t t_end = row_ptr[r + 1];
      S = t_end - t_row;
      n_keep = quarter ? (int)(S / quarter) : 1;
      ok = t_end >= t_row && t_end <= total_slots && (t_row & 7u) == 0 && n_keep >= 1 && n_keep <= 4 &&
           (uint32_t)n_keep * quarter == S;
      if (quarter == 0) ok = t_end == t_row;
    } else {
      ok = t_row == (uint32_t)r * S;
    }
    const uint32_t *qrow = (const uint32_t *)qparams + (INT4 ? (size_t)r * (size_t)(cols / group) : 0);
    float acc = 0.f;
    if (ok) {
      const uint32_t n = (uint32_t)n_keep;
      const bool one = n != 3 && g4 % (8u / n) == 0, two = (n + 6) / n <= g4;
#define EGT_ROW(N, Q) row_dot<VAL_KIND, N, Q, X_IN_LDS>(values, idx, qrow, t_row, S >> 3, g4, inv_g4, lane, xv)
#define EGT_ROW_N(N) (one ? EGT_ROW(N, Q_ONE) : two ? EGT_ROW(N, Q_TWO) : EGT_ROW(N, Q_EACH))
      switch (n_keep) {                                  // the same for all lanes of the wave
        case 1: acc = EGT_ROW_N(1); break;
        case 2: acc = EGT_ROW_N(2); break;
        case 3: acc = two ? EGT_ROW(3, Q_TWO) : EGT_ROW(3, Q_EACH); break;
        default: acc = EGT_ROW_N(4); break;
      }
#undef EGT_ROW_N
#undef EGT_ROW
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) y[r] = ok ? __float2half(acc) : __ushort_as_half((uint16_t)0x7E00);
  }
}

// Dense group-quantised INT4 GEMV, one wave per row, lanes stride over 8-column words.
__global__ __launch_bounds__(256) void k_int4_generic(const uint8_t *__restrict__ q,
                                                       const uint16_t *__restrict__ qparams,
                                                       int rows, int cols, int group,
                                                       const __half *__restrict__ x,
                                                       __half *__restrict__ y) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int G = cols / group;
  const uint32_t *qr = (const uint32_t *)(q + (size_t)r * (cols >> 1));
  float acc = 0.f;
  for (int w = lane; w < (cols >> 3); w += 64) {
    const uint32_t nib = qr[w];
    const int c0 = 8 * w;                                   // group % 8 == 0: one group per word
    const uint16_t *p = qparams + ((size_t)r * G + c0 / group) * 2;
    const float s = __half2float(__ushort_as_half(p[0])), z = __half2float(__ushort_as_half(p[1]));
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      part = fmaf((float)((nib >> (4 * k)) & 15) - z, __half2float(x[c0 + k]), part);
    acc = fmaf(s, part, acc);
  }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) y[r] = __float2half(acc);
}

// The same product in units of four columns (two bytes of codes): serves groups that are a
// multiple of 4 but not of 8 columns, where an 8-column word would straddle two groups.
__global__ __launch_bounds__(256) void k_int4_generic4(const uint8_t *__restrict__ q,
                                                        const uint16_t *__restrict__ qparams,
                                                        int rows, int cols, int group,
                                                        const __half *__restrict__ x,
                                                        __half *__restrict__ y) {
  const int lane = threadIdx.x & 63;
  const int r = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int G = cols / group;
  const uint16_t *qr = (const uint16_t *)(q + (size_t)r * (cols >> 1));
  float acc = 0.f;
  for (int u = lane; u < (cols >> 2); u += 64) {
    const uint32_t nib = qr[u];
    const int c0 = 4 * u;                                   // group % 4 == 0: one group per unit
    const uint16_t *p = qparams + ((size_t)r * G + c0 / group) * 2;
    const float s = __half2float(__ushort_as_half(p[0])), z = __half2float(__ushort_as_half(p[1]));
    float part = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      part = fmaf((float)((nib >> (4 * k)) & 15) - z, __half2float(x[c0 + k]), part);
    acc = fmaf(s, part, acc);
  }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) y[r] = __float2half(acc);
}

hipError_t launch_sparse_generic(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                 int64_t ldy, int M, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  const dim3 block(256);
  const int mt = M == 1 ? 1 : 4;
  const dim3 grid((w.rows + 3) / 4, (M + mt - 1) / mt);
  const int paired = w.val_kind == EGT_VAL_INT4_PAIRED ? 1 : 0;
  if (M == 1 && w.cols <= 131072) {                   // (the kernel divides by multiplication: exact for rows this wide and less)
    const bool x_in_lds = w.cols <= 32768;              // x through LDS while it fits (64 KB)
    const size_t lds = x_in_lds ? 2 * (((size_t)w.cols + 31) & ~(size_t)31) : 0;   // (the swizzle stays inside 32 halves)
#define EGT_GO1(KIND, RAGGED, XL)                                                                \
  launch(k_sparse_generic_m1<KIND, RAGGED, XL>, dim3(std::min((w.rows + 15) / 16, 512)), dim3(1024), lds, stream, w.row_ptr, \
         (const uint8_t *)w.values, w.idx, w.qparams, w.rows, w.cols, w.n_keep, w.total_slots, w.group_size, \
         (const __half *)X, (__half *)Y)
#define EGT_GO1_X(KIND, RAGGED) (x_in_lds ? EGT_GO1(KIND, RAGGED, true) : EGT_GO1(KIND, RAGGED, false))
#define EGT_GO1_R(KIND) (w.n_keep == 0 ? EGT_GO1_X(KIND, true) : EGT_GO1_X(KIND, false))
    if (w.val_kind == EGT_VAL_INT4) return EGT_GO1_R(EGT_VAL_INT4);
    if (w.val_kind == EGT_VAL_INT4_PAIRED) return EGT_GO1_R(EGT_VAL_INT4_PAIRED);
    return EGT_GO1_R(EGT_VAL_FP16);
#undef EGT_GO1_R
#undef EGT_GO1_X
#undef EGT_GO1
  }
#define EGT_GO(KIND, MT, RAGGED)                                                                 \
  launch(k_sparse_generic<KIND, MT, RAGGED>, grid, block, 0, stream, w.row_ptr, (const uint8_t *)w.values, \
         w.idx, w.qparams, w.rows, w.cols, w.n_keep, w.total_slots, w.group_size, paired, (const __half *)X, ldx, \
         (__half *)Y, ldy, M)
#define EGT_GO_MT(KIND, RAGGED) (mt == 1 ? EGT_GO(KIND, 1, RAGGED) : EGT_GO(KIND, 4, RAGGED))
  const bool int4 = w.val_kind != EGT_VAL_FP16;
  if (w.n_keep == 0)                                  // rows of different lengths
    return int4 ? EGT_GO_MT(EGT_VAL_INT4, true) : EGT_GO_MT(EGT_VAL_FP16, true);
  return int4 ? EGT_GO_MT(EGT_VAL_INT4, false) : EGT_GO_MT(EGT_VAL_FP16, false);
#undef EGT_GO_MT
#undef EGT_GO
}

hipError_t launch_int4_generic(const uint8_t *q, const uint16_t *qparams, int rows, int cols,
                               int group, const uint16_t *x, uint16_t *y, hipStream_t stream) {
  if (rows == 0) return hipSuccess;
  if (group % 8 != 0)
    return launch(k_int4_generic4, dim3((rows + 3) / 4), dim3(256), 0, stream, q, qparams, rows, cols,
                  group, (const __half *)x, (__half *)y);
  return launch(k_int4_generic, dim3((rows + 3) / 4), dim3(256), 0, stream, q, qparams, rows, cols,
                group, (const __half *)x, (__half *)y);
}

}  // namespace egt
