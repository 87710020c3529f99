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
