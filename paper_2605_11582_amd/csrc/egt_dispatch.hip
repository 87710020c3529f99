// Kernel selection for the device entry points.
#include "egt_device.h"

#include "egt_tune.h"

namespace egt {

hipError_t launch_sparse(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                         int64_t ldy, int M, hipStream_t stream) {
  if (w.val_kind == EGT_VAL_INT4_PAIRED) {            // tuned for M = 1 at 2:4; everything else slot by slot
    if (M == 1 && sparse_m1_paired_supported(w)) return launch_sparse_m1_paired(w, X, Y, stream);
    return launch_sparse_generic(w, X, ldx, Y, ldy, M, stream);
  }
  if (M == 1 && sparse_m1_supported(w)) return launch_sparse_m1(w, X, Y, stream);
  if (M == 1 && sparse_m1_n1_supported(w)) return launch_sparse_m1_n1(w, X, Y, stream);
  // 16-byte loads of X: token rows must start on a 16-byte boundary there
  if (M >= 2 && ldx % 8 == 0 && sparse_m1_tokens_supported(w, M) && !tune_flag("EGT_NO_M1T"))
    return launch_sparse_m1_tokens(w, X, ldx, Y, ldy, M, stream);
  if (M >= 2 && sparse_smallm_supported(w, ldx, M)) return launch_sparse_smallm(w, X, ldx, Y, ldy, M, stream);
  return launch_sparse_generic(w, X, ldx, Y, ldy, M, stream);
}

hipError_t launch_int4(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                       const uint16_t *x, uint16_t *y, hipStream_t stream) {
  if (int4_m1_supported(cols, group)) return launch_int4_m1(q, qparams, rows, cols, group, x, y, stream);
  return launch_int4_generic(q, qparams, rows, cols, group, x, y, stream);
}

hipError_t launch_sparse_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                               int count, hipStream_t stream) {
  if (ws[0].val_kind == EGT_VAL_INT4_PAIRED) {        // no batched form: one launch each
    for (int k = 0; k < count; ++k) {
      const hipError_t e = launch_sparse(ws[k], xs[k], ws[k].cols, ys[k], ws[k].rows, 1, stream);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (sparse_m1_supported(ws[0])) return launch_sparse_m1_batch(ws, xs, ys, count, stream);
  if (sparse_m1_n1_supported(ws[0])) return launch_sparse_m1_n1_batch(ws, xs, ys, count, stream);
  for (int k = 0; k < count; ++k) {                   // shapes without a tuned kernel: one launch each
    const hipError_t e = launch_sparse_generic(ws[k], xs[k], ws[k].cols, ys[k], ws[k].rows, 1, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_sparse_gemm_batch(const egt_2bitcsr *ws, const uint16_t *const *Xs, int64_t ldx, uint16_t *const *Ys,
                                    int64_t ldy, int M, int count, hipStream_t stream) {
  const egt_2bitcsr &w = ws[0];
  // the small-M kernel where a single call would take it (M = 1 and the few-token form of the M = 1 kernel have
  // batched forms of their own or none: one launch per member there)
  const bool tokens_form = M >= 2 && ldx % 8 == 0 && sparse_m1_tokens_supported(w, M) && !tune_flag("EGT_NO_M1T");
  if (count >= 2 && M >= 2 && w.val_kind != EGT_VAL_INT4_PAIRED && !tokens_form && sparse_smallm_supported(w, ldx, M))
    return launch_sparse_smallm_batch(ws, Xs, ldx, Ys, ldy, M, count, stream);
  for (int k = 0; k < count; ++k) {
    const hipError_t e = launch_sparse(ws[k], Xs[k], ldx, Ys[k], ldy, M, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_int4_batch(const uint8_t *const *qs, const uint16_t *const *qps, int rows, int cols,
                             int group, const uint16_t *const *xs, uint16_t *const *ys, int count,
                             hipStream_t stream) {
  if (int4_m1_supported(cols, group)) return launch_int4_m1_batch(qs, qps, rows, cols, group, xs, ys, count, stream);
  for (int k = 0; k < count; ++k) {
    const hipError_t e = launch_int4_generic(qs[k], qps[k], rows, cols, group, xs[k], ys[k], stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace egt
