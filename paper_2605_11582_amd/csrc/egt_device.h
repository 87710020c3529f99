// Internal declarations shared by the device translation units of the library.
#ifndef EGT_DEVICE_H
#define EGT_DEVICE_H

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "egt.h"

namespace egt {

// Launch through hipLaunchKernel so that the status is the launch's own return
// value (hipGetLastError may carry a stale, unrelated code of the calling thread).
template <typename... P, typename... A>
inline hipError_t launch(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         A... args) {
  auto pack = [&](P... p) {
    void *argv[] = {(void *)&p...};
    return hipLaunchKernel((const void *)kernel, grid, block, argv, lds, stream);
  };
  return pack(static_cast<P>(args)...);
}

// code of the most recent failing HIP call made by this library on this thread
void note_hip_error(hipError_t e);

// generic, slot-by-slot kernels (any shape the format allows)
hipError_t launch_sparse_generic(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                 int64_t ldy, int M, hipStream_t stream);
hipError_t launch_int4_generic(const uint8_t *q, const uint16_t *qparams, int rows, int cols,
                               int group, const uint16_t *x, uint16_t *y, hipStream_t stream);

// M = 1 kernels on the sparse matrix cores (2:4 only; see sparse_m1_supported)
bool sparse_m1_supported(const egt_2bitcsr &w);
hipError_t launch_sparse_m1(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream);
bool sparse_m1_paired_supported(const egt_2bitcsr &w);      // INT4 values in the paired nibble order
hipError_t launch_sparse_m1_paired(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream);

// M = 1, 1:4 sparsity (see sparse_m1_n1_supported)
bool sparse_m1_n1_supported(const egt_2bitcsr &w);
hipError_t launch_sparse_m1_n1(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream);

// 2 <= M <= 64 on the sparse matrix cores (2:4 and 1:4; see sparse_smallm_supported)
bool sparse_smallm_supported(const egt_2bitcsr &w, int64_t ldx, int M);
hipError_t launch_sparse_smallm(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                int64_t ldy, int M, hipStream_t stream);
hipError_t launch_sparse_smallm_batch(const egt_2bitcsr *ws, const uint16_t *const *Xs, int64_t ldx, uint16_t *const *Ys,
                                      int64_t ldy, int M, int count, hipStream_t stream);
// any number of 2:4 (or of 1:4) INT4 small-M products in one launch (egt_gemm_stack_plan / egt_gemm_stack_run)
bool smallm_stack_item_ok(const egt_2bitcsr &w, int M);
int smallm_stack_blocks(int M, int n_keep, int rows);
void smallm_stack_shape(int M, int n_keep, int &block_threads, int &lds_bytes);
void smallm_stack_entry(const egt_2bitcsr &w, const uint16_t *X, uint16_t *Y, int M, void *entry);
hipError_t launch_smallm_stack(const void *table_dev, int count, int M, int n_keep, int grid_x, hipStream_t stream);
// (dispatch: identically shaped members; falls back to one launch per member where no batched kernel applies)
hipError_t launch_sparse_gemm_batch(const egt_2bitcsr *ws, const uint16_t *const *Xs, int64_t ldx, uint16_t *const *Ys,
                                    int64_t ldy, int M, int count, hipStream_t stream);

// the same with K split over workgroups and FP32 partial sums in a workspace of the caller
// (sparse_smallm_split_bytes: false if this shape and M do not use the split form)
bool sparse_smallm_split_bytes(const egt_2bitcsr &w, int64_t ldx, int M, size_t &bytes);
hipError_t launch_sparse_smallm_split(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                      int64_t ldy, int M, float *ws, hipStream_t stream);

// dense INT4, M = 1, on the matrix cores (group sizes 32 << j; see int4_m1_supported)
bool int4_m1_supported(int cols, int group);
hipError_t launch_int4_m1(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                          const uint16_t *x, uint16_t *y, hipStream_t stream);

// 2:4 INT4, 2..4 activation rows on the M = 1 kernel's row-per-wave mapping
bool sparse_m1_tokens_supported(const egt_2bitcsr &w, int M);
hipError_t launch_sparse_m1_tokens(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                   int64_t ldy, int M, hipStream_t stream);

// batched forms: `count` identically shaped matrices in one launch (count <= 4)
hipError_t launch_sparse_m1_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                                  int count, hipStream_t stream);
hipError_t launch_sparse_m1_n1_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                                     int count, hipStream_t stream);
hipError_t launch_int4_m1_batch(const uint8_t *const *qs, const uint16_t *const *qps, int rows, int cols,
                                int group, const uint16_t *const *xs, uint16_t *const *ys, int count,
                                hipStream_t stream);

// dispatchers: pick the tuned kernel for the shape, else the generic one
hipError_t launch_sparse(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                         int64_t ldy, int M, hipStream_t stream);
hipError_t launch_int4(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                       const uint16_t *x, uint16_t *y, hipStream_t stream);

hipError_t launch_sparse_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                               int count, hipStream_t stream);
hipError_t launch_int4_batch(const uint8_t *const *qs, const uint16_t *const *qps, int rows, int cols,
                             int group, const uint16_t *const *xs, uint16_t *const *ys, int count,
                             hipStream_t stream);

}  // namespace egt
#endif
