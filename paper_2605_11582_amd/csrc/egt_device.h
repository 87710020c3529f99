// Internal declarations shared by the device translation units of the library.
#ifndef EGT_DEVICE_H
#define EGT_DEVICE_H

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "egt.h"

namespace egt {

// generic, slot-by-slot kernels (any shape the format allows)
hipError_t launch_sparse_generic(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                 int64_t ldy, int M, hipStream_t stream);
hipError_t launch_int4_generic(const uint8_t *q, const uint16_t *qparams, int rows, int cols,
                               int group, const uint16_t *x, uint16_t *y, hipStream_t stream);

// dispatchers: pick the tuned kernel for the shape, else the generic one
hipError_t launch_sparse(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                         int64_t ldy, int M, hipStream_t stream);
hipError_t launch_int4(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                       const uint16_t *x, uint16_t *y, hipStream_t stream);

}  // namespace egt
#endif
