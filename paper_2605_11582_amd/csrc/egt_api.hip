// Device entry points of the C ABI: argument checks on the host, then dispatch to
// a kernel.  Nothing here synchronises or allocates.
#include "egt_device.h"

#include "egt_tune.h"

#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

namespace {

// `pointers`: also require the buffers (a size query looks at the shape only)
egt_status check_view(const egt_2bitcsr *w, bool pointers = true) {
  if (!w) return EGT_ERR_NULL;
  if (w->rows < 0 || w->cols < 0 || w->cols % 32 != 0) return EGT_ERR_SHAPE;
  if (w->n_keep < 0 || w->n_keep > 4) return EGT_ERR_SHAPE;
  // n_keep == 0: rows of different lengths; the buffers hold total_slots whole index words
  if (w->n_keep == 0 && (w->total_slots % 8 != 0 || (uint64_t)w->total_slots > (uint64_t)w->rows * (uint64_t)w->cols))
    return EGT_ERR_SHAPE;
  if (w->val_kind == EGT_VAL_INT4 || w->val_kind == EGT_VAL_INT4_PAIRED) {
    if (w->group_size <= 0 || w->group_size % 4 != 0 || w->cols % w->group_size != 0)
      return EGT_ERR_SHAPE;
    if (pointers && !w->qparams && w->rows != 0) return EGT_ERR_NULL;
  } else if (w->val_kind == EGT_VAL_FP16) {
    if (w->group_size != 0) return EGT_ERR_SHAPE;
  } else {
    return EGT_ERR_SHAPE;
  }
  if ((uint64_t)w->rows * (uint64_t)w->n_keep * (uint64_t)(w->cols / 4) >= (1ull << 32))
    return EGT_ERR_SHAPE;
  if (w->rows == 0 || !pointers) return EGT_OK;     // empty matrix: its buffers may be NULL
  if (!w->row_ptr || !w->values || !w->idx) return EGT_ERR_NULL;
  return EGT_OK;
}

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

thread_local hipError_t g_last_hip_error = hipSuccess;

inline egt_status done(hipError_t e) {
  if (e == hipSuccess) return EGT_OK;
  g_last_hip_error = e;
  return EGT_ERR_HIP;
}

// Streams `n16` 16-byte words; every workgroup folds what it read into one word.
// Each thread keeps U independent 128-bit loads in flight.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void fold_and_store(uint32_t acc, uint32_t *__restrict__ sink) {
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
  __shared__ uint32_t part[4];
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) sink[blockIdx.x] = part[0] ^ part[1] ^ part[2] ^ part[3];
}

// Grid-stride form for large buffers: a fixed number of workgroups walks the buffer.
template <int U>
__global__ __launch_bounds__(256) void k_stream_read(const u32x4 *__restrict__ src, size_t n16,
                                                      uint32_t *__restrict__ sink) {
  uint32_t acc = 0;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 a = src[i];
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
  fold_and_store(acc, sink);
}

// One-shot form, the launch shape of the M = 1 kernels: every workgroup owns U consecutive
// 4 KB pieces and each of its threads requests its U words before it looks at any of them,
// so the whole buffer is requested within the first moments of the kernel.  Words past the
// end are read from a clamped address and do not enter the fold.
template <int U>
__global__ __launch_bounds__(256) void k_stream_read_shot(const u32x4 *__restrict__ src, size_t n16,
                                                           uint32_t *__restrict__ sink) {
  const size_t base = (size_t)blockIdx.x * (256 * U) + threadIdx.x;
  u32x4 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t i = base + 256 * u;
    v[u] = __builtin_nontemporal_load(src + (i < n16 ? i : n16 - 1));
  }
  uint32_t acc = 0;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const uint32_t f = v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    acc ^= base + 256 * u < n16 ? f : 0u;
  }
  fold_and_store(acc, sink);
}

// Device memory of the allocation-free entry point: the partial sums of the split small-M
// kernels go here instead of into a caller's workspace.  Every GPU the library runs on
// holds its own copy of the array, at its own address, until the process ends.  In host
// code the array's name is only a handle: the address kernels can use comes from
// hipGetSymbolAddress, asked once per device with that device current, and is kept.
static __device__ __align__(256) unsigned char scratch[EGT_STATIC_SCRATCH_BYTES];

hipError_t static_scratch(void **out) {
  constexpr int MAX_DEVICES = 64;
  static std::mutex mu;
  static void *addr[MAX_DEVICES] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *out = addr[dev];
  return hipSuccess;
}

}  // namespace

namespace egt {
void note_hip_error(hipError_t e) { g_last_hip_error = e; }
}  // namespace egt

extern "C" {

const char *egt_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

egt_status egt_int4_gemv(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                         const uint16_t *x, uint16_t *y, void *stream) {
  if (rows < 0 || cols < 0 || group <= 0 || group % 4 != 0 || cols % group != 0)
    return EGT_ERR_SHAPE;
  if (rows == 0) return EGT_OK;                     // nothing to compute, pointers not examined
  if (!q || !qparams || !x || !y) return EGT_ERR_NULL;
  if (!aligned16(q) || !aligned16(qparams) || !aligned16(x)) return EGT_ERR_BUFFER;
  return done(egt::launch_int4(q, qparams, rows, cols, group, x, y, (hipStream_t)stream));
}

egt_status egt_sparse_gemm_smallm(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx,
                                  uint16_t *Y, int64_t ldy, int M, void *stream) {
  const egt_status st = check_view(w);
  if (st != EGT_OK) return st;
  if (M < 1 || M > 64 || ldx < w->cols || ldy < w->rows) return EGT_ERR_SHAPE;
  if (w->rows == 0) return EGT_OK;                  // nothing to compute, pointers not examined
  if (!X || !Y) return EGT_ERR_NULL;
  if (!aligned16(w->row_ptr) || !aligned16(w->values) || !aligned16(w->idx) ||
      (w->qparams && !aligned16(w->qparams)) || !aligned16(X))
    return EGT_ERR_BUFFER;
  return done(egt::launch_sparse(*w, X, ldx, Y, ldy, M, (hipStream_t)stream));
}

egt_status egt_sparse_gemm_smallm_ws_bytes(const egt_2bitcsr *w, int64_t ldx, int M, size_t *bytes) {
  if (!bytes) return EGT_ERR_NULL;
  const egt_status st = check_view(w, false);
  if (st != EGT_OK) return st;
  if (M < 1 || M > 64 || ldx < w->cols) return EGT_ERR_SHAPE;
  size_t need = 0;
  // (token rows of X off 16-byte boundaries: the split kernels do not apply, the call is the one-launch form)
  if (w->rows > 0 && ldx % 8 == 0) egt::sparse_smallm_split_bytes(*w, ldx, M, need);
  *bytes = need;
  return EGT_OK;
}

egt_status egt_sparse_gemm_smallm_ws(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                     int64_t ldy, int M, void *workspace, size_t workspace_bytes, void *stream) {
  const egt_status st = check_view(w);
  if (st != EGT_OK) return st;
  if (M < 1 || M > 64 || ldx < w->cols || ldy < w->rows) return EGT_ERR_SHAPE;
  if (w->rows == 0) return EGT_OK;
  size_t need = 0;
  const bool split = egt::sparse_smallm_split_bytes(*w, ldx, M, need) && ldx % 8 == 0;
  if (!split) return egt_sparse_gemm_smallm(w, X, ldx, Y, ldy, M, stream);   // no workspace needed: the one-launch form
  if (!X || !Y || !workspace) return EGT_ERR_NULL;
  if (workspace_bytes < need) return EGT_ERR_SHAPE;
  if (!aligned16(w->row_ptr) || !aligned16(w->values) || !aligned16(w->idx) || (w->qparams && !aligned16(w->qparams)) ||
      !aligned16(X) || !aligned16(workspace))
    return EGT_ERR_BUFFER;
  return done(egt::launch_sparse_smallm_split(*w, X, ldx, Y, ldy, M, (float *)workspace, (hipStream_t)stream));
}

egt_status egt_sparse_gemm_smallm_static(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                         int64_t ldy, int M, void *stream) {
  const egt_status st = check_view(w);
  if (st != EGT_OK) return st;
  if (M < 1 || M > 64 || ldx < w->cols || ldy < w->rows) return EGT_ERR_SHAPE;
  if (w->rows == 0) return EGT_OK;
  size_t need = 0;
  const bool split = egt::sparse_smallm_split_bytes(*w, ldx, M, need) && ldx % 8 == 0;
  if (!split) return egt_sparse_gemm_smallm(w, X, ldx, Y, ldy, M, stream);   // no partial sums in memory: nothing to place
  if (need > EGT_STATIC_SCRATCH_BYTES) return EGT_ERR_UNSUPPORTED;           // beyond the built-in buffer
  if (!X || !Y) return EGT_ERR_NULL;
  if (!aligned16(w->row_ptr) || !aligned16(w->values) || !aligned16(w->idx) || (w->qparams && !aligned16(w->qparams)) ||
      !aligned16(X))
    return EGT_ERR_BUFFER;
  void *ws = nullptr;
  const hipError_t e = static_scratch(&ws);
  if (e != hipSuccess) return done(e);
  // every partial sum the second kernel reads is written by the first: nothing to clear
  return done(egt::launch_sparse_smallm_split(*w, X, ldx, Y, ldy, M, (float *)ws, (hipStream_t)stream));
}

egt_status egt_sparse_gemv(const egt_2bitcsr *w, const uint16_t *x, uint16_t *y, void *stream) {
  if (!w) return EGT_ERR_NULL;
  return egt_sparse_gemm_smallm(w, x, w->cols, y, w->rows, 1, stream);
}

egt_status egt_sparse_gemv_batch(const egt_2bitcsr *w, const uint16_t *const *x, uint16_t *const *y,
                                 int count, void *stream) {
  if (!w || !x || !y) return EGT_ERR_NULL;
  if (count < 1 || count > 4) return EGT_ERR_SHAPE;
  for (int k = 0; k < count; ++k) {
    const egt_status st = check_view(&w[k]);
    if (st != EGT_OK) return st;
    if (w[k].rows != w[0].rows || w[k].cols != w[0].cols || w[k].n_keep != w[0].n_keep ||
        w[k].group_size != w[0].group_size || w[k].val_kind != w[0].val_kind)
      return EGT_ERR_SHAPE;
  }
  if (w[0].rows == 0) return EGT_OK;
  for (int k = 0; k < count; ++k) {
    if (!x[k] || !y[k]) return EGT_ERR_NULL;
    if (!aligned16(w[k].row_ptr) || !aligned16(w[k].values) || !aligned16(w[k].idx) ||
        (w[k].qparams && !aligned16(w[k].qparams)) || !aligned16(x[k]))
      return EGT_ERR_BUFFER;
  }
  return done(egt::launch_sparse_batch(w, x, y, count, (hipStream_t)stream));
}

egt_status egt_sparse_gemm_smallm_batch(const egt_2bitcsr *w, const uint16_t *const *X, int64_t ldx,
                                        uint16_t *const *Y, int64_t ldy, int M, int count, void *stream) {
  if (!w || !X || !Y) return EGT_ERR_NULL;
  if (count < 1 || count > 4) return EGT_ERR_SHAPE;
  for (int k = 0; k < count; ++k) {
    const egt_status st = check_view(&w[k]);
    if (st != EGT_OK) return st;
    if (w[k].rows != w[0].rows || w[k].cols != w[0].cols || w[k].n_keep != w[0].n_keep ||
        w[k].group_size != w[0].group_size || w[k].val_kind != w[0].val_kind || w[k].total_slots != w[0].total_slots)
      return EGT_ERR_SHAPE;
  }
  if (M < 1 || M > 64 || ldx < w[0].cols || ldy < w[0].rows) return EGT_ERR_SHAPE;
  if (w[0].rows == 0) return EGT_OK;
  for (int k = 0; k < count; ++k) {
    if (!X[k] || !Y[k]) return EGT_ERR_NULL;
    if (!aligned16(w[k].row_ptr) || !aligned16(w[k].values) || !aligned16(w[k].idx) ||
        (w[k].qparams && !aligned16(w[k].qparams)) || !aligned16(X[k]))
      return EGT_ERR_BUFFER;
  }
  return done(egt::launch_sparse_gemm_batch(w, X, ldx, Y, ldy, M, count, (hipStream_t)stream));
}

// descriptors, then one 32-bit word per workgroup, rounded up to 16 bytes
static uint64_t gemm_table_bytes(int count, int grid_x) {
  return (uint64_t)count * EGT_STACK_ENTRY_BYTES + (((uint64_t)grid_x * 4 + 15) & ~(uint64_t)15);
}

egt_status egt_gemm_stack_plan(const egt_gemm_item *items, int count, int M, void *table, size_t table_bytes,
                               egt_gemm_plan *plan) {
  if (!items || !plan) return EGT_ERR_NULL;
  if (count < 1 || count > 65535 || M < 2 || M > 64) return EGT_ERR_SHAPE;
  uint64_t nwg = 0;
  for (int k = 0; k < count; ++k) {
    const egt_2bitcsr *w = items[k].sparse;
    if (!w) return EGT_ERR_NULL;
    const egt_status st = check_view(w);
    if (st != EGT_OK) return st;
    if (w->rows != 0 && (!items[k].X || !items[k].Y)) return EGT_ERR_NULL;
    if (!aligned16(w->row_ptr) || !aligned16(w->values) || !aligned16(w->idx) || !aligned16(w->qparams) ||
        !aligned16(items[k].X))
      return EGT_ERR_BUFFER;
    if (!egt::smallm_stack_item_ok(*w, M)) return EGT_ERR_UNSUPPORTED;
    if (w->n_keep != items[0].sparse->n_keep) return EGT_ERR_UNSUPPORTED;   // one storage form per table (one kernel)
    const int blocks = egt::smallm_stack_blocks(M, w->n_keep, w->rows);
    if (blocks > 0xFFFF) return EGT_ERR_UNSUPPORTED;                         // (the list names a workgroup's place in 16 bits)
    nwg += (uint64_t)blocks;
  }
  if (nwg > (1u << 24)) return EGT_ERR_UNSUPPORTED;
  const int n_keep = items[0].sparse->n_keep;
  egt_gemm_plan out;
  std::memset(&out, 0, sizeof(out));
  out.count = count;
  out.M = M;
  out.n_keep = n_keep;
  out.grid_x = (int32_t)nwg;
  egt::smallm_stack_shape(M, n_keep, out.block_threads, out.lds_bytes);
  out.table_bytes = gemm_table_bytes(count, out.grid_x);
  if (table) {
    if ((uint64_t)table_bytes < out.table_bytes) return EGT_ERR_SHAPE;
    // Descriptors in the order of falling row length (a stable sort): a workgroup walks all of K, so the matrices
    // with the longest rows start first and the launch ends on short workgroups.  The order of the table is
    // nobody's business but the kernel's: every descriptor names its own X and Y.
    std::vector<int> order((size_t)count);
    for (int k = 0; k < count; ++k) order[(size_t)k] = k;
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return items[a].sparse->cols > items[b].sparse->cols; });
    std::memset(table, 0, (size_t)out.table_bytes);
    uint32_t *list = (uint32_t *)((uint8_t *)table + (size_t)count * EGT_STACK_ENTRY_BYTES);
    for (int k = 0; k < count; ++k) {
      const egt_gemm_item &it = items[order[(size_t)k]];
      egt::smallm_stack_entry(*it.sparse, it.X, it.Y, M, (uint8_t *)table + (size_t)k * EGT_STACK_ENTRY_BYTES);
      const int blocks = egt::smallm_stack_blocks(M, n_keep, it.sparse->rows);
      for (int x = 0; x < blocks; ++x) *list++ = ((uint32_t)k << 16) | (uint32_t)x;   // matrix, place in the matrix
    }
  }
  *plan = out;
  return EGT_OK;
}

egt_status egt_gemm_stack_run(const void *table_dev, const egt_gemm_plan *plan, void *stream) {
  if (!table_dev || !plan) return EGT_ERR_NULL;
  if (!aligned16(table_dev)) return EGT_ERR_BUFFER;
  if (plan->count < 1 || plan->count > 65535 || plan->M < 2 || plan->M > 64 || (plan->n_keep != 1 && plan->n_keep != 2) ||
      (plan->n_keep == 1 && plan->M > 32))
    return EGT_ERR_SHAPE;
  int threads, lds;
  egt::smallm_stack_shape(plan->M, plan->n_keep, threads, lds);
  if (plan->grid_x < 0 || plan->grid_x > (1 << 24) || plan->block_threads != threads || plan->lds_bytes != lds ||
      plan->table_bytes != gemm_table_bytes(plan->count, plan->grid_x))
    return EGT_ERR_SHAPE;
  if (plan->grid_x == 0) return EGT_OK;               // every matrix is empty
  return done(egt::launch_smallm_stack(table_dev, plan->count, plan->M, plan->n_keep, plan->grid_x, (hipStream_t)stream));
}

egt_status egt_int4_gemv_batch(const uint8_t *const *q, const uint16_t *const *qparams, int rows,
                               int cols, int group, const uint16_t *const *x, uint16_t *const *y,
                               int count, void *stream) {
  if (!q || !qparams || !x || !y) return EGT_ERR_NULL;
  if (count < 1 || count > 4) return EGT_ERR_SHAPE;
  if (rows < 0 || cols < 0 || group <= 0 || group % 4 != 0 || cols % group != 0)
    return EGT_ERR_SHAPE;
  if (rows == 0) return EGT_OK;
  for (int k = 0; k < count; ++k) {
    if (!q[k] || !qparams[k] || !x[k] || !y[k]) return EGT_ERR_NULL;
    if (!aligned16(q[k]) || !aligned16(qparams[k]) || !aligned16(x[k])) return EGT_ERR_BUFFER;
  }
  return done(egt::launch_int4_batch(q, qparams, rows, cols, group, x, y, count, (hipStream_t)stream));
}

egt_status egt_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream) {
  if (!src || !sink) return EGT_ERR_NULL;
  if (bytes % 16 != 0) return EGT_ERR_SHAPE;
  if (!aligned16(src)) return EGT_ERR_BUFFER;
  if (bytes == 0) return EGT_OK;
  const size_t n16 = bytes / 16;
  // loads in flight per thread; shape 0 = one-shot (one workgroup per U * 4 KB, at most 4096
  // of them), shape k > 0 = k * 256 workgroups walking the buffer
  int unroll = 8, shape = 0;
  egt::tune_pair("EGT_READ_TUNE", unroll, shape);
  if (unroll != 4 && unroll != 8 && unroll != 16) unroll = 8;
  shape = shape < 0 ? 0 : shape > 16 ? 16 : shape;
  const hipStream_t st = (hipStream_t)stream;
  const u32x4 *p = (const u32x4 *)src;
  const size_t shot_blocks = (n16 + 256 * (size_t)unroll - 1) / (256 * (size_t)unroll);
  if (shape == 0 && shot_blocks <= 4096) {
    const dim3 grid((unsigned)shot_blocks), block(256);
    switch (unroll) {
      case 4: return done(egt::launch(k_stream_read_shot<4>, grid, block, 0, st, p, n16, sink));
      case 16: return done(egt::launch(k_stream_read_shot<16>, grid, block, 0, st, p, n16, sink));
      default: return done(egt::launch(k_stream_read_shot<8>, grid, block, 0, st, p, n16, sink));
    }
  }
  if (shape == 0) shape = 8;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * (size_t)shape) blocks = 256 * (size_t)shape;
  const dim3 grid((unsigned)blocks), block(256);
  switch (unroll) {
    case 4: return done(egt::launch(k_stream_read<4>, grid, block, 0, st, p, n16, sink));
    case 16: return done(egt::launch(k_stream_read<16>, grid, block, 0, st, p, n16, sink));
    default: return done(egt::launch(k_stream_read<8>, grid, block, 0, st, p, n16, sink));
  }
}

}  // extern "C"
