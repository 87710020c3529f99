/* egt.h - C ABI of the SparseGemv library for MI355X (gfx950).
 *
 * The library implements the decode-time product y = W.x of the paper's
 * "Revised Kernel" section (Sec. 3.3): W is a weight matrix compressed offline by
 * group-wise INT4 quantisation (Sec. 3.2 "Adaptive Group-Wise Quantization") and
 * N:4 semi-structured pruning (Sec. 3.2 "Sparsification"), stored in the
 * index-compressed CSR variant of Sec. 3.3 "Sparse Index Structure" (called
 * 2bit-CSR here); x is an FP16 activation vector.  A small-M form serves the
 * parallel verification step of Sec. 3.4, where several candidate tokens pass
 * through the same linear layers at once.
 *
 * General rules
 *  - Plain C linkage, no exceptions cross the boundary, no global state; every
 *    call is thread-safe with respect to the library (buffers are the caller's).
 *  - The library never allocates or frees device memory and keeps no handles.
 *    Every buffer is owned by the caller.
 *  - "HOST" functions take host pointers and run on the CPU.  "DEVICE" functions
 *    take device pointers (16-byte aligned), enqueue kernels on `stream`
 *    (a hipStream_t passed as void*, NULL = the default stream) and return
 *    without synchronising.
 *  - A device call on a matrix with rows == 0 is a no-op that returns EGT_OK
 *    without looking at the buffer pointers.
 *  - Argument errors are detected on the host before anything is written or
 *    launched; outputs are untouched when a call returns an error.
 *  - FP16 numbers cross the boundary as their IEEE binary16 bit patterns
 *    (uint16_t).
 *
 * The 2bit-CSR format (canonical layout)
 *    R rows, K columns, K % 32 == 0.  Columns are cut into 4-groups [4c, 4c+4).
 *    n = n_keep (1..4) entries of every 4-group own a slot; a row has
 *    S = n*K/4 slots in ascending column order and the in-group offsets (0..3)
 *    of one 4-group are strictly ascending.
 *      row_ptr  uint32[R+1]   first slot of each row (slot units); rows are
 *                             uniform, so row_ptr[r] = r*S.
 *      idx      uint16[T/8]   T = R*S.  Slot t lives in word t>>3 at bits
 *                             [2*(t&7), 2*(t&7)+1]: the first slot of a word
 *                             sits in its least-significant bits, so
 *                             offset = (word >> 2*(t&7)) & 3.
 *      values   INT4: uint8[T/2], slot t in byte t>>1, low nibble for even t.
 *               FP16: uint16[T], raw bits of the kept weight (+0.0 for padding).
 *      qparams  INT4 only: uint16[R][K/g][2] = FP16 bits of {scale s, zero z} of
 *               the group of g consecutive *dense* columns; z is an integer
 *               0..15; a code q decodes to s*(q - z).
 *    Quantiser (per row and group, over the kept values V of the group):
 *      xmin = min(0, min V), xmax = max(0, max V),
 *      s = fp16((xmax - xmin)/15) rounded once to nearest-even, s = 1 if that is 0,
 *      z = clamp(rint(-xmin/s), 0, 15), q = clamp(rint(v/s) + z, 0, 15),
 *      all in binary64 with rint = ties-to-even.
 *    A 4-group whose mask keeps fewer than n entries is padded with the
 *    smallest unused offsets; padding slots hold an exact zero (q = z or +0.0).
 *
 * Rows of different lengths (Sec. 3.2 makes N of N:4 adaptive; Sec. 3.3 gives the format
 * CSR-like row pointers): a matrix packed by egt_pack_2bitcsr_rows keeps n_r in 1..4
 * entries per 4-group in row r, row r has S_r = n_r*K/4 slots, row_ptr is the running sum
 * of the S_r and T = row_ptr[R].  Such a view has n_keep = 0 and says T in total_slots.
 * Everything else (slot order, index words, nibbles, qparams per row and dense group) is
 * as above; a row starts on a whole index word and a whole byte because K % 32 == 0.
 */
#ifndef EGT_H
#define EGT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EGT_OK = 0,
  EGT_ERR_NULL = 1,        /* a required pointer is NULL                                  */
  EGT_ERR_SHAPE = 2,       /* rows/cols/n_keep/group/M/leading dimension out of range     */
  EGT_ERR_MASK = 3,        /* a 4-group of the mask keeps more than n_keep entries        */
  EGT_ERR_NONFINITE = 4,   /* a kept weight is NaN or Inf                                 */
  EGT_ERR_BUFFER = 5,      /* inconsistent buffer contents (e.g. row_ptr not uniform)     */
  EGT_ERR_UNSUPPORTED = 6, /* valid format, but no kernel covers it                       */
  EGT_ERR_HIP = 7          /* the HIP runtime reported an error at launch                 */
} egt_status;

/* EGT_VAL_INT4_PAIRED: INT4 values in a second nibble order (Sec. 3.3 reorders what it
 * stores so that plain bit operations recover it; this is that idea applied to the codes).
 * Inside every word of eight slots - the 32 bits of values that one index word speaks for -
 * slot j sits in nibble (j >> 1) + 4 (j & 1): the nibbles of the word, from the low bits,
 * hold the slots 0, 2, 4, 6, 1, 3, 5, 7, so that `word & 0x000F000F` is the slot pair (0, 1),
 * `word & 0x00F000F0` the pair (2, 3), and the same two masks on `word >> 8` the pairs
 * (4, 5) and (6, 7): the pairs a matrix-core operand register wants, without a byte
 * permute.  Everything else (index words, parameters, sizes, row pointers) is as for
 * EGT_VAL_INT4.  The M = 1 kernels for 2:4 with groups of 128 columns and more are tuned
 * for it; every other call takes it through the slot-by-slot kernels. */
typedef enum { EGT_VAL_INT4 = 0, EGT_VAL_FP16 = 1, EGT_VAL_INT4_PAIRED = 2 } egt_val_kind;

/* A view of one matrix in 2bit-CSR.  The struct itself lives in host memory.
 * Its pointer fields are host pointers for pack/unpack and device pointers for
 * the GEMV calls.  The library never owns them. */
typedef struct {
  int32_t rows, cols;    /* R = output features, K = input features (reduction axis) */
  int32_t n_keep;        /* n of n:4                                                  */
  int32_t group_size;    /* g, along dense K; INT4 only; 0 for FP16 values            */
  int32_t val_kind;      /* egt_val_kind                                              */
  uint32_t *row_ptr;     /* [R+1]                                                     */
  void *values;          /* INT4: T/2 bytes; FP16: 2*T bytes                          */
  uint16_t *idx;         /* [T/8]                                                     */
  uint16_t *qparams;     /* INT4: [R][K/g][2]; FP16 values: NULL                      */
  uint32_t total_slots;  /* rows of different lengths (n_keep == 0) only: T, the extent
                            of values and idx that the caller vouches for                */
} egt_2bitcsr;

/* Text for a status code (static storage, never NULL). */
const char *egt_status_str(egt_status status);

/* Text of the HIP error behind the most recent EGT_ERR_HIP returned to the
 * calling thread ("no error" if there was none).  Diagnostic aid. */
const char *egt_last_hip_error(void);

/* HOST.  Byte sizes of the four buffers {row_ptr, values, idx, qparams} of a
 * matrix (Sec. 3.3 "Sparse Index Structure").  EGT_ERR_SHAPE unless
 * cols % 32 == 0, n_keep in 1..4 and, for INT4, group > 0, group % 4 == 0 and
 * cols % group == 0 (group must be 0 for FP16 values). */
egt_status egt_2bitcsr_sizes(int rows, int cols, int n_keep, int group, int val_kind,
                             size_t bytes[4]);

/* HOST.  N:4 magnitude pruning mask (Sec. 3.2 "Sparsification"; Eq. (3) with a
 * constant activation norm and gradient reduces to |W_ij|).  w: rows x cols FP16
 * bits, row stride ldw elements.  mask: rows x cols bytes, row stride ldm, set to
 * 1 for the n_keep entries of largest magnitude of every 4-group (equal
 * magnitudes: lower column wins; -0.0 has magnitude 0), else 0.  cols % 4 == 0. */
egt_status egt_prune_n4(const uint16_t *w, int64_t ldw, int rows, int cols, int n_keep,
                        uint8_t *mask, int64_t ldm);

/* HOST.  N:4 pruning mask by the importance score of Eq. (3) (Sec. 3.2
 * "Sparsification"): I_ij = |W_ij| * ||X_j||_2 + |W_ij| * |dE/dW_ij|, evaluated in
 * float64 as written (two products, one sum, no fused multiply-add).  act_norm: cols
 * floats, the activation norm of every input feature; grad_abs: rows x cols floats,
 * row stride ldg, the gradient magnitudes, or NULL for a zero gradient term.  The
 * n_keep entries of largest score of every 4-group are kept (equal scores: lower column
 * wins).  EGT_ERR_NONFINITE if a weight, norm or gradient is NaN or infinite or a norm
 * or gradient is negative; the mask is untouched then. */
egt_status egt_prune_n4_importance(const uint16_t *w, int64_t ldw, const float *act_norm,
                                   const float *grad_abs, int64_t ldg, int rows, int cols,
                                   int n_keep, uint8_t *mask, int64_t ldm);

/* HOST.  Encoder of Sec. 3.3 "Sparse Index Structure" fused with the quantiser of
 * Sec. 3.2: dense FP16 W + 0/1 mask + group size -> 2bit-CSR.  `out` has its five
 * scalars ignored on input and filled on success; its four buffers are
 * caller-allocated HOST memory of the sizes egt_2bitcsr_sizes reports (qparams
 * may be NULL for FP16 values).  Errors: EGT_ERR_MASK when a 4-group keeps more
 * than n_keep entries, EGT_ERR_NONFINITE when a kept weight is NaN/Inf. */
egt_status egt_pack_2bitcsr(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                            int rows, int cols, int n_keep, int group, int val_kind,
                            egt_2bitcsr *out);

/* HOST.  The encoder for rows of different lengths: row r keeps row_n_keep[r] in 1..4
 * entries per 4-group (a 4-group of row r whose mask keeps more is EGT_ERR_MASK).  `out`
 * gets n_keep = 0 and total_slots; its buffers have the sizes egt_2bitcsr_sizes_rows
 * reports.  A 2:4 matrix in which half of the rows are 1:4 moves a quarter fewer bytes
 * than the 2:4 matrix with those rows padded. */
egt_status egt_2bitcsr_sizes_rows(int rows, int cols, const int32_t *row_n_keep, int group, int val_kind,
                                  size_t bytes[4]);
egt_status egt_pack_2bitcsr_rows(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                                 int rows, int cols, const int32_t *row_n_keep, int group, int val_kind,
                                 egt_2bitcsr *out);

/* HOST.  The same encoder with a group size per row (Sec. 3.2 "Adaptive Group-Wise
 * Quantization": channels found sensitive get more, smaller groups, robust ones fewer).
 * row_group: rows entries, each a multiple of `group` that divides cols (else
 * EGT_ERR_SHAPE); NULL means `group` for every row.  Row r is quantised in groups of
 * row_group[r] columns.  The stored parameters keep the granularity `group`
 * (out->group_size = group): a coarser group repeats its {scale, zero} pair, so the
 * device kernels and egt_unpack_2bitcsr read the result like any other matrix; the
 * bytes moved are those of the finest group size.  INT4 values only. */
egt_status egt_pack_2bitcsr_rowgroups(const uint16_t *w, int64_t ldw, const uint8_t *mask, int64_t ldm,
                                      int rows, int cols, int n_keep, int group, int val_kind,
                                      const int32_t *row_group, egt_2bitcsr *out);

/* HOST.  Inverse of the encoder: writes the decoded matrix (FP16 bits; s*(q-z)
 * rounded once to FP16 for INT4 values; 0 where no slot exists) and the mask of
 * positions that own a slot.  Either output may be NULL.  EGT_ERR_BUFFER when
 * row_ptr is not the uniform progression (n_keep = 0: not a running sum of whole rows of
 * 1..4 entries per 4-group that ends at total_slots) or offsets are not ascending. */
egt_status egt_unpack_2bitcsr(const egt_2bitcsr *in, uint16_t *w_dense, int64_t ldw,
                              uint8_t *mask, int64_t ldm);

/* HOST.  Dense group-wise INT4 quantiser of the earlier "Gemv" kernel that
 * Sec. 3.3 starts from: every column kept, same quantiser as above.
 * q: rows x cols/2 bytes (column c in byte c>>1, low nibble for even c);
 * qparams: [rows][cols/group][2] FP16 bits.  cols % group == 0, group % 4 == 0. */
egt_status egt_quant_int4(const uint16_t *w, int64_t ldw, int rows, int cols, int group,
                          uint8_t *q, uint16_t *qparams);

/* DEVICE.  y[r] = sum_c s(r,c/g) * (q(r,c) - z(r,c/g)) * x[c]: the dense
 * weight-only INT4 GEMV (Sec. 3.3, "previous generation of Gemv").  x: cols FP16,
 * y: rows FP16 (FP32 accumulation, one rounding at the end). */
egt_status egt_int4_gemv(const uint8_t *q, const uint16_t *qparams, int rows, int cols,
                         int group, const uint16_t *x, uint16_t *y, void *stream);

/* DEVICE.  SparseGemv (Sec. 3.3 "Computational Acceleration"): y = W.x for W in
 * 2bit-CSR with INT4 or FP16 values.  x: cols FP16, y: rows FP16.  A row whose
 * row_ptr entry is not r*S yields NaN in y[r] (the kernel checks it).  Rows of
 * different lengths (n_keep = 0) are followed through row_ptr by a slot-by-slot kernel;
 * a row whose pointers do not describe a whole row of 1..4 entries per 4-group that
 * starts on an index word and ends inside total_slots yields NaN and is never read. */
egt_status egt_sparse_gemv(const egt_2bitcsr *w, const uint16_t *x, uint16_t *y, void *stream);

/* DEVICE.  Small-M form for tree-based parallel verification (Sec. 3.4): the M
 * candidate rows of X go through the same compressed matrix in one call.
 * X: M x K row-major with row stride ldx; Y: M x R row-major with row stride ldy;
 * Y[m][r] = sum_k W[r][k] * X[m][k]; 1 <= M <= 64. */
egt_status egt_sparse_gemm_smallm(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx,
                                  uint16_t *Y, int64_t ldy, int M, void *stream);

/* The same product with K split over workgroups (Sec. 3.4: the cost of a verification step
 * grows with the number of candidates; from about five candidates on, what grows is the
 * traffic of X, which every compute unit of the one-launch form reads in full).  The grid is
 * cut into row blocks x K slices, a workgroup reads only its slice of X, the FP32 partial
 * sums of the slices pass through `workspace` (DEVICE memory of the caller, 16-byte
 * aligned) and a second kernel adds them in slice order, so results are reproducible
 * run to run; they differ from egt_sparse_gemm_smallm's in the order of the FP32 additions
 * only.  The workspace is dead after the call's kernels have run; calls that share one
 * must not overlap.
 * egt_sparse_gemm_smallm_ws_bytes (HOST): the bytes this matrix and M need; 0 where the
 * split form is not the faster one (it is for 2:4 INT4 with groups of 64 columns and more
 * and either M > 32 with K >= 8192 or at least 8192 rows - there the slice of X of a
 * workgroup stays in LDS - or M > 16, K >= 8192 and at most 4096 rows: the down projection
 * under verification), in which case egt_sparse_gemm_smallm_ws ignores the workspace and is
 * the one-launch call.
 * EGT_ERR_SHAPE when workspace_bytes is smaller than required. */
egt_status egt_sparse_gemm_smallm_ws_bytes(const egt_2bitcsr *w, int64_t ldx, int M, size_t *bytes);
egt_status egt_sparse_gemm_smallm_ws(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx,
                                     uint16_t *Y, int64_t ldy, int M, void *workspace,
                                     size_t workspace_bytes, void *stream);

/* DEVICE.  egt_sparse_gemm_smallm_ws for callers that cannot allocate device memory and
 * have no workspace to hand over: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The partial sums go to a buffer of
 * EGT_STATIC_SCRATCH_BYTES that is part of the library's device image (every GPU the library
 * runs on holds it until the process ends); the call allocates and frees nothing.  A
 * matrix and M whose partial sums need more give EGT_ERR_UNSUPPORTED (use the workspace
 * form); where the split form does not apply the call is egt_sparse_gemm_smallm.  All
 * calls on one GPU share that buffer: calls that overlap on one GPU (two streams, two
 * threads) race, whoever makes them must order them.  Results equal
 * egt_sparse_gemm_smallm_ws's bit for bit. */
#define EGT_STATIC_SCRATCH_BYTES (16u << 20) /* 64 tokens: eleven slices x 4096 rows or four slices x 11008 rows of FP32 */
egt_status egt_sparse_gemm_smallm_static(const egt_2bitcsr *w, const uint16_t *X, int64_t ldx,
                                         uint16_t *Y, int64_t ldy, int M, void *stream);

/* DEVICE.  `count` (1..4) independent products y[k] = W[k].x[k] of identically shaped
 * matrices (same rows, cols, n_keep, group_size, val_kind; else EGT_ERR_SHAPE) in one
 * launch: the q/k/v or gate/up projections of a decoder layer.  Sec. 3.3 starts from
 * one kernel per linear layer; fusing the launches removes the fixed cost a short
 * kernel cannot amortise.  w: array of `count` views; x, y: arrays of `count` device
 * pointers (host arrays of device pointers).  Results equal those of `count` separate
 * egt_sparse_gemv / egt_int4_gemv calls bit for bit. */
egt_status egt_sparse_gemv_batch(const egt_2bitcsr *w, const uint16_t *const *x, uint16_t *const *y,
                                 int count, void *stream);
egt_status egt_int4_gemv_batch(const uint8_t *const *q, const uint16_t *const *qparams, int rows,
                               int cols, int group, const uint16_t *const *x, uint16_t *const *y,
                               int count, void *stream);

/* DEVICE.  The same for 1 <= M <= 64 activation rows (Sec. 3.4: all candidates of a trie level
 * pass the q/k/v or the gate/up projections together): Y[k] = X[k] . W[k]^T for `count` (1..4)
 * identically shaped matrices in one launch.  X, Y: host arrays of `count` device pointers
 * (the members may share one X); every X[k] has leading dimension ldx, every Y[k] ldy; the
 * other arguments are those of egt_sparse_gemm_smallm.  Where no batched kernel takes the
 * shape or M (one to four tokens at K = 4096, the paired nibble order, shapes of the
 * slot-by-slot kernel) the members run as one launch each.  Results equal those of `count`
 * separate egt_sparse_gemm_smallm calls bit for bit. */
egt_status egt_sparse_gemm_smallm_batch(const egt_2bitcsr *w, const uint16_t *const *X, int64_t ldx,
                                        uint16_t *const *Y, int64_t ldy, int M, int count, void *stream);

/* Several products of different shapes and storage forms in one launch (Sec. 3.3 starts
 * from one kernel per linear layer; Sec. 3.2 makes the stack a layer-adaptive mix of 2:4,
 * 1:4 and dense INT4 layers): the fixed cost of a launch, about half the time of a GEMV of
 * a few megabytes, is paid once per table instead of once per matrix.
 *
 * An item is one product y = W.x.  `sparse` != NULL: W is that 2bit-CSR view (INT4 values,
 * n_keep 2 with group_size >= 64 or n_keep 1 with group_size >= 128; device buffers); the
 * fields q .. group are ignored.  `sparse` == NULL: W is dense INT4 (q, qparams, rows, cols,
 * group as for egt_int4_gemv, group >= 128).  x: cols FP16, y: rows FP16, device pointers.
 * Shapes outside those of the matrix-core kernels give EGT_ERR_UNSUPPORTED. */
typedef struct {
  const egt_2bitcsr *sparse;
  const uint8_t *q;
  const uint16_t *qparams;
  int32_t rows, cols, group;
  const uint16_t *x;
  uint16_t *y;
} egt_gemv_item;

#define EGT_STACK_ENTRY_BYTES 160 /* bytes of one descriptor in the table */
enum { EGT_STACK_AUTO = 0, EGT_STACK_GRID = 1, EGT_STACK_RESIDENT = 2 };

/* One launch of a planned table.  A table whose matrices all run well in one kernel is one
 * part.  A table that holds 1:4 matrices beside others is two: the 1:4 kernel body needs
 * twice the registers of the others, and a kernel that carries every body runs every
 * matrix at the occupancy of the widest one (the three-way mix of a 7B stack: 783 us in
 * one kernel, 480 us in two).  The parts' tables follow each other in the table. */
typedef struct {
  int32_t count;         /* matrices of the part                                             */
  int32_t mode;          /* 0: one grid of short-lived workgroups per matrix;
                            1: resident workgroups that walk a list of row blocks            */
  int32_t grid_x;        /* mode 0: workgroups of the largest matrix; mode 1: workgroups     */
  int32_t block_threads; /* threads per workgroup (a multiple of 64)                         */
  int32_t lds_bytes;     /* dynamic LDS per workgroup                                        */
  int32_t x_pieces;      /* 16-byte pieces of x a thread stages: 2, 4 or 8                   */
  int32_t forms;         /* storage forms in the table: bit 0 2:4, bit 1 1:4, bit 2 dense    */
  int32_t nitems;        /* mode 1: row blocks in the list                                   */
  int32_t part_offset;   /* mode 1: LDS offset of the partial sums                           */
  int32_t reserved;
  uint64_t table_bytes;  /* bytes of the part's table                                        */
} egt_stack_part;

#define EGT_STACK_MAX_PARTS 2
typedef struct {
  int32_t count;         /* matrices in the table                                            */
  int32_t nparts;        /* launches                                                         */
  egt_stack_part part[EGT_STACK_MAX_PARTS];
  uint64_t table_bytes;  /* bytes of the whole table                                         */
} egt_stack_plan;

/* HOST.  Checks `count` (1..65535) items, chooses the launch form and writes the launch
 * shape to *plan.  With table == NULL that is all (a size query: plan->table_bytes says how
 * large the table is); otherwise the table - the matrix descriptors, EGT_STACK_ENTRY_BYTES
 * each, followed in mode 1 by the list of row blocks - is written to `table`, HOST memory
 * of the caller with room for `table_bytes` >= plan->table_bytes bytes (else EGT_ERR_SHAPE).
 * The caller copies the table to 16-byte aligned device memory it owns (the library
 * allocates nothing) and may run it any number of times.  Nothing is written when an
 * error is returned.  Items with rows == 0 are legal and compute nothing.
 * `form`: EGT_STACK_AUTO picks mode 1 for tables of 2:4 and dense INT4 matrices with at
 * least 2048 (dense) or 4096 (2:4) columns that hold 32 MB or more (below that a workgroup
 * would see too few rows to make walking a list pay) and mode 0 otherwise; EGT_STACK_GRID
 * and EGT_STACK_RESIDENT ask for mode 0 or mode 1 (EGT_ERR_UNSUPPORTED if the shapes do not
 * allow mode 1).  Mode 1 sizes the launch for the 256 compute units of an MI355X.  The
 * form is chosen per part (with EGT_STACK_RESIDENT every part has to allow mode 1); 1:4
 * matrices take mode 1 with 2048, 4096 or 8192 to 16384 columns and groups of 128 and more. */
egt_status egt_gemv_stack_plan(const egt_gemv_item *items, int count, int form, void *table,
                               size_t table_bytes, egt_stack_plan *plan);

/* DEVICE.  Runs every product of a planned table, one launch per part, on `stream`.  table_dev:
 * the device copy of the table egt_gemv_stack_plan wrote; it and every buffer it names
 * must stay valid until the launch has completed.  The products are independent: no y may
 * alias an x or another y of the same table.  Each y[r] is computed by the same code as
 * in egt_sparse_gemv / egt_int4_gemv (a broken row_ptr entry gives NaN in that row). */
egt_status egt_gemv_stack_run(const void *table_dev, const egt_stack_plan *plan, void *stream);

/* A verification step through a stack of layers (Sec. 3.4 "Parallel Verification Trigger":
 * one step checks M candidate tokens against every layer): any number of small-M products
 * Y_k = X_k . W_k^T of different shapes in one launch.  A single product has to spread one
 * matrix over the whole chip; a table of them lets every compute unit work on several
 * matrices at once with small workgroups, which more than halves the time per product
 * (and the fixed cost of a launch is paid once per table).  Items: W an INT4 2bit-CSR view
 * (device buffers), all of a table of one storage form - 2:4 with group_size >= 64 and cols
 * a multiple of 64, or (Sec. 3.2's sparser layers) 1:4 with group_size >= 128, cols a
 * multiple of 128 and at most 32 tokens; X: M x cols FP16 with the token rows back to back
 * (ldx = cols), Y: M x rows FP16 (ldy = rows), device pointers, X 16-byte aligned.  Other
 * shapes, and tables that mix the two forms, give EGT_ERR_UNSUPPORTED: a mix runs as one
 * table per form, anything else as single products. */
typedef struct {
  const egt_2bitcsr *sparse;
  const uint16_t *X;
  uint16_t *Y;
} egt_gemm_item;

typedef struct {
  int32_t count;         /* matrices in the table                                            */
  int32_t M;             /* tokens of every product (2..64)                                  */
  int32_t grid_x;        /* workgroups of the launch (0: every matrix is empty)              */
  int32_t block_threads; /* threads per workgroup                                            */
  int32_t lds_bytes;     /* dynamic LDS per workgroup                                        */
  int32_t n_keep;        /* storage form of every matrix of the table: 2 (2:4) or 1 (1:4)    */
  uint64_t table_bytes;  /* the descriptors and 4 bytes per workgroup, a multiple of 16      */
} egt_gemm_plan;

/* HOST.  As egt_gemv_stack_plan: checks `count` (1..65535) items for M tokens each, writes
 * the launch shape to *plan and, with table != NULL, one descriptor per item and the list
 * of the launch's workgroups to `table` (HOST memory of the caller, table_bytes >= plan->table_bytes, else EGT_ERR_SHAPE), which
 * the caller copies to 16-byte aligned device memory.  Items with rows == 0 compute
 * nothing.  Nothing is written when an error is returned. */
egt_status egt_gemm_stack_plan(const egt_gemm_item *items, int count, int M, void *table,
                               size_t table_bytes, egt_gemm_plan *plan);

/* DEVICE.  Runs every product of the table in one launch on `stream`.  The table and every
 * buffer it names stay valid until the launch has completed; no Y may alias an X or another
 * Y of the table.  Each Y[m][r] is the FP16 rounding of an FP32 sum of the same products as
 * in egt_sparse_gemm_smallm; the sum runs in another order (along the row from its first
 * column to its last), so the two may differ in the last bit.  The result
 * does not depend on the other items of the table or on the run.  A broken row_ptr entry
 * gives NaN in that row. */
egt_status egt_gemm_stack_run(const void *table_dev, const egt_gemm_plan *plan, void *stream);

/* HOST.  Cost model of the parallel-verification trigger (Sec. 3.4 "Parallel
 * Verification Trigger"): the paper observes that the cost of a verification step grows
 * linearly with the number of candidate tokens while an autoregressive step costs a
 * constant.  egt_fit_verify_cost fits t(M) ~ a + b*M by least squares to n >= 2 measured
 * points (m[i] >= 1, not all equal).  egt_trigger_depth returns in *best the depth d in
 * [0, depth) that maximises  remaining[d] * t_ar - (a + b * cand[d])  - the time of
 * generating the remaining tokens one by one minus the time of verifying cand[d]
 * candidates in one step - and that maximum in *benefit; *best = -1 and *benefit = 0 when
 * no depth has a positive benefit (never trigger).  Equal benefits: the smaller depth. */
egt_status egt_fit_verify_cost(const int *m, const double *t, int n, double *a, double *b);
egt_status egt_trigger_depth(double t_ar, double a, double b, const int *cand, const int *remaining,
                             int depth, int *best, double *benefit);

/* DEVICE.  Measurement aid: streams `bytes` (a multiple of 16) from `src` with
 * 128-bit loads and folds them into one 32-bit word per workgroup written to
 * `sink` (at least 4096 words).  Gives the read bandwidth a kernel of that size
 * can reach at all on the device; not part of the method. */
egt_status egt_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EGT_H */
