// M = 1 SparseGemv for 1:4 sparsity (the sparser of the two layer-adaptive settings
// of Sec. 3.2 "Sparsification") on the gfx950 sparse matrix cores.
//
// The matrix instruction wants two values per four dense columns; a 1:4 group has
// one.  Each slot therefore becomes the pair {value, 0} and its 2-bit offset is
// spread to the even index field of the pair (the odd field belongs to the zero and
// may hold anything).  Everything else follows the 2:4 kernel: a chunk is 32 slots
// = 16 B of nibbles + 8 B of index words, which now span 128 dense columns (exactly
// one quantisation group of 128); a tile is 64 consecutive chunks, lane (i, kb)
// owns chunk 4 i + kb, column n of B holds the activations of chunks 4 n .. 4 n + 3,
// and D[i][i] is the dot product of a quad (512 dense columns) with x.  Eight
// instructions (four slots each) finish a chunk.
#include "egt_n1_body.h"

#include "egt_tune.h"

namespace egt {

template <int KIND, int TPI, int XP, int QW, int NI>
__global__ __launch_bounds__(1024) void k_sparse_m1_n1(const uint32_t *__restrict__ row_ptr,
                                                        const uint8_t *__restrict__ values,
                                                        const uint8_t *__restrict__ idx,
                                                        const uint8_t *__restrict__ qparams,
                                                        const __half *__restrict__ x,
                                                        __half *__restrict__ y, const M1N1Geom g) {
  k_sparse_m1_n1_body<KIND, TPI, XP, QW, NI>(row_ptr, values, idx, qparams, x, y, g);
}

template <int KIND, int TPI, int XP, int QW, int NI>
__global__ __launch_bounds__(1024) void k_sparse_m1_n1_batch(const GemvBatch b, const M1N1Geom g) {
  k_sparse_m1_n1_body<KIND, TPI, XP, QW, NI>(pick4(b.row_ptr, blockIdx.y), pick4(b.values, blockIdx.y),
                                     pick4(b.idx, blockIdx.y), pick4(b.qparams, blockIdx.y),
                                     pick4(b.x, blockIdx.y), pick4(b.y, blockIdx.y), g);
}

// Shapes covered: 1:4; K = 2048 or 4096 (several rows per tile) or a multiple of 128
// from 8192 up to 4 tiles per row (four waves per phase stage x); INT4 groups of 32 << j.
bool sparse_m1_n1_supported(const egt_2bitcsr &w) {
  if (w.n_keep != 1) return false;
  const bool multirow = w.cols == 2048 || w.cols == 4096;
  if (!multirow && (w.cols < 8192 || w.cols % 128 != 0 || w.cols > 4 * 8192)) return false;
  if (w.val_kind == EGT_VAL_INT4) {
    const int gm = w.group_size / 32;
    if (w.group_size % 32 != 0 || (gm & (gm - 1)) != 0) return false;
  }
  return true;
}

hipError_t launch_sparse_m1_n1_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                                     int count, hipStream_t stream) {
  const egt_2bitcsr &w = ws[0];
  if (w.rows == 0 || count == 0) return hipSuccess;
  GemvBatch b = {};
  for (int k = 0; k < count; ++k) {
    b.row_ptr[k] = ws[k].row_ptr; b.values[k] = (const uint8_t *)ws[k].values;
    b.idx[k] = (const uint8_t *)ws[k].idx; b.qparams[k] = (const uint8_t *)ws[k].qparams;
    b.x[k] = (const __half *)xs[k]; b.y[k] = (__half *)ys[k];
  }
  M1N1Geom g;
  // FP16 values: one row per tile, contiguous-kilobyte loads (NI load instructions per tile)
  const bool lin = w.val_kind == EGT_VAL_FP16 && !tune_flag("EGT_M1N1_NOLIN");
  int ni;
  n1_geometry(w, lin, g, ni);
  int tpi = g.phases == 1 ? 2 : 4, wpp = 4;
  if (lin) tpi = ni == 4 ? 2 : 4;
  tune_pair("EGT_M1N1_TUNE", tpi, wpp);
  if (wpp < 1) wpp = 1;
  if (wpp * g.phases > 16) wpp = 16 / g.phases;
  if (tpi != 1 && tpi != 2 && tpi != 4) tpi = 2;
  if (w.val_kind == EGT_VAL_FP16 && tpi == 4 && ni != 1 && ni != 2) tpi = 2;   // 64 B of values per lane and tile
  if (lin && ni < 4) tpi = 4;
  if (lin && ni == 4) tpi = 2;
  if (w.val_kind == EGT_VAL_INT4 && w.group_size < 128) tpi = 2;
  LaunchShape ls;
  if (!n1_block_shape(g, lin, ni, wpp, tpi, 4, ls)) return hipErrorInvalidConfiguration;
  const dim3 grid(ls.nblocks, count), block(64 * ls.nwaves);
  const size_t lds = ls.lds;
  const int xp = ls.xp;
#define EGT_GO5(KIND, TPI, XP, QW, NI)                                                          \
  (count > 1 ? launch(k_sparse_m1_n1_batch<KIND, TPI, XP, QW, NI>, grid, block, lds, stream, b, g)  \
             : launch(k_sparse_m1_n1<KIND, TPI, XP, QW, NI>, grid, block, lds, stream, b.row_ptr[0], \
                      b.values[0], b.idx[0], b.qparams[0], b.x[0], b.y[0], g))
#define EGT_GO4(KIND, TPI, XP, QW) EGT_GO5(KIND, TPI, XP, QW, 0)
#define EGT_GO3(KIND, TPI, XP) EGT_GO4(KIND, TPI, XP, 1)
#define EGT_GO(KIND, TPI)                                                                       \
  (xp <= 1 ? EGT_GO3(KIND, TPI, 1) : xp == 2 ? EGT_GO3(KIND, TPI, 2) : EGT_GO3(KIND, TPI, 4))
#define EGT_GOL(TPI, NI)                                                                        \
  (xp <= 1 ? EGT_GO5(EGT_VAL_FP16, TPI, 1, 1, NI) : xp == 2 ? EGT_GO5(EGT_VAL_FP16, TPI, 2, 1, NI) \
                                                            : EGT_GO5(EGT_VAL_FP16, TPI, 4, 1, NI))
  if (lin) return ni == 1 ? EGT_GOL(4, 1) : ni == 2 ? EGT_GOL(4, 2) : EGT_GOL(2, 4);
  if (w.val_kind == EGT_VAL_INT4 && w.group_size < 128) {   // narrow groups: one launch shape each
    if (w.group_size == 64)
      return xp <= 1 ? EGT_GO4(EGT_VAL_INT4, 2, 1, 2) : xp == 2 ? EGT_GO4(EGT_VAL_INT4, 2, 2, 2)
                                                                : EGT_GO4(EGT_VAL_INT4, 2, 4, 2);
    return xp <= 1 ? EGT_GO4(EGT_VAL_INT4, 2, 1, 4) : xp == 2 ? EGT_GO4(EGT_VAL_INT4, 2, 2, 4)
                                                              : EGT_GO4(EGT_VAL_INT4, 2, 4, 4);
  }
  if (w.val_kind == EGT_VAL_INT4) {
    switch (tpi) {
      case 1: return EGT_GO(EGT_VAL_INT4, 1);
      case 4: return EGT_GO(EGT_VAL_INT4, 4);
      default: return EGT_GO(EGT_VAL_INT4, 2);
    }
  }
  switch (tpi) {
    case 1: return EGT_GO(EGT_VAL_FP16, 1);
    default: return EGT_GO(EGT_VAL_FP16, 2);
  }
#undef EGT_GO
#undef EGT_GO3
#undef EGT_GO4
#undef EGT_GO5
#undef EGT_GOL
}

hipError_t launch_sparse_m1_n1(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream) {
  return launch_sparse_m1_n1_batch(&w, &x, &y, 1, stream);
}

}  // namespace egt
