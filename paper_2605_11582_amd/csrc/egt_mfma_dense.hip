// Dense group-quantised INT4 GEMV (M = 1) on the gfx950 matrix cores.
//
// Same "diagonal" mapping as the sparse kernel, with v_mfma_f32_16x16x32_f16:
// a chunk is 32 dense columns = 16 B of nibbles, a tile is 64 consecutive chunks
// (2048 columns), lane (i, kb) = i + 16 kb owns chunk 4 i + kb, and column n of B
// carries the activations of chunks 4 n .. 4 n + 3.  B lane (n, kb) then holds the
// activations of its *own* chunk, and D[i][i] is the dot product of one quad
// = 128 dense columns = exactly one quantisation group (group size 128).
//
// Because a diagonal element covers one group, the scale and the zero point are
// applied after the matrix instruction: the nibbles go in as 64 + q (one byte
// permute and one and-or per pair, exact), and the kernel finishes a group as
//   s * ( sum (64 + q) x  -  (64 + z) * sum x ),
// where sum x over the group does not depend on the row: it is computed once per
// wave by the same instruction with an all-ones A operand.  Groups of 256, 512, ...
// columns work the same way (neighbouring quads share their parameters).
// Groups of 32 or 64 columns are narrower than a quad; there a lane's chunk lies in
// one group and the lane applies zero point and scale to its values before the
// matrix instruction (template parameter PRE), two more packed operations per pair.
#include "egt_dense_body.h"

#include "egt_tune.h"

namespace egt {

template <int TPI, int XP, bool PRE>
__global__ __launch_bounds__(1024) void k_int4_m1(const uint8_t *__restrict__ q,
                                                   const uint8_t *__restrict__ qparams,
                                                   const __half *__restrict__ x,
                                                   __half *__restrict__ y, const DenseGeom g) {
  k_int4_m1_body<TPI, XP, PRE>(q, qparams, x, y, g);
}

template <int TPI, int XP, bool PRE>
__global__ __launch_bounds__(1024) void k_int4_m1_batch(const GemvBatch b, const DenseGeom g) {
  k_int4_m1_body<TPI, XP, PRE>(pick4(b.values, blockIdx.y), pick4(b.qparams, blockIdx.y),
                          pick4(b.x, blockIdx.y), pick4(b.y, blockIdx.y), g);
}

// Shapes covered: group size 32 << j; K = 512 or 1024 (several rows per tile) or a
// multiple of 128 from 2048 up to 16 tiles per row.
bool int4_m1_supported(int cols, int group) {
  const int gm = group / 32;
  if (group % 32 != 0 || (gm & (gm - 1)) != 0 || cols % group != 0) return false;
  if (cols == 512 || cols == 1024) return true;
  return cols >= 2048 && cols % 128 == 0 && cols <= 16 * 2048;
}

hipError_t launch_int4_m1_batch(const uint8_t *const *qs, const uint16_t *const *qps, int rows, int cols,
                                int group, const uint16_t *const *xs, uint16_t *const *ys, int count,
                                hipStream_t stream) {
  if (rows == 0 || count == 0) return hipSuccess;
  GemvBatch b = {};
  for (int k = 0; k < count; ++k) {
    b.values[k] = qs[k]; b.qparams[k] = (const uint8_t *)qps[k];
    b.x[k] = (const __half *)xs[k]; b.y[k] = (__half *)ys[k];
  }
  DenseGeom g;
  bool pre;
  dense_geometry(rows, cols, group, g, pre);
  int tpi = 4, wpp = g.phases == 1 ? 4 : (g.phases <= 8 ? 2 : 1);   // measured; K = 11008 (6 phases): 7.65 us with 2, 8.24 with 1
  tune_pair("EGT_DENSE_TUNE", tpi, wpp);
  if (wpp < 1) wpp = 1;
  if (wpp * g.phases > 16) wpp = 16 / g.phases;
  if (tpi != 1 && tpi != 2 && tpi != 4 && tpi != 8) tpi = 4;
  LaunchShape ls;
  if (!dense_block_shape(g, wpp, tpi, 4, ls)) return hipErrorInvalidConfiguration;
  const dim3 grid(ls.nblocks, count), block(64 * ls.nwaves);
  const size_t lds = ls.lds;
  const int xp = ls.xp;
#define EGT_GO4(TPI, XP, PRE)                                                                    \
  (count > 1 ? launch(k_int4_m1_batch<TPI, XP, PRE>, grid, block, lds, stream, b, g)               \
             : launch(k_int4_m1<TPI, XP, PRE>, grid, block, lds, stream, b.values[0],             \
                      b.qparams[0], b.x[0], b.y[0], g))
#define EGT_GO3(TPI, XP) (pre ? EGT_GO4(TPI, XP, true) : EGT_GO4(TPI, XP, false))
#define EGT_GO(TPI) (xp <= 1 ? EGT_GO3(TPI, 1) : xp == 2 ? EGT_GO3(TPI, 2) : EGT_GO3(TPI, 4))
  switch (tpi) {
    case 1: return EGT_GO(1);
    case 2: return EGT_GO(2);
    case 8: return EGT_GO(8);
    default: return EGT_GO(4);
  }
#undef EGT_GO
#undef EGT_GO3
#undef EGT_GO4
}

hipError_t launch_int4_m1(const uint8_t *q, const uint16_t *qparams, int rows, int cols, int group,
                          const uint16_t *x, uint16_t *y, hipStream_t stream) {
  return launch_int4_m1_batch(&q, &qparams, rows, cols, group, &x, &y, 1, stream);
}

}  // namespace egt
