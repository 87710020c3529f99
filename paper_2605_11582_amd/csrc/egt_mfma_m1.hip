// M = 1 SparseGemv on the gfx950 sparse matrix cores.
//
// The 2:4 compressed operand of v_smfmac_f32_16x16x64_f16 is what 2bit-CSR
// stores: per 4 dense columns two FP16 values plus two 2-bit in-group offsets,
// eight offsets to a 16-bit word with the first one in the low bits.  A lane
// feeds the instruction 8 values (4 VGPRs) and one 16-bit half of an index
// register, so one uint16 idx word of the format is the index operand of one
// instruction as it stands; no index arithmetic is executed at all.
//
// Mapping ("diagonal" scheme).  Work is cut into chunks of 64 dense columns =
// 32 slots = 16 B of nibbles + 8 B of idx words.  A tile is 64 consecutive
// chunks, one per lane, so every load instruction of a wave reads one
// contiguous kilobyte.  The instruction computes D[i][n] = sum_k A[i][k] B[k][n]
// where lane (i, kb) = i + 16 kb supplies A[i][16 kb .. 16 kb + 15].  Lane
// (i, kb) is given chunk 4 i + kb of the tile, and column n of B is loaded with
// the activations of the dense columns of chunks 4 n .. 4 n + 3.  Then
// D[i][i] is the dot product of four consecutive chunks (a "quad", 256 dense
// columns) with x, and the other 240 outputs are ignored.  The matrix cores
// are otherwise idle in a GEMV, so the waste costs nothing, while the gather
// of x by runtime indices - the expensive part on vector ALUs - disappears.
// B depends only on the column position of the tile, so it is loaded once per
// wave and reused for every row the wave processes.
//
// Four instructions (one per dword of the lane's nibbles) finish a tile.
// Loads are never predicated: lanes or tiles that fall outside the matrix read a
// clamped (valid) address and their result is either multiplied by a zero of B
// or not stored.
#include "egt_m1_body.h"

#include "egt_tune.h"

namespace egt {

// One matrix per launch, one whole tile per row (K = 4096), INT4 values: the headline shape.
template <int TPI, int XP, int QW, bool PAIRED = false>
__global__ __launch_bounds__(1024) void k_sparse_m1_one(const uint32_t *__restrict__ row_ptr,
                                                         const uint8_t *__restrict__ values,
                                                         const uint8_t *__restrict__ idx,
                                                         const uint8_t *__restrict__ qparams,
                                                         const __half *__restrict__ x,
                                                         __half *__restrict__ y, const M1Geom g) {
  // Workgroups [0, hi_blocks) take TPI tiles per wave, the rest TPI - 1: the launcher picks a
  // workgroup count that is a multiple of the compute units and spreads the rows evenly
  // (11008 rows in workgroups of 16 are 688 workgroups, 2.7 per compute unit: some units
  // would get three, some two, and the kernel ends with the slowest).
  const int nw = blockDim.x >> 6;
  if constexpr (TPI > 1) {
    if ((int)blockIdx.x >= g.hi_blocks) {
      k_sparse_m1_body<EGT_VAL_INT4, TPI - 1, XP, QW, false, 1, true, PAIRED>(
          row_ptr, values, idx, qparams, x, y, g, (g.hi_blocks * TPI + ((int)blockIdx.x - g.hi_blocks) * (TPI - 1)) * nw);
      return;
    }
  }
  k_sparse_m1_body<EGT_VAL_INT4, TPI, XP, QW, false, 1, true, PAIRED>(row_ptr, values, idx, qparams, x, y, g,
                                                                      (int)blockIdx.x * nw * TPI);
}

// One matrix per launch: the pointers are plain kernel arguments.
template <int KIND, int TPI, int XP, int QW, bool LIN, bool PAIRED = false>
__global__ __launch_bounds__(1024) void k_sparse_m1(const uint32_t *__restrict__ row_ptr,
                                                     const uint8_t *__restrict__ values,
                                                     const uint8_t *__restrict__ idx,
                                                     const uint8_t *__restrict__ qparams,
                                                     const __half *__restrict__ x,
                                                     __half *__restrict__ y, const M1Geom g) {
  k_sparse_m1_body<KIND, TPI, XP, QW, LIN, 1, false, PAIRED>(row_ptr, values, idx, qparams, x, y, g);
}

// Several tokens (2 <= M <= MT), one matrix.
template <int KIND, int TPI, int XP, int MT>
__global__ __launch_bounds__((MT > 2 || KIND == EGT_VAL_FP16) ? 512 : 1024) void k_sparse_m1_tokens(const uint32_t *__restrict__ row_ptr,
                                                                           const uint8_t *__restrict__ values,
                                                                           const uint8_t *__restrict__ idx,
                                                                           const uint8_t *__restrict__ qparams,
                                                                           const __half *__restrict__ x,
                                                                           __half *__restrict__ y, const M1Geom g) {
  k_sparse_m1_body<KIND, TPI, XP, 1, KIND == EGT_VAL_FP16, MT>(row_ptr, values, idx, qparams, x, y, g);
}

// Several identically shaped matrices per launch, selected by blockIdx.y.
template <int KIND, int TPI, int XP, int QW, bool LIN>
__global__ __launch_bounds__(1024) void k_sparse_m1_batch(const GemvBatch b, const M1Geom g) {
  k_sparse_m1_body<KIND, TPI, XP, QW, LIN, 1>(pick4(b.row_ptr, blockIdx.y), pick4(b.values, blockIdx.y),
                                  pick4(b.idx, blockIdx.y), pick4(b.qparams, blockIdx.y),
                                  pick4(b.x, blockIdx.y), pick4(b.y, blockIdx.y), g);
}

// Shapes the diagonal kernel covers: 2:4; K = 1024 or 2048 (several rows per tile)
// or a multiple of 64 from 4096 up to 8 tiles per row (more would not leave two waves per
// phase in a 16-wave workgroup to stage x in four pieces per thread); INT4 groups of 32 << j.
bool sparse_m1_supported(const egt_2bitcsr &w) {
  if (w.n_keep != 2) return false;
  const bool multirow = w.cols == 1024 || w.cols == 2048;
  if (!multirow && (w.cols < 4096 || w.cols % 64 != 0 || w.cols > 8 * 4096)) return false;
  if (w.val_kind == EGT_VAL_INT4) {
    const int gm = w.group_size / 32;
    if (w.group_size % 32 != 0 || (gm & (gm - 1)) != 0) return false;
  }
  return true;
}

hipError_t launch_sparse_m1_batch(const egt_2bitcsr *ws, const uint16_t *const *xs, uint16_t *const *ys,
                                  int count, hipStream_t stream) {
  const egt_2bitcsr &w = ws[0];
  if (w.rows == 0 || count == 0) return hipSuccess;
  GemvBatch b = {};
  for (int k = 0; k < count; ++k) {
    b.row_ptr[k] = ws[k].row_ptr; b.values[k] = (const uint8_t *)ws[k].values;
    b.idx[k] = (const uint8_t *)ws[k].idx; b.qparams[k] = (const uint8_t *)ws[k].qparams;
    b.x[k] = (const __half *)xs[k]; b.y[k] = (__half *)ys[k];
  }
  M1Geom g;
  m1_geometry(w, g);
  const bool multirow = g.mr_shift >= 0;
  const bool g32 = w.val_kind == EGT_VAL_INT4 && w.group_size == 32;
  // tuning knobs: tiles per wave, waves per phase per block
  // measured optima: 4 tiles per wave and 4 waves per phase for one phase, 2 waves per phase
  // for several - except three phases (K = 11008: 6.97 against 7.30 us with 2 and 4)
  int tpi = g.phases == 3 ? 2 : 4, wpp = (g.phases == 1 || g.phases == 3) ? 4 : 2;
  tune_pair("EGT_M1_TUNE", tpi, wpp);
  if (wpp < 1) wpp = 1;
  if (wpp * g.phases > 16) wpp = 16 / g.phases;
  if (tpi != 1 && tpi != 2 && tpi != 4 && tpi != 8) tpi = 4;
  if (w.val_kind == EGT_VAL_FP16 && tpi == 8) tpi = 4;
  if (g32) tpi = 4;
  const bool lin = w.val_kind == EGT_VAL_FP16 && !multirow && !tune_flag("EGT_M1_NOLIN");
  LaunchShape ls;
  if (!m1_block_shape(g, lin, wpp, tpi, 1, 4, ls)) {
    // (a developer build's knobs may ask for a workgroup too small to stage x: the shipped shape then)
    tpi = (g.phases == 3 || g32) ? (g32 ? 4 : 2) : 4;
    wpp = (g.phases == 1 || g.phases == 3) ? 4 : 2;
    if (wpp * g.phases > 16) wpp = 16 / g.phases;
    if (!m1_block_shape(g, lin, wpp, tpi, 1, 4, ls)) return hipErrorInvalidConfiguration;
  }
  const dim3 grid(ls.nblocks, count), block(64 * ls.nwaves);
  const size_t lds = ls.lds;
  const int xp = ls.xp;
#define EGT_GO5(KIND, TPI, XP, QW, LIN)                                                         \
  (count > 1 ? launch(k_sparse_m1_batch<KIND, TPI, XP, QW, LIN>, grid, block, lds, stream, b, g)    \
             : launch(k_sparse_m1<KIND, TPI, XP, QW, LIN>, grid, block, lds, stream, b.row_ptr[0], \
                      b.values[0], b.idx[0], b.qparams[0], b.x[0], b.y[0], g))
#define EGT_GO4(KIND, TPI, XP, QW) EGT_GO5(KIND, TPI, XP, QW, false)
#define EGT_GO3(KIND, TPI, XP) EGT_GO4(KIND, TPI, XP, 1)
#define EGT_GOL(TPI) (xp <= 1 ? EGT_GO5(EGT_VAL_FP16, TPI, 1, 1, true) : xp == 2 ? EGT_GO5(EGT_VAL_FP16, TPI, 2, 1, true) \
                                                                                  : EGT_GO5(EGT_VAL_FP16, TPI, 4, 1, true))
#define EGT_GO(KIND, TPI)                                                                       \
  (xp <= 1 ? EGT_GO3(KIND, TPI, 1) : xp == 2 ? EGT_GO3(KIND, TPI, 2) : EGT_GO3(KIND, TPI, 4))
  if (count == 1 && w.val_kind == EGT_VAL_INT4 && !g32 && g.nchunks == 64 && !tune_flag("EGT_M1_NOONE")) {
    // an even spread over the compute units while all workgroups are resident at once: the
    // smallest multiple of 256 workgroups that covers the rows at tpi tiles per wave, a part
    // of them with one tile less
    int nb = ls.nblocks;
    g.hi_blocks = nb;
    const int per_hi = ls.nwaves * tpi, per_lo = ls.nwaves * (tpi - 1);
    const int even = 256 * ((g.ntiles + 256 * per_hi - 1) / (256 * per_hi));
    if (tpi > 1 && even <= 1024 && even * per_lo < g.ntiles && !tune_flag("EGT_M1_NOEVEN")) {
      nb = even;
      g.hi_blocks = (g.ntiles - nb * per_lo + ls.nwaves - 1) / ls.nwaves;
    }
    const dim3 grid(nb);
#define EGT_ONE(TPI, XP)                                                                        \
  launch(k_sparse_m1_one<TPI, XP, 1>, grid, block, lds, stream, b.row_ptr[0], b.values[0], b.idx[0], b.qparams[0], \
         b.x[0], b.y[0], g)
    if (xp <= 2) {                                     // (at least four waves: x in one or two pieces per thread)
      switch (tpi) {
        case 1: return xp <= 1 ? EGT_ONE(1, 1) : EGT_ONE(1, 2);
        case 2: return xp <= 1 ? EGT_ONE(2, 1) : EGT_ONE(2, 2);
        case 8: return xp <= 1 ? EGT_ONE(8, 1) : EGT_ONE(8, 2);
        default: return xp <= 1 ? EGT_ONE(4, 1) : EGT_ONE(4, 2);
      }
    }
#undef EGT_ONE
  }
  if (g32)                                             // groups of 32: one launch shape
    return xp <= 1 ? EGT_GO4(EGT_VAL_INT4, 4, 1, 2) : xp == 2 ? EGT_GO4(EGT_VAL_INT4, 4, 2, 2)
                                                              : EGT_GO4(EGT_VAL_INT4, 4, 4, 2);
  if (w.val_kind == EGT_VAL_INT4) {
    switch (tpi) {
      case 1: return EGT_GO(EGT_VAL_INT4, 1);
      case 2: return EGT_GO(EGT_VAL_INT4, 2);
      case 8: return EGT_GO(EGT_VAL_INT4, 8);
      default: return EGT_GO(EGT_VAL_INT4, 4);
    }
  }
  if (lin) {
    switch (tpi) {
      case 1: return EGT_GOL(1);
      case 2: return EGT_GOL(2);
      default: return EGT_GOL(4);
    }
  }
  switch (tpi) {
    case 1: return EGT_GO(EGT_VAL_FP16, 1);
    case 2: return EGT_GO(EGT_VAL_FP16, 2);
    default: return EGT_GO(EGT_VAL_FP16, 4);
  }
#undef EGT_GO
#undef EGT_GO3
#undef EGT_GO4
#undef EGT_GO5
#undef EGT_GOL
}

// The paired nibble order (EGT_VAL_INT4_PAIRED): the shapes of sparse_m1_supported with one
// {scale, zero} pair per chunk, at the default tiles per wave.
bool sparse_m1_paired_supported(const egt_2bitcsr &w) {
  if (w.val_kind != EGT_VAL_INT4_PAIRED || w.group_size < 64) return false;
  egt_2bitcsr c = w;
  c.val_kind = EGT_VAL_INT4;
  return sparse_m1_supported(c);
}

hipError_t launch_sparse_m1_paired(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  egt_2bitcsr c = w;
  c.val_kind = EGT_VAL_INT4;
  M1Geom g;
  m1_geometry(c, g);
  g.nib_mask = 0x000F000Fu; g.nib_magic = 0x64006400u; g.nib_magic2 = 0x54005400u;
  const int tpi = g.phases == 3 ? 2 : 4;
  int wpp = (g.phases == 1 || g.phases == 3) ? 4 : 2;
  if (wpp * g.phases > 16) wpp = 16 / g.phases;
  LaunchShape ls;
  if (!m1_block_shape(g, false, wpp, tpi, 1, 4, ls)) return hipErrorInvalidConfiguration;
  const dim3 block(64 * ls.nwaves);
#define EGT_ARGS w.row_ptr, (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams, (const __half *)x, (__half *)y, g
  if (g.nchunks == 64 && ls.xp <= 2) {                 // one tile per row: rows spread evenly, see launch_sparse_m1_batch
    int nb = ls.nblocks;
    g.hi_blocks = nb;
    const int per_hi = ls.nwaves * tpi, per_lo = ls.nwaves * (tpi - 1);
    const int even = 256 * ((g.ntiles + 256 * per_hi - 1) / (256 * per_hi));
    if (even <= 1024 && even * per_lo < g.ntiles) {
      nb = even;
      g.hi_blocks = (g.ntiles - nb * per_lo + ls.nwaves - 1) / ls.nwaves;
    }
    return ls.xp <= 1 ? launch(k_sparse_m1_one<4, 1, 1, true>, dim3(nb), block, ls.lds, stream, EGT_ARGS)
                      : launch(k_sparse_m1_one<4, 2, 1, true>, dim3(nb), block, ls.lds, stream, EGT_ARGS);
  }
  const dim3 grid(ls.nblocks);
#define EGT_P(TPI) (ls.xp <= 1 ? launch(k_sparse_m1<EGT_VAL_INT4, TPI, 1, 1, false, true>, grid, block, ls.lds, stream, EGT_ARGS) \
                    : ls.xp == 2 ? launch(k_sparse_m1<EGT_VAL_INT4, TPI, 2, 1, false, true>, grid, block, ls.lds, stream, EGT_ARGS) \
                                 : launch(k_sparse_m1<EGT_VAL_INT4, TPI, 4, 1, false, true>, grid, block, ls.lds, stream, EGT_ARGS))
  return tpi == 2 ? EGT_P(2) : EGT_P(4);
#undef EGT_P
#undef EGT_ARGS
}

// Several-token form: 2:4, M = 2..4, INT4 values (groups of 64 << j) or FP16 values.  Used
// where it is the faster one: a row is one tile (K = 4096; with more tiles per row the
// K-split kernel wins, except for two tokens with FP16 values), and for three or four tokens
// with INT4 values (about 220 registers, two waves per SIMD) all workgroups must be resident
// at once (at most 8192 rows).
bool sparse_m1_tokens_supported(const egt_2bitcsr &w, int M) {
  if (M < 2 || M > 4 || w.n_keep != 2) return false;
  // FP16 values, two tokens: also up to four tiles per row (12.3 against 14.0 us on
  // 4096 x 11008, 8.7 against 11.0 us on 4096 x 8192)
  if (w.val_kind == EGT_VAL_FP16 && M == 2 && w.cols % 64 == 0 && w.cols > 4096 && w.cols <= 16384) return true;
  // INT4 values, two tokens, two tiles per row (K up to 8192: 6.3 against 7.4 us on 4096 x 8192,
  // 26.4 against 28.1 us on 28672 x 8192; with three tiles per row the K-split kernel is faster)
  const bool two_tiles = w.val_kind == EGT_VAL_INT4 && M == 2 && w.cols % 64 == 0 && w.cols > 4096 && w.cols <= 8192;
  if (w.cols != 4096 && !two_tiles) return false;
  if (w.val_kind == EGT_VAL_FP16) return true;
  if (M > 2 && w.rows > 8192) return false;
  const int gm = w.group_size / 64;
  return w.group_size % 64 == 0 && (gm & (gm - 1)) == 0;
}

hipError_t launch_sparse_m1_tokens(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                   int64_t ldy, int M, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  M1Geom g;
  m1_geometry(w, g);
  const bool f16 = w.val_kind == EGT_VAL_FP16;
  g.M = M; g.ldx = ldx; g.ldy = ldy;
  const int mt = M == 2 ? 2 : 4;
  // four tokens take about 200 registers: two waves per SIMD, workgroups of at most 8 waves;
  // FP16 values (64 B per lane and tile): two tiles per wave
  int tpi = (f16 && g.phases < 3) ? 2 : 4, wpp = g.phases == 1 ? 4 : 2;
  tune_pair("EGT_M1T_TUNE", tpi, wpp);
  if (f16 && mt == 4) tpi = 2;                        // the only four-token form with FP16 values
  if (wpp < 1) wpp = 1;
  const int max_waves = (mt > 2 || f16) ? 8 : 16;
  if (wpp * g.phases > max_waves) wpp = max_waves / g.phases;
  if (wpp < 1) return hipErrorInvalidConfiguration;
  if (tpi != 2 && tpi != 4) tpi = f16 ? 2 : 4;
  LaunchShape ls;
  if (!m1_block_shape(g, f16, wpp, tpi, mt, 4, ls)) return hipErrorInvalidConfiguration;
  const dim3 grid(ls.nblocks), block(64 * ls.nwaves);
  const size_t lds = ls.lds;
  const int xp = ls.xp;
#define EGT_T3(KIND, TPI, XP, MT)                                                               \
  launch(k_sparse_m1_tokens<KIND, TPI, XP, MT>, grid, block, lds, stream, w.row_ptr, (const uint8_t *)w.values, \
         (const uint8_t *)w.idx, (const uint8_t *)w.qparams, (const __half *)X, (__half *)Y, g)
#define EGT_T2(KIND, TPI, MT) (xp <= 1 ? EGT_T3(KIND, TPI, 1, MT) : xp == 2 ? EGT_T3(KIND, TPI, 2, MT) : EGT_T3(KIND, TPI, 4, MT))
  if (f16 && mt == 4) return EGT_T2(EGT_VAL_FP16, 2, 4);
  if (f16) return tpi == 2 ? EGT_T2(EGT_VAL_FP16, 2, 2) : EGT_T2(EGT_VAL_FP16, 4, 2);
  if (mt == 2) return tpi == 2 ? EGT_T2(EGT_VAL_INT4, 2, 2) : EGT_T2(EGT_VAL_INT4, 4, 2);
  return tpi == 2 ? EGT_T2(EGT_VAL_INT4, 2, 4) : EGT_T2(EGT_VAL_INT4, 4, 4);
#undef EGT_T2
#undef EGT_T3
}

hipError_t launch_sparse_m1(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream) {
  return launch_sparse_m1_batch(&w, &x, &y, 1, stream);
}

}  // namespace egt
