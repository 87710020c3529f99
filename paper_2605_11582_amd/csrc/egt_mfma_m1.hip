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
#include "egt_mfma_common.h"

#include "egt_tune.h"

namespace egt {

// Eight INT4 codes of one dword (slot k in bits 4k..4k+3) -> four half2 registers
// {slot 2p, slot 2p+1} holding s*(q - z).  Byte p of the dword carries the pair:
// the low nibble becomes the mantissa of 1024 + q, the high nibble (left in
// place) the mantissa of 64 + q; one packed subtract removes both offsets and z
// exactly, one packed multiply applies the scale (a single rounding to FP16).
__device__ __forceinline__ u4 dequant8(uint32_t d, uint32_t off, uint32_t s2, uint32_t mask, uint32_t magic) {
  u4 r;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t t = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)p * 0x00010001u);
    r[p] = pk_mul_f16(pk_sub_f16(and_or(t, mask, magic), off), s2);
  }
  return r;
}

// Geometry of a launch, computed on the host.
struct M1Geom {
  int rows;
  int nchunks;         // cols / 64
  int ntiles;          // tiles per phase = ceil(rows / rows_per_tile)
  int phases;          // tiles per row (row-tile mode), else 1
  int mr_shift;        // multi-row mode: log2(nchunks) (nchunks = 16 or 32); -1 in row-tile mode
  int gshift;          // INT4 group = 64 << gshift dense columns
  int groups_per_row;  // cols / group
  uint32_t last_chunk; // rows * nchunks - 1
  int part_offset;     // byte offset of the per-phase partial sums in LDS
  int xtok;            // LDS bytes of the staged activations of one token
  int M;               // tokens (activation rows): 1, or up to MT in the several-token form
  int64_t ldx, ldy;    // row strides of X and Y in elements (several-token form)
  uint32_t nib_mask;   // 0x00F0000F: low nibble of the low half, high nibble of the high half
  uint32_t nib_magic;  // 0x54006400: FP16 {1024.0, 64.0}
};

// One wave = TPI tiles, all loaded before the first is consumed.
// XP = 16 B pieces of x each thread stages (ceil(pieces / block size)).
// QW = {scale, zero} pairs per chunk: 1 for groups of 64 columns and more, 2 for groups
// of 32 (dwords 0, 1 of a chunk then belong to the first group, 2, 3 to the second).
// LIN (FP16 values, one row per tile): every load instruction of a wave reads one
// contiguous kilobyte of values - instruction k takes the 16-byte piece 64 k + lane of the
// tile (8 slots = 16 dense columns = one idx word) - instead of each lane reading its own
// chunk of 64 B.  Lane (i, kb) then multiplies pieces i + 16 kb + 64 k, k = 0..3, and
// column n of B carries the activations of the pieces n + 16 kb + 64 k.
// MT > 1: the several-token form (2 <= M <= MT activation rows).  The dequantised A
// registers of a tile feed MT instructions, one per token, each with the B operand of
// its own token (32 registers per token, loaded once per wave); everything about the
// weights - the loads, the dequantisation - is done once, as for one token.
template <int KIND, int TPI, int XP, int QW, bool LIN, int MT>
__device__ __forceinline__ void k_sparse_m1_body(const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
    const uint8_t *__restrict__ idx, const uint8_t *__restrict__ qparams, const __half *__restrict__ x,
    __half *__restrict__ y, const M1Geom &g) {
  extern __shared__ __align__(16) uint8_t xs[];       // staged x, then [phases][rows of this block] floats
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = blockDim.x >> 6;
  const int wpp = nwaves / g.phases;                  // waves per phase in this block
  float *part = (float *)(xs + g.part_offset);
  const int phase = wave / wpp;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;                         // chunk of this lane inside a tile
  const bool multirow = g.mr_shift >= 0;
  const int rpt = multirow ? (64 >> g.mr_shift) : 1;  // rows per tile
  const int c = multirow ? (cit & (g.nchunks - 1)) : cit + 64 * phase;   // chunk inside the row
  const int rsub = multirow ? (cit >> g.mr_shift) : 0;
  const int c_ld = min(c, g.nchunks - 1);

  // ---- x: the block's threads fetch it once, 16 B pieces, before anything else is
  //      requested, so that it is the first data to come back
  const int npieces = g.nchunks * 8;                   // 8 halfs per piece
  const int lds_pieces = multirow ? npieces : g.phases * 512;
  u4 xp[MT][XP];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const __half *xm = MT == 1 ? x : x + (int64_t)min(m, g.M - 1) * g.ldx;   // a token past M repeats the last one
#pragma unroll
    for (int j = 0; j < XP; ++j) {
      const int pi = threadIdx.x + j * blockDim.x;
      xp[m][j] = *(const u4 *)(xm + 8 * min(pi, npieces - 1));
    }
  }

  constexpr int XSH = LIN ? 4 : 5;                    // x in LDS: one 16 B pad per 2^XSH pieces
  const int tile0 = (blockIdx.x * wpp + wslot) * TPI;
  // The lanes that will store read their row pointers before the tiles are requested (loads
  // return in order, so the small ones go first and never make the wave wait for a tile):
  // lane j < 16 finishes tile (j >> 2) of each batch of four tiles.
  const int sum_steps = multirow ? (g.mr_shift - 4) : 2;       // log2(quad groups per row)
  constexpr int NB = (TPI + 3) / 4;
  uint32_t rp[NB];
  int rrow[NB];
  bool st[NB];
#pragma unroll
  for (int bt = 0; bt < NB; ++bt) {
    const int t = 4 * bt + ((lane >> 2) & 3);
    const int tr = tile0 + t;
    rrow[bt] = tr * rpt + ((lane & 3) >> sum_steps);
    st[bt] = lane < 16 && t < TPI && tr < g.ntiles && rrow[bt] < g.rows &&
             ((lane & 3) & ((1 << sum_steps) - 1)) == 0;
    rp[bt] = st[bt] ? row_ptr[rrow[bt]] : 0u;
  }

  // several tiles per row: the threads that add the phases up at the end fetch the row
  // pointer of their row now (wpp * TPI * MT <= 64 <= blockDim: one output per thread)
  uint32_t rp_fin = 0;
  if (g.phases > 1 && (int)threadIdx.x < wpp * TPI * MT) {
    const int r = blockIdx.x * (wpp * TPI) + (int)threadIdx.x / MT;
    if (r < g.rows) rp_fin = row_ptr[r];
  }

  // ---- issue every load of the wave's TPI tiles
  u4 nib[TPI][KIND == EGT_VAL_INT4 ? 1 : 4];
  u2 iw[TPI];
  uint32_t iwl[LIN ? TPI : 1][4];                     // LIN: the idx word of each piece
  uint32_t qp[TPI][QW];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    const int tr = min(tile0 + t, g.ntiles - 1);      // uniform
    if constexpr (LIN) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uint32_t piece = (uint32_t)min(256 * phase + 64 * k + lane, 4 * g.nchunks - 1);   // inside the row (clamped)
        const uint32_t gp = (uint32_t)tr * (uint32_t)(4 * g.nchunks) + piece;
        nib[t][k] = ld_stream<u4>(values + 16ull * gp);
        iwl[t][k] = ld_stream<uint16_t>(idx + 2ull * gp);
      }
      continue;
    }
    uint32_t chunk;
    if (multirow) chunk = min((uint32_t)tr * 64u + (uint32_t)cit, g.last_chunk);
    else chunk = (uint32_t)tr * (uint32_t)g.nchunks + (uint32_t)c_ld;
    iw[t] = ld_stream<u2>(idx + 8ull * chunk);
    qp[t][0] = 0;
    if (KIND == EGT_VAL_INT4) {
      nib[t][0] = ld_stream<u4>(values + 16ull * chunk);
      const int r = min(tr * rpt + rsub, g.rows - 1);
      if (QW == 2) {
        const u2 v = ld_stream<u2>(qparams + 4ull * ((uint32_t)r * (uint32_t)g.groups_per_row + 2u * (uint32_t)c_ld));
        qp[t][0] = v[0];
        qp[t][QW - 1] = v[1];
      } else {
        qp[t][0] = ld_stream<uint32_t>(qparams + 4ull * ((uint32_t)r * (uint32_t)g.groups_per_row + (uint32_t)(c_ld >> g.gshift)));
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) nib[t][k] = ld_stream<u4>(values + 64ull * chunk + 16 * k);
    }
  }
  // ---- x through LDS.  Piece p lives at byte 16 p + 16 (p >> 5): one 16 B pad after
  //      every 512 B, so that the 16-lane reads below, whose addresses are 512 B
  //      apart, fall into different banks.  Pieces past the end of x are zero.
#pragma unroll
  for (int m = 0; m < MT; ++m) {
#pragma unroll
    for (int j = 0; j < XP; ++j) {
      const int pi = threadIdx.x + j * blockDim.x;
      if (pi < lds_pieces) {
        u4 v = xp[m][j];
        if (pi >= npieces) v = u4{0, 0, 0, 0};
        *(u4 *)(xs + m * g.xtok + 16 * pi + 16 * (pi >> XSH)) = v;
      }
    }
  }
  __syncthreads();
  // B operand: column n = lane & 15 holds the activations of chunks 4n .. 4n+3;
  // lane (n, b) supplies k-octets b (first 8 halfs) and 4 + b (last 8 halfs)
  u8v bx[MT][4];
  if constexpr (LIN) {
    const int n = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = 2 * h + (b >> 1), sub = b & 1;  // the A lane (n, kba) this octet multiplies
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int pi = 2 * (256 * phase + 64 * k + n + 16 * kba) + sub;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const u4 v = *(const u4 *)(xs + m * g.xtok + 16 * pi + 16 * (pi >> XSH));
#pragma unroll
          for (int j = 0; j < 4; ++j) bx[m][k][4 * h + j] = v[j];
        }
      }
    }
  } else {
    const int n = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = (4 * h + b) >> 1, sub = b & 1;  // the A lane (n, kba) this octet multiplies
      int cb = 4 * n + kba;
      cb = multirow ? (cb & (g.nchunks - 1)) : cb + 64 * phase;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int pi = 8 * cb + 2 * d + sub;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
          const u4 v = *(const u4 *)(xs + m * g.xtok + 16 * pi + 16 * (pi >> 5));
#pragma unroll
          for (int k = 0; k < 4; ++k) bx[m][d][4 * h + k] = v[k];
        }
      }
    }
  }

  // ---- consume
  const uint32_t magic = in_vgpr(g.nib_magic);
  float s[TPI][MT];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    f4 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = f4{0.f, 0.f, 0.f, 0.f};
    uint32_t s2[QW], off[QW];
#pragma unroll
    for (int k = 0; k < QW; ++k) {
      s2[k] = off[k] = 0;
      if (KIND == EGT_VAL_INT4) {
        s2[k] = __builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x01000100u);                            // {s, s}
        off[k] = pk_add_f16(__builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x03020302u), g.nib_magic);  // {1024+z, 64+z}
      }
    }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      u4 a;
      if (KIND == EGT_VAL_INT4) a = dequant8(nib[t][0][d], off[d * QW / 4], s2[d * QW / 4], g.nib_mask, magic);
      else a = nib[t][d];
      if constexpr (LIN) {
#pragma unroll
        for (int m = 0; m < MT; ++m)
          acc[m] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[m][d]), acc[m], (int)iwl[t][d], 0, 0);
        continue;
      }
      const int iword = d < 2 ? (int)iw[t][0] : (int)iw[t][1];
#pragma unroll
      for (int m = 0; m < MT; ++m) {
        if (d & 1)
          acc[m] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[m][d]), acc[m], iword, 0, 1);
        else
          acc[m] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[m][d]), acc[m], iword, 0, 0);
      }
    }
    // D[q][q] sits in lane q + 16 (q / 4), register q % 4: lane 20 kb collects the
    // four diagonals of quads 4 kb .. 4 kb + 3 from its three right neighbours
#pragma unroll
    for (int m = 0; m < MT; ++m)
      s[t][m] = acc[m][0] + row_shl<1>(acc[m][1]) + row_shl<2>(acc[m][2]) + row_shl<3>(acc[m][3]);
  }
  // ---- lane j < 16 fetches tile (j >> 2), quad group (j & 3); then sum the groups of a row
  const int src_lane = 20 * (lane & 3);
#pragma unroll
  for (int m = 0; m < MT; ++m) {
#pragma unroll
    for (int bt = 0; bt < NB; ++bt) {
      float v = 0.f;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (4 * bt + k < TPI) {
          const float gk = __shfl(s[4 * bt + k][m], src_lane, 64);
          v = ((lane >> 2) & 3) == k ? gk : v;
        }
      }
      if (sum_steps >= 1) v += quad_xor1(v);
      if (sum_steps >= 2) v += quad_xor2(v);
      if (st[bt] && (MT == 1 || m < g.M)) {
        const int r = rrow[bt];
        if (g.phases == 1) {
          const bool ok = rp[bt] == (uint32_t)r * (uint32_t)(g.nchunks * 32);
          y[(int64_t)m * g.ldy + r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
        } else {
          part[(phase * (wpp * TPI) + wslot * TPI + 4 * bt + ((lane >> 2) & 3)) * MT + m] = v;
        }
      }
    }
  }
  if (g.phases > 1) {
    __syncthreads();
    const int per = wpp * TPI;                        // rows handled by this block
    const int j = threadIdx.x;
    if (j < per * MT) {
      const int jr = j / MT, m = j - jr * MT;
      const int r = blockIdx.x * per + jr;
      if (r < g.rows && (MT == 1 || m < g.M)) {
        float v = 0.f;
        for (int p = 0; p < g.phases; ++p) v += part[(p * per + jr) * MT + m];
        const bool ok = rp_fin == (uint32_t)r * (uint32_t)(g.nchunks * 32);
        y[(int64_t)m * g.ldy + r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
      }
    }
  }
}

// One matrix per launch: the pointers are plain kernel arguments.
template <int KIND, int TPI, int XP, int QW, bool LIN>
__global__ __launch_bounds__(1024) void k_sparse_m1(const uint32_t *__restrict__ row_ptr,
                                                     const uint8_t *__restrict__ values,
                                                     const uint8_t *__restrict__ idx,
                                                     const uint8_t *__restrict__ qparams,
                                                     const __half *__restrict__ x,
                                                     __half *__restrict__ y, const M1Geom g) {
  k_sparse_m1_body<KIND, TPI, XP, QW, LIN, 1>(row_ptr, values, idx, qparams, x, y, g);
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
  g.rows = w.rows;
  g.nchunks = w.cols / 64;
  const bool multirow = g.nchunks < 64;
  g.mr_shift = multirow ? (g.nchunks == 16 ? 4 : 5) : -1;
  const int rpt = multirow ? 64 / g.nchunks : 1;
  g.phases = multirow ? 1 : (g.nchunks + 63) / 64;
  g.ntiles = (w.rows + rpt - 1) / rpt;
  g.gshift = 0;
  g.groups_per_row = 0;
  const bool g32 = w.val_kind == EGT_VAL_INT4 && w.group_size == 32;
  if (w.val_kind == EGT_VAL_INT4) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.last_chunk = (uint32_t)w.rows * (uint32_t)g.nchunks - 1u;
  g.nib_mask = 0x00F0000Fu;
  g.nib_magic = 0x54006400u;
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
  const int nwaves = wpp * g.phases;
  const int tiles_per_block = wpp * tpi;
  const dim3 grid((g.ntiles + tiles_per_block - 1) / tiles_per_block, count), block(64 * nwaves);
  const int lds_pieces = multirow ? g.nchunks * 8 : g.phases * 512;
  const bool lin = w.val_kind == EGT_VAL_FP16 && !multirow && !tune_flag("EGT_M1_NOLIN");
  g.part_offset = lin ? 16 * lds_pieces + 16 * ((lds_pieces + 15) >> 4) : 16 * lds_pieces + 16 * ((lds_pieces + 31) >> 5);
  g.xtok = g.part_offset; g.M = 1; g.ldx = 0; g.ldy = 0;
  const size_t lds = g.part_offset + (g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block : 0);
  const int xp = (lds_pieces + 64 * nwaves - 1) / (64 * nwaves);
  if (xp > 4) return hipErrorInvalidConfiguration;
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
  g.rows = w.rows;
  g.nchunks = w.cols / 64;
  g.mr_shift = -1;
  g.phases = (g.nchunks + 63) / 64;
  g.ntiles = w.rows;
  const bool f16 = w.val_kind == EGT_VAL_FP16;
  g.gshift = 0; g.groups_per_row = 0;
  if (!f16) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.last_chunk = (uint32_t)w.rows * (uint32_t)g.nchunks - 1u;
  g.nib_mask = 0x00F0000Fu;
  g.nib_magic = 0x54006400u;
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
  const int nwaves = wpp * g.phases;
  const int tiles_per_block = wpp * tpi;
  const dim3 grid((g.ntiles + tiles_per_block - 1) / tiles_per_block), block(64 * nwaves);
  const int lds_pieces = g.phases * 512;
  // (x in LDS is padded once per 16 pieces for the contiguous-kilobyte form, else once per 32)
  g.xtok = f16 ? 16 * lds_pieces + 16 * ((lds_pieces + 15) >> 4) : 16 * lds_pieces + 16 * ((lds_pieces + 31) >> 5);
  g.part_offset = mt * g.xtok;
  const size_t lds = g.part_offset + (g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block * mt : 0);
  const int xp = (lds_pieces + 64 * nwaves - 1) / (64 * nwaves);
  if (xp > 4) return hipErrorInvalidConfiguration;
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
