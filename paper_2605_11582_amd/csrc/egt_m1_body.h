// Device body of the 2:4 M = 1 kernel (and its several-token form) with its launch
// geometry, shared by the single-matrix, batched and multi-matrix launchers.
#ifndef EGT_M1_BODY_H
#define EGT_M1_BODY_H

#include "egt_mfma_common.h"

// EGT_ABLATE (developer build, -DEGT_ABLATE=<bits>): stages of the 2:4 M = 1 kernel switched
// off for timing; the results are then wrong on purpose.  The loads, their order and the
// launch shape stay as they are, and every loaded register still reaches the stored value,
// so nothing that is timed can be optimised away.
//   bit 0: no dequantisation (the raw nibble dword goes to the instruction four times)
//   bit 1: no matrix instructions (the operands are folded into the sum with shifts, xors and
//          one add; the shifts keep equal registers from cancelling)
//   bit 2: no cross-lane reduction (each storing lane stores its own partial value)
//   bit 3: x is not staged through LDS (no LDS write, no barrier, B operand = the raw pieces)
#ifndef EGT_ABLATE
#define EGT_ABLATE 0
#endif

namespace egt {

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
  int wpp, wpp_inv;    // waves per phase in a workgroup, ceil(65536 / wpp)
  int hi_blocks;       // k_sparse_m1_one: workgroups [0, hi_blocks) take TPI tiles per wave, the others TPI - 1
  int64_t ldx, ldy;    // row strides of X and Y in elements (several-token form)
  uint32_t nib_mask;   // 0x00F0000F: low nibble of the low half, high nibble of the high half
  uint32_t nib_magic;  // 0x54006400: FP16 {1024.0, 64.0}
  // (paired nibble order: nib_mask 0x000F000F, nib_magic {1024.0, 1024.0}, nib_magic2 {64.0, 64.0})
  uint32_t nib_magic2;
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
// ONE: the matrix has exactly one whole tile per row (K = 4096) - the shape of most
// projections of a 7B decoder and of the headline workload; tiles per row, rows per tile
// and chunks per row are then constants and the index arithmetic of the general form
// (two integer divisions before the first request goes out) folds away.
// PAIRED: the INT4 codes are stored in the paired nibble order (EGT_VAL_INT4_PAIRED).
template <int KIND, int TPI, int XP, int QW, bool LIN, int MT, bool ONE = false, bool PAIRED = false>
__device__ __forceinline__ void k_sparse_m1_body(const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
    const uint8_t *__restrict__ idx, const uint8_t *__restrict__ qparams, const __half *__restrict__ x,
    __half *__restrict__ y, const M1Geom &g, int tile_base = -1) {
  extern __shared__ __align__(16) uint8_t xs[];       // staged x, then [phases][rows of this block] floats
  const int g_phases = ONE ? 1 : g.phases, g_mr_shift = ONE ? -1 : g.mr_shift, g_nchunks = ONE ? 64 : g.nchunks;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // waves per phase in this workgroup; (wave * wpp_inv) >> 16 = wave / wpp for wave < 16
  // (both from the host: integer divisions here would delay the first request)
  const int wpp = ONE ? (int)(blockDim.x >> 6) : g.wpp;
  float *part = (float *)(xs + g.part_offset);
  const int phase = ONE ? 0 : (wave * g.wpp_inv) >> 16;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;                         // chunk of this lane inside a tile
  const bool multirow = g_mr_shift >= 0;
  const int rpt = multirow ? (64 >> g_mr_shift) : 1;  // rows per tile
  const int c = multirow ? (cit & (g_nchunks - 1)) : cit + 64 * phase;   // chunk inside the row
  const int rsub = multirow ? (cit >> g_mr_shift) : 0;
  const int c_ld = min(c, g_nchunks - 1);

  // ---- x: the block's threads fetch it once, 16 B pieces, before anything else is
  //      requested, so that it is the first data to come back
  const int npieces = g_nchunks * 8;                   // 8 halfs per piece
  const int lds_pieces = multirow ? npieces : g_phases * 512;
  u4 xp[MT][XP];
#pragma unroll
  for (int m = 0; m < MT; ++m) {
    const __half *xm = MT == 1 ? x : x + (int64_t)min(m, g.M - 1) * g.ldx;   // a token past M repeats the last one
    x_request<XP>(xm, npieces, xp[m]);
  }

  constexpr int XSH = LIN ? 4 : 5;                    // x in LDS: one 16 B pad per 2^XSH pieces
  // first tile of this wave; tile_base >= 0: the caller says where the workgroup's tiles start
  // (workgroups of one launch may differ in their tiles per wave)
  const int tile0 = tile_base >= 0 ? tile_base + wslot * TPI : (blockIdx.x * wpp + wslot) * TPI;
  // The lanes that will store read their row pointers before the tiles are requested (loads
  // return in order, so the small ones go first and never make the wave wait for a tile):
  // lane j < 16 finishes tile (j >> 2) of each batch of four tiles.
  const int sum_steps = multirow ? (g_mr_shift - 4) : 2;       // log2(quad groups per row)
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
  if (g_phases > 1 && (int)threadIdx.x < wpp * TPI * MT) {
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
        const uint32_t piece = (uint32_t)min(256 * phase + 64 * k + lane, 4 * g_nchunks - 1);   // inside the row (clamped)
        const uint32_t gp = (uint32_t)tr * (uint32_t)(4 * g_nchunks) + piece;
        nib[t][k] = ld_stream<u4>(values + 16ull * gp);
        iwl[t][k] = ld_stream<uint16_t>(idx + 2ull * gp);
      }
      continue;
    }
    uint32_t chunk;
    if (multirow) chunk = min((uint32_t)tr * 64u + (uint32_t)cit, g.last_chunk);
    else chunk = (uint32_t)tr * (uint32_t)g_nchunks + (uint32_t)c_ld;
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
  if (!(EGT_ABLATE & 8)) {
#pragma unroll
    for (int m = 0; m < MT; ++m) x_store<XP, XSH>(xs + m * g.xtok, xp[m], npieces, lds_pieces);
    __syncthreads();
  }
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
      cb = multirow ? (cb & (g_nchunks - 1)) : cb + 64 * phase;
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

  if (EGT_ABLATE & 8) {
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
      for (int d = 0; d < 4; ++d)
#pragma unroll
        for (int j = 0; j < 8; ++j) bx[m][d][j] = xp[m][(d + j) % XP][j & 3];
  }

  // ---- consume
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t magic2 = PAIRED ? in_vgpr(g.nib_magic2) : 0u;
  float s[TPI][MT];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    f4 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = f4{0.f, 0.f, 0.f, 0.f};
    uint32_t s2[QW], off[QW], off2[QW];
#pragma unroll
    for (int k = 0; k < QW; ++k) {
      s2[k] = off[k] = off2[k] = 0;
      if (KIND == EGT_VAL_INT4) {
        s2[k] = __builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x01000100u);                            // {s, s}
        const uint32_t zz = __builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x03020302u);                // {z, z}
        off[k] = pk_add_f16(zz, g.nib_magic);          // {1024+z, 64+z}; paired order: {1024+z, 1024+z}
        if (PAIRED) off2[k] = pk_add_f16(zz, g.nib_magic2);                                         // {64+z, 64+z}
      }
    }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      u4 a;
      if (KIND == EGT_VAL_INT4) {
        if (EGT_ABLATE & 1) a = u4{nib[t][0][d], nib[t][0][d] ^ off[0], nib[t][0][d] ^ s2[0], nib[t][0][d]};
        else if (PAIRED) a = dequant8_paired(nib[t][0][d], off[d * QW / 4], off2[d * QW / 4], s2[d * QW / 4], g.nib_mask,
                                             g.nib_mask << 4, magic, magic2);
        else a = dequant8(nib[t][0][d], off[d * QW / 4], s2[d * QW / 4], g.nib_mask, magic);
      } else {
        a = nib[t][d];
      }
      if (EGT_ABLATE & 2) {
        const int iw_abl = LIN ? (int)iwl[t][d] : (d < 2 ? (int)iw[t][0] : (int)iw[t][1]);
#pragma unroll
        for (int m = 0; m < MT; ++m)
          acc[m][0] += __builtin_bit_cast(float, a[0] ^ (a[1] >> 1) ^ (a[2] << 1) ^ (a[3] >> 2) ^ bx[m][d][0] ^ (uint32_t)iw_abl);
        continue;
      }
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
    for (int m = 0; m < MT; ++m) {
      if (EGT_ABLATE & 4) s[t][m] = acc[m][0] + acc[m][1] + acc[m][2] + acc[m][3];
      else s[t][m] = acc[m][0] + row_shl<1>(acc[m][1]) + row_shl<2>(acc[m][2]) + row_shl<3>(acc[m][3]);
    }
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
          const float gk = (EGT_ABLATE & 4) ? s[4 * bt + k][m] : __shfl(s[4 * bt + k][m], src_lane, 64);
          v = ((lane >> 2) & 3) == k ? gk : v;
        }
      }
      if (!(EGT_ABLATE & 4)) {
        if (sum_steps >= 1) v += quad_xor1(v);
        if (sum_steps >= 2) v += quad_xor2(v);
      }
      if (st[bt] && (MT == 1 || m < g.M)) {
        const int r = rrow[bt];
        if (g_phases == 1) {
          const bool ok = rp[bt] == (uint32_t)r * (uint32_t)(g_nchunks * 32);
          y[(int64_t)m * g.ldy + r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
        } else {
          part[(phase * (wpp * TPI) + wslot * TPI + 4 * bt + ((lane >> 2) & 3)) * MT + m] = v;
        }
      }
    }
  }
  if (g_phases > 1) {
    __syncthreads();
    const int per = wpp * TPI;                        // rows handled by this block
    const int j = threadIdx.x;
    if (j < per * MT) {
      const int jr = j / MT, m = j - jr * MT;
      const int r = blockIdx.x * per + jr;
      if (r < g.rows && (MT == 1 || m < g.M)) {
        float v = 0.f;
        for (int p = 0; p < g_phases; ++p) v += part[(p * per + jr) * MT + m];
        const bool ok = rp_fin == (uint32_t)r * (uint32_t)(g_nchunks * 32);
        y[(int64_t)m * g.ldy + r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
      }
    }
  }
}

// Geometry of a 2:4 matrix for the diagonal kernel (everything that does not depend on the
// block shape).  `lin`: the contiguous-kilobyte form of FP16 values.
inline void m1_geometry(const egt_2bitcsr &w, M1Geom &g) {
  g.rows = w.rows;
  g.nchunks = w.cols / 64;
  const bool multirow = g.nchunks < 64;
  g.mr_shift = multirow ? (g.nchunks == 16 ? 4 : 5) : -1;
  const int rpt = multirow ? 64 / g.nchunks : 1;
  g.phases = multirow ? 1 : (g.nchunks + 63) / 64;
  g.ntiles = (w.rows + rpt - 1) / rpt;
  g.gshift = 0;
  g.groups_per_row = 0;
  if (w.val_kind == EGT_VAL_INT4) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.last_chunk = (uint32_t)w.rows * (uint32_t)g.nchunks - 1u;
  g.nib_mask = 0x00F0000Fu;
  g.nib_magic = 0x54006400u;
  g.nib_magic2 = 0;
  g.M = 1; g.ldx = 0; g.ldy = 0;
  g.hi_blocks = 0;
}

// Block shape for `wpp` waves per phase and `tpi` tiles per wave, `mt` tokens; fills the
// LDS offsets of the geometry.  False when x cannot be staged in `max_xp` pieces per thread.
inline bool m1_block_shape(M1Geom &g, bool lin, int wpp, int tpi, int mt, int max_xp, LaunchShape &ls) {
  const bool multirow = g.mr_shift >= 0;
  ls.nwaves = wpp * g.phases;
  ls.tpi = tpi;
  g.wpp = wpp; g.wpp_inv = (65536 + wpp - 1) / wpp;
  const int tiles_per_block = wpp * tpi;
  ls.nblocks = (g.ntiles + tiles_per_block - 1) / tiles_per_block;
  const int lds_pieces = multirow ? g.nchunks * 8 : g.phases * 512;
  // x in LDS is padded once per 16 pieces for the contiguous-kilobyte form, else once per 32
  g.xtok = lin ? 16 * lds_pieces + 16 * ((lds_pieces + 15) >> 4) : 16 * lds_pieces + 16 * ((lds_pieces + 31) >> 5);
  g.part_offset = mt * g.xtok;
  ls.lds = g.part_offset + (g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block * mt : 0);
  ls.xp = (lds_pieces + 64 * ls.nwaves - 1) / (64 * ls.nwaves);
  return ls.xp <= max_xp;
}

}  // namespace egt
#endif
