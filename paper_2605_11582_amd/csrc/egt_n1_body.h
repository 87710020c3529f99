// Device body of the 1:4 M = 1 kernel with its launch geometry, shared by the
// single-matrix, batched and multi-matrix launchers.
#ifndef EGT_N1_BODY_H
#define EGT_N1_BODY_H

#include "egt_mfma_common.h"

namespace egt {

struct M1N1Geom {
  int rows;
  int nchunks;         // cols / 128
  int ntiles;
  int phases;
  int mr_shift;        // multi-row mode: log2(nchunks) (16 or 32); -1 in row-tile mode
  int gshift;          // INT4 group = 128 << gshift dense columns
  int groups_per_row;
  uint32_t last_chunk;
  int part_offset;
  uint32_t m8, m4, m2; // masks of spread_idx, passed in so that they live in registers
  uint32_t nib_mask;   // 0x00F0000F
  uint32_t nib_magic;  // 0x54006400: FP16 {1024.0, 64.0}
  int wpp, wpp_inv;    // waves per phase in a workgroup, ceil(65536 / wpp)
};

// QW = {scale, zero} pairs per chunk of 128 dense columns: 1 for groups of 128 and more,
// 2 for groups of 64, 4 for groups of 32.
// NI > 0 (FP16 values): a tile is one row (one phase of it: up to 64 NI pieces of 16 bytes,
// a piece being 8 slots = 32 dense columns = one 16-bit index word) and load instruction k
// of a wave reads the contiguous kilobyte of pieces 64 k + lane.  Lane (i, kb) then owns the
// pieces 64 k + 16 kb + i, k < NI, each good for two matrix instructions (slots 0..3 and
// 4..7), and column n of B carries the activations under the pieces 64 k + 16 kb + n.
// NI = 0: every lane reads the 64 B of its own chunk.
template <int KIND, int TPI, int XP, int QW, int NI>
__device__ __forceinline__ void k_sparse_m1_n1_body(const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
    const uint8_t *__restrict__ idx, const uint8_t *__restrict__ qparams, const __half *__restrict__ x,
    __half *__restrict__ y, const M1N1Geom &g) {
  extern __shared__ __align__(16) uint8_t xs[];       // staged x, then [phases][rows of this block] floats
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // waves per phase in this workgroup; (wave * wpp_inv) >> 16 = wave / wpp for wave < 16
  // (both from the host: integer divisions here would delay the first request)
  const int wpp = g.wpp;
  float *part = (float *)(xs + g.part_offset);
  const int phase = (wave * g.wpp_inv) >> 16;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;
  const bool multirow = g.mr_shift >= 0;
  const int rpt = multirow ? (64 >> g.mr_shift) : 1;
  const int c = multirow ? (cit & (g.nchunks - 1)) : cit + 64 * phase;
  const int rsub = multirow ? (cit >> g.mr_shift) : 0;
  const int c_ld = min(c, g.nchunks - 1);

  // ---- x first (16 B pieces, 16 per chunk)
  const int npieces = g.nchunks * 16;
  constexpr bool LIN = NI > 0;
  constexpr int XSH = LIN ? 4 : 6;                    // x in LDS: one 16 B pad per 2^XSH pieces
  const int lds_pieces = LIN ? g.phases * NI * 256 : multirow ? npieces : g.phases * 1024;
  u4 xp[XP];
  x_request<XP>(x, npieces, xp);

  const int tile0 = (blockIdx.x * wpp + wslot) * TPI;
  // several tiles per row: the threads that add the phases up at the end fetch the row
  // pointer of their row now (wpp * TPI <= 64 <= blockDim: one output per thread)
  uint32_t rp_fin = 0;
  if (g.phases > 1 && (int)threadIdx.x < wpp * TPI) {
    const int r = blockIdx.x * (wpp * TPI) + (int)threadIdx.x;
    if (r < g.rows) rp_fin = row_ptr[r];
  }
  u4 nib[TPI][KIND == EGT_VAL_INT4 ? 1 : 4];
  u2 iw[TPI];
  uint32_t iwl[LIN ? TPI : 1][LIN ? NI : 1];          // LIN: the index word of each piece
  uint32_t qp[TPI][QW];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    const int tr = min(tile0 + t, g.ntiles - 1);
    if constexpr (LIN) {
#pragma unroll
      for (int k = 0; k < NI; ++k) {
        const uint32_t piece = (uint32_t)min(NI * 64 * phase + 64 * k + lane, 4 * g.nchunks - 1);   // inside the row (clamped)
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
      const uint8_t *qrow = qparams + 4ull * ((uint32_t)r * (uint32_t)g.groups_per_row);
      if (QW == 4) {
        const u4 v = ld_stream<u4>(qrow + 16u * (uint32_t)c_ld);
#pragma unroll
        for (int k = 0; k < QW; ++k) qp[t][k] = v[k & 3];
      } else if (QW == 2) {
        const u2 v = ld_stream<u2>(qrow + 8u * (uint32_t)c_ld);
#pragma unroll
        for (int k = 0; k < QW; ++k) qp[t][k] = v[k & 1];
      } else {
        qp[t][0] = ld_stream<uint32_t>(qrow + 4u * (uint32_t)(c_ld >> g.gshift));
      }
    } else {
#pragma unroll
      for (int k = 0; k < 4; ++k) nib[t][k] = ld_stream<u4>(values + 64ull * chunk + 16 * k);
    }
  }
  const int sum_steps = multirow ? (g.mr_shift - 4) : 2;
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

  // ---- x through LDS: piece p at byte 16 p + 16 (p >> 6), one 16 B pad per KiB (the
  //      16 lanes of a B read are 1 KiB apart); zero past the end of x
  x_store<XP, XSH>(xs, xp, npieces, lds_pieces);
  __syncthreads();
  // B operand of instruction m: the 16 dense columns 16 m .. 16 m + 15 of each chunk
  u8v bx[8];
  if constexpr (LIN) {
    // instruction 2 k + e multiplies slots 4 e .. 4 e + 3 (16 dense columns) of the pieces
    // 64 k + 16 kb + n: x pieces 4 P + 2 e and 4 P + 2 e + 1
    const int n = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = 2 * h + (b >> 1), sub = b & 1;
#pragma unroll
      for (int k = 0; k < NI; ++k) {
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int pi = 4 * (NI * 64 * phase + 64 * k + 16 * kba + n) + 2 * e + sub;
          const u4 v = *(const u4 *)(xs + 16 * pi + 16 * (pi >> XSH));
#pragma unroll
          for (int j = 0; j < 4; ++j) bx[2 * k + e][4 * h + j] = v[j];
        }
      }
    }
  } else {
    const int n = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = (4 * h + b) >> 1, sub = b & 1;
      int cb = 4 * n + kba;
      cb = multirow ? (cb & (g.nchunks - 1)) : cb + 64 * phase;
#pragma unroll
      for (int m = 0; m < 8; ++m) {
        const int pi = 16 * cb + 2 * m + sub;
        const u4 v = *(const u4 *)(xs + 16 * pi + 16 * (pi >> 6));
#pragma unroll
        for (int k = 0; k < 4; ++k) bx[m][4 * h + k] = v[k];
      }
    }
  }

  // ---- consume
  const uint32_t magic = in_vgpr(g.nib_magic);
  float s[TPI];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    uint32_t s2[QW], off[QW];
#pragma unroll
    for (int k = 0; k < QW; ++k) {
      s2[k] = off[k] = 0;
      if (KIND == EGT_VAL_INT4) {
        s2[k] = __builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x01000100u);                            // {s, s}
        off[k] = pk_add_f16(__builtin_amdgcn_perm(qp[t][k], qp[t][k], 0x03020302u), g.nib_magic);  // {1024+z, 64+z}
      }
    }
    if constexpr (LIN) {
#pragma unroll
      for (int k = 0; k < NI; ++k) {
        const int iword = (int)spread_idx(iwl[t][k], g.m8, g.m4, g.m2);
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const uint32_t v0 = nib[t][k][2 * e], v1 = nib[t][k][2 * e + 1];
          const u4 a = {v0 & 0xFFFFu, v0 >> 16, v1 & 0xFFFFu, v1 >> 16};
          if (e)
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[2 * k + e]), acc, iword, 0, 1);
          else
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[2 * k + e]), acc, iword, 0, 0);
        }
      }
      s[t] = acc[0] + row_shl<1>(acc[1]) + row_shl<2>(acc[2]) + row_shl<3>(acc[3]);
      continue;
    }
    const uint32_t sp[4] = {spread_idx(iw[t][0] & 0xFFFFu, g.m8, g.m4, g.m2), spread_idx(iw[t][0] >> 16, g.m8, g.m4, g.m2),
                            spread_idx(iw[t][1] & 0xFFFFu, g.m8, g.m4, g.m2), spread_idx(iw[t][1] >> 16, g.m8, g.m4, g.m2)};
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      u4 a;
      if (KIND == EGT_VAL_INT4) {
        // slots 4 m .. 4 m + 3 = bytes 2 (m & 1), 2 (m & 1) + 1 of dword m >> 1
        const uint32_t d = nib[t][0][m >> 1];
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          // the two slots of a byte are dequantised as a pair, then split into {w, 0} registers
          const uint32_t t2 = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)(2 * (m & 1) + p) * 0x00010001u);
          const uint32_t pair = pk_mul_f16(pk_sub_f16(and_or(t2, g.nib_mask, magic), off[m * QW / 8]), s2[m * QW / 8]);
          a[2 * p] = pair & 0xFFFFu;
          a[2 * p + 1] = pair >> 16;
        }
      } else {
        // FP16 values: slots 4 m .. 4 m + 3 are two dwords of the lane's 64 B
        const uint32_t v0 = nib[t][m >> 1][2 * (m & 1)], v1 = nib[t][m >> 1][2 * (m & 1) + 1];
        a[0] = v0 & 0xFFFFu; a[1] = v0 >> 16; a[2] = v1 & 0xFFFFu; a[3] = v1 >> 16;
      }
      const int iword = (int)sp[m >> 1];
      if (m & 1)
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[m]), acc, iword, 0, 1);
      else
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[m]), acc, iword, 0, 0);
    }
    s[t] = acc[0] + row_shl<1>(acc[1]) + row_shl<2>(acc[2]) + row_shl<3>(acc[3]);
  }
  const int src_lane = 20 * (lane & 3);
#pragma unroll
  for (int bt = 0; bt < NB; ++bt) {
    float v = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      if (4 * bt + k < TPI) {
        const float gk = __shfl(s[4 * bt + k], src_lane, 64);
        v = ((lane >> 2) & 3) == k ? gk : v;
      }
    }
    if (sum_steps >= 1) v += quad_xor1(v);
    if (sum_steps >= 2) v += quad_xor2(v);
    if (st[bt]) {
      const int r = rrow[bt];
      if (g.phases == 1) {
        const bool ok = rp[bt] == (uint32_t)r * (uint32_t)(g.nchunks * 32);
        y[r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
      } else {
        part[phase * (wpp * TPI) + wslot * TPI + 4 * bt + ((lane >> 2) & 3)] = v;
      }
    }
  }
  if (g.phases > 1) {
    __syncthreads();
    const int per = wpp * TPI;
    const int j = threadIdx.x;
    if (j < per) {
      const int r = blockIdx.x * per + j;
      if (r < g.rows) {
        float v = 0.f;
        for (int p = 0; p < g.phases; ++p) v += part[p * per + j];
        const bool ok = rp_fin == (uint32_t)r * (uint32_t)(g.nchunks * 32);
        y[r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
      }
    }
  }
}

// Geometry of a 1:4 matrix (everything that does not depend on the block shape).  `lin`:
// the contiguous-kilobyte form of FP16 values, with `ni` load instructions per tile.
inline void n1_geometry(const egt_2bitcsr &w, bool lin, M1N1Geom &g, int &ni) {
  g.rows = w.rows;
  g.nchunks = w.cols / 128;
  ni = !lin ? 0 : g.nchunks == 16 ? 1 : g.nchunks == 32 ? 2 : 4;
  const bool multirow = !lin && g.nchunks < 64;
  g.mr_shift = multirow ? (g.nchunks == 16 ? 4 : 5) : -1;
  const int rpt = multirow ? 64 / g.nchunks : 1;
  g.phases = (g.nchunks + 63) / 64;
  g.ntiles = (w.rows + rpt - 1) / rpt;
  g.gshift = 0;
  g.groups_per_row = 0;
  if (w.val_kind == EGT_VAL_INT4) {
    while ((128 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.last_chunk = (uint32_t)w.rows * (uint32_t)g.nchunks - 1u;
  g.m8 = 0x00FF00FFu; g.m4 = 0x0F0F0F0Fu; g.m2 = 0x33333333u;
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
}

// Block shape for `wpp` waves per phase and `tpi` tiles per wave; fills the LDS offset of
// the geometry.  False when x cannot be staged in `max_xp` pieces per thread.
inline bool n1_block_shape(M1N1Geom &g, bool lin, int ni, int wpp, int tpi, int max_xp, LaunchShape &ls) {
  const bool multirow = g.mr_shift >= 0;
  ls.nwaves = wpp * g.phases;
  ls.tpi = tpi;
  g.wpp = wpp; g.wpp_inv = (65536 + wpp - 1) / wpp;
  const int tiles_per_block = wpp * tpi;
  ls.nblocks = (g.ntiles + tiles_per_block - 1) / tiles_per_block;
  const int lds_pieces = lin ? g.phases * ni * 256 : multirow ? g.nchunks * 16 : g.phases * 1024;
  g.part_offset = lin ? 16 * lds_pieces + 16 * ((lds_pieces + 15) >> 4) : 16 * lds_pieces + 16 * ((lds_pieces + 63) >> 6);
  ls.lds = g.part_offset + (g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block : 0);
  ls.xp = (lds_pieces + 64 * ls.nwaves - 1) / (64 * ls.nwaves);
  return ls.xp <= max_xp;
}

}  // namespace egt
#endif
