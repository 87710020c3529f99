// Device body of the dense INT4 M = 1 kernel with its launch geometry, shared by the
// single-matrix, batched and multi-matrix launchers.
#ifndef EGT_DENSE_BODY_H
#define EGT_DENSE_BODY_H

#include "egt_mfma_common.h"

namespace egt {

// Eight INT4 codes of one dword (column k in bits 4k..4k+3) -> four half2
// registers {col 2p, col 2p+1} holding 64 + q.  Byte p of the dword holds the odd
// column in its high nibble; byte p of (dword << 4) holds the even one there.
__device__ __forceinline__ u4 nibbles_to_f16(uint32_t d, uint32_t mask, uint32_t magic) {
  const uint32_t dsh = d << 4;
  u4 r;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t t = __builtin_amdgcn_perm(d, dsh, 0x0c040c00u + (uint32_t)p * 0x00010001u);
    r[p] = and_or(t, mask, magic);
  }
  return r;
}

// One diagonal element of a dense tile, s * (sum (64 + q) x - (64 + z) * sum x), from the
// instruction's sum `diag`, the group's {scale, zero} bits and the sum of x over the group.
// The rounding steps are spelled out (one fused multiply-add, one multiply) so that every
// kernel that finishes a tile gets the same bits whatever the compiler contracts elsewhere.
__device__ __forceinline__ float dense_finish(float diag, uint32_t qp, float xq) {
  const float sc = __half2float(__ushort_as_half((uint16_t)(qp & 0xFFFFu)));
  const float zp = __half2float(__ushort_as_half((uint16_t)(qp >> 16)));
  return __fmul_rn(sc, __fmaf_rn(-(64.f + zp), xq, diag));
}

struct DenseGeom {
  int rows;
  int nchunks;         // cols / 32
  int ntiles;          // tiles per phase = ceil(rows / rows_per_tile)
  int phases;          // tiles per row (row-tile mode), else 1
  int mr_shift;        // multi-row mode: log2(nchunks) (16 or 32 chunks per row); else -1
  int groups_per_row;  // cols / group
  int gs;              // group = 128 << gs columns (scaled after the instruction) or 32 << gs (before)
  uint32_t last_chunk; // rows * nchunks - 1
  int part_offset;     // byte offset of the per-phase partial sums in LDS
  uint32_t nib_mask;   // 0x00F000F0: the nibble of each half that becomes a mantissa
  uint32_t nib_magic;  // 0x54005400: FP16 64.0 in both halves
  int wpp, wpp_inv;    // waves per phase in a workgroup, ceil(65536 / wpp)
};

template <int TPI, int XP, bool PRE>
__device__ __forceinline__ void k_int4_m1_body(const uint8_t *__restrict__ q, const uint8_t *__restrict__ qparams,
    const __half *__restrict__ x, __half *__restrict__ y, const DenseGeom &g) {
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
  const int cit = 4 * i + kb;                         // chunk of this lane inside a tile
  const bool multirow = g.mr_shift >= 0;
  const int rpt = multirow ? (64 >> g.mr_shift) : 1;  // rows per tile
  const int c = multirow ? (cit & (g.nchunks - 1)) : cit + 64 * phase;   // chunk inside the row
  const int c_ld = min(c, g.nchunks - 1);

  // ---- x first: 16 B pieces, fetched once per block
  const int npieces = g.nchunks * 4;
  const int lds_pieces = multirow ? npieces : g.phases * 256;
  u4 xp[XP];
  x_request<XP>(x, npieces, xp);

  // ---- every load of the wave's TPI tiles: nibbles of the own chunk, and the
  //      {scale, zero} of the quad (lane & 15), whose diagonal this lane may hold
  const int tile0 = (blockIdx.x * wpp + wslot) * TPI;
  const int ql = lane & 15;
  const int qrow = multirow ? ((4 * ql) >> g.mr_shift) : 0;
  const int rsub = multirow ? (cit >> g.mr_shift) : 0;
  const int qgrp = PRE ? (c_ld >> g.gs)
                       : multirow ? ((((4 * ql) & (g.nchunks - 1)) >> 2) >> g.gs)
                                  : min((16 * phase + ql) >> g.gs, g.groups_per_row - 1);
  u4 nib[TPI];
  uint32_t qp[TPI];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    const int tr = min(tile0 + t, g.ntiles - 1);      // uniform
    uint32_t chunk;
    if (multirow) chunk = min((uint32_t)tr * 64u + (uint32_t)cit, g.last_chunk);
    else chunk = (uint32_t)tr * (uint32_t)g.nchunks + (uint32_t)c_ld;
    nib[t] = ld_stream<u4>(q + 16ull * chunk);
    const int r = min(tr * rpt + (PRE ? rsub : qrow), g.rows - 1);
    qp[t] = ld_stream<uint32_t>(qparams + 4ull * ((uint32_t)r * (uint32_t)g.groups_per_row + (uint32_t)qgrp));
  }
  const int sum_steps = multirow ? (g.mr_shift - 4) : 2;       // log2(quad groups per row)
  constexpr int NB = (TPI + 3) / 4;
  int rrow[NB];
  bool st[NB];
#pragma unroll
  for (int bt = 0; bt < NB; ++bt) {
    const int t = 4 * bt + ((lane >> 2) & 3);
    const int tr = tile0 + t;
    rrow[bt] = tr * rpt + ((lane & 3) >> sum_steps);
    st[bt] = lane < 16 && t < TPI && tr < g.ntiles && rrow[bt] < g.rows &&
             ((lane & 3) & ((1 << sum_steps) - 1)) == 0;
  }

  // ---- x through LDS: piece p at byte 16 p + 16 (p >> 4), i.e. one 16 B pad per
  //      256 B, so that lanes 256 B apart hit different banks; zero past the end
  x_store<XP, 4>(xs, xp, npieces, lds_pieces);
  __syncthreads();
  // B operand: lane (n, kb) holds the activations of chunk 4 n + kb, 8 per instruction
  u4 bx[4];
  {
    const int cb = multirow ? c : cit + 64 * phase;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int pi = 4 * cb + d;
      bx[d] = *(const u4 *)(xs + 16 * pi + 16 * (pi >> 4));
    }
  }
  // sum of x over each quad: every row of D gets the column sums of B
  f4 xsum = {0.f, 0.f, 0.f, 0.f};
  if (!PRE) {
    const u4 ones = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
#pragma unroll
    for (int d = 0; d < 4; ++d)
      xsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, ones), __builtin_bit_cast(h8, bx[d]), xsum, 0, 0, 0);
  }
  const float xq = xsum[0];                           // quad (lane & 15)

  // ---- consume
  const uint32_t magic = in_vgpr(g.nib_magic);
  float s[TPI];
#pragma unroll
  for (int t = 0; t < TPI; ++t) {
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    uint32_t s2 = 0, off = 0;
    if (PRE) {
      s2 = __builtin_amdgcn_perm(qp[t], qp[t], 0x01000100u);                            // {s, s}
      off = pk_add_f16(__builtin_amdgcn_perm(qp[t], qp[t], 0x03020302u), g.nib_magic);  // {64 + z, 64 + z}
    }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      u4 a = nibbles_to_f16(nib[t][d], g.nib_mask, magic);
      if (PRE) {
#pragma unroll
        for (int p = 0; p < 4; ++p) a[p] = pk_mul_f16(pk_sub_f16(a[p], off), s2);
      }
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, bx[d]), acc, 0, 0, 0);
    }
    // lane 20 kb + v holds D[4 kb + v][4 kb + v] in register v = lane & 3
    const float diag = select4(lane & 3, acc[0], acc[1], acc[2], acc[3]);
    float val = diag;
    if (!PRE) val = dense_finish(diag, qp[t], xq);
    s[t] = val + row_shl<1>(val) + row_shl<2>(val) + row_shl<3>(val);   // valid in lanes 20 kb
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
      if (g.phases == 1) y[rrow[bt]] = __float2half(v);
      else part[phase * (wpp * TPI) + wslot * TPI + 4 * bt + ((lane >> 2) & 3)] = v;
    }
  }
  if (g.phases > 1) {
    __syncthreads();
    const int per = wpp * TPI;                        // rows handled by this block
    for (int j = threadIdx.x; j < per; j += blockDim.x) {
      const int r = blockIdx.x * per + j;
      if (r < g.rows) {
        float v = 0.f;
        for (int p = 0; p < g.phases; ++p) v += part[p * per + j];
        y[r] = __float2half(v);
      }
    }
  }
}

// Geometry of a dense INT4 matrix (everything that does not depend on the block shape).
// Groups of 128 columns and more are scaled after the matrix instruction, narrower ones
// before it (`pre`).
inline void dense_geometry(int rows, int cols, int group, DenseGeom &g, bool &pre) {
  g.rows = rows;
  g.nchunks = cols / 32;
  const bool multirow = g.nchunks < 64;
  g.mr_shift = multirow ? (g.nchunks == 16 ? 4 : 5) : -1;
  const int rpt = multirow ? 64 / g.nchunks : 1;
  g.phases = multirow ? 1 : (g.nchunks + 63) / 64;
  g.ntiles = (rows + rpt - 1) / rpt;
  g.groups_per_row = cols / group;
  pre = group < 128;
  g.gs = 0;
  while (((pre ? 32 : 128) << g.gs) < group) ++g.gs;
  g.last_chunk = (uint32_t)rows * (uint32_t)g.nchunks - 1u;
  g.nib_mask = 0x00F000F0u;
  g.nib_magic = 0x54005400u;
}

// Block shape for `wpp` waves per phase and `tpi` tiles per wave; fills the LDS offset of
// the geometry.  False when x cannot be staged in `max_xp` pieces per thread.
inline bool dense_block_shape(DenseGeom &g, int wpp, int tpi, int max_xp, LaunchShape &ls) {
  const bool multirow = g.mr_shift >= 0;
  ls.nwaves = wpp * g.phases;
  ls.tpi = tpi;
  g.wpp = wpp; g.wpp_inv = (65536 + wpp - 1) / wpp;
  const int tiles_per_block = wpp * tpi;
  ls.nblocks = (g.ntiles + tiles_per_block - 1) / tiles_per_block;
  const int lds_pieces = multirow ? g.nchunks * 4 : g.phases * 256;
  g.part_offset = 16 * lds_pieces + 16 * ((lds_pieces + 15) >> 4);
  ls.lds = g.part_offset + (g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block : 0);
  ls.xp = (lds_pieces + 64 * ls.nwaves - 1) / (64 * ls.nwaves);
  return ls.xp <= max_xp;
}

}  // namespace egt
#endif
