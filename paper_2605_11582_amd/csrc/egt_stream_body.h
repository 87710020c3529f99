// Streaming form of the M = 1 kernels for tables that are much larger than what the device
// holds in flight at once (a decoder stack: gigabytes).
//
// The single-matrix kernels are one-shot: every wave requests all of its tiles at once,
// waits, computes, and leaves.  That is the right shape for a matrix of a few megabytes -
// the whole matrix is on its way within a microsecond - but as a stream of short-lived
// workgroups it leaves the memory system idle whenever a workgroup starts up or drains.
// Here the planner cuts the concatenation of all matrices into spans of equal byte count, one
// per workgroup (eight per compute unit, two of them resident at a time: 24 waves, each with
// its own requests in flight; spans this short also even out the finish), so a workgroup
// streams one contiguous stretch of the table; a span is a short
// list of work items, an item being a block of consecutive rows of one matrix.  Per item the
// workgroup stages x in LDS once; every wave then owns one tile column of the rows (a
// "phase": 4096 dense columns at 2:4, 2048 for dense INT4), keeps the B operand of that
// column in registers for the whole item and streams its tiles through a ring of DEPTH
// register sets: tile j is consumed while tiles j + 1 .. j + DEPTH are on their way.  Every
// request is issued unconditionally - a tile past the end of the item is requested out of
// range of its buffer resource, which returns zeros and moves no data - so the loop has
// no branch around a load and the compiler's own wait counts are exact.
//
// Tile arithmetic, operand mapping, LDS layout of x and the order of every floating-point
// addition are those of the single-matrix kernels (egt_m1_body.h, egt_dense_body.h): the
// results are the same bits.
#ifndef EGT_STREAM_BODY_H
#define EGT_STREAM_BODY_H

#include "egt_dense_body.h"
#include "egt_m1_body.h"
#include "egt_n1_body.h"

namespace egt {

enum : int32_t { FORM_S24 = 0, FORM_S14 = 1, FORM_DENSE = 2 };

// One matrix of a streamed table (device memory of the caller, written by the planner).
struct StreamMatrix {
  const uint32_t *row_ptr;   // 2:4 only
  const uint8_t *values;     // nibbles
  const uint8_t *idx;        // 2:4 only
  const uint8_t *qparams;
  const __half *x;
  __half *y;
  int32_t form;              // FORM_S24, FORM_S14 or FORM_DENSE
  int32_t rows;
  int32_t nchunks;           // cols / 64 (2:4), cols / 128 (1:4) or cols / 32 (dense)
  int32_t phases;            // tiles per row
  int32_t gshift;            // 2:4: group = 64 << gshift columns; 1:4 and dense: group = 128 << gshift
  int32_t groups_per_row;
  uint32_t val_bytes, idx_bytes, qp_bytes;   // extents of the arrays (buffer resources)
  int32_t item_rows;         // rows of a work item of this matrix at most
  int32_t mr_shift;          // 1:4 with rows of 16 or 32 chunks: log2(chunks per row), a tile is 64 chunks = 4 or 2 rows; else -1
};

// One work item: `nrows` consecutive rows of matrix `matrix` starting at `row0`.
struct StreamItem {
  uint32_t matrix;
  uint32_t row0;
  uint32_t nrows;
  uint32_t reserved;
};

constexpr int STREAM_MAX_ITEM_ROWS = 2048;           // rows of an item at most (16 B of partial sums per row and tile)
constexpr uint32_t STREAM_OFF_RANGE = 0xFFFFFFF0u;   // lane offset past any buffer: zeros, no traffic
#ifndef EGT_STREAM_NT
#define EGT_STREAM_NT 2
#endif
constexpr int STREAM_NT = EGT_STREAM_NT;             // cache policy of the weight requests: 2 = non-temporal

// Pointers that arrive through a table in memory are generic to the compiler; loads through
// them would be flat operations, which count against both wait counters and break the
// in-order accounting of the tile ring.  They all point to device memory.
typedef __attribute__((address_space(1))) const u4 global_u4;
typedef __attribute__((address_space(1))) const uint32_t global_u32;
typedef __attribute__((address_space(1))) uint16_t global_u16;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t stream_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// x of one matrix into LDS, in the layout of the single-matrix kernel of its form, in two
// halves: the requests go out first (before the first tiles are requested, so that x is
// the first data to return), the LDS writes follow once the tiles are on their way.
template <int XP>
__device__ __forceinline__ void stream_x_request(u4 (&xp)[XP], const __half *__restrict__ x, int npieces, int nthreads) {
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int pi = threadIdx.x + j * nthreads;
    xp[j] = *(global_u4 *)(x + 8 * min(pi, npieces - 1));
  }
}
template <int XP>
__device__ __forceinline__ void stream_x_store(const u4 (&xp)[XP], uint8_t *xs, int npieces, int lds_pieces, int pad_shift,
                                               int nthreads) {
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int pi = threadIdx.x + j * nthreads;
    if (pi < lds_pieces) {
      u4 v = xp[j];
      if (pi >= npieces) v = u4{0, 0, 0, 0};
      *(u4 *)(xs + 16 * pi + 16 * (pi >> pad_shift)) = v;
    }
  }
}

// ---- 2:4 sparse INT4, one {scale, zero} pair per chunk -------------------------------
// `part`: partial sums of the item, [row][phase][4] floats.
template <int XP, int DEPTH>
__device__ __forceinline__ void stream_item_s24(const StreamMatrix &m, uint8_t *xs, float *part, int row0, int nrows,
                                                uint32_t nib_mask, uint32_t nib_magic, int nthreads) {
  u4 xp[XP];
  stream_x_request<XP>(xp, m.x, m.nchunks * 8, nthreads);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = nthreads >> 6;
  const int wpp = nwaves / m.phases;
  const int phase = wave / wpp;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;
  const int c_ld = min(cit + 64 * phase, m.nchunks - 1);
  const int n = nrows > wslot ? (nrows - wslot + wpp - 1) / wpp : 0;     // tiles of this wave

  const __amdgpu_buffer_rsrc_t r_val = stream_rsrc(m.values, m.val_bytes), r_idx = stream_rsrc(m.idx, m.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = stream_rsrc(m.qparams, m.qp_bytes);
  const uint32_t l_val = 16u * (uint32_t)c_ld, l_idx = 8u * (uint32_t)c_ld, l_qp = 4u * (uint32_t)(c_ld >> m.gshift);
  u4 nib[DEPTH];
  u2 iw[DEPTH];
  uint32_t qp[DEPTH];
  auto request = [&](int slot, int j) {
    const bool on = j < n;                                                // uniform
    const uint32_t row = (uint32_t)(row0 + wslot + (on ? j : 0) * wpp);
    const uint32_t cu = row * (uint32_t)m.nchunks;
    nib[slot] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? l_val : STREAM_OFF_RANGE, 16u * cu, STREAM_NT);
    iw[slot] = __builtin_amdgcn_raw_buffer_load_b64(r_idx, on ? l_idx : STREAM_OFF_RANGE, 8u * cu, STREAM_NT);
    qp[slot] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, on ? l_qp : STREAM_OFF_RANGE,
                                                    4u * row * (uint32_t)m.groups_per_row, STREAM_NT);
  };
  // (the requests of a ring slot stay together and the slots in order: the wait before a
  //  tile is consumed counts the requests made after it)
  static_for<0, DEPTH>([&](auto d) {
    request(d.v, d.v);
    __builtin_amdgcn_sched_barrier(0);
  });
  stream_x_store<XP>(xp, xs, m.nchunks * 8, m.phases * 512, 5, nthreads);
  lds_barrier();

  // B operand of this wave's tile column (see egt_m1_body.h): column n = lane & 15 holds the
  // activations of chunks 4n .. 4n+3; lane (n, b) supplies k-octets b and 4 + b
  u8v bx[4];
  {
    const int nn = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = (4 * h + b) >> 1, sub = b & 1;
      const int cb = 4 * nn + kba + 64 * phase;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const int pi = 8 * cb + 2 * d + sub;
        const u4 v = *(const u4 *)(xs + 16 * pi + 16 * (pi >> 5));
#pragma unroll
        for (int k = 0; k < 4; ++k) bx[d][4 * h + k] = v[k];
      }
    }
  }
  const uint32_t magic = in_vgpr(nib_magic);
  float *my_part = part + 4 * phase + (lane >> 4);                       // + 4 * phases * row
  const bool writer = (lane == 0) | (lane == 20) | (lane == 40) | (lane == 60);

  for (int j0 = 0; j0 < n; j0 += DEPTH) {
    static_for<0, DEPTH>([&](auto d) {
      const int j = j0 + d.v;
      if (j < n) {                                                        // uniform; the requests stay outside
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        const uint32_t q = qp[d.v];
        const uint32_t s2 = __builtin_amdgcn_perm(q, q, 0x01000100u);                           // {s, s}
        const uint32_t off = pk_add_f16(__builtin_amdgcn_perm(q, q, 0x03020302u), nib_magic);   // {1024+z, 64+z}
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
          const u4 a = dequant8(nib[d.v][dd], off, s2, nib_mask, magic);
          const int iword = dd < 2 ? (int)iw[d.v][0] : (int)iw[d.v][1];
          if (dd & 1)
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[dd]), acc, iword, 0, 1);
          else
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[dd]), acc, iword, 0, 0);
        }
        const float s = acc[0] + row_shl<1>(acc[1]) + row_shl<2>(acc[2]) + row_shl<3>(acc[3]);
        if (writer) my_part[4 * m.phases * (wslot + j * wpp)] = s;
      }
      __builtin_amdgcn_sched_barrier(0);
      request(d.v, j + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    });
  }
}

// ---- 1:4 sparse INT4, one {scale, zero} pair per chunk of 128 columns -------------------
// A tile is 64 chunks: one row's share of a phase, or (rows of 16 or 32 chunks) 4 or 2 whole
// rows.  `part`: [tile][phase][4] floats, the four quarter sums of a tile (a quarter belongs
// to one row: quarters per row = 4, 2 or 1).  Every slot becomes the pair {value, 0} with its
// offset in the even index field, eight instructions per tile, as in egt_n1_body.h.
template <int XP, int DEPTH>
__device__ __forceinline__ void stream_item_s14(const StreamMatrix &m, uint8_t *xs, float *part, int row0, int nrows,
                                                uint32_t nib_mask, uint32_t nib_magic, int nthreads) {
  u4 xp[XP];
  stream_x_request<XP>(xp, m.x, m.nchunks * 16, nthreads);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = nthreads >> 6;
  const int wpp = nwaves / m.phases;
  const int phase = wave / wpp;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;
  const bool multirow = m.mr_shift >= 0;
  const int rpt_shift = multirow ? 6 - m.mr_shift : 0;                    // log2(rows per tile)
  const int c = multirow ? (cit & (m.nchunks - 1)) : cit + 64 * phase;
  const int rsub = multirow ? (cit >> m.mr_shift) : 0;
  const int c_ld = min(c, m.nchunks - 1);
  const int ntiles = (nrows + (1 << rpt_shift) - 1) >> rpt_shift;         // tiles of the item (row0 is a multiple of rows per tile)
  const int n = ntiles > wslot ? (ntiles - wslot + wpp - 1) / wpp : 0;    // tiles of this wave

  const __amdgpu_buffer_rsrc_t r_val = stream_rsrc(m.values, m.val_bytes), r_idx = stream_rsrc(m.idx, m.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = stream_rsrc(m.qparams, m.qp_bytes);
  // lane part of the chunk number: the tile's 64 chunks in lane order, or chunk c_ld of the row
  const uint32_t l_chunk = multirow ? (uint32_t)cit : (uint32_t)c_ld;
  const uint32_t l_qp = 4u * ((uint32_t)rsub * (uint32_t)m.groups_per_row + (uint32_t)(c_ld >> m.gshift));
  u4 nib[DEPTH];
  u2 iw[DEPTH];
  uint32_t qp[DEPTH];
  auto request = [&](int slot, int j) {
    const bool on = j < n;                                                // uniform
    const uint32_t tile = (uint32_t)((row0 >> rpt_shift) + wslot + (on ? j : 0) * wpp);
    const uint32_t cu = multirow ? 64u * tile : tile * (uint32_t)m.nchunks;                 // first chunk of the tile / of its row
    // (a tile that reaches past the last row is cut off by the buffer resources: zeros)
    nib[slot] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? 16u * l_chunk : STREAM_OFF_RANGE, 16u * cu, STREAM_NT);
    iw[slot] = __builtin_amdgcn_raw_buffer_load_b64(r_idx, on ? 8u * l_chunk : STREAM_OFF_RANGE, 8u * cu, STREAM_NT);
    qp[slot] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, on ? l_qp : STREAM_OFF_RANGE,
                                                    4u * (tile << rpt_shift) * (uint32_t)m.groups_per_row, STREAM_NT);
  };
  static_for<0, DEPTH>([&](auto d) {
    request(d.v, d.v);
    __builtin_amdgcn_sched_barrier(0);
  });
  stream_x_store<XP>(xp, xs, m.nchunks * 16, multirow ? m.nchunks * 16 : m.phases * 1024, 6, nthreads);
  lds_barrier();

  // B operand of instruction mm: the 16 dense columns 16 mm .. 16 mm + 15 of each chunk
  u8v bx[8];
  {
    const int nn = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = (4 * h + b) >> 1, sub = b & 1;
      int cb = 4 * nn + kba;
      cb = multirow ? (cb & (m.nchunks - 1)) : cb + 64 * phase;
#pragma unroll
      for (int mm = 0; mm < 8; ++mm) {
        const int pi = 16 * cb + 2 * mm + sub;
        const u4 v = *(const u4 *)(xs + 16 * pi + 16 * (pi >> 6));
#pragma unroll
        for (int k = 0; k < 4; ++k) bx[mm][4 * h + k] = v[k];
      }
    }
  }
  const uint32_t magic = in_vgpr(nib_magic);
  const uint32_t m8 = in_vgpr(0x00FF00FFu), m4 = in_vgpr(0x0F0F0F0Fu), m2 = in_vgpr(0x33333333u);
  float *my_part = part + 4 * phase + (lane >> 4);                       // + 4 * phases * tile
  const bool writer = (lane == 0) | (lane == 20) | (lane == 40) | (lane == 60);

  for (int j0 = 0; j0 < n; j0 += DEPTH) {
    static_for<0, DEPTH>([&](auto d) {
      const int j = j0 + d.v;
      if (j < n) {                                                        // uniform; the requests stay outside
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        const uint32_t q = qp[d.v];
        const uint32_t s2 = __builtin_amdgcn_perm(q, q, 0x01000100u);                           // {s, s}
        const uint32_t off = pk_add_f16(__builtin_amdgcn_perm(q, q, 0x03020302u), nib_magic);   // {1024+z, 64+z}
        const uint32_t sp[4] = {spread_idx(iw[d.v][0] & 0xFFFFu, m8, m4, m2), spread_idx(iw[d.v][0] >> 16, m8, m4, m2),
                                spread_idx(iw[d.v][1] & 0xFFFFu, m8, m4, m2), spread_idx(iw[d.v][1] >> 16, m8, m4, m2)};
#pragma unroll
        for (int mm = 0; mm < 8; ++mm) {
          // slots 4 mm .. 4 mm + 3 = bytes 2 (mm & 1), 2 (mm & 1) + 1 of dword mm >> 1: the two slots of a byte
          // are dequantised as a pair, then split into {w, 0} registers
          const uint32_t dw = nib[d.v][mm >> 1];
          u4 a;
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t t2 = __builtin_amdgcn_perm(dw, dw, 0x0c000c00u + (uint32_t)(2 * (mm & 1) + p) * 0x00010001u);
            const uint32_t pair = pk_mul_f16(pk_sub_f16(and_or(t2, nib_mask, magic), off), s2);
            a[2 * p] = pair & 0xFFFFu;
            a[2 * p + 1] = pair >> 16;
          }
          const int iword = (int)sp[mm >> 1];
          if (mm & 1)
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[mm]), acc, iword, 0, 1);
          else
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[mm]), acc, iword, 0, 0);
        }
        const float s = acc[0] + row_shl<1>(acc[1]) + row_shl<2>(acc[2]) + row_shl<3>(acc[3]);
        if (writer) my_part[4 * m.phases * (wslot + j * wpp)] = s;
      }
      __builtin_amdgcn_sched_barrier(0);
      request(d.v, j + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    });
  }
}

// ---- dense INT4, groups of 128 columns and more ---------------------------------------
template <int XP, int DEPTH>
__device__ __forceinline__ void stream_item_dense(const StreamMatrix &m, uint8_t *xs, float *part, int row0, int nrows,
                                                  uint32_t nib_mask, uint32_t nib_magic, int nthreads) {
  u4 xp[XP];
  stream_x_request<XP>(xp, m.x, m.nchunks * 4, nthreads);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = nthreads >> 6;
  const int wpp = nwaves / m.phases;
  const int phase = wave / wpp;
  const int wslot = wave - phase * wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;
  const int c = cit + 64 * phase;
  const int c_ld = min(c, m.nchunks - 1);
  const int ql = lane & 15;
  const int qgrp = min((16 * phase + ql) >> m.gshift, m.groups_per_row - 1);
  const int n = nrows > wslot ? (nrows - wslot + wpp - 1) / wpp : 0;

  const __amdgpu_buffer_rsrc_t r_val = stream_rsrc(m.values, m.val_bytes), r_qp = stream_rsrc(m.qparams, m.qp_bytes);
  const uint32_t l_val = 16u * (uint32_t)c_ld, l_qp = 4u * (uint32_t)qgrp;
  u4 nib[DEPTH];
  uint32_t qp[DEPTH];
  auto request = [&](int slot, int j) {
    const bool on = j < n;
    const uint32_t row = (uint32_t)(row0 + wslot + (on ? j : 0) * wpp);
    nib[slot] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? l_val : STREAM_OFF_RANGE, 16u * row * (uint32_t)m.nchunks, STREAM_NT);
    qp[slot] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, on ? l_qp : STREAM_OFF_RANGE,
                                                    4u * row * (uint32_t)m.groups_per_row, STREAM_NT);
  };
  // (the requests of a ring slot stay together and the slots in order: the wait before a
  //  tile is consumed counts the requests made after it)
  static_for<0, DEPTH>([&](auto d) {
    request(d.v, d.v);
    __builtin_amdgcn_sched_barrier(0);
  });
  stream_x_store<XP>(xp, xs, m.nchunks * 4, m.phases * 256, 4, nthreads);
  lds_barrier();

  // B operand: lane (n, kb) holds the activations of its own chunk (see egt_dense_body.h)
  u4 bx[4];
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const int pi = 4 * c + d;
    bx[d] = *(const u4 *)(xs + 16 * pi + 16 * (pi >> 4));
  }
  f4 xsum = {0.f, 0.f, 0.f, 0.f};
  {
    const u4 ones = {0x3C003C00u, 0x3C003C00u, 0x3C003C00u, 0x3C003C00u};
#pragma unroll
    for (int d = 0; d < 4; ++d)
      xsum = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, ones), __builtin_bit_cast(h8, bx[d]), xsum, 0, 0, 0);
  }
  const float xq = xsum[0];
  const uint32_t magic = in_vgpr(nib_magic);
  float *my_part = part + 4 * phase + (lane >> 4);
  const bool writer = (lane == 0) | (lane == 20) | (lane == 40) | (lane == 60);

  for (int j0 = 0; j0 < n; j0 += DEPTH) {
    static_for<0, DEPTH>([&](auto d) {
      const int j = j0 + d.v;
      if (j < n) {
        f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
          const u4 a = nibbles_to_f16(nib[d.v][dd], nib_mask, magic);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, bx[dd]), acc, 0, 0, 0);
        }
        const float diag = select4(lane & 3, acc[0], acc[1], acc[2], acc[3]);
        const float val = dense_finish(diag, qp[d.v], xq);
        const float s = val + row_shl<1>(val) + row_shl<2>(val) + row_shl<3>(val);
        if (writer) my_part[4 * m.phases * (wslot + j * wpp)] = s;
      }
      __builtin_amdgcn_sched_barrier(0);
      request(d.v, j + DEPTH);
      __builtin_amdgcn_sched_barrier(0);
    });
  }
}

// Persistent kernel: workgroup b takes the items first[b] .. first[b + 1] - 1.
// FORMS: bit 0 2:4 items present, bit 2 dense items present.
// FORMS == 2: a table of 1:4 matrices (a launch of its own: their body needs more registers).
template <int XP, int FORMS, int DEPTH_S, int DEPTH_D>
__device__ __forceinline__ void stream_body(const uint8_t *__restrict__ matrices, const uint32_t *__restrict__ first,
                                            const StreamItem *__restrict__ items, int entry_bytes, int part_offset,
                                            int nthreads) {
  extern __shared__ __align__(16) uint8_t xs[];       // staged x, then the partial sums of the item
  float *part = (float *)(xs + part_offset);
  const int it_end = (int)first[blockIdx.x + 1];
  for (int it = (int)first[blockIdx.x]; it < it_end; ++it) {
    const StreamItem item = items[it];
    const StreamMatrix m = *(const StreamMatrix *)(matrices + (size_t)item.matrix * (size_t)entry_bytes);
    const int row0 = (int)item.row0;
    const int nrows = (int)item.nrows;
    const bool sparse = (FORMS & 1) && (!(FORMS & 4) || m.form == FORM_S24);
    // (x of this item goes into LDS only after every wave has left the previous item's loop,
    //  whose closing barrier is behind us; the sums of the previous item are read before the
    //  barrier inside the item function, this item's sums are written after it)
    if (FORMS == 2) {
      stream_item_s14<XP, DEPTH_S>(m, xs, part, row0, nrows, 0x00F0000Fu, 0x54006400u, nthreads);
      lds_barrier();
      // a thread per row: the quarter sums of its row pairwise, then the tiles of the row in ascending
      // order - the order of the single-matrix kernel
      const int rpt_shift = m.mr_shift >= 0 ? 6 - m.mr_shift : 0;
      for (int t = (int)threadIdx.x; t < nrows; t += nthreads) {
        const int r = row0 + t;
        const uint32_t rp = *(global_u32 *)(m.row_ptr + r);
        const float *p = part + 4 * m.phases * (t >> rpt_shift);
        const int sub = t & ((1 << rpt_shift) - 1);
        float v = 0.f;
        if (rpt_shift == 2) v = p[sub];
        else if (rpt_shift == 1) v = p[2 * sub] + p[2 * sub + 1];
        else for (int ph = 0; ph < m.phases; ++ph) v += (p[4 * ph] + p[4 * ph + 1]) + (p[4 * ph + 2] + p[4 * ph + 3]);
        const bool ok = rp == (uint32_t)r * (uint32_t)(m.nchunks * 32);
        *(global_u16 *)(m.y + r) = ok ? __half_as_ushort(__float2half(v)) : (uint16_t)0x7E00;
      }
      continue;
    }
    if (sparse) stream_item_s24<XP, DEPTH_S>(m, xs, part, row0, nrows, 0x00F0000Fu, 0x54006400u, nthreads);
    else stream_item_dense<XP, DEPTH_D>(m, xs, part, row0, nrows, 0x00F000F0u, 0x54005400u, nthreads);
    lds_barrier();
    // a thread per row adds the partial sums in the order of the single-matrix kernels: the
    // four quarter sums of a tile pairwise, then the tiles of the row in ascending order
    for (int t = (int)threadIdx.x; t < nrows; t += nthreads) {
      const int r = row0 + t;
      uint32_t rp = 0;
      if (sparse) rp = *(global_u32 *)(m.row_ptr + r);
      const float *p = part + 4 * m.phases * t;
      float v = 0.f;
      for (int ph = 0; ph < m.phases; ++ph) v += (p[4 * ph] + p[4 * ph + 1]) + (p[4 * ph + 2] + p[4 * ph + 3]);
      bool ok = true;
      if (sparse) ok = rp == (uint32_t)r * (uint32_t)(m.nchunks * 32);
      *(global_u16 *)(m.y + r) = ok ? __half_as_ushort(__float2half(v)) : (uint16_t)0x7E00;
    }
  }
}

}  // namespace egt
#endif
