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
#include "egt_device.h"

namespace egt {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ uint32_t pk_add_f16(uint32_t a, uint32_t b) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, a) + __builtin_bit_cast(h2, b));
}
__device__ __forceinline__ uint32_t pk_mul_f16(uint32_t a, uint32_t b) {
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, a) * __builtin_bit_cast(h2, b));
}

// Eight INT4 codes of one dword (slot k in bits 4k..4k+3) -> four half2 registers
// {slot 2p, slot 2p+1} holding s*(q - z).  Byte p of the dword carries the pair:
// the low nibble becomes the mantissa of 1024 + q, the high nibble (left in
// place) the mantissa of 64 + q; one packed add removes both offsets and z
// exactly, one packed multiply applies the scale (a single rounding to FP16).
__device__ __forceinline__ u4 dequant8(uint32_t d, uint32_t neg_off, uint32_t s2) {
  u4 r;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t t = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)p * 0x00010001u);
    const uint32_t h = (t & 0x00F0000Fu) | 0x54006400u;
    r[p] = pk_mul_f16(pk_add_f16(h, neg_off), s2);
  }
  return r;
}

// Geometry of a launch, computed on the host.
struct M1Geom {
  int rows, cols;
  int nchunks;        // cols / 64
  int rows_per_tile;  // 1, or 64 / nchunks when a row is shorter than a tile
  int phases;         // tiles per row (1 when rows_per_tile >= 1 covers the row)
  int ntile_rows;     // ceil(rows / rows_per_tile): tiles per phase
  int tiles_per_wave;
  int group;          // INT4 group size (multiple of 64), 0 for FP16 values
};

// TPI tiles are loaded together before any of them is consumed.
template <int KIND, int TPI>
__global__ __launch_bounds__(256) void k_sparse_m1(const uint32_t *__restrict__ row_ptr,
                                                    const uint8_t *__restrict__ values,
                                                    const uint8_t *__restrict__ idx,
                                                    const uint16_t *__restrict__ qparams,
                                                    const __half *__restrict__ x,
                                                    __half *__restrict__ y, const M1Geom g) {
  extern __shared__ float part[];                     // [phases][waves-per-phase * tiles_per_wave]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  const int wpp = nwaves / g.phases;                  // waves per phase in this block
  const int phase = wave / wpp;
  const int wslot = wave % wpp;
  const int i = lane & 15, kb = lane >> 4;
  const int cit = 4 * i + kb;                         // chunk of this lane inside a tile

  // ---- B operand: activations for column n = lane & 15, k-octets (lane >> 4) and 4 + (lane >> 4)
  u8v bx[4];
  {
    const int n = lane & 15, b = lane >> 4;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int kba = (4 * h + b) >> 1, sub = b & 1;  // the A lane (n, kba) this octet multiplies
      int c = 4 * n + kba;                             // its chunk inside the tile
      c = g.rows_per_tile > 1 ? c % g.nchunks : c + 64 * phase;
      const bool ok = c < g.nchunks;
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        u4 v = {0, 0, 0, 0};
        if (ok) v = *(const u4 *)(x + 64 * c + 16 * d + 8 * sub);
        bx[d][4 * h + 0] = v[0]; bx[d][4 * h + 1] = v[1];
        bx[d][4 * h + 2] = v[2]; bx[d][4 * h + 3] = v[3];
      }
    }
  }

  const int S_row = g.cols >> 1;                      // slots per row (2:4)
  const int tile0 = (blockIdx.x * wpp + wslot) * g.tiles_per_wave;
  for (int tb = 0; tb < g.tiles_per_wave; tb += TPI) {
    u4 nib[TPI][KIND == EGT_VAL_INT4 ? 1 : 4];
    uint2 iw[TPI];
    uint32_t qp[TPI];
    bool act[TPI];
    // ---- issue every load of TPI tiles
#pragma unroll
    for (int t = 0; t < TPI; ++t) {
      const int tr = tile0 + tb + t;                  // tile row index
      int r, c;                                       // matrix row and chunk-in-row of this lane
      if (g.rows_per_tile > 1) { r = tr * g.rows_per_tile + cit / g.nchunks; c = cit % g.nchunks; }
      else { r = tr; c = cit + 64 * phase; }
      act[t] = tr < g.ntile_rows && r < g.rows && c < g.nchunks;
      iw[t] = make_uint2(0u, 0u);
      qp[t] = 0;
#pragma unroll
      for (int k = 0; k < (KIND == EGT_VAL_INT4 ? 1 : 4); ++k) nib[t][k] = u4{0, 0, 0, 0};
      if (act[t]) {
        const size_t chunk = (size_t)r * g.nchunks + c;            // global chunk id
        iw[t] = *(const uint2 *)(idx + 8 * chunk);
        if (KIND == EGT_VAL_INT4) {
          nib[t][0] = *(const u4 *)(values + 16 * chunk);
          qp[t] = *(const uint32_t *)(qparams + 2 * ((size_t)r * (g.cols / g.group) + (64 * c) / g.group));
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) nib[t][k] = *(const u4 *)(values + 64 * chunk + 16 * k);
        }
      }
    }
    // ---- consume them
#pragma unroll
    for (int t = 0; t < TPI; ++t) {
      f4 acc = {0.f, 0.f, 0.f, 0.f};
      uint32_t s2 = 0, neg_off = 0;
      if (KIND == EGT_VAL_INT4) {
        s2 = __builtin_amdgcn_perm(qp[t], qp[t], 0x01000100u);               // {s, s}
        const uint32_t z2 = __builtin_amdgcn_perm(qp[t], qp[t], 0x03020302u); // {z, z}
        neg_off = pk_add_f16(z2, 0x54006400u) ^ 0x80008000u;                  // -{1024 + z, 64 + z}
      }
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        u4 a;
        if (KIND == EGT_VAL_INT4) a = dequant8(nib[t][0][d], neg_off, s2);
        else a = nib[t][d];
        const int iword = d < 2 ? (int)iw[t].x : (int)iw[t].y;
        if (d & 1)
          acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 1);
        else
          acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 0);
      }
      // D[q][q] of quad q sits in lane q + 16 (q / 4), register q % 4
      float cand = (lane & 2) ? ((lane & 1) ? acc[3] : acc[2]) : ((lane & 1) ? acc[1] : acc[0]);
      float v = __shfl(cand, (lane & 15) + 16 * ((lane & 15) >> 2), 64);     // lane l: quad l % 16
      // sum the quads of one row: 16 / rows_per_tile consecutive quads
      const int qpr = 16 / g.rows_per_tile;
      for (int o = 1; o < qpr; o <<= 1) v += __shfl_xor(v, o, 64);
      const int tr = tile0 + tb + t;
      if (tr < g.ntile_rows && lane < 16 && (lane % qpr) == 0) {
        const int r = tr * g.rows_per_tile + lane / qpr;
        if (r < g.rows) {
          if (g.phases == 1) {
            const bool ok = row_ptr[r] == (uint32_t)r * (uint32_t)S_row;
            y[r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
          } else {
            part[phase * (wpp * g.tiles_per_wave) + wslot * g.tiles_per_wave + tb + t] = v;
          }
        }
      }
    }
  }
  if (g.phases > 1) {
    __syncthreads();
    const int per = wpp * g.tiles_per_wave;           // rows handled by this block
    for (int j = threadIdx.x; j < per; j += blockDim.x) {
      const int r = blockIdx.x * per + j;
      if (r < g.rows) {
        float v = 0.f;
        for (int p = 0; p < g.phases; ++p) v += part[p * per + j];
        const bool ok = row_ptr[r] == (uint32_t)r * (uint32_t)S_row;
        y[r] = ok ? __float2half(v) : __ushort_as_half((uint16_t)0x7E00);
      }
    }
  }
}

// Shapes the diagonal kernel covers: 2:4, K a multiple of 256 that either divides
// 4096 or is at least 4096 (at most 16 tiles per row), INT4 groups of a multiple of 64.
bool sparse_m1_supported(const egt_2bitcsr &w) {
  if (w.n_keep != 2 || w.cols % 256 != 0) return false;
  if (w.cols < 4096 && 4096 % w.cols != 0) return false;
  if (w.cols > 16 * 4096) return false;
  if (w.val_kind == EGT_VAL_INT4 && w.group_size % 64 != 0) return false;
  return true;
}

hipError_t launch_sparse_m1(const egt_2bitcsr &w, const uint16_t *x, uint16_t *y, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  M1Geom g;
  g.rows = w.rows; g.cols = w.cols; g.nchunks = w.cols / 64;
  g.rows_per_tile = g.nchunks >= 64 ? 1 : 64 / g.nchunks;
  g.phases = g.nchunks >= 64 ? (g.nchunks + 63) / 64 : 1;
  g.ntile_rows = (w.rows + g.rows_per_tile - 1) / g.rows_per_tile;
  g.group = w.group_size;
  constexpr int TPI = 4;
  g.tiles_per_wave = TPI;
  const int wpp = g.phases == 1 ? 4 : (g.phases <= 2 ? 2 : 1);   // waves per phase in a block
  const int nwaves = wpp * g.phases;
  const int tiles_per_block = wpp * g.tiles_per_wave;
  const dim3 grid((g.ntile_rows + tiles_per_block - 1) / tiles_per_block), block(64 * nwaves);
  const size_t lds = g.phases > 1 ? sizeof(float) * g.phases * tiles_per_block : 0;
  if (w.val_kind == EGT_VAL_INT4)
    return launch(k_sparse_m1<EGT_VAL_INT4, TPI>, grid, block, lds, stream, w.row_ptr,
                  (const uint8_t *)w.values, (const uint8_t *)w.idx, w.qparams, (const __half *)x,
                  (__half *)y, g);
  return launch(k_sparse_m1<EGT_VAL_FP16, TPI>, grid, block, lds, stream, w.row_ptr,
                (const uint8_t *)w.values, (const uint8_t *)w.idx, w.qparams, (const __half *)x,
                (__half *)y, g);
}

}  // namespace egt
