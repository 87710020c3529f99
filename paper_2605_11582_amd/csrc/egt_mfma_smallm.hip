// Small-M SparseGemm (2 <= M <= 64 activation rows) on the gfx950 sparse matrix
// cores: the parallel-verification form of the product, Y[m][r] = sum_k W[r][k] X[m][k].
//
// Mapping.  The 16 rows of the A operand of v_smfmac_f32_16x16x64_f16 are 16 matrix
// rows (a row tile) and the 16 columns of B are 16 activation rows (a token group), so
// all 256 outputs of an instruction are used.  K is walked in steps of 256 dense
// columns.  In a step, lane (i, kb) = i + 16 kb holds chunk kb of row i (a chunk is 64
// dense columns = 16 B of nibbles + 8 B of idx words); its four dwords feed four
// instructions.  Instruction d therefore sees, as its k-range [16 kb, 16 kb + 16), the
// dense columns 64 kb + 16 d .. + 15 of the step: any fixed permutation of k is fine
// as long as B follows it, and B is read from LDS with exactly that permutation.
#include "egt_mfma_common.h"

#include <cstdio>
#include <cstdlib>

namespace egt {

__device__ __forceinline__ u4 dequant8_sm(uint32_t d, uint32_t off, uint32_t s2, uint32_t mask, uint32_t magic) {
  u4 r;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t t = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)p * 0x00010001u);
    r[p] = pk_mul_f16(pk_sub_f16(and_or(t, mask, magic), off), s2);
  }
  return r;
}

// The waves of a workgroup split K between them: in phase p, wave w
// owns K-step p * waves + w (256 dense columns) of every row tile of the workgroup
// (at most NIT of them, 16 rows each) and keeps its 16 x 16 sums in registers over
// the phases.  Its slice of X (16 tokens x 256 columns per token group) is fetched
// with fully coalesced loads and turned into the B operand layout through a private
// LDS region (token rows padded against bank conflicts; no workgroup barrier).
// A operand, INT4: lane 4 r + c fetches chunk c of row r of the step, so that four
// neighbouring lanes read 64 contiguous bytes, and a lane permutation (ds_bpermute)
// hands the chunk to lane (i, kb) = (r, c) of the matrix instruction.  FP16 values
// are fetched by lane (i, kb) directly (64 B per lane).
// The loads of phase p + 1 (A and the first token group of X) are requested while
// phase p is computed.  Loads return in the order of their requests, so a request
// for X that follows a request for A waits for A: with NT = 2 token groups the second
// group of a phase is requested before the A tiles of the next phase and nothing
// needed soon queues behind the long latency of A.  More than 16 NT tokens are
// handled in passes over the same rows (the weights of the later passes come from
// the caches).  After the last phase the waves leave their sums in LDS, one barrier
// later 4-lane groups add them up over the waves in wave order (a fixed order: the
// result does not depend on timing) and store four consecutive rows of a token.
struct SmallMKsGeom {
  int rows, M;
  int nchunks;         // cols / 64
  int nsteps;          // cols / 256
  int ntiles;          // ceil(rows / 16)
  int gshift;
  int groups_per_row;
  int vec_store;       // Y and ldy allow 8-byte stores of four rows
  uint32_t val_bytes, idx_bytes, qp_bytes, x_bytes;   // extents of the arrays
  int64_t ldx, ldy;
  uint32_t nib_mask, nib_magic;
};

template <int KIND, int QW>
struct ATile {                        // A operand of one row tile, one K-step
  u4 nib[KIND == EGT_VAL_INT4 ? 1 : 4];
  u2 iw;
  uint32_t qp[QW];                    // {scale, zero} of the chunk; two for groups of 32 columns
};

constexpr int KS_PAIR = 1024 + 32;                 // LDS bytes of a pair of tokens
constexpr int KS_REGION = 8 * KS_PAIR;             // LDS bytes per wave for X

__device__ __forceinline__ uint32_t lane_perm(int byte_addr, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_ds_bpermute(byte_addr, (int)v);
}
// Buffer resource over `bytes` bytes at p: loads through it take a 32-bit lane offset
// plus a 32-bit wave-uniform offset (scalar registers, scalar arithmetic) and return
// zero past the end instead of faulting.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
// Explicit waits around the loads that write LDS directly: they count as vector-memory
// operations, return in request order with the register loads, and nothing else tells a
// following LDS read that their data has landed (or a following load of that kind that
// the reads of the data it replaces are done).  The statements also keep the compiler
// from moving memory operations across them.
template <int N>
__device__ __forceinline__ void wait_vmem() {       // at most N vector-memory operations still pending
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wait_lds() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}
template <int N>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {     // value of lane N of the 4-lane group
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, N * 0x55, 0xf, 0xf, true);
}

template <int KIND, int NT, int NIT, int NWMAX, int QW>
__global__ __launch_bounds__(64 * NWMAX) void k_sparse_smallm_ks(const uint32_t *__restrict__ row_ptr,
                                                                  const uint8_t *__restrict__ values,
                                                                  const uint8_t *__restrict__ idx,
                                                                  const uint8_t *__restrict__ qparams,
                                                                  const __half *__restrict__ X,
                                                                  __half *__restrict__ Y,
                                                                  const SmallMKsGeom g) {
  extern __shared__ __align__(16) uint8_t xs[];       // X regions, later the partial sums
  constexpr bool INT4 = KIND == EGT_VAL_INT4;
  constexpr int VW = INT4 ? 1 : 4;
  constexpr bool HOLD = NT > 1;                       // A operands of a phase are kept for all token groups
  constexpr int PART = NIT * NT * 1024;               // bytes of partial sums per wave
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int i = lane & 15, kb = lane >> 4;
  const int li = INT4 ? (lane >> 2) : i, lc = INT4 ? (lane & 3) : kb;   // row, chunk this lane fetches
  const int from = 4 * (4 * i + kb);                  // lane that fetched the chunk of lane (i, kb), as a byte address
  const int nit = (g.ntiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;   // <= NIT
  const int phases = (g.nsteps + nw - 1) / nw;
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
  uint8_t *region = xs + wave * KS_REGION;
  const int ngroups = (g.M + 15) >> 4;
  // Row pointers of the workgroup's rows are requested first and checked at the end
  // (flags in LDS behind the regions): a row whose pointer is not r * S yields NaN.
  uint32_t *flags = (uint32_t *)(xs + nw * (KS_REGION > PART ? KS_REGION : PART));
  const int frow = 16 * ((int)blockIdx.x + (int)(threadIdx.x >> 4) * (int)gridDim.x) + (int)(threadIdx.x & 15);
  const bool fcheck = (int)threadIdx.x < 16 * nit && frow < g.rows;
  const uint32_t frp = fcheck ? row_ptr[frow] : 0u;

  const __amdgpu_buffer_rsrc_t r_val = make_rsrc(values, g.val_bytes), r_idx = make_rsrc(idx, g.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = make_rsrc(qparams, g.qp_bytes), r_x = make_rsrc(X, g.x_bytes);
  auto load_a = [&](ATile<KIND, QW> &a, int it, int step) {
    const int rt = (int)blockIdx.x + min(it, nit - 1) * (int)gridDim.x;       // a tile past the end repeats the last one
    const int s = min(step, g.nsteps - 1);
    const uint32_t rel = (uint32_t)min(li, g.rows - 1 - 16 * rt);            // row inside the tile (clamped)
    const uint32_t cl = rel * (uint32_t)g.nchunks + (uint32_t)lc;             // lane part of the chunk number
    const uint32_t cu = (uint32_t)(16 * rt) * (uint32_t)g.nchunks + (uint32_t)(4 * s);   // uniform part
    a.iw = __builtin_amdgcn_raw_buffer_load_b64(r_idx, 8u * cl, 8u * cu, 0);
    a.qp[0] = 0;
    if (INT4) {
      a.nib[0] = __builtin_amdgcn_raw_buffer_load_b128(r_val, 16u * cl, 16u * cu, 0);
      if (QW == 2) {                                  // groups 8 s + 2 lc and the next one
        const uint32_t qu = (uint32_t)(16 * rt) * (uint32_t)g.groups_per_row + (uint32_t)(8 * s);
        const u2 v = __builtin_amdgcn_raw_buffer_load_b64(
            r_qp, 4u * (rel * (uint32_t)g.groups_per_row + 2u * (uint32_t)lc), 4u * qu, 0);
        a.qp[0] = v[0];
        a.qp[QW - 1] = v[1];
      } else {
        const uint32_t qu = (uint32_t)(16 * rt) * (uint32_t)g.groups_per_row + (uint32_t)((4 * s) >> g.gshift);
        a.qp[0] = __builtin_amdgcn_raw_buffer_load_b32(
            r_qp, 4u * (rel * (uint32_t)g.groups_per_row + (uint32_t)(lc >> g.gshift)), 4u * qu, 0);
      }
    } else {
#pragma unroll
      for (int k = 0; k < VW; ++k)
        a.nib[k] = __builtin_amdgcn_raw_buffer_load_b128(r_val, 64u * cl + 16u * k, 64u * cu, 0);
    }
  };
  // fetched form -> operand form: lane (i, kb) takes what lane 4 i + kb fetched
  auto to_operand = [&](ATile<KIND, QW> &a) {
    if (INT4) {
#pragma unroll
      for (int d = 0; d < 4; ++d) a.nib[0][d] = lane_perm(from, a.nib[0][d]);
      a.iw[0] = lane_perm(from, a.iw[0]);
      a.iw[1] = lane_perm(from, a.iw[1]);
#pragma unroll
      for (int k = 0; k < QW; ++k) a.qp[k] = lane_perm(from, a.qp[k]);
    }
  };
  // This wave's slice of X for token group j (16 tokens x 512 B) goes from global memory
  // straight into its LDS region, no registers in between: instruction u covers tokens
  // 2 u and 2 u + 1, lane l delivers to byte 16 l of the kilobyte at 1056 u.  The odd token
  // of a pair has neighbouring 16-byte pieces swapped (piece q at slot q ^ 1) and pairs are
  // 32 B apart modulo the bank cycle, so the sixteen lanes of a B read (one token each, same
  // piece) fall into different banks.
  // Pairs of tokens past M are not fetched and the odd token past an odd M repeats token
  // M - 1: whatever LDS holds there only reaches columns of the products that are never
  // stored.
  const int xtl = lane >> 5;
  const uint32_t xoff_lo = 16u * (uint32_t)((lane & 31) ^ xtl);               // both halves read the same token
  const uint32_t xoff_hi = xoff_lo + (uint32_t)xtl * (uint32_t)(2 * g.ldx);
  auto dma_x = [&](int j, int step) {
    const uint32_t xs0 = 512u * (uint32_t)min(step, g.nsteps - 1);
    asm volatile("" ::: "memory");                    // the eight requests stay together, in program order
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int t0 = 16 * j + 2 * u;
      if (t0 < g.M)                                   // uniform
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(region + KS_PAIR * u),
                                                 16, t0 + 1 < g.M ? xoff_hi : xoff_lo,
                                                 xs0 + (uint32_t)t0 * (uint32_t)(2 * g.ldx), 0, 0);
    }
    asm volatile("" ::: "memory");
  };
  // B operand: lane (n, b) holds token n, k-octets b and 4 + b of each 16-column group d,
  // i.e. piece q = 16 h + 8 (b >> 1) + 2 d + (b & 1) for h = 0, 1
  auto read_b = [&](u8v (&bx)[4]) {
    const int n = lane & 15, b = lane >> 4;
    const uint8_t *base0 = region + KS_PAIR * (n >> 1) + 512 * (n & 1) + 16 * (8 * (b >> 1) + ((b ^ n) & 1));
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        const u4 v = *(const u4 *)(base0 + 256 * h + 32 * d);
#pragma unroll
        for (int k = 0; k < 4; ++k) bx[d][4 * h + k] = v[k];
      }
    }
  };
  auto dequant = [&](const ATile<KIND, QW> &t, u4 (&av)[4]) {
    uint32_t s2[QW], off[QW];
#pragma unroll
    for (int k = 0; k < QW; ++k) {
      s2[k] = off[k] = 0;
      if (INT4) {
        s2[k] = __builtin_amdgcn_perm(t.qp[k], t.qp[k], 0x01000100u);
        off[k] = pk_add_f16(__builtin_amdgcn_perm(t.qp[k], t.qp[k], 0x03020302u), g.nib_magic);
      }
    }
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      if (INT4) av[d] = dequant8_sm(t.nib[0][d], off[d * QW / 4], s2[d * QW / 4], g.nib_mask, magic);
      else av[d] = t.nib[d];
    }
  };
  auto mfma4 = [&](const u4 (&av)[4], const u2 iw, const u8v (&bx)[4], f4 &acc) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const int iword = d < 2 ? (int)iw[0] : (int)iw[1];
      if (d & 1)
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[d]), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 1);
      else
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[d]), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 0);
    }
  };

  for (int j0 = 0; j0 < ngroups; j0 += NT) {          // passes of NT token groups
    ATile<KIND, QW> raw[NIT];
    f4 acc[NIT][NT];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
      for (int jj = 0; jj < NT; ++jj) acc[it][jj] = f4{0.f, 0.f, 0.f, 0.f};
    dma_x(j0, wave);
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_a(raw[it], it, wave);

    // A wave whose last step lies past K (K-steps not a multiple of the waves) skips
    // that phase; it is the last one, nothing is requested in it.
    for (int p = 0; p < phases && p * nw + wave < g.nsteps; ++p) {
      const int step = p * nw + wave;
      const bool more = p + 1 < phases;
      constexpr int NA = NIT * (INT4 ? 3 : 5);         // loads of the A tiles of one phase (any QW)
      u8v bx[4];
      ATile<KIND, QW> t[NIT];
      wait_vmem<0>();                                 // X and the A tiles of this phase have arrived
      read_b(bx);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        t[it] = raw[it];
        to_operand(t[it]);
      }
      wait_lds();                                     // the region and the fetch registers are free again
      if (HOLD) {
        // requests, in this order: X of the second token group, then the A tiles of the
        // next phase; X of the next phase follows after the second group has been read
        if (j0 + 1 < ngroups) dma_x(j0 + 1, step);
        else if (more) dma_x(j0, step + nw);
        if (more) {
#pragma unroll
          for (int it = 0; it < NIT; ++it) load_a(raw[it], it, step + nw);
        }
        u4 held[NIT][4];
#pragma unroll
        for (int it = 0; it < NIT; ++it) dequant(t[it], held[it]);
#pragma unroll
        for (int jj = 0; jj < NT; ++jj) {
          if (j0 + jj < ngroups) {                    // uniform
            if (jj > 0) {
              if (more) wait_vmem<NA>(); else wait_vmem<0>();
              read_b(bx);
              wait_lds();
              if (jj + 1 < NT && j0 + jj + 1 < ngroups) dma_x(j0 + jj + 1, step);
              else if (more) dma_x(j0, step + nw);
            }
#pragma unroll
            for (int it = 0; it < NIT; ++it)
              if (it < nit) mfma4(held[it], t[it].iw, bx, acc[it][jj]);
          }
        }
      } else {
        if (more) dma_x(j0, step + nw);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          if (it < nit) {
            u4 av[4];
            dequant(t[it], av);
            mfma4(av, t[it].iw, bx, acc[it][0]);
          }
          if (more) load_a(raw[it], it, step + nw);  // into the registers this tile has just left
        }
      }
    }
    wait_vmem<0>();                                   // a wave that left early may still have X on its way

    // ---- partial sums to LDS: tile (it, jj) of wave w at w * PART + (it * NT + jj) * 1024,
    //      float 4 * lane + v = D[row 4 (lane >> 4) + v][token lane & 15]
    __syncthreads();                                  // every wave is done with its X region
    if (threadIdx.x < 16 * NIT) flags[threadIdx.x] = (fcheck && frp == (uint32_t)frow * S_row) ? 1u : 0u;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
      for (int jj = 0; jj < NT; ++jj)
        if (it < nit) *(f4 *)(xs + wave * PART + (it * NT + jj) * 1024 + 16 * lane) = acc[it][jj];
    __syncthreads();
    for (int unit = threadIdx.x; unit < NIT * NT * 256; unit += (int)blockDim.x) {
      const int tj = unit >> 8, it = tj / NT, jj = tj % NT;
      if (it >= nit || j0 + jj >= ngroups) continue;  // uniform over a wave
      const int v = unit & 3, sl = (unit >> 2) & 63;  // register v of lane sl of the tile
      const float *src = (const float *)xs + unit;
      float part[NWMAX];
#pragma unroll
      for (int w = 0; w < NWMAX; ++w) part[w] = src[min(w, nw - 1) * (PART / 4)];
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NWMAX; ++w) sum += w < nw ? part[w] : 0.f;
      const int row0 = 16 * ((int)blockIdx.x + it * (int)gridDim.x) + 4 * (sl >> 4);
      const int row = row0 + v;
      const int tok = 16 * (j0 + jj) + (sl & 15);
      uint32_t hv = 0x7E00u;
      if (flags[16 * it + 4 * (sl >> 4) + v]) hv = __half_as_ushort(__float2half(sum));
      const uint32_t h1 = quad_bcast<1>(hv), h2 = quad_bcast<2>(hv), h3 = quad_bcast<3>(hv);
      if (tok < g.M) {
        __half *dst = Y + (int64_t)tok * g.ldy + row;
        if (g.vec_store && row0 + 3 < g.rows) {
          if (v == 0) *(u2 *)dst = u2{hv | (h1 << 16), h2 | (h3 << 16)};
        } else if (row < g.rows) {
          *dst = __ushort_as_half((uint16_t)hv);
        }
      }
    }
    __syncthreads();                                  // the next pass writes X regions again
  }
}

// Shapes covered: 2:4, K a multiple of 256, INT4 groups of 32 << j.
bool sparse_smallm_supported(const egt_2bitcsr &w) {
  if (w.n_keep != 2 || w.cols % 256 != 0 || w.cols < 256) return false;
  if (w.val_kind == EGT_VAL_INT4) {
    const int gm = w.group_size / 32;
    if (w.group_size % 32 != 0 || (gm & (gm - 1)) != 0) return false;
  }
  return true;
}

template <int KIND, int NT, int NIT, int NWMAX, int QW = 1>
static hipError_t go_ks(const egt_2bitcsr &w, const uint16_t *X, uint16_t *Y, const SmallMKsGeom &g, int nw,
                        int nblocks, hipStream_t stream) {
  const size_t x_bytes = (size_t)nw * KS_REGION, p_bytes = (size_t)nw * NIT * NT * 1024;
  const size_t lds = (x_bytes > p_bytes ? x_bytes : p_bytes) + 64 * NIT;   // + row-pointer flags
  return launch(k_sparse_smallm_ks<KIND, NT, NIT, NWMAX, QW>, dim3(nblocks), dim3(64 * nw), lds, stream, w.row_ptr,
                (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams,
                (const __half *)X, (__half *)Y, g);
}

hipError_t launch_sparse_smallm(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                int64_t ldy, int M, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  const bool int4 = w.val_kind == EGT_VAL_INT4;
  SmallMKsGeom g;
  g.rows = w.rows; g.M = M;
  g.nchunks = w.cols / 64;
  g.nsteps = w.cols / 256;
  g.ntiles = (w.rows + 15) / 16;
  g.gshift = 0; g.groups_per_row = 0;
  if (int4) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.ldx = ldx; g.ldy = ldy;
  g.vec_store = ((uintptr_t)Y % 8 == 0 && ldy % 4 == 0) ? 1 : 0;
  const uint64_t chunks = (uint64_t)w.rows * g.nchunks;
  const uint64_t vb = chunks * (int4 ? 16 : 64), xb = ((uint64_t)(M - 1) * ldx + w.cols) * 2;
  if (vb >= (1ull << 32) || xb >= (1ull << 32)) return hipErrorInvalidValue;   // 32-bit offsets
  g.val_bytes = (uint32_t)vb; g.idx_bytes = (uint32_t)(chunks * 8);
  g.qp_bytes = (uint32_t)((uint64_t)w.rows * g.groups_per_row * 4); g.x_bytes = (uint32_t)xb;
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
  // One workgroup per compute unit while its row tiles fit the registers (NIT of them);
  // up to 16 tokens with 16 waves of 128 registers, more with 8 waves of 256.
  const bool wide = M > 16 || !int4;                  // 8 waves, two token groups per pass
  const int nit_max = wide ? 4 : 3;
  int nwmax = wide ? 8 : 16, blocks_per_cu = 1;
  if (const char *e = getenv("EGT_SM_TUNE")) sscanf(e, "%d,%d", &nwmax, &blocks_per_cu);
  if (nwmax < 1 || nwmax > (wide ? 8 : 16)) return hipErrorInvalidValue;
  const int nw = g.nsteps < nwmax ? g.nsteps : nwmax;
  int nblocks = 256 * blocks_per_cu;
  if (nblocks * nit_max < g.ntiles) nblocks = (g.ntiles + nit_max - 1) / nit_max;
  if (nblocks > g.ntiles) nblocks = g.ntiles;
  const bool one = nblocks == g.ntiles;               // one row tile per workgroup
  if (int4 && w.group_size == 32) {
    if (!wide) return one ? go_ks<EGT_VAL_INT4, 1, 1, 16, 2>(w, X, Y, g, nw, nblocks, stream)
                          : go_ks<EGT_VAL_INT4, 1, 3, 16, 2>(w, X, Y, g, nw, nblocks, stream);
    return one ? go_ks<EGT_VAL_INT4, 2, 1, 8, 2>(w, X, Y, g, nw, nblocks, stream)
               : go_ks<EGT_VAL_INT4, 2, 4, 8, 2>(w, X, Y, g, nw, nblocks, stream);
  }
  if (int4) {
    if (!wide) return one ? go_ks<EGT_VAL_INT4, 1, 1, 16>(w, X, Y, g, nw, nblocks, stream)
                          : go_ks<EGT_VAL_INT4, 1, 3, 16>(w, X, Y, g, nw, nblocks, stream);
    return one ? go_ks<EGT_VAL_INT4, 2, 1, 8>(w, X, Y, g, nw, nblocks, stream)
               : go_ks<EGT_VAL_INT4, 2, 4, 8>(w, X, Y, g, nw, nblocks, stream);
  }
  if (M <= 16) return one ? go_ks<EGT_VAL_FP16, 1, 1, 8>(w, X, Y, g, nw, nblocks, stream)
                          : go_ks<EGT_VAL_FP16, 1, 4, 8>(w, X, Y, g, nw, nblocks, stream);
  return one ? go_ks<EGT_VAL_FP16, 2, 1, 8>(w, X, Y, g, nw, nblocks, stream)
             : go_ks<EGT_VAL_FP16, 2, 4, 8>(w, X, Y, g, nw, nblocks, stream);
}

}  // namespace egt
