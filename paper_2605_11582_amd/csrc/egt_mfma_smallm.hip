// Small-M SparseGemm (2 <= M <= 64 activation rows) on the gfx950 sparse matrix
// cores: the parallel-verification form of the product, Y[m][r] = sum_k W[r][k] X[m][k].
//
// Mapping.  Here the 16 rows of the A operand of v_smfmac_f32_16x16x64_f16 are 16
// matrix rows and the 16 columns of B are 16 activation rows (tokens), so all 256
// outputs of an instruction are used.  A wave owns one row tile (16 rows) and
// walks K in steps of 256 dense columns.  In a step, lane (i, kb) = i + 16 kb loads
// the chunk (64 dense columns = 16 B of nibbles + 8 B of idx words) number kb of
// row i; its four dwords feed four instructions.  Instruction d therefore sees,
// as its k-range [16 kb, 16 kb + 16), the dense columns 64 kb + 16 d .. + 15 of the
// step - any fixed permutation of k is fine as long as B follows it, and B is
// read from LDS with exactly that permutation.
// The activations of a step (M tokens x 256 columns) are staged in LDS once per
// workgroup and shared by its waves; token rows are padded by 16 B so that the
// 16 lanes of a B read, one token each, fall into different banks.
// The dequantised A registers of a step are reused for every group of 16 tokens.
#include "egt_mfma_common.h"

#include <cstdio>
#include <cstdlib>

namespace egt {

// Here a wave-wide load touches 16 rows x 64 B, i.e. half cache lines whose other half
// is read by a neighbouring wave a moment later: ordinary (cached) loads, not
// streaming ones, or the line is dropped and fetched twice.
template <typename T>
__device__ __forceinline__ T ld_plain(const void *p) {
  return *(const T *)p;
}

__device__ __forceinline__ u4 dequant8_sm(uint32_t d, uint32_t off, uint32_t s2, uint32_t mask, uint32_t magic) {
  u4 r;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t t = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)p * 0x00010001u);
    r[p] = pk_mul_f16(pk_sub_f16(and_or(t, mask, magic), off), s2);
  }
  return r;
}

struct SmallMGeom {
  int rows, M;
  int nchunks;         // cols / 64
  int nsteps;          // cols / 256
  int gshift;          // INT4 group = 64 << gshift
  int groups_per_row;
  int64_t ldx, ldy;
  uint32_t nib_mask, nib_magic;
};

constexpr int TOKEN_STRIDE = 528;     // 256 halfs + 16 B pad

// NT = groups of 16 tokens, PF = K-steps of A kept in flight, XPT = 16 B pieces of X
// each thread stages per step.
template <int KIND, int NT, int PF, int XPT>
__global__ __launch_bounds__(256) void k_sparse_smallm(const uint32_t *__restrict__ row_ptr,
                                                        const uint8_t *__restrict__ values,
                                                        const uint8_t *__restrict__ idx,
                                                        const uint8_t *__restrict__ qparams,
                                                        const __half *__restrict__ X,
                                                        __half *__restrict__ Y, const SmallMGeom g) {
  extern __shared__ __align__(16) uint8_t xs[];       // two buffers of 16 NT tokens
  constexpr int VW = KIND == EGT_VAL_INT4 ? 1 : 4;    // dwordx4 loads of values per chunk
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nthreads = blockDim.x;
  const int i = lane & 15, kb = lane >> 4;
  const int r0 = (blockIdx.x * (nthreads >> 6) + wave) * 16;
  const int r_ld = min(r0 + i, g.rows - 1);           // row this lane loads (clamped)
  const uint32_t row_chunk0 = (uint32_t)r_ld * (uint32_t)g.nchunks;
  const int buf_bytes = 16 * NT * TOKEN_STRIDE;

  // row pointers of the four rows this lane will store
  uint32_t rp[4];
#pragma unroll
  for (int v = 0; v < 4; ++v) rp[v] = row_ptr[min(r0 + 4 * kb + v, g.rows - 1)];

  // ---- staging of X: linear piece index e -> (token, piece)
  u4 xr[XPT];
  auto load_x = [&](int step) {
    const int s = min(step, g.nsteps - 1);
#pragma unroll
    for (int j = 0; j < XPT; ++j) {
      const int e = threadIdx.x + j * nthreads;
      const int tok = min(e >> 5, g.M - 1), piece = e & 31;
      xr[j] = *(const u4 *)(X + (int64_t)tok * g.ldx + 256 * s + 8 * piece);
    }
  };
  auto store_x = [&](int step) {
    uint8_t *buf = xs + (step & 1) * buf_bytes;
#pragma unroll
    for (int j = 0; j < XPT; ++j) {
      const int e = threadIdx.x + j * nthreads;
      const int tok = e >> 5, piece = e & 31;
      if (tok < 16 * NT) {
        u4 v = xr[j];
        if (tok >= g.M) v = u4{0, 0, 0, 0};
        *(u4 *)(buf + tok * TOKEN_STRIDE + 16 * piece) = v;
      }
    }
  };

  // ---- A operand of a step
  u4 nib[PF][VW];
  u2 iw[PF];
  uint32_t qp[PF];
  auto load_a = [&](int slot, int step) {
    const int s = min(step, g.nsteps - 1);
    const uint32_t chunk = row_chunk0 + (uint32_t)(4 * s + kb);
    iw[slot] = ld_plain<u2>(idx + 8ull * chunk);
    qp[slot] = 0;
    if (KIND == EGT_VAL_INT4) {
      nib[slot][0] = ld_plain<u4>(values + 16ull * chunk);
      qp[slot] = ld_plain<uint32_t>(qparams + 4ull * ((uint32_t)r_ld * (uint32_t)g.groups_per_row +
                                                        (uint32_t)((4 * s + kb) >> g.gshift)));
    } else {
#pragma unroll
      for (int k = 0; k < VW; ++k) nib[slot][k] = ld_plain<u4>(values + 64ull * chunk + 16 * k);
    }
  };

  load_x(0);
#pragma unroll
  for (int u = 0; u < PF; ++u) load_a(u, u);

  f4 acc[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc[j] = f4{0.f, 0.f, 0.f, 0.f};
  const uint32_t magic = in_vgpr(g.nib_magic);
  // LDS byte offset of this lane's B reads: token (lane & 15), octets b and 4 + b
  const int n = lane & 15, b = lane >> 4;
  const int boff0 = n * TOKEN_STRIDE + 16 * (8 * (b >> 1) + (b & 1));              // h = 0
  const int boff1 = n * TOKEN_STRIDE + 16 * (8 * ((4 + b) >> 1) + (b & 1));        // h = 1

  for (int s0 = 0; s0 < g.nsteps; s0 += PF) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int s = s0 + u;
      if (s < g.nsteps) {                              // uniform
        store_x(s);
        __syncthreads();
        load_x(s + 1);
        const uint8_t *buf = xs + (s & 1) * buf_bytes;
        uint32_t s2 = 0, off = 0;
        if (KIND == EGT_VAL_INT4) {
          s2 = __builtin_amdgcn_perm(qp[u], qp[u], 0x01000100u);
          off = pk_add_f16(__builtin_amdgcn_perm(qp[u], qp[u], 0x03020302u), g.nib_magic);
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          u4 a;
          if (KIND == EGT_VAL_INT4) a = dequant8_sm(nib[u][0][d], off, s2, g.nib_mask, magic);
          else a = nib[u][d];
          const int iword = d < 2 ? (int)iw[u][0] : (int)iw[u][1];
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            const uint8_t *tb = buf + 16 * j * TOKEN_STRIDE + 32 * d;
            const u4 lo = *(const u4 *)(tb + boff0);
            const u4 hi = *(const u4 *)(tb + boff1);
            const u8v bv = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            if (d & 1)
              acc[j] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bv), acc[j], iword, 0, 1);
            else
              acc[j] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h16, bv), acc[j], iword, 0, 0);
          }
        }
        load_a(u, s + PF);
      }
    }
  }

  // ---- D[row 4 kb + v][token n] of tile j -> Y[16 j + n][r0 + 4 kb + v]
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int tok = 16 * j + n;
    if (tok < g.M) {
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = r0 + 4 * kb + v;
        if (r < g.rows) {
          const bool ok = rp[v] == (uint32_t)r * S_row;
          Y[(int64_t)tok * g.ldy + r] = ok ? __float2half(acc[j][v]) : __ushort_as_half((uint16_t)0x7E00);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------
// K-split form.  The waves of a workgroup split K between them: in phase p, wave w
// owns K-step p * waves + w (256 dense columns).  It fetches its slice of X
// (16 tokens x 256 columns) with fully coalesced loads, turns it into the B operand
// layout through a private LDS region (token rows padded against bank conflicts, no
// workgroup barrier involved) and keeps B in registers while the workgroup walks over
// its (at most four) row tiles, whose A operands are all requested up front.  Each
// wave leaves its partial 16 x 16 products in its own region; after one barrier 256
// threads add them over the waves into running sums, and Y is stored after the last
// phase.  K <= 4096 is one phase.  Groups of 16 tokens are handled one after the other.
struct SmallMKsGeom {
  int rows, M;
  int nchunks;         // cols / 64
  int nsteps;          // cols / 256
  int ntiles;          // ceil(rows / 16)
  int gshift;
  int groups_per_row;
  int64_t ldx, ldy;
  uint32_t nib_mask, nib_magic;
};

template <int KIND>
struct ATile {                        // A operand of one row tile, one K-step
  u4 nib[KIND == EGT_VAL_INT4 ? 1 : 4];
  u2 iw;
  uint32_t qp;
};

constexpr int KS_MAX_ITEMS = 4;                    // row tiles per workgroup
constexpr int KS_REGION = 16 * TOKEN_STRIDE;       // LDS bytes per wave

template <int KIND>
__global__ __launch_bounds__(1024) void k_sparse_smallm_ks(const uint32_t *__restrict__ row_ptr,
                                                            const uint8_t *__restrict__ values,
                                                            const uint8_t *__restrict__ idx,
                                                            const uint8_t *__restrict__ qparams,
                                                            const __half *__restrict__ X,
                                                            __half *__restrict__ Y,
                                                            const SmallMKsGeom g) {
  extern __shared__ __align__(16) uint8_t xs[];       // [waves][KS_REGION]
  constexpr int VW = KIND == EGT_VAL_INT4 ? 1 : 4;
  constexpr int INFL = KIND == EGT_VAL_INT4 ? 3 : 2;  // row tiles whose A operand is in flight together
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int i = lane & 15, kb = lane >> 4;
  const int nit = (g.ntiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;   // <= KS_MAX_ITEMS
  const int phases = (g.nsteps + nw - 1) / nw;
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
  uint8_t *region = xs + wave * KS_REGION;
  // role of this thread in the cross-wave sum: row tile rit, register sv of lane sl
  const int rit = threadIdx.x >> 8, sv = (threadIdx.x >> 6) & 3, sl = threadIdx.x & 63;
  const int srow = 16 * ((int)blockIdx.x + rit * (int)gridDim.x) + 4 * (sl >> 4) + sv;
  const bool summing = rit < nit && srow < g.rows;

  auto load_a = [&](ATile<KIND> &a, int it, int step) {
    const int rt = min((int)blockIdx.x + it * (int)gridDim.x, g.ntiles - 1);
    const int r = min(16 * rt + i, g.rows - 1);
    const int s = min(step, g.nsteps - 1);
    const uint32_t chunk = (uint32_t)r * (uint32_t)g.nchunks + (uint32_t)(4 * s + kb);
    a.iw = ld_plain<u2>(idx + 8ull * chunk);
    a.qp = 0;
    if (KIND == EGT_VAL_INT4) {
      a.nib[0] = ld_plain<u4>(values + 16ull * chunk);
      a.qp = ld_plain<uint32_t>(qparams + 4ull * ((uint32_t)r * (uint32_t)g.groups_per_row +
                                                   (uint32_t)((4 * s + kb) >> g.gshift)));
    } else {
#pragma unroll
      for (int k = 0; k < VW; ++k) a.nib[k] = ld_plain<u4>(values + 64ull * chunk + 16 * k);
    }
  };

  const int ngroups = (g.M + 15) >> 4;
  bool first = true;
  for (int j = 0; j < ngroups; ++j) {
    float run = 0.f;
    const uint32_t rp = summing ? row_ptr[srow] : 0u;
    for (int p = 0; p < phases; ++p) {
      const int step = p * nw + wave;
      // ---- this wave's slice of X: 8 coalesced loads of two token rows each
      u4 xr[8];
      const bool step_ok = step < g.nsteps;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int tok = 16 * j + 2 * u + (lane >> 5);
        xr[u] = *(const u4 *)(X + (int64_t)min(tok, g.M - 1) * g.ldx + 256 * min(step, g.nsteps - 1) + 8 * (lane & 31));
      }
      ATile<KIND> a[INFL];
#pragma unroll
      for (int it = 0; it < INFL; ++it)
        if (it < nit) load_a(a[it], it, step);
      // the regions are read by the summing threads of the previous round: wait for them
      if (!first) __syncthreads();
      first = false;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int tl = 2 * u + (lane >> 5);
        u4 v = xr[u];
        if (16 * j + tl >= g.M || !step_ok) v = u4{0, 0, 0, 0};
        *(u4 *)(region + tl * TOKEN_STRIDE + 16 * (lane & 31)) = v;
      }
      // B operand: lane (n, b) reads token n, k-octets b and 4 + b of each 16-column group d
      u8v bx[4];
      {
        const int n = lane & 15, b = lane >> 4;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int kba = (4 * h + b) >> 1, sub = b & 1;
#pragma unroll
          for (int d = 0; d < 4; ++d) {
            const u4 v = *(const u4 *)(region + n * TOKEN_STRIDE + 16 * (8 * kba + 2 * d + sub));
#pragma unroll
            for (int k = 0; k < 4; ++k) bx[d][4 * h + k] = v[k];
          }
        }
      }

      auto compute = [&](const ATile<KIND> &at, int it) {
        f4 acc = {0.f, 0.f, 0.f, 0.f};
        uint32_t s2 = 0, off = 0;
        if (KIND == EGT_VAL_INT4) {
          s2 = __builtin_amdgcn_perm(at.qp, at.qp, 0x01000100u);
          off = pk_add_f16(__builtin_amdgcn_perm(at.qp, at.qp, 0x03020302u), g.nib_magic);
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
          u4 av;
          if (KIND == EGT_VAL_INT4) av = dequant8_sm(at.nib[0][d], off, s2, g.nib_mask, magic);
          else av = at.nib[d];
          const int iword = d < 2 ? (int)at.iw[0] : (int)at.iw[1];
          if (d & 1)
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 1);
          else
            acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av), __builtin_bit_cast(h16, bx[d]), acc, iword, 0, 0);
        }
        float *out = (float *)(region + it * 1024);   // B has been read: the region is free
#pragma unroll
        for (int v = 0; v < 4; ++v) out[v * 64 + lane] = acc[v];
      };
#pragma unroll
      for (int it0 = 0; it0 < KS_MAX_ITEMS; it0 += INFL) {
        if (it0 < nit) {
          if (it0 > 0) {
#pragma unroll
            for (int it = 0; it < INFL; ++it)
              if (it0 + it < nit) load_a(a[it], it0 + it, step);
          }
#pragma unroll
          for (int it = 0; it < INFL; ++it)
            if (it0 + it < nit) compute(a[it], it0 + it);
        }
      }
      __syncthreads();
      if (summing) {                                  // all reads issued together, then added in wave order
        const float *src = (const float *)(xs + rit * 1024) + (threadIdx.x & 255);
        float part[16];
#pragma unroll
        for (int w = 0; w < 16; ++w) part[w] = w < nw ? src[w * (KS_REGION / 4)] : 0.f;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < 16; ++w) sum += part[w];
        run += sum;
      }
    }
    // ---- store: thread (rit, sv, sl) owns D[row 4 (sl >> 4) + sv][token sl & 15] of row tile rit
    const int tok = 16 * j + (sl & 15);
    if (summing && tok < g.M) {
      const bool ok = rp == (uint32_t)srow * S_row;
      Y[(int64_t)tok * g.ldy + srow] = ok ? __float2half(run) : __ushort_as_half((uint16_t)0x7E00);
    }
  }
}

// Shapes covered: 2:4, K a multiple of 256, INT4 groups of 64 << j.
bool sparse_smallm_supported(const egt_2bitcsr &w) {
  if (w.n_keep != 2 || w.cols % 256 != 0 || w.cols < 256) return false;
  if (w.val_kind == EGT_VAL_INT4) {
    const int gm = w.group_size / 64;
    if (w.group_size % 64 != 0 || (gm & (gm - 1)) != 0) return false;
  }
  return true;
}

static hipError_t launch_sparse_smallm_steps(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx,
                                             uint16_t *Y, int64_t ldy, int M, hipStream_t stream);

hipError_t launch_sparse_smallm(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                int64_t ldy, int M, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  const int nsteps = w.cols / 256;
  int nw = nsteps < 16 ? nsteps : 16;                 // waves per workgroup
  int blocks_per_cu = 1;
  if (const char *e = getenv("EGT_SM_TUNE")) sscanf(e, "%d,%d", &nw, &blocks_per_cu);
  if (nw < 1 || nw > 16) return launch_sparse_smallm_steps(w, X, ldx, Y, ldy, M, stream);
  SmallMKsGeom g;
  g.rows = w.rows; g.M = M;
  g.nchunks = w.cols / 64;
  g.nsteps = nsteps;
  g.ntiles = (w.rows + 15) / 16;
  g.gshift = 0; g.groups_per_row = 0;
  if (w.val_kind == EGT_VAL_INT4) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.ldx = ldx; g.ldy = ldy;
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
  int nblocks = 256 * blocks_per_cu;                  // one (or more) workgroup per compute unit
  if (nblocks * KS_MAX_ITEMS < g.ntiles) nblocks = (g.ntiles + KS_MAX_ITEMS - 1) / KS_MAX_ITEMS;
  if (nblocks > g.ntiles) nblocks = g.ntiles;
  const dim3 grid(nblocks), block(64 * nw);
  const size_t lds = (size_t)nw * KS_REGION;
  if (w.val_kind == EGT_VAL_INT4)
    return launch(k_sparse_smallm_ks<EGT_VAL_INT4>, grid, block, lds, stream, w.row_ptr,
                  (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams,
                  (const __half *)X, (__half *)Y, g);
  return launch(k_sparse_smallm_ks<EGT_VAL_FP16>, grid, block, lds, stream, w.row_ptr,
                (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams,
                (const __half *)X, (__half *)Y, g);
}

// K-step form (any K that is a multiple of 256): used when K is too wide for one
// workgroup to cover it with 16 waves.
static hipError_t launch_sparse_smallm_steps(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                int64_t ldy, int M, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  SmallMGeom g;
  g.rows = w.rows; g.M = M;
  g.nchunks = w.cols / 64;
  g.nsteps = w.cols / 256;
  g.gshift = 0; g.groups_per_row = 0;
  if (w.val_kind == EGT_VAL_INT4) {
    while ((64 << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.ldx = ldx; g.ldy = ldy;
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
  const int nt = M <= 16 ? 1 : (M <= 32 ? 2 : 4);
  const int row_tiles = (w.rows + 15) / 16;
  const int nw = row_tiles >= 512 ? 2 : 1;            // waves (row tiles) per workgroup
  // 16 B pieces per thread per step = 16 nt tokens * 32 pieces / (64 nw threads)
  const int xpt = 8 * nt / nw;
  const dim3 grid((row_tiles + nw - 1) / nw), block(64 * nw);
  const size_t lds = 2 * 16 * nt * TOKEN_STRIDE;
#define EGT_GO(KIND, NT, PF, XPT)                                                               \
  launch(k_sparse_smallm<KIND, NT, PF, XPT>, grid, block, lds, stream, w.row_ptr,                \
         (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams,          \
         (const __half *)X, (__half *)Y, g)
#define EGT_PICK(KIND, PF)                                                                       \
  switch (xpt) {                                                                                 \
    case 2: return EGT_GO(KIND, 1, PF, 2);   /* nt 1, nw 4 */                                    \
    case 4: return nt == 1 ? EGT_GO(KIND, 1, PF, 4) : EGT_GO(KIND, 2, PF, 4);                    \
    case 8: return nt == 1 ? EGT_GO(KIND, 1, PF, 8) : nt == 2 ? EGT_GO(KIND, 2, PF, 8)           \
                                                               : EGT_GO(KIND, 4, PF, 8);         \
    case 16: return nt == 2 ? EGT_GO(KIND, 2, PF, 16) : EGT_GO(KIND, 4, PF, 16);                 \
    default: return EGT_GO(KIND, 4, PF, 32); /* nt 4, nw 1 */                                    \
  }
  if (w.val_kind == EGT_VAL_INT4) { EGT_PICK(EGT_VAL_INT4, 4) }
  EGT_PICK(EGT_VAL_FP16, 2)
#undef EGT_PICK
#undef EGT_GO
}

}  // namespace egt
