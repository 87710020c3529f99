// Small-M SparseGemm for 17 <= M <= 64 tokens with the activations held still in LDS.
//
// Sec. 3.4 puts all candidates of a trie level through the linear layers at once; its
// cost "scales with the number of candidates".  On this device the part that scales is
// X, not W: in the one-launch kernel (egt_mfma_smallm.hip) every compute unit owns row
// tiles over the whole of K and therefore pulls the whole of X (M * K * 2 bytes) through
// its XCD's L2 once per token group, which costs 3.5 us per group of 16 tokens on
// 11008 x 4096 against 5 us for the weights.  (Measured with stages compiled out, 11008 x
// 4096, M = 64, both kernels: tile requests alone 9.9 us, + X 1.5, + products 4.0, + the
// partial sums' store and write-back 4.0: the stages of such a short kernel do not overlap.)
//
// Here the grid is cut in two dimensions: workgroup (row block b, K slice s) owns the row
// tiles of block b over the K-steps of slice s only.  A slice is short enough (<= 16 / NG
// steps of 256 columns for NG token groups) for its part of X - all M tokens - to sit in
// LDS (<= 132 KB of the 160 KB) for the whole life of the workgroup: X is fetched once per
// workgroup, straight from global memory into LDS, and every wave then streams the weights
// of its own row tiles past it.  A wave owns whole tiles (all steps of the slice, all
// token groups), so there is no sum across waves; the 16 x 16 FP32 sums of a (tile, slice,
// group) go to the caller's workspace, and k_smallm_sum_slices adds the slices in
// ascending order and rounds once: the result does not depend on timing.
//
// Operand layout, X layout in LDS, dequantisation and the lane exchange of the A tiles are
// those of the one-launch kernel (2:4, INT4, one {scale, zero} pair per 64-column chunk).
#include "egt_mfma_common.h"

namespace egt {

struct SmallMXsGeom {
  int rows, M;
  int nchunks;         // cols / 64
  int nsteps;          // nchunks / 4 (K is a multiple of 256 here)
  int ntiles;          // ceil(rows / 16)
  int gshift;          // group = 64 << gshift columns
  int groups_per_row;
  int nslices;         // K slices; slice s owns the steps [s * nsteps / nslices, (s + 1) * nsteps / nslices)
  int row_blocks;      // row block b owns the tiles [b * ntiles / row_blocks, (b + 1) * ntiles / row_blocks)
  uint32_t val_bytes, idx_bytes, qp_bytes, x_bytes, rp_bytes;   // extents of the arrays
  int64_t ldx;
  float *ws;           // 16 x 16 sums as the matrix instruction leaves them: ws[((s * ntiles + tile) * NG + grp) * 256 + 4 * lane + j]
                       // is token 16 grp + (lane & 15), row 16 tile + 4 (lane >> 4) + j of slice s
  uint32_t nib_mask, nib_magic;
};

constexpr int XS_PAIR = 1024 + 32;                   // LDS bytes of a pair of tokens of one step (512 B each)
constexpr int XS_REGION = 8 * XS_PAIR;               // one step, one token group
constexpr int XS_MAX_REGIONS = 16;                   // 135 168 B
constexpr int XS_T = 2;                              // row tiles a wave works on at a time

__device__ __forceinline__ uint32_t xs_lane_perm(int byte_addr, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_ds_bpermute(byte_addr, (int)v);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t xs_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// What a lane fetched of one row tile over the steps of a slice (lane 4 r + c: chunk c of
// row r of every step), and the row pointer lane r < 16 checks.
template <int SPS>
struct XsTile {
  u4 nib[SPS];
  u2 iw[SPS];
  uint32_t qp[SPS];
  uint32_t rp;
};

// NG: token groups of 16 (2..4).  SPS: K-steps of a slice at most (NG * SPS <= 16).
// T: row tiles a wave works on at a time.
template <int NG, int SPS, int T>
__global__ __launch_bounds__(512) void k_smallm_xs(const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
                                                   const uint8_t *__restrict__ idx, const uint8_t *__restrict__ qparams,
                                                   const __half *__restrict__ X, const SmallMXsGeom g) {
  static_assert(NG * SPS <= XS_MAX_REGIONS, "the slice of X fits LDS");
  extern __shared__ __align__(16) uint8_t xs[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int slice = (int)blockIdx.x % g.nslices, rb = (int)blockIdx.x / g.nslices;
  const int step0 = slice * g.nsteps / g.nslices;
  const int sps = (slice + 1) * g.nsteps / g.nslices - step0;           // <= SPS (host)
  const int tile0 = rb * g.ntiles / g.row_blocks, tile1 = (rb + 1) * g.ntiles / g.row_blocks;

  const __amdgpu_buffer_rsrc_t r_val = xs_rsrc(values, g.val_bytes), r_idx = xs_rsrc(idx, g.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = xs_rsrc(qparams, g.qp_bytes), r_x = xs_rsrc(X, g.x_bytes);
  const __amdgpu_buffer_rsrc_t r_rp = xs_rsrc(row_ptr, g.rp_bytes);
  const uint32_t off_range = 0xFFFFFFF0u;             // past every buffer: zeros, no traffic

  // ---- X of the slice: region (step ls, group grp) at (ls * NG + grp) * XS_REGION; request u
  //      of a region brings tokens 2 u, 2 u + 1 of the group (lane l: 16 bytes at 16 l of the
  //      kilobyte; the odd token has neighbouring pieces swapped, see the one-launch kernel)
  {
    const int xtl = lane >> 5;
    const int slot_piece = (lane & 31) ^ xtl;
    const uint32_t off_lo = 16u * (uint32_t)slot_piece;
    const uint32_t off_hi = off_lo + (uint32_t)xtl * (uint32_t)(2 * g.ldx);
    asm volatile("" ::: "memory");
    for (int q = wave; q < sps * NG * 8; q += nw) {
      const int u = q & 7, rg = q >> 3, grp = rg % NG, ls = rg / NG;
      const int t0 = 16 * grp + 2 * u;
      if (t0 < g.M)                                   // uniform; the odd token past an odd M repeats token M - 1
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(xs + rg * XS_REGION + XS_PAIR * u),
                                                 16, t0 + 1 < g.M ? off_hi : off_lo,
                                                 (uint32_t)(512 * (step0 + ls)) + (uint32_t)t0 * (uint32_t)(2 * g.ldx), 0, 0);
    }
    asm volatile("" ::: "memory");
  }

  // ---- A tiles
  const int i = lane & 15, kb = lane >> 4;
  const int li = lane >> 2, lc = lane & 3;            // row, chunk this lane fetches
  const int from = 4 * (4 * i + kb);                  // lane that fetched the chunk of lane (i, kb), as a byte address
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
  // Requests for T tiles, step by step (the first step of every tile arrives first, and
  // the products of a step start as soon as its data is there); T * (3 SPS + 1) requests,
  // whatever the slice and the tiles: those past the end are made out of range.
  auto load_tiles = [&](XsTile<SPS> (&a)[T], int t) {
    uint32_t cl[T], ql[T], cu0[T], qu[T];
    bool on[T];
#pragma unroll
    for (int k = 0; k < T; ++k) {
      on[k] = t + k < tile1;                                                  // uniform
      const int tt = on[k] ? t + k : tile0;
      const uint32_t rel = (uint32_t)min(li, g.rows - 1 - 16 * tt);           // row inside the tile (clamped)
      cl[k] = rel * (uint32_t)g.nchunks + (uint32_t)lc;                       // lane part of the chunk number
      ql[k] = rel * (uint32_t)g.groups_per_row;
      cu0[k] = (uint32_t)(16 * tt) * (uint32_t)g.nchunks;
      qu[k] = 4u * (uint32_t)(16 * tt) * (uint32_t)g.groups_per_row;
      // lanes 0..15 fetch the row pointers of the tile (rows past the end: the last row's)
      const uint32_t prow = (uint32_t)min(16 * tt + i, g.rows - 1);
      a[k].rp = __builtin_amdgcn_raw_buffer_load_b32(r_rp, on[k] ? 4u * prow : off_range, 0u, 0);
    }
#pragma unroll
    for (int ls = 0; ls < SPS; ++ls) {
#pragma unroll
      for (int k = 0; k < T; ++k) {
        const bool live = on[k] && ls < sps;                                  // uniform
        const uint32_t cu = cu0[k] + (uint32_t)(4 * (step0 + ls));
        a[k].iw[ls] = __builtin_amdgcn_raw_buffer_load_b64(r_idx, live ? 8u * cl[k] : off_range, live ? 8u * cu : 0u, 0);
        a[k].nib[ls] = __builtin_amdgcn_raw_buffer_load_b128(r_val, live ? 16u * cl[k] : off_range, live ? 16u * cu : 0u, 0);
        const uint32_t chunk = (uint32_t)(4 * (step0 + ls) + lc);
        a[k].qp[ls] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, live ? 4u * (ql[k] + (chunk >> g.gshift)) : off_range,
                                                           live ? qu[k] : 0u, 0);
      }
    }
  };
  // B operand of instruction m of a step: lane (n, b) holds token n, k-octets b and 4 + b
  auto read_b = [&](const uint8_t *region, int m, u8v &bx) {
    const int n = lane & 15, b = lane >> 4;
    const uint8_t *base0 = region + XS_PAIR * (n >> 1) + 512 * (n & 1) + 16 * (8 * (b >> 1) + ((b ^ n) & 1));
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u4 v = *(const u4 *)(base0 + 256 * h + 32 * m);
#pragma unroll
      for (int k = 0; k < 4; ++k) bx[4 * h + k] = v[k];
    }
  };

  // A wave takes its tiles T at a time: every B operand read from LDS then serves T tiles
  // (the LDS reads are what bounds this kernel: 1 KB per instruction operand), and the
  // T * NG matrix instructions that follow a read are independent of each other.
  XsTile<SPS> a[T];
  int t = tile0 + T * wave;
  load_tiles(a, t);
  asm volatile("" ::: "memory");
  wait_vmem<T * (3 * SPS + 1)>();                     // requests return in order: this wave's part of X has arrived,
  lds_barrier();                                      // the tile requests stay in flight across the barrier
  if (t >= tile1) return;                             // a wave without tiles only helped to fetch X (no barrier follows)

  for (;;) {
    f4 acc[T][NG];
#pragma unroll
    for (int k = 0; k < T; ++k)
#pragma unroll
      for (int grp = 0; grp < NG; ++grp) acc[k][grp] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ls = 0; ls < SPS; ++ls) {
      if (ls < sps) {                                 // uniform
        u4 av[T][4];
        uint32_t iw0[T], iw1[T];
#pragma unroll
        for (int k = 0; k < T; ++k) {
          // fetched form -> operand form: lane (i, kb) takes what lane 4 i + kb fetched
          u4 nib;
#pragma unroll
          for (int d = 0; d < 4; ++d) nib[d] = xs_lane_perm(from, a[k].nib[ls][d]);
          iw0[k] = xs_lane_perm(from, a[k].iw[ls][0]);
          iw1[k] = xs_lane_perm(from, a[k].iw[ls][1]);
          const uint32_t qp = xs_lane_perm(from, a[k].qp[ls]);
          const uint32_t s2 = __builtin_amdgcn_perm(qp, qp, 0x01000100u);
          const uint32_t off = pk_add_f16(__builtin_amdgcn_perm(qp, qp, 0x03020302u), g.nib_magic);
#pragma unroll
          for (int d = 0; d < 4; ++d) av[k][d] = dequant8(nib[d], off, s2, g.nib_mask, magic);
        }
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          u8v bx[NG];
#pragma unroll
          for (int grp = 0; grp < NG; ++grp) read_b(xs + (ls * NG + grp) * XS_REGION, m, bx[grp]);
#pragma unroll
          for (int k = 0; k < T; ++k) {
            const int iword = (int)(m < 2 ? iw0[k] : iw1[k]);
#pragma unroll
            for (int grp = 0; grp < NG; ++grp) {
              if (m & 1)
                acc[k][grp] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[k][m]), __builtin_bit_cast(h16, bx[grp]),
                                                                       acc[k][grp], iword, 0, 1);
              else
                acc[k][grp] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[k][m]), __builtin_bit_cast(h16, bx[grp]),
                                                                       acc[k][grp], iword, 0, 0);
            }
          }
        }
      }
    }
    // ---- a row whose pointer is not r * S yields NaN; lane (n, b) stores rows 4 b .. 4 b + 3 of token n
#pragma unroll
    for (int k = 0; k < T; ++k) {
      const int tk = t + k;
      if (tk < tile1) {                               // uniform
        const bool rp_ok = lane >= 16 || a[k].rp == (uint32_t)min(16 * tk + i, g.rows - 1) * S_row;
        const uint32_t okmask = (uint32_t)__ballot(rp_ok) >> (4 * kb);
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) {
          f4 v = acc[k][grp];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            if (!((okmask >> j) & 1u)) v[j] = __builtin_nanf("");
          // one contiguous kilobyte per tile and token group
          *(f4 *)(g.ws + (((int64_t)slice * g.ntiles + tk) * NG + grp) * 256 + 4 * lane) = v;
        }
      }
    }
    t += T * nw;
    if (t >= tile1) break;                            // uniform
    load_tiles(a, t);
  }
}

// Shapes this form takes: 2:4, INT4, one {scale, zero} pair per chunk (groups of 64 << j),
// K a multiple of 256, 17..64 tokens whose rows start on 16-byte boundaries.
bool sparse_smallm_xs_plan(const egt_2bitcsr &w, int64_t ldx, int M, bool force, SmallMXsGeom &g, int &ng, int &sps_cap, int &nw,
                           size_t &lds) {
  if (w.val_kind != EGT_VAL_INT4 || w.n_keep != 2 || M < 17 || M > 64 || w.rows < 1) return false;
  // Where it is the faster form (measured against the one-launch kernel and the split with
  // X re-fetched per workgroup): more than 32 tokens on long rows or on many rows.  The
  // partial sums cost a write-back at the end of the kernel, a second launch and their read;
  // that is recovered only where X, not W, dominates the one-launch kernel.
  if (!force && !(M > 32 && (w.cols >= 8192 || w.rows >= 8192))) return false;
  if (w.cols % 256 != 0 || w.cols < 256 || ldx % 8 != 0) return false;
  const int gm = w.group_size / 64;
  if (w.group_size % 64 != 0 || gm < 1 || (gm & (gm - 1)) != 0) return false;
  const uint64_t chunks = (uint64_t)w.rows * (uint64_t)(w.cols / 64);
  const uint64_t xbytes = ((uint64_t)(M - 1) * (uint64_t)ldx + (uint64_t)w.cols) * 2;
  if (chunks * 16 >= (1ull << 32) || xbytes >= (1ull << 32)) return false;       // 32-bit offsets
  g.rows = w.rows; g.M = M;
  g.nchunks = w.cols / 64;
  g.nsteps = g.nchunks / 4;
  g.ntiles = (w.rows + 15) / 16;
  g.gshift = 0;
  while ((64 << g.gshift) < w.group_size) ++g.gshift;
  g.groups_per_row = w.cols / w.group_size;
  ng = (M + 15) / 16;
  sps_cap = ng == 4 ? 4 : ng == 3 ? 5 : 8;
  g.nslices = (g.nsteps + sps_cap - 1) / sps_cap;
  if (g.nslices < 2 || g.nslices > 256) return false;    // one slice: nothing to add up, the one-launch kernel does it
  g.row_blocks = 256 / g.nslices;                    // one workgroup per compute unit
  if (g.row_blocks > g.ntiles) g.row_blocks = g.ntiles;
  if (g.row_blocks < 1) g.row_blocks = 1;
  g.val_bytes = (uint32_t)(chunks * 16); g.idx_bytes = (uint32_t)(chunks * 8);
  g.qp_bytes = (uint32_t)((uint64_t)w.rows * (uint64_t)g.groups_per_row * 4);
  g.x_bytes = (uint32_t)xbytes;
  g.rp_bytes = (uint32_t)(4 * ((uint64_t)w.rows + 1));
  g.ldx = ldx;
  g.ws = nullptr;
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
  // waves: the tile pairs of a row block spread as evenly as they go over at most 8 waves
  const int tpb = (g.ntiles + g.row_blocks - 1) / g.row_blocks;
  const int units = (tpb + XS_T - 1) / XS_T;
  const int per_wave = (units + 7) / 8;
  nw = (units + per_wave - 1) / per_wave;
  if (nw < 4) nw = 4;                                 // X of the slice is fetched by all waves
  const int sps_max = (g.nsteps + g.nslices - 1) / g.nslices;
  lds = (size_t)sps_max * (size_t)ng * XS_REGION;
  return true;
}

// Y[m][r] = FP16( sum over the K slices, in slice order, of the 16 x 16 sums of k_smallm_xs ).
// One thread per lane of a (tile, token group): four consecutive rows of one token.
__global__ __launch_bounds__(256) void k_smallm_xs_sum(const float *__restrict__ ws, int nslices, int ntiles, int ng, int M, int rows,
                                                       __half *__restrict__ Y, int64_t ldy, int vec_store) {
  const int64_t unit = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);        // (tile, group)
  if (unit >= (int64_t)ntiles * ng) return;
  const int lane = threadIdx.x & 63, tile = (int)(unit / ng), grp = (int)(unit % ng);
  const int tok = 16 * grp + (lane & 15), row0 = 16 * tile + 4 * (lane >> 4);
  // four slices are requested before the first is added (one memory latency per four slices, not per slice);
  // the additions stay in ascending slice order
  f4 sum = f4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < nslices; s0 += 4) {
    f4 p[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      p[k] = *(const f4 *)(ws + (((int64_t)min(s0 + k, nslices - 1) * ntiles + tile) * ng + grp) * 256 + 4 * lane);
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (s0 + k < nslices) sum += p[k];
  }
  if (tok >= M || row0 >= rows) return;
  uint32_t h[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) h[j] = sum[j] != sum[j] ? 0x7E00u : (uint32_t)__half_as_ushort(__float2half(sum[j]));
  __half *dst = Y + (int64_t)tok * ldy + row0;
  if (vec_store && row0 + 3 < rows) {
    *(u2 *)dst = u2{h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (row0 + j < rows) dst[j] = __ushort_as_half((uint16_t)h[j]);
  }
}

template <int NG, int SPS>
static hipError_t go_xs(const egt_2bitcsr &w, const uint16_t *X, const SmallMXsGeom &g, int nw, size_t lds, hipStream_t stream) {
  // more than 64 KB of dynamic LDS has to be asked for once per kernel and device
  static thread_local int asked_dev = -1;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (asked_dev != dev) {
    e = hipFuncSetAttribute((const void *)k_smallm_xs<NG, SPS, XS_T>, hipFuncAttributeMaxDynamicSharedMemorySize, XS_MAX_REGIONS * XS_REGION);
    if (e != hipSuccess) return e;
    asked_dev = dev;
  }
  return launch(k_smallm_xs<NG, SPS, XS_T>, dim3(g.row_blocks * g.nslices), dim3(64 * nw), lds, stream, w.row_ptr,
                (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams, (const __half *)X, g);
}

size_t sparse_smallm_xs_bytes(const egt_2bitcsr &w, int64_t ldx, int M, bool force) {
  SmallMXsGeom g;
  int ng, cap, nw;
  size_t lds;
  if (!sparse_smallm_xs_plan(w, ldx, M, force, g, ng, cap, nw, lds)) return 0;
  return sizeof(float) * 256 * (size_t)g.nslices * (size_t)g.ntiles * (size_t)ng;
}

hipError_t launch_sparse_smallm_xs(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y, int64_t ldy, int M,
                                   float *ws, bool force, hipStream_t stream) {
  SmallMXsGeom g;
  int ng, cap, nw;
  size_t lds;
  if (!sparse_smallm_xs_plan(w, ldx, M, force, g, ng, cap, nw, lds)) return hipErrorInvalidValue;
  g.ws = ws;
  hipError_t e;
  if (ng == 4) e = go_xs<4, 4>(w, X, g, nw, lds, stream);
  else if (ng == 3) e = go_xs<3, 5>(w, X, g, nw, lds, stream);
  else e = go_xs<2, 8>(w, X, g, nw, lds, stream);
  if (e != hipSuccess) return e;
  const int vec_store = ((uintptr_t)Y % 8 == 0 && ldy % 4 == 0) ? 1 : 0;
  return launch(k_smallm_xs_sum, dim3((unsigned)(((int64_t)g.ntiles * ng + 3) / 4)), dim3(256), 0, stream, (const float *)ws, g.nslices,
                g.ntiles, ng, M, w.rows, (__half *)Y, ldy, vec_store);
}

}  // namespace egt
