// Small-M SparseGemm (2 <= M <= 64 activation rows) on the gfx950 sparse matrix
// cores: the parallel-verification form of the product, Y[m][r] = sum_k W[r][k] X[m][k].
//
// Mapping.  The 16 rows of the A operand of v_smfmac_f32_16x16x64_f16 are 16 matrix
// rows (a row tile) and the 16 columns of B are 16 activation rows (a token group), so
// all 256 outputs of an instruction are used.  K is walked in steps of four chunks; a
// chunk is 16 B of nibbles (or 64 B of FP16 values) + 8 B of idx words = 32 slots, i.e.
// 64 dense columns at 2:4 and 128 at 1:4.  In a step, lane (i, kb) = i + 16 kb holds
// chunk kb of row i.
//   2:4: its four dwords feed four instructions; instruction d sees, as its k-range
//        [16 kb, 16 kb + 16), the dense columns 64 kb + 16 d .. + 15 of the step.
//   1:4: the instruction wants two values per four columns, so every slot becomes the
//        pair {value, 0} with its offset in the even index field (spread_idx); eight
//        instructions finish the step, instruction m takes slots 4 m .. 4 m + 3 of the
//        chunk = the dense columns 128 kb + 16 m .. + 15.
// Any fixed permutation of k is fine as long as B follows it, and B is read from LDS
// with exactly that permutation.
//
// The waves of a workgroup split K between them: in phase p, wave w owns K-step
// p * waves + w of every row tile of the workgroup (at most NIT of them) and keeps its
// 16 x 16 sums in registers over the phases.  Its slice of X goes from global memory
// straight into a private LDS region (no registers in between, no workgroup barrier).
// A operand, INT4: lane 4 r + c fetches chunk c of row r of the step, so that four
// neighbouring lanes read 64 contiguous bytes, and a lane permutation (ds_bpermute)
// hands the chunk to lane (i, kb) = (r, c) of the matrix instruction.  FP16 values at
// 2:4 use another assignment (LINA below): instruction k takes chunk k and lane (i, kb)
// its piece kb, what a lane fetches is its operand; at 1:4 lane (i, kb) fetches the 64 B
// of its chunk.
// The loads of phase p + 1 are requested while phase p is computed.  Loads return in
// the order of their requests, so a request for X that follows a request for A waits
// for A: with NT = 2 token groups the second group of a phase is requested before the
// A tiles of the next phase and nothing needed soon queues behind the long latency of
// A.  More than 16 NT tokens are handled in passes over the same rows (the weights of
// the later passes come from the caches).  In the last phase nothing is requested any
// more and the row tiles are consumed as they arrive.  Then the waves leave their sums
// in LDS, one barrier later 4-lane groups add them up over the waves in wave order (a
// fixed order: the result does not depend on timing) and store four consecutive rows of
// a token.  Row tiles past the last one of a workgroup are requested out of range of the
// buffer resources (zeros, no traffic), so every wave issues the same number of loads.
// A last step that K fills only partly: chunks past the end are fetched from a clamped
// (valid) address and enter with scale 0 (FP16: value 0), the pieces of X past the end
// are overwritten with zeros in LDS.
#include "egt_mfma_common.h"

#include "egt_tune.h"

#include <cstring>

namespace egt {

struct SmallMKsGeom {
  int rows, M;
  int nchunks;         // cols / 64 (2:4) or cols / 128 (1:4)
  int nsteps;          // ceil(nchunks / 4)
  int kpieces;         // cols / 8: 16-byte pieces of a row of X
  int ntiles;          // ceil(rows / 16)
  int gshift;          // one {scale, zero} pair per chunk: group = chunk << gshift columns
  int groups_per_row;
  int vec_store;       // Y and ldy allow 8-byte stores of four rows
  uint32_t val_bytes, idx_bytes, qp_bytes, x_bytes;   // extents of the arrays
  int64_t ldx, ldy;
  uint32_t nib_mask, nib_magic;                        // 0x00F0000F, FP16 {1024.0, 64.0}
  uint32_t m8, m4, m2;                                 // masks of spread_idx
  // K split over workgroups (blockIdx.y = slice s of nslices: the K-steps
  // [s * nsteps / nslices, (s + 1) * nsteps / nslices)), and where the FP32 partial sums of
  // slice s, token m, row r go: ws[(s * M + m) * ws_ld + r]
  int nslices;
  int64_t ws_ld;
  float *ws;
};

template <int KIND, int QW>
struct ATile {                        // A operand of one row tile, one K-step
  static constexpr int VW = KIND == EGT_VAL_INT4 ? 1 : 4;        // 16-byte value registers per lane
  // Vector-memory requests that fetch one tile: the index words, then either the nibbles
  // and the quantisation parameters (any QW: one request) or VW requests of FP16 values.
  // The kernel waits with hand-counted `s_waitcnt vmcnt(n)`; every n is a multiple of
  // this number, and every request in load_a names its ordinal below it (TileRequest).
  static constexpr int LOADS = KIND == EGT_VAL_INT4 ? 3 : 1 + VW;
  u4 nib[VW];
  u2 iw;
  uint32_t qp[QW];                    // {scale, zero} pairs of the chunk (QW > 1: groups narrower than a chunk)
};
// Tag of the ORD-th request of a tile: a request added to load_a without raising
// ATile::LOADS (and with it every wait count) does not compile.
template <int ORD, int LOADS>
struct TileRequest {
  static_assert(ORD >= 0 && ORD < LOADS, "a tile request beyond the count the vmcnt waits are built on");
};

constexpr int KS_PAIR = 1024 + 32;                 // 2:4: LDS bytes of a pair of tokens (512 B each)
constexpr int KS_TOKEN_N1 = 1024 + 16;             // 1:4: LDS bytes of a token (1 KiB)

__device__ __forceinline__ uint32_t lane_perm(int byte_addr, uint32_t v) {
  return (uint32_t)__builtin_amdgcn_ds_bpermute(byte_addr, (int)v);
}
// Buffer resource over `bytes` bytes at p: loads through it take a 32-bit lane offset
// plus a 32-bit wave-uniform offset (scalar registers, scalar arithmetic).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}
template <int N>
__device__ __forceinline__ uint32_t quad_bcast(uint32_t v) {     // value of lane N of the 4-lane group
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, N * 0x55, 0xf, 0xf, true);
}

// KIND: INT4 or FP16 values.  NT: token groups per pass.  NIT: row tiles per workgroup.
// NWMAX: waves per workgroup at most.  QW: {scale, zero} pairs per chunk.  N1: 1:4.
// RND: a workgroup may own more than NIT row tiles and takes them in rounds.
// KS: the grid's y dimension splits K; a workgroup walks only the K-steps of its slice and
// leaves FP32 partial sums in the caller's workspace (k_smallm_sum_slices finishes them).
template <int KIND, int NT, int NIT, int NWMAX, int QW, bool N1, bool RND, bool KS = false>
__device__ __forceinline__ void smallm_ks_body(const uint32_t *__restrict__ row_ptr, const uint8_t *__restrict__ values,
                                               const uint8_t *__restrict__ idx, const uint8_t *__restrict__ qparams,
                                               const __half *__restrict__ X, __half *__restrict__ Y, const SmallMKsGeom g) {
  extern __shared__ __align__(16) uint8_t xs[];       // X regions, later the partial sums
  static_assert(!(N1 && NT > 1), "1:4 runs one token group per pass");
  constexpr bool INT4 = KIND == EGT_VAL_INT4;
  constexpr int VW = ATile<KIND, QW>::VW;
  constexpr int LPT = ATile<KIND, QW>::LOADS;         // requests per tile: the unit of every vmcnt wait below
  constexpr bool HOLD = NT > 1;                       // A operands of a phase are kept for all token groups
  // FP16 values at 2:4: instruction k of a step takes chunk k, lane (i, kb) its 16-byte
  // piece kb, so the four lanes of a row fetch 64 contiguous bytes and what a lane
  // fetches is its operand.  (Otherwise lane (i, kb) owns chunk kb for all instructions.)
  constexpr bool LINA = !INT4 && !N1;
  // DEEP: the A tiles are requested two phases ahead (two sets of fetch registers); X,
  // which has one LDS region per wave, stays one phase ahead.
  constexpr bool DEEP = LINA && !HOLD;
  constexpr int NM = N1 ? 8 : 4;                      // matrix instructions per step
  constexpr int PIECES = N1 ? 64 : 32;                // 16-byte pieces of a token row in a step
  constexpr int REGION = N1 ? 16 * KS_TOKEN_N1 : 8 * KS_PAIR;   // LDS bytes per wave for X
  constexpr int PART = NIT * NT * 1024;               // bytes of partial sums per wave
  // SEP: the partial sums have LDS of their own behind the X regions, so the first loads
  // of the next pass can be requested before the sums of this pass are added up and
  // stored (8-wave forms with two token groups per pass; the others put them over the X regions)
  constexpr bool SEP = HOLD;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = blockDim.x >> 6;
  const int i = lane & 15, kb = lane >> 4;
  // row, chunk this lane fetches (LINA: of the index words only)
  const int li = (INT4 || LINA) ? (lane >> 2) : i, lc = (INT4 || LINA) ? (lane & 3) : kb;
  const int from = 4 * (4 * i + kb);                  // lane that fetched the chunk of lane (i, kb), as a byte address
  // Row tiles of this workgroup: blockIdx.x + k * gridDim.x, k < mytiles, taken NIT at a time
  // (rounds); round rr holds tiles_of(rr) of them.
  const int mytiles = (g.ntiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;
  const int rounds = RND ? (mytiles + NIT - 1) / NIT : 1;
  auto tiles_of = [&](int rr) { return RND ? min(NIT, mytiles - rr * NIT) : mytiles; };
  // the K-steps of this workgroup: [step0, nsteps)
  const int step0 = KS ? (int)blockIdx.y * g.nsteps / g.nslices : 0;
  const int nsteps = KS ? ((int)blockIdx.y + 1) * g.nsteps / g.nslices : g.nsteps;
  const int phases = (nsteps - step0 + nw - 1) / nw;
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
  uint8_t *region = xs + wave * REGION;
  const int ngroups = (g.M + 15) >> 4;
  // Row pointers of the workgroup's rows are requested first and checked at the end
  // (flags in LDS behind the regions): a row whose pointer is not r * S yields NaN.
  // (not SEP: a wave's partial sums go to the start of its own X region, which no other
  //  wave touches: no barrier between the last read of X and the sums)
  static_assert(PART <= REGION, "partial sums of a wave fit its X region");
  constexpr int PSTRIDE = SEP ? PART : REGION;        // bytes from one wave's partial sums to the next
  uint8_t *parts = SEP ? xs + nw * REGION : xs;
  uint32_t *flags = (uint32_t *)(xs + nw * (SEP ? REGION + PART : REGION));
  const int frow0 = 16 * ((int)blockIdx.x + (int)(threadIdx.x >> 4) * (int)gridDim.x) + (int)(threadIdx.x & 15);
  auto flag_row = [&](int rr) {                       // the row whose pointer this thread checks in round rr
    return RND ? frow0 + 16 * rr * NIT * (int)gridDim.x : frow0;
  };
  auto flag_checked = [&](int rr) { return (int)threadIdx.x < 16 * tiles_of(rr) && flag_row(rr) < g.rows; };
  auto load_rp = [&](int rr) { return flag_checked(rr) ? row_ptr[flag_row(rr)] : 0u; };
  const bool fcheck0 = flag_checked(0);
  uint32_t frp = fcheck0 ? row_ptr[frow0] : 0u, frp_next = 0;

  const __amdgpu_buffer_rsrc_t r_val = make_rsrc(values, g.val_bytes), r_idx = make_rsrc(idx, g.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = make_rsrc(qparams, g.qp_bytes), r_x = make_rsrc(X, g.x_bytes);
  auto load_a = [&](ATile<KIND, QW> &a, int it, int step, int rr) {
    // A tile past the last one of the round is requested out of range of the buffers: such a
    // request returns zeros and moves no data (the count of requests per phase stays fixed).
    const int nit_r = RND ? tiles_of(rr) : mytiles;
    const bool on = it < nit_r;                                               // uniform
    const uint32_t off_range = 0xFFFFFFF0u;
    const int rt = (int)blockIdx.x + ((RND ? rr * NIT : 0) + min(it, nit_r - 1)) * (int)gridDim.x;
    const int s = min(step, nsteps - 1);
    // (the lane offsets are recomputed at every request: kept across the loops they would
    //  occupy a dozen registers)
    const uint32_t rel = (uint32_t)min((int)in_vgpr((uint32_t)li), g.rows - 1 - 16 * rt);   // row inside the tile (clamped)
    const uint32_t lcc = (uint32_t)min((int)in_vgpr((uint32_t)lc), g.nchunks - 1 - 4 * s);  // chunk inside the step (clamped)
    const uint32_t cl = rel * (uint32_t)g.nchunks + lcc;                      // lane part of the chunk number
    const uint32_t cu = on ? (uint32_t)(16 * rt) * (uint32_t)g.nchunks + (uint32_t)(4 * s) : 0u;   // uniform part
    (void)TileRequest<0, LPT>{};
    a.iw = __builtin_amdgcn_raw_buffer_load_b64(r_idx, on ? 8u * cl : off_range, 8u * cu, 0);
    a.qp[0] = 0;
    if (INT4) {
      (void)TileRequest<1, LPT>{};
      a.nib[0] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? 16u * cl : off_range, 16u * cu, 0);
      (void)TileRequest<2, LPT>{};                    // one of the three forms below
      const uint32_t qrow_l = rel * (uint32_t)g.groups_per_row;
      const uint32_t qrow_u = on ? (uint32_t)(16 * rt) * (uint32_t)g.groups_per_row : 0u;
      if (QW == 4) {
        const u4 v = __builtin_amdgcn_raw_buffer_load_b128(r_qp, on ? 4u * (qrow_l + 4u * lcc) : off_range,
                                                           on ? 4u * (qrow_u + 16u * (uint32_t)s) : 0u, 0);
#pragma unroll
        for (int k = 0; k < QW; ++k) a.qp[k] = v[k & 3];
      } else if (QW == 2) {
        const u2 v = __builtin_amdgcn_raw_buffer_load_b64(r_qp, on ? 4u * (qrow_l + 2u * lcc) : off_range,
                                                          on ? 4u * (qrow_u + 8u * (uint32_t)s) : 0u, 0);
#pragma unroll
        for (int k = 0; k < QW; ++k) a.qp[k] = v[k & 1];
      } else {
        a.qp[0] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, on ? 4u * (qrow_l + (lcc >> g.gshift)) : off_range,
                                                       on ? 4u * (qrow_u + (uint32_t)((4 * s) >> g.gshift)) : 0u, 0);
      }
    } else if (LINA) {
      const uint32_t vrow = (uint32_t)min((int)in_vgpr((uint32_t)i), g.rows - 1 - 16 * rt);
      const uint32_t vl = on ? 64u * vrow * (uint32_t)g.nchunks + 16u * (uint32_t)kb : off_range;
      (void)TileRequest<VW, LPT>{};                   // requests 1 .. VW
#pragma unroll
      for (int k = 0; k < VW; ++k)                    // chunk k of the step (clamped: uniform)
        a.nib[k] = __builtin_amdgcn_raw_buffer_load_b128(r_val, vl, on ? 64u * (cu + (uint32_t)min(k, g.nchunks - 1 - 4 * s)) : 0u, 0);
    } else {
      (void)TileRequest<VW, LPT>{};                   // requests 1 .. VW
#pragma unroll
      for (int k = 0; k < VW; ++k)
        a.nib[k] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? 64u * cl + 16u * k : off_range, 64u * cu, 0);
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
    } else if (LINA) {
      // The index word of chunk c (four 16-bit fields, one per piece) was fetched by lane
      // 4 r + c; instruction k wants field kb of the word of chunk k in lane (i, kb):
      // a 4 x 4 transpose over the four lanes of the row, then the lane exchange.
      const uint32_t c = (uint32_t)(lane & 3);
      const uint32_t lo_sel = 0x0c0c0100u + c * 0x0202u, hi_sel = 0x01000c0cu + c * 0x02020000u;
      const uint32_t a0 = quad_bcast<0>(a.iw[0]), b0 = quad_bcast<0>(a.iw[1]);
      const uint32_t a1 = quad_bcast<1>(a.iw[0]), b1 = quad_bcast<1>(a.iw[1]);
      const uint32_t a2 = quad_bcast<2>(a.iw[0]), b2 = quad_bcast<2>(a.iw[1]);
      const uint32_t a3 = quad_bcast<3>(a.iw[0]), b3 = quad_bcast<3>(a.iw[1]);
      const uint32_t w01 = __builtin_amdgcn_perm(b0, a0, lo_sel) | __builtin_amdgcn_perm(b1, a1, hi_sel);
      const uint32_t w23 = __builtin_amdgcn_perm(b2, a2, lo_sel) | __builtin_amdgcn_perm(b3, a3, hi_sel);
      a.iw[0] = lane_perm(from, w01);
      a.iw[1] = lane_perm(from, w23);
    }
  };
  // This wave's slice of X for token group j goes from global memory straight into its
  // LDS region: lane l of a request delivers to byte 16 l of one kilobyte.
  //   2:4 (512 B per token): request u covers tokens 2 u and 2 u + 1 and lands at
  //     1056 u.  The odd token of a pair has neighbouring 16-byte pieces swapped (piece
  //     q at slot q ^ 1) and pairs are 32 B apart modulo the bank cycle, so the sixteen
  //     lanes of a B read (one token each, same piece) fall into different banks.
  //   1:4 (1 KiB per token): request u is token u and lands at 1040 u.
  // Pairs (tokens) past M are not fetched and the odd token past an odd M repeats token
  // M - 1: whatever LDS holds there only reaches columns of the products that are never
  // stored.  Pieces past the end of a row of X repeat the last one (and are zeroed later).
  const int xtl = lane >> 5;
  const int slot_piece = N1 ? lane : ((lane & 31) ^ xtl);      // piece of X this lane delivers
  auto dma_x = [&](int j, int step) {
    const int s = min(step, nsteps - 1);
    const int vp = min(PIECES, g.kpieces - PIECES * s);         // pieces of the step inside K
    const uint32_t xs0 = (uint32_t)(16 * PIECES) * (uint32_t)s;
    const uint32_t off_lo = 16u * (uint32_t)min(slot_piece, vp - 1);
    const uint32_t off_hi = off_lo + (uint32_t)xtl * (uint32_t)(2 * g.ldx);
    asm volatile("" ::: "memory");                    // the requests stay together, in program order
    if (N1) {
#pragma unroll
      for (int u = 0; u < 16; ++u) {
        const int t0 = 16 * j + u;
        if (t0 < g.M)                                 // uniform
          __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(region + KS_TOKEN_N1 * u),
                                                   16, off_lo, xs0 + (uint32_t)t0 * (uint32_t)(2 * g.ldx), 0, 0);
      }
    } else {
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t0 = 16 * j + 2 * u;
        if (t0 < g.M)                                 // uniform
          __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(region + KS_PAIR * u),
                                                   16, t0 + 1 < g.M ? off_hi : off_lo,
                                                   xs0 + (uint32_t)t0 * (uint32_t)(2 * g.ldx), 0, 0);
      }
    }
    asm volatile("" ::: "memory");
  };
  // the pieces of a partly filled step that lie past K become zeros
  auto zero_tail = [&](int step) {
    const int vp = g.kpieces - PIECES * step;
    if (vp < PIECES && slot_piece >= vp) {
#pragma unroll
      for (int u = 0; u < (N1 ? 16 : 8); ++u)
        *(u4 *)(region + (N1 ? KS_TOKEN_N1 : KS_PAIR) * u + 16 * lane) = u4{0, 0, 0, 0};
    }
  };
  // B operand: lane (n, b) holds token n, k-octets b and 4 + b of the 16-column group of
  // each instruction, i.e. the pieces 16 h + 8 (b >> 1) + 2 d + (b & 1) of the step at 2:4
  // and 32 h + 16 (b >> 1) + 2 m + (b & 1) at 1:4, for h = 0, 1
  auto read_b = [&](u8v (&bx)[NM]) {
    const int n = lane & 15, b = lane >> 4;
    // (LINA: pieces 8 m + b and 8 m + 4 + b, instruction m being chunk m of the step)
    const uint8_t *base0 = N1     ? region + KS_TOKEN_N1 * n + 16 * (16 * (b >> 1) + (b & 1))
                           : LINA ? region + KS_PAIR * (n >> 1) + 512 * (n & 1) + 16 * (b ^ (n & 1))
                                  : region + KS_PAIR * (n >> 1) + 512 * (n & 1) + 16 * (8 * (b >> 1) + ((b ^ n) & 1));
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const u4 v = *(const u4 *)(base0 + (N1 ? 512 : LINA ? 64 : 256) * h + (LINA ? 128 : 32) * m);
#pragma unroll
        for (int k = 0; k < 4; ++k) bx[m][4 * h + k] = v[k];
      }
    }
  };
  // operands of the NM instructions of a step: values av[m], index words iwv[m >> 1]
  // (instruction m takes the low half of its word for even m, the high half for odd m)
  auto operands = [&](const ATile<KIND, QW> &t, int step, u4 (&av)[NM], uint32_t (&iwv)[NM / 2]) {
    const bool live = 4 * step + kb < g.nchunks;      // false: a chunk past the end of K
    uint32_t s2[QW], off[QW];
#pragma unroll
    for (int k = 0; k < QW; ++k) {
      s2[k] = off[k] = 0;
      if (INT4) {
        s2[k] = __builtin_amdgcn_perm(t.qp[k], t.qp[k], 0x01000100u);
        if (!live) s2[k] = 0;
        off[k] = pk_add_f16(__builtin_amdgcn_perm(t.qp[k], t.qp[k], 0x03020302u), g.nib_magic);
      }
    }
    if (N1) {
      iwv[0] = spread_idx(t.iw[0] & 0xFFFFu, g.m8, g.m4, g.m2);
      iwv[1] = spread_idx(t.iw[0] >> 16, g.m8, g.m4, g.m2);
      iwv[NM / 2 - 2] = spread_idx(t.iw[1] & 0xFFFFu, g.m8, g.m4, g.m2);
      iwv[NM / 2 - 1] = spread_idx(t.iw[1] >> 16, g.m8, g.m4, g.m2);
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        if constexpr (INT4) {
          // slots 4 m .. 4 m + 3 = bytes 2 (m & 1), 2 (m & 1) + 1 of dword m >> 1; the two
          // slots of a byte are dequantised as a pair, then split into {w, 0} registers
          const uint32_t d = t.nib[0][(m >> 1) & 3];
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t t2 = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)(2 * (m & 1) + p) * 0x00010001u);
            const uint32_t pair = pk_mul_f16(pk_sub_f16(and_or(t2, g.nib_mask, magic), off[m * QW / 8]), s2[m * QW / 8]);
            av[m][2 * p] = pair & 0xFFFFu;
            av[m][2 * p + 1] = pair >> 16;
          }
        } else {
          const uint32_t v0 = live ? t.nib[(m >> 1) & 3][2 * (m & 1)] : 0u;
          const uint32_t v1 = live ? t.nib[(m >> 1) & 3][2 * (m & 1) + 1] : 0u;
          av[m] = u4{v0 & 0xFFFFu, v0 >> 16, v1 & 0xFFFFu, v1 >> 16};
        }
      }
    } else if constexpr (LINA) {
      iwv[0] = t.iw[0];
      iwv[NM / 2 - 1] = t.iw[1];
#pragma unroll
      for (int d = 0; d < NM; ++d) av[d] = 4 * step + d < g.nchunks ? t.nib[d & 3] : u4{0, 0, 0, 0};   // uniform
    } else {
      iwv[0] = t.iw[0];
      iwv[NM / 2 - 1] = t.iw[1];
#pragma unroll
      for (int d = 0; d < NM; ++d) {
        if constexpr (INT4) av[d] = dequant8(t.nib[0][d & 3], off[(d & 3) * QW / 4], s2[(d & 3) * QW / 4], g.nib_mask, magic);
        else av[d] = live ? t.nib[d & 3] : u4{0, 0, 0, 0};
      }
    }
  };
  auto mfma_step = [&](const u4 (&av)[NM], const uint32_t (&iwv)[NM / 2], const u8v (&bx)[NM], f4 &acc) {
#pragma unroll
    for (int m = 0; m < NM; ++m) {
      const int iword = (int)iwv[m >> 1];
      if (m & 1)
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[m]), __builtin_bit_cast(h16, bx[m]), acc, iword, 0, 1);
      else
        acc = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[m]), __builtin_bit_cast(h16, bx[m]), acc, iword, 0, 0);
    }
  };

  ATile<KIND, QW> raw[NIT], raw2[DEEP ? NIT : 1];
  // first requests of a pass: X and the A tiles of phase 0 (DEEP: and the tiles of phase 1)
  auto start_pass = [&](int rr, int j) {
    dma_x(j, step0 + wave);
#pragma unroll
    for (int it = 0; it < NIT; ++it) load_a(raw[it], it, step0 + wave, rr);
    if (DEEP && phases > 1) {
#pragma unroll
      for (int it = 0; it < NIT; ++it) load_a(raw2[it], it, step0 + wave + nw, rr);
    }
  };
  start_pass(0, 0);
  int r = 0;                                          // the round being computed
  for (int j0 = 0; RND || j0 < ngroups;) {            // work items: (round r, pass of NT token groups from j0)
    const int nit = tiles_of(r);
    f4 acc[NIT][NT];
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
      for (int jj = 0; jj < NT; ++jj) acc[it][jj] = f4{0.f, 0.f, 0.f, 0.f};

    // A wave whose last step lies past K (K-steps not a multiple of the waves) skips
    // that phase; it is the last one, nothing is requested in it.
    // DEEP: pending at the top of phase p are, in request order, A(p), X(p), A(p + 1)
    auto deep_phase = [&](ATile<KIND, QW> (&cur)[NIT], int p) {
      constexpr int NA = NIT * LPT;
      const int step = step0 + p * nw + wave;
      u8v bx[NM];
      ATile<KIND, QW> t[NIT];
      if (p + 1 >= phases) {
        // last phase: the tiles are consumed as they arrive
        wait_vmem<(NIT - 1) * LPT>();
        zero_tail(step);
        read_b(bx);
        static_for<0, NIT>([&](auto ic) {
          constexpr int it = decltype(ic)::v;
          if constexpr (it > 0) wait_vmem<(NIT - 1 - it) * LPT>();
          if (it < nit) {
            ATile<KIND, QW> tl = cur[it];
            to_operand(tl);
            u4 av[NM];
            uint32_t iwv[NM / 2];
            operands(tl, step, av, iwv);
            mfma_step(av, iwv, bx, acc[it][0]);
          }
        });
        return;
      }
      wait_vmem<NA>();
      zero_tail(step);
      read_b(bx);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        t[it] = cur[it];
        to_operand(t[it]);
      }
      wait_lds();
      if (p + 1 < phases) dma_x(j0, step + nw);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        if (it < nit) {
          u4 av[NM];
          uint32_t iwv[NM / 2];
          operands(t[it], step, av, iwv);
          mfma_step(av, iwv, bx, acc[it][0]);
        }
        if (p + 2 < phases) load_a(cur[it], it, step + 2 * nw, r);
      }
    };
    if constexpr (DEEP) {
      for (int p = 0; p < phases && step0 + p * nw + wave < nsteps; p += 2) {
        deep_phase(raw, p);
        if (p + 1 < phases && step0 + (p + 1) * nw + wave < nsteps) deep_phase(raw2, p + 1);
      }
    }
    for (int p = 0; !DEEP && p < phases && step0 + p * nw + wave < nsteps; ++p) {
      const int step = step0 + p * nw + wave;
      const bool more = p + 1 < phases;
      constexpr int NA = NIT * LPT;                    // loads of the A tiles of one phase (any QW)
      u8v bx[NM];
      ATile<KIND, QW> t[NIT];
      if constexpr (!HOLD) {
        if (!more) {
          // Last phase: nothing more is requested, so the tiles are consumed as they arrive
          // (loads return in request order: X first, then tile 0, 1, ...).
          wait_vmem<(NIT - 1) * LPT>();
          zero_tail(step);
          read_b(bx);
          static_for<0, NIT>([&](auto ic) {
            constexpr int it = decltype(ic)::v;
            if constexpr (it > 0) wait_vmem<(NIT - 1 - it) * LPT>();
            if (it < nit) {
              ATile<KIND, QW> tl = raw[it];
              to_operand(tl);
              u4 av[NM];
              uint32_t iwv[NM / 2];
              operands(tl, step, av, iwv);
              mfma_step(av, iwv, bx, acc[it][0]);
            }
          });
          continue;
        }
      }
      wait_vmem<0>();                                 // X and the A tiles of this phase have arrived
      zero_tail(step);
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
          for (int it = 0; it < NIT; ++it) load_a(raw[it], it, step + nw, r);
        }
        u4 held[NIT][NM];
        uint32_t hiw[NIT][NM / 2];
#pragma unroll
        for (int it = 0; it < NIT; ++it) operands(t[it], step, held[it], hiw[it]);
#pragma unroll
        for (int jj = 0; jj < NT; ++jj) {
          if (j0 + jj < ngroups) {                    // uniform
            if (jj > 0) {
              if (more) wait_vmem<NA>(); else wait_vmem<0>();
              zero_tail(step);
              read_b(bx);
              wait_lds();
              if (jj + 1 < NT && j0 + jj + 1 < ngroups) dma_x(j0 + jj + 1, step);
              else if (more) dma_x(j0, step + nw);
            }
#pragma unroll
            for (int it = 0; it < NIT; ++it)
              if (it < nit) mfma_step(held[it], hiw[it], bx, acc[it][jj]);
          }
        }
      } else {
        if (more) dma_x(j0, step + nw);
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          if (it < nit) {
            u4 av[NM];
            uint32_t iwv[NM / 2];
            operands(t[it], step, av, iwv);
            mfma_step(av, iwv, bx, acc[it][0]);
          }
          if (more) load_a(raw[it], it, step + nw, r);  // into the registers this tile has just left
        }
      }
    }
    // the next work item: the next pass over the same row tiles, else the next round
    const bool same_round = j0 + NT < ngroups;
    const int rn = (!RND || same_round) ? r : r + 1, jn = same_round ? j0 + NT : 0;
    const bool more_work = RND ? rn < rounds : same_round;   // uniform over the workgroup
    if (SEP) {
      if (more_work) {                                // (the region is free)
        if (!same_round) frp_next = load_rp(rn);
        start_pass(rn, jn);
      }
    } else {
      wait_vmem<0>();                                 // a wave that left early may still have X on its way
    }

    // ---- partial sums to LDS: tile (it, jj) of wave w at w * PSTRIDE + (it * NT + jj) * 1024,
    //      float 4 * lane + v = D[row 4 (lane >> 4) + v][token lane & 15]
    if (threadIdx.x < 16 * NIT)
      flags[threadIdx.x] = ((RND ? flag_checked(r) : fcheck0) && frp == (uint32_t)flag_row(r) * S_row) ? 1u : 0u;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
      for (int jj = 0; jj < NT; ++jj)
        if (it < nit) *(f4 *)(parts + wave * PSTRIDE + (it * NT + jj) * 1024 + 16 * lane) = acc[it][jj];
    lds_barrier();
    for (int unit = threadIdx.x; unit < NIT * NT * 256; unit += (int)blockDim.x) {
      const int tj = unit >> 8, it = tj / NT, jj = tj % NT;
      if (it >= nit || j0 + jj >= ngroups) continue;  // uniform over a wave
      const int v = unit & 3, sl = (unit >> 2) & 63;  // register v of lane sl of the tile
      const float *src = (const float *)parts + unit;
      float part[NWMAX];
#pragma unroll
      for (int w = 0; w < NWMAX; ++w) part[w] = src[min(w, nw - 1) * (PSTRIDE / 4)];
      float sum = 0.f;
#pragma unroll
      for (int w = 0; w < NWMAX; ++w) sum += w < nw ? part[w] : 0.f;
      const int row0 = 16 * ((int)blockIdx.x + (r * NIT + it) * (int)gridDim.x) + 4 * (sl >> 4);
      const int row = row0 + v;
      const int tok = 16 * (j0 + jj) + (sl & 15);
      if constexpr (KS) {
        // partial sum of this slice; a row with a broken pointer gets NaN from every slice
        if (tok < g.M && row < g.rows)
          g.ws[((int64_t)blockIdx.y * g.M + tok) * g.ws_ld + row] = flags[16 * it + 4 * (sl >> 4) + v] ? sum : __builtin_nanf("");
        continue;
      }
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
    if (!more_work) break;
    lds_barrier();                                    // the next work item writes the partial sums (and X regions) again
    if (!SEP) {
      if (!same_round) frp_next = load_rp(rn);
      start_pass(rn, jn);
    }
    if (!same_round) frp = frp_next;
    r = rn;
    j0 = jn;
  }
}

template <int KIND, int NT, int NIT, int NWMAX, int QW, bool N1, bool RND, bool KS = false>
__global__ __launch_bounds__(64 * NWMAX) void k_sparse_smallm_ks(const uint32_t *__restrict__ row_ptr,
                                                                  const uint8_t *__restrict__ values,
                                                                  const uint8_t *__restrict__ idx,
                                                                  const uint8_t *__restrict__ qparams,
                                                                  const __half *__restrict__ X,
                                                                  __half *__restrict__ Y,
                                                                  const SmallMKsGeom g) {
  smallm_ks_body<KIND, NT, NIT, NWMAX, QW, N1, RND, KS>(row_ptr, values, idx, qparams, X, Y, g);
}

// Up to four identically shaped products (the q/k/v or gate/up projections under the same
// tokens or under tokens of their own) in one launch: blockIdx.y names the member, whose
// workgroups run the very body of the single-matrix kernel.
struct SmallMBatch {
  const uint32_t *row_ptr[EGT_MAX_BATCH];
  const uint8_t *values[EGT_MAX_BATCH], *idx[EGT_MAX_BATCH], *qparams[EGT_MAX_BATCH];
  const __half *X[EGT_MAX_BATCH];
  __half *Y[EGT_MAX_BATCH];
};
template <int KIND, int NT, int NIT, int NWMAX, int QW, bool N1, bool RND>
__global__ __launch_bounds__(64 * NWMAX) void k_sparse_smallm_ks_batch(const SmallMBatch b, const SmallMKsGeom g) {
  const unsigned k = blockIdx.y;
  smallm_ks_body<KIND, NT, NIT, NWMAX, QW, N1, RND, false>(pick4(b.row_ptr, k), pick4(b.values, k), pick4(b.idx, k), pick4(b.qparams, k),
                                                           pick4(b.X, k), pick4(b.Y, k), g);
}

// Shapes covered: 2:4 with K a multiple of 64, 1:4 with K a multiple of 128; INT4 groups
// of 32 << j; token rows of X on a dword boundary; values and X below 4 GiB each (the
// loads take 32-bit offsets).
bool sparse_smallm_supported(const egt_2bitcsr &w, int64_t ldx, int M) {
  if (w.n_keep != 1 && w.n_keep != 2) return false;
  if (w.val_kind != EGT_VAL_INT4 && w.val_kind != EGT_VAL_FP16) return false;   // the paired nibble order has no small-M kernel
  const int chunk = w.n_keep == 1 ? 128 : 64;
  if (w.cols % chunk != 0 || w.cols < chunk || ldx % 2 != 0) return false;
  const uint64_t vbytes = (uint64_t)w.rows * (w.cols / chunk) * (w.val_kind == EGT_VAL_INT4 ? 16 : 64);
  const uint64_t xbytes = ((uint64_t)(M - 1) * ldx + w.cols) * 2;
  if (vbytes >= (1ull << 32) || xbytes >= (1ull << 32)) return false;
  if (w.val_kind == EGT_VAL_INT4) {
    const int gm = w.group_size / 32;
    if (w.group_size % 32 != 0 || (gm & (gm - 1)) != 0) return false;
  }
  return true;
}

// Y[m][r] = FP16( sum over the K slices, in slice order, of the partial sums the split
// kernel left in the workspace ).  One thread per output; a NaN partial (broken row
// pointer) gives the library's NaN pattern.
__global__ __launch_bounds__(256) void k_smallm_sum_slices(const float *__restrict__ ws, int64_t ws_ld, int nslices, int M,
                                                           int rows, __half *__restrict__ Y, int64_t ldy) {
  const int r = blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
  if (r >= rows) return;
  // (four slices requested before the first is added; the additions stay in ascending slice order)
  float sum = 0.f;
  for (int s0 = 0; s0 < nslices; s0 += 4) {
    float p[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) p[k] = ws[((int64_t)min(s0 + k, nslices - 1) * M + m) * ws_ld + r];
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (s0 + k < nslices) sum += p[k];
  }
  Y[(int64_t)m * ldy + r] = sum != sum ? __ushort_as_half((uint16_t)0x7E00) : __float2half(sum);
}

template <int KIND, int NT, int NIT, int NWMAX, int QW, bool N1, bool RND, bool KS = false>
static hipError_t go_ks(const egt_2bitcsr &w, const uint16_t *X, uint16_t *Y, const SmallMKsGeom &g, int nw,
                        int nblocks, hipStream_t stream, const SmallMBatch *batch = nullptr, int count = 1) {
  const size_t region = N1 ? 16 * KS_TOKEN_N1 : 8 * KS_PAIR;
  const size_t x_bytes = (size_t)nw * region, p_bytes = (size_t)nw * NIT * NT * 1024;
  // partial sums behind the X regions where the kernel keeps them apart (NT > 1), else at
  // the start of each wave's own region; + row-pointer flags
  const size_t lds = (NT > 1 ? x_bytes + p_bytes : x_bytes) + 64 * NIT;
  if constexpr (!KS) {
    if (batch)
      return launch(k_sparse_smallm_ks_batch<KIND, NT, NIT, NWMAX, QW, N1, RND>, dim3(nblocks, count), dim3(64 * nw), lds, stream, *batch, g);
  }
  return launch(k_sparse_smallm_ks<KIND, NT, NIT, NWMAX, QW, N1, RND, KS>, dim3(nblocks, KS ? g.nslices : 1), dim3(64 * nw),
                lds, stream, w.row_ptr, (const uint8_t *)w.values, (const uint8_t *)w.idx, (const uint8_t *)w.qparams,
                (const __half *)X, (__half *)Y, g);
}

static void smallm_geometry(const egt_2bitcsr &w, int64_t ldx, uint16_t *Y, int64_t ldy, int M, SmallMKsGeom &g, int &qw) {
  const bool int4 = w.val_kind == EGT_VAL_INT4, n1 = w.n_keep == 1;
  const int chunk = n1 ? 128 : 64;
  g.rows = w.rows; g.M = M;
  g.nchunks = w.cols / chunk;
  g.nsteps = (g.nchunks + 3) / 4;
  g.kpieces = w.cols / 8;
  g.ntiles = (w.rows + 15) / 16;
  g.gshift = 0; g.groups_per_row = 0;
  qw = 1;                                             // {scale, zero} pairs per chunk
  if (int4) {
    if (w.group_size < chunk) qw = chunk / w.group_size;
    while ((chunk << g.gshift) < w.group_size) ++g.gshift;
    g.groups_per_row = w.cols / w.group_size;
  }
  g.ldx = ldx; g.ldy = ldy;
  g.vec_store = ((uintptr_t)Y % 8 == 0 && ldy % 4 == 0) ? 1 : 0;
  const uint64_t chunks = (uint64_t)w.rows * g.nchunks;
  g.val_bytes = (uint32_t)(chunks * (int4 ? 16 : 64)); g.idx_bytes = (uint32_t)(chunks * 8);
  g.qp_bytes = (uint32_t)((uint64_t)w.rows * g.groups_per_row * 4);
  g.x_bytes = (uint32_t)(((uint64_t)(M - 1) * ldx + w.cols) * 2);
  g.nib_mask = 0x00F0000Fu; g.nib_magic = 0x54006400u;
  g.m8 = 0x00FF00FFu; g.m4 = 0x0F0F0F0Fu; g.m2 = 0x33333333u;
  g.nslices = 1; g.ws_ld = 0; g.ws = nullptr;
}

// K split over workgroups: at larger M every compute unit pulls the whole of X (M * K * 2
// bytes) through its XCD's L2, which is what bounds the one-launch kernel when K is large
// and the rows are few (the down projection: 4096 x 11008).  With the grid cut into row
// blocks x K slices a workgroup needs only its slice of X, at the price of FP32 partial
// sums that pass through a workspace and a second, small kernel that adds them in slice
// order.  That price is only recovered where a workgroup still gets by with one round of
// row tiles (a second round would fetch its X slice again), and measured it is: 2:4 INT4,
// one {scale, zero} pair per chunk, more than 16 tokens, K >= 8192 and at most 256 row
// tiles - four slices, a quarter of the row tiles per workgroup column (4096 x 11008:
// 21.9 against 24.9 us at M = 64, 14.3 against 14.9 at M = 32; with more rows, e.g.
// 11008 x 4096, every split measured was slower than the one-launch kernel).
// Returns the number of slices (1: no split) and the row blocks.
static int smallm_slices(const egt_2bitcsr &w, int M, int &row_blocks) {
  row_blocks = 0;
  if (w.val_kind != EGT_VAL_INT4 || w.n_keep != 2 || w.group_size < 64 || w.rows < 16) return 1;
  const int nsteps = (w.cols / 64 + 3) / 4, ntiles = (w.rows + 15) / 16;
  int s = (M > 16 && nsteps >= 32 && ntiles <= 256) ? 4 : 1;
  int blocks = (ntiles + 3) / 4;
  tune_pair("EGT_SM_KS", s, blocks);                   // developer build: any split, for timing
  if (M < 5 || s < 2 || s > 16 || s > nsteps) return 1;
  if (blocks < 1) blocks = 1;
  if (blocks > ntiles) blocks = ntiles;
  row_blocks = blocks;
  return s;
}

// the form with X held still in LDS (egt_mfma_smallm_xs.hip)
size_t sparse_smallm_xs_bytes(const egt_2bitcsr &w, int64_t ldx, int M, bool force);
hipError_t launch_sparse_smallm_xs(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y, int64_t ldy, int M,
                                   float *ws, bool force, hipStream_t stream);
static bool use_xs(const egt_2bitcsr &w, int64_t ldx, int M, size_t &bytes, bool &force) {
  force = tune_flag("EGT_SM_XS");                     // developer build: wherever the form applies
  if (tune_flag("EGT_SM_NOXS")) return false;
  bytes = sparse_smallm_xs_bytes(w, ldx, M, force);
  return bytes != 0;
}

bool sparse_smallm_split_bytes(const egt_2bitcsr &w, int64_t ldx, int M, size_t &bytes) {
  int row_blocks;
  bytes = 0;
  if (!sparse_smallm_supported(w, ldx, M)) return false;
  bool force;
  if (use_xs(w, ldx, M, bytes, force)) return true;
  const int s = smallm_slices(w, M, row_blocks);
  if (s < 2) return false;
  bytes = sizeof(float) * (size_t)s * (size_t)M * (size_t)w.rows;
  return true;
}

hipError_t launch_sparse_smallm_split(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y, int64_t ldy, int M,
                                      float *ws, hipStream_t stream) {
  if (w.rows == 0) return hipSuccess;
  {
    size_t xs_bytes;
    bool force;
    if (use_xs(w, ldx, M, xs_bytes, force)) return launch_sparse_smallm_xs(w, X, ldx, Y, ldy, M, ws, force, stream);
  }
  SmallMKsGeom g;
  int qw, row_blocks;
  smallm_geometry(w, ldx, Y, ldy, M, g, qw);
  g.nslices = smallm_slices(w, M, row_blocks);
  g.ws = ws; g.ws_ld = w.rows;
  const bool wide = M > 16;
  const int nwmax = wide ? 8 : 16;
  const int min_steps = g.nsteps / g.nslices;          // the shortest slice
  const int nw = min_steps < nwmax ? min_steps : nwmax;
  const int nblocks = row_blocks;
  const bool one = nblocks == g.ntiles;
  hipError_t e;
#define EGT_KSS(NT, NIT, NWMAX)                                                                              \
  ((NIT > 1 && (int64_t)nblocks * NIT < g.ntiles) ? go_ks<EGT_VAL_INT4, NT, NIT, NWMAX, 1, false, (NIT > 1), true>(w, X, Y, g, nw, nblocks, stream) \
                                                  : go_ks<EGT_VAL_INT4, NT, NIT, NWMAX, 1, false, false, true>(w, X, Y, g, nw, nblocks, stream))
  if (!wide) e = one ? EGT_KSS(1, 1, 16) : EGT_KSS(1, 3, 16);
  else e = one ? EGT_KSS(2, 1, 8) : EGT_KSS(2, 4, 8);
#undef EGT_KSS
  if (e != hipSuccess) return e;
  return launch(k_smallm_sum_slices, dim3((w.rows + 255) / 256, M), dim3(256), 0, stream, (const float *)ws, g.ws_ld,
                g.nslices, M, w.rows, (__half *)Y, ldy);
}

static hipError_t smallm_one_launch(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                    int64_t ldy, int M, hipStream_t stream, const SmallMBatch *batch, int count) {
  if (w.rows == 0) return hipSuccess;
  const bool int4 = w.val_kind == EGT_VAL_INT4, n1 = w.n_keep == 1;
  SmallMKsGeom g;
  int qw;
  {
    const uint64_t chunks = (uint64_t)w.rows * (uint64_t)(w.cols / (n1 ? 128 : 64));
    const uint64_t vb = chunks * (int4 ? 16 : 64), xb = ((uint64_t)(M - 1) * ldx + w.cols) * 2;
    if (vb >= (1ull << 32) || xb >= (1ull << 32)) return hipErrorInvalidValue;   // 32-bit offsets
  }
  smallm_geometry(w, ldx, Y, ldy, M, g, qw);
  if (batch)                                          // 8-byte stores only where every member's Y allows them
    for (int k = 0; k < count; ++k)
      if ((uintptr_t)batch->Y[k] % 8 != 0) g.vec_store = 0;
  // One workgroup per compute unit while its row tiles fit the registers (NIT of them).
  // 2:4 INT4, up to 16 tokens: 16 waves of 128 registers; everything else 8 waves of 256
  // (more than 16 tokens at 2:4: two token groups per pass).
  const bool wide = n1 || M > 16 || !int4;
  const bool f16x = !int4 && !n1 && M <= 16;          // FP16 values at 2:4, one token group
  int nwmax = wide ? 8 : 16, blocks_per_cu = 1;
  if (f16x && g.ntiles <= 256) nwmax = 16;            // one tile per workgroup: 16 waves of 128 registers
  {
    const int nwcap = (wide && !f16x) ? 8 : 16;
    tune_pair("EGT_SM_TUNE", nwmax, blocks_per_cu);
    nwmax = nwmax < 1 ? 1 : nwmax > nwcap ? nwcap : nwmax;
    blocks_per_cu = blocks_per_cu < 1 ? 1 : blocks_per_cu > 4 ? 4 : blocks_per_cu;
  }
  int nblocks = 256 * blocks_per_cu;                  // more row tiles than nblocks * NIT: rounds in the kernel
  if (nblocks > g.ntiles) nblocks = g.ntiles;
  const bool one = nblocks == g.ntiles;               // one row tile per workgroup
  if (f16x && !one && nwmax > 8) nwmax = 8;           // several tiles with FP16 values: 8 waves of 256 registers
  const int nw = g.nsteps < nwmax ? g.nsteps : nwmax;
  // (NIT > 1: the form with rounds only where a workgroup owns more than NIT row tiles)
#define EGT_KS(KIND, NT, NIT, NWMAX, QW, N1)                                                     \
  ((NIT > 1 && (int64_t)nblocks * NIT < g.ntiles) ? go_ks<KIND, NT, NIT, NWMAX, QW, N1, (NIT > 1)>(w, X, Y, g, nw, nblocks, stream, batch, count) \
                                                  : go_ks<KIND, NT, NIT, NWMAX, QW, N1, false>(w, X, Y, g, nw, nblocks, stream, batch, count))
  if (n1) {
    if (!int4) return one ? EGT_KS(EGT_VAL_FP16, 1, 1, 8, 1, true) : EGT_KS(EGT_VAL_FP16, 1, 4, 8, 1, true);
    if (qw == 4) return one ? EGT_KS(EGT_VAL_INT4, 1, 1, 8, 4, true) : EGT_KS(EGT_VAL_INT4, 1, 4, 8, 4, true);
    if (qw == 2) return one ? EGT_KS(EGT_VAL_INT4, 1, 1, 8, 2, true) : EGT_KS(EGT_VAL_INT4, 1, 4, 8, 2, true);
    return one ? EGT_KS(EGT_VAL_INT4, 1, 1, 8, 1, true) : EGT_KS(EGT_VAL_INT4, 1, 4, 8, 1, true);
  }
  if (int4 && qw == 2) {
    if (!wide) return one ? EGT_KS(EGT_VAL_INT4, 1, 1, 16, 2, false) : EGT_KS(EGT_VAL_INT4, 1, 3, 16, 2, false);
    return one ? EGT_KS(EGT_VAL_INT4, 2, 1, 8, 2, false) : EGT_KS(EGT_VAL_INT4, 2, 4, 8, 2, false);
  }
  if (int4) {
    if (!wide) return one ? EGT_KS(EGT_VAL_INT4, 1, 1, 16, 1, false) : EGT_KS(EGT_VAL_INT4, 1, 3, 16, 1, false);
    return one ? EGT_KS(EGT_VAL_INT4, 2, 1, 8, 1, false) : EGT_KS(EGT_VAL_INT4, 2, 4, 8, 1, false);
  }
  if (M <= 16) {
    if (one) return nw > 8 ? EGT_KS(EGT_VAL_FP16, 1, 1, 16, 1, false) : EGT_KS(EGT_VAL_FP16, 1, 1, 8, 1, false);
    return EGT_KS(EGT_VAL_FP16, 1, 4, 8, 1, false);
  }
  return one ? EGT_KS(EGT_VAL_FP16, 2, 1, 8, 1, false) : EGT_KS(EGT_VAL_FP16, 2, 4, 8, 1, false);
#undef EGT_KS
}

hipError_t launch_sparse_smallm(const egt_2bitcsr &w, const uint16_t *X, int64_t ldx, uint16_t *Y,
                                int64_t ldy, int M, hipStream_t stream) {
  return smallm_one_launch(w, X, ldx, Y, ldy, M, stream, nullptr, 1);
}

// ---- Any number of small-M products in one launch (a verification pass through a whole
// stack of 2:4 INT4 layers): a table in device memory of the caller holds a descriptor per
// matrix - pointers and geometry - and behind them a list of the workgroups of the launch.
// The single product has to spread one matrix over the whole chip: one 16-wave workgroup per
// compute unit, K split over its waves.  Such a workgroup runs its loads, products and the
// sum across waves one after the other, and nothing else is resident to fill the gaps.  A
// table offers many matrices at once, so the stack uses smaller workgroups, few per matrix,
// and the compute units work on several matrices at the same time (16 layers of a 7B stack,
// 1.3 GB: 347 us at 16 tokens against 951 us of single products replayed from a graph, 594
// against 2008 us at 64 tokens).  The host writes the descriptors in the order of falling row
// length, so that the launch ends on short workgroups.
struct SmallMStackEntry {
  uint64_t row_ptr, values, idx, qparams, X, Y;      // device addresses
  SmallMKsGeom g;
};
static_assert(sizeof(SmallMStackEntry) <= EGT_STACK_ENTRY_BYTES, "descriptor larger than the published entry size");

// Rows, not K, are split over the waves.
// With K split over the waves (the kernels above; the stack ran on that body first, 4 waves
// and three row tiles a round) every wave stages its own slice of X, and a round of
// row tiles pulls the whole of X through the L2: at 16 tokens and three tiles a round that is
// 128 KB of X for 61 KB of weights, and the counters show it (16 layers of a 7B stack: 5.9 GB
// from the L2 to the compute units for 1.36 GB of weights and tokens).  A table offers
// enough row tiles to fill the chip without cutting K, so here a workgroup of 8 waves owns 8
// consecutive row tiles for all of K, one tile per wave, in rounds of four K-steps (1024
// columns): the token rows of a round (32 KB) are staged once per workgroup - each wave
// requests an eighth - and read by all waves, and every wave keeps the sums of its tile in
// registers from the first K-step to the last: no sum across waves, the results go from the
// registers to Y.
// What a wave requests of its tile follows the cache lines.  A request of the kernel above
// covers one K-step of 16 rows: 64 B of nibbles, 32 B of idx words and 8 B of scales per row.
// There the waves of a workgroup ask for neighbouring K-steps at the same time; a wave that
// walks its rows alone, one K-step after the other, finds the rest of each line gone from the
// caches a step later (measured that way: 4.6 GB fetched for 1.36 GB).  Here a request covers
// 8 rows x 8 chunks - two K-steps, 128 B of nibbles per row - and the requests of a round are
// issued together.
// X of round j + 1 and the A tiles of round j + 2 are requested while round j is computed
// (two regions in LDS, one barrier a round, two sets of fetch registers).
// More than 16 tokens: NG token groups of 16.  The token rows of all groups are staged per
// round, the operands of a K-step are dequantised once and serve every group (NG sums per
// wave), and a round is two K-steps, so that the regions still fit: up to 32 tokens two
// groups and 8 waves (two workgroups per compute unit), beyond four groups and 16 waves.
#ifndef EGT_RS_WAVES
#define EGT_RS_WAVES 8
#endif
#ifndef EGT_RS_Q
#define EGT_RS_Q 4
#endif
constexpr int RS_WAVES = EGT_RS_WAVES, RS_Q = EGT_RS_Q, RS_BUFS = 2;
// LDS bytes of the token rows of one K-step and token group: 2:4 eight pairs of tokens (256 columns), 1:4 sixteen
// tokens of 512 columns
constexpr int rs_step_bytes(bool n1) { return n1 ? 16 * KS_TOKEN_N1 : 8 * KS_PAIR; }
// NG token groups of 16 (M <= 16 NG), rounds of Q K-steps: LDS bytes of a workgroup
constexpr int rs_lds_bytes(int ng, int q, bool n1 = false) { return RS_BUFS * ng * q * rs_step_bytes(n1); }

// N1: 1:4 sparsity (chunks of 128 columns, eight instructions a K-step, a request of X per token).
template <int NG, int Q, int W, bool N1 = false>
__global__ __launch_bounds__(64 * W, 4) void k_smallm_rows(const uint8_t *__restrict__ table, int count) {
  constexpr int RS_WAVES = W, RS_Q = Q, RS_STEP = rs_step_bytes(N1), RS_REGION = NG * Q * RS_STEP;
  constexpr int XREQ = N1 ? 16 : 8;                   // requests of X per K-step and token group
  constexpr int NM = N1 ? 8 : 4;                      // matrix instructions per K-step
  constexpr int PIECES = N1 ? 64 : 32;                // 16-byte pieces of a token row in a K-step
  constexpr int RS_REQ = NG * Q * XREQ / W;           // requests of X a wave issues per round
  static_assert(RS_REQ * W == NG * Q * XREQ && Q % 2 == 0, "the waves share the requests of a round evenly");
  extern __shared__ __align__(16) uint8_t xs[];       // RS_BUFS regions of RS_REGION bytes
  typedef __attribute__((address_space(1))) const uint32_t *g_u32;
  typedef __attribute__((address_space(1))) const uint8_t *g_u8;
  typedef __attribute__((address_space(1))) const __half *g_h;
  typedef __attribute__((address_space(1))) __half *g_hw;
  typedef ATile<EGT_VAL_INT4, 1> Tile;
  constexpr int LPT = Tile::LOADS;
  // the list behind the descriptors names the matrix (high half) and the workgroup's place in it (low half)
  const uint32_t where = ((const uint32_t *)(table + (size_t)count * EGT_STACK_ENTRY_BYTES))[blockIdx.x];
  const int wg = (int)(where & 0xFFFFu);
  const SmallMStackEntry *e = (const SmallMStackEntry *)(table + (size_t)(where >> 16) * EGT_STACK_ENTRY_BYTES);
  const SmallMKsGeom g = e->g;
  const uint32_t *row_ptr = (const uint32_t *)(g_u32)e->row_ptr;
  __half *Y = (__half *)(g_hw)e->Y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = lane & 15, kb = lane >> 4;            // operand form: row i of the tile, chunk kb of the step
  // this wave's row tile (a wave past the last tile has none, but still stages its share of X
  // and meets the barriers)
  const int tile = wg * RS_WAVES + wave;
  const bool has_tile = tile < g.ntiles;
  const int nsteps = g.nsteps, nrounds = (nsteps + RS_Q - 1) / RS_Q;
  const uint32_t magic = in_vgpr(g.nib_magic);
  const uint32_t S_row = (uint32_t)g.nchunks * 32u;
  // row pointers first, checked at the end: a row whose pointer is not r * S yields NaN
  const int frow = 16 * tile + lane;
  const bool fchecked = has_tile && lane < 16 && frow < g.rows;
  const uint32_t frp = fchecked ? row_ptr[frow] : 0u;

  const __amdgpu_buffer_rsrc_t r_val = make_rsrc((const uint8_t *)(g_u8)e->values, g.val_bytes);
  const __amdgpu_buffer_rsrc_t r_idx = make_rsrc((const uint8_t *)(g_u8)e->idx, g.idx_bytes);
  const __amdgpu_buffer_rsrc_t r_qp = make_rsrc((const uint8_t *)(g_u8)e->qparams, g.qp_bytes);
  const __amdgpu_buffer_rsrc_t r_x = make_rsrc((const __half *)(g_h)e->X, g.x_bytes);
  const uint32_t off_range = 0xFFFFFFF0u;             // past every buffer: such a request returns zeros and moves no data
  // A round of a tile is 16 rows x 16 chunks.  A request covers 8 rows x 8 chunks - lane
  // (r, c) = (lane >> 3, lane & 7, see below) fetches chunk 8 p + c of row 8 h + r: 128 contiguous bytes
  // of nibbles per row, whole cache lines - so four requests (h, p) per array fetch the round,
  // and request (h, p) holds the K-steps 2 p and 2 p + 1 of half h of the rows.
  struct RoundRegs {
    u4 nib[2][Q / 2];
    u2 iw[2][Q / 2];
    uint32_t qp[2][Q / 2];
  };
  // (rows 4 to 7 of a request keep their chunks in the other order of halves - lane (r, c) fetches chunk c ^ (r & 4):
  //  the lanes that a lane permutation reads for rows r and r + 4 then lie in different LDS banks)
  const int r8 = lane >> 3, c8 = (lane & 7) ^ ((lane >> 3) & 4);
  auto load_half = [&](RoundRegs &a, int round, int p) {   // the requests (0, p) and (1, p): 2 * LPT of them
    const bool on = has_tile && RS_Q * round + 2 * p < nsteps;                // uniform
    const int c0 = 4 * RS_Q * round + 8 * p;                                  // first chunk of the request
    const uint32_t lcc = (uint32_t)min((int)in_vgpr((uint32_t)c8), g.nchunks - 1 - c0);       // chunk inside the request (clamped)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t rel = (uint32_t)min(8 * h + r8, max(g.rows - 1 - 16 * tile, 0));          // row inside the tile (clamped)
      const uint32_t cl = rel * (uint32_t)g.nchunks + lcc;                    // lane part of the chunk number
      const uint32_t cu = on ? (uint32_t)(16 * tile) * (uint32_t)g.nchunks + (uint32_t)c0 : 0u;   // uniform part
      (void)TileRequest<0, LPT>{};
      a.iw[h][p] = __builtin_amdgcn_raw_buffer_load_b64(r_idx, on ? 8u * cl : off_range, 8u * cu, 0);
      (void)TileRequest<1, LPT>{};
      a.nib[h][p] = __builtin_amdgcn_raw_buffer_load_b128(r_val, on ? 16u * cl : off_range, 16u * cu, 0);
      (void)TileRequest<2, LPT>{};
      const uint32_t qrow_l = rel * (uint32_t)g.groups_per_row;
      const uint32_t qrow_u = on ? (uint32_t)(16 * tile) * (uint32_t)g.groups_per_row : 0u;
      a.qp[h][p] = __builtin_amdgcn_raw_buffer_load_b32(r_qp, on ? 4u * (qrow_l + (lcc >> g.gshift)) : off_range,
                                                        on ? 4u * (qrow_u + (uint32_t)(c0 >> g.gshift)) : 0u, 0);
    }
  };
  // operand of K-step q of the round: lane (i, kb) takes chunk 4 (q & 1) + kb of row i & 7 from
  // request (i >> 3, q >> 1): one lane permutation of either half, then the choice between them
  // (the chunk sits in lane 8 (i & 7) + (chunk ^ (i & 4)) of the request)
  const int from_even = 4 * (8 * (i & 7) + (kb ^ (i & 4)));
  const bool upper = i >= 8;
  auto pick = [&](int from, uint32_t lo, uint32_t hi) {
    const uint32_t a = lane_perm(from, lo), b = lane_perm(from, hi);
    return upper ? b : a;
  };
  auto to_operand = [&](const RoundRegs &a, int q, Tile &t) {
    const int from = from_even ^ (16 * (q & 1)), p = q >> 1;
#pragma unroll
    for (int d = 0; d < 4; ++d) t.nib[0][d] = pick(from, a.nib[0][p][d], a.nib[1][p][d]);
    t.iw[0] = pick(from, a.iw[0][p][0], a.iw[1][p][0]);
    t.iw[1] = pick(from, a.iw[0][p][1], a.iw[1][p][1]);
    t.qp[0] = pick(from, a.qp[0][p], a.qp[1][p]);
  };
  // X of a round: one request per token group, K-step and pair of tokens, each landing in one
  // kilobyte of the region ([group][K-step][pair], a K-step in the layout of the kernel above:
  // lane l delivers to byte 16 l; the odd token of a pair has neighbouring pieces swapped).
  // Every wave issues the same number of them, so that the wait counts are fixed; a pair past
  // M or a step past K asks out of range.
  const int xtl = lane >> 5;
  const int slot_piece = N1 ? lane : ((lane & 31) ^ xtl);   // piece of X this lane delivers
  auto dma_x = [&](int round, int buf) {
    asm volatile("" ::: "memory");                    // the requests stay together, in program order
#pragma unroll
    for (int k = 0; k < RS_REQ; ++k) {
      const int r = wave * RS_REQ + k;                // request r of the round: token group, K-step, pair of tokens (1:4: token)
      const int gq = r / XREQ, u = r % XREQ;          // (group, K-step) as one index: the region's order
      const int grp = gq / RS_Q, t0 = 16 * grp + (N1 ? u : 2 * u);
      const int step = RS_Q * round + gq % RS_Q;
      const int vp = max(1, min(PIECES, g.kpieces - PIECES * step));   // pieces of the step inside K
      const uint32_t off_lo = 16u * (uint32_t)min(slot_piece, vp - 1);
      const uint32_t off_hi = N1 ? off_lo : off_lo + (uint32_t)xtl * (uint32_t)(2 * g.ldx);
      const bool on = t0 < g.M && step < nsteps;      // uniform
      __builtin_amdgcn_raw_ptr_buffer_load_lds(r_x, (__attribute__((address_space(3))) void *)(xs + buf * RS_REGION + gq * RS_STEP + (N1 ? KS_TOKEN_N1 : KS_PAIR) * u), 16,
                                               on ? (t0 + 1 < g.M ? off_hi : off_lo) : off_range,
                                               on ? (uint32_t)(16 * PIECES) * (uint32_t)step + (uint32_t)t0 * (uint32_t)(2 * g.ldx) : 0u, 0, 0);
    }
    asm volatile("" ::: "memory");
  };
  // the pieces of a partly filled step that lie past K become zeros (the issuing wave's own requests)
  auto zero_tail = [&](int round, int buf) {
#pragma unroll
    for (int k = 0; k < RS_REQ; ++k) {
      const int r = wave * RS_REQ + k;
      const int vp = g.kpieces - PIECES * (RS_Q * round + (r / XREQ) % RS_Q);
      if (vp > 0 && vp < PIECES && slot_piece >= vp)
        *(u4 *)(xs + buf * RS_REGION + (r / XREQ) * RS_STEP + (N1 ? KS_TOKEN_N1 : KS_PAIR) * (r % XREQ) + 16 * lane) = u4{0, 0, 0, 0};
    }
  };
  // B operand of instruction m of a K-step (as in the kernel above: lane (n, b) holds token n,
  // k-octets b and 4 + b of the instruction's 16-column group)
  const int b_off = N1 ? KS_TOKEN_N1 * (lane & 15) + 16 * (16 * (lane >> 5) + ((lane >> 4) & 1))
                       : KS_PAIR * ((lane & 15) >> 1) + 512 * (lane & 1) + 16 * (8 * (lane >> 5) + (((lane >> 4) ^ lane) & 1));
  auto read_b = [&](const uint8_t *region, int m) {
    const u4 lo = *(const u4 *)(region + b_off + 32 * m), hi = *(const u4 *)(region + b_off + (N1 ? 512 : 256) + 32 * m);
    return u8v{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  };

  f4 acc[NG];
#pragma unroll
  for (int grp = 0; grp < NG; ++grp) acc[grp] = f4{0.f, 0.f, 0.f, 0.f};
  // The A tiles are requested two rounds ahead (two sets of fetch registers), X one round
  // ahead.  Requests in a round, in this order: X(j + 1), then A(j + 2) - so that at the top
  // of round j the requests still allowed to be pending are exactly the RS_Q * LPT of A(j + 1).
  // The barrier is issued with its own wait counts: a fence would wait for every pending
  // request, the LDS-bound ones of X among them, and give the depth away.
  RoundRegs raw0, raw1;
#pragma unroll
  for (int p = 0; p < RS_Q / 2; ++p) load_half(raw0, 0, p);
  dma_x(0, 0);
  if (nrounds > 1) {
#pragma unroll
    for (int p = 0; p < RS_Q / 2; ++p) load_half(raw1, 1, p);
  }
  int buf = 0;                                        // region of round j: j % 2
  auto round = [&](RoundRegs &cur, int j) {
    if (j + 1 < nrounds) wait_vmem<RS_Q * LPT>(); else wait_vmem<0>();   // A(j) and this wave's share of X(j) have arrived
    zero_tail(j, buf);
    // X(j) of every wave has landed; nobody reads the region of round j - 1 any more
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    if (j + 1 < nrounds) dma_x(j + 1, buf ^ 1);
#pragma unroll
    for (int q = 0; q < RS_Q; ++q) {
      // (a step past K, a wave without a tile: requested out of range, zeros with scale 0)
      const int step = RS_Q * j + q;
      Tile t;
      to_operand(cur, q, t);
      // (both K-steps of a pair of requests consumed: their fetch registers are free again)
      if ((q & 1) && j + 2 < nrounds) {
        wait_lds();
        load_half(cur, j + 2, q >> 1);
      }
      const bool live = 4 * step + kb < g.nchunks;    // false: a chunk past the end of K
      const uint32_t s2 = live ? __builtin_amdgcn_perm(t.qp[0], t.qp[0], 0x01000100u) : 0u;
      const uint32_t off = pk_add_f16(__builtin_amdgcn_perm(t.qp[0], t.qp[0], 0x03020302u), g.nib_magic);
      // the operands of the step's instructions serve every token group
      u4 av[NM];
      uint32_t iwv[NM / 2];
      if constexpr (N1) {
        // every slot becomes the pair {value, 0} with its offset in the even index field; instruction m takes
        // slots 4 m .. 4 m + 3 of the chunk: bytes 2 (m & 1), 2 (m & 1) + 1 of dword m >> 1
        iwv[0] = spread_idx(t.iw[0] & 0xFFFFu, g.m8, g.m4, g.m2);
        iwv[1] = spread_idx(t.iw[0] >> 16, g.m8, g.m4, g.m2);
        iwv[2] = spread_idx(t.iw[1] & 0xFFFFu, g.m8, g.m4, g.m2);
        iwv[3] = spread_idx(t.iw[1] >> 16, g.m8, g.m4, g.m2);
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const uint32_t d = t.nib[0][m >> 1];
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const uint32_t t2 = __builtin_amdgcn_perm(d, d, 0x0c000c00u + (uint32_t)(2 * (m & 1) + p) * 0x00010001u);
            const uint32_t pair = pk_mul_f16(pk_sub_f16(and_or(t2, g.nib_mask, magic), off), s2);
            av[m][2 * p] = pair & 0xFFFFu;
            av[m][2 * p + 1] = pair >> 16;
          }
        }
      } else {
        iwv[0] = t.iw[0];
        iwv[1] = t.iw[1];
#pragma unroll
        for (int m = 0; m < NM; ++m) av[m] = dequant8(t.nib[0][m], off, s2, g.nib_mask, magic);
      }
#pragma unroll
      for (int grp = 0; grp < NG; ++grp) {
        if (NG > 1 && 16 * grp >= g.M) continue;      // uniform
        const uint8_t *bregion = xs + buf * RS_REGION + (grp * RS_Q + q) * RS_STEP;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
          const u8v bx = read_b(bregion, m);          // (read per instruction: 8 registers of B at a time)
          const int iword = (int)iwv[m >> 1];
          if (m & 1)
            acc[grp] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[m]), __builtin_bit_cast(h16, bx), acc[grp], iword, 0, 1);
          else
            acc[grp] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(__builtin_bit_cast(h8, av[m]), __builtin_bit_cast(h16, bx), acc[grp], iword, 0, 0);
        }
      }
    }
    buf ^= 1;
  };
  for (int j = 0; j < nrounds; j += 2) {
    round(raw0, j);
    if (j + 1 < nrounds) round(raw1, j + 1);
  }
  // register v of lane l = D[row 4 (l >> 4) + v][token l & 15]: four consecutive rows of one token
  const uint64_t good = __builtin_amdgcn_ballot_w64(fchecked && frp == (uint32_t)frow * S_row);
  if (!has_tile) return;
  const int row0 = 16 * tile + 4 * (lane >> 4);
#pragma unroll
  for (int grp = 0; grp < NG; ++grp) {
    const int tok = 16 * grp + (lane & 15);
    if (tok >= g.M) continue;
    uint32_t hv[4];
#pragma unroll
    for (int v = 0; v < 4; ++v)
      hv[v] = ((good >> (4 * (lane >> 4) + v)) & 1) ? (uint32_t)__half_as_ushort(__float2half(acc[grp][v])) : 0x7E00u;
    __half *dst = Y + (int64_t)tok * g.ldy + row0;
    if (g.vec_store && row0 + 3 < g.rows) {
      *(u2 *)dst = u2{hv[0] | (hv[1] << 16), hv[2] | (hv[3] << 16)};
    } else {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (row0 + v < g.rows) dst[v] = __ushort_as_half((uint16_t)hv[v]);
    }
  }
}

// Shapes the stack takes: INT4 with one {scale, zero} pair per chunk, 2:4 (up to 64 tokens) or 1:4 (up to 32: the
// token rows of a K-step are twice as long).
bool smallm_stack_item_ok(const egt_2bitcsr &w, int M) {
  if (w.val_kind != EGT_VAL_INT4) return false;
  if (!(w.n_keep == 2 && w.group_size >= 64) && !(w.n_keep == 1 && w.group_size >= 128 && M <= 32)) return false;
  return sparse_smallm_supported(w, w.cols, M);
}

static int stack_waves(int M, bool n1) { return M <= (n1 ? 16 : 32) ? RS_WAVES : 16; }

// workgroups of a matrix: one per row tile and wave
int smallm_stack_blocks(int M, int n_keep, int rows) {
  const int ntiles = (rows + 15) / 16, w = stack_waves(M, n_keep == 1);
  return (ntiles + w - 1) / w;
}

void smallm_stack_shape(int M, int n_keep, int &block_threads, int &lds_bytes) {
  const bool n1 = n_keep == 1;
  block_threads = 64 * stack_waves(M, n1);
  if (n1) lds_bytes = rs_lds_bytes(M <= 16 ? 1 : 2, 2, true);
  else lds_bytes = M <= 16 ? rs_lds_bytes(1, RS_Q) : M <= 32 ? rs_lds_bytes(2, 2) : rs_lds_bytes(4, 2);
}

// Descriptor of one item into 160 bytes of the table.
void smallm_stack_entry(const egt_2bitcsr &w, const uint16_t *X, uint16_t *Y, int M, void *entry) {
  SmallMStackEntry e;
  std::memset(&e, 0, sizeof(e));
  int qw;
  smallm_geometry(w, w.cols, Y, w.rows, M, e.g, qw);
  e.row_ptr = (uint64_t)(uintptr_t)w.row_ptr; e.values = (uint64_t)(uintptr_t)w.values; e.idx = (uint64_t)(uintptr_t)w.idx;
  e.qparams = (uint64_t)(uintptr_t)w.qparams; e.X = (uint64_t)(uintptr_t)X; e.Y = (uint64_t)(uintptr_t)Y;
  std::memset(entry, 0, EGT_STACK_ENTRY_BYTES);
  std::memcpy(entry, &e, sizeof(e));
}

hipError_t launch_smallm_stack(const void *table_dev, int count, int M, int n_keep, int grid_x, hipStream_t stream) {
  int threads, lds;
  smallm_stack_shape(M, n_keep, threads, lds);
  const dim3 grid(grid_x), block(threads);
  const uint8_t *t = (const uint8_t *)table_dev;
  if (n_keep == 1) {
    if (M <= 16) return launch(k_smallm_rows<1, 2, RS_WAVES, true>, grid, block, (size_t)lds, stream, t, count);
    return launch(k_smallm_rows<2, 2, 16, true>, grid, block, (size_t)lds, stream, t, count);
  }
  if (M <= 16) return launch(k_smallm_rows<1, RS_Q, RS_WAVES>, grid, block, (size_t)lds, stream, t, count);
  if (M <= 32) return launch(k_smallm_rows<2, 2, RS_WAVES>, grid, block, (size_t)lds, stream, t, count);
  return launch(k_smallm_rows<4, 2, 16>, grid, block, (size_t)lds, stream, t, count);
}

// `count` (2..4) identically shaped members in one launch (the caller has checked the shapes
// and that sparse_smallm_supported holds for them).
hipError_t launch_sparse_smallm_batch(const egt_2bitcsr *ws, const uint16_t *const *Xs, int64_t ldx, uint16_t *const *Ys,
                                      int64_t ldy, int M, int count, hipStream_t stream) {
  SmallMBatch b;
  for (int k = 0; k < EGT_MAX_BATCH; ++k) {
    const int j = k < count ? k : 0;                  // unused slots repeat member 0
    b.row_ptr[k] = ws[j].row_ptr; b.values[k] = (const uint8_t *)ws[j].values; b.idx[k] = (const uint8_t *)ws[j].idx;
    b.qparams[k] = (const uint8_t *)ws[j].qparams; b.X[k] = (const __half *)Xs[j]; b.Y[k] = (__half *)Ys[j];
  }
  return smallm_one_launch(ws[0], Xs[0], ldx, Ys[0], ldy, M, stream, &b, count);
}

}  // namespace egt
