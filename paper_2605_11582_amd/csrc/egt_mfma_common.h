// Register-level helpers shared by the matrix-core kernels.
#ifndef EGT_MFMA_COMMON_H
#define EGT_MFMA_COMMON_H

#include "egt_device.h"

namespace egt {

typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16 __attribute__((ext_vector_type(16)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef uint32_t u8v __attribute__((ext_vector_type(8)));
typedef uint32_t u2 __attribute__((ext_vector_type(2)));

// streaming load: the weights are used once, keep them from displacing x in the caches
template <typename T>
__device__ __forceinline__ T ld_stream(const void *p) {
  return __builtin_nontemporal_load((const T *)p);
}

__device__ __forceinline__ uint32_t pk_sub_f16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, a) - __builtin_bit_cast(h2, b));
}
__device__ __forceinline__ uint32_t pk_add_f16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, a) + __builtin_bit_cast(h2, b));
}
__device__ __forceinline__ uint32_t pk_mul_f16(uint32_t a, uint32_t b) {
  return __builtin_bit_cast(uint32_t, __builtin_bit_cast(h2, a) * __builtin_bit_cast(h2, b));
}
// (a & mask) | magic.  The compiler fuses this into one v_and_or_b32 only when mask
// and magic are register values: the three-operand encoding takes no literal, so
// callers pass them in from kernel arguments instead of writing constants.  (Inline
// assembly is not an option here: results that feed a matrix instruction need wait
// states the compiler only inserts for instructions it emitted itself.)
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t magic) {
  return (a & mask) | magic;
}
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

// The same for the paired nibble order (EGT_VAL_INT4_PAIRED): the word holds the slots
// 0, 2, 4, 6, 1, 3, 5, 7 from its low nibble up, so slot pair (0, 1) is `d & 0x000F000F`,
// (2, 3) is `d & 0x00F000F0`, and (4, 5), (6, 7) the same of d >> 8: one shift and four
// and-ors instead of four byte permutes and four and-ors.  Both halves of a register carry
// the same offset: 1024 (mask_lo, magic_lo, off_lo = {1024 + z} twice) or 64.
__device__ __forceinline__ u4 dequant8_paired(uint32_t d, uint32_t off_lo, uint32_t off_hi, uint32_t s2, uint32_t mask_lo,
                                              uint32_t mask_hi, uint32_t magic_lo, uint32_t magic_hi) {
  const uint32_t d8 = d >> 8;
  u4 r;
  r[0] = pk_mul_f16(pk_sub_f16(and_or(d, mask_lo, magic_lo), off_lo), s2);
  r[1] = pk_mul_f16(pk_sub_f16(and_or(d, mask_hi, magic_hi), off_hi), s2);
  r[2] = pk_mul_f16(pk_sub_f16(and_or(d8, mask_lo, magic_lo), off_lo), s2);
  r[3] = pk_mul_f16(pk_sub_f16(and_or(d8, mask_hi, magic_hi), off_hi), s2);
  return r;
}
// Pins a wave-uniform value into a vector register (an empty statement for the
// assembler): with the mask in a scalar and the magic in a vector register the
// fused and-or respects the one-scalar-operand limit of the encoding.
__device__ __forceinline__ uint32_t in_vgpr(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}
// value of lane (l + N) of the same 16-lane row, 0 past the end of the row
template <int N>
__device__ __forceinline__ float row_shl(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x100 + N, 0xf, 0xf, true));
}
// value of lane (l ^ 1) / (l ^ 2) inside each group of four lanes
__device__ __forceinline__ float quad_xor1(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));
}
__device__ __forceinline__ float quad_xor2(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));
}


// 16-bit index word (8 fields of 2 bits) -> 32 bits with field j at bits [4j, 4j+1]: the
// index operand of an instruction whose compressed values are {value, 0} pairs (1:4).
// The masks 0x00FF00FF, 0x0F0F0F0F, 0x33333333 are passed in so that they live in registers.
__device__ __forceinline__ uint32_t spread_idx(uint32_t w, uint32_t m8, uint32_t m4, uint32_t m2) {
  uint32_t t = (w | (w << 8)) & m8;
  t = (t | (t << 4)) & m4;
  return (t | (t << 2)) & m2;
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
// f(IC<0>), f(IC<1>), ... f(IC<N - 1>): a loop whose index is a compile-time constant
template <int V>
struct IC { static constexpr int v = V; };
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (I < N) {
    f(IC<I>{});
    static_for<I + 1, N>(f);
  }
}
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store of the wave; where loads for later work are in flight
// across the barrier on purpose, that wait would give the overlap away.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// x through LDS, the two halves every row-per-wave kernel shares (Sec. 3.3 "Accelerate
// Memory Access": the activations are fetched once per workgroup and shared, laid out so
// that the reads do not collide on banks).  x_request: each thread asks for XP 16-byte
// pieces (thread t: pieces t, t + blockDim, ...; a piece past the end of x repeats the last
// one) before anything else is requested, so that x is the first data to come back.
// x_store: piece p goes to byte 16 p + 16 (p >> XSH) of `xs` - one 16-byte pad after every
// 2^XSH pieces, which puts the 16 lanes of a B operand read on different banks; pieces past
// the end of x (up to lds_pieces, what the B reads may touch) are zeros.
template <int XP>
__device__ __forceinline__ void x_request(const __half *x, int npieces, u4 (&xp)[XP]) {
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int pi = threadIdx.x + j * blockDim.x;
    xp[j] = *(const u4 *)(x + 8 * min(pi, npieces - 1));
  }
}
template <int XP, int XSH>
__device__ __forceinline__ void x_store(uint8_t *xs, const u4 (&xp)[XP], int npieces, int lds_pieces) {
#pragma unroll
  for (int j = 0; j < XP; ++j) {
    const int pi = threadIdx.x + j * blockDim.x;
    if (pi < lds_pieces) {
      u4 v = xp[j];
      if (pi >= npieces) v = u4{0, 0, 0, 0};
      *(u4 *)(xs + 16 * pi + 16 * (pi >> XSH)) = v;
    }
  }
}

// Block shape of a launch of one of the M = 1 kernels, derived on the host from the matrix
// geometry, the waves per workgroup and the tiles per wave.
struct LaunchShape {
  int nblocks;   // workgroups along x
  int nwaves;    // waves per workgroup
  int tpi;       // tiles per wave
  int xp;        // 16-byte pieces of x each thread stages
  size_t lds;    // dynamic LDS bytes
};

// Pointer table of a batched launch: up to EGT_MAX_BATCH identically shaped matrices,
// selected by blockIdx.y (a single product is a batch of one).
constexpr int EGT_MAX_BATCH = 4;
struct GemvBatch {
  const uint32_t *row_ptr[EGT_MAX_BATCH];
  const uint8_t *values[EGT_MAX_BATCH];
  const uint8_t *idx[EGT_MAX_BATCH];
  const uint8_t *qparams[EGT_MAX_BATCH];
  const __half *x[EGT_MAX_BATCH];
  __half *y[EGT_MAX_BATCH];
};

// Member `i` of a pointer table by scalar selects: all four entries arrive with the
// kernel arguments, so no load depends on the index.
template <typename T>
__device__ __forceinline__ T pick4(T const (&a)[EGT_MAX_BATCH], unsigned i) {
  const T lo = (i & 1) ? a[1] : a[0];
  const T hi = (i & 1) ? a[3] : a[2];
  return (i & 2) ? hi : lo;
}

// Index of the four-lane group, (lane >> 2) & 3, selects among four values.
__device__ __forceinline__ float select4(int k, float a0, float a1, float a2, float a3) {
  return (k & 2) ? ((k & 1) ? a3 : a2) : ((k & 1) ? a1 : a0);
}

}  // namespace egt
#endif
