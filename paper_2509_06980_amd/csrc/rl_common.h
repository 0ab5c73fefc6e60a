// Shared device helpers and memory-layout functions for the rollout kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned int)))) unsigned int u32x4;  // one 16-byte load

#define RL_PAGE 16  // tokens per KV page

__host__ __device__ __forceinline__ float bf2f(bf16_t x) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)x << 16;
  return c.f;
}
// round-to-nearest-even (finite inputs)
__host__ __device__ __forceinline__ bf16_t f2bf(float f) {
  union { uint32_t u; float f; } c;
  c.f = f;
  uint32_t u = c.u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float ldf(const float* p) { return *p; }
__device__ __forceinline__ float ldf(const bf16_t* p) { return bf2f(*p); }
__device__ __forceinline__ void stf(float* p, float v) { *p = v; }
__device__ __forceinline__ void stf(bf16_t* p, float v) { *p = f2bf(v); }

// ---------------------------------------------------------------------------------------
// "A-tile" layout of a bf16 activation matrix X[rows, K] that feeds an MFMA GEMM as the
// row operand.  Rows are grouped in tiles of 128, K in blocks of 16; inside one
// (tile, k-block) the 4 KB are four 32x32x16 MFMA operands (32 rows each) stored in lane
// order: lane = row % 32 + 32 * ((k % 16) / 8), 8 consecutive k per lane.  A GEMM workgroup
// therefore copies its K-chunk of a tile into LDS as one contiguous block, and each
// ds_read_b128 of an operand is conflict free.  Requires K % 16 == 0; the buffer holds
// ceil(rows / 128) * 128 rows.
// ---------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ size_t atile_off(int row, int k, int K) {
  int mt = row >> 7, r = row & 127;
  int mb = r >> 5, kb = k >> 4;
  int lane = (r & 31) + (((k >> 3) & 1) << 5);
  return ((((size_t)mt * (K >> 4) + kb) * 4 + mb) * 64 + lane) * 8 + (k & 7);
}

// ---------------------------------------------------------------------------------------
// KV cache.  One page holds RL_PAGE tokens of one layer; pool layout [page][kv_head][block].
// Plain block (fp32 mode, or head_dim != 128): [token][d].
// MFMA block (bf16, head_dim 128, 4 KB for K and 4 KB for V):
//   K: the 16 tokens x 128 dims are four 16x16x32 row operands (32 dims each) in lane
//      order: lane = token + 16 * ((d % 32) / 8), 8 consecutive d per lane.
//   V: stored transposed for the P.V product: eight 16x16x16 operands (16 dims each) whose
//      lane = d % 16 + 16 * (token / 4) holds 4 consecutive tokens; two operands are
//      interleaved per 16-byte lane slot so that one 16-byte load feeds two MFMAs.
// ---------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ int kswz_off(int tok, int d) {
  return ((((d >> 5) * 4 + ((d >> 3) & 3)) * 16 + tok) << 3) + (d & 7);
}
__host__ __device__ __forceinline__ int vswz_off(int tok, int d) {
  int jb = d >> 4, lane = (d & 15) + ((tok >> 2) << 4);
  return ((((jb >> 1) * 64 + lane) * 2 + (jb & 1)) << 2) + (tok & 3);
}

// 8-bit cache variant (OCP FP8 E4M3 codes, head_dim 128, 2 KB for K and 2 KB for V per block): the
// same operand orders with one byte per element, packed so that a lane still loads 16 bytes at a
// time.  K: the 16-byte lane slot holds the lane's 8 dims of two consecutive 32-dim operands.
// V: the slot holds the lane's 4 tokens of four consecutive 16-dim operands.
__host__ __device__ __forceinline__ int kswz8_off(int tok, int d) {
  int lane = tok + (((d >> 3) & 3) << 4);
  return (((((d >> 6) * 64 + lane) << 1) + ((d >> 5) & 1)) << 3) + (d & 7);
}
__host__ __device__ __forceinline__ int vswz8_off(int tok, int d) {
  int jb = d >> 4, lane = (d & 15) + ((tok >> 2) << 4);
  return (((((jb >> 2) * 64 + lane) << 2) + (jb & 3)) << 2) + (tok & 3);
}
// E4M3 code of x: round to nearest even, magnitudes above the largest finite value stored as it.
__device__ __forceinline__ uint32_t f2e4m3x4(float a, float b, float c, float d) {
  a = fminf(fmaxf(a, -448.f), 448.f); b = fminf(fmaxf(b, -448.f), 448.f);
  c = fminf(fmaxf(c, -448.f), 448.f); d = fminf(fmaxf(d, -448.f), 448.f);
  int p = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
  p = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, p, true);
  return (uint32_t)p;
}
__device__ __forceinline__ uint8_t f2e4m3(float a) { return (uint8_t)(f2e4m3x4(a, a, a, a) & 0xffu); }
// Four E4M3 codes (one 32-bit word) -> four bf16 (exact), element order kept.
__device__ __forceinline__ void e4m3x4_to_bf16(uint32_t w, uint32_t* lo, uint32_t* hi) {
  *lo = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false));
  *hi = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true));
}
// Two raw 16-byte lane slots of an 8-bit block -> the four 16-byte operand registers that the
// bf16 block of the same tokens would have delivered (same rule for keys and values).
__device__ __forceinline__ void expand_e4m3_block(const u32x4 (&raw)[2], u32x4 (&out)[4]) {
#pragma unroll
  for (int i = 0; i < 4; i++) {
    uint32_t a, b, c, d;
    e4m3x4_to_bf16(raw[i >> 1][2 * (i & 1)], &a, &b);
    e4m3x4_to_bf16(raw[i >> 1][2 * (i & 1) + 1], &c, &d);
    out[i] = (u32x4){a, b, c, d};
  }
}

template <bool SWZ>
__device__ __forceinline__ int kblk_off(int tok, int d, int D) {
  return SWZ ? kswz_off(tok, d) : tok * D + d;
}
template <bool SWZ>
__device__ __forceinline__ int vblk_off(int tok, int d, int D) {
  return SWZ ? vswz_off(tok, d) : tok * D + d;
}

// Reductions over the four lanes {n, n + 16, n + 32, n + 48} (the four token groups of one MFMA
// column) with the gfx950 row-swap instructions: swapping a register with itself puts lanes
// i and i ^ 16 (i ^ 32) side by side; every lane ends with the result.  Plain VALU, no LDS path.
__device__ __forceinline__ float quad_max(float x) {
  unsigned a = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
  unsigned r0 = r[0], r1 = r[1];
  float y = fmaxf(__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1));
  unsigned b = __builtin_bit_cast(unsigned, y);
  auto q = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  unsigned q0 = q[0], q1 = q[1];
  return fmaxf(__builtin_bit_cast(float, q0), __builtin_bit_cast(float, q1));
}
__device__ __forceinline__ float quad_sum(float x) {
  unsigned a = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane16_swap(a, a, false, false);
  unsigned r0 = r[0], r1 = r[1];
  float y = __builtin_bit_cast(float, r0) + __builtin_bit_cast(float, r1);
  unsigned b = __builtin_bit_cast(unsigned, y);
  auto q = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  unsigned q0 = q[0], q1 = q[1];
  return __builtin_bit_cast(float, q0) + __builtin_bit_cast(float, q1);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
