// Device helpers shared by the kernels: bfloat16 conversion and splitting,
// MFMA operand types, LDS tile addressing.  gfx950 (CDNA4) only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace snn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

// ---------------------------------------------------------------- bfloat16
// Round to nearest, ties to even.  Inputs are finite here (no NaN handling).
__device__ __forceinline__ uint32_t bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_value(uint32_t bits) { return __uint_as_float(bits << 16); }

// Piece `plane` of the three-way split x = hi + mid + lo with each piece a bfloat16.
// plane 0: hi = rne(x); plane 1: mid = rne(x - hi); plane 2: lo = rne(x - hi - mid).
__device__ __forceinline__ uint32_t bf16_piece(float x, int plane) {
  uint32_t hi = bf16_bits(x);
  if (plane == 0) return hi;
  float r1 = x - bf16_value(hi);
  uint32_t mid = bf16_bits(r1);
  if (plane == 1) return mid;
  float r2 = r1 - bf16_value(mid);
  return bf16_bits(r2);
}
__device__ __forceinline__ uint32_t pack2(uint32_t lo16, uint32_t hi16) { return lo16 | (hi16 << 16); }

// "HL" form of a value entering a bfloat16 product with better than bfloat16 accuracy:
// hi = bf16(x) in bits 0..15, lo = bf16(x - hi) in bits 16..31; hi + lo = x to 2^-16 relative.
// (The casts compile to v_cvt_pk_bf16_f32.)
__device__ __forceinline__ uint32_t pack_hl(float x) {
  const __bf16 h = (__bf16)x;
  const __bf16 l = (__bf16)(x - (float)h);
  return (uint32_t)__builtin_bit_cast(unsigned short, h) | ((uint32_t)__builtin_bit_cast(unsigned short, l) << 16);
}

// Two 0/1 bytes -> two bfloat16 (0.0 or 1.0) in one dword: bytes sit in bits 0 and 16.
__device__ __forceinline__ uint32_t spikes2_to_bf16(uint32_t two_bytes_spread) {
  return (two_bytes_spread & 0x00010001u) * 0x3F80u;
}

// ---------------------------------------------------------------- buffer addressing
// Global accesses of the hot kernels go through buffer instructions: a 128-bit resource
// (base, size), a per-lane byte offset kept in one register, and a scalar byte offset.  The
// per-step or per-tile address arithmetic then runs on the scalar unit, and a lane offset
// beyond the size reads zero / drops the store.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
constexpr int OOB = 0x7FFFFF00;          // beyond any buffer here

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, unsigned bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ uint32_t ld_b8(rsrc_t r, int voff, int soff) {
  return (uint32_t)__builtin_amdgcn_raw_buffer_load_b8(r, voff, soff, 0);
}
// POLICY: 0 = default, NT = non-temporal (data streamed once; see scan.hpp).
constexpr int NT = 2;
template <int POLICY = 0> __device__ __forceinline__ uint32_t ld_b32(rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, POLICY);
}
template <int POLICY = 0> __device__ __forceinline__ u32x2 ld_b64(rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, POLICY);
}
template <int POLICY = 0> __device__ __forceinline__ u32x4 ld_b128(rsrc_t r, int voff, int soff) {
  return __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, POLICY);
}
__device__ __forceinline__ void st_b8(rsrc_t r, int voff, int soff, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b8((unsigned char)v, r, voff, soff, 0);
}
__device__ __forceinline__ void st_b16(rsrc_t r, int voff, int soff, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b16((unsigned short)v, r, voff, soff, 0);
}
__device__ __forceinline__ void st_b32(rsrc_t r, int voff, int soff, uint32_t v) {
  __builtin_amdgcn_raw_buffer_store_b32(v, r, voff, soff, 0);
}
__device__ __forceinline__ void st_b64(rsrc_t r, int voff, int soff, u32x2 v) {
  __builtin_amdgcn_raw_buffer_store_b64(v, r, voff, soff, 0);
}
// A 16-byte store reads its four data registers over several cycles, and an instruction
// that overwrites one of them must keep its distance.  The compiler keeps that distance only
// for stores without a scalar offset register; with one, a write to the first data register
// directly behind the store was seen to reach memory in place of the stored value on gfx950.
// So the whole offset of a 16-byte store goes through the vector register.
__device__ __forceinline__ void st_b128(rsrc_t r, int voff, int soff, u32x4 v) {
  __builtin_amdgcn_raw_buffer_store_b128(v, r, (int)((unsigned)voff + (unsigned)soff), 0, 0);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (vmcnt(0)), which would expose the full memory latency at each
// barrier and defeat the register prefetch ring of the product kernels.  Here only the LDS
// counter is drained; global loads stay in flight and are waited for where their registers
// are first used.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---------------------------------------------------------------- LDS operand tiles
// An operand tile holds ROWS rows of 64 contraction elements as bfloat16: 128 bytes per row,
// split in eight 16-byte chunks.  Chunk c of row r lives at chunk slot c ^ swz(r); the
// permutation keeps both the 16-byte fragment reads (32 consecutive rows, same chunk) and
// the transposing stores (rows 4 or 2 apart, same chunk) spread over all banks.
__device__ __forceinline__ int tile_swz(int row) { return (row ^ (row >> 3)) & 7; }
__device__ __forceinline__ int tile_off(int row, int chunk) {   // byte offset
  return row * 128 + ((chunk ^ tile_swz(row)) << 4);
}

}  // namespace snn
