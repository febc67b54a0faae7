// MFMA building blocks for gfx950 (64-wide wavefronts).
//
// v_mfma_f32_16x16x32_bf16 computes D[16x16] += A[16x32] * B[32x16]:
//   A: lane l holds row (l % 16), columns 8*(l / 16) .. 8*(l / 16) + 7
//   B: lane l holds column (l % 16), rows 8*(l / 16) .. +7
//   D: lane l holds column (l % 16), rows 4*(l / 16) .. 4*(l / 16) + 3
// so a lane is addressed as (r, q) = (l % 16, l / 16) throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mhcl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16 bytes as a native vector (HIP's uint4 is a struct and is kept out of the
// register tiles: arrays of it tend to be left on the stack)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x4 mfma16(const u32x4 &a, const u32x4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// the same tile shape and lane layout with fp16 operands
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x4 mfma16h(const u32x4 &a, const u32x4 &b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
// two fp32 -> packed fp16 pair, round to nearest even
__device__ __forceinline__ uint32_t cvt_pk_f16(float lo, float hi) {
  f16x2 r;
  r[0] = static_cast<_Float16>(lo);
  r[1] = static_cast<_Float16>(hi);
  return __builtin_bit_cast(uint32_t, r);
}

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t cvt_pk_bf16(float lo, float hi) {
  bf16x2 r;
  r[0] = static_cast<__bf16>(lo);
  r[1] = static_cast<__bf16>(hi);
  return __builtin_bit_cast(uint32_t, r);
}

// Packed layouts of the projection matrix W [K, M] (fp32) as bf16 pairs
// W = hi + lo (hi = bf16(W), lo = bf16(W - hi): ~16 mantissa bits together).
//
// Stream tensors are read in MFMA lane order: at K step s (32 columns) lane
// (r, q) reads the 16 bytes of token r at columns 32 s + 8 q .. + 7; kernels
// issue two or more consecutive steps back to back so that the four lanes of a
// token consume whole 128-byte lines per visit.
//
// "B layout" (W as the right operand, contraction over K):
//   block (s, j, p): K step s (32 rows), logit tile j (16 columns), part p
//   (0 = hi, 1 = lo); 64 lanes x 8 bf16; lane (r, q), element e is
//   W[32 s + 8 q + e][16 j + r]  (0 beyond M).  Block index (s * NT + j) * 2 + p.
//
// "A layout" (W as the left operand, contraction over the logits):
//   block (S, h, ms, p): 64-row step S, quarter h = 2 u + hh (u, hh in 0..1),
//   logit step ms (32 logits), part p; lane (r, q), element e is
//   W[64 S + 32 u + 8 (r / 4) + 4 hh + (r % 4)][32 ms + 8 q + e].
//   Block index ((S * 4 + h) * MS + ms) * 2 + p.
//   With B = per-token vectors [32 logits x 16 tokens], quarter h leaves lane
//   (token, q) holding rows 64 S + 32 u + 8 q + 4 hh + 0..3: over hh = 0, 1 the
//   same 8 consecutive rows that lane loads from a stream tensor at step 2 S + u.
inline int logit_tiles(int M) { return (M + 15) / 16; }
inline int logit_steps(int M) { return (M + 31) / 32; }
inline size_t packed_b_bytes(int K, int M) { return static_cast<size_t>(K / 32) * logit_tiles(M) * 2 * 1024; }
inline size_t packed_a_bytes(int K, int M) { return static_cast<size_t>(K / 64) * 4 * logit_steps(M) * 2 * 1024; }

}  // namespace mhcl
