// Register layouts of the gfx950 MFMA instructions used by the bf16 path, and the index maps
// the kernels agree on.  Device-side only.
//
// v_mfma_f32_32x32x16_{bf16,f16}  D[32x32] += A[32x16] * B[16x32], one wavefront (64 lanes):
//   lane l = (m, g) with m = l % 32, g = l / 32
//   A: lane holds A[m][8g .. 8g+7]          (8 bf16, 4 VGPRs)
//   B: lane holds B[8g .. 8g+7][m]          (8 bf16)
//   D: lane holds D[8*(r/4) + 4g + r%4][m]  for r = 0..15
// The operator is evaluated "tokens along N": a lane owns one token (column) and, in its
// 16 accumulator registers per row block, 16 rows.  Row and contraction indices may be
// permuted freely as long as both operands of a product agree; the maps below pick the
// permutations that make every lane's rows contiguous in memory:
//   lane (t, g), row block mb, register r  <->  row  g*(R/2) + 16*mb + r   (R rows in total)
// so a lane owns R/2 consecutive rows (channels or features) of its token.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace linattn {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(2 * sizeof(_Float16)))) _Float16 f16x2;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;

// Two fp32 -> packed bf16 pair (round to nearest even, one v_cvt_pk_bf16_f32), lo in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// Two fp32 -> packed fp16 pair (round to nearest even, one v_cvt_pk_f16_f32).
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  f32x2 v = {lo, hi};
  f16x2 r = __builtin_convertvector(v, f16x2);
  return __builtin_bit_cast(uint32_t, r);
}

// Packed bf16 pair -> packed fp16 pair.  Exact for 2^-14 <= |x| < 65520; smaller values lose
// bits below 2^-24, larger ones become infinity.
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t u) {
  return pack_f16x2(__builtin_bit_cast(float, u << 16), __builtin_bit_cast(float, u & 0xffff0000u));
}

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ __forceinline__ f16x8 as_f16x8(uint4 v) { return __builtin_bit_cast(f16x8, v); }

// A-operand row i (0..31) of row block mb  <->  actual row, for R rows in total.
// Inverse of the accumulator layout: row i lands in lane group (i/4)%2, register 4*(i/8) + i%4.
template <int R>
__device__ __forceinline__ constexpr int owned_row(int mb, int i) {
  return ((i / 4) % 2) * (R / 2) + 16 * mb + 4 * (i / 8) + (i % 4);
}

// Index maps of the query pass out^T = S^T phi(q)^T for head width D.
template <int D>
struct ApplyLayout {
  static constexpr int HALF = D / 2;      // features per softmax half (Eq. 5)
  static constexpr int KS = D / 16;       // k-steps over the D features of phi
  static constexpr int MB = D / 32;       // row blocks over the D output channels
  static constexpr int MBZ = MB + 1;      // + one block whose rows 0 and 4 carry z (the normaliser)
  // Feature of phi (order of Eq. 5: softmax(+u) first) that lane group g feeds as element e of
  // k-step ks: each lane owns HALF/2 consecutive features of each half.
  __device__ static constexpr int feature(int ks, int g, int e) {
    return (ks < KS / 2 ? 0 : HALF) + g * (HALF / 2) + 8 * (ks % (KS / 2)) + e;
  }
  // Output channel carried by A-operand row m of row block mb.
  __device__ static constexpr int channel(int mb, int m) { return owned_row<D>(mb, m); }
  // Output channel carried by B-operand column c of column block mb when the operands are swapped
  // (Y = phi S, tokens on the accumulator rows): a lane then holds MB adjacent channels of each of
  // its 16 token rows, and 32 lanes cover one whole row of d channels.
  __device__ static constexpr int channel_cols(int mb, int c) { return MB * c + mb; }
};

}  // namespace linattn
