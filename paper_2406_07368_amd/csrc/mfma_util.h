// Helpers shared by the matrix-core kernels: LDS fragment loads (row reads and the
// gfx950 transpose reads), the 32x32x16 bf16 MFMA, accumulator -> bf16 operand packing.
#pragma once
#include "common.h"

namespace linattn {

constexpr int HALO = 8;   // value rows kept from the previous group for the conv taps (Kc-1 <= 7)

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4* lds_s16x4_ptr;

__device__ __forceinline__ bf16x8 lds_row8(const uint16_t* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ bf16x4 lds_row4(const uint16_t* p) { return *reinterpret_cast<const bf16x4*>(p); }

__device__ __forceinline__ bf16x8 cat4(bf16x4 a, bf16x4 b) {
  return __builtin_shufflevector(a, b, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Transpose load: the 16 lanes of a block read a 4 x 16 tile (4 rows, 16 columns,
// each lane 8 bytes of one row) and lane j receives column j of the 4 rows.
__device__ __forceinline__ bf16x4 lds_tr4(const uint16_t* p) {
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  return __builtin_bit_cast(bf16x4, r);
}

// MFMA operand with lanes <-> 32 consecutive columns (col0 + lane%32) of a row-major
// bf16 array and registers <-> rows row0 + 8*(lane/32) + 0..7.
__device__ __forceinline__ bf16x8 tr_operand(const uint16_t* base, int stride, int row0, int col0, int lane) {
  const int j = lane & 15;
  const uint16_t* p = base + (row0 + 8 * (lane >> 5) + (j >> 2)) * stride + col0 + 16 * ((lane >> 4) & 1) + 4 * (j & 3);
  return cat4(lds_tr4(p), lds_tr4(p + 4 * stride));
}

// The same with registers <-> the rows in the order in which a 32 x 32 accumulator holds its row index: registers
// 0..3 <-> rows row0 + 4 (lane / 32) + 0..3, registers 4..7 <-> rows row0 + 8 + 4 (lane / 32) + 0..3.  An accumulator
// packed with pack8(acc, 0) / pack8(acc, 8) is then the other operand of a product over rows row0 .. row0 + 15 /
// row0 + 16 .. row0 + 31 without its values ever passing through LDS.
__device__ __forceinline__ bf16x8 tr_operand_acc_order(const uint16_t* base, int stride, int row0, int col0, int lane) {
  const int j = lane & 15;
  const uint16_t* p = base + (row0 + 4 * (lane >> 5) + (j >> 2)) * stride + col0 + 16 * ((lane >> 4) & 1) + 4 * (j & 3);
  return cat4(lds_tr4(p), lds_tr4(p + 8 * stride));
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& x, int o) {
  u32x4 r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = pack_bf16x2(x[o + 2 * i], x[o + 2 * i + 1]);
  return __builtin_bit_cast(bf16x8, r);
}

// Eight accumulator values as the sum of two bf16 operands: hi = bf16(x), lo = bf16(x - hi).  A product with hi and
// one with lo carries sixteen significant bits of x where one operand carries eight.
__device__ __forceinline__ void split8(const f32x16& x, int o, bf16x8& hi, bf16x8& lo) {
  u32x4 h, l;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    h[i] = pack_bf16x2(x[o + 2 * i], x[o + 2 * i + 1]);
    l[i] = pack_bf16x2(x[o + 2 * i] - bf16_lo_to_f32(h[i]), x[o + 2 * i + 1] - bf16_hi_to_f32(h[i]));
  }
  hi = __builtin_bit_cast(bf16x8, h);
  lo = __builtin_bit_cast(bf16x8, l);
}


// phi(x) = elu(x) + 1 as max(x + 1, min(2^(x log2 e), 1)): for x > 0 the clamped exponential is 1 < x + 1,
// for x <= 0 the exponential is >= x + 1 (convexity), so the maximum picks the right branch without a select.
__device__ __forceinline__ float phi_elu1_max(float x) {
  const float e = __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(x * 1.44269504088896340736f), 0.f, 1.f);
  return fmaxf(x + 1.f, e);
}

// phi on four packed bf16 pairs -> four packed bf16 pairs.  `relu` is uniform over a launch: one branch
// per call, no select per element.
__device__ __forceinline__ u32x4 phi_pack8(u32x4 x, int relu) {
  u32x4 y;
  if (!relu) {
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = pack_bf16x2(phi_elu1_max(bf16_lo_to_f32(x[i])), phi_elu1_max(bf16_hi_to_f32(x[i])));
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = pack_bf16x2(fmaxf(bf16_lo_to_f32(x[i]), 0.f), fmaxf(bf16_hi_to_f32(x[i]), 0.f));
  }
  return y;
}

// The same without a branch on the feature map: with one = 1 for elu + 1 and 0 for max(x, 0), phi(x) =
// max(x + one, one * min(exp(x), 1)).  For callers inside unrolled loops, where a branch per call would cut the loop
// into basic blocks with a full wait at the end of each.
__device__ __forceinline__ float phi_nb(float x, float one) {
  return fmaxf(x + one, one * __builtin_amdgcn_fmed3f(__builtin_amdgcn_exp2f(x * 1.44269504088896340736f), 0.f, 1.f));
}
__device__ __forceinline__ u32x4 phi_pack8_nb(u32x4 x, float one) {
  u32x4 y;
#pragma unroll
  for (int i = 0; i < 4; ++i) y[i] = pack_bf16x2(phi_nb(bf16_lo_to_f32(x[i]), one), phi_nb(bf16_hi_to_f32(x[i]), one));
  return y;
}
__device__ __forceinline__ void phi_split8_nb(u32x4 x, float one, u32x4& hi, u32x4& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float f0 = phi_nb(bf16_lo_to_f32(x[i]), one), f1 = phi_nb(bf16_hi_to_f32(x[i]), one);
    hi[i] = pack_bf16x2(f0, f1);
    lo[i] = pack_bf16x2(f0 - bf16_lo_to_f32(hi[i]), f1 - bf16_hi_to_f32(hi[i]));
  }
}

// phi on four packed bf16 pairs as the sum of two bf16 terms: hi = bf16(phi(x)), lo = bf16(phi(x) - hi).
// phi(x) = x + 1 of a bf16 x needs more significant bits than one bf16 has; hi + lo carries sixteen, so a
// product (hi + lo) * v that enters the fp32 state is off by 2^-17 of itself instead of 2^-9.  max(x, 0)
// of a bf16 x is a bf16: lo = 0.
__device__ __forceinline__ void phi_split8(u32x4 x, int relu, u32x4& hi, u32x4& lo) {
  if (!relu) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float f0 = phi_elu1_max(bf16_lo_to_f32(x[i])), f1 = phi_elu1_max(bf16_hi_to_f32(x[i]));
      hi[i] = pack_bf16x2(f0, f1);
      lo[i] = pack_bf16x2(f0 - bf16_lo_to_f32(hi[i]), f1 - bf16_hi_to_f32(hi[i]));
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      hi[i] = pack_bf16x2(fmaxf(bf16_lo_to_f32(x[i]), 0.f), fmaxf(bf16_hi_to_f32(x[i]), 0.f));
      lo[i] = 0u;
    }
  }
}

}  // namespace linattn
