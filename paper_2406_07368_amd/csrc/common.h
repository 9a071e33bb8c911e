// Shared device helpers for the gfx950 kernels: vector types, bf16 <-> fp32,
// the feature map, and typed 8-element global loads/stores.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace linattn {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// phi(x) = elu(x) + 1 (Sec. 3: kernel embedding of queries and keys; elu+1 is
// the embedding of the kernelised attention the paper builds on).
__device__ __forceinline__ float phi_elu1(float x) { return x > 0.f ? x + 1.f : __expf(x); }
// Either feature map; `relu` is uniform over a launch.
__device__ __forceinline__ float phi_any(float x, int relu) { return relu ? fmaxf(x, 0.f) : phi_elu1(x); }

__device__ __forceinline__ float bf16_lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Two floats -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2 x = {lo, hi};
  bf16x2 y = __builtin_convertvector(x, bf16x2);
  return __builtin_bit_cast(uint32_t, y);
}
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return (uint16_t)(pack_bf16x2(f, 0.f) & 0xffffu);
}

// ---- typed access to rows of q/k/v/out/hist ------------------------------------
// IoF32 / IoBf16: load `8 consecutive elements` as floats, store 8 floats.
struct F32Raw8 { f32x4 lo, hi; };

struct IoF32 {
  typedef float elem;
  typedef F32Raw8 raw8;     // 8 elements as they lie in memory: requested early, converted where they are used
  static __device__ __forceinline__ raw8 load_raw8(const void* base, int64_t idx) {
    const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + idx);
    return raw8{p[0], p[1]};
  }
  // The value has to be in its registers here: a request whose only uses sit under a condition is otherwise moved
  // down to them by the compiler, behind every request issued in between, with a wait for all of those.
  static __device__ __forceinline__ void needed_here(const raw8& r) { asm volatile("" ::"v"(r.lo[0]), "v"(r.hi[0])); }
  static __device__ __forceinline__ void unpack8(const raw8& r, float (&x)[8]) {
    x[0] = r.lo[0]; x[1] = r.lo[1]; x[2] = r.lo[2]; x[3] = r.lo[3];
    x[4] = r.hi[0]; x[5] = r.hi[1]; x[6] = r.hi[2]; x[7] = r.hi[3];
  }
  static __device__ __forceinline__ void load8(const void* base, int64_t idx, float (&x)[8]) {
    const f32x4* p = reinterpret_cast<const f32x4*>(static_cast<const float*>(base) + idx);
    f32x4 a = p[0], b = p[1];
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3];
    x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
  static __device__ __forceinline__ void store8(void* base, int64_t idx, const float (&x)[8]) {
    f32x4* p = reinterpret_cast<f32x4*>(static_cast<float*>(base) + idx);
    p[0] = f32x4{x[0], x[1], x[2], x[3]};
    p[1] = f32x4{x[4], x[5], x[6], x[7]};
  }
  static __device__ __forceinline__ float load1(const void* base, int64_t idx) {
    return static_cast<const float*>(base)[idx];
  }
  static __device__ __forceinline__ void store1(void* base, int64_t idx, float x) {
    static_cast<float*>(base)[idx] = x;
  }
};

struct IoBf16 {
  typedef uint16_t elem;
  typedef u32x4 raw8;
  static __device__ __forceinline__ raw8 load_raw8(const void* base, int64_t idx) {
    return *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + idx);
  }
  static __device__ __forceinline__ void needed_here(const raw8& r) { asm volatile("" ::"v"(r[0])); }
  static __device__ __forceinline__ void unpack8(const raw8& r, float (&x)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = bf16_lo_to_f32(r[i]);
      x[2 * i + 1] = bf16_hi_to_f32(r[i]);
    }
  }
  static __device__ __forceinline__ void load8(const void* base, int64_t idx, float (&x)[8]) {
    u32x4 r = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(base) + idx);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = bf16_lo_to_f32(r[i]);
      x[2 * i + 1] = bf16_hi_to_f32(r[i]);
    }
  }
  static __device__ __forceinline__ void store8(void* base, int64_t idx, const float (&x)[8]) {
    u32x4 r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = pack_bf16x2(x[2 * i], x[2 * i + 1]);
    *reinterpret_cast<u32x4*>(static_cast<uint16_t*>(base) + idx) = r;
  }
  static __device__ __forceinline__ float load1(const void* base, int64_t idx) {
    return bf16_bits_to_f32(static_cast<const uint16_t*>(base)[idx]);
  }
  static __device__ __forceinline__ void store1(void* base, int64_t idx, float x) {
    static_cast<uint16_t*>(base)[idx] = f32_to_bf16_bits(x);
  }
};

// Sums across lanes without the LDS crossbar (hundreds of them per step: as ds_bpermute they were the
// bottleneck).  Within a row of 16 lanes: DPP modifiers on the add; across rows: the lane-swap instructions.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xf, 0xf, false));
}
// every lane gets the sum over its group of N consecutive lanes (N = 8 or 16, groups aligned)
template <int N>
__device__ __forceinline__ float sum_lanes(float x) {
  x = dpp_add<0xB1>(x);                 // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);                 // quad_perm [2,3,0,1]
  x = dpp_add<0x141>(x);                // row_half_mirror: the other quad of each 8
  if (N == 16) x = dpp_add<0x140>(x);   // row_mirror: the other half of each 16
  return x;
}
// the same for the largest value
template <int CTRL>
__device__ __forceinline__ float dpp_max(float x) {
  return fmaxf(x, __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(0, (int)__float_as_uint(x), CTRL, 0xf, 0xf, false)));
}
template <int N>
__device__ __forceinline__ float max_lanes(float x) {
  x = dpp_max<0xB1>(x);
  x = dpp_max<0x4E>(x);
  x = dpp_max<0x141>(x);
  if (N == 16) x = dpp_max<0x140>(x);
  return x;
}

}  // namespace linattn
