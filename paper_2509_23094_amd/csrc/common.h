// Device-side helpers shared by the gfx950 kernels: storage types, MFMA
// fragments for 64-wide wavefronts, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace d2c {

typedef __bf16 bf16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return static_cast<float>(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return static_cast<bf16>(x); }

// A 16-byte fragment: what one lane feeds to the matrix core for one step along
// the contraction axis.  For bf16 it is one 16x16x32 operand (8 values); for
// float it is four consecutive 16x16x4 operands (lane group g = lane/16 owns
// four consecutive k, used one per instruction; both operands use the same
// rule so the contraction pairs matching k).
template <typename T> struct Frag;
template <> struct Frag<bf16> {
  static constexpr int kElems = 8;     // elements per 16-byte lane fragment
  static constexpr int kStep = 32;     // contraction length covered by the 4 lane groups
  u32x4 raw;
};
template <> struct Frag<float> {
  static constexpr int kElems = 4;
  static constexpr int kStep = 16;
  u32x4 raw;
};

// acc[16x16] += A_frag * B_frag.  Lane l holds row (or column) l%16 of its
// operand and contraction offsets (l/16)*kElems ..; acc element j is
// D[4*(l/16)+j][l%16].
__device__ __forceinline__ void mfma16(f32x4& acc, const Frag<bf16>& a, const Frag<bf16>& b) {
  acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a.raw),
                                                __builtin_bit_cast(bf16x8, b.raw), acc, 0, 0, 0);
}
__device__ __forceinline__ void mfma16(f32x4& acc, const Frag<float>& a, const Frag<float>& b) {
  const f32x4 af = __builtin_bit_cast(f32x4, a.raw), bf = __builtin_bit_cast(f32x4, b.raw);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, bf.x, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, bf.y, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, bf.z, acc, 0, 0, 0);
  acc = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, bf.w, acc, 0, 0, 0);
}

__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }
__device__ __forceinline__ u32x2 ld8(const void* p) { return *reinterpret_cast<const u32x2*>(p); }

// Full-wave reductions in a fixed order (xor butterfly): every lane ends with
// the same value, and the same inputs always give the same bits.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Position of x in the ascending array a[0..n), or -1.
__device__ __forceinline__ int find_sorted(const int32_t* a, int n, int x) {
  int lo = 0, hi = n;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    int v = a[mid];
    if (v < x) lo = mid + 1; else hi = mid;
  }
  return (lo < n && a[lo] == x) ? lo : -1;
}

}  // namespace d2c
