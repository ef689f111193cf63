// Shared device-side types and small helpers for the gfx950 prefill kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp {

typedef __bf16 bf16;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;          // CDNA wavefront width
constexpr int kKvBlock = 16;       // tokens per KV-cache block
constexpr int kOpsPerLayer = 9;

// Eight consecutive elements of the storage type, loaded/stored as one vector and handled in
// fp32 registers.  bf16: one 16-byte access; fp32: two 16-byte accesses.
// SiLU(gate) * up in fp32: the one formula both the stand-alone operator and the fused GEMM
// epilogue use, so the two give the same bits.
__device__ __forceinline__ float silu_mul_f32(float g, float u) {
  return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;   // v_rcp_f32 (1 ulp) instead of the IEEE division sequence
}

template <typename T> struct Vec8;

template <> struct Vec8<bf16> {
  static __device__ __forceinline__ f32x8 load(const bf16* p) {
    bf16x8 v = *reinterpret_cast<const bf16x8*>(p);
    return __builtin_convertvector(v, f32x8);
  }
  static __device__ __forceinline__ void store(bf16* p, f32x8 v) {
    *reinterpret_cast<bf16x8*>(p) = __builtin_convertvector(v, bf16x8);
  }
};

template <> struct Vec8<float> {
  static __device__ __forceinline__ f32x8 load(const float* p) {
    f32x4 a = *reinterpret_cast<const f32x4*>(p);
    f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
    return f32x8{a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  }
  static __device__ __forceinline__ void store(float* p, f32x8 v) {
    *reinterpret_cast<f32x4*>(p) = f32x4{v[0], v[1], v[2], v[3]};
    *reinterpret_cast<f32x4*>(p + 4) = f32x4{v[4], v[5], v[6], v[7]};
  }
};

__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
__device__ __forceinline__ float to_f32(float v) { return v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return static_cast<T>(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

}  // namespace fp
