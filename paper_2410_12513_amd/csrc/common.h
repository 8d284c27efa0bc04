// Device helpers shared by the decode and prefill kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace first {

constexpr int WG = 256;          // threads per workgroup in every kernel of this library
constexpr int WAVES = WG / 64;   // wavefronts per workgroup

struct bf16 { uint16_t v; };     // raw upper half of an fp32
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));   // 16 bytes that stay in registers (arrays of HIP's uint4 tend to end up in scratch)

template <typename T> struct Vec;                // elements per 16-byte vector
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<bf16>  { static constexpr int N = 8; };

__device__ __forceinline__ float bf2f(uint32_t b) { return __uint_as_float(b << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return bf2f(x.v); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { bf16 r; r.v = f2bf(x); return r; }
// value after a round trip through the storage type
template <typename T> __device__ __forceinline__ float round_to(float x) { return to_f32(from_f32<T>(x)); }

// One 16-byte global/LDS load widened to fp32.
__device__ __forceinline__ void load_vec(const float* p, float (&o)[4]) {
  const float4 v = *reinterpret_cast<const float4*>(p);
  o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
}
__device__ __forceinline__ void load_vec(const bf16* p, float (&o)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
  o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xffff0000u);
  o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xffff0000u);
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

// Sum over the 256 threads of a workgroup in a fixed order; red: LDS float[WAVES].
// Ends with every thread holding the total.  Contains two barriers.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) t += red[w];
  return t;
}

// Workgroup barrier that orders LDS traffic only: unlike __syncthreads() it does not wait
// for outstanding global loads, so prefetches stay in flight across it.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ float sigmoidf(float z) { return 1.0f / (1.0f + expf(-z)); }
__device__ __forceinline__ float siluf(float z) { return z / (1.0f + expf(-z)); }

// (value, index) pair ordered as greedy decoding needs it: larger value first, then the
// lower index on exact ties.
struct Best { float v; int i; };
__device__ __forceinline__ bool better(const Best& a, const Best& b) {
  return a.v > b.v || (a.v == b.v && a.i < b.i);
}

// The split activation vectors of the (up to) 16 sequences of a pass are kept in the order the
// MFMA A operand wants them: block s = elements 32 s .. 32 s + 31 of all 16 slots is 1 KB, lane
// l = slot + 16 g of a wave owns its 16 bytes l (slot's elements 32 s + 8 g .. + 8).  One A load
// of a wave is then 1 KB contiguous instead of sixteen 64-byte pieces one vector pitch apart.
__host__ __device__ __forceinline__ size_t bg_aidx(int slot, int k) {
  return ((size_t)(k >> 5) << 9) + (size_t)((((k >> 3) & 3) << 4) + slot) * 8 + (k & 7);
}


}  // namespace first
