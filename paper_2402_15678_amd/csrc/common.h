// Shared device helpers and the internal launcher interface (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mn {

typedef uint16_t bf16_t;  // raw bf16 pattern
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

constexpr int WAVE = 64;

// fp32 -> bf16, round to nearest even (inputs are finite).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) { return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16); }

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Store<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf2f(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f2bf(v); }
};

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

// Sum over a block of NW waves; every thread gets the result.  `red` holds NW floats.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NW; ++i) t += red[i];
  return t;
}

// ---- per-row metadata produced by the prepare kernel ----
struct RowInfo {
  const int32_t* row_seq;   // [M] sequence of row m
  const int32_t* row_j;     // [M] offset inside its sequence
  const int32_t* row_pos;   // [M] absolute position ctx_b + j, or -1 when the sequence is disabled
  const int32_t* row_tok;   // [M] input token
  const int32_t* seq_row0;  // [B+1] first row of sequence b
  const int32_t* seq_ctx;   // [B] ctx_b as read at the start of the step (0 for disabled sequences)
  const int32_t* seq_ok;    // [B] 1 = enabled
};

struct KvView {
  void* k;  // [num_blocks][Hkv][hd/8][bs][8]
  void* v;  // [num_blocks][Hkv][hd][bs]
  const int32_t* block_tables;
  int block_size, num_blocks, max_blocks_per_seq;
};

}  // namespace mn
