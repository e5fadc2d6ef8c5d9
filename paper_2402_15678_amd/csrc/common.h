// Shared device helpers and the internal launcher interface (gfx950 only, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mn {

typedef uint16_t bf16_t;  // raw bf16 pattern (the type weights and embeddings of bf16 models arrive in)
typedef _Float16 f16_t;   // activation type and KV page type in bf16 models (see the note below)
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Precision note.  In bf16 models the weights arrive as bf16.  Every bf16 value
// in the normal fp16 range is exactly representable in fp16 (8 significant bits into 11), so the
// weights are re-encoded as fp16 once, when they are packed, the KV pages hold fp16 (the library writes
// them and reads them back), and all products run on the fp16 MFMA with fp32 accumulation, while the
// activations between kernels (norm output, queries, attention output, FFN activation, softmax
// probabilities) are kept in fp16: 8x less rounding error per stage than bf16 activations at the
// same MFMA rate and the same HBM traffic.  bf16 magnitudes below 2^-14 lose low bits in the re-encoding
// (absolute error below 2^-24), which is far below every tolerance.

constexpr int WAVE = 64;

// fp32 -> bf16, round to nearest even (inputs are finite).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// two fp32 -> packed fp16, round to nearest even
__device__ __forceinline__ uint32_t pack2h(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}
// The fp16 range guard.  Activations handed from one kernel to the next are fp16 (see the precision note), so
// a value beyond +-65504 would turn into an infinity and poison its row without a trace.  Every conversion
// of a computed activation therefore saturates (NaN becomes -65504) and reports: `bad` is set when the value
// was not within the range, and the kernel ORs MN_DEV_RANGE into the call's status word once at its end.
constexpr float F16_MAX = 65504.f;
__device__ __forceinline__ float sat_h(float v, bool& bad) {
  bad |= !(__builtin_fabsf(v) <= F16_MAX);
  return __builtin_fminf(__builtin_fmaxf(v, -F16_MAX), F16_MAX);
}
__device__ __forceinline__ uint32_t pack2h_sat(float lo, float hi, bool& bad) { return pack2h(sat_h(lo, bad), sat_h(hi, bad)); }
// 8 bf16 (16 bytes) -> 8 fp16, exact for magnitudes in [2^-14, 65504]
__device__ __forceinline__ f16x8 bf16x8_to_f16x8(u32x4 u) {
  union { f16x8 v; uint32_t w[4]; } r;
  const uint32_t in[4] = {u[0], u[1], u[2], u[3]};
#pragma unroll
  for (int i = 0; i < 4; ++i)
    r.w[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(in[i] << 16),
                                                                     __uint_as_float(in[i] & 0xffff0000u)));
  return r.v;
}

__device__ __forceinline__ f16x8 bf16x8_to_f16x8(uint4 u) { return bf16x8_to_f16x8((u32x4){u.x, u.y, u.z, u.w}); }

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Store<f16_t> {
  static __device__ __forceinline__ float load(const f16_t* p) { return (float)*p; }
  static __device__ __forceinline__ void store(f16_t* p, float v) { *p = (f16_t)v; }
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

// 64 lanes x 16 bytes, global (g + OFFSET) -> LDS at lds_base + 16 * lane.  The instruction adds its
// immediate offset to BOTH addresses, so the LDS base handed to it is lowered by the same amount.  The load
// is invisible to the compiler's wait-count bookkeeping: the kernel waits for these loads itself
// (wait_vm) and issues no other memory load while one of them may still be needed.
// STREAM: the data is read once (weights, KV pages): the load carries the non-temporal hint, so the line does not
// push out of the L2 what the kernels share and re-read (activation tiles, partial sums, code).
template <int OFFSET, bool STREAM = false>
__device__ __forceinline__ void dma16(const char* g, uint32_t lds_base) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off offset:%2 nt" ::"v"(g), "s"(lds_base - (uint32_t)OFFSET), "n"(OFFSET) : "memory");
  else
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off offset:%2" ::"v"(g), "s"(lds_base - (uint32_t)OFFSET), "n"(OFFSET) : "memory");
}
// wait until at most N of this wave's memory loads are outstanding (they complete in order)
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(((N & 15) | ((N >> 4) << 14)) | (7 << 4) | (15 << 8));
  asm volatile("" ::: "memory");
}

// ---- per-row metadata produced by the prepare kernel ----
struct RowInfo {
  const int32_t* row_seq;   // [M] sequence of row m
  const int32_t* row_j;     // [M] offset inside its sequence
  const int32_t* row_pos;   // [M] absolute position ctx_b + j, or -1 when the sequence is disabled
  const int32_t* row_tok;   // [M] input token
  const int32_t* row_slot;  // [M] where the row's K/V go: physical block * block_size + offset, or -1 (disabled)
  const int32_t* seq_row0;  // [B+1] first row of sequence b
  const int32_t* seq_ctx;   // [B] ctx_b as read at the start of the step (0 for disabled sequences)
  const int32_t* seq_ok;    // [B] 1 = enabled
  const int32_t* attn_tps;  // [1] key tiles (32 keys) one attention workgroup should take: sets the KV splits per sequence
};

struct KvView {
  void* k;  // [num_blocks][Hkv][hd/8][bs][8]
  void* v;  // [num_blocks][Hkv][hd][bs]
  const int32_t* block_tables;
  int block_size, num_blocks, max_blocks_per_seq;
};

}  // namespace mn
