// Two measuring sticks for the box the library runs on: a plain streaming read and a dense fp16 MFMA
// loop.  They do no work of the method; bench.py times them beside the verification step so that the
// roofline fractions it prints can also be read against what this very chip sustains.
#include "common.h"
#include "../../include/minions_verify.h"

namespace mn {

// every thread reads 4 x 16 bytes per trip, 1 KB per wave instruction, the whole grid striding over the buffer;
// the loads carry the non-temporal hint, as the weight and KV streams of the library do
__global__ void __launch_bounds__(256) probe_stream_kernel(const u32x4* __restrict__ p, size_t n16, uint32_t* sink) {
  u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 1024;
  for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < n16; i += stride) {
    const u32x4 v0 = __builtin_nontemporal_load(p + i), v1 = __builtin_nontemporal_load(p + i + 256),
                v2 = __builtin_nontemporal_load(p + i + 512), v3 = __builtin_nontemporal_load(p + i + 768);
    acc ^= v0 ^ v1 ^ v2 ^ v3;
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u && sink) *sink = acc[0];  // (keeps the loads alive)
}

// eight independent accumulator chains of the 16x16x32 fp16 MFMA per wave, two waves per SIMD.
// DATA = false: every operand element is the same small constant (few bits toggle: the loop holds the
// boost clock); DATA = true: four A and four B fragments of random sign and mantissa, magnitudes in
// [0.5, 1), so the multipliers see what a real product feeds them (the power management then settles at
// a lower clock: this is the rate a dense product can hope for on this chip).
template <bool DATA>
__global__ void __launch_bounds__(512, 1) probe_mfma_kernel(int iters, float* sink) {
  f32x4 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
  f16x8 a[4], b[4];
  uint32_t h = (uint32_t)threadIdx.x * 2654435761u + 12345u;
#pragma unroll
  for (int f = 0; f < 8; ++f) {
    u32x4 bits;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      h = h * 1664525u + 1013904223u;
      // two halves per word: sign and mantissa from the generator, exponent of 0.5 (or the constant 0.5)
      bits[e] = DATA ? (((h >> 8) & 0x83ff83ffu) | 0x38003800u) : 0x38003800u;
    }
    if (f < 4) a[f] = __builtin_bit_cast(f16x8, bits);
    else b[f - 4] = __builtin_bit_cast(f16x8, bits);
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i & 7] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[i & 3], b[(i >> 2) & 3], acc[i & 7], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) t += acc[i][0];
  if (t == 12345.678f && sink) *sink = t;
}

}  // namespace mn

extern "C" mn_status mn_probe_stream_read(const void* buf, size_t bytes, void* stream) {
  if (!buf) return MN_ENULL;
  if (bytes < (1u << 20) || (reinterpret_cast<uintptr_t>(buf) & 15u)) return MN_EINVAL;
  mn::probe_stream_kernel<<<2048, 256, 0, (hipStream_t)stream>>>(reinterpret_cast<const mn::u32x4*>(buf), bytes / 16, nullptr);
  return hipGetLastError() == hipSuccess ? MN_OK : MN_EHIP;
}

static mn_status probe_mfma(bool data, int iters, double* flop, void* stream) {
  if (iters < 1 || iters > (1 << 22)) return MN_EINVAL;
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
    return MN_EHIP;
  if (data) mn::probe_mfma_kernel<true><<<cus, 512, 0, (hipStream_t)stream>>>(iters, nullptr);
  else mn::probe_mfma_kernel<false><<<cus, 512, 0, (hipStream_t)stream>>>(iters, nullptr);
  if (flop) *flop = (double)iters * 32.0 * (2.0 * 16 * 16 * 32) * 8.0 * (double)cus;  // 8 waves per workgroup, one per CU
  return hipGetLastError() == hipSuccess ? MN_OK : MN_EHIP;
}

extern "C" mn_status mn_probe_mfma(int iters, double* flop, void* stream) { return probe_mfma(false, iters, flop, stream); }

extern "C" mn_status mn_probe_mfma_data(int iters, double* flop, void* stream) { return probe_mfma(true, iters, flop, stream); }
