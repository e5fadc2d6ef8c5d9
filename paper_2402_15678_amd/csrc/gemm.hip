// Projection GEMMs of the verification forward: out[m][n] = sum_k a[m][k] * w[n][k].
//
// The verification step scores only M = sum_b (k_b + 1) rows (tens to a few hundred) against
// matrices of 10^8..10^9 parameters, so every weight byte is needed exactly once per step and
// the kernel is a weight streamer: weights go HBM -> registers (bf16 widened exactly to fp16) ->
// MFMA with no staging (both operands are contiguous along k, which is what the 16x16x32 MFMA
// wants: 8 consecutive k per lane), the small fp16 activation tile is shared by the four waves of
// a workgroup through LDS, and all M rows of a chunk are covered by one workgroup so no weight
// byte is read twice.
#include "launch.h"
#include "../../include/minions_verify.h"

#include <cstdlib>

namespace mn {

constexpr int KB = 64;            // k elements per main-loop iteration (two MFMA k-steps)
constexpr int LDS_ROW = KB + 8;   // padded row of the activation tile, in fp16 elements (144 bytes)

// Workgroup = 4 waves; wave w owns NTW 16-column tiles; every wave covers all MT 16-row tiles.
// MFMA orientation: the weight fragment is the row operand (rows = output columns n), the
// activation fragment is the column operand (columns = rows m of the output), so a lane ends up
// with 4 consecutive n for one m.
template <int MT, int NTW>
__global__ void __launch_bounds__(256) gemm_w16_kernel(const f16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                        float* __restrict__ out, const float* __restrict__ bias,
                                                        int M, int N, int K, int k_per_split) {
  __shared__ __attribute__((aligned(16))) f16_t s_a[2][16 * MT * LDS_ROW];
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int n_wg = blockIdx.x * (64 * NTW);
  const int split = blockIdx.y;
  const int m0 = blockIdx.z * (16 * MT);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_iter = (k_end - k_begin) / KB;

  // weight rows of this lane (clamped: rows past N are computed on valid memory and dropped)
  const bf16_t* wrow[NTW];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt) {
    int n = n_wg + (wave * NTW + nt) * 16 + l16;
    n = n < N ? n : N - 1;
    wrow[nt] = W + (size_t)n * K + k_begin + g * 8;
  }

  // activation tile staging: 16*MT rows x 8 chunks of 16 bytes, spread over 256 threads
  constexpr int A_CHUNKS = 16 * MT * (KB / 8);
  constexpr int A_PER_THREAD = (A_CHUNKS + 255) / 256;
  uint4 a_stage[A_PER_THREAD];
  auto load_a = [&](int kb) {
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
      const int c = i * 256 + tid;
      const int r = c >> 3, ch = c & 7;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (c < A_CHUNKS && m0 + r < M) v = *reinterpret_cast<const uint4*>(A + (size_t)(m0 + r) * K + kb + ch * 8);
      a_stage[i] = v;
    }
  };
  auto store_a = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
      const int c = i * 256 + tid;
      const int r = c >> 3, ch = c & 7;
      if (c < A_CHUNKS) *reinterpret_cast<uint4*>(&s_a[buf][r * LDS_ROW + ch * 8]) = a_stage[i];
    }
  };

  f32x4 acc[NTW][MT];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  f16x8 wcur[NTW][2];
  uint4 wnxt[NTW][2];  // raw bf16 of the next iteration, widened when it becomes current
  if (n_iter > 0) {
    load_a(k_begin);
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      wcur[nt][0] = bf16x8_to_f16x8(*reinterpret_cast<const uint4*>(wrow[nt]));
      wcur[nt][1] = bf16x8_to_f16x8(*reinterpret_cast<const uint4*>(wrow[nt] + 32));
    }
    store_a(0);
  }
  __syncthreads();

  for (int it = 0; it < n_iter; ++it) {
    const int buf = it & 1;
    const bool more = it + 1 < n_iter;
    if (more) {
      const int koff = (it + 1) * KB;
      load_a(k_begin + koff);
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        wnxt[nt][0] = *reinterpret_cast<const uint4*>(wrow[nt] + koff);
        wnxt[nt][1] = *reinterpret_cast<const uint4*>(wrow[nt] + koff + 32);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      f16x8 bfrag[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
        bfrag[mt] = *reinterpret_cast<const f16x8*>(&s_a[buf][(mt * 16 + l16) * LDS_ROW + ks * 32 + g * 8]);
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wcur[nt][ks], bfrag[mt], acc[nt][mt], 0, 0, 0);
    }
    if (more) {
      store_a(buf ^ 1);
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        wcur[nt][0] = bf16x8_to_f16x8(wnxt[nt][0]);
        wcur[nt][1] = bf16x8_to_f16x8(wnxt[nt][1]);
      }
    }
    __syncthreads();
  }

  // epilogue: lane holds D[n = base + 4g + i][m = mt*16 + l16]
  float* o = out + (size_t)split * M * N;
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt) {
    const int n = n_wg + (wave * NTW + nt) * 16 + g * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 16 + l16;
      if (m >= M || n >= N) continue;
      f32x4 v = acc[nt][mt];
      if (bias && split == 0) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n + i < N) v[i] += bias[n + i];
      }
      float* p = o + (size_t)m * N + n;
      if (n + 3 < N && (N & 3) == 0) {
        *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n + i < N) p[i] = v[i];
      }
    }
  }
}

// fp32 model (the small configuration): one wave per output column, lanes split k, up to 8 rows
// at a time.  Plain FMA; the summation order is fixed (per-lane partial sums, then a xor tree).
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W,
                                                       float* __restrict__ out, const float* __restrict__ bias, int M,
                                                       int N, int K) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = blockIdx.x * 4 + wave;
  const int m0 = blockIdx.y * 8;
  if (n >= N) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  const float* wr = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float w = wr[k];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      if (m0 + i < M) acc[i] = fmaf(A[(size_t)(m0 + i) * K + k], w, acc[i]);
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float s = wave_sum(acc[i]);
    if (lane == 0 && m0 + i < M) out[(size_t)(m0 + i) * N + n] = s + (bias ? bias[n] : 0.f);
  }
}

// out[i] = sum_s partials[s][i], ascending s
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ p, int S, size_t stride,
                                                              float* __restrict__ out, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float v = 0.f;
    for (int s = 0; s < S; ++s) v += p[(size_t)s * stride + i];
    out[i] = v;
  }
}

void launch_reduce_partials(const float* partials, int S, size_t stride, float* out, size_t n, hipStream_t st) {
  if (n == 0) return;
  size_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  reduce_partials_kernel<<<(int)blocks, 256, 0, st>>>(partials, S, stride, out, n);
}

// ---- launch geometry -------------------------------------------------------------------------
struct GemmTune {
  int ntw;      // 0 = automatic
  int split;    // 0 = automatic
  int target;   // workgroups to aim for
};
static GemmTune tune() {
  static GemmTune t = [] {
    GemmTune x{0, 0, 512};
    if (const char* e = getenv("MN_GEMM_NTW")) x.ntw = atoi(e);
    if (const char* e = getenv("MN_GEMM_SPLIT")) x.split = atoi(e);
    if (const char* e = getenv("MN_GEMM_TARGET_WGS")) x.target = atoi(e);
    return x;
  }();
  return t;
}

static int pick_ntw(int N) {
  const int t = tune().ntw;
  if (t == 2 || t == 4) return t;
  return (N >= 24576) ? 4 : 2;
}

int gemm_pick_split(int M, int N, int K, int dtype) {
  if (dtype != MN_DT_BF16) return 1;
  const int forced = tune().split;
  const int n_wg = 64 * pick_ntw(N);
  const int nblocks = (N + n_wg - 1) / n_wg;
  int s = 1;
  if (forced >= 1) s = forced;
  else
    while (s < MN_MAX_SPLIT_K && nblocks * s < tune().target && K / (s * 2) >= 512) s *= 2;
  if (s > MN_MAX_SPLIT_K) s = MN_MAX_SPLIT_K;
  while (s > 1 && (K / KB) < s) s >>= 1;
  return s;
}

template <int MT>
static void launch_bf16_mt(const GemmArgs& a, int ntw, int m_chunks, hipStream_t st) {
  const int n_wg = 64 * ntw;
  const int iters = a.K / KB;
  const int per = (iters + a.split_k - 1) / a.split_k;  // iterations per split
  dim3 grid((a.N + n_wg - 1) / n_wg, a.split_k, m_chunks);
  const f16_t* A = reinterpret_cast<const f16_t*>(a.a);
  const bf16_t* W = reinterpret_cast<const bf16_t*>(a.w);
  if (ntw == 4)
    gemm_w16_kernel<MT, 4><<<grid, 256, 0, st>>>(A, W, a.out, a.bias, a.M, a.N, a.K, per * KB);
  else
    gemm_w16_kernel<MT, 2><<<grid, 256, 0, st>>>(A, W, a.out, a.bias, a.M, a.N, a.K, per * KB);
}

void launch_gemm(const GemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return;
  if (a.dtype != MN_DT_BF16) {
    dim3 grid((a.N + 3) / 4, (a.M + 7) / 8);
    gemm_f32_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const float*>(a.a), reinterpret_cast<const float*>(a.w),
                                          a.out, a.bias, a.M, a.N, a.K);
    return;
  }
  const int ntw = pick_ntw(a.N);
  const int tiles = (a.M + 15) / 16;
  // row tiles per workgroup: everything in one chunk up to 9 tiles (144 rows), else chunks of 8
  if (tiles <= 1) launch_bf16_mt<1>(a, ntw, 1, st);
  else if (tiles <= 2) launch_bf16_mt<2>(a, ntw, 1, st);
  else if (tiles <= 3) launch_bf16_mt<3>(a, ntw, 1, st);
  else if (tiles <= 4) launch_bf16_mt<4>(a, ntw, 1, st);
  else if (tiles <= 6) launch_bf16_mt<6>(a, ntw, 1, st);
  else if (tiles <= 9) launch_bf16_mt<9>(a, ntw, 1, st);
  else launch_bf16_mt<8>(a, ntw, (tiles + 7) / 8, st);
}

}  // namespace mn
