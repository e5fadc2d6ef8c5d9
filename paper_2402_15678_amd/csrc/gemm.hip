// Projection GEMMs of the verification forward: out[m][n] = sum_k a[m][k] * w[n][k].
//
// The verification step scores only M = sum_b (k_b + 1) rows (tens to a few hundred) against
// matrices of 10^8..10^9 parameters, so every weight byte is needed exactly once per step and
// the kernel is a weight streamer: weights go HBM -> registers (bf16 widened exactly to fp16) ->
// MFMA with no staging (both operands are contiguous along k, which is what the 16x16x32 MFMA
// wants: 8 consecutive k per lane), the small fp16 activation tile is shared by the four waves of
// a workgroup through LDS, and all M rows of a chunk are covered by one workgroup so no weight
// byte is read twice.
//
// Weight layout ("packed"): HBM only streams near its peak when every workgroup reads long
// contiguous runs, so the matrices of bf16 models are stored pre-tiled for this kernel.  A matrix
// [N][K] is cut into blocks of 128 output columns x 128 k; block (nb, kb) is the 32 KB at offset
// (nb * K/128 + kb) * 32 KB, so one workgroup walks one contiguous stream.  Inside a block the
// fragment of wave w, column tile nt, k-step ks is the 1 KB at ((w*2 + nt)*4 + ks) KB, stored in
// lane order: lane l holds output column (w*2 + nt)*16 + l%16, k = ks*32 + (l/16)*8 .. +7.
// Rows past N are zero.  pack_weight_kernel converts from row-major.
#include "launch.h"
#include "../../include/minions_verify.h"

#include <cstdlib>
#include <type_traits>

namespace mn {

constexpr int KSTEP = 32;         // k elements per MFMA
constexpr int KS = 4;             // MFMA k-steps per main-loop iteration
constexpr int KB = KS * KSTEP;    // k elements per main-loop iteration (128)
constexpr int LDS_ROW = KB;       // row of the activation tile in fp16 elements: 256 bytes, unpadded (see lds_slot)
constexpr int NWG = 128;          // output columns per workgroup
constexpr int WBLOCK = NWG * KB;  // elements of one packed 128 x 128 weight block (32 KB)

// The activation tile keeps 256-byte rows (two buffers of a 144-row tile for two workgroups per CU
// must fit the 160 KB of LDS, so there is no room for padding) and rotates the sixteen 16-byte
// chunks of row r by 2r instead: byte address r*256 + ((chunk + 2r) mod 16)*16.  That is the bank
// pattern of a 288-byte row stride, which the LDS conflict counter reads as zero for this kernel's
// ds_read_b128 pattern (16 rows x one chunk per quarter wave); 272-byte rows conflict on 40 % of
// the LDS cycles.
__device__ __forceinline__ int lds_slot(int row, int chunk) { return row * LDS_ROW + (((chunk + 2 * row) & 15) << 3); }

template <int MT>
constexpr size_t gemm_smem_bytes() { return (size_t)2 * 16 * MT * LDS_ROW * sizeof(f16_t); }

// Workgroup = 4 waves; wave w owns NTW 16-column tiles; every wave covers all MT 16-row tiles.
// MFMA orientation: the weight fragment is the row operand (rows = output columns n), the
// activation fragment is the column operand (columns = rows m of the output), so a lane ends up
// with 4 consecutive n for one m.
//
// Pipeline per wave: the raw bf16 weight fragments of iterations it+1 and it+2 are in flight in a
// two-slot register ring while iteration it runs on the MFMA (the slot of iteration it is widened
// to fp16 at the top of the iteration and refilled at once for it+2); the activation tile of
// iteration it+1 travels global -> registers -> the other LDS buffer during the same time.
//
// Epilogues: EPI_PARTIAL stores the fp32 partial sums of this split ([S][M][N], bias on split 0).
// EPI_SWIGLU (Llama first FFN projection, one split): the matrix was packed with gate and up rows
// interleaved per 16-column tile, so a wave's two tiles are gate and up of the same 16 FFN
// columns; it stores silu(gate) * up as fp16 [M][F] and nothing else.
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1 };

template <int MT, int NTW, int EPI>
__global__ void __launch_bounds__(256, 2) gemm_w16_kernel(const f16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                           void* __restrict__ out_, const float* __restrict__ bias,
                                                           int M, int N, int K, int k_per_split) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gemm_smem[];
  f16_t* s_a = reinterpret_cast<f16_t*>(gemm_smem);  // [2][16*MT][LDS_ROW]
  constexpr int TILE = 16 * MT * LDS_ROW;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int n_wg = blockIdx.x * (64 * NTW);
  const int split = blockIdx.y;
  const int m0 = blockIdx.z * (16 * MT);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_iter = (k_end - k_begin) / KB;

  // this wave's stream inside the workgroup's contiguous run of 32 KB blocks
  const bf16_t* wbase = W + ((size_t)blockIdx.x * (K / KB) + k_begin / KB) * (size_t)WBLOCK + wave * (NTW * KS * 512) + lane * 8;

  // Activation tile staging: 16*MT rows x 16 chunks of 16 bytes = MT chunks per thread.  Every load in the main loop is unconditional, with
  // clamped addresses (rows past M re-read row M-1 and feed output rows that are never stored;
  // iterations past the end re-read the last block), so the compiler can count outstanding loads and
  // wait for exactly the ones it needs instead of draining the queue.
  constexpr int CPR = KB / 8;  // chunks per row
  static_assert(16 * MT * CPR == MT * 256, "one chunk per thread per row tile");
  const int a_r0 = tid / CPR, a_ch = tid % CPR;  // chunk i of this thread: row a_r0 + 16 i, 16-byte chunk a_ch
  const f16_t* a_base = A + k_begin + a_ch * 8;
  const int a_dst0 = lds_slot(a_r0, a_ch);  // rows 16 apart share the rotation: (2 * 16) mod 16 == 0
  const int last = n_iter - 1;
  const bf16_t* wlane = wbase;

#define MN_LOAD_A(STAGE, LO, CNT, IT)                                                              \
  _Pragma("unroll") for (int i_ = 0; i_ < (CNT); ++i_) {                                           \
    const int row_ = min(m0 + a_r0 + 16 * ((LO) + i_), M - 1);                                     \
    STAGE[i_] = *reinterpret_cast<const u32x4*>(a_base + (size_t)row_ * K + (IT) * KB);            \
  }
#define MN_STORE_A(STAGE, LO, CNT, BUF)                                                            \
  _Pragma("unroll") for (int i_ = 0; i_ < (CNT); ++i_)                                             \
    *reinterpret_cast<u32x4*>(&s_a[(BUF) * TILE + a_dst0 + ((LO) + i_) * 16 * LDS_ROW]) = STAGE[i_];
#define MN_W_PTR(IT, NT, KS_) \
  reinterpret_cast<const u32x4*>(wlane + (size_t)min((IT), last) * WBLOCK + ((NT) * KS + (KS_)) * 512)

  f32x4 acc[NTW][MT];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (n_iter > 0) {  // (uniform per workgroup)
    u32x4 ring0[NTW][KS], ring1[NTW][KS];  // raw bf16 fragments of the next two iterations
    {
      u32x4 st0[MT];
      MN_LOAD_A(st0, 0, MT, 0)
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          ring0[nt][ks] = *MN_W_PTR(0, nt, ks);
          ring1[nt][ks] = *MN_W_PTR(1, nt, ks);
        }
      MN_STORE_A(st0, 0, MT, 0)
      // Land the first two ring slots before the loop (an empty asm that reads them).  The compiler sizes
      // its in-loop waits by the shortest distance between a load and its use over all paths; without
      // this the short prologue path would halve the prefetch depth of every iteration.
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          asm volatile("" : "+v"(ring0[nt][ks]));
          asm volatile("" : "+v"(ring1[nt][ks]));
        }
    }
    __syncthreads();

#ifndef MN_ABLATE
#define MN_ABLATE 0
#endif
#if MN_ABLATE & 1  // experiment: no LDS reads / MFMAs, keep the weight stream alive
#define MN_ABLATE_GROUPS 0
#define MN_ABLATE_SKIP_COMPUTE(W) { acc[0][0][0] += (float)W[0][0] + (float)W[1][0]; }
#else
#define MN_ABLATE_GROUPS 2
#define MN_ABLATE_SKIP_COMPUTE(W)
#endif
// One iteration on ring slot RING.  Issue order matters because loads return in order: the next
// activation tile (L2 hits, needed at the end of this iteration) goes first, then, k-step by k-step, the
// weight refills for iteration it+2 (HBM, needed two iterations from now), so waiting for the tile
// never waits for a refill.  The row tiles of a k-step run in two groups to keep the live set small.
#define MN_GEMM_ITER(RING, IT)                                                                              \
  {                                                                                                         \
    const int it_ = (IT);                                                                                   \
    const int buf_ = it_ & 1;                                                                               \
    const int nxt_ = min(it_ + 1, last);                                                                    \
    u32x4 sa_[MT];                                                                                          \
    if (!(MN_ABLATE & 2)) { MN_LOAD_A(sa_, 0, MT, nxt_) }                                                   \
    /* a compiler-level memory fence: without it the loads above are sunk to the stores at the bottom */    \
    asm volatile("" ::: "memory");                                                                          \
    const f16_t* tile_ = s_a + buf_ * TILE;                                                                 \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                                     \
      f16x8 wcur_[NTW];                                                                                     \
      _Pragma("unroll") for (int nt = 0; nt < NTW; ++nt) {                                                  \
        wcur_[nt] = bf16x8_to_f16x8(RING[nt][ks]);                                                          \
        RING[nt][ks] = *MN_W_PTR(it_ + 2, nt, ks);                                                          \
      }                                                                                                     \
      MN_ABLATE_SKIP_COMPUTE(wcur_)                                                                         \
      _Pragma("unroll") for (int grp = 0; grp < MN_ABLATE_GROUPS; ++grp) {                                  \
        constexpr int G0 = (MT + 1) / 2;                                                                    \
        const int lo_ = grp ? G0 : 0, cnt_ = grp ? MT - G0 : G0;                                            \
        f16x8 bfrag_[G0];                                                                                   \
        _Pragma("unroll") for (int i = 0; i < G0; ++i)                                                      \
          if (i < cnt_)                                                                                     \
            bfrag_[i] = *reinterpret_cast<const f16x8*>(&tile_[(lo_ + i) * 16 * LDS_ROW + lds_slot(l16, ks * 4 + g)]); \
        _Pragma("unroll") for (int nt = 0; nt < NTW; ++nt)                                                  \
          _Pragma("unroll") for (int i = 0; i < G0; ++i)                                                    \
            if (i < cnt_)                                                                                   \
              acc[nt][lo_ + i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wcur_[nt], bfrag_[i], acc[nt][lo_ + i], 0, 0, 0); \
        __builtin_amdgcn_sched_barrier(0);                                                                  \
      }                                                                                                     \
    }                                                                                                       \
    if (!(MN_ABLATE & 2)) { MN_STORE_A(sa_, 0, MT, buf_ ^ 1) }                                              \
    if (!(MN_ABLATE & 4)) __syncthreads();                                                                  \
  }

    // pairs of iterations with no branch inside the loop (a conditional second half would give the
    // compiler a short path that shrinks every wait), then the odd one out
    int it = 0;
    for (; it + 1 < n_iter; it += 2) {
      MN_GEMM_ITER(ring0, it)
      MN_GEMM_ITER(ring1, it + 1)
    }
    if (it < n_iter) MN_GEMM_ITER(ring0, it)
#undef MN_GEMM_ITER
  }
#undef MN_LOAD_A
#undef MN_STORE_A
#undef MN_W_PTR

  // epilogue: lane holds D[n = base + 4g + i][m = mt*16 + l16]
  if constexpr (EPI == EPI_SWIGLU) {
    static_assert(NTW == 2, "gate and up tiles of one wave");
    f16_t* act = reinterpret_cast<f16_t*>(out_);
    const int F = N >> 1;
    const int f = blockIdx.x * 64 + wave * 16 + g * 4;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int m = m0 + mt * 16 + l16;
      if (m >= M || f >= F) continue;
      const f32x4 gt = acc[0][mt], up = acc[1][mt];
      float r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) r[i] = gt[i] / (1.f + __expf(-gt[i])) * up[i];
      *reinterpret_cast<uint2*>(act + (size_t)m * F + f) = make_uint2(pack2h(r[0], r[1]), pack2h(r[2], r[3]));
    }
  } else {
    float* o = reinterpret_cast<float*>(out_) + (size_t)split * M * N;
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
}

// Row-major [N][K] bf16 -> the packed layout described at the top.  One thread per 16-byte piece.
// With half > 0 (Llama gate||up, N = 2*half) packed column tile 2t holds gate rows [16t, 16t+16)
// and tile 2t+1 the up rows half + [16t, 16t+16).
__global__ void __launch_bounds__(256) pack_weight_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N,
                                                          int K, int half) {
  const size_t pieces = (size_t)((N + NWG - 1) / NWG) * (K / KB) * (WBLOCK / 8);
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < pieces; idx += (size_t)gridDim.x * blockDim.x) {
    const size_t blk = idx / (WBLOCK / 8);
    const int p = (int)(idx % (WBLOCK / 8));
    const int nb = (int)(blk / (K / KB)), kb = (int)(blk % (K / KB));
    const int frag = p >> 6, lane = p & 63;
    const int tile = frag / KS, ks = frag % KS;
    const int prow = nb * NWG + tile * 16 + (lane & 15);
    const int k = kb * KB + ks * KSTEP + (lane >> 4) * 8;
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (prow < N) {
      int srow = prow;
      if (half > 0) {
        const int t = prow >> 4, r = prow & 15;
        srow = ((t & 1) ? half : 0) + (t >> 1) * 16 + r;
      }
      v = *reinterpret_cast<const uint4*>(src + (size_t)srow * K + k);
    }
    *reinterpret_cast<uint4*>(dst + idx * 8) = v;
  }
}

size_t packed_weight_elems(int N, int K) { return (size_t)((N + NWG - 1) / NWG) * NWG * (size_t)K; }

void launch_pack_weight(const void* src, void* dst, int N, int K, int half, hipStream_t st) {
  const size_t pieces = packed_weight_elems(N, K) / 8;
  size_t blocks = (pieces + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  pack_weight_kernel<<<(int)blocks, 256, 0, st>>>(reinterpret_cast<const bf16_t*>(src), reinterpret_cast<bf16_t*>(dst), N, K, half);
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
  int split;    // 0 = automatic
  int target;   // workgroups to aim for
};
static GemmTune tune() {
  static GemmTune t = [] {
    GemmTune x{0, 512};
    if (const char* e = getenv("MN_GEMM_SPLIT")) x.split = atoi(e);
    if (const char* e = getenv("MN_GEMM_TARGET_WGS")) x.target = atoi(e);
    return x;
  }();
  return t;
}

int gemm_pick_split(int M, int N, int K, int dtype) {
  if (dtype != MN_DT_BF16) return 1;
  const int forced = tune().split;
  const int nblocks = (N + NWG - 1) / NWG;
  const int iters = K / KB;
  // as many splits as keep the whole grid resident at once (two workgroups per CU), each split at
  // least 16 iterations long (measured: shorter splits lose more to ramp-up and partial sums than
  // the extra workgroups win)
  int s = forced >= 1 ? forced : tune().target / nblocks;
  if (forced < 1 && s > iters / 16) s = iters / 16;
  if (s > MN_MAX_SPLIT_K) s = MN_MAX_SPLIT_K;
  if (s < 1) s = 1;
  // drop splits that would get no iteration
  const int per = (iters + s - 1) / s;
  return (iters + per - 1) / per;
}

template <int MT>
static void launch_bf16_mt(const GemmArgs& a, int m_chunks, hipStream_t st) {
  const int iters = a.K / KB;
  const int per = (iters + a.split_k - 1) / a.split_k;  // iterations per split
  dim3 grid((a.N + NWG - 1) / NWG, a.split_k, m_chunks);
  const f16_t* A = reinterpret_cast<const f16_t*>(a.a);
  const bf16_t* W = reinterpret_cast<const bf16_t*>(a.w);
  constexpr size_t smem = gemm_smem_bytes<MT>();
  static bool attr_set = false;  // once per instantiation: allow more than 64 KB of dynamic LDS
  if (!attr_set) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_w16_kernel<MT, 2, EPI_PARTIAL>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_w16_kernel<MT, 2, EPI_SWIGLU>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    attr_set = true;
  }
  if (a.swiglu_act)
    gemm_w16_kernel<MT, 2, EPI_SWIGLU><<<grid, 256, smem, st>>>(A, W, a.swiglu_act, nullptr, a.M, a.N, a.K, per * KB);
  else
    gemm_w16_kernel<MT, 2, EPI_PARTIAL><<<grid, 256, smem, st>>>(A, W, a.out, a.bias, a.M, a.N, a.K, per * KB);
}

void launch_gemm(const GemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return;
  if (a.dtype != MN_DT_BF16) {
    dim3 grid((a.N + 3) / 4, (a.M + 7) / 8);
    gemm_f32_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const float*>(a.a), reinterpret_cast<const float*>(a.w),
                                          a.out, a.bias, a.M, a.N, a.K);
    return;
  }
  const int tiles = (a.M + 15) / 16;
  // row tiles per workgroup: everything in one chunk up to 9 tiles (144 rows), else chunks of 8
  if (tiles <= 1) launch_bf16_mt<1>(a, 1, st);
  else if (tiles <= 2) launch_bf16_mt<2>(a, 1, st);
  else if (tiles <= 3) launch_bf16_mt<3>(a, 1, st);
  else if (tiles <= 4) launch_bf16_mt<4>(a, 1, st);
  else if (tiles <= 6) launch_bf16_mt<6>(a, 1, st);
  else if (tiles <= 9) launch_bf16_mt<9>(a, 1, st);
  else launch_bf16_mt<8>(a, (tiles + 7) / 8, st);
}

}  // namespace mn
