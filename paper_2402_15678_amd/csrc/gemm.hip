// Projection GEMMs of the verification forward: out[m][n] = sum_k a[m][k] * w[n][k].
//
// The verification step scores only M = sum_b (k_b + 1) rows (tens to a few hundred) against
// matrices of 10^8..10^9 parameters, so every weight byte is needed exactly once per step and
// the kernel is a weight streamer: weights go HBM -> registers -> MFMA with no staging and no
// conversion (the packed matrices hold the bf16 values re-encoded as fp16, see below) (both operands are contiguous along k, which is what the 16x16x32 MFMA
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
// Rows past N are zero.  pack_weight_kernel converts from row-major and re-encodes every bf16 value as
// the fp16 value the MFMA consumes (same two bytes per parameter; every bf16 value of magnitude in
// [2^-14, 65504] is an fp16 value, smaller ones land on the fp16 subnormal grid with an absolute
// error under 2^-24, larger ones do not occur in weights), so the main loop spends no vector
// instruction on the weight stream: the widening used to take more issue slots than the MFMAs.
#include "launch.h"
#include "tune.h"
#include "../../include/minions_verify.h"

#include <mutex>
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


// Workgroup = 4 waves; wave w owns NTW 16-column tiles; every wave covers all MT 16-row tiles.
// MFMA orientation: the weight fragment is the row operand (rows = output columns n), the
// activation fragment is the column operand (columns = rows m of the output), so a lane ends up
// with 4 consecutive n for one m.
//
// Pipeline per wave: the raw bf16 weight fragments of iterations it+1 and it+2 are in flight in a
// two-slot register ring while iteration it runs on the MFMA (the slot of iteration it is consumed
// k-step by k-step and refilled at once for it+2); the activation tile of
// iteration it+1 travels global -> registers -> the other LDS buffer during the same time.
//
// Epilogues: EPI_PARTIAL stores the fp32 partial sums of this split ([S][M][N], bias on split 0).
// EPI_SWIGLU (Llama first FFN projection, one split): the matrix was packed with gate and up rows
// interleaved per 16-column tile, so a wave's two tiles are gate and up of the same 16 FFN
// columns; it stores silu(gate) * up as fp16 [M][F] and nothing else.
// EPI_RELU (OPT first FFN projection, one split): stores max(sum + bias, 0) as fp16 [M][N].
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_RELU = 2 };

template <int MT, int NTW, int EPI, int NW, int RD>
__global__ void __launch_bounds__(NW * 64, (MT * NTW > 24 || NW > 4) ? 1 : 2) gemm_w16_kernel(const f16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                           void* __restrict__ out_, const float* __restrict__ bias,
                                                           int M, int N, int K, int k_per_split, int m_chunks, int gx,
                                                           int n_split, int32_t* __restrict__ status) {
  // two activation-tile buffers as separate objects: the compiler then knows that a DMA into one
  // does not touch the reads of the other
  __shared__ __attribute__((aligned(1024))) f16_t s_a0[16 * MT * LDS_ROW];
  __shared__ __attribute__((aligned(1024))) f16_t s_a1[16 * MT * LDS_ROW];
  // NW = 4: 128 columns per workgroup, two workgroups per CU.  NW = 5..8: up to 256 columns per
  // workgroup, one workgroup per CU: the activation tile is then fetched once for all of them, which
  // cuts the L2 -> LDS traffic and the load-unit time it costs.
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  constexpr int WPB = 8 / NTW;                                  // waves per 128-column block
  const int nblk_all = (N + NWG - 1) / NWG;
  // Grid: 1-D, mapped by hand, because workgroup ids are dealt round-robin over the 8 XCDs and each XCD has
  // its own L2.  One row chunk: all workgroups of a k-split run on the same XCDs (8 / n_split of them each,
  // or n_split / 8 splits per XCD), so an XCD's L2 fetches only the k range of the activations its splits
  // need: with the split as the slow grid index every XCD fetched the whole activation matrix (measured:
  // +67 MB of HBM fetch on the 470 MB down projection, +19 MB on the 134-168 MB ones).  Split counts that
  // neither divide 8 nor are a multiple of it keep the plain order.  More rows than one chunk holds
  // (M > 144): the row chunks of one (column group, split) pair get consecutive slots on the SAME XCD, so
  // the chunks run together and the weight block comes from HBM once and from that XCD's L2 for the others.
  int bx, split, bz = 0;
  {
    const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
    if (m_chunks > 1) {
      const int pair = (slot / m_chunks) * 8 + xcd;
      if (pair >= gx * n_split) return;  // (whole workgroup)
      bz = slot % m_chunks;
      bx = pair % gx;
      split = pair / gx;
    } else if (n_split <= 8 && 8 % n_split == 0) {
      const int r = 8 / n_split;         // XCDs per split
      split = xcd / r;
      bx = slot * r + xcd % r;
    } else if (n_split % 8 == 0) {
      const int q = n_split >> 3;        // splits per XCD
      split = (slot % q) * 8 + xcd;
      bx = slot / q;
    } else {
      split = id / gx;
      bx = id % gx;
    }
    if (bx >= gx || split >= n_split) return;  // (whole workgroup: padding of the grid)
  }
  // A workgroup covers NW consecutive wave slices (16*NTW columns each) of the matrix, whatever NW is: the
  // launcher picks the wave count that makes the grid fill the chip (7 waves = 224 columns give the
  // 57344-column matrix exactly 256 workgroups).  All waves share the activation tile.
  const int wslice = bx * NW + wave;                            // this wave's slice of the matrix
  const int nblk = wslice / WPB;                                // its 128-column block ...
  const int w4 = wslice % WPB;                                  // ... and its place inside the block
  const int nblk_rd = min(nblk, nblk_all - 1);                  // past the end: re-read the last block, store nothing
  const int n_wg = nblk * NWG;
  const int m0 = bz * (16 * MT);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_iter = (k_end - k_begin) / KB;

  // this wave's stream inside the workgroup's contiguous run of 32 KB blocks
  const bf16_t* wbase = W + ((size_t)nblk_rd * (K / KB) + k_begin / KB) * (size_t)WBLOCK + w4 * (NTW * KS * 512) + lane * 8;

  // Activation tile: 16*MT rows x 256 bytes = 4*MT chunks of 1 KB (four rows each).  Wave w brings in
  // chunks w, w + NW, ... with direct global->LDS loads (no staging registers, no ds_write): a wave
  // load drops lane i's 16 bytes at chunk base + 16 i, so lane i fetches the piece that belongs there
  // under the rotated layout: row = 4c + i/16, k-chunk = (i%16 - 2 row) mod 16.  Rows past M re-read row
  // M-1 (they feed output rows that are never stored); every load in the loop is unconditional.
  constexpr int A_PER_WAVE = (4 * MT + NW - 1) / NW;
  const f16_t* a_lane[A_PER_WAVE];
#pragma unroll
  for (int i = 0; i < A_PER_WAVE; ++i) {
    const int row = 4 * (i * NW + wave) + (lane >> 4);
    const int kc = ((lane & 15) - 2 * row) & 15;
    a_lane[i] = A + (size_t)min(m0 + row, M - 1) * K + k_begin + kc * 8;
  }
  const int last = n_iter - 1;
  const bf16_t* wlane = wbase;

#define MN_DMA_A(DST, IT)                                                                            \
  _Pragma("unroll") for (int i_ = 0; i_ < A_PER_WAVE; ++i_)                                          \
    if ((4 * MT) % NW == 0 || i_ * NW + wave < 4 * MT) /* wave-uniform */                            \
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(a_lane[i_] + (IT) * KB),     \
                                       (__attribute__((address_space(3))) void*)((DST) + (i_ * NW + wave) * 512), 16, 0, 0);
// Weight loads carry the non-temporal hint: a matrix is read once per step, and with the ordinary policy its
// 134-940 MB went through the L2s like everything else and pushed out what the kernels share and re-read (the
// activation tiles every workgroup fetches, the partial sums the next kernel reads, the code).  Measured on the
// whole step at 144 rows: 31.8 -> 29.5 ms, alternating runs on one box.
#define MN_W_PTR(IT, NT, KS_) \
  reinterpret_cast<const u32x4*>(wlane + (size_t)min((IT), last) * WBLOCK + ((NT) * KS + (KS_)) * 512)
#define MN_W_LOAD(IT, NT, KS_) __builtin_nontemporal_load(MN_W_PTR(IT, NT, KS_))
// Wait until at most N (8 or 16) of this wave's memory loads are outstanding (loads complete in order).
// The wait is the compiler's own s_waitcnt builtin, so its wait-count bookkeeping sees it, fenced on
// both sides so that no load moves across it.  Encoding (gfx9 family): vmcnt = bits [3:0] and [15:14],
// expcnt [6:4] = 7 and lgkmcnt [11:8] = 15 mean "do not wait".
#define MN_WAIT_VM(N)                                                                   \
  {                                                                                     \
    asm volatile("" ::: "memory");                                                      \
    __builtin_amdgcn_s_waitcnt((((N) & 15) | (((N) >> 4) << 14)) | (7 << 4) | (15 << 8)); \
    asm volatile("" ::: "memory");                                                      \
  }

  f32x4 acc[NTW][MT];
#pragma unroll
  for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[nt][mt] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (n_iter > 0) {  // (uniform per workgroup)
    // raw bf16 fragments of the next RD iterations (RD = 2: two slots, used alternately; RD = 1: the
    // wide-column variant for many rows, where the registers go to accumulators instead)
    u32x4 ring0[NTW][KS], ring1[RD == 2 ? NTW : 1][RD == 2 ? KS : 1];
    MN_DMA_A(s_a0, 0)
    asm volatile("" ::: "memory");
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        ring0[nt][ks] = MN_W_LOAD(0, nt, ks);
        if constexpr (RD == 2) ring1[nt][ks] = MN_W_LOAD(1, nt, ks);
      }
    // Everything lands before the loop.  Waiting for the tile and slot 0 only (slot 1 asked for behind slot 0,
    // at most 8 loads outstanding) would let the first pass overlap with the arrival of slot 1, but the compiler's
    // wait-count bookkeeping answers loads pending at the loop's entry with an s_waitcnt vmcnt(0) inside the loop
    // (with or without the register pins below), which drains the load queue on every pass.
    MN_WAIT_VM(0);
    __builtin_amdgcn_s_barrier();

// One iteration on ring slot RING, reading tile CUR and bringing the next tile into NXT.  Issue order
// matters because loads complete in order: the tile loads go first (L2 hits, needed at the end of this
// iteration), then the NTW*KS = 8 weight refills for iteration it+RD (HBM, needed two iterations from now).
// The compiler-level fences keep the groups apart, so "at most 8 outstanding" at the bottom means exactly
// "the tile has landed" without waiting for any refill.
// A fragment register is refilled only BEHIND the k-step that multiplies out of it (the refill of k-step ks
// goes out at the top of k-step ks+1, the last one at the bottom of the iteration): the old value is dead by
// then, the load can land in the same register, and the ring stays where it is from one pass of the loop to
// the next.  With the refill issued before its k-step's MFMAs the fragment had to be copied aside first, its
// registers moved by one set per refill, and the compiler put them back at the loop's back edge with a row of
// moves behind an s_waitcnt vmcnt(0): a full drain of the load queue every second iteration.
// A wave raises its priority for the MFMAs of a k-step and drops it for what lies between (refills, fragment reads
// of the next k-step): of the two waves that share a SIMD the one that is multiplying is not held up by the other's
// load issue (measured: 1.3 % of the projections' time at 144 rows, three alternating runs on one box; priority 3
// and the inverse assignment gain less or nothing).
#define MN_PRIO_HI __builtin_amdgcn_s_setprio(1);
#define MN_PRIO_LO __builtin_amdgcn_s_setprio(0);
#define MN_GEMM_REFILL(RING, KS_)                                                                           \
  _Pragma("unroll") for (int nt = 0; nt < NTW; ++nt) RING[nt][KS_] = MN_W_LOAD(it_ + RD, nt, KS_);
#define MN_GEMM_ITER(RING, CUR, NXT, IT)                                                                    \
  {                                                                                                         \
    const int it_ = (IT);                                                                                   \
    const int nxt_ = min(it_ + 1, last);                                                                    \
    /* pin this iteration's ring slot below the previous barrier: the compiler otherwise hoists its      */ \
    /* first use above it, where the tile loads are still pending and every wait becomes a full drain    */ \
    _Pragma("unroll") for (int nt = 0; nt < NTW; ++nt)                                                      \
      _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(RING[nt][ks]));              \
    MN_DMA_A(NXT, nxt_)                                                                                     \
    asm volatile("" ::: "memory");                                                                          \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                                     \
      if (ks > 0) MN_GEMM_REFILL(RING, ks - 1)                                                              \
      MN_PRIO_HI                                                                                            \
      _Pragma("unroll") for (int grp = 0; grp < 2; ++grp) {                                                 \
        constexpr int G0 = (MT + 1) / 2;                                                                    \
        const int lo_ = grp ? G0 : 0, cnt_ = grp ? MT - G0 : G0;                                            \
        f16x8 bfrag_[G0];                                                                                   \
        _Pragma("unroll") for (int i = 0; i < G0; ++i)                                                      \
          if (i < cnt_)                                                                                     \
            bfrag_[i] = *reinterpret_cast<const f16x8*>(&CUR[(lo_ + i) * 16 * LDS_ROW + lds_slot(l16, ks * 4 + g)]); \
        _Pragma("unroll") for (int nt = 0; nt < NTW; ++nt)                                                  \
          _Pragma("unroll") for (int i = 0; i < G0; ++i)                                                    \
            if (i < cnt_)                                                                                   \
              acc[nt][lo_ + i] = __builtin_amdgcn_mfma_f32_16x16x32_f16(                                    \
                  __builtin_bit_cast(f16x8, RING[nt][ks]) /* packed weights are fp16 already */, bfrag_[i], \
                  acc[nt][lo_ + i], 0, 0, 0);                                                               \
        /* scheduling fence after every k-step (after every row-tile group, or none, is the same within noise) */ \
        if (grp == 1) __builtin_amdgcn_sched_barrier(0);                                                    \
      }                                                                                                     \
      MN_PRIO_LO                                                                                            \
    }                                                                                                       \
    MN_GEMM_REFILL(RING, KS - 1)                                                                            \
    MN_WAIT_VM(NTW * KS);                                                                                   \
    __builtin_amdgcn_s_barrier();                                                                           \
  }

    // pairs of iterations with no branch inside the loop (a conditional second half would give the
    // compiler a short path that shrinks every wait), then the odd one out
    int it = 0;
    for (; it + 1 < n_iter; it += 2) {
      MN_GEMM_ITER(ring0, s_a0, s_a1, it)
      if constexpr (RD == 2) MN_GEMM_ITER(ring1, s_a1, s_a0, it + 1)
      else MN_GEMM_ITER(ring0, s_a1, s_a0, it + 1)
    }
    if (it < n_iter) MN_GEMM_ITER(ring0, s_a0, s_a1, it)
#undef MN_GEMM_ITER
#undef MN_GEMM_REFILL
#undef MN_PRIO_HI
#undef MN_PRIO_LO
  }
#undef MN_DMA_A
#undef MN_W_PTR
#undef MN_W_LOAD
#undef MN_WAIT_VM

  // epilogue: lane holds D[n = base + 4g + i][m = mt*16 + l16]
  bool bad = false;  // an fp16 activation left the fp16 range (saturated; reported once below)
  if constexpr (EPI == EPI_SWIGLU) {
    static_assert(NTW % 2 == 0, "gate and up tiles alternate inside a wave");
    f16_t* act = reinterpret_cast<f16_t*>(out_);
    const int F = N >> 1;
#pragma unroll
    for (int pr = 0; pr < NTW / 2; ++pr) {
      const int f = nblk * 64 + (w4 * (NTW / 2) + pr) * 16 + g * 4;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + mt * 16 + l16;
        if (m >= M || f >= F) continue;
        const f32x4 gt = acc[2 * pr][mt], up = acc[2 * pr + 1][mt];
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = gt[i] / (1.f + __expf(-gt[i])) * up[i];
        *reinterpret_cast<uint2*>(act + (size_t)m * F + f) = make_uint2(pack2h_sat(r[0], r[1], bad), pack2h_sat(r[2], r[3], bad));
      }
    }
  } else if constexpr (EPI == EPI_RELU) {
    f16_t* act = reinterpret_cast<f16_t*>(out_);
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
      const int n = n_wg + (w4 * NTW + nt) * 16 + g * 4;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int m = m0 + mt * 16 + l16;
        if (m >= M || n >= N) continue;
        f32x4 v = acc[nt][mt];
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = fmaxf(v[i] + ((bias && n + i < N) ? bias[n + i] : 0.f), 0.f);
        f16_t* p = act + (size_t)m * N + n;
        if (n + 3 < N && (N & 3) == 0) {
          *reinterpret_cast<uint2*>(p) = make_uint2(pack2h_sat(r[0], r[1], bad), pack2h_sat(r[2], r[3], bad));
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < N) p[i] = (f16_t)sat_h(r[i], bad);
        }
      }
    }
  } else {
    float* o = reinterpret_cast<float*>(out_) + (size_t)split * M * N;
    // (row tile outside, column tile inside: the wave's two column tiles are the two 64-byte halves of the same
    // 128-byte lines, and stored back to back they leave the L2 as whole lines; with the column tile outside the
    // halves were stored far apart and the down projection's 38 MB of partial sums cost 51 MB of HBM writes)
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
      for (int nt = 0; nt < NTW; ++nt) {
        const int n = n_wg + (w4 * NTW + nt) * 16 + g * 4;
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
  if (EPI != EPI_PARTIAL && bad && status) atomicOr(status, MN_DEV_RANGE);
}

// ------------------------------------------------------------------------------------------
// Many rows (M > 144): the MFMA-bound regime.  Both operands go through LDS.
// ------------------------------------------------------------------------------------------
// Workgroup = 8 waves (one per CU, two per SIMD) on a tile of 32*AT rows x 256 columns: wave (wm, wn)
// owns AT x 4 tiles of 16 x 16 (16*AT rows x 64 columns: 4*AT accumulator registers per tile row), so one
// k-step of 32 costs it AT + 4 fragment reads (1 KB each) for 4*AT MFMAs: with the weights streamed to
// registers instead, a wave cannot hold more than one iteration of lead once the accumulators take
// 100+ registers, and the counters showed it waiting for memory two thirds of its life.
// Everything arrives by direct global->LDS loads (no staging registers), one barrier per k-step:
//  * weights: a k-step is 16 column tiles x 1 KB, contiguous in the packed layout, landing as they are
//    in a ring of four stages, two to three k-steps ahead;
//  * activations: blocks of 64 k (32*AT rows x 128 bytes: whole cache lines; 64-byte row pieces cost the
//    L2 twice the requests), double-buffered, one to two k-steps ahead.  A load instruction brings
//    8 rows; the eight 16-byte pieces of row r are exchanged by XOR with (r/2) mod 8, which makes the
//    operand reads (16 rows x one piece per quarter wave) as fast as contiguous ones (measured).
// Loads complete in order, so "at most n outstanding" names exactly which have landed: the waits below
// count the loads issued after the ones needed next.
// Grid: as for the streaming kernel with several row chunks: the row blocks of one (column group, split)
// pair sit on consecutive slots of the same XCD and share the weights through its L2.
constexpr int BIG_NST = 4;                 // weight stages in LDS
constexpr int BIG_W_BYTES = 16 * 1024;     // 16 column tiles x 1 KB per k-step

template <int AT, int EPI>
__global__ void __launch_bounds__(512, 1) gemm_big_kernel(const f16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                          void* __restrict__ out_, const float* __restrict__ bias, int M,
                                                          int N, int K, int k_per_split, int m_chunks, int gx,
                                                          int n_split, int32_t* __restrict__ status) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  constexpr int A_TILE = 32 * AT * 128;                  // one 64-k block of activations
  constexpr int W_BASE = 2 * A_TILE;
  constexpr int UA = (4 * AT + 7) / 8;                   // activation loads per wave and block (8 rows each; spare
                                                         // slots of an odd AT repeat the last chunk)
  constexpr int UW = 2;                                  // weight loads per wave and k-step
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int wm = wave >> 2, wn = wave & 3;
  // id -> (column group, split, row block): the row blocks of a pair on consecutive slots of one XCD, and all
  // pairs of a k-split on the same XCDs (see the streaming kernel), so that an XCD's L2 holds the weights of
  // a pair once for its row blocks and fetches only its splits' k range of the activations
  const int id = blockIdx.x, xcd = id & 7, slot = id >> 3;
  const int li = slot / m_chunks, bz = slot % m_chunks;
  int bx, split;
  if (n_split <= 8 && 8 % n_split == 0) {
    const int r = 8 / n_split;
    split = xcd / r;
    bx = li * r + xcd % r;
  } else if (n_split % 8 == 0) {
    const int q = n_split >> 3;
    split = (li % q) * 8 + xcd;
    bx = li / q;
  } else {
    const int pair = li * 8 + xcd;
    bx = pair % gx;
    split = pair / gx;
  }
  if (bx >= gx || split >= n_split) return;  // (whole workgroup: padding of the grid)
  const int nblk_all = (N + NWG - 1) / NWG;
  const int m0 = bz * (32 * AT);
  const int k_begin = split * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_stage = (k_end - k_begin) / KSTEP;         // a multiple of 4 (splits are cut at 128 k)
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem);

  // ---- loader role of this lane ----
  const char* a_src[UA];     // activation piece at block 0
  const char* w_src[UW];     // weight piece at k-step 0
#pragma unroll
  for (int j = 0; j < UA; ++j) {
    const int c = min(wave * UA + j, 4 * AT - 1);        // 8-row chunk of the tile
    const int row = m0 + 8 * c + (lane >> 3);
    const int piece = (lane & 7) ^ (4 * (c & 1) + (lane >> 4));  // key = ((row mod 16) / 2)
    a_src[j] = reinterpret_cast<const char*>(A + (size_t)min(row, M - 1) * K + k_begin + 8 * piece);
  }
#pragma unroll
  for (int j = 0; j < UW; ++j) {
    const int wt = wave * UW + j;                        // column tile of the 256-column group
    const int nblk = min(bx * 2 + (wt >> 3), nblk_all - 1);
    w_src[j] = reinterpret_cast<const char*>(W + ((size_t)nblk * (K / KB) + k_begin / KB) * (size_t)WBLOCK +
                                             (size_t)(wt & 7) * (KS * 512) + lane * 8);
  }
  const int last_stage = n_stage - 1, last_blk = (n_stage >> 1) - 1;
  // block JB of the split -> activation buffer JB % 2; k-step ST -> weight stage ST % 4 (past the end: repeats)
#define MN_BIG_DMA_A1(JB, J)                                                                                \
  {                                                                                                         \
    const size_t off_ = (size_t)min((JB), last_blk) * (2 * KSTEP * sizeof(f16_t));                \
    dma16<0>(a_src[J] + off_, __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)((JB) & 1) * A_TILE +         \
                                                             (uint32_t)min(wave * UA + (J), 4 * AT - 1) * 1024u)); \
  }
#define MN_BIG_DMA_W1(ST, J)                                                                                \
  {                                                                                                         \
    const int st_ = min((ST), last_stage);                                                        \
    const size_t off_ = ((size_t)(st_ >> 2) * WBLOCK + (size_t)(st_ & 3) * 512) * sizeof(bf16_t);           \
    dma16<0, true>(w_src[J] + off_, __builtin_amdgcn_readfirstlane(lds0 + W_BASE + (uint32_t)((ST) & (BIG_NST - 1)) * BIG_W_BYTES + \
                                                             (uint32_t)(wave * UW + (J)) * 1024u));         \
  }
#define MN_BIG_DMA_A(JB) { _Pragma("unroll") for (int j = 0; j < UA; ++j) MN_BIG_DMA_A1(JB, j) }
#define MN_BIG_DMA_W(ST) { _Pragma("unroll") for (int j = 0; j < UW; ++j) MN_BIG_DMA_W1(ST, j) }
  // The loads go out one at a time between the MFMA groups, spread over the two k-steps of a block:
  //   lower half of even k-step st:  pieces C0 .. C0+C1-1 of A(jb+1)
  //   upper half of even k-step st:  the last C2 pieces of A(jb+1), then W(st+3)
  //   lower half of odd k-step st+1: W(st+4)
  //   upper half of odd k-step st+1: pieces 0 .. C0-1 of A(jb+2)
  // (every target was last read before the barrier the issuing half comes after), so that the eight
  // waves do not queue at the CU's address unit at the same moment: worth 0-3 % against one burst at
  // the start of the k-step.
  constexpr int C0 = (UA + 2) / 3, C1 = (UA - C0 + 1) / 2, C2 = UA - C0 - C1;
  static_assert(C0 <= 4 && C1 <= 4 && C2 + UW <= 4, "one load per MFMA group");
#define MN_BIG_DMA_LOW(ODD, JB, ST, G)                                                                      \
  {                                                                                                         \
    if (ODD) {                                                                                              \
      if ((G) < UW) MN_BIG_DMA_W1((ST) + 4, (G) < UW ? (G) : 0)                                             \
    } else if ((G) < C1) MN_BIG_DMA_A1((JB) + 1, (G) < C1 ? C0 + (G) : 0)                                   \
  }
#define MN_BIG_DMA_HIGH(ODD, JB, ST, G)                                                                     \
  {                                                                                                         \
    if (ODD) {                                                                                              \
      if ((G) < C0) MN_BIG_DMA_A1((JB) + 2, (G) < C0 ? (G) : 0)                                             \
    } else if ((G) < C2) MN_BIG_DMA_A1((JB) + 1, (G) < C2 ? C0 + C1 + (G) : 0)                              \
    else if ((G) < C2 + UW) MN_BIG_DMA_W1((ST) + 3, ((G) >= C2 && (G) < C2 + UW) ? (G) - C2 : 0)            \
  }

  f32x4 acc[AT][4];
#pragma unroll
  for (int a = 0; a < AT; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = (f32x4){0.f, 0.f, 0.f, 0.f};

  if (n_stage > 0) {  // (uniform per workgroup)
    const uint32_t a_row = (uint32_t)(wm * AT) * 2048u + (uint32_t)l16 * 128u;
    const uint32_t key = (uint32_t)(l16 >> 1) & 7u;
    const uint32_t a_rd0 = a_row + ((uint32_t)g ^ key) * 16u;          // first k-step of a block
    const uint32_t a_rd1 = a_row + ((uint32_t)(4 + g) ^ key) * 16u;    // second
    const uint32_t w_rd = (uint32_t)W_BASE + (uint32_t)(wn * 4) * 1024u + (uint32_t)lane * 16u;
    // One k-step = two halves of 2*AT MFMAs: the lower AT/2 row tiles before the barrier, the upper ones
    // behind it.  Every operand is asked for half a k-step before its first use, into registers the
    // previous half has just given up: the upper activation fragments at the start of the k-step (while
    // the lower half multiplies), the next k-step's lower fragments right behind the barrier that
    // publishes them, and its weight fragment b as soon as the upper half is through with column tile b
    // (no copy of the weight fragments is needed to keep them alive across the barrier).
    //   ABUF/HALF: activation buffer and its half of this k-step; N*: of the next one, NWST its weight
    //   stage; WAIT: loads that may still be in flight when the next k-step's data must have landed
    constexpr int H_ = AT / 2;
    f16x8 wf[4], af[AT];
#define MN_BIG_READ_LOW(ABUF, HALF)                                                                         \
  {                                                                                                         \
    const unsigned char* sl_ = smem + (ABUF) * A_TILE + ((HALF) ? a_rd1 : a_rd0);                           \
    _Pragma("unroll") for (int a = 0; a < H_; ++a) af[a] = *reinterpret_cast<const f16x8*>(sl_ + a * 2048); \
  }
#define MN_BIG_READ_W(WST, B_) wf[B_] = *reinterpret_cast<const f16x8*>(smem + w_rd + (WST) * BIG_W_BYTES + (B_) * 1024);
#define MN_BIG_STEP(ABUF, HALF, NABUF, NHALF, NWST, WAIT, ODD, JB, ST)                                                 \
  {                                                                                                         \
    const unsigned char* sa_ = smem + (ABUF) * A_TILE + ((HALF) ? a_rd1 : a_rd0);                           \
    _Pragma("unroll") for (int a = H_; a < AT; ++a) af[a] = *reinterpret_cast<const f16x8*>(sa_ + a * 2048); \
    __builtin_amdgcn_sched_barrier(0);                                                                      \
    _Pragma("unroll") for (int b = 0; b < 4; ++b) {                                                         \
      _Pragma("unroll") for (int a = 0; a < H_; ++a)                                                        \
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[b], af[a], acc[a][b], 0, 0, 0);               \
      __builtin_amdgcn_sched_barrier(0);                                                                    \
      MN_BIG_DMA_LOW(ODD, JB, ST, b)                                                                        \
      __builtin_amdgcn_sched_barrier(0);                                                                    \
    }                                                                                                       \
    wait_vm<(WAIT)>();                                                                                      \
    __syncthreads();                                                                                        \
    MN_BIG_READ_LOW(NABUF, NHALF)                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                                      \
    _Pragma("unroll") for (int b = 0; b < 4; ++b) {                                                         \
      _Pragma("unroll") for (int a = H_; a < AT; ++a)                                                       \
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(wf[b], af[a], acc[a][b], 0, 0, 0);               \
      __builtin_amdgcn_sched_barrier(0);                                                                    \
      MN_BIG_READ_W(NWST, b)                                                                                \
      MN_BIG_DMA_HIGH(ODD, JB, ST, b)                                                                       \
      __builtin_amdgcn_sched_barrier(0);                                                                    \
    }                                                                                                       \
  }
    // issue order (per wave): A(0) W(0) W(1) W(2) A(1)[0..C0) | k-step 0: A(1)[C0..C0+C1) . A(1)[C0+C1..UA) W(3) |
    // k-step 1: W(4) . A(2)[0..C0) | ...
    MN_BIG_DMA_A(0)
    MN_BIG_DMA_W(0)
    MN_BIG_DMA_W(1)
    MN_BIG_DMA_W(2)
#pragma unroll
    for (int j = 0; j < C0; ++j) MN_BIG_DMA_A1(1, j)
    wait_vm<2 * UW + C0>();  // A(0), W(0) landed
    __syncthreads();
    MN_BIG_READ_LOW(0, 0)
#pragma unroll
    for (int b = 0; b < 4; ++b) MN_BIG_READ_W(0, b)
    for (int st = 0; st < n_stage; st += 2) {
      const int jb = st >> 1;
      // even k-step: W(st+1) must have landed; W(st+2) and the first C0+C1 pieces of A(jb+1) may be in flight
      MN_BIG_STEP(jb & 1, 0, jb & 1, 1, (st + 1) & 3, UW + C0 + C1, 0, jb, st)
      // odd k-step: W(st+2) and A(jb+1) must have landed; W(st+3), W(st+4) may be in flight
      MN_BIG_STEP(jb & 1, 1, (jb + 1) & 1, 0, (st + 2) & 3, 2 * UW, 1, jb, st)
    }
    wait_vm<0>();  // the repeats past the end must land before the LDS is given back
#undef MN_BIG_STEP
#undef MN_BIG_READ_W
#undef MN_BIG_READ_LOW
  }
#undef MN_BIG_DMA_LOW
#undef MN_BIG_DMA_HIGH
#undef MN_BIG_DMA_A
#undef MN_BIG_DMA_W
#undef MN_BIG_DMA_A1
#undef MN_BIG_DMA_W1

  // epilogue: lane holds D[n = 16*(wn*4 + b) + 4g + i][m = 16*(wm*AT + a) + l16] of the workgroup tile
  bool bad = false;  // an fp16 activation left the fp16 range (saturated; reported once below)
  const int n_wg = bx * 256;
  if constexpr (EPI == EPI_SWIGLU) {
    f16_t* act = reinterpret_cast<f16_t*>(out_);
    const int F = N >> 1;
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const int f = (bx * 8 + wn * 2 + pr) * 16 + g * 4;
#pragma unroll
      for (int a = 0; a < AT; ++a) {
        const int m = m0 + (wm * AT + a) * 16 + l16;
        if (m >= M || f >= F) continue;
        const f32x4 gt = acc[a][2 * pr], up = acc[a][2 * pr + 1];
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = gt[i] / (1.f + __expf(-gt[i])) * up[i];
        *reinterpret_cast<uint2*>(act + (size_t)m * F + f) = make_uint2(pack2h_sat(r[0], r[1], bad), pack2h_sat(r[2], r[3], bad));
      }
    }
  } else if constexpr (EPI == EPI_RELU) {
    f16_t* act = reinterpret_cast<f16_t*>(out_);
#pragma unroll
    for (int b = 0; b < 4; ++b) {
      const int n = n_wg + (wn * 4 + b) * 16 + g * 4;
#pragma unroll
      for (int a = 0; a < AT; ++a) {
        const int m = m0 + (wm * AT + a) * 16 + l16;
        if (m >= M || n >= N) continue;
        const f32x4 v = acc[a][b];
        float r[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) r[i] = fmaxf(v[i] + ((bias && n + i < N) ? bias[n + i] : 0.f), 0.f);
        f16_t* p = act + (size_t)m * N + n;
        if (n + 3 < N && (N & 3) == 0) {
          *reinterpret_cast<uint2*>(p) = make_uint2(pack2h_sat(r[0], r[1], bad), pack2h_sat(r[2], r[3], bad));
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n + i < N) p[i] = (f16_t)sat_h(r[i], bad);
        }
      }
    }
  } else {
    float* o = reinterpret_cast<float*>(out_) + (size_t)split * M * N;
    // (row tile outside, the wave's four column tiles inside: two whole 128-byte lines per row, back to back)
#pragma unroll
    for (int a = 0; a < AT; ++a) {
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int n = n_wg + (wn * 4 + b) * 16 + g * 4;
        const int m = m0 + (wm * AT + a) * 16 + l16;
        if (m >= M || n >= N) continue;
        f32x4 v = acc[a][b];
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
  if (EPI != EPI_PARTIAL && bad && status) atomicOr(status, MN_DEV_RANGE);
}

// Row-major [N][K] bf16 -> the packed layout described at the top.  One thread per 16-byte piece.
// With half > 0 (Llama gate||up, N = 2*half) packed column tile 2t holds gate rows [16t, 16t+16)
// and tile 2t+1 the up rows half + [16t, 16t+16).
__global__ void __launch_bounds__(256) pack_weight_kernel(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int N,
                                                          int K, int half, int32_t* __restrict__ status) {
  bool bad = false;
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
    // re-encode once, here, instead of in every pass over the matrix: the same conversion the kernels
    // apply to bf16 data in registers (exact for magnitudes in [2^-14, 65504], below that truncated to
    // the fp16 subnormal grid, an absolute error under 2^-24).  A weight beyond the fp16 range (or not a
    // number) is saturated and reported: bf16 patterns with magnitude bits above those of 65504 (0x477F)
    const uint32_t w4[4] = {v.x, v.y, v.z, v.w};
    uint32_t c4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      uint32_t lo = w4[i] & 0xFFFFu, hi = w4[i] >> 16;
      if ((lo & 0x7FFFu) > 0x477Fu) { bad = true; lo = (lo & 0x8000u) | 0x477Fu; }
      if ((hi & 0x7FFFu) > 0x477Fu) { bad = true; hi = (hi & 0x8000u) | 0x477Fu; }
      c4[i] = lo | (hi << 16);
    }
    const f16x8 h = bf16x8_to_f16x8(make_uint4(c4[0], c4[1], c4[2], c4[3]));
    *reinterpret_cast<f16x8*>(dst + idx * 8) = h;
  }
  if (bad && status) atomicOr(status, MN_DEV_RANGE);
}

size_t packed_weight_elems(int N, int K) { return (size_t)((N + NWG - 1) / NWG) * NWG * (size_t)K; }

void launch_pack_weight(const void* src, void* dst, int N, int K, int half, int32_t* status, hipStream_t st) {
  const size_t pieces = packed_weight_elems(N, K) / 8;
  size_t blocks = (pieces + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  pack_weight_kernel<<<(int)blocks, 256, 0, st>>>(reinterpret_cast<const bf16_t*>(src), reinterpret_cast<bf16_t*>(dst), N, K, half, status);
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
static GemmTune tune() { return GemmTune{MN_TUNE("MN_GEMM_SPLIT", 0), MN_TUNE("MN_GEMM_TARGET_WGS", 512)}; }

// rows from which the big-tile kernel takes over (0: above 144)
static int big_min_m() { return MN_TUNE("MN_GEMM_BIG_MIN_M", 0); }

// Shape of the grid for one projection: waves per workgroup (each wave owns 32 columns; all waves of a
// workgroup share the activation tile, so more waves mean less L2 -> LDS traffic per weight byte) and
// k-splits.  Goal: every CU streams (a CU's share of the HBM rate is bounded by what its waves keep in
// flight), the whole grid is resident at once, and every split runs at least 16 iterations (measured:
// shorter splits lose more to ramp-up and partial sums than the extra workgroups win).
struct GemmPlan {
  int nw, split;
};
static GemmPlan gemm_plan(int M, int N, int K, int forced_split) {
  const int forced_nw = MN_TUNE("MN_GEMM_NW", 0);
  const int slices = ((N + NWG - 1) / NWG) * 4;  // 32-column wave slices of the padded matrix
  const int iters = K / KB;
  if (forced_split < 1 && tune().split >= 1) forced_split = tune().split;
  auto splits_for = [&](int gx, int slots, int min_iters = 16) {
    int s = forced_split >= 1 ? forced_split : slots / gx;
    if (forced_split < 1 && s > iters / min_iters) s = iters / min_iters;
    if (s > MN_MAX_SPLIT_K) s = MN_MAX_SPLIT_K;
    if (s < 1) s = 1;
    const int per = (iters + s - 1) / s;  // drop splits that would get no iteration
    return (iters + per - 1) / per;
  };
  GemmPlan best{4, 1};
  // (tuning builds: the plan of the projection with N output columns by hand)
  if (MN_TUNE("MN_GEMM_PLAN_N", 0) == N && MN_TUNE("MN_GEMM_PLAN_K", 0) == K && M > 96 && M <= 144)
    return GemmPlan{MN_TUNE("MN_GEMM_PLAN_NW", 4), MN_TUNE("MN_GEMM_PLAN_SPLIT", 1)};
  if (M > 144 || (big_min_m() > 0 && M >= big_min_m())) {  // big-tile kernel: 256-column groups x row blocks, one workgroup per CU
    const int gx = (slices / 4 + 1) / 2;
    int rb = 1 << 30;
    for (int at : {10, 8, 6}) rb = min(rb, (M + 32 * at - 1) / (32 * at) * at);  // (rows padded least; see big_at)
    int blocks = 1;
    for (int at : {10, 8, 6})
      if ((M + 32 * at - 1) / (32 * at) * at == rb) { blocks = (M + 32 * at - 1) / (32 * at); break; }
    if (M <= 160) blocks = 1;
    best.nw = 8;
    best.split = splits_for(gx * blocks, tune().target / 2);
    return best;
  }
  if (M <= 96) {
    // up to six row tiles: 4-wave workgroups.  Few rows make an iteration cheap, so a split may be as short
    // as 8 iterations, and one workgroup per CU is enough (measured at 40 rows: the 5120 x 5120 matrix
    // gains 30 % from 5 splits over 2, the 20480-column one loses with any split)
    const int gx = (slices + 3) / 4;
    best.split = splits_for(gx, tune().target / 2, 8);
    // small matrices (the drafting models: a few hundred KB per projection) would leave most of the chip
    // idle at that rule, and their time is launch and memory latency rather than bandwidth: splits as short
    // as one iteration, up to about a hundred workgroups
    if (gx * best.split < 64) best.split = splits_for(gx, 96, 1);
    return best;
  }
  int best_cus = 0, best_waves = 0;
  for (int nw = 8; nw >= 4; --nw) {
    if (forced_nw && nw != forced_nw) continue;
    const int gx = (slices + nw - 1) / nw;
    const int slots = nw == 4 ? tune().target : tune().target / 2;  // 4 waves: two workgroups per CU
    const int sp = splits_for(gx, slots);
    const int wgs = gx * sp;
    const int cus = wgs < 256 ? wgs : 256;
    const int waves = (wgs < slots ? wgs : slots) * nw;
    // fewer waves per workgroup only when that puts clearly more CUs (or waves) to work (measured at 144
    // rows: 224 -> 256 CUs, 8 -> 7 waves, gains 2 % on the 57344-column matrix since the ring keeps its
    // registers (nothing before); 160 -> 256 gains 6 % on the 10240-column one)
    if (best_cus == 0 || cus * 100 >= best_cus * 112 || (cus >= best_cus && waves * 100 >= best_waves * 115)) {
      best = GemmPlan{nw, sp};
      best_cus = cus;
      best_waves = waves;
    }
  }
  // Short splits pay more for ramp-up, tail and partial sums than they win: where the plan above cuts k into
  // pieces of fewer than 24 iterations, one 4-wave workgroup per CU with fewer, longer splits is faster if it
  // still covers nine CUs in ten (measured at 144 rows on the 10240 x 8192 matrix: 4 waves x 80 column groups
  // x 3 splits = 240 workgroups take 49.8 us against 52.5 for 5 x 64 x 4, and write a quarter less partial sums)
  if (!forced_nw && forced_split < 1 && best.split > 1 && (iters + best.split - 1) / best.split < 24) {
    const int gx4 = (slices + 3) / 4;
    const int sp4 = 256 / gx4;
    if (sp4 >= 1 && sp4 < best.split && gx4 * sp4 * 10 >= 256 * 9) best = GemmPlan{4, sp4};
  }
  return best;
}

int gemm_pick_split(int M, int N, int K, int dtype) {
  if (dtype != MN_DT_BF16) return 1;
  return gemm_plan(M, N, K, 0).split;
}

template <int MT, int NW, int NTW = 2, int RD = 2>
static void launch_bf16_mt(const GemmArgs& a, int m_chunks, hipStream_t st) {
  const int iters = a.K / KB;
  const int per = (iters + a.split_k - 1) / a.split_k;  // iterations per split
  const int slices = ((a.N + NWG - 1) / NWG) * (8 / NTW);
  const int gx = (slices + NW - 1) / NW;
  // 1-D grids; the kernel maps the id to (column group, split, row chunk) itself
  dim3 grid(gx * a.split_k, 1, 1);
  if (m_chunks > 1) grid = dim3(((gx * a.split_k + 7) / 8) * 8 * m_chunks, 1, 1);
  else if (a.split_k <= 8 && 8 % a.split_k == 0) grid = dim3(8 * ((gx + 8 / a.split_k - 1) / (8 / a.split_k)), 1, 1);
  const f16_t* A = reinterpret_cast<const f16_t*>(a.a);
  const bf16_t* W = reinterpret_cast<const bf16_t*>(a.w);
  if (a.swiglu_act)
    gemm_w16_kernel<MT, NTW, EPI_SWIGLU, NW, RD><<<grid, NW * 64, 0, st>>>(A, W, a.swiglu_act, nullptr, a.M, a.N, a.K, per * KB, m_chunks, gx, a.split_k, a.dev_status);
  else if (a.relu_act)
    gemm_w16_kernel<MT, NTW, EPI_RELU, NW, RD><<<grid, NW * 64, 0, st>>>(A, W, a.relu_act, a.bias, a.M, a.N, a.K, per * KB, m_chunks, gx, a.split_k, a.dev_status);
  else
    gemm_w16_kernel<MT, NTW, EPI_PARTIAL, NW, RD><<<grid, NW * 64, 0, st>>>(A, W, a.out, a.bias, a.M, a.N, a.K, per * KB, m_chunks, gx, a.split_k, a.dev_status);
}

// rows per workgroup of the big-tile kernel: the AT (row tiles per wave, two waves deep) that pads M least
static int big_at(int M) {
  if (M <= 160) return 5;
  int best = 10, best_rows = 1 << 30;
  for (int at : {10, 8, 6}) {
    const int rb = (M + 32 * at - 1) / (32 * at);
    if (rb * 32 * at < best_rows) {
      best_rows = rb * 32 * at;
      best = at;
    }
  }
  return best;
}

template <int AT>
static hipError_t launch_big(const GemmArgs& a, hipStream_t st) {
  const int iters = a.K / KB;
  const int per = (iters + a.split_k - 1) / a.split_k;  // 128-k blocks per split
  const int gx = ((a.N + NWG - 1) / NWG + 1) / 2;       // 256-column groups
  const int rb = (a.M + 32 * AT - 1) / (32 * AT);
  int per_xcd = (gx * a.split_k + 7) / 8;               // (column group, split) pairs per XCD
  if (a.split_k <= 8 && 8 % a.split_k == 0) per_xcd = (gx + 8 / a.split_k - 1) / (8 / a.split_k);
  else if (a.split_k % 8 == 0) per_xcd = (a.split_k / 8) * gx;
  const dim3 grid(8 * per_xcd * rb, 1, 1);
  const size_t smem = (size_t)2 * 32 * AT * 128 + (size_t)BIG_NST * BIG_W_BYTES;
  const f16_t* A = reinterpret_cast<const f16_t*>(a.a);
  const bf16_t* W = reinterpret_cast<const bf16_t*>(a.w);
  // once per process and instantiation, whichever thread comes first; a refusal is returned by every call
  // and nothing is launched
  static std::once_flag attr_once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [] {
    const void* fns[3] = {reinterpret_cast<const void*>(gemm_big_kernel<AT, EPI_PARTIAL>),
                          reinterpret_cast<const void*>(gemm_big_kernel<AT, EPI_SWIGLU>),
                          reinterpret_cast<const void*>(gemm_big_kernel<AT, EPI_RELU>)};
    for (const void* f : fns) {
      const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e != hipSuccess) attr_err = e;
    }
  });
  if (attr_err != hipSuccess) return attr_err;
  if (a.swiglu_act)
    gemm_big_kernel<AT, EPI_SWIGLU><<<grid, 512, smem, st>>>(A, W, a.swiglu_act, nullptr, a.M, a.N, a.K, per * KB, rb, gx, a.split_k, a.dev_status);
  else if (a.relu_act)
    gemm_big_kernel<AT, EPI_RELU><<<grid, 512, smem, st>>>(A, W, a.relu_act, a.bias, a.M, a.N, a.K, per * KB, rb, gx, a.split_k, a.dev_status);
  else
    gemm_big_kernel<AT, EPI_PARTIAL><<<grid, 512, smem, st>>>(A, W, a.out, a.bias, a.M, a.N, a.K, per * KB, rb, gx, a.split_k, a.dev_status);
  return hipSuccess;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.dtype != MN_DT_BF16) {
    dim3 grid((a.N + 3) / 4, (a.M + 7) / 8);
    gemm_f32_kernel<<<grid, 256, 0, st>>>(reinterpret_cast<const float*>(a.a), reinterpret_cast<const float*>(a.w),
                                          a.out, a.bias, a.M, a.N, a.K);
    return hipSuccess;
  }
  const int tiles = (a.M + 15) / 16;
  // row tiles per workgroup: everything in one chunk up to 9 tiles (144 rows), else chunks of 8
  if (tiles <= 1) launch_bf16_mt<1, 4>(a, 1, st);
  else if (tiles <= 2) launch_bf16_mt<2, 4>(a, 1, st);
  else if (tiles <= 3) launch_bf16_mt<3, 4>(a, 1, st);
  else if (tiles <= 4) launch_bf16_mt<4, 4>(a, 1, st);
  else if (tiles <= 6) launch_bf16_mt<6, 4>(a, 1, st);
  else if (tiles <= 9 && !(big_min_m() > 0 && a.M >= big_min_m())) {
    switch (gemm_plan(a.M, a.N, a.K, a.split_k).nw) {
      case 8: launch_bf16_mt<9, 8>(a, 1, st); break;
      case 7: launch_bf16_mt<9, 7>(a, 1, st); break;
      case 6: launch_bf16_mt<9, 6>(a, 1, st); break;
      case 5: launch_bf16_mt<9, 5>(a, 1, st); break;
      default: launch_bf16_mt<9, 4>(a, 1, st); break;
    }
  }
  else {
    if (!MN_TUNE("MN_GEMM_BIG", 1)) {  // 0 = chunks of the streaming kernel
      launch_bf16_mt<8, 4>(a, (tiles + 7) / 8, st);
    } else {
      switch (big_at(a.M)) {
        case 5: return launch_big<5>(a, st);
        case 10: return launch_big<10>(a, st);
        case 8: return launch_big<8>(a, st);
        default: return launch_big<6>(a, st);
      }
    }
  }
  return hipSuccess;
}

}  // namespace mn
