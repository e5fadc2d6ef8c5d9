// Multi-token paged attention against an existing KV cache (paper section 4: paged attention
// extended to more than one input token per sequence once a cache exists).  Query row j of
// sequence b sees the cached keys [0, ctx_b) and the new keys 0..j of its own sequence.
//
// The keys and values of the scored tokens themselves are in the pages already: the tentative append
// (rope_append_kernel) runs before attention, so the kernels here read nothing but pages.
//
// Three kernels:
//  * attn_mfma_kernel  fp16 pages / fp16 queries, head_dim 128, 16-token blocks.  The G*q_b query rows that share one
//    KV head (grouped-query attention stacks the group's heads on top of the speculated tokens)
//    are the column index of every MFMA, so each K/V byte is read once per KV head.  Key tiles go
//    HBM -> LDS by direct loads, already in the operand order of the MFMAs of all the
//    waves: the page layouts put 8 consecutive contraction elements in 16 bytes for both
//    products (head-dim chunks for K, tokens for V).  The KV range of a sequence is split across
//    workgroups; partial (max, sum, output) triples are merged by attn_merge_kernel.
//  * attn_fewrow_kernel  fp16 pages / fp16 queries, head_dim 64, at most 4 stacked query rows per KV head
//    (a small drafting model decoding token by token): wide loads, plain FMA.
//  * attn_generic_kernel  any storage type / head_dim / block size; plain FMA, one (row, head)
//    per workgroup.  Used by the fp32 model and as the fallback.
#include "launch.h"
#include "tune.h"
#include "../../include/minions_verify.h"

#include <mutex>

namespace mn {

// ------------------------------------------------------------------------------------------
// generic kernel
// ------------------------------------------------------------------------------------------
constexpr int GEN_THREADS = 256;

// TA: activation type of q and out; T: storage type of the KV pages
template <typename TA, typename T>
__global__ void __launch_bounds__(GEN_THREADS) attn_generic_kernel(AttnArgs a) {
  __shared__ float s_q[256];
  __shared__ float s_p[GEN_THREADS];
  __shared__ int s_pb[GEN_THREADS];
  __shared__ float s_red[GEN_THREADS / 64];
  __shared__ float s_acc[GEN_THREADS];
  const int h = blockIdx.x, m = blockIdx.y, tid = threadIdx.x;
  const int hd = a.hd, bs = a.kv.block_size;
  const int b = a.rows.row_seq[m];
  const int pos = a.rows.row_pos[m];
  TA* o = reinterpret_cast<TA*>(a.out) + ((size_t)m * a.H + h) * hd;
  if (pos < 0) {
    for (int e = tid; e < hd; e += GEN_THREADS) Store<TA>::store(o + e, 0.f);
    return;
  }
  const int nkeys = pos + 1;
  const int kh = h / (a.H / a.Hkv);
  const float scale = rsqrtf((float)hd);
  const TA* q = reinterpret_cast<const TA*>(a.q) + ((size_t)m * a.H + h) * hd;
  for (int e = tid; e < hd; e += GEN_THREADS) s_q[e] = Store<TA>::load(q + e) * scale;
  __syncthreads();
  const T* Kp = reinterpret_cast<const T*>(a.kv.k);
  const T* Vp = reinterpret_cast<const T*>(a.kv.v);
  const int32_t* bt = a.kv.block_tables + (size_t)b * a.kv.max_blocks_per_seq;
  const int ng = GEN_THREADS / hd;  // key groups in the PV phase
  const int e_own = tid % hd, kg = tid / hd;
  float run_m = -INFINITY, run_l = 0.f, acc = 0.f;
  for (int k0 = 0; k0 < nkeys; k0 += GEN_THREADS) {
    const int key = k0 + tid;
    float s = -INFINITY;
    int pb = 0;
    if (key < nkeys) {
      pb = bt[key / bs];
      const int off = key % bs;
      float d = 0.f;
      const T* kb = Kp + ((size_t)pb * a.Hkv + kh) * (size_t)hd * bs;
      for (int c = 0; c < hd / 8; ++c) {
        const T* kk = kb + ((size_t)c * bs + off) * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) d = fmaf(s_q[c * 8 + i], Store<T>::load(kk + i), d);
      }
      s = d;
    }
    // chunk maximum
    float cm = wave_max(s);
    __syncthreads();
    if ((tid & 63) == 0) s_red[tid >> 6] = cm;
    __syncthreads();
    cm = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    const float new_m = fmaxf(run_m, cm);  // finite: key k0 is always visible
    const float alpha = __expf(run_m - new_m);
    const float p = (key < nkeys) ? __expf(s - new_m) : 0.f;
    s_p[tid] = p;
    s_pb[tid] = pb;
    const float ps = block_sum<GEN_THREADS / 64>(p, s_red);  // also orders the s_p / s_pb writes
    run_l = run_l * alpha + ps;
    run_m = new_m;
    acc *= alpha;
    const int cnt = min(GEN_THREADS, nkeys - k0);
    if (kg < ng) {
      for (int i = kg; i < cnt; i += ng) {
        const int key2 = k0 + i;
        const T* vb = Vp + ((size_t)s_pb[i] * a.Hkv + kh) * (size_t)hd * bs;
        acc = fmaf(s_p[i], Store<T>::load(vb + (size_t)e_own * bs + key2 % bs), acc);
      }
    }
    __syncthreads();
  }
  s_acc[tid] = (kg < ng) ? acc : 0.f;
  __syncthreads();
  if (tid < hd) {
    float t = 0.f;
    for (int g2 = 0; g2 < ng; ++g2) t += s_acc[g2 * hd + tid];
    Store<TA>::store(o + tid, t / run_l);
  }
}

// ------------------------------------------------------------------------------------------
// MFMA kernel (fp16 pages, fp16 queries, head_dim 128, block 16)
// ------------------------------------------------------------------------------------------
// Workgroup (4 waves) = one (KV head, sequence, row group, KV split).  The R = G*q_b query rows that share the
// KV head are cut into 16-row column tiles; wave w owns tiles w, w+4, (w+8) and keeps their query
// fragments (pre-multiplied by log2(e)/sqrt(hd)) in registers.
//
// Both products have the query row as the MFMA column index (S^T = K Q^T, O^T = V^T P^T): softmax
// statistics are per-lane scalars.  Inside a tile the K rows are permuted (S^T row 4g'+r of half t
// is key 8g' + 4t + r) so that the lane group g of the first product's output holds keys
// 8g..8g+7, exactly the operand order of the second product and 16 contiguous bytes of a V page.
//
// Data path of a key tile (32 keys = two blocks, 16 KB): HBM -> LDS by direct loads (no staging
// registers) into one of NS slots, already in MFMA fragment order (a wave load drops lane i's 16 bytes
// at slot base + 16 i, so lane i asks for the piece that belongs there); after the issuing waves' wait and
// a barrier every wave's MFMAs read it as it came.  Three tiles are in flight or landed ahead of the one being
// multiplied, and the loads of tile i+3 are issued before the wait for tile i+1, so the memory queue never runs
// dry while the waves wait for one another.
//
// The kernel is bound by instruction issue and LDS latency, not by HBM, at 128 query rows per KV head,
// hence: tiles that lie wholly inside the cached context take a branch-free body (no mask);
// the accumulators of the first product start at minus the running reference, so the
// scores come out already shifted; the reference moves lazily; the row sums are one more MFMA with
// an all-ones operand (they add exactly the fp16 probabilities the second product uses, and need no
// cross-lane reduction); the K fragments of the next tile and the V fragments of this one are read
// into registers early, and the phases are ordered so that every batch of MFMAs has independent
// vector work beside it (the softmax of tile ct beside the products of its neighbour).
constexpr int HD = 128;
constexpr int BS = 16;
constexpr int KT = 32;                         // keys per tile (two blocks)
constexpr int TILE_HALFS = 2 * KT * HD;        // fp16 elements of K + V of one tile
constexpr int TILE_BYTES = TILE_HALFS * 2;     // 16 KB
constexpr int NS = 4;                          // tile slots in LDS (a ring of 8, seven tiles of lead, is slower: measured)
constexpr int MAX_CT = 2;                      // column tiles per wave; a workgroup covers 64 * MAX_CT stacked rows
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LAZY_MAX = 6.f;                // the reference moves when a score exceeds it by 2^6

__device__ __forceinline__ float max3(float x, float y, float z) { return __builtin_fmaxf(__builtin_fmaxf(x, y), z); }

// Online-softmax step of one column tile on one key tile.  S0/S1: scores of keys 8g+0..3 / 8g+4..7 of
// this lane's query row, already minus the reference (negm4 = -reference in all four elements, 0 while
// nothing was seen).  Returns the probabilities as the B operand of the second product.
template <bool MASK>
__device__ __forceinline__ f16x8 softmax_tile(const f32x4& S0, const f32x4& S1, float& run_m, f32x4& negm4, float& thr,
                                              f32x4 (&O)[8], f32x4& L, int keyg, int lim) {
  float sc[8] = {S0[0], S0[1], S0[2], S0[3], S1[0], S1[1], S1[2], S1[3]};
  if (MASK) {
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (keyg + e > lim) sc[e] = -INFINITY;
  }
  float tm = max3(max3(sc[0], sc[1], sc[2]), max3(sc[3], sc[4], sc[5]), __builtin_fmaxf(sc[6], sc[7]));
  // thr is -inf until the row has seen a key, LAZY_MAX afterwards: probabilities up to 2^6 are fine
  // in fp16 and in the fp32 accumulators, so the common tile needs no exchange and no rescale
  if (__any(tm > thr)) {
    tm = __builtin_fmaxf(tm, __shfl_xor(tm, 16, 64));
    tm = __builtin_fmaxf(tm, __shfl_xor(tm, 32, 64));
    const bool fresh = run_m == -INFINITY;
    float d = fresh ? tm : __builtin_fmaxf(tm, 0.f);  // how far the reference moves (shifted units)
    if (d == -INFINITY) d = 0.f;                      // still nothing visible
    const float alpha = fresh ? 1.f : __builtin_amdgcn_exp2f(-d);
    if (!(fresh && tm == -INFINITY)) run_m = d - negm4[0];
    const float nm = (run_m == -INFINITY) ? 0.f : -run_m;
    negm4 = (f32x4){nm, nm, nm, nm};
    thr = (run_m == -INFINITY) ? -INFINITY : LAZY_MAX;
#pragma unroll
    for (int e = 0; e < 8; ++e) sc[e] -= d;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      O[u][0] *= alpha; O[u][1] *= alpha; O[u][2] *= alpha; O[u][3] *= alpha;
    }
    L[0] *= alpha; L[1] *= alpha; L[2] *= alpha; L[3] *= alpha;
  }
  union { f16x8 v; uint32_t u[4]; } pf;
#pragma unroll
  for (int e = 0; e < 4; ++e)
    pf.u[e] = pack2h(__builtin_amdgcn_exp2f(sc[2 * e]), __builtin_amdgcn_exp2f(sc[2 * e + 1]));
  return pf.v;
}

template <int N> struct IntC { static constexpr int value = N; };

// KV splits of a sequence with n_tiles key tiles when a workgroup should take about tps of them
__device__ __forceinline__ int seq_splits(int n_tiles, int tps, int n_splits_max) {
  return max(1, min(n_splits_max, (n_tiles + tps - 1) / max(tps, 1)));
}

// Partials: o_part [split][M][H][HD] fp32 (unnormalised), ml_part [split][M][H][2] = (max in log2 units, sum)
// NW waves per workgroup.  Waves 0-3 are the loaders (the tile's 16 fragments are dealt to four waves); with 5 or
// 6 waves the others only multiply: a stack of 65-96 query rows (5 or 6 column tiles, e.g. 8 query heads per KV
// head x 9-12 scored positions) then gives every wave one column tile, where four waves would leave one of them
// two tiles' worth of products and softmax per key tile while the other three wait at the barrier.
template <int CTW, int NW>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) attn_mfma_kernel(AttnArgs a, float* __restrict__ o_part,
                                                                             float* __restrict__ ml_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16_t* s_kv = reinterpret_cast<f16_t*>(smem);                          // [NS][16 fragments][64 lanes][8]
  int32_t* s_bidx = reinterpret_cast<int32_t*>(smem + NS * TILE_BYTES);  // physical block of every block of the split
  // Work list: workgroup (item, KV head) takes record `item` of the list attn_plan_kernel wrote for this step:
  // {sequence, row group, split, splits of the sequence, first row, rows, enabled, context}.  The list holds
  // only workgroups that have work, longest first, and the KV head is the fast index: workgroup ids are dealt
  // round-robin over the 8 XCDs and, inside an XCD, over its CUs, strictly in id order, so work has to be
  // dense in the id space (with the split as the fast grid index a batch that used 2 of 16 possible splits
  // ran on 2 of the 8 XCDs; with an often empty second row group next to the sequence index the real
  // workgroups shared half of the CUs) and long items must not queue behind short ones.
  // Row group rg: column tiles [NW*CTW*rg, NW*CTW*(rg+1)) of the stack; sequences with more than 16*NW*CTW stacked
  // rows get a workgroup per group (each streams the keys again).
  const int item = blockIdx.x / a.Hkv, kvh = blockIdx.x % a.Hkv;
  const int4 rec0 = reinterpret_cast<const int4*>(a.items)[2 * item];
  const int4 rec1 = reinterpret_cast<const int4*>(a.items)[2 * item + 1];
  const int b = rec0.x, rg = rec0.y, split = rec0.z, my_splits = rec0.w;
  if (b < 0) return;                      // past the end of the list (whole workgroup)
  const int row0 = rec1.x, qb = rec1.y, ok = rec1.z, ctx = rec1.w;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int G = a.H / a.Hkv;
  const int R = G * qb;                   // query rows sharing this KV head; row r = j*G + gi
  const int NT16 = (R + 15) >> 4;         // column tiles in use
  const int tile0 = NW * CTW * rg;        // first column tile of this workgroup
  const bool loader = wave < 4;           // (wave-uniform)
  if (qb <= 0 || tile0 >= NT16 || split >= my_splits) return;  // (whole workgroup; the list holds no such record)
  const int nkeys = ok ? ctx + qb : 0;
  const int n_tiles = (nkeys + KT - 1) / KT;
  const int t_begin = (int)(((long)n_tiles * split) / my_splits);
  const int t_end = (int)(((long)n_tiles * (split + 1)) / my_splits);
  const int n_my = max(0, t_end - t_begin);
  const int nct = ok ? min(CTW, max(0, (NT16 - tile0 - wave + NW - 1) / NW)) : 0;  // real column tiles of this wave

  // block table of this split -> LDS (the dependent chain table -> address -> load would otherwise
  // cost an L2 round trip per tile); entries past the last mapped block repeat the last one
  const int32_t* bt = a.kv.block_tables + (size_t)b * a.kv.max_blocks_per_seq;
  const int last_blk = ok ? (nkeys - 1) / BS : 0;
  for (int i = tid; i < 2 * n_my; i += NW * 64) s_bidx[i] = bt[min(2 * t_begin + i, last_blk)];

  // ---- Q fragments -> registers, scaled by log2(e)/sqrt(hd) (one more fp16 rounding of q, 2^-11), so
  // the scores come out of the first product in log2 units.  Rows past R are zero. ----
  const float sscale = rsqrtf((float)HD) * LOG2E;
  const f16_t* Q = reinterpret_cast<const f16_t*>(a.q);
  f16x8 qf[CTW][4];
  f32x4 O[CTW][8], L[CTW], negm4[CTW];
  float run_m[CTW], thr[CTW];
  int lim[CTW];
#pragma unroll
  for (int ct = 0; ct < CTW; ++ct) {
    run_m[ct] = -INFINITY;
    thr[ct] = -INFINITY;
    negm4[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
    L[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const int r = (tile0 + wave + NW * ct) * 16 + l16;
    lim[ct] = ctx + min(r / G, qb - 1);  // last visible key of this lane's query row
#pragma unroll
    for (int u = 0; u < 8; ++u) O[ct][u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      f16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
      if (r < R) {
        v = *reinterpret_cast<const f16x8*>(Q + ((size_t)(row0 + r / G) * a.H + kvh * G + r % G) * HD + 32 * s + 8 * g);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (f16_t)((float)v[e] * sscale);
      }
      qf[ct][s] = v;
    }
  }

  // Loader role of this thread: the pieces of its own lane in K fragments (t = 0, 1; head-dim step s = wave)
  // and V fragments (u = wave, wave + 4).  K: S^T row l16 = 4g'+r of half t <-> key 8g' + 4t + r of the
  // tile, head-dim chunk 4*wave + g (t = 1: +64 bytes).  V: head-dim row 16u + l16, keys 8g..8g+7
  // (u + 4: +2048 bytes).
  const int kkey0 = 8 * (l16 >> 2) + (l16 & 3);  // key inside the tile for t = 0 (t = 1: + 4)
  const int kchunk = 4 * wave + g;
  const int ksel = l16 >> 3, vsel = g >> 1;      // which of the tile's two blocks the pieces live in
  const uint32_t blk_bytes = (uint32_t)a.Hkv * (HD * BS) * (uint32_t)sizeof(f16_t);
  const uint32_t blk_last = (uint32_t)max(a.kv.num_blocks - 1, 0);
  const size_t head_bytes = (size_t)kvh * (HD * BS) * sizeof(f16_t);
  const char* kbase = reinterpret_cast<const char*>(a.kv.k) + head_bytes + ((size_t)kchunk * BS + (kkey0 & (BS - 1))) * 8 * sizeof(f16_t);
  const char* vbase = reinterpret_cast<const char*>(a.kv.v) + head_bytes + ((size_t)(16 * wave + l16) * BS + 8 * (g & 1)) * sizeof(f16_t);
  // LDS byte address of fragment `wave` of slot 0 (wave-uniform)
  const uint32_t lds_w = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem + (uint32_t)wave * 1024u);
  __syncthreads();  // block indices are in LDS; every load issued so far has been consumed

  if (ok && n_my > 0) {
    const int ti_last = n_my - 1;
    // all loads of tile TI of the split -> slot SLOT (tiles past the end repeat the last one)
#define MN_ATT_DMA(TI, SLOT)                                                                      \
  if (loader) {                                                                                   \
    const int t_ = min((TI), ti_last);                                                            \
    /* (the clamp costs two instructions and keeps a damaged table from becoming a wild address) */ \
    const char* kp_ = kbase + (uint64_t)min((uint32_t)s_bidx[2 * t_ + ksel], blk_last) * blk_bytes; \
    const char* vp_ = vbase + (uint64_t)min((uint32_t)s_bidx[2 * t_ + vsel], blk_last) * blk_bytes; \
    const uint32_t l_ = __builtin_amdgcn_readfirstlane(lds_w + (uint32_t)(SLOT) * TILE_BYTES);    \
    dma16<0, true>(kp_, l_);                                                                  \
    dma16<4 * 8 * 2, true>(kp_, l_ + 4 * 1024);                                               \
    dma16<0, true>(vp_, l_ + 8 * 1024);                                                       \
    dma16<64 * BS * 2, true>(vp_, l_ + 12 * 1024);                                            \
  }
    f16x8 kf[8];  // K fragments of the tile about to be multiplied
    // prologue: tiles 0 .. NS-2 on their way; tile 0 landed and its K fragments in registers
#pragma unroll
    for (int t = 0; t < NS - 1; ++t) MN_ATT_DMA(t, t)
    wait_vm<4 * (NS - 2)>();
    __syncthreads();
#pragma unroll
    for (int f = 0; f < 8; ++f) kf[f] = *reinterpret_cast<const f16x8*>(s_kv + (f * 64 + lane) * 8);

    // Iteration i: slot i%NS holds tile i (its K fragments already in kf); tile i+1 landed or
    // landing in slot (i+1)%NS, tiles i+2 .. i+NS-2 in flight; slot (i+NS-1)%NS, which held tile i-1, is free
    // since the last barrier.  SLOW: the tile reaches past ctx: the scores are masked (causal order among
    // the scored tokens, keys past the sequence end), and the V slots past the sequence end, which may hold anything
    // (0 * garbage must stay 0), are read as zeros.
    const f16x8 ones = {1, 1, 1, 1, 1, 1, 1, 1};
    auto iter = [&](auto nct_c, auto slow_c, int i) {
      constexpr int NCT = decltype(nct_c)::value;
      constexpr bool SLOW = decltype(slow_c)::value != 0;
      constexpr int NC = NCT > 0 ? NCT : 1;
      const int cur = i & (NS - 1), nxt = (i + 1) & (NS - 1);
      MN_ATT_DMA(i + NS - 1, (i + NS - 1) & (NS - 1))
      f16x8 vf[8];
      if (NCT > 0) {
#pragma unroll
        for (int u = 0; u < 8; ++u) vf[u] = *reinterpret_cast<const f16x8*>(s_kv + cur * TILE_HALFS + ((8 + u) * 64 + lane) * 8);
      }
      if (SLOW && NCT > 0) {
        const int past = (t_begin + i) * KT + 8 * g + 8 - nkeys;  // how many of this lane's 8 keys lie past the end
        if (past > 0) {
#pragma unroll
          for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (e >= 8 - past) vf[u][e] = (f16_t)0.f;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // first product of column tile 0
      f32x4 S0[NC], S1[NC];
      f16x8 P[NC];
      const int keyg = (t_begin + i) * KT + 8 * g;
      if (NCT > 0) {
        S0[0] = negm4[0];
        S1[0] = negm4[0];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          S0[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[s], qf[0][s], S0[0], 0, 0, 0);
          S1[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[4 + s], qf[0][s], S1[0], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      // first product of column tile ct beside the softmax of tile ct-1
#pragma unroll
      for (int ct = 1; ct < NCT; ++ct) {
        S0[ct] = negm4[ct];
        S1[ct] = negm4[ct];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          S0[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[s], qf[ct][s], S0[ct], 0, 0, 0);
          S1[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[4 + s], qf[ct][s], S1[ct], 0, 0, 0);
        }
        P[ct - 1] = softmax_tile<SLOW>(S0[ct - 1], S1[ct - 1], run_m[ct - 1], negm4[ct - 1], thr[ct - 1], O[ct - 1], L[ct - 1], keyg, lim[ct - 1]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // every LDS read of tile i has been issued; tile i+1 has landed once every loader's own wait is over
      // (the NS-2 tiles behind it may stay in flight): hand over
      wait_vm<4 * (NS - 2)>();
      __syncthreads();
#pragma unroll
      for (int f = 0; f < 8; ++f) kf[f] = *reinterpret_cast<const f16x8*>(s_kv + nxt * TILE_HALFS + (f * 64 + lane) * 8);
      __builtin_amdgcn_sched_barrier(0);
      // second product of tiles 0..NCT-2 beside the softmax of the last tile, then the last second product
      if (NCT > 0) {
#pragma unroll
        for (int ct = 0; ct + 1 < NCT; ++ct) {
#pragma unroll
          for (int u = 0; u < 8; ++u) O[ct][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[u], P[ct], O[ct][u], 0, 0, 0);
          L[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, P[ct], L[ct], 0, 0, 0);
        }
        P[NCT - 1] = softmax_tile<SLOW>(S0[NCT - 1], S1[NCT - 1], run_m[NCT - 1], negm4[NCT - 1], thr[NCT - 1], O[NCT - 1], L[NCT - 1], keyg, lim[NCT - 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int u = 0; u < 8; ++u) O[NCT - 1][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[u], P[NCT - 1], O[NCT - 1][u], 0, 0, 0);
        L[NCT - 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ones, P[NCT - 1], L[NCT - 1], 0, 0, 0);
      }
    };
    // fast iterations: tiles that lie wholly below ctx
    const int n_fast = min(n_my, max(0, ctx / KT - t_begin));
    int i = 0;
    if (nct == CTW) {
      for (; i < n_fast; ++i) iter(IntC<CTW>{}, IntC<0>{}, i);
      for (; i < n_my; ++i) iter(IntC<CTW>{}, IntC<1>{}, i);
    } else if (nct == 0) {
      for (; i < n_my; ++i) iter(IntC<0>{}, IntC<1>{}, i);
    } else {
      if constexpr (CTW > 1) {
        if (nct == 1) {
          for (; i < n_fast; ++i) iter(IntC<1>{}, IntC<0>{}, i);
          for (; i < n_my; ++i) iter(IntC<1>{}, IntC<1>{}, i);
        }
      }
    }
    wait_vm<0>();  // the loads of the tiles past the end must land before the LDS is given back
#undef MN_ATT_DMA
  }

  // ---- output: lane holds O^T[hd = 16u + 4g + i][row = tile*16 + l16]; every lane has its row's sum ----
#pragma unroll
  for (int ct = 0; ct < CTW; ++ct) {
    const int tile = tile0 + wave + NW * ct;
    const int r = tile * 16 + l16;
    if (tile >= NT16 || r >= R) continue;
    const float l = L[ct][0];
    const int j = r / G, gi = r % G;
    const int m = row0 + j, h = kvh * G + gi;
    if (my_splits == 1) {
      const float inv = (ok && l > 0.f) ? 1.f / l : 0.f;
      f16_t* o = reinterpret_cast<f16_t*>(a.out) + ((size_t)m * a.H + h) * HD + 4 * g;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const f32x4 v = O[ct][u];
        *reinterpret_cast<uint2*>(o + 16 * u) = make_uint2(pack2h(v[0] * inv, v[1] * inv), pack2h(v[2] * inv, v[3] * inv));
      }
    } else {
      float* o = o_part + (((size_t)split * a.M + m) * a.H + h) * HD + 4 * g;
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const f32x4 v = O[ct][u];
        *reinterpret_cast<float4*>(o + 16 * u) = make_float4(v[0], v[1], v[2], v[3]);
      }
      if (g == 0) {
        float* ml = ml_part + (((size_t)split * a.M + m) * a.H + h) * 2;
        ml[0] = run_m[ct];
        ml[1] = l;
      }
    }
  }
}

// One wave per (row, head): merge the split partials, normalise, store fp16.  Rows of sequences that ran as
// one split were written in final form by the attention kernel and are left alone.
__global__ void __launch_bounds__(256) attn_merge_kernel(const float* __restrict__ o_part, const float* __restrict__ ml_part,
                                                         int n_splits_max, int M, int H,
                                                         const int32_t* __restrict__ row_splits, f16_t* __restrict__ out) {
  const int wid = (blockIdx.x * 256 + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (wid >= M * H) return;
  // (one read decides: most rows of a ragged batch have nothing to merge; the bound keeps a damaged entry from
  // reaching past the partials)
  const int n_splits = min(row_splits[wid / H], n_splits_max);
  if (n_splits <= 1) return;
  float gm = -INFINITY;
  for (int s = 0; s < n_splits; ++s) gm = fmaxf(gm, ml_part[((size_t)s * M * H + wid) * 2]);
  const float ms = (gm == -INFINITY) ? 0.f : gm;
  float l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float* ml = ml_part + ((size_t)s * M * H + wid) * 2;
    const float f = __builtin_amdgcn_exp2f(ml[0] - ms);
    l += ml[1] * f;
    const float2 v = *reinterpret_cast<const float2*>(o_part + ((size_t)s * M * H + wid) * HD + lane * 2);
    o0 += v.x * f;
    o1 += v.y * f;
  }
  const float inv = l > 0.f ? 1.f / l : 0.f;
  *reinterpret_cast<uint32_t*>(out + (size_t)wid * HD + lane * 2) = pack2h(o0 * inv, o1 * inv);
}

// ------------------------------------------------------------------------------------------
// few-row kernel (fp16 pages, fp16 queries, head_dim 64, 16-token blocks, at most 4 stacked rows per KV head)
// ------------------------------------------------------------------------------------------
// The shape of a small model decoding one token per sequence (the SSMs that draft for the vote): one or
// a few query rows against the whole context.  There is nothing for a matrix instruction to share, the
// job is to keep the K/V pages streaming with wide loads.  Workgroup = one (KV head, sequence), 8 or 16 waves;
// a wave takes the key range in steps of four blocks (64 keys):
//  * K: lane (token t = lane % 16, group g = lane / 16) loads head-dim chunks g and g + 4 of token t of
//    each of the four blocks (16 bytes each, a quarter wave reads 256 contiguous bytes), multiplies
//    them with its part of q and adds up over the four groups with two cross-lane steps; group g then
//    keeps the score of block g: one key per lane;
//  * softmax: running maximum per wave (log2 units), per-lane partial sums of the probabilities;
//  * V: lane = head dimension; the 64 probabilities go through LDS (read back as broadcasts) and meet
//    the 16 tokens x 4 blocks of that dimension (32 contiguous bytes per block).
// The waves' (max, sum, output) are merged through LDS.
constexpr int FR_HD = 64;

// the two fp16 values of a 32-bit word of a page
__device__ __forceinline__ float h_lo(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[0]; }
__device__ __forceinline__ float h_hi(uint32_t w) { return (float)__builtin_bit_cast(f16x2, w)[1]; }

template <int RR, int FR_NW>  // rows held, waves per workgroup
__global__ void __launch_bounds__(FR_NW * 64) attn_fewrow_kernel(AttnArgs a) {
  __shared__ __attribute__((aligned(16))) float s_p[FR_NW][RR][64];
  __shared__ float s_o[FR_NW][RR][64];
  __shared__ float s_m[FR_NW][RR], s_l[FR_NW][RR];
  const int kvh = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = lane & 15, g = lane >> 4;
  const int G = a.H / a.Hkv;
  // (the sequence's scalars in one round trip, as in the MFMA kernel)
  const int row0 = a.rows.seq_row0[b], row1 = a.rows.seq_row0[b + 1];
  const int seq_ok = a.rows.seq_ok[b];
  const int ctx = a.rows.seq_ctx[b];
  asm volatile("" ::"r"(seq_ok), "r"(ctx));
  const int qb = row1 - row0;
  if (qb <= 0) return;                       // (whole workgroup)
  const int R = min(G * qb, RR);             // stacked rows r = j*G + gi (the host launches RR >= G * max_q)
  f16_t* out = reinterpret_cast<f16_t*>(a.out);
  if (!seq_ok) {                             // disabled sequence: zeros (whole workgroup)
    if (wave < R) out[((size_t)(row0 + wave / G) * a.H + kvh * G + wave % G) * FR_HD + lane] = (f16_t)0.f;
    return;
  }
  const f16_t* Q = reinterpret_cast<const f16_t*>(a.q);
  const int n_pk = ctx + qb;                 // the cached keys and this step's own
  const float sscale = rsqrtf((float)FR_HD) * LOG2E;

  float qf[RR][16];   // q of row r, head-dim chunks g and g + 4 (the lane's share of a dot product)
  float m[RR], l[RR], acc[RR];
  int lim[RR];        // keys [0, lim) of the pages are visible to row r
#pragma unroll
  for (int r = 0; r < RR; ++r) {
    m[r] = -INFINITY;
    l[r] = 0.f;
    acc[r] = 0.f;
    lim[r] = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) qf[r][i] = 0.f;
    if (r < R) {
      const f16_t* qp = Q + ((size_t)(row0 + r / G) * a.H + kvh * G + r % G) * FR_HD;
      const f16x8 p0 = *reinterpret_cast<const f16x8*>(qp + 8 * g);
      const f16x8 p1 = *reinterpret_cast<const f16x8*>(qp + 8 * (g + 4));
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        qf[r][i] = (float)p0[i] * sscale;
        qf[r][8 + i] = (float)p1[i] * sscale;
      }
      lim[r] = min(n_pk, ctx + r / G + 1);
    }
  }

  const int32_t* bt = a.kv.block_tables + (size_t)b * a.kv.max_blocks_per_seq;
  const int last_blk = max(0, (n_pk - 1) / BS);
  const uint32_t blk_last = (uint32_t)max(a.kv.num_blocks - 1, 0);
  const size_t head_stride = (size_t)FR_HD * BS * sizeof(f16_t);  // one (block, KV head) of K or of V
  const char* Kb = reinterpret_cast<const char*>(a.kv.k) + (size_t)kvh * head_stride + (size_t)(g * BS + t) * 16;
  const char* Vb = reinterpret_cast<const char*>(a.kv.v) + (size_t)kvh * head_stride + (size_t)lane * (BS * sizeof(f16_t));
  const int n_steps = (n_pk + 63) >> 6;
  for (int s = wave; s < n_steps; s += FR_NW) {
    uint4 kp[4][2], vp[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t blk = min((uint32_t)bt[min(4 * s + i, last_blk)], blk_last);
      const size_t off = (size_t)blk * a.Hkv * head_stride;
      kp[i][0] = *reinterpret_cast<const uint4*>(Kb + off);
      kp[i][1] = *reinterpret_cast<const uint4*>(Kb + off + 4 * BS * 16);
      vp[i][0] = *reinterpret_cast<const uint4*>(Vb + off);
      vp[i][1] = *reinterpret_cast<const uint4*>(Vb + off + 16);
    }
    if ((s + 1) * 64 > n_pk) {               // (wave-uniform) V slots past the sequence end may hold anything, and
#pragma unroll                               // 0 * garbage must stay 0: read them as zeros
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          uint32_t w[4] = {vp[i][c].x, vp[i][c].y, vp[i][c].z, vp[i][c].w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int tok = (4 * s + i) * BS + 8 * c + 2 * j;
            w[j] &= (tok < n_pk ? 0x0000ffffu : 0u) | (tok + 1 < n_pk ? 0xffff0000u : 0u);
          }
          vp[i][c] = make_uint4(w[0], w[1], w[2], w[3]);
        }
    }
    const int key = (4 * s + g) * BS + t;    // the key whose score this lane keeps
#pragma unroll
    for (int r = 0; r < RR; ++r) {
      float sv = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float d = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const uint4 w = kp[i][c];
          const float* qq = &qf[r][8 * c];
          d = fmaf(qq[0], h_lo(w.x), d); d = fmaf(qq[1], h_hi(w.x), d);
          d = fmaf(qq[2], h_lo(w.y), d); d = fmaf(qq[3], h_hi(w.y), d);
          d = fmaf(qq[4], h_lo(w.z), d); d = fmaf(qq[5], h_hi(w.z), d);
          d = fmaf(qq[6], h_lo(w.w), d); d = fmaf(qq[7], h_hi(w.w), d);
        }
        d += __shfl_xor(d, 16);
        d += __shfl_xor(d, 32);
        if (g == i) sv = d;
      }
      if (key >= lim[r]) sv = -INFINITY;
      const float new_m = fmaxf(m[r], wave_max(sv));
      const float alpha = (m[r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m[r] - new_m);
      const float p = (sv == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(sv - new_m);
      m[r] = new_m;
      l[r] = l[r] * alpha + p;
      acc[r] *= alpha;
      s_p[wave][r][lane] = p;
    }
    // (the wave reads back what it has just written: LDS operations of one wave stay in order)
#pragma unroll
    for (int r = 0; r < RR; ++r) {
      float o = acc[r];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float4* pp = reinterpret_cast<const float4*>(&s_p[wave][r][16 * i]);
        const float4 p0 = pp[0], p1 = pp[1], p2 = pp[2], p3 = pp[3];
        const uint4 v0 = vp[i][0], v1 = vp[i][1];
        o = fmaf(p0.x, h_lo(v0.x), o); o = fmaf(p0.y, h_hi(v0.x), o);
        o = fmaf(p0.z, h_lo(v0.y), o); o = fmaf(p0.w, h_hi(v0.y), o);
        o = fmaf(p1.x, h_lo(v0.z), o); o = fmaf(p1.y, h_hi(v0.z), o);
        o = fmaf(p1.z, h_lo(v0.w), o); o = fmaf(p1.w, h_hi(v0.w), o);
        o = fmaf(p2.x, h_lo(v1.x), o); o = fmaf(p2.y, h_hi(v1.x), o);
        o = fmaf(p2.z, h_lo(v1.y), o); o = fmaf(p2.w, h_hi(v1.y), o);
        o = fmaf(p3.x, h_lo(v1.z), o); o = fmaf(p3.y, h_hi(v1.z), o);
        o = fmaf(p3.z, h_lo(v1.w), o); o = fmaf(p3.w, h_hi(v1.w), o);
      }
      acc[r] = o;
    }
  }

#pragma unroll
  for (int r = 0; r < RR; ++r) {
    const float lt = wave_sum(l[r]);
    s_o[wave][r][lane] = acc[r];
    if (lane == 0) {
      s_m[wave][r] = m[r];
      s_l[wave][r] = lt;
    }
  }
  __syncthreads();
  {
    const int r = wave;                      // wave r merges row r (R <= 4 <= FR_NW)
    if (r < R) {
      float gm = -INFINITY;
#pragma unroll
      for (int w = 0; w < FR_NW; ++w) gm = fmaxf(gm, s_m[w][r]);
      float lt = 0.f, o = 0.f;
#pragma unroll
      for (int w = 0; w < FR_NW; ++w) {
        const float f = (s_m[w][r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(s_m[w][r] - gm);
        lt += f * s_l[w][r];
        o += f * s_o[w][r][lane];
      }
      out[((size_t)(row0 + r / G) * a.H + kvh * G + r % G) * FR_HD + lane] = (f16_t)(lt > 0.f ? o / lt : 0.f);
    }
  }
}

static bool fewrow_supported(const AttnArgs& a, int G) {
  return a.dtype == MN_DT_BF16 && a.hd == FR_HD && a.kv.block_size == BS && a.Hkv > 0 && a.H % a.Hkv == 0 &&
         G * a.max_q <= 4;
}

// ------------------------------------------------------------------------------------------
// launch
// ------------------------------------------------------------------------------------------
// The list of workgroups of the MFMA kernel for this step (the same for every layer): one record of 8 int32 per
// (sequence, row group, KV split) that has work: {sequence, row group, split, splits of the sequence, first
// row, rows, enabled, context}.  Sequences are ordered by descending key tiles per workgroup (ties by index),
// so the longest workgroups start first and the short ones fill the end of the launch; the records of the
// grid past the last real one get sequence = -1.  One workgroup; ranking is a comparison of every pair of
// sequences (B <= 4096, once per step).
__global__ void __launch_bounds__(1024) attn_plan_kernel(RowInfo rows, int B, int G, int tiles16_per_wg, int n_splits_max,
                                                         int grid_items, int32_t* __restrict__ items, int M,
                                                         int32_t* __restrict__ row_splits) {
  __shared__ int s_key[MN_MAX_BATCH], s_cnt[MN_MAX_BATCH], s_spl[MN_MAX_BATCH];
  __shared__ int s_total;
  const int tid = threadIdx.x;
  const int tps = rows.attn_tps[0];
  for (int m = tid; m < M; m += blockDim.x) row_splits[m] = 0;   // rows of no sequence (a disabled batch) merge nothing
  for (int b = tid; b < B; b += blockDim.x) {
    const int q = rows.seq_row0[b + 1] - rows.seq_row0[b];
    const int n_tiles = rows.seq_ok[b] ? (rows.seq_ctx[b] + q + KT - 1) / KT : 0;
    const int nt16 = (G * q + 15) >> 4;
    const int n_rg = q > 0 ? (nt16 + tiles16_per_wg - 1) / tiles16_per_wg : 0;
    const int spl = seq_splits(n_tiles, tps, n_splits_max);
    s_spl[b] = spl;
    s_cnt[b] = n_rg * spl;                       // a disabled sequence keeps one workgroup per row group: it writes zeros
    s_key[b] = (n_tiles + spl - 1) / spl;
  }
  __syncthreads();
  for (int b = tid; b < B; b += blockDim.x) {
    const int key = s_key[b], cnt = s_cnt[b], spl = s_spl[b];
    int off = 0, total = 0;
    for (int b2 = 0; b2 < B; ++b2) {
      const int c = s_cnt[b2], k2 = s_key[b2];
      total += c;
      if (k2 > key || (k2 == key && b2 < b)) off += c;
    }
    if (b == 0) s_total = total;
    const int row0 = rows.seq_row0[b], q = rows.seq_row0[b + 1] - row0, ok = rows.seq_ok[b], ctx = rows.seq_ctx[b];
    for (int j = 0; j < q; ++j) row_splits[row0 + j] = spl;   // for the merge: which rows have partials at all
    for (int i = 0; i < cnt; ++i) {
      if (off + i >= grid_items) break;        // (cannot happen: the grid holds every real record)
      int4* rec = reinterpret_cast<int4*>(items) + 2 * (size_t)(off + i);
      rec[0] = make_int4(b, i / spl, i % spl, spl);
      rec[1] = make_int4(row0, q, ok, ctx);
    }
  }
  __syncthreads();
  for (int i = s_total + tid; i < grid_items; i += blockDim.x)
    reinterpret_cast<int4*>(items)[2 * (size_t)i] = make_int4(-1, 0, 0, 1);
}

// Fewest key tiles a workgroup should take: below that the lead-in of a workgroup, the fp32 partial it writes and the
// merge launch behind cost as much as the parallelism wins (measured at 33 tiles per sequence and 128 (sequence, KV
// head) pairs: one split 2.10 ms of attention per step, two splits + merge 2.13-2.17, three or four 2.8-2.9; 16 and
// 32 give the same times at the other benchmark shapes, where the batch size decides the splits).
int attention_min_tiles() {
  const int x = MN_TUNE("MN_ATTN_MIN_TILES", 32);
  return x > 0 ? x : 32;
}

// 1.25 workgroups with work per CU: measured flat between 1 and 1.3 per CU, slower beyond (every further split of
// a sequence writes and re-reads one more fp32 partial of its rows, and workgroups beyond the 512 that are
// resident at once start when the first ones end)
int attention_target_workgroups() {
  const int x = MN_TUNE("MN_ATTN_WGS", 320);
  return x > 0 ? x : 320;
}

// Largest number of KV splits any sequence of the batch may get (it sizes the partials and bounds the work list;
// every sequence then takes what its own length asks for, see seq_splits): one per attention_min_tiles() key
// tiles of the longest context, 16 at most.
static int pick_splits(int max_ctx) {
  const int forced = MN_TUNE("MN_ATTN_SPLITS", 0);
  const int tiles = (max_ctx + KT - 1) / KT;
  int s = forced > 0 ? forced : tiles / attention_min_tiles();
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return s;
}

bool attention_mfma_supported(int H, int Hkv, int hd, int block_size, int dtype) {
  const int off = MN_TUNE("MN_ATTN_GENERIC", 0);
  return !off && dtype == MN_DT_BF16 && hd == HD && block_size == BS && Hkv > 0 && H % Hkv == 0;
}

static size_t mfma_smem_bytes(int tiles_per_split) {
  return (size_t)NS * TILE_BYTES + (size_t)(2 * tiles_per_split + 2) * sizeof(int32_t);
}

size_t attention_scratch_bytes(int M, int H, int hd, int max_ctx, int dtype) {
  if (dtype != MN_DT_BF16 || hd != HD) return 256;
  return (size_t)16 * M * H * (HD + 2) * sizeof(float) + 256;
}

// Records the work list must hold: a sequence of q rows has at most G q / 64 + 1 row groups (a workgroup covers
// at least 64 stacked rows) of at most 16 splits each.
size_t attention_items_capacity(int B, int M, int H, int Hkv) {
  const size_t G = Hkv > 0 ? (size_t)(H / Hkv) : 1;
  return 16 * (G * (size_t)(M > 0 ? M : 0) / 64 + (size_t)(B > 0 ? B : 0)) + 16;
}

// Shape of the MFMA launch, from what the host knows (largest row count of a sequence, longest context).
struct MfmaShape {
  int ctw, nw, n_rg, n_splits, grid_items;
};
static MfmaShape mfma_shape(const AttnArgs& a) {
  const int G = a.Hkv > 0 ? a.H / a.Hkv : 1;
  // the kernel covers NW * CTW column tiles of 16 stacked query rows per workgroup (4 waves with one or two tiles
  // each, or 5-6 waves with one tile each when that gives every wave the same work); longer stacks are cut into
  // row groups
  const int nt16_max = (G * a.max_q + 15) / 16;
  MfmaShape s;
  s.ctw = nt16_max <= 4 ? 1 : MAX_CT;
  s.nw = 4;
  if ((nt16_max == 5 || nt16_max == 6) && MN_TUNE("MN_ATTN_NW", 0) != 4) { s.ctw = 1; s.nw = nt16_max; }
  s.n_rg = (nt16_max + s.nw * s.ctw - 1) / (s.nw * s.ctw);
  s.n_splits = pick_splits(a.max_ctx);
  const size_t bound = (size_t)a.B * s.n_rg * s.n_splits;
  s.grid_items = (int)(bound < a.items_capacity ? bound : a.items_capacity);
  return s;
}
static bool mfma_path(const AttnArgs& a) {
  // (the block-index staging of the longest context must fit the LDS beside the tile ring: about 390 000 tokens;
  // longer contexts take the generic kernel)
  return attention_mfma_supported(a.H, a.Hkv, a.hd, a.kv.block_size, a.dtype) && a.scratch != nullptr &&
         mfma_smem_bytes((a.max_ctx + KT - 1) / KT + 1) <= 160 * 1024 &&
         a.scratch_bytes >= attention_scratch_bytes(a.M, a.H, a.hd, a.max_ctx, a.dtype) && a.items != nullptr &&
         a.row_splits != nullptr &&
         a.items_capacity >= attention_items_capacity(a.B, a.M, a.H, a.Hkv);
}

void launch_attention_plan(const AttnArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.B <= 0 || !mfma_path(a)) return;
  const MfmaShape s = mfma_shape(a);
  attn_plan_kernel<<<1, 1024, 0, st>>>(a.rows, a.B, a.H / a.Hkv, s.nw * s.ctw, s.n_splits, s.grid_items, a.items, a.M,
                                       a.row_splits);
}

hipError_t launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.B <= 0) return hipSuccess;
  const int G = a.Hkv > 0 ? a.H / a.Hkv : 1;
  if (mfma_path(a)) {
    const MfmaShape sh = mfma_shape(a);
    const int n_splits = sh.n_splits;
    float* o_part = a.scratch;
    float* ml_part = a.scratch + (size_t)n_splits * a.M * a.H * HD;
    // The block-index staging holds every block of the longest context: how many splits a sequence gets is
    // decided on the device from the whole batch (a large batch leaves even its longest sequence in one piece), so
    // a workgroup may have to walk all of a sequence's key tiles.  (Sized for the most splits instead, the array
    // was too short whenever the device chose fewer, and only the allocation granularity of the LDS covered it.)
    const int tiles_per_split = (a.max_ctx + KT - 1) / KT + 1;
    const size_t smem = mfma_smem_bytes(tiles_per_split);
    // once per process, whichever thread comes first; a refusal is returned by every call and nothing is launched
    static std::once_flag attr_once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(attr_once, [] {
      const void* fns[4] = {reinterpret_cast<const void*>(attn_mfma_kernel<1, 4>), reinterpret_cast<const void*>(attn_mfma_kernel<2, 4>),
                            reinterpret_cast<const void*>(attn_mfma_kernel<1, 5>), reinterpret_cast<const void*>(attn_mfma_kernel<1, 6>)};
      for (const void* f : fns) {
        const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) attr_err = e;
      }
    });
    if (attr_err != hipSuccess) return attr_err;
    const unsigned grid = (unsigned)a.Hkv * (unsigned)sh.grid_items;
    if (sh.nw == 5) attn_mfma_kernel<1, 5><<<grid, 320, smem, st>>>(a, o_part, ml_part);
    else if (sh.nw == 6) attn_mfma_kernel<1, 6><<<grid, 384, smem, st>>>(a, o_part, ml_part);
    else if (sh.ctw == 1) attn_mfma_kernel<1, 4><<<grid, 256, smem, st>>>(a, o_part, ml_part);
    else attn_mfma_kernel<2, 4><<<grid, 256, smem, st>>>(a, o_part, ml_part);
    if (n_splits > 1) {
      const int waves = a.M * a.H;
      attn_merge_kernel<<<(waves + 3) / 4, 256, 0, st>>>(o_part, ml_part, n_splits, a.M, a.H, a.row_splits, reinterpret_cast<f16_t*>(a.out));
    }
    return hipSuccess;
  }
  if (!MN_TUNE("MN_ATTN_GENERIC", 0) && fewrow_supported(a, G)) {
    const dim3 fg(a.Hkv, a.B);
    const int rr = G * a.max_q;
    // a single row leaves registers for 16 waves (one step of 64 keys each at 1024 keys of context)
    if (rr <= 1) attn_fewrow_kernel<1, 16><<<fg, 1024, 0, st>>>(a);
    else if (rr <= 2) attn_fewrow_kernel<2, 8><<<fg, 512, 0, st>>>(a);
    else attn_fewrow_kernel<4, 8><<<fg, 512, 0, st>>>(a);
    return hipSuccess;
  }
  dim3 grid(a.H, a.M);
  if (a.dtype == MN_DT_BF16) attn_generic_kernel<f16_t, f16_t><<<grid, GEN_THREADS, 0, st>>>(a);
  else attn_generic_kernel<float, float><<<grid, GEN_THREADS, 0, st>>>(a);
  return hipSuccess;
}

}  // namespace mn
