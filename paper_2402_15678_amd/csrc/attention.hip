// Multi-token paged attention against an existing KV cache (paper section 4: paged attention
// extended to more than one input token per sequence once a cache exists).  Query row j of
// sequence b sees the cached keys [0, ctx_b) and the new keys 0..j of its own sequence.
//
// Two kernels:
//  * attn_mfma_kernel  bf16 pages / fp16 queries, head_dim 128, 16-token blocks.  The G*q_b query rows that share one
//    KV head (grouped-query attention stacks the group's heads on top of the speculated tokens)
//    are the column index of every MFMA, so each K/V byte is read once per KV head.  K and V
//    fragments go HBM -> registers (bf16 widened exactly to fp16) -> MFMA directly: the page layouts put 8 consecutive
//    contraction elements in 16 bytes for both products (head-dim chunks for K, tokens for V).
//    The KV range of a sequence is split across workgroups; partial (max, sum, output) triples
//    are merged by attn_merge_kernel.
//  * attn_generic_kernel  any storage type / head_dim / block size; plain FMA, one (row, head)
//    per workgroup.  Used by the fp32 model and as the fallback.
#include "launch.h"
#include "../../include/minions_verify.h"

#include <cstdlib>

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
  const int ctx = a.rows.seq_ctx[b], row0 = a.rows.seq_row0[b];
  const TA* Kn = reinterpret_cast<const TA*>(a.knew);
  const TA* Vn = reinterpret_cast<const TA*>(a.vnew);
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
      if (Kn && key >= ctx) {
        const TA* kk = Kn + ((size_t)(row0 + key - ctx) * a.Hkv + kh) * hd;
        for (int e = 0; e < hd; ++e) d = fmaf(s_q[e], Store<TA>::load(kk + e), d);
      } else {
        const T* kb = Kp + ((size_t)pb * a.Hkv + kh) * (size_t)hd * bs;
        for (int c = 0; c < hd / 8; ++c) {
          const T* kk = kb + ((size_t)c * bs + off) * 8;
#pragma unroll
          for (int i = 0; i < 8; ++i) d = fmaf(s_q[c * 8 + i], Store<T>::load(kk + i), d);
        }
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
        float v;
        if (Vn && key2 >= ctx) {
          v = Store<TA>::load(Vn + ((size_t)(row0 + key2 - ctx) * a.Hkv + kh) * hd + e_own);
        } else {
          const T* vb = Vp + ((size_t)s_pb[i] * a.Hkv + kh) * (size_t)hd * bs;
          v = Store<T>::load(vb + (size_t)e_own * bs + key2 % bs);
        }
        acc = fmaf(s_p[i], v, acc);
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
// MFMA kernel (bf16 pages, fp16 queries, head_dim 128, block 16)
// ------------------------------------------------------------------------------------------
// Workgroup (4 waves) = one (KV split, KV head, sequence).  The R = G*q_b query rows that share the
// KV head are cut into 16-row column tiles; wave w owns tiles w, w+4, (w+8).  Key tiles of 32 keys
// (two blocks) travel HBM -> registers (raw bf16, a ring of PF tiles in flight per workgroup) ->
// widened once to fp16 -> LDS in MFMA fragment order -> every wave's MFMAs, so each K/V byte is
// loaded and converted once per KV head.  Q sits in LDS for the whole kernel.
//
// Both products have the query row as the MFMA column index (S^T = K Q^T, O^T = V^T P^T): softmax
// statistics are per-lane scalars.  Inside a tile the K rows are permuted (S^T row 4g'+r of half t
// is key 8g' + 4t + r) so that the lane group g of the first product's output holds keys
// 8g..8g+7, exactly the operand order of the second product and 16 contiguous bytes of a V page.
constexpr int HD = 128;
constexpr int BS = 16;
constexpr int KT = 32;                         // keys per tile (two blocks)
constexpr int TILE_BYTES = 2 * KT * HD * 2;    // K + V of one tile in fp16: 16 KB
constexpr int PF = 2;                          // key tiles in flight in registers per workgroup
constexpr int MAX_CT = 3;                      // column tiles per wave at most (R <= 192)
constexpr float LOG2E = 1.4426950408889634f;

// Q in LDS: 256-byte rows with the sixteen 16-byte chunks of row r rotated by 2r (bank pattern of a
// 288-byte stride: conflict-free for 16 rows x one chunk per quarter wave).
__device__ __forceinline__ int q_slot(int row, int chunk) { return row * HD + (((chunk + 2 * row) & 15) << 3); }

struct TileAddr {  // what a thread needs to fetch its four 16-byte pieces of a key tile
  const bf16_t* k[2];
  const bf16_t* v[2];
};

// Partials: o_part [split][M][H][HD] fp32 (unnormalised), ml_part [split][M][H][2] = (max in log2 units, sum)
template <int CTW>
__global__ void __launch_bounds__(256, 2) attn_mfma_kernel(AttnArgs a, int n_splits, int nt16_max,
                                                           float* __restrict__ o_part, float* __restrict__ ml_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16_t* s_kv = reinterpret_cast<f16_t*>(smem);                       // [2][16 fragments][64 lanes][8]
  f16_t* s_q = reinterpret_cast<f16_t*>(smem + 2 * TILE_BYTES);       // [nt16_max*16][HD], rotated chunks
  int32_t* s_bt = reinterpret_cast<int32_t*>(smem + 2 * TILE_BYTES + (size_t)nt16_max * 16 * HD * sizeof(f16_t));
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int G = a.H / a.Hkv;
  const int row0 = a.rows.seq_row0[b];
  const int qb = a.rows.seq_row0[b + 1] - row0;
  if (qb <= 0) return;
  const int ok = a.rows.seq_ok[b];
  const int ctx = a.rows.seq_ctx[b];
  const int R = G * qb;                   // query rows sharing this KV head; row r = j*G + gi
  const int NT16 = (R + 15) >> 4;         // column tiles in use (<= 4*CTW, checked by the launcher)
  const int nkeys = ok ? ctx + qb : 0;
  const int n_tiles = (nkeys + KT - 1) / KT;
  const int t_begin = (int)(((long)n_tiles * split) / n_splits);
  const int t_end = (int)(((long)n_tiles * (split + 1)) / n_splits);

  // ---- Q -> LDS (zero rows past R) ----
  const float sscale = rsqrtf((float)HD) * LOG2E;
  const f16_t* Q = reinterpret_cast<const f16_t*>(a.q);
  for (int c = tid; c < NT16 * 16 * (HD / 8); c += 256) {
    const int r = c >> 4, ch = c & 15;
    // Q is scaled by log2(e)/sqrt(hd) once here (one more fp16 rounding of q, 2^-11), so the scores
    // come out of the first product in log2 units
    f16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (r < R) {
      const int j = r / G, gi = r % G;
      v = *reinterpret_cast<const f16x8*>(Q + ((size_t)(row0 + j) * a.H + kvh * G + gi) * HD + ch * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (f16_t)((float)v[e] * sscale);
    }
    *reinterpret_cast<f16x8*>(&s_q[q_slot(r, ch)]) = v;
  }

  f32x4 O[CTW][8];
  float run_m[CTW], run_l[CTW];
  int lim[CTW];
  bool mine[CTW];
#pragma unroll
  for (int ct = 0; ct < CTW; ++ct) {
    run_m[ct] = -INFINITY;
    run_l[ct] = 0.f;
    const int tile = wave + 4 * ct;
    mine[ct] = ok && tile < NT16;
    const int r = tile * 16 + l16;
    lim[ct] = ctx + min(r / G, qb - 1);  // last visible key of this lane's query row
#pragma unroll
    for (int u = 0; u < 8; ++u) O[ct][u] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }

  const bf16_t* Kp = reinterpret_cast<const bf16_t*>(a.kv.k);
  const bf16_t* Vp = reinterpret_cast<const bf16_t*>(a.kv.v);
  const f16_t* Kn = reinterpret_cast<const f16_t*>(a.knew);
  const f16_t* Vn = reinterpret_cast<const f16_t*>(a.vnew);
  const int32_t* bt = a.kv.block_tables + (size_t)b * a.kv.max_blocks_per_seq;
  const size_t head_off = (size_t)kvh * (HD * BS);
  const size_t blk_stride = (size_t)a.Hkv * (HD * BS);
  // Loader role of this thread: K pieces (t = 0, 1; head-dim step s = wave) and V pieces (u = wave, wave + 4).
  // K piece: S^T row l16 = 4g'+r of half t <-> key 8g' + 4t + r of the tile; head-dim chunk 4*wave + g.
  const int kkey0 = 8 * (l16 >> 2) + (l16 & 3);      // key inside the tile for t = 0 (t = 1: + 4)
  const int kchunk = 4 * wave + g;

  // block table of this split -> LDS (the dependent chain table -> address -> load would otherwise
  // cost an L2 round trip per tile); entries past the last mapped block repeat the last one
  const int n_my = max(0, t_end - t_begin);
  const int last_blk = ok ? (nkeys - 1) / BS : 0;
  for (int i = tid; i < 2 * n_my; i += 256) s_bt[i] = bt[min(2 * t_begin + i, last_blk)];
  __syncthreads();

  auto tile_addr = [&](int ti) {  // ti: tile index inside the split
    TileAddr ta;
    const int pb0 = s_bt[2 * ti], pb1 = s_bt[2 * ti + 1];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int kk = kkey0 + 4 * t;
      ta.k[t] = Kp + (size_t)(kk < BS ? pb0 : pb1) * blk_stride + head_off + ((size_t)kchunk * BS + (kk & (BS - 1))) * 8;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
      ta.v[i] = Vp + (size_t)(g < 2 ? pb0 : pb1) * blk_stride + head_off + (size_t)(16 * (wave + 4 * i) + l16) * BS + 8 * (g & 1);
    return ta;
  };
  // LDS fragment slots this thread fills: K fragment (t*4 + wave), V fragment 8 + wave + 4i
  auto frag_ptr = [&](int buf, int f, int ln) { return s_kv + (size_t)buf * (TILE_BYTES / 2) + ((size_t)f * 64 + ln) * 8; };

  // ---- one key tile on this wave's column tiles; `tail` tiles apply the causal mask ----
  auto compute = [&](int buf, int key0, bool tail) {
    f32x4 S0[CTW], S1[CTW];
#pragma unroll
    for (int ct = 0; ct < CTW; ++ct) S0[ct] = S1[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const f16x8 k0 = *reinterpret_cast<const f16x8*>(frag_ptr(buf, s, lane));
      const f16x8 k1 = *reinterpret_cast<const f16x8*>(frag_ptr(buf, 4 + s, lane));
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct) {
        if (!mine[ct]) continue;
        const f16x8 qf = *reinterpret_cast<const f16x8*>(&s_q[q_slot((wave + 4 * ct) * 16 + l16, 4 * s + g)]);
        S0[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k0, qf, S0[ct], 0, 0, 0);
        S1[ct] = __builtin_amdgcn_mfma_f32_16x16x32_f16(k1, qf, S1[ct], 0, 0, 0);
      }
    }
    f16x8 P[CTW];
#pragma unroll
    for (int ct = 0; ct < CTW; ++ct) {
      if (!mine[ct]) continue;
      // lane holds keys key0 + 8g + e, e = 0..7 (S0 -> e 0..3, S1 -> e 4..7) of query row l16;
      // the scores are already in log2 units (Q was scaled when it was staged)
      float sc[8];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        sc[e] = S0[ct][e];
        sc[4 + e] = S1[ct][e];
      }
      if (tail) {
#pragma unroll
        for (int e = 0; e < 8; ++e)
          if (key0 + 8 * g + e > lim[ct]) sc[e] = -INFINITY;
      }
      float tm = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
      // Lazy maximum: the reference only moves (a cross-lane exchange and a rescale of the accumulator)
      // when some row's scores exceed it by more than 2^6; until then probabilities up to 64 are fine
      // in fp16 and in the fp32 sums.
      if (__any(tm > run_m[ct] + 6.f)) {
        tm = fmaxf(tm, __shfl_xor(tm, 16, 64));
        tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
        const float new_m = fmaxf(run_m[ct], tm);
        const float m_safe = (new_m == -INFINITY) ? 0.f : new_m;
        const float alpha = __builtin_amdgcn_exp2f(run_m[ct] - m_safe);
        run_m[ct] = new_m;
        run_l[ct] *= alpha;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          O[ct][u][0] *= alpha; O[ct][u][1] *= alpha; O[ct][u][2] *= alpha; O[ct][u][3] *= alpha;
        }
      }
      const float m_ref = (run_m[ct] == -INFINITY) ? 0.f : run_m[ct];
      float ps = 0.f;
      float p[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[e] = __builtin_amdgcn_exp2f(sc[e] - m_ref);
        ps += p[e];
      }
      run_l[ct] += ps;  // per-lane partial sum; lane groups are added at the end
      union { f16x8 v; uint32_t u[4]; } pf;
#pragma unroll
      for (int e = 0; e < 4; ++e) pf.u[e] = pack2h(p[2 * e], p[2 * e + 1]);
      P[ct] = pf.v;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const f16x8 vf = *reinterpret_cast<const f16x8*>(frag_ptr(buf, 8 + u, lane));
#pragma unroll
      for (int ct = 0; ct < CTW; ++ct) {
        if (!mine[ct]) continue;
        O[ct][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf, P[ct], O[ct][u], 0, 0, 0);
      }
    }
  };

  // ---- loop over this split's key tiles; the raw pages of the next PF tiles are in flight in registers ----
  if (ok && n_my > 0) {
    const int ti_last = n_my - 1;
    u32x4 ring[PF][4];  // raw bf16 pieces of the next PF tiles
#define MN_ATT_LOAD(SLOT, TI)                                                                    \
  {                                                                                              \
    const TileAddr ta_ = tile_addr(min((TI), ti_last));                                          \
    ring[SLOT][0] = *reinterpret_cast<const u32x4*>(ta_.k[0]);                                   \
    ring[SLOT][1] = *reinterpret_cast<const u32x4*>(ta_.k[1]);                                   \
    ring[SLOT][2] = *reinterpret_cast<const u32x4*>(ta_.v[0]);                                   \
    ring[SLOT][3] = *reinterpret_cast<const u32x4*>(ta_.v[1]);                                   \
  }
    // widen the four pieces of ring slot SLOT and put them into LDS buffer BUF as tile TI of the split;
    // tiles that reach past ctx take this step's own keys from the fp16 side buffers and zero the slots
    // past the sequence end (stale slots may hold anything: 0 * garbage must stay 0)
    auto fill = [&](const u32x4 (&r)[4], int buf, int ti) {
      const int key0 = (t_begin + ti) * KT;
      f16x8 kf[2] = {bf16x8_to_f16x8(r[0]), bf16x8_to_f16x8(r[1])};
      f16x8 vf[2] = {bf16x8_to_f16x8(r[2]), bf16x8_to_f16x8(r[3])};
      if (key0 + KT > ctx) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const int key = key0 + kkey0 + 4 * t;
          if (Kn && key >= ctx && key < nkeys)
            kf[t] = *reinterpret_cast<const f16x8*>(Kn + ((size_t)(row0 + key - ctx) * a.Hkv + kvh) * HD + kchunk * 8);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int hd = 16 * (wave + 4 * i) + l16;
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int key = key0 + 8 * g + e;
            if (key >= nkeys) vf[i][e] = (f16_t)0.f;
            else if (Vn && key >= ctx) vf[i][e] = Vn[((size_t)(row0 + key - ctx) * a.Hkv + kvh) * HD + hd];
          }
        }
      }
      *reinterpret_cast<f16x8*>(frag_ptr(buf, wave, lane)) = kf[0];
      *reinterpret_cast<f16x8*>(frag_ptr(buf, 4 + wave, lane)) = kf[1];
      *reinterpret_cast<f16x8*>(frag_ptr(buf, 8 + wave, lane)) = vf[0];
      *reinterpret_cast<f16x8*>(frag_ptr(buf, 12 + wave, lane)) = vf[1];
    };
    // prologue: tile 0 -> LDS buffer 0, tiles 1 and 2 in flight
    MN_ATT_LOAD(0, 0)
    MN_ATT_LOAD(1, 1)
    fill(ring[0], 0, 0);
    MN_ATT_LOAD(0, 2)
    __syncthreads();
// iteration i: LDS[i&1] holds tile i; ring slot SLOT holds tile i+1 (in flight or landed), the other
// slot tile i+2.  Fill the other LDS buffer with tile i+1, refill the slot with tile i+3, compute tile i.
#define MN_ATT_ITER(SLOT, I)                                                                     \
  {                                                                                              \
    const int i_ = (I);                                                                          \
    fill(ring[SLOT], (i_ + 1) & 1, min(i_ + 1, ti_last));                                        \
    MN_ATT_LOAD(SLOT, i_ + 3)                                                                    \
    asm volatile("" ::: "memory");                                                               \
    compute(i_ & 1, (t_begin + i_) * KT, (t_begin + i_) * KT + KT > ctx);                        \
    __syncthreads();                                                                             \
  }
    int i = 0;
    for (; i + 1 < n_my; i += 2) {
      MN_ATT_ITER(1, i)
      MN_ATT_ITER(0, i + 1)
    }
    if (i < n_my) MN_ATT_ITER(1, i)
#undef MN_ATT_ITER
#undef MN_ATT_LOAD
  }

  // ---- output: lane holds O^T[hd = 16u + 4g + i][row = tile*16 + l16] ----
#pragma unroll
  for (int ct = 0; ct < CTW; ++ct) {
    const int tile = wave + 4 * ct;
    const int r = tile * 16 + l16;
    if (tile >= NT16 || r >= R) continue;
    float l = run_l[ct];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    const int j = r / G, gi = r % G;
    const int m = row0 + j, h = kvh * G + gi;
    if (n_splits == 1) {
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

// One wave per (row, head): merge the split partials, normalise, store fp16.
__global__ void __launch_bounds__(256) attn_merge_kernel(const float* __restrict__ o_part, const float* __restrict__ ml_part,
                                                         int n_splits, int M, int H, f16_t* __restrict__ out) {
  const int wid = (blockIdx.x * 256 + threadIdx.x) >> 6, lane = threadIdx.x & 63;
  if (wid >= M * H) return;
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
// launch
// ------------------------------------------------------------------------------------------
static int attn_target_wgs() {
  static int t = [] {
    const char* e = getenv("MN_ATTN_TARGET_WGS");
    return e ? atoi(e) : 512;  // two workgroups per CU
  }();
  return t;
}

static int pick_splits(int B, int Hkv, int max_ctx) {
  static int forced = [] {
    const char* e = getenv("MN_ATTN_SPLITS");
    return e ? atoi(e) : 0;
  }();
  const int tiles = (max_ctx + KT - 1) / KT;
  int s = forced > 0 ? forced : (attn_target_wgs() + B * Hkv - 1) / (B * Hkv);
  const int cap = (tiles + 7) / 8;  // at least eight key tiles per split
  if (s > cap) s = cap;
  if (s > 16) s = 16;
  if (s < 1) s = 1;
  return s;
}

bool attention_mfma_supported(int H, int Hkv, int hd, int block_size, int dtype) {
  static int off = [] {
    const char* e = getenv("MN_ATTN_GENERIC");
    return e ? atoi(e) : 0;
  }();
  return !off && dtype == MN_DT_BF16 && hd == HD && block_size == BS && Hkv > 0 && H % Hkv == 0;
}

static size_t mfma_smem_bytes(int nt16_max, int tiles_per_split) {
  return (size_t)2 * TILE_BYTES + (size_t)nt16_max * 16 * HD * sizeof(f16_t) + (size_t)(2 * tiles_per_split + 2) * sizeof(int32_t);
}

size_t attention_scratch_bytes(int M, int H, int hd, int max_ctx, int dtype) {
  if (dtype != MN_DT_BF16 || hd != HD) return 256;
  return (size_t)16 * M * H * (HD + 2) * sizeof(float) + 256;
}

void launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.B <= 0) return;
  const int G = a.Hkv > 0 ? a.H / a.Hkv : 1;
  // the MFMA kernel stacks at most 4 * MAX_CT column tiles of 16 query rows per KV head
  const int nt16_max = (G * a.max_q + 15) / 16;
  const bool mfma = attention_mfma_supported(a.H, a.Hkv, a.hd, a.kv.block_size, a.dtype) && nt16_max <= 4 * MAX_CT &&
                    a.scratch != nullptr &&
                    a.scratch_bytes >= attention_scratch_bytes(a.M, a.H, a.hd, a.max_ctx, a.dtype);
  if (mfma) {
    const int n_splits = pick_splits(a.B, a.Hkv, a.max_ctx);
    float* o_part = a.scratch;
    float* ml_part = a.scratch + (size_t)n_splits * a.M * a.H * HD;
    const int tiles_per_split = ((a.max_ctx + KT - 1) / KT + n_splits - 1) / n_splits + 1;
    const size_t smem = mfma_smem_bytes(nt16_max, tiles_per_split);
    static bool attr_set = false;
    if (!attr_set) {
      const int most = 160 * 1024;
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<1>), hipFuncAttributeMaxDynamicSharedMemorySize, most);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<2>), hipFuncAttributeMaxDynamicSharedMemorySize, most);
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<3>), hipFuncAttributeMaxDynamicSharedMemorySize, most);
      attr_set = true;
    }
    dim3 grid(n_splits, a.Hkv, a.B);
    if (nt16_max <= 4) attn_mfma_kernel<1><<<grid, 256, smem, st>>>(a, n_splits, nt16_max, o_part, ml_part);
    else if (nt16_max <= 8) attn_mfma_kernel<2><<<grid, 256, smem, st>>>(a, n_splits, nt16_max, o_part, ml_part);
    else attn_mfma_kernel<3><<<grid, 256, smem, st>>>(a, n_splits, nt16_max, o_part, ml_part);
    if (n_splits > 1) {
      const int waves = a.M * a.H;
      attn_merge_kernel<<<(waves + 3) / 4, 256, 0, st>>>(o_part, ml_part, n_splits, a.M, a.H, reinterpret_cast<f16_t*>(a.out));
    }
    return;
  }
  dim3 grid(a.H, a.M);
  if (a.dtype == MN_DT_BF16) attn_generic_kernel<f16_t, bf16_t><<<grid, GEN_THREADS, 0, st>>>(a);
  else attn_generic_kernel<float, float><<<grid, GEN_THREADS, 0, st>>>(a);
}

}  // namespace mn
