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
// MFMA kernel (bf16, head_dim 128, block 16)
// ------------------------------------------------------------------------------------------
constexpr int HD = 128;
constexpr int BS = 16;
constexpr int KT = 32;                 // keys per tile (two blocks)
constexpr int CT = 4;                  // 16-row column tiles per wave (64 query rows)
constexpr int Q_ROW = HD + 8;          // padded LDS row of Q, fp16 elements
constexpr int MAX_RG = 4;              // row groups of 64 rows per workgroup
constexpr int MERGE_RG = 2;              // row groups that can need a wave merge (KW > 1 only when RG <= 2)
constexpr float LOG2E = 1.4426950408889634f;

// Partials: o_part [split][M][H][HD] fp32 (unnormalised), ml_part [split][M][H][2] = (max in log2 units, sum)
__global__ void __launch_bounds__(256) attn_mfma_kernel(AttnArgs a, int n_splits, float* __restrict__ o_part,
                                                        float* __restrict__ ml_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  f16_t* s_q = reinterpret_cast<f16_t*>(smem);  // [RG*64][Q_ROW]; later reused for the wave merge
  const int split = blockIdx.x, kvh = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, g = lane >> 4;
  const int G = a.H / a.Hkv;
  const int row0 = a.rows.seq_row0[b];
  const int qb = a.rows.seq_row0[b + 1] - row0;
  const int ok = a.rows.seq_ok[b];
  const int ctx = a.rows.seq_ctx[b];
  const int R = G * qb;  // query rows sharing this KV head; row r = j*G + gi
  if (qb <= 0) return;
  const int RG = (R + 63) >> 6;            // row groups in use (1..4)
  const int KW = (RG == 1) ? 4 : (RG == 2 ? 2 : 1);  // waves that interleave over key tiles
  const int rg = wave / KW, kw = wave % KW;
  const bool active = ok && rg < RG;
  const int nkeys = ok ? ctx + qb : 0;
  const int n_tiles = (nkeys + KT - 1) / KT;
  const int t_begin = (int)(((long)n_tiles * split) / n_splits);
  const int t_end = (int)(((long)n_tiles * (split + 1)) / n_splits);

  // ---- Q -> LDS (zero rows past R) ----
  const f16_t* Q = reinterpret_cast<const f16_t*>(a.q);
  for (int c = tid; c < RG * 64 * (HD / 8); c += 256) {
    const int r = c / (HD / 8), ch = c % (HD / 8);
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    if (r < R) {
      const int j = r / G, gi = r % G;
      v = *reinterpret_cast<const uint4*>(Q + ((size_t)(row0 + j) * a.H + kvh * G + gi) * HD + ch * 8);
    }
    *reinterpret_cast<uint4*>(&s_q[r * Q_ROW + ch * 8]) = v;
  }
  __syncthreads();

  const float sscale = rsqrtf((float)HD) * LOG2E;
  f32x4 O[CT][8];
  float run_m[CT], run_l[CT];
  int lim[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    run_m[ct] = -INFINITY;
    run_l[ct] = 0.f;
    const int r = rg * 64 + ct * 16 + l16;
    lim[ct] = ctx + min(r / G, qb - 1);  // last visible key of this lane's query row
#pragma unroll
    for (int u = 0; u < 8; ++u) O[ct][u] = (f32x4){0.f, 0.f, 0.f, 0.f};
  }
  const int n_ct = active ? min(CT, (R - rg * 64 + 15) >> 4) : 0;

  const bf16_t* Kp = reinterpret_cast<const bf16_t*>(a.kv.k);
  const bf16_t* Vp = reinterpret_cast<const bf16_t*>(a.kv.v);
  const f16_t* Kn = reinterpret_cast<const f16_t*>(a.knew);
  const f16_t* Vn = reinterpret_cast<const f16_t*>(a.vnew);
  const int32_t* bt = a.kv.block_tables + (size_t)b * a.kv.max_blocks_per_seq;
  // lane constants of the K operand: S^T row i = l16 = 4g'+r  <->  key 8g' + 4t + r of the tile
  const int kg_ = l16 >> 2, kr_ = l16 & 3;

  if (active) {
    for (int T = t_begin + kw; T < t_end; T += KW) {
      const int key0 = T * KT;
      const int pb0 = bt[2 * T];
      const int pb1 = (key0 + BS < nkeys) ? bt[2 * T + 1] : pb0;
      const bool tail = key0 + KT > ctx;  // the tile holds keys of this step (masking, side-buffer reads)
      // ---- K fragments: [t][s] ----
      f16x8 kf[2][4];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int kk = 8 * kg_ + 4 * t + kr_;  // key inside the tile
        const int pb = (kk < BS) ? pb0 : pb1;
        const int key = key0 + kk;
        if (tail && Kn && key >= ctx && key < nkeys) {
          // a key of this step: read the unrounded row from the side buffer
          const f16_t* base = Kn + ((size_t)(row0 + key - ctx) * a.Hkv + kvh) * HD + g * 8;
#pragma unroll
          for (int s = 0; s < 4; ++s) kf[t][s] = *reinterpret_cast<const f16x8*>(base + 32 * s);
        } else {
          const bf16_t* base = Kp + ((size_t)pb * a.Hkv + kvh) * (size_t)(HD * BS) + (kk & (BS - 1)) * 8;
#pragma unroll
          for (int s = 0; s < 4; ++s)
            kf[t][s] = bf16x8_to_f16x8(*reinterpret_cast<const uint4*>(base + (size_t)(4 * s + g) * (BS * 8)));
        }
      }
      // ---- V fragments: [u], keys 8g..8g+7 of the tile ----
      f16x8 vf[8];
      {
        const int pb = (g < 2) ? pb0 : pb1;
        const bf16_t* base = Vp + ((size_t)pb * a.Hkv + kvh) * (size_t)(HD * BS) + (8 * (g & 1));
#pragma unroll
        for (int u = 0; u < 8; ++u) vf[u] = bf16x8_to_f16x8(*reinterpret_cast<const uint4*>(base + (size_t)(16 * u + l16) * BS));
        if (key0 + KT > nkeys) {
          // stale slots past the sequence end may hold anything: zero them so 0 * garbage stays 0
#pragma unroll
          for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (key0 + 8 * g + e >= nkeys) vf[u][e] = (f16_t)0.f;
        }
        if (tail && Vn) {
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const int key = key0 + 8 * g + e;
            if (key >= ctx && key < nkeys) {
              const f16_t* src = Vn + ((size_t)(row0 + key - ctx) * a.Hkv + kvh) * HD + l16;
#pragma unroll
              for (int u = 0; u < 8; ++u) vf[u][e] = src[16 * u];
            }
          }
        }
      }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        if (ct >= n_ct) continue;
        // ---- S^T = K Q^T for 32 keys x 16 rows ----
        f32x4 S0 = (f32x4){0.f, 0.f, 0.f, 0.f}, S1 = S0;
        const f16_t* qrow = &s_q[(rg * 64 + ct * 16 + l16) * Q_ROW + g * 8];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const f16x8 qf = *reinterpret_cast<const f16x8*>(qrow + s * 32);
          S0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[0][s], qf, S0, 0, 0, 0);
          S1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(kf[1][s], qf, S1, 0, 0, 0);
        }
        // lane holds keys key0 + 8g + e, e = 0..7 (S0 -> e 0..3, S1 -> e 4..7) of row l16
        float sc[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          sc[e] = S0[e] * sscale;
          sc[4 + e] = S1[e] * sscale;
        }
        if (tail) {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (key0 + 8 * g + e > lim[ct]) sc[e] = -INFINITY;
        }
        float tm = fmaxf(fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3])), fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
        tm = fmaxf(tm, __shfl_xor(tm, 16, 64));
        tm = fmaxf(tm, __shfl_xor(tm, 32, 64));
        const float new_m = fmaxf(run_m[ct], tm);
        const float m_safe = (new_m == -INFINITY) ? 0.f : new_m;
        const float alpha = __builtin_amdgcn_exp2f(run_m[ct] - m_safe);
        run_m[ct] = new_m;
        float ps = 0.f;
        float p[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          p[e] = __builtin_amdgcn_exp2f(sc[e] - m_safe);
          ps += p[e];
        }
        run_l[ct] = run_l[ct] * alpha + ps;  // per-lane partial sum; lane groups are added at the end
        union { f16x8 v; uint32_t u[4]; } pf;
#pragma unroll
        for (int e = 0; e < 4; ++e) pf.u[e] = pack2h(p[2 * e], p[2 * e + 1]);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          f32x4 o = O[ct][u];
          o[0] *= alpha; o[1] *= alpha; o[2] *= alpha; o[3] *= alpha;
          O[ct][u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vf[u], pf.v, o, 0, 0, 0);
        }
      }
    }
  }
  // per-row sums over the four lane groups
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    float l = run_l[ct];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    run_l[ct] = l;
  }

  // ---- merge the KW waves of a row group through LDS (wave kw=0 accumulates) ----
  __syncthreads();  // everyone is done with s_q
  float* s_o = reinterpret_cast<float*>(smem);                 // [MERGE_RG][CT][8][4][64]
  float* s_ml = s_o + MERGE_RG * CT * 8 * 4 * 64;              // [MERGE_RG][CT][2][64]
  for (int step = 1; step < KW; ++step) {
    if (active && kw == step) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) s_o[(((rg * CT + ct) * 8 + u) * 4 + i) * 64 + lane] = O[ct][u][i];
        s_ml[((rg * CT + ct) * 2 + 0) * 64 + lane] = run_m[ct];
        s_ml[((rg * CT + ct) * 2 + 1) * 64 + lane] = run_l[ct];
      }
    }
    __syncthreads();
    if (active && kw == 0) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        const float om = s_ml[((rg * CT + ct) * 2 + 0) * 64 + lane];
        const float ol = s_ml[((rg * CT + ct) * 2 + 1) * 64 + lane];
        const float nm = fmaxf(run_m[ct], om);
        const float ms = (nm == -INFINITY) ? 0.f : nm;
        const float fa = __builtin_amdgcn_exp2f(run_m[ct] - ms), fb = __builtin_amdgcn_exp2f(om - ms);
        run_m[ct] = nm;
        run_l[ct] = run_l[ct] * fa + ol * fb;
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i)
            O[ct][u][i] = O[ct][u][i] * fa + s_o[(((rg * CT + ct) * 8 + u) * 4 + i) * 64 + lane] * fb;
      }
    }
    __syncthreads();
  }

  // ---- output: lane holds O^T[hd = 16u + 4g + i][row = rg*64 + ct*16 + l16] ----
  if (rg < RG && kw == 0) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const int r = rg * 64 + ct * 16 + l16;
      if (r >= R) continue;
      const int j = r / G, gi = r % G;
      const int m = row0 + j, h = kvh * G + gi;
      if (n_splits == 1) {
        const float inv = (ok && run_l[ct] > 0.f) ? 1.f / run_l[ct] : 0.f;
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
          ml[1] = run_l[ct];
        }
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
    return e ? atoi(e) : 256;  // one workgroup per CU: more splits cost more in partial sums than they gain
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
  const int cap = (tiles + 3) / 4;  // at least four key tiles per split
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

static size_t mfma_smem_bytes(int rg_max) {
  const size_t q = (size_t)rg_max * 64 * Q_ROW * sizeof(f16_t);
  // the merge area is needed by any sequence with at most MERGE_RG row groups, whatever the batch maximum is
  const size_t merge = (size_t)MERGE_RG * CT * (8 * 4 + 2) * 64 * sizeof(float);
  return q > merge ? q : merge;
}

size_t attention_scratch_bytes(int M, int H, int hd, int max_ctx, int dtype) {
  if (dtype != MN_DT_BF16 || hd != HD) return 256;
  return (size_t)16 * M * H * (HD + 2) * sizeof(float) + 256;
}

void launch_attention(const AttnArgs& a, hipStream_t st) {
  if (a.M <= 0 || a.B <= 0) return;
  const int G = a.Hkv > 0 ? a.H / a.Hkv : 1;
  // the MFMA kernel stacks at most MAX_RG*64 query rows per KV head
  const bool mfma = attention_mfma_supported(a.H, a.Hkv, a.hd, a.kv.block_size, a.dtype) &&
                    (long)G * a.max_q <= MAX_RG * 64 && a.scratch != nullptr &&
                    a.scratch_bytes >= attention_scratch_bytes(a.M, a.H, a.hd, a.max_ctx, a.dtype);
  if (mfma) {
    const int n_splits = pick_splits(a.B, a.Hkv, a.max_ctx);
    float* o_part = a.scratch;
    float* ml_part = a.scratch + (size_t)n_splits * a.M * a.H * HD;
    const int rg_max = (G * a.max_q + 63) / 64;
    const size_t smem = mfma_smem_bytes(rg_max);
    static bool attr_set = false;
    if (!attr_set) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)mfma_smem_bytes(MAX_RG));
      attr_set = true;
    }
    dim3 grid(n_splits, a.Hkv, a.B);
    attn_mfma_kernel<<<grid, 256, smem, st>>>(a, n_splits, o_part, ml_part);
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
