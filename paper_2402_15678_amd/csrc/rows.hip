// Row-wise kernels of the verification forward: row bookkeeping, embedding + LayerNorm/RMSNorm with
// the residual update folded in, rotary embedding + tentative KV append, FFN activation, vocabulary
// argmax.  The paper (section 4) only states that every scored token's cache entry is addressed
// by a logical block id and an offset; the decoder body is the standard pre-norm one.
#include "launch.h"
#include "../../include/minions_verify.h"

namespace mn {

// ------------------------------------------------------------------------------------------
// prepare: validate the batch on the device and lay out the packed rows
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024) prepare_kernel(PrepArgs a) {
  __shared__ int32_t s_row0[MN_MAX_BATCH + 1];
  __shared__ int32_t s_ok[MN_MAX_BATCH];
  __shared__ int32_t s_nb[MN_MAX_BATCH];  // blocks each sequence needs mapped (0: nothing to check)
  __shared__ int s_bad;
  __shared__ unsigned long long s_tiles;
  const int tid = threadIdx.x;
  if (tid == 0) { s_bad = 0; s_tiles = 0ull; }
  __syncthreads();
  // pass 1: per-sequence validation
  for (int b = tid; b < a.B; b += blockDim.x) {
    const int k = a.spec_len[b];
    const int ctx = a.ctx_lens[b];
    int ok = 1;
    int flags = 0;
    int nb = 0;
    if (k < 0 || k > a.k_max) { ok = 0; flags |= MN_DEV_SPEC_LEN; }
    s_row0[b + 1] = (k < 0 || k > a.k_max) ? 1 : k + 1;
    if (ok) {
      const long need = (long)ctx + k + 1;
      if (ctx < 0 || need > (long)a.max_blocks_per_seq * a.block_size) { ok = 0; flags |= MN_DEV_BLOCK_TABLE; }
      if (ok && need > a.max_pos) { ok = 0; flags |= MN_DEV_TOKEN; }
      // the host sized the attention launch (key tiles per split, block-index staging) for max_ctx keys
      if (ok && need > a.max_ctx) { ok = 0; flags |= MN_DEV_CTX; }
      if (ok) nb = (int)((need + a.block_size - 1) / a.block_size);
    }
    s_ok[b] = ok;
    s_nb[b] = ok ? nb : 0;
    if (flags) {
      if (a.dev_status) atomicOr(a.dev_status, flags);
      if (flags & MN_DEV_SPEC_LEN) atomicOr(&s_bad, 1);
    }
  }
  __syncthreads();
  // pass 1b: every mapped block of every sequence, all threads side by side (a long context has
  // hundreds of table entries; one thread walking them is a chain of dependent loads)
  for (long idx = tid; idx < (long)a.B * a.max_blocks_per_seq; idx += blockDim.x) {
    const int b = (int)(idx / a.max_blocks_per_seq), i = (int)(idx % a.max_blocks_per_seq);
    if (i >= s_nb[b]) continue;
    const int pb = a.block_tables[idx];
    if (pb < 0 || pb >= a.num_blocks) {
      atomicAnd(&s_ok[b], 0);
      if (a.dev_status) atomicOr(a.dev_status, MN_DEV_BLOCK_TABLE);
    }
  }
  // pass 1c: every input token of every sequence that passed the shape checks, likewise
  if (a.last_tok) {
    for (long idx = tid; idx < (long)a.B * (a.k_max + 1); idx += blockDim.x) {
      const int b = (int)(idx / (a.k_max + 1)), j = (int)(idx % (a.k_max + 1));
      if (s_nb[b] == 0 || j >= s_row0[b + 1]) continue;  // (s_row0[b+1] still holds q_b = k_b + 1 here)
      const int tok = (j == 0) ? a.last_tok[b] : a.voted[(size_t)b * a.k_max + j - 1];
      if (tok < 0 || tok >= a.vocab) {
        atomicAnd(&s_ok[b], 0);
        if (a.dev_status) atomicOr(a.dev_status, MN_DEV_TOKEN);
      }
    }
  }
  __syncthreads();
  if (tid == 0) {
    s_row0[0] = 0;
    for (int b = 0; b < a.B; ++b) s_row0[b + 1] += s_row0[b];
    if (s_row0[a.B] != a.M) {
      s_bad = 1;
      if (a.dev_status) atomicOr(a.dev_status, MN_DEV_SPEC_LEN);
    }
  }
  __syncthreads();
  const bool bad = s_bad != 0;
  // a device spec_len that disagrees with the launch geometry disables the whole batch
  if (bad) {
    if (tid == 0 && a.attn_tps) a.attn_tps[0] = 1 << 20;
    for (int b = tid; b <= a.B; b += blockDim.x) a.seq_row0[b] = 0;
    for (int b = tid; b < a.B; b += blockDim.x) { a.seq_ctx[b] = 0; a.seq_ok[b] = 0; }
    for (int m = tid; m < a.M; m += blockDim.x) { a.row_seq[m] = 0; a.row_j[m] = 0; a.row_pos[m] = -1; a.row_tok[m] = 0; a.row_slot[m] = -1; }
    return;
  }
  for (int b = tid; b <= a.B; b += blockDim.x) a.seq_row0[b] = s_row0[b];
  for (int b = tid; b < a.B; b += blockDim.x) {
    const int ok = s_ok[b];
    const int ctx = ok ? a.ctx_lens[b] : 0;
    a.seq_ctx[b] = ctx;
    a.seq_ok[b] = ok;
    const int r0 = s_row0[b], q = s_row0[b + 1] - s_row0[b];
    for (int j = 0; j < q; ++j) {
      a.row_seq[r0 + j] = b;
      a.row_j[r0 + j] = j;
      a.row_pos[r0 + j] = ok ? ctx + j : -1;
      // where the row's K/V are written, looked up once per step instead of once per layer and head
      a.row_slot[r0 + j] = ok ? a.block_tables[(size_t)b * a.max_blocks_per_seq + (ctx + j) / a.block_size] * a.block_size +
                                    (ctx + j) % a.block_size
                              : -1;
      a.row_tok[r0 + j] = (ok && a.last_tok) ? ((j == 0) ? a.last_tok[b] : a.voted[(size_t)b * a.k_max + j - 1]) : 0;
    }
    // key tiles of 32, once per group of 128 (query position x head) rows: the work of the sequence in units of
    // one workgroup's tile (integer sum: order-free)
    if (ok && q > 0)
      atomicAdd(&s_tiles, (unsigned long long)((ctx + q + 31) >> 5) * (unsigned long long)((q * max(a.q_per_kv, 1) + 127) >> 7));
  }
  __syncthreads();
  // Balance of the attention grid: a workgroup should take about (all key tiles x KV heads) / (the number of
  // workgroups aimed for) tiles, at least 32 (below that the lead-in of a workgroup and the partial sums cost more than
  // the parallelism wins).  Long sequences of a ragged batch are then cut into more splits than short ones.
  if (tid == 0 && a.attn_tps) {
    const unsigned long long w = (unsigned long long)max(a.attn_wgs, 1);
    const unsigned long long per = (s_tiles * (unsigned long long)max(a.kv_heads, 1) + w - 1) / w;
    a.attn_tps[0] = (int)min(max(per, (unsigned long long)max(a.attn_min_tiles, 1)), (unsigned long long)(1 << 20));
  }
}

// cos/sin of the rotary angles, evaluated in double once per step and shared by all layers.
__global__ void rope_table_kernel(const int32_t* __restrict__ row_pos, int half, float base, float* __restrict__ c,
                                  float* __restrict__ s) {
  const int m = blockIdx.x;
  const int p = row_pos[m] < 0 ? 0 : row_pos[m];
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double inv = pow((double)base, -2.0 * (double)i / (double)(2 * half));
    const double ang = (double)p * inv;
    c[(size_t)m * half + i] = (float)cos(ang);
    s[(size_t)m * half + i] = (float)sin(ang);
  }
}

void launch_prepare(const PrepArgs& a, hipStream_t st) {
  // one workgroup; 1024 threads walk the block tables side by side (32 sequences x 512 blocks took 45 us with 256)
  prepare_kernel<<<1, 1024, 0, st>>>(a);
  if (a.rope_half > 0 && a.M > 0) rope_table_kernel<<<a.M, 64, 0, st>>>(a.row_pos, a.rope_half, a.rope_base, a.rope_cos, a.rope_sin);
}

// ------------------------------------------------------------------------------------------
// norm: x += sum of partials + bias (or x = embedding), then LayerNorm / RMSNorm -> h
// ------------------------------------------------------------------------------------------
constexpr int NORM_THREADS = 1024;  // 16 waves per row: the row's partial sums are many independent streams
constexpr int NORM_MAX_VEC = 2;     // float4 per thread: d <= 1024*2*4 = 8192

template <typename T>
__device__ __forceinline__ float4 load4(const T* p);
template <>
__device__ __forceinline__ float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <>
__device__ __forceinline__ float4 load4<bf16_t>(const bf16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xFFFF0000u), __uint_as_float(u.y << 16),
                     __uint_as_float(u.y & 0xFFFF0000u));
}
template <>
__device__ __forceinline__ float4 load4<f16_t>(const f16_t* p) {
  const uint2 u = *reinterpret_cast<const uint2*>(p);
  const f16x2 a = __builtin_bit_cast(f16x2, u.x), b = __builtin_bit_cast(f16x2, u.y);
  return make_float4((float)a[0], (float)a[1], (float)b[0], (float)b[1]);
}
// (fp16 stores saturate and set `bad`, see sat_h)
template <typename T>
__device__ __forceinline__ void store4(T* p, float4 v, bool& bad);
template <>
__device__ __forceinline__ void store4<f16_t>(f16_t* p, float4 v, bool& bad) {
  *reinterpret_cast<uint2*>(p) = make_uint2(pack2h_sat(v.x, v.y, bad), pack2h_sat(v.z, v.w, bad));
}
template <>
__device__ __forceinline__ void store4<float>(float* p, float4 v, bool&) { *reinterpret_cast<float4*>(p) = v; }
// one element in the activation type TA / the page storage type T; fp16 saturates to the fp16 range
template <typename T>
__device__ __forceinline__ void store1(T* p, float v, bool& bad) { Store<T>::store(p, v); }
template <>
__device__ __forceinline__ void store1<f16_t>(f16_t* p, float v, bool& bad) { *p = (f16_t)sat_h(v, bad); }

// T: storage type of the embedding tables; TA: activation type of the normalised output
template <typename T, typename TA>
__global__ void __launch_bounds__(NORM_THREADS) norm_kernel(NormArgs a) {
  __shared__ float red[NORM_THREADS / 64];
  const int m = blockIdx.x;
  const int tid = threadIdx.x;
  const int d = a.d;
  const int nvec = d >> 2;
  float4 v[NORM_MAX_VEC];
  float* xr = a.x + (size_t)m * d;
  const bool embed = a.tok_emb != nullptr;
  const T* te = embed ? reinterpret_cast<const T*>(a.tok_emb) + (size_t)a.row_tok[m] * d : nullptr;
  const int pos = (embed && a.pos_emb) ? (a.row_pos[m] < 0 ? 0 : a.row_pos[m]) : 0;
  const T* pe = (embed && a.pos_emb) ? reinterpret_cast<const T*>(a.pos_emb) + (size_t)pos * d : nullptr;
  float sum = 0.f;
#pragma unroll
  for (int it = 0; it < NORM_MAX_VEC; ++it) {
    const int i4 = it * NORM_THREADS + tid;
    float4 r = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i4 < nvec) {
      const int e = i4 << 2;
      if (embed) {
        r = load4<T>(te + e);
        if (pe) {
          const float4 p = load4<T>(pe + e);
          r.x += p.x; r.y += p.y; r.z += p.z; r.w += p.w;
        }
      } else {
        r = *reinterpret_cast<const float4*>(xr + e);
        if (a.partials) {
          // fixed summation order: residual, then partial 0, 1, ..., then the bias.  The partials are
          // fetched eight at a time before any is added (indices past the end repeat the last one and are
          // not added): one memory round trip per batch instead of one per partial
          for (int s0 = 0; s0 < a.n_partials; s0 += 8) {
            float4 p[8];
#pragma unroll
            for (int j = 0; j < 8; ++j)
              p[j] = *reinterpret_cast<const float4*>(a.partials + ((size_t)min(s0 + j, a.n_partials - 1) * a.M + m) * d + e);
#pragma unroll
            for (int j = 0; j < 8; ++j)
              if (s0 + j < a.n_partials) { r.x += p[j].x; r.y += p[j].y; r.z += p[j].z; r.w += p[j].w; }
          }
        }
        if (a.bias) {
          const float4 p = *reinterpret_cast<const float4*>(a.bias + e);
          r.x += p.x; r.y += p.y; r.z += p.z; r.w += p.w;
        }
      }
      if (embed || a.partials || a.bias) *reinterpret_cast<float4*>(xr + e) = r;
      sum += (r.x + r.y) + (r.z + r.w);
    }
    v[it] = r;
  }
  const float inv_d = 1.f / (float)d;
  float mean = 0.f;
  if (a.shift) mean = block_sum<NORM_THREADS / 64>(sum, red) * inv_d;
  float sq = 0.f;
#pragma unroll
  for (int it = 0; it < NORM_MAX_VEC; ++it) {
    const int i4 = it * NORM_THREADS + tid;
    if (i4 < nvec) {
      const float4 r = v[it];
      const float a0 = r.x - mean, a1 = r.y - mean, a2 = r.z - mean, a3 = r.w - mean;
      sq += (a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3);
    }
  }
  const float var = block_sum<NORM_THREADS / 64>(sq, red) * inv_d;
  const float rstd = 1.f / sqrtf(var + a.eps);
  TA* hr = reinterpret_cast<TA*>(a.h) + (size_t)m * d;
  bool bad = false;
#pragma unroll
  for (int it = 0; it < NORM_MAX_VEC; ++it) {
    const int i4 = it * NORM_THREADS + tid;
    if (i4 < nvec) {
      const int e = i4 << 2;
      const float4 r = v[it];
      const float4 g = *reinterpret_cast<const float4*>(a.gain + e);
      float4 o = make_float4((r.x - mean) * rstd * g.x, (r.y - mean) * rstd * g.y, (r.z - mean) * rstd * g.z,
                             (r.w - mean) * rstd * g.w);
      if (a.shift) {
        const float4 sh = *reinterpret_cast<const float4*>(a.shift + e);
        o.x += sh.x; o.y += sh.y; o.z += sh.z; o.w += sh.w;
      }
      store4<TA>(hr + e, o, bad);
    }
  }
  if (bad && a.dev_status) atomicOr(a.dev_status, MN_DEV_RANGE);
}

void launch_norm(const NormArgs& a, hipStream_t st) {
  if (a.M <= 0) return;
  if (a.dtype == MN_DT_BF16) norm_kernel<bf16_t, f16_t><<<a.M, NORM_THREADS, 0, st>>>(a);
  else norm_kernel<float, float><<<a.M, NORM_THREADS, 0, st>>>(a);
}

// ------------------------------------------------------------------------------------------
// rotary embedding + tentative KV append
// ------------------------------------------------------------------------------------------
// grid (ceil((H + 2 Hkv) / heads per block), M), 256 threads: a block takes 512 / hd consecutive heads of one row
// (one-wave blocks were bound by the rate at which workgroups can be dispatched: 11520 of them at the 70B shape);
// thread (head, t) owns the pair (t, t + hd/2) of its head.
// TA: activation type of the query buffer; T: storage type of the KV pages
constexpr int ROPE_THREADS = 256;
template <typename TA, typename T>
__global__ void __launch_bounds__(ROPE_THREADS) rope_append_kernel(RopeAppendArgs a) {
  const int m = blockIdx.y;
  const int hd = a.hd, half = hd >> 1;
  const int head = blockIdx.x * (ROPE_THREADS / half) + (int)threadIdx.x / half;
  const int t = (int)threadIdx.x % half;
  if (head >= a.H + 2 * a.Hkv) return;
  const int slot = a.rows.row_slot[m];  // (asked for first: the stores at the end wait for nothing else)
  const int ncols = (a.H + 2 * a.Hkv) * hd;
  const int c0 = head * hd + t, c1 = c0 + half;
  float v0 = 0.f, v1 = 0.f;
  // partials fetched eight at a time before any is added (see norm_kernel); the order of the sum is fixed
  for (int s0 = 0; s0 < a.n_partials; s0 += 8) {
    float p0[8], p1[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float* p = a.qkv + ((size_t)min(s0 + j, a.n_partials - 1) * a.M + m) * ncols;
      p0[j] = p[c0];
      p1[j] = p[c1];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < a.n_partials) { v0 += p0[j]; v1 += p1[j]; }
  }
  if (a.bias) { v0 += a.bias[c0]; v1 += a.bias[c1]; }
  const bool is_v = head >= a.H + a.Hkv;
  if (a.rope_cos && !is_v) {
    const float c = a.rope_cos[(size_t)m * half + t], s = a.rope_sin[(size_t)m * half + t];
    const float r0 = v0 * c - v1 * s;
    const float r1 = v1 * c + v0 * s;
    v0 = r0; v1 = r1;
  }
  bool bad = false;
  if (head < a.H) {
    TA* q = reinterpret_cast<TA*>(a.q) + ((size_t)m * a.H + head) * hd;
    store1<TA>(q + t, v0, bad);
    store1<TA>(q + t + half, v1, bad);
    if (bad && a.dev_status) atomicOr(a.dev_status, MN_DEV_RANGE);
    return;
  }
  if (slot < 0) return;  // disabled sequence: nothing is written to the cache (and nothing reported)
  const int bs = a.kv.block_size;
  const int pb = slot / bs;
  const int off = slot % bs;
  if (!is_v) {
    const int kh = head - a.H;
    T* base = reinterpret_cast<T*>(a.kv.k) + ((size_t)pb * a.Hkv + kh) * (size_t)hd * bs;
    // [hd/8][bs][8]
    store1<T>(base + ((size_t)(t >> 3) * bs + off) * 8 + (t & 7), v0, bad);
    const int t1 = t + half;
    store1<T>(base + ((size_t)(t1 >> 3) * bs + off) * 8 + (t1 & 7), v1, bad);
  } else {
    const int vh = head - a.H - a.Hkv;
    T* base = reinterpret_cast<T*>(a.kv.v) + ((size_t)pb * a.Hkv + vh) * (size_t)hd * bs;
    // [hd][bs]
    store1<T>(base + (size_t)t * bs + off, v0, bad);
    store1<T>(base + (size_t)(t + half) * bs + off, v1, bad);
  }
  if (bad && a.dev_status) atomicOr(a.dev_status, MN_DEV_RANGE);
}

void launch_rope_append(const RopeAppendArgs& a, hipStream_t st) {
  if (a.M <= 0) return;
  const int per_block = ROPE_THREADS / (a.hd / 2);  // head_dim is one of 8 ... 256: hd/2 divides 256
  dim3 grid((a.H + 2 * a.Hkv + per_block - 1) / per_block, a.M);
  if (a.dtype == MN_DT_BF16) rope_append_kernel<f16_t, f16_t><<<grid, ROPE_THREADS, 0, st>>>(a);
  else rope_append_kernel<float, float><<<grid, ROPE_THREADS, 0, st>>>(a);
}

// ------------------------------------------------------------------------------------------
// FFN activation on the first projection's partial sums
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) act_kernel(ActArgs a) {
  const size_t nvec = (size_t)a.M * (a.F >> 2);
  const int ncols = a.swiglu ? 2 * a.F : a.F;
  bool bad = false;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (size_t)gridDim.x * blockDim.x) {
    const int m = (int)(i / (a.F >> 2));
    const int f = (int)(i % (a.F >> 2)) << 2;
    float4 g = make_float4(0.f, 0.f, 0.f, 0.f), u = g;
    for (int s = 0; s < a.n_partials; ++s) {
      const float* p = a.partials + ((size_t)s * a.M + m) * ncols;
      const float4 x = *reinterpret_cast<const float4*>(p + f);
      g.x += x.x; g.y += x.y; g.z += x.z; g.w += x.w;
      if (a.swiglu) {
        const float4 y = *reinterpret_cast<const float4*>(p + a.F + f);
        u.x += y.x; u.y += y.y; u.z += y.z; u.w += y.w;
      }
    }
    float4 o;
    if (a.swiglu) {
      o.x = g.x / (1.f + __expf(-g.x)) * u.x;
      o.y = g.y / (1.f + __expf(-g.y)) * u.y;
      o.z = g.z / (1.f + __expf(-g.z)) * u.z;
      o.w = g.w / (1.f + __expf(-g.w)) * u.w;
    } else {
      if (a.bias) {
        const float4 bb = *reinterpret_cast<const float4*>(a.bias + f);
        g.x += bb.x; g.y += bb.y; g.z += bb.z; g.w += bb.w;
      }
      o = make_float4(fmaxf(g.x, 0.f), fmaxf(g.y, 0.f), fmaxf(g.z, 0.f), fmaxf(g.w, 0.f));
    }
    store4<T>(reinterpret_cast<T*>(a.act) + (size_t)m * a.F + f, o, bad);
  }
  if (bad && a.dev_status) atomicOr(a.dev_status, MN_DEV_RANGE);
}

void launch_act(const ActArgs& a, hipStream_t st) {
  if (a.M <= 0) return;
  const size_t nvec = (size_t)a.M * (a.F >> 2);
  int blocks = (int)((nvec + 255) / 256);
  if (blocks > 4096) blocks = 4096;
  if (a.dtype == MN_DT_BF16) act_kernel<f16_t><<<blocks, 256, 0, st>>>(a);
  else act_kernel<float><<<blocks, 256, 0, st>>>(a);
}

// ------------------------------------------------------------------------------------------
// vocabulary argmax: lowest id attaining the row maximum; NaN never wins
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void arg_better(float& bv, int& bi, float v, int i) {
  if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

__global__ void __launch_bounds__(256) argmax_rows_kernel(const float* __restrict__ logits, int M, int V, RowInfo rows,
                                                          int k_max, int32_t* __restrict__ greedy, int B) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int tid = threadIdx.x;
  if ((int)blockIdx.x >= M) {
    // padding blocks: one per sequence
    const int b = blockIdx.x - M;
    const int q = rows.seq_ok[b] ? rows.seq_row0[b + 1] - rows.seq_row0[b] : 0;
    for (int j = q + tid; j <= k_max; j += blockDim.x) greedy[(size_t)b * (k_max + 1) + j] = -1;
    return;
  }
  const int m = blockIdx.x;
  const float* r = logits + (size_t)m * V;
  float bv = -INFINITY;
  int bi = 0x7FFFFFFF;
  if ((V & 3) == 0) {
    // 16-byte pieces, eight in flight per thread before any is looked at (one piece per round trip is bound
    // by memory latency); a thread's indices grow, and ties between threads are settled by arg_better
    const float4* r4 = reinterpret_cast<const float4*>(r);
    const int n4 = V >> 2;
    for (int i0 = tid; i0 < n4; i0 += 8 * 256) {
      float4 p[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) p[u] = r4[min(i0 + u * 256, n4 - 1)];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i4 = i0 + u * 256;
        if (i4 < n4) {
          arg_better(bv, bi, p[u].x, 4 * i4);
          arg_better(bv, bi, p[u].y, 4 * i4 + 1);
          arg_better(bv, bi, p[u].z, 4 * i4 + 2);
          arg_better(bv, bi, p[u].w, 4 * i4 + 3);
        }
      }
    }
  } else {
    for (int i = tid; i < V; i += blockDim.x) arg_better(bv, bi, r[i], i);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    arg_better(bv, bi, ov, oi);
  }
  if ((tid & 63) == 0) { sv[tid >> 6] = bv; si[tid >> 6] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int w = 1; w < 4; ++w) arg_better(bv, bi, sv[w], si[w]);
    if (bi >= V) bi = 0;
    const int b = rows.row_seq[m];
    if (rows.seq_ok[b]) greedy[(size_t)b * (k_max + 1) + rows.row_j[m]] = bi;
  }
}

void launch_argmax_rows(const float* logits, int M, int V, const RowInfo& rows, int k_max, int32_t* greedy, int B,
                        hipStream_t st) {
  if (M + B <= 0) return;
  argmax_rows_kernel<<<M + B, 256, 0, st>>>(logits, M, V, rows, k_max, greedy, B);
}

}  // namespace mn
