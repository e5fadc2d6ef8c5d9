// Stochastic verification (paper section 2.1, the general rule; longest-prefix acceptance on argmax
// tokens is its temperature -> 0 case).  For every scored position the kernel decides whether the
// speculated token survives (kept outright when the SSM's probability q does not exceed the LLM's o,
// otherwise rejected with probability 1 - o/q) and, where it does not, or at the position after the
// last speculated token, draws a token from max(0, o - q) renormalised (from o itself after the last
// one).  The result has the layout of the greedy token array, with a surviving position holding its
// own speculated token, so the same acceptance and commit kernel turns it into the step's output:
// the first position whose entry differs from the speculated token is the first rejection.
//
// Arithmetic: fp64 throughout (the scores arrive as fp32).  A decision compares a 53-bit uniform
// number with a ratio or a running sum known to about 1e-14 relative, so it is reproducible by any
// other fp64 evaluation of the same definition except on a set of measure ~1e-14.
// Random numbers: Philox-4x32 with 10 rounds (Salmon et al., SC 2011), key = seed, counter =
// (sequence, position, step + consumer tag): a position's numbers do not depend on the batch it is scored in.
//
// The same file holds the drafting side of the rule: draft_sample_kernel draws an SSM's next token from
// its own q = softmax(scores / T) and writes q out for the verifier.
#include "launch.h"
#include "../../include/minions_verify.h"

namespace mn {

__device__ __forceinline__ void philox4x32_10(uint32_t c[4], uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c[0]), lo0 = 0xD2511F53u * c[0];
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c[2]), lo1 = 0xCD9E8D57u * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
}

// 27 + 26 random bits -> [0, 1)
__device__ __forceinline__ double unit_double(uint32_t hi, uint32_t lo) {
  return ((double)(hi >> 5) * 67108864.0 + (double)(lo >> 6)) * (1.0 / 9007199254740992.0);
}

constexpr int SV_THREADS = 256;
constexpr int SV_TILE = 1024;  // tokens per tile: a wave owns 256 of them, a lane 4 consecutive ones
constexpr int SV_MAX_TILES = 2048;

// Fixed-order sum of one double per thread: thread 0 adds the 256 values in thread order.
__device__ __forceinline__ double block_sum_ordered(double v, double* s_buf, int tid) {
  __syncthreads();
  s_buf[tid] = v;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int i = 0; i < SV_THREADS; ++i) t += s_buf[i];
    s_buf[SV_THREADS] = t;
  }
  __syncthreads();
  return s_buf[SV_THREADS];
}

struct DrawShared {
  double buf[SV_THREADS + 1];
  double tile[SV_MAX_TILES];  // mass of every tile
  double target[2];           // target inside the chosen tile, total mass
  int pick[2];                // chosen tile, chosen token
};

// Inverse-CDF draw over the vocabulary: the first token, in token order, whose running sum of mass(v)
// exceeds u times the total; -1 when the total is not positive.  Tokens are walked in tiles of 1024:
// thread t of the workgroup holds tokens tile*1024 + 4t .. 4t+3 (coalesced 16-byte pieces), so a prefix
// over (tile, thread, element) is a prefix in token order.  The per-tile masses are summed first, one
// thread finds the tile that holds the target, and that tile alone is scanned.  Every thread of the
// workgroup calls it; the result is uniform.  mass(v) must return the same value every time it is asked.
template <typename F>
__device__ int cdf_draw(F mass, int V, double u, DrawShared& sh, int tid) {
  const int n_tiles = (V + SV_TILE - 1) / SV_TILE;
  for (int t = 0; t < n_tiles; ++t) {
    double m = 0.0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = t * SV_TILE + 4 * tid + e;
      if (v < V) m += mass(v);
    }
    const double ts = block_sum_ordered(m, sh.buf, tid);
    if (tid == 0) sh.tile[t] = ts;
  }
  __syncthreads();
  if (tid == 0) {
    double total = 0.0;
    for (int t = 0; t < n_tiles; ++t) total += sh.tile[t];
    const double target = u * total;
    double before = 0.0;
    int t = 0;
    while (t < n_tiles - 1 && before + sh.tile[t] <= target) before += sh.tile[t++];
    sh.target[0] = target - before;
    sh.target[1] = total;
    sh.pick[0] = t;
    sh.pick[1] = 0x7fffffff;
  }
  __syncthreads();
  if (!(sh.target[1] > 0.0)) return -1;  // (whole workgroup)
  const int tile = sh.pick[0];
  const double target = sh.target[0];
  double m4[4], mine = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int v = tile * SV_TILE + 4 * tid + e;
    m4[e] = v < V ? mass(v) : 0.0;
    mine += m4[e];
  }
  sh.buf[tid] = mine;
  __syncthreads();
  double cum = 0.0;
  for (int i = 0; i < tid; ++i) cum += sh.buf[i];  // thread order = token order
  int hit = 0x7fffffff, last_pos = -1;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    cum += m4[e];
    const int v = tile * SV_TILE + 4 * tid + e;
    if (m4[e] > 0.0) {
      last_pos = v;
      if (cum > target && hit == 0x7fffffff) hit = v;
    }
  }
  if (hit != 0x7fffffff) atomicMin(&sh.pick[1], hit);
  __syncthreads();
  if (sh.pick[1] == 0x7fffffff) {  // rounding left the target at the tile's end: its last token with mass (whole workgroup)
    __syncthreads();
    if (tid == 0) sh.pick[1] = -1;
    __syncthreads();
    if (last_pos >= 0) atomicMax(&sh.pick[1], last_pos);
    __syncthreads();
  }
  return sh.pick[1];
}

// Largest score of a row and Z = sum_v exp((l_v - max) / T), both uniform over the workgroup.
__device__ __forceinline__ void row_max_and_z(const float* __restrict__ L, int V, double temperature, float* s_max,
                                              double* s_buf, int tid, double& dmx, double& Z) {
  float mx = -INFINITY;
  for (int v = tid; v < V; v += SV_THREADS) mx = fmaxf(mx, L[v]);
  s_max[tid] = mx;
  __syncthreads();
  for (int s = SV_THREADS / 2; s > 0; s >>= 1) {
    if (tid < s) s_max[tid] = fmaxf(s_max[tid], s_max[tid + s]);
    __syncthreads();
  }
  dmx = (double)s_max[0];
  double zp = 0.0;
  const int n_tiles = (V + SV_TILE - 1) / SV_TILE;
  for (int t = 0; t < n_tiles; ++t) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int v = t * SV_TILE + 4 * tid + e;
      if (v < V) zp += exp(((double)L[v] - dmx) / temperature);
    }
  }
  Z = block_sum_ordered(zp, s_buf, tid);
}

// The top byte of the counter's last word names the consumer of the numbers, so that the verifier
// (0) and the drafting SSMs (1 + index) never share a stream under one seed; steps are below 2^56.
__device__ __forceinline__ void position_uniforms(uint32_t b, uint32_t j, uint32_t step_lo, uint32_t step_hi,
                                                  uint32_t consumer, uint32_t seed_lo, uint32_t seed_hi, double& u0,
                                                  double& u1) {
  uint32_t w[4] = {b, j, step_lo, (step_hi & 0x00ffffffu) | (consumer << 24)};
  philox4x32_10(w, seed_lo, seed_hi);
  u0 = unit_double(w[0], w[1]);
  u1 = unit_double(w[2], w[3]);
}

// One workgroup per (position j, sequence b).
__global__ void __launch_bounds__(SV_THREADS) verify_sample_kernel(
    const float* __restrict__ logits, const int32_t* __restrict__ voted, const float* __restrict__ draft_probs,
    const int32_t* __restrict__ spec_len, const int32_t* __restrict__ greedy, int B, int k_max, int M, int V,
    double temperature, uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo, uint32_t step_hi,
    int32_t* __restrict__ sampled, int32_t* dev_status) {
  __shared__ DrawShared sh;
  __shared__ float s_max[SV_THREADS];
  __shared__ int s_int[2];  // rows before this sequence, bad flag
  const int j = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  int32_t* out = sampled + (size_t)b * (k_max + 1) + j;

  if (tid < 2) s_int[tid] = 0;
  __syncthreads();
  {  // rows of the sequences before b (integer sum: order-free)
    int part = 0, bad = 0;
    for (int i = tid; i < b; i += SV_THREADS) {
      const int k = spec_len[i];
      if (k < 0 || k > k_max) bad = 1;
      part += k + 1;
    }
    if (part) atomicAdd(&s_int[0], part);
    if (bad) atomicOr(&s_int[1], 1);
  }
  __syncthreads();
  const int k_b = spec_len[b];
  const int row = s_int[0] + j;
  const bool seq_ok = !s_int[1] && k_b >= 0 && k_b <= k_max && greedy[(size_t)b * (k_max + 1)] >= 0;
  if (!seq_ok || j > k_b || row >= M) {  // (whole workgroup)
    if (tid == 0) {
      *out = -1;
      if (seq_ok && j <= k_b && dev_status) atomicOr(dev_status, MN_DEV_SPEC_LEN);  // rows do not add up to M
    }
    return;
  }
  const float* L = logits + (size_t)row * V;
  double dmx, Z;
  row_max_and_z(L, V, temperature, s_max, sh.buf, tid, dmx, Z);
  double u_acc, u_res;
  position_uniforms((uint32_t)b, (uint32_t)j, step_lo, step_hi, 0u, seed_lo, seed_hi, u_acc, u_res);

  // ---- does the speculated token survive? ----
  bool keep = false;
  int x = -1;
  const float* Q = nullptr;
  if (j < k_b) {
    x = voted[(size_t)b * k_max + j];
    Q = draft_probs + ((size_t)b * k_max + j) * V;
    if (x >= 0 && x < V) {
      const double ox = exp(((double)L[x] - dmx) / temperature) / Z;
      const double qx = (double)Q[x];
      keep = (qx <= ox) || (u_acc < ox / qx);
    }
  }
  if (keep) {  // (whole workgroup: x, Q, Z, the random numbers are uniform over it)
    if (tid == 0) *out = x;
    return;
  }
  // ---- a token from max(0, o - q); without q (position k_b) from o.  When nothing of o lies above q (a q that
  // sums above 1) the replacement comes from o without the rejected token, so that it still differs from what
  // it replaces (the acceptance reads "first entry that differs" as the first rejection); and when all of o
  // sits on that token there is nothing else to emit: it stays ----
  int tok = -1;
  if (Q) {
    tok = cdf_draw([&](int v) { return fmax(0.0, exp(((double)L[v] - dmx) / temperature) / Z - (double)Q[v]); }, V,
                   u_res, sh, tid);
    if (tok < 0) tok = cdf_draw([&](int v) { return v == x ? 0.0 : exp(((double)L[v] - dmx) / temperature) / Z; }, V, u_res, sh, tid);
    if (tok < 0) tok = x;
  } else {
    tok = cdf_draw([&](int v) { return exp(((double)L[v] - dmx) / temperature) / Z; }, V, u_res, sh, tid);
  }
  if (tid == 0) *out = tok;
}

// One workgroup per sequence: token ~ q = softmax(scores / T) of a drafting SSM, and q itself in fp32.
// The draw is taken from the fp32 values that are written out, so what the verifier is later told is
// exactly the distribution the token came from.
__global__ void __launch_bounds__(SV_THREADS) draft_sample_kernel(const float* __restrict__ logits, int V,
                                                                  double temperature, uint32_t seed_lo, uint32_t seed_hi,
                                                                  uint32_t step_lo, uint32_t step_hi, uint32_t consumer,
                                                                  uint32_t t_pos, int32_t* __restrict__ tokens,
                                                                  long token_stride, float* __restrict__ probs,
                                                                  long probs_stride) {
  __shared__ DrawShared sh;
  __shared__ float s_max[SV_THREADS];
  const int b = blockIdx.x, tid = threadIdx.x;
  const float* L = logits + (size_t)b * V;
  double dmx, Z;
  row_max_and_z(L, V, temperature, s_max, sh.buf, tid, dmx, Z);
  double u_unused, u;
  position_uniforms((uint32_t)b, t_pos, step_lo, step_hi, consumer, seed_lo, seed_hi, u_unused, u);
  auto q32 = [&](int v) { return (float)(exp(((double)L[v] - dmx) / temperature) / Z); };
  if (probs) {
    float* P = probs + (size_t)b * probs_stride;
    for (int v = tid; v < V; v += SV_THREADS) P[v] = q32(v);
  }
  const int tok = cdf_draw([&](int v) { return (double)q32(v); }, V, u, sh, tid);
  if (tid == 0) tokens[(size_t)b * token_stride] = tok;
}

void launch_verify_sample(const float* logits, const int32_t* voted, const float* draft_probs, const int32_t* spec_len,
                          const int32_t* greedy, int B, int k_max, int M, int V, double temperature, uint64_t seed,
                          uint64_t step, int32_t* sampled, int32_t* dev_status, hipStream_t st) {
  if (B <= 0) return;
  verify_sample_kernel<<<dim3(k_max + 1, B), SV_THREADS, 0, st>>>(
      logits, voted, draft_probs, spec_len, greedy, B, k_max, M, V, temperature, (uint32_t)seed, (uint32_t)(seed >> 32),
      (uint32_t)step, (uint32_t)(step >> 32), sampled, dev_status);
}

void launch_draft_sample(const float* logits, int B, int V, double temperature, uint64_t seed, uint64_t step, int ssm,
                         int t_pos, int32_t* tokens, long token_stride, float* probs, long probs_stride, hipStream_t st) {
  if (B <= 0) return;
  draft_sample_kernel<<<B, SV_THREADS, 0, st>>>(logits, V, temperature, (uint32_t)seed, (uint32_t)(seed >> 32),
                                                (uint32_t)step, (uint32_t)(step >> 32), (uint32_t)(1 + ssm),
                                                (uint32_t)t_pos, tokens, token_stride, probs, probs_stride);
}

int verify_sample_max_vocab() { return SV_TILE * SV_MAX_TILES; }

}  // namespace mn
