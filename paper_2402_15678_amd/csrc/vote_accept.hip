// Integer kernels of the verification step: the majority vote over SSM drafts (paper section 3.2,
// "Tree-based Weighted Majority Decision"), longest-prefix acceptance with KV commit (section
// 2.1 in its greedy case; section 4 for the deletion of rejected tokens' cache entries), and the
// speculation quality metric with the SSM weight update that closes the loop (section 3.2,
// equation ACR).
#include "launch.h"
#include "../../include/minions_verify.h"

namespace mn {

// One thread per sequence.  The token tree is never materialised: `alive` is the set of drafts
// whose prefix equals the path chosen so far, which is exactly the subtree below the current node.
// A child's weight is accumulated in fp32 in ascending draft order (the order is part of the result).
__global__ void vote_kernel(const int32_t* __restrict__ drafts, const int32_t* __restrict__ spec_len,
                            const float* __restrict__ ssm_w, int B, int n, int k_max, int mode,
                            int32_t* __restrict__ voted, int32_t* __restrict__ voted_ssm, int32_t* dev_status) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t* D = drafts + (size_t)b * n * k_max;
  int k = spec_len[b];
  if (k < 0 || k > k_max) {
    if (dev_status) atomicOr(dev_status, MN_DEV_DRAFTS);
    for (int t = 0; t < k_max; ++t) voted[(size_t)b * k_max + t] = -1;
    voted_ssm[b] = -1;
    return;
  }
  const uint64_t all = (n >= 64) ? ~0ull : ((1ull << n) - 1ull);
  uint64_t alive = all;
  for (int t = 0; t < k; ++t) {
    const uint64_t pool = (mode == MN_VOTE_TREE) ? alive : all;
    uint64_t todo = pool;  // drafts whose token at this level has not been weighed yet
    int best_tok = -1;
    float best_w = 0.f;
    bool have = false;
    uint64_t best_set = 0;
    while (todo) {
      const int j = __ffsll((unsigned long long)todo) - 1;
      const int tok = D[(size_t)j * k_max + t];
      float W = 0.f;
      uint64_t same = 0;
      uint64_t rest = pool;
      while (rest) {
        const int j2 = __ffsll((unsigned long long)rest) - 1;
        rest &= rest - 1;
        if (D[(size_t)j2 * k_max + t] == tok) {
          W += ssm_w[j2];
          same |= 1ull << j2;
        }
      }
      todo &= ~same;
      if (!have || W > best_w) {
        have = true;
        best_w = W;
        best_tok = tok;
        best_set = same;
      }
    }
    voted[(size_t)b * k_max + t] = best_tok;
    if (mode == MN_VOTE_TREE) alive = best_set;
  }
  for (int t = k; t < k_max; ++t) voted[(size_t)b * k_max + t] = -1;
  int ssm = -1;
  if (mode == MN_VOTE_TREE) {
    ssm = __ffsll((unsigned long long)alive) - 1;
  } else {
    for (int j = 0; j < n && ssm < 0; ++j) {
      bool eq = true;
      for (int t = 0; t < k && eq; ++t) eq = D[(size_t)j * k_max + t] == voted[(size_t)b * k_max + t];
      if (eq) ssm = j;
    }
  }
  voted_ssm[b] = ssm;
}

void launch_vote(const int32_t* drafts, const int32_t* spec_len, const float* ssm_w, int B, int n, int k_max, int mode,
                 int32_t* voted, int32_t* voted_ssm, int32_t* dev_status, hipStream_t st) {
  if (B <= 0) return;
  const int bs = 64;
  vote_kernel<<<(B + bs - 1) / bs, bs, 0, st>>>(drafts, spec_len, ssm_w, B, n, k_max, mode, voted, voted_ssm,
                                                dev_status);
}

// One thread per sequence: longest matching prefix, emitted tokens, context advance.
__global__ void accept_commit_kernel(const int32_t* __restrict__ voted, const int32_t* __restrict__ greedy,
                                     const int32_t* __restrict__ spec_len, int B, int k_max, int32_t* ctx_lens,
                                     int block_size, int max_blocks_per_seq, int32_t* __restrict__ accepted_len,
                                     int32_t* __restrict__ out_tokens, int32_t* __restrict__ n_out,
                                     int32_t* __restrict__ next_last_tok, int32_t* __restrict__ blocks_in_use,
                                     int32_t* dev_status) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const int32_t* g = greedy + (size_t)b * (k_max + 1);
  int32_t* o = out_tokens + (size_t)b * (k_max + 1);
  const int k = spec_len[b];
  const int ctx = ctx_lens[b];
  bool ok = (k >= 0 && k <= k_max && g[0] >= 0);
  if (k < 0 || k > k_max) {
    if (dev_status) atomicOr(dev_status, MN_DEV_SPEC_LEN);
  }
  int a = 0;
  if (ok) {
    const int32_t* v = voted + (size_t)b * k_max;
    while (a < k && v[a] == g[a]) ++a;
    const long cap = (long)max_blocks_per_seq * block_size;
    if ((long)ctx + a + 1 > cap) {
      ok = false;
      if (dev_status) atomicOr(dev_status, MN_DEV_BLOCK_TABLE);
    }
  }
  if (!ok) {
    for (int t = 0; t <= k_max; ++t) o[t] = -1;
    accepted_len[b] = 0;
    n_out[b] = 0;
    next_last_tok[b] = -1;
    blocks_in_use[b] = (ctx + block_size - 1) / block_size;
    return;
  }
  for (int t = 0; t <= k_max; ++t) o[t] = (t <= a) ? g[t] : -1;
  accepted_len[b] = a;
  n_out[b] = a + 1;
  next_last_tok[b] = g[a];
  const int nc = ctx + a + 1;
  ctx_lens[b] = nc;
  blocks_in_use[b] = (nc + block_size - 1) / block_size;
}

void launch_accept_commit(const int32_t* voted, const int32_t* greedy, const int32_t* spec_len, int B, int k_max,
                          int32_t* ctx_lens, int block_size, int max_blocks_per_seq, int32_t* accepted_len,
                          int32_t* out_tokens, int32_t* n_out, int32_t* next_last_tok, int32_t* blocks_in_use,
                          int32_t* dev_status, hipStream_t st) {
  if (B <= 0) return;
  const int bs = 64;
  accept_commit_kernel<<<(B + bs - 1) / bs, bs, 0, st>>>(voted, greedy, spec_len, B, k_max, ctx_lens, block_size,
                                                        max_blocks_per_seq, accepted_len, out_tokens, n_out,
                                                        next_last_tok, blocks_in_use, dev_status);
}

// Average acceptance rate per SSM and the multiplicative weight update (section 3.2, equation ACR).
// Thread i owns SSM i and walks the batch in ascending order: ACR_i is the mean, in fp64, of
// accepted_len / spec_len over the verified outputs whose voted SSM is i (outputs with nothing
// speculated, or that the step did not verify, are not in the set).  An SSM that won no vote keeps its
// weight and reports NaN.  The sum is sequential, so the result does not depend on the launch.
__global__ void acr_update_kernel(const int32_t* __restrict__ voted_ssm, const int32_t* __restrict__ accepted_len,
                                  const int32_t* __restrict__ spec_len, const int32_t* __restrict__ n_out, int B, int n,
                                  double reward_threshold, double punish_threshold, float reward_factor,
                                  float punish_factor, float* ssm_w, double* __restrict__ acr) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  double sum = 0.0;
  int cnt = 0;
  for (int b = 0; b < B; ++b) {
    const int k = spec_len[b];
    if (voted_ssm[b] != i || k <= 0 || (n_out && n_out[b] <= 0)) continue;
    sum += (double)accepted_len[b] / (double)k;
    ++cnt;
  }
  if (cnt == 0) {
    if (acr) acr[i] = __longlong_as_double(0x7ff8000000000000ll);
    return;
  }
  const double r = sum / (double)cnt;
  if (acr) acr[i] = r;
  if (r > reward_threshold) ssm_w[i] = ssm_w[i] * reward_factor;
  else if (r < punish_threshold) ssm_w[i] = ssm_w[i] * punish_factor;
}

void launch_acr_update(const int32_t* voted_ssm, const int32_t* accepted_len, const int32_t* spec_len,
                       const int32_t* n_out, int B, int n, double reward_threshold, double punish_threshold,
                       float reward_factor, float punish_factor, float* ssm_w, double* acr, hipStream_t st) {
  if (n <= 0) return;
  acr_update_kernel<<<1, 64, 0, st>>>(voted_ssm, accepted_len, spec_len, n_out, B, n, reward_threshold, punish_threshold,
                                      reward_factor, punish_factor, ssm_w, acr);
}

}  // namespace mn
