// Internal launchers: one per kernel family.  Host-side shape checks happen in api.hip; the
// launchers assume validated arguments and only translate them into grids.
#pragma once
#include "common.h"

namespace mn {

// ---- vote_accept.hip ----
void launch_vote(const int32_t* drafts, const int32_t* spec_len, const float* ssm_w, int B, int n, int k_max, int mode,
                 int32_t* voted, int32_t* voted_ssm, int32_t* dev_status, hipStream_t st);
void launch_acr_update(const int32_t* voted_ssm, const int32_t* accepted_len, const int32_t* spec_len,
                       const int32_t* n_out, int B, int n, double reward_threshold, double punish_threshold,
                       float reward_factor, float punish_factor, float* ssm_w, double* acr, hipStream_t st);
void launch_accept_commit(const int32_t* voted, const int32_t* greedy, const int32_t* spec_len, int B, int k_max,
                          int32_t* ctx_lens, int block_size, int max_blocks_per_seq, int32_t* accepted_len,
                          int32_t* out_tokens, int32_t* n_out, int32_t* next_last_tok, int32_t* blocks_in_use,
                          int32_t* dev_status, hipStream_t st);

// ---- stochastic.hip ----
void launch_verify_sample(const float* logits, const int32_t* voted, const float* draft_probs, const int32_t* spec_len,
                          const int32_t* greedy, int B, int k_max, int M, int V, double temperature, uint64_t seed,
                          uint64_t step, int32_t* sampled, int32_t* dev_status, hipStream_t st);
void launch_draft_sample(const float* logits, int B, int V, double temperature, uint64_t seed, uint64_t step, int ssm,
                         int t_pos, int32_t* tokens, long token_stride, float* probs, long probs_stride, hipStream_t st);
int verify_sample_max_vocab();

// ---- rows.hip ----
struct PrepArgs {
  const int32_t *last_tok, *voted, *spec_len, *ctx_lens, *block_tables;
  int B, k_max, M, vocab, max_pos, block_size, num_blocks, max_blocks_per_seq;
  int max_ctx;       // the host's bound on ctx_b + k_b + 1 (it sized the attention launch)
  int rope_half;     // head_dim/2 for rotary models, 0 otherwise
  float rope_base;
  int32_t *row_seq, *row_j, *row_pos, *row_tok, *row_slot, *seq_row0, *seq_ctx, *seq_ok;
  int32_t* attn_tps;           // [1] out: key tiles per attention workgroup (see RowInfo)
  int kv_heads;                // KV heads of the model (the attention grid has one workgroup row per KV head)
  int q_per_kv;                // query heads per KV head (a workgroup covers 128 rows of query position x head)
  int attn_wgs;                // number of attention workgroups to aim for
  int attn_min_tiles;          // fewest key tiles a workgroup should take
  float *rope_cos, *rope_sin;  // [M][rope_half]
  int32_t* dev_status;
};
void launch_prepare(const PrepArgs& a, hipStream_t st);

struct NormArgs {
  // source of the row: either the residual stream x (+ partial sums + bias), or the embeddings
  float* x;               // [M][d] residual stream, updated in place
  const float* partials;  // [S][M][d] or null
  int n_partials;
  const float* bias;      // [d] or null
  const void* tok_emb;    // when non-null the row is tok_emb[row_tok] (+ pos_emb[row_pos])
  const void* pos_emb;
  const int32_t *row_tok, *row_pos;
  const float *gain, *shift;  // shift null => RMSNorm
  float eps;
  void* h;                // [M][d] normalised output in the activation type
  int M, d, dtype;
  int32_t* dev_status;    // MN_DEV_RANGE is OR-ed in when an fp16 output saturates, or null
};
void launch_norm(const NormArgs& a, hipStream_t st);

struct RopeAppendArgs {
  const float* qkv;  // [S][M][(H+2Hkv)*hd] partial sums
  int n_partials;
  const float* bias;  // [(H+2Hkv)*hd] or null
  const float *rope_cos, *rope_sin;  // [M][hd/2] or null (no rotation)
  RowInfo rows;
  KvView kv;
  void* q;  // [M][H][hd] activation type
  int M, H, Hkv, hd, dtype;
  int32_t* dev_status;  // MN_DEV_RANGE is OR-ed in when an fp16 output saturates, or null
};
void launch_rope_append(const RopeAppendArgs& a, hipStream_t st);

// act[m][f] = relu(sum_s p[s][m][f] + b[f])  or  silu(gate) * up with gate = column f, up = column F + f
struct ActArgs {
  const float* partials;  // [S][M][ncols]
  int n_partials;
  const float* bias;
  void* act;  // [M][F] activation type
  int M, F, swiglu, dtype;
  int32_t* dev_status;  // MN_DEV_RANGE is OR-ed in when an fp16 output saturates, or null
};
void launch_act(const ActArgs& a, hipStream_t st);

void launch_argmax_rows(const float* logits, int M, int V, const RowInfo& rows, int k_max, int32_t* greedy, int B,
                        hipStream_t st);

// ---- gemm.hip ----
struct GemmArgs {
  const void* a;  // [M][K] activation type (fp32 in fp32 models, fp16 in bf16 models)
  const void* w;  // fp32 models: [N][K] row-major; bf16 models: the packed layout of gemm.hip
  float* out;     // [S][M][N] fp32 partial sums (S = split_k); bias added to split 0 when given
  void* swiglu_act;  // non-null: fused SwiGLU epilogue, fp16 [M][N/2] (bf16 models, split_k == 1, interleaved packing)
  void* relu_act;    // non-null: fused bias + ReLU epilogue, fp16 [M][N] (bf16 models, split_k == 1)
  const float* bias;
  int M, N, K, split_k, dtype;
  int32_t* dev_status;  // MN_DEV_RANGE is OR-ed in when a fused fp16 epilogue saturates a value, or null
};
int gemm_pick_split(int M, int N, int K, int dtype);
size_t packed_weight_elems(int N, int K);
void launch_pack_weight(const void* src, void* dst, int N, int K, int half, int32_t* status, hipStream_t st);
// hipSuccess, or the error of a one-time kernel attribute setting that failed (nothing is launched then)
hipError_t launch_gemm(const GemmArgs& a, hipStream_t st);
void launch_reduce_partials(const float* partials, int S, size_t stride, float* out, size_t n, hipStream_t st);

// ---- attention.hip ----
struct AttnArgs {
  const void* q;  // [M][H][hd] activation type
  void* out;      // [M][H*hd] activation type
  RowInfo rows;
  KvView kv;      // every key is read from the pages, this step's own (appended before the call) included
  int B, M, H, Hkv, hd, dtype, max_ctx;
  int max_q;       // largest number of rows of one sequence (host knowledge)
  float* scratch;  // split-KV partials
  size_t scratch_bytes;
  int32_t* items;        // work list of the MFMA kernel, 8 int32 per record (see launch_attention_plan), or null
  size_t items_capacity; // records the buffer holds
  int32_t* row_splits;   // [M] KV splits of the row's sequence (written by the plan, read by the merge), or null
};
size_t attention_scratch_bytes(int M, int H, int hd, int max_ctx, int dtype);
bool attention_mfma_supported(int H, int Hkv, int hd, int block_size, int dtype);
int attention_min_tiles();  // fewest key tiles an attention workgroup should take (32)
int attention_target_workgroups();  // attention workgroups with work the plan aims for (320)
size_t attention_items_capacity(int B, int M, int H, int Hkv);
// once per step, after the row bookkeeping and before the first launch_attention: the list of workgroups
void launch_attention_plan(const AttnArgs& a, hipStream_t st);
// hipSuccess, or the error of a one-time kernel attribute setting that failed (nothing is launched then)
hipError_t launch_attention(const AttnArgs& a, hipStream_t st);

}  // namespace mn
