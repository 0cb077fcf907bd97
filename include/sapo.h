/*
 * sapo.h - C ABI of the MI355X (gfx950) implementation of the per-node hot path of
 * Swarm sAmpling Policy Optimization (SAPO).
 *
 * One node-round of Algorithm 1 spends its accelerator time in two places:
 *   - "Generate rollouts": for each question q of the batch, the policy pi^n produces a
 *     rollout R^n(q) = {a_1 .. a_L} of L sampled answers (Sec. 3.1, Algorithm 1)
 *                                                        -> sapo_rollout_generate
 *   - re-encoding every rollout of the training set T^n (own and swarm-shared) and
 *     computing its token-level values under the node's own policy, however unlikely the
 *     rollout is under it (Sec. 3.2), plus the group-relative advantages GRPO consumes
 *     (Sec. 4.2; zero-advantage groups, Sec. 3.2 and Sec. 5)
 *                                                        -> sapo_score_logprobs
 *
 * The policy is a decoder-only LM with RMSNorm, rotary positions (rotate-half pairing),
 * grouped-query attention, a SwiGLU FFN and an (optionally tied) LM head.
 *
 * Conventions
 *   - Every pointer marked "dev" is device (HBM) memory of the current HIP device, owned by
 *     the caller; the library never frees or reallocates caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: they return before the GPU has finished.  Outputs are valid after the
 *     stream has been synchronised.
 *   - The only allocations the library makes are the packed weight copy owned by a
 *     sapo_weights handle; rollout and scoring calls run entirely inside the caller's
 *     workspace.
 *   - Every function returning int returns SAPO_OK or a negative error code and writes
 *     nothing to its outputs when it rejects its arguments.  sapo_last_error() gives a
 *     human-readable message for the calling thread's last failure.
 *   - Token ids in inputs must lie in [0, vocab); this is not checked on the device.
 *   - Sequences of a rollout are ordered s = p * G + g (prompt-major); group of s is s / G.
 *   - Threads: calls that use the same sapo_weights handle, or the same workspace, must not
 *     overlap (a handle caches the captured decode step of its last rollout call); the first
 *     call of each kind in a process sets kernel attributes and must not race with another
 *     first call.  Different handles with different workspaces may be used from different
 *     threads after that.
 *   - A rollout call on a non-default stream replays one captured decode step (HIP graph);
 *     the calls with a stop token additionally synchronise the stream every 32 steps.
 *   - Environment (read when a handle is created / at every rollout call; for measurements and tests):
 *       SAPO_FORCE_GENERIC=1  a new sapo_weights handle uses the shape-generic kernels even for shapes the
 *                             matrix-core kernels accept
 *       SAPO_NO_GRAPH=1       rollout calls launch every decode step eagerly instead of replaying a graph
 *       SAPO_NO_COMPACT=1     rollout calls with a stop token keep ended sequences in the decode batch
 */
#ifndef SAPO_H
#define SAPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SAPO_OK = 0,
  SAPO_EINVAL = -1,     /* null pointer, non-positive size, negative temperature, S % G != 0, ... */
  SAPO_ESHAPE = -2,     /* model config the kernels cannot run (Hq % Hkv != 0, odd head_dim, ...) */
  SAPO_EWORKSPACE = -3, /* workspace smaller than the matching *_workspace_bytes() */
  SAPO_EHIP = -4        /* HIP runtime error (allocation, launch); see sapo_last_error() */
};

enum { SAPO_DTYPE_F32 = 0, SAPO_DTYPE_BF16 = 1 };

typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
  float rms_eps, rope_theta;
  int32_t tied_embeddings; /* 1: the LM head is the embedding matrix */
  int32_t dtype;           /* SAPO_DTYPE_*: storage type of weights, activations and KV cache */
  int32_t kv_page_tokens;  /* tokens per KV-cache page; must be 16 */
  int32_t max_seq;         /* longest sequence (prompt + generated) any call will use */
} sapo_model_config;

typedef struct sapo_weights sapo_weights; /* opaque, library-owned */

/*
 * Build the library's packed copy of the model weights.
 * tensors: host array of dev pointers in this order, matrices row-major
 *   [out_features, in_features] (y = x W^T), element type per cfg->dtype (fp32 or bf16),
 *   RMSNorm gains always fp32:
 *     embed[vocab, d];
 *     per layer: attn_norm[d], wq[Hq*hd, d], wk[Hkv*hd, d], wv[Hkv*hd, d], wo[d, Hq*hd],
 *                ffn_norm[d], w_gate[F, d], w_up[F, d], w_down[d, F];
 *     final_norm[d];
 *     lm_head[vocab, d]  (ignored, may be NULL, when tied_embeddings = 1).
 *   n_tensors must be 1 + 9 * n_layers + 2.
 * The copy is complete once `stream` has been synchronised; after that the caller may free
 * the originals.  Allocates device memory: bf16 models whose shapes fit the MFMA tiles keep two
 * fragment-ordered copies of every matrix (one per MFMA shape, for decode and for prefill/scoring)
 * besides the embedding table, about three times the model size; other models about once.
 *
 * Number format of the matrix-core path (bf16 models whose shapes fit the MFMA tiles;
 * sapo_weights_uses_mfma() tells): the packed matrices hold the bf16 weights' values as IEEE half,
 * and activations and the KV cache are rounded to half.  Half represents a bf16 value exactly for
 * 2^-14 <= |w| <= 65504; smaller non-zero weights keep an absolute error below 3e-8
 * (sapo_weights_half_stats counts them).  A weight beyond +-65504, infinite or NaN cannot be held:
 * the call then fails with SAPO_EINVAL (so does sapo_weights_update, which leaves the handle's
 * matrices unusable until it is filled again with valid weights), and because the answer needs the
 * packing kernels' counters the call waits for `stream` on this path.  An activation beyond
 * +-65504 is clamped to +-65504 (never infinite): the results stay finite but no longer follow the
 * definition; sapo_debug_half_clamped counts such values for a given batch.  The operand of a
 * projection after an RMSNorm is (residual row x gain), normalised after the product, so the clamp
 * is reached when |residual x gain| exceeds 65504, whatever the row's norm.
 */
int sapo_weights_create(const sapo_model_config* cfg, const void* const* tensors, int n_tensors,
                        void* stream, sapo_weights** out);
void sapo_weights_destroy(sapo_weights* w);
/*
 * New values for an existing handle (Algorithm 1: the updated policy replaces pi^n for the next round).
 * `tensors` as for sapo_weights_create with the handle's own configuration.  The handle's buffers are
 * refilled in place on `stream` - nothing is allocated, and the decode step captured by an earlier
 * rollout call stays valid - so no call that uses the handle may overlap with this one.  Biases set
 * with sapo_weights_set_qkv_bias keep their values until set again.
 */
int sapo_weights_update(sapo_weights* w, const void* const* tensors, int n_tensors, void* stream);
/*
 * out2[0] = 1 when the handle runs on the 16-bit matrix-core path, else 0; out2[1] = the number of
 * non-zero weight values below half's normal range (2^-14) at the last create / update (host ints).
 */
int sapo_weights_half_stats(const sapo_weights* w, int64_t* out2);

/*
 * Optional biases on the query / key / value projections of one layer (the decoder family the
 * paper's experiments ran, Sec. 4, carries them; sapo_weights_create builds a model without):
 * q = W_q x + bq, k = W_k x + bk, v = W_v x + bv, before the rotary embedding.
 *   bq dev fp32 [Hq*hd], bk, bv dev fp32 [Hkv*hd]; copied (complete once `stream` is synchronised).
 * May be called again to replace them.  Not to be called while a call using `w` is in flight.
 */
int sapo_weights_set_qkv_bias(sapo_weights* w, int layer, const float* bq, const float* bk, const float* bv,
                              void* stream);

/* Workspace sizes in bytes (0 on invalid arguments). */
size_t sapo_rollout_workspace_bytes(const sapo_weights* w, int P, int Lp, int G, int max_new);
size_t sapo_score_workspace_bytes(const sapo_weights* w, int S, int T);
size_t sapo_debug_logits_workspace_bytes(const sapo_weights* w, int S, int T, int n);

/*
 * Rollout generation (Sec. 3.1; Algorithm 1 "Generate rollouts").
 * For each of the P prompts, G completions of exactly max_new tokens are sampled
 * autoregressively from the policy at the given temperature.  Token t of sequence s is
 *   argmax_v ( z_v / temperature + g_v ),  g_v = -ln(-ln u_v)
 * (an exact sample of softmax(z / temperature)), with u_v from Philox4x32-10 keyed on
 * (seed, s, t, v); temperature == 0 is greedy argmax of z; ties go to the lowest id.
 *   prompts       dev int32 [P, Lp]
 *   out_tokens    dev int32 [P*G, max_new]   generated tokens only
 *   out_logprobs  dev fp32  [P*G, max_new]   log softmax(z)[token] at temperature 1
 *   workspace     dev, >= sapo_rollout_workspace_bytes(w, P, Lp, G, max_new), 256-byte aligned
 * Requires Lp >= 1, Lp + max_new <= cfg.max_seq.
 * A step whose logits are not numbers (NaN from non-finite weights set behind the library's back, or
 * a decode step that gave up its bounded wait) yields token -1 with log-prob 0 for that row instead
 * of an id; the row's later steps continue from id 0.  A caller that sees -1 discards the row.
 */
int sapo_rollout_generate(const sapo_weights* w, const int32_t* prompts, int P, int Lp, int G,
                          int max_new, float temperature, uint64_t seed, int32_t* out_tokens,
                          float* out_logprobs, void* workspace, size_t workspace_bytes,
                          void* stream);

/*
 * Rollout generation with a stop token (answers of different lengths, Sec. 3.1: an answer a_i(q)
 * ends where the policy ends it).  As sapo_rollout_generate, and in addition: the first stop_token a
 * sequence samples ends it (the token and its log-prob are kept); the rest of its row is stop_token
 * with log-prob 0.  The noise is keyed on (seed, sequence, step), so a row equals the row of the
 * plain call up to and including its stop.  Every 32 steps the host reads a counter (this call then
 * synchronises the stream) and returns early once every sequence has ended.  On the matrix-core
 * path with more than 64 sequences, ended sequences also leave the batch: once the running ones fit 256
 * (then 64) rows, the decode step goes on with that many rows.  A row of the result is then still the
 * sample the definition above describes for its sequence (same noise, same cache), computed by the
 * kernels of the smaller batch, whose logits differ from the larger batch's by fp32 summation order.
 *   stop_token   a vocabulary id
 *   out_lengths  dev int32 [P*G]   tokens generated including the stop token; max_new if none
 */
int sapo_rollout_generate_stop(const sapo_weights* w, const int32_t* prompts, int P, int Lp, int G,
                               int max_new, float temperature, uint64_t seed, int32_t stop_token,
                               int32_t* out_tokens, float* out_logprobs, int32_t* out_lengths,
                               void* workspace, size_t workspace_bytes, void* stream);
/*
 * Figures of the last rollout call made on this handle (host ints, for logs and tests):
 *   out4[0] decode steps enqueued (max_new - 1 unless every sequence ended early)
 *   out4[1] times the batch was compacted
 *   out4[2] rows per decode step at the end of the call
 *   out4[3] ended sequences at the last look (0 without a stop token)
 */
int sapo_rollout_last_stats(const sapo_weights* w, int32_t* out4);


/*
 * Rollout generation for prompts of different lengths (questions are presented directly as prompts,
 * Sec. 3.1; real question sets are not of one length), with an optional stop token.
 *   prompts      dev int32 [P, Lp_max]   prompt p occupies the first prompt_lens[p] entries of its row;
 *                                        the rest of the row is padding (any vocabulary ids)
 *   prompt_lens  HOST int32 [P]          1 <= prompt_lens[p] <= Lp_max; copied to the device on `stream`:
 *                                        keep it unchanged until the stream has been synchronised
 *   stop_token   a vocabulary id, or -1 for none (then out_lengths may be NULL)
 * Sequence s = p * G + g continues prompt p from position prompt_lens[p]; everything else is as in
 * sapo_rollout_generate / sapo_rollout_generate_stop: the result for prompt p equals what a call with
 * that prompt alone at its own length returns for the same sequence indices.  Workspace:
 * sapo_rollout_workspace_bytes(w, P, Lp_max, G, max_new).  Requires Lp_max + max_new <= cfg.max_seq.
 */
int sapo_rollout_generate_ragged(const sapo_weights* w, const int32_t* prompts, const int32_t* prompt_lens,
                                 int P, int Lp_max, int G, int max_new, float temperature, uint64_t seed,
                                 int32_t stop_token, int32_t* out_tokens, float* out_logprobs,
                                 int32_t* out_lengths, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Scoring pass (Sec. 3.2: token-level values of any rollout under the node's own policy;
 * Sec. 4.2: GRPO's group-relative advantage).
 *   tokens           dev int32 [S, T]   prompt + completion of every training-set sequence
 *   completion_mask  dev uint8 [S, T]   non-zero where a log-prob is wanted
 *   rewards          dev fp32  [S]
 *   out_logprobs     dev fp32  [S, T]   log softmax(z_{t-1})[tokens[s, t]] where the mask is
 *                                       set and t >= 1; 0.0 elsewhere
 *   out_advantages   dev fp32  [S]      per group of G consecutive sequences:
 *                                       (r - mean) / (population std + 1e-6); exactly 0 for a
 *                                       group whose rewards are all equal
 * Requires S % G == 0, T <= cfg.max_seq.
 */
int sapo_score_logprobs(const sapo_weights* w, const int32_t* tokens,
                        const uint8_t* completion_mask, const float* rewards, int S, int T, int G,
                        float* out_logprobs, float* out_advantages, void* workspace,
                        size_t workspace_bytes, void* stream);

/*
 * The same at a temperature: out_logprobs = log softmax(z_{t-1} / temperature)[tokens[s, t]], the
 * log-probs of the distribution a rollout at that temperature was sampled from (the rollout calls
 * themselves return the policy's log-probs at temperature 1).  temperature > 0.
 */
int sapo_score_logprobs_at(const sapo_weights* w, const int32_t* tokens,
                           const uint8_t* completion_mask, const float* rewards, int S, int T, int G,
                           float temperature, float* out_logprobs, float* out_advantages,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * Test hook: teacher-forced logits z (Sec. 3.2's re-encoding, before the log-softmax) at n
 * chosen (sequence, position) pairs: out_logits[i, :] are the logits after consuming
 * tokens[s_i, 0 .. t_i].
 *   tokens dev int32 [S, T]; positions dev int32 [n, 2] = (s, t); out_logits dev fp32 [n, vocab]
 */
int sapo_debug_logits(const sapo_weights* w, const int32_t* tokens, int S, int T,
                      const int32_t* positions, int n, float* out_logits, void* workspace,
                      size_t workspace_bytes, void* stream);

/*
 * Test hook for the number format stated at sapo_weights_create: runs the teacher-forced forward
 * pass of Sec. 3.2 over tokens[S, T] and counts, over every layer, the half-precision activation
 * values that sit at the clamp +-65504 (projection operands, rotated queries, attention outputs,
 * SwiGLU outputs, the LM head's operand).  0 means no activation of this batch was clamped (a
 * value that is exactly 65504 by itself also counts).  Always 0 for models on the shape-generic
 * kernels, which keep activations in the weights' own type.  Synchronises `stream`.
 *   tokens dev int32 [S, T]; out_count host; workspace dev, >= sapo_debug_logits_workspace_bytes(w, S, T, 1)
 */
int sapo_debug_half_clamped(const sapo_weights* w, const int32_t* tokens, int S, int T,
                            int64_t* out_count, void* workspace, size_t workspace_bytes,
                            void* stream);

/*
 * Training-set assembly (Sec. 3.2; Algorithm 1 "Assemble training set": SampleSelf and
 * SampleExternal).  A datapoint is one question's whole rollout: G consecutive rows of a pool.
 * n_local datapoints are drawn uniformly without replacement from the node's own pool, then n_ext
 * from the swarm pool after discarding the datapoints whose G rewards are all equal (zero
 * advantage; the filter the paper's experiments use).  Draw: datapoint g of a pool gets the key
 * Philox4x32-10(counter (g, 0, 0, stream), key seed)[0], stream 2 for the own pool and 1 for the
 * swarm pool; the sample is the eligible datapoints with the smallest (key, g), in that order.
 *   local_tokens  dev int32 [n_local_pool * G, T]   local_rewards  dev fp32 [n_local_pool * G]
 *   ext_tokens    dev int32 [n_ext_pool * G, T]     ext_rewards    dev fp32 [n_ext_pool * G]
 *   out_tokens    dev int32 [(n_local + n_ext) * G, T]   own datapoints first
 *   out_rewards   dev fp32  [(n_local + n_ext) * G]
 *   out_source    dev int32 [n_local + n_ext]   g for own datapoint g, n_local_pool + g for swarm
 *                                               datapoint g, -1 for a slot the pool could not fill
 *                                               (its rows are zero)
 *   out_counts    dev int32 [2]                 datapoints taken from the own / the swarm pool
 *   workspace     dev, >= sapo_assemble_workspace_bytes(n_local_pool, n_ext_pool), 256-byte aligned
 * Pools may be empty (pointers may then be NULL); each holds at most 16384 datapoints.
 * Exact (integer work).  n_ext = 0 is plain local fine-tuning.
 */
size_t sapo_assemble_workspace_bytes(int n_local_pool, int n_ext_pool);
int sapo_assemble_training_set(const int32_t* local_tokens, const float* local_rewards, int n_local_pool,
                               const int32_t* ext_tokens, const float* ext_rewards, int n_ext_pool, int G,
                               int T, int n_local, int n_ext, uint64_t seed, int32_t* out_tokens,
                               float* out_rewards, int32_t* out_source, int32_t* out_counts,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Clipped surrogate of the local policy update (Sec. 4.2: GRPO with the KL weight at zero and
 * asymmetric clipping, eps_low = 0.2, eps_high = 0.28), consuming what the two calls above produce.
 * Per masked token: rho = exp(logp_new - logp_old), A = advantages[s],
 *   term = min(rho A, clip(rho, 1 - eps_low, 1 + eps_high) A);
 * loss = - (sum of term) / (number of masked tokens), 0 when nothing is masked (the section does
 * not print the normalisation; this is the token-level mean of the recipe it cites).
 *   logp_new, logp_old  dev fp32 [S, T]   only read where the mask is set
 *   completion_mask     dev uint8 [S, T]
 *   advantages          dev fp32 [S]
 *   out_loss            dev fp32 [1]
 *   out_dlogp           dev fp32 [S, T] or NULL: d loss / d logp_new = -A rho / N where the unclipped
 *                       branch is the minimum (A >= 0 and rho <= 1 + eps_high, or A < 0 and
 *                       rho >= 1 - eps_low), 0 elsewhere and where the mask is clear
 *   workspace           dev, >= sapo_surrogate_workspace_bytes(), 256-byte aligned
 * rho and the branch are taken in fp32, the sums in fp64 in a fixed order (no atomics).
 * Returns SAPO_EINVAL for NULL buffers, non-positive sizes or eps outside [0, 1) / [0, inf).
 */
size_t sapo_surrogate_workspace_bytes(void);
int sapo_clipped_surrogate(const float* logp_new, const float* logp_old, const uint8_t* completion_mask,
                           const float* advantages, int S, int T, float eps_low, float eps_high,
                           float* out_loss, float* out_dlogp, void* workspace, size_t workspace_bytes,
                           void* stream);

/*
 * sapo_clipped_surrogate for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the
 * workspace, same kernels, same results bit for bit.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine): its scratch (256 block partials and the totals, 4112 bytes) is a file-scope
 * device array of the library, one copy per GPU, held until the process ends; its address is looked up on the
 * first call on a device.  The caller still passes inputs and outputs (device pointers).
 *   S * T at most SAPO_SURROGATE_NOALLOC_MAX_TOKENS; larger inputs are rejected with SAPO_EINVAL (as are NULL buffers,
 *   non-positive sizes and clip bounds out of range); SAPO_EHIP when the array's address cannot be obtained.
 * Every call on a GPU uses that GPU's one array (each call overwrites all of it before reading it, so nothing
 * carries over from the previous call): two calls that overlap in time on one GPU - different streams or
 * threads - race; run them in order.
 */
#define SAPO_SURROGATE_NOALLOC_MAX_TOKENS (1L << 28)
int sapo_clipped_surrogate_noalloc(const float* logp_new, const float* logp_old, const uint8_t* completion_mask,
                                   const float* advantages, int S, int T, float eps_low, float eps_high,
                                   float* out_loss, float* out_dlogp, void* stream);

/*
 * The local policy update (Algorithm 1, the PolicyGradient step; Sec. 4.2: GRPO with the KL weight
 * at zero, the clipped surrogate above, Adam with its default hyper-parameters: learning rate
 * 1e-3, beta1 0.9, beta2 0.999, eps 1e-8, no weight decay).
 *
 * A trainer owns fp32 master copies of every tensor of the model (embedding, projection matrices,
 * RMSNorm gains, the LM head when it is untied), their gradient and the two Adam moments: four
 * times the model in fp32, allocated by sapo_trainer_create and released by sapo_trainer_destroy.
 *   cfg, tensors, n_tensors   as for sapo_weights_create (device pointers, element type per
 *                             cfg->dtype, gains fp32); bf16 values become the fp32 masters unchanged.
 *                             head_dim at most 128.  Projection biases: sapo_trainer_set_qkv_bias.
 *   opt                       Adam's constants, or NULL for the defaults named above
 * Complete once `stream` has been synchronised.
 */
typedef struct { float lr, beta1, beta2, eps; } sapo_adam_config;
typedef struct sapo_trainer sapo_trainer; /* opaque, library-owned */
int sapo_trainer_create(const sapo_model_config* cfg, const void* const* tensors, int n_tensors,
                        const sapo_adam_config* opt, void* stream, sapo_trainer** out);
void sapo_trainer_destroy(sapo_trainer* tr);
/* Workspace of one update over S sequences of T tokens (every layer's activations are kept for the
 * backward pass: about 4 (4 d + 2 Hq hd + 2 Hkv hd + 3 F) bytes per token and layer, plus score
 * matrices, a chunk of logits and packed GEMM operands); 0 on invalid arguments (T < 2 or
 * T > max_seq).  At most 8192 tokens per sequence. */
size_t sapo_trainer_workspace_bytes(const sapo_trainer* tr, int S, int T);
/* The same when the update is to run S_micro <= S sequences at a time (see sapo_policy_update). */
size_t sapo_trainer_workspace_bytes_for(const sapo_trainer* tr, int S, int T, int S_micro);
/*
 * One update on the training set: teacher-forced forward pass under the masters, loss =
 * sapo_clipped_surrogate(logp_new, logp_old, mask, advantages), backward pass, one Adam step on
 * every tensor.
 *   tokens           dev int32 [S, T]   the assembled training set (prompt + completion per row)
 *   completion_mask  dev uint8 [S, T]   a set entry at t = 0 has no prediction behind it: it enters the
 *                                       loss with logp_new = 0 and carries no gradient
 *   logp_old         dev fp32 [S, T]    log-probs of the policy that is being improved (the scoring
 *                                       call's output); read where the mask is set
 *   advantages       dev fp32 [S]
 *   out_loss         dev fp32 [1]       the loss before the step
 *   out_logp_new     dev fp32 [S, T] or NULL: the log-probs under the masters before the step (0 where
 *                                       the mask is clear)
 *   workspace        dev, 256-byte aligned.  With sapo_trainer_workspace_bytes(tr, S, T) bytes the whole set
 *                    goes through forward and backward at once; with less, the call works through it in
 *                    micro-batches of the largest number of sequences whose activations fit
 *                    (sapo_trainer_workspace_bytes_for gives the size for a chosen number), adding their
 *                    gradients up before the one Adam step: the same update up to the order of fp32
 *                    additions.  SAPO_EWORKSPACE if not even one sequence fits.
 * fp32 values throughout (the large matrix products are formed from bf16 pieces on the matrix cores
 * with the accuracy of fp32 products), every sum in a fixed order (no atomics): the same call on the
 * same state gives the same bits.  The LM head runs only on the rows that predict a masked token; the host
 * sizes its products from their number, so the call waits once, at its start, for a small kernel that lists
 * them (and for whatever `stream` held before); everything else is enqueued and the call returns before the
 * update has finished.  The trainer's state is updated in place, so calls on one trainer must not overlap.  Errors: SAPO_EINVAL (NULL, sizes, eps), SAPO_EWORKSPACE.
 */
int sapo_policy_update(sapo_trainer* tr, const int32_t* tokens, const uint8_t* completion_mask,
                       const float* logp_old, const float* advantages, int S, int T, float eps_low,
                       float eps_high, float* out_loss, float* out_logp_new, void* workspace,
                       size_t workspace_bytes, void* stream);
/*
 * The masters in the model's storage type, for a new sapo_weights_create (the policy the next
 * round's rollouts are generated with): tensors_out is a host array of n_tensors device buffers in
 * the order and with the sizes of `tensors` above; matrices are written as cfg->dtype (bf16: round
 * to nearest even), gains as fp32.
 */
int sapo_trainer_export(const sapo_trainer* tr, void* const* tensors_out, int n_tensors, void* stream);
/*
 * Biases on the query / key / value projections of the trainer's model (the counterpart of
 * sapo_weights_set_qkv_bias): set copies bq dev fp32 [Hq*hd], bk, bv dev fp32 [Hkv*hd] into the masters
 * of `layer`; once any layer has been set, every layer's biases (zero where not set) are trained with
 * the rest.  get copies the masters out (dev fp32, same sizes) for the next sapo_weights_set_qkv_bias.
 */
int sapo_trainer_set_qkv_bias(sapo_trainer* tr, int layer, const float* bq, const float* bk, const float* bv,
                              void* stream);
int sapo_trainer_get_qkv_bias(const sapo_trainer* tr, int layer, float* bq, float* bk, float* bv, void* stream);
/*
 * Arithmetic of the update's large matrix products (projections and LM head; forward and backward).
 *   pieces = 3 (default): every fp32 operand is the exact sum of three bf16 values and a product is the
 *                sum of the six largest of the nine partial products: the accuracy of an fp32 product.
 *   pieces = 2: every operand is rounded to 16 significant bits (two bf16 values) and a product is the
 *                sum of three partial products: relative error below 2^-16 per product, of either sign,
 *                at half the matrix-core work.
 *   pieces = 1: operands rounded to bf16 (nearest even), fp32 accumulation: plain mixed precision,
 *                several times faster; gradients then carry the relative error of bf16 operands
 *                (about 2^-8 of a contraction's sum of absolute terms).
 * Masters, gradients, Adam and every other step stay fp32 either way.
 */
int sapo_trainer_set_matmul_pieces(sapo_trainer* tr, int pieces);
/* Number of Adam steps taken (-1 for NULL). */
int sapo_trainer_steps(const sapo_trainer* tr);
/*
 * Test hook: copies one tensor of the trainer's state to out (dev fp32 [n], n = the tensor's element
 * count).  what: 0 masters, 1 the last update's gradient, 2 / 3 Adam's first / second moment.  Tensor
 * n_tensors + l is layer l's bias vector [bq | bk | bv].
 */
int sapo_trainer_read(const sapo_trainer* tr, int what, int tensor, float* out, size_t n, void* stream);

/*
 * The current device as the runtime reports it (host ints, for the measurement's record):
 * out4 = {compute units, peak shader clock MHz, memory clock MHz, memory bus width in bits}.
 */
int sapo_device_info(int32_t* out4);

/*
 * Measurement hook: one launch of a kernel that only reads `bytes` bytes at `buf` (dev, 16-byte aligned; 2048
 * workgroups, 16-byte non-temporal loads): timed by the caller, it gives the streaming read bandwidth a kernel
 * can reach on the machine, as context for the HBM roofline figures.  sink: dev, 4 bytes (normally left alone).
 */
int sapo_debug_read_probe(const void* buf, size_t bytes, void* sink, void* stream);
/*
 * Measurement hook: one launch of a kernel that only issues matrix-core instructions on registers (n_workgroups
 * workgroups of 4 waves, two resident per compute unit; per wave `iters` rounds of 8 independent 32x32x16 half
 * MFMAs on the 6 KiB at `operands`: dev, 16-byte aligned, half values, read once).  *out_flops (host) = the
 * flops the launch executes; timed by the caller, it gives the rate the matrix cores sustain on the machine with
 * these operand values, as context for the MFMA roofline figures.  sink: dev, 4 bytes (normally left alone).
 */
int sapo_debug_mfma_probe(const void* operands, int n_workgroups, int iters, double* out_flops, void* sink,
                          void* stream);

/*
 * Test hook: the sampler's noise.  out[i] = g for (seed, seq, step, v = v0 + i), i < n.
 * out dev fp32 [n].
 */
int sapo_debug_gumbel(uint64_t seed, uint32_t seq, uint32_t step, uint32_t v0, int n, float* out,
                      void* stream);

/*
 * Per-kernel timing for benchmarks.  Between sapo_profile_start() and sapo_profile_stop() every
 * kernel launch the library makes carries two HIP events that receive the kernel's own start and
 * end timestamps on its stream (launches are no longer replayed from a captured graph while it is
 * on; do not time throughput then).  sapo_profile_stop() synchronises the device
 * and fills, per kernel symbol i < sapo_profile_kernel_count(), the summed duration in ms and the
 * number of launches (host arrays of at least sapo_profile_kernel_count() entries).  Not
 * thread-safe; at most 200000 launches are recorded.
 */
int sapo_profile_kernel_count(void);
const char* sapo_profile_kernel_name(int i);
int sapo_profile_start(void);
int sapo_profile_stop(double* total_ms, int64_t* launches, int n);
/* Message for the calling thread's last failed call ("" if none). */
const char* sapo_last_error(void);

/* 1 if this weights handle runs on the MFMA (bf16, tile-aligned) kernels, 0 if on the
 * shape-generic kernels. */
int sapo_weights_uses_mfma(const sapo_weights* w);

#ifdef __cplusplus
}
#endif
#endif /* SAPO_H */
