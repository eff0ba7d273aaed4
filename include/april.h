/*
 * april.h - C ABI of the MI355X-native APRIL rollout engine.
 *
 * APRIL (Active Partial Rollouts in Reinforcement Learning) schedules the rollout
 * phase of RL post-training: every step keeps N' > N rollouts in flight, stops as
 * soon as N of them are complete, parks the unfinished ones in a continuation
 * buffer and resumes them, ahead of new requests, at the next step (paper,
 * Section 2.2, the four-item description of the method).  With N' == N the same
 * call is the wait-for-all baseline of the paper's "standard setting"
 * (Section 3.1).
 *
 * The library owns the whole hot path on ONE gfx950 GPU: paged KV cache, prefill,
 * the batched decode loop (HIP kernels), the sampler, and a device-side scheduler
 * that counts finished rollouts and compacts the live batch without a host round
 * trip per token.  There is no CPU fallback: every call fails with APRIL_EDEVICE
 * when no GPU is usable.
 *
 * Conventions
 *   - all functions return APRIL_OK (0) or a negative error code; the message is
 *     available from april_last_error();
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory on the context's GPU; each argument says which one it is;
 *   - a context is single-threaded; calls on one context must not overlap;
 *   - matrices are row-major [out_features, in_features] (y = W x).
 */
#ifndef APRIL_H
#define APRIL_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define APRIL_OK        0
#define APRIL_EINVAL   -1   /* bad argument / unsupported configuration          */
#define APRIL_ENOMEM   -2   /* device memory or KV pool cannot hold the request   */
#define APRIL_ESTARVED -3   /* fewer than N_target rollouts can ever complete     */
#define APRIL_EHANDLE  -4   /* unknown / stale buffer handle or request id        */
#define APRIL_EDEVICE  -5   /* HIP error, or no usable GPU                        */

#define APRIL_DTYPE_FP32 0
#define APRIL_DTYPE_BF16 1
#define APRIL_MEM_KV      1   /* memory tags of april_memory_pause / april_memory_resume */
#define APRIL_MEM_WEIGHTS 2
#define APRIL_SAMPLER_GREEDY 0
#define APRIL_SAMPLER_TOPK   1   /* top-k, then (top_p < 1) the nucleus of the k candidates            */
#define APRIL_SAMPLER_CATEGORICAL 2   /* temperature sampling over the whole vocabulary (the paper's
                                         rollout setting, appendix: rollout temperature, no truncation) */

typedef struct april_ctx    april_ctx;     /* opaque; owns all device state            */
typedef struct april_buffer april_buffer;  /* opaque handle: a continuation buffer     */

/* Model and engine configuration (host memory, read during april_init only).
 * The network is a pre-norm decoder: RMSNorm, q/k/v projections without bias,
 * rotary embedding (pair (i, i + head_dim/2), angle pos * rope_theta^(-2i/head_dim)),
 * causal attention with n_q_heads / n_kv_heads query heads sharing one KV head,
 * output projection + residual, RMSNorm, SwiGLU MLP (or routed experts) + residual,
 * final RMSNorm, untied LM head.  The paper names only the model family it runs
 * (Section 3.1); the rollout itself is Eq. 1's a ~ pi(theta_k). */
typedef struct {
  int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int32_t n_experts, experts_per_tok, d_expert_ffn;  /* 0,0,0 => dense MLP                */
  int32_t dtype;             /* APRIL_DTYPE_*: type of weights, KV cache, GEMM operands   */
  float   rope_theta, rms_eps;
  int32_t kv_block_tokens;   /* tokens per KV page; must be 16                            */
  int64_t kv_pool_bytes;     /* 0 => sized for max_inflight sequences of max_ctx tokens,
                                but at most the free device memory less a reserve for the
                                workspaces (max(12 GiB, 1/16 of the device))              */
  int32_t max_inflight;      /* sequence slots (in flight + parked + surplus-complete)    */
  int32_t max_ctx;           /* max prompt + generated tokens of one sequence             */
  int32_t sampler;           /* APRIL_SAMPLER_*                                           */
  int32_t top_k;             /* 1..64 for the top-k sampler                               */
  float   temperature;       /* > 0, top-k sampler only                                   */
  uint64_t seed;             /* Philox key of the sampler                                 */
  int32_t eos_token;         /* -1: only length limits end a rollout                      */
  int32_t debug_logits;      /* 1: parity mode, logits of watched requests are kept       */
  float   top_p;             /* top-k sampler: keep the shortest prefix of the k candidates
                                (descending) whose probabilities, renormalised over the k
                                candidates, reach top_p; 0 or >= 1: no nucleus cut (the paper's
                                appendix lists an evaluation top_p)                          */
  int32_t logprobs;          /* 1: keep log softmax(logits / temperature)[token] over the whole
                                vocabulary for every generated token (what a trainer's
                                importance ratio needs, Section 2.2) and return it            */
  int32_t n_samples_per_prompt;  /* G > 1: instance-level completion (Section 3.2.3; Section 3.1
                                runs 32 x 8): every input instance is a group of G rollouts
                                (april_request.group_id), admitted together; a step stops once
                                N_target / G groups have all members complete and returns those
                                groups whole; complete members of an unfinished group wait in the
                                buffer.  N_target and N_overprovision stay rollout counts and must
                                be multiples of G.  0 or 1: every rollout on its own             */
  int32_t pausable;          /* 1: the KV pool and the weights live in reserved virtual address
                                ranges whose physical memory april_memory_pause can release    */
  void*   stream;            /* hipStream_t to run on (e.g. torch's current), or NULL     */
} april_model_cfg;

/* One named weight tensor.  `data` is host or device memory (on_device says which),
 * borrowed for the duration of april_init only: the library keeps its own copy in
 * the layout its kernels want.  Element type: float for APRIL_DTYPE_FP32, bf16 bit
 * patterns (uint16) for APRIL_DTYPE_BF16; norm gains are always float.
 * Names (l = layer index): tok_emb [vocab,d]; attn_norm.l [d]; wq.l [Hq*dh,d];
 * wk.l, wv.l [Hkv*dh,d]; wo.l [d,Hq*dh]; mlp_norm.l [d]; w_gate.l, w_up.l [F,d];
 * w_down.l [d,F]; final_norm [d]; lm_head [vocab,d]; for experts: router.l [E,d],
 * e_gate.l, e_up.l [E,Fe,d], e_down.l [E,d,Fe]. */
typedef struct {
  const char* name;
  const void* data;
  int64_t     nbytes;
  int32_t     on_device;
} april_tensor;

/* A new rollout request (host memory, borrowed during the call).
 * forced_len > 0: the rollout is complete exactly when it has generated
 * min(forced_len, max_new) tokens (synthetic long-tail workloads); 0: only max_new
 * and the EOS token end it.  forced_tokens (may be NULL): teacher forcing for
 * parity tests - generated token i is replaced by forced_tokens[i] for
 * i < n_forced_tokens after the sampler has run. */
typedef struct {
  int64_t        request_id;
  const int32_t* tokens;          /* prompt, host */
  int32_t        n_tokens;
  int32_t        forced_len;
  const int32_t* forced_tokens;   /* host, or NULL */
  int32_t        n_forced_tokens;
  int64_t        group_id;        /* input instance (n_samples_per_prompt > 1): its G requests are
                                     consecutive in new_reqs; ignored otherwise                  */
} april_request;

/* Result of one step.  Every pointer is host memory owned by the context and valid
 * until the next april_rollout_step / april_destroy on that context. */
typedef struct {
  int32_t  n_completed;           /* == N_target on success                                */
  const int64_t* request_id;      /* [n_completed], completion order (iteration, then id)  */
  const int32_t* const* tokens;   /* [n_completed] generated tokens only                   */
  const int32_t* n_tokens;        /* [n_completed]                                         */
  const int32_t* n_resumes;       /* [n_completed] steps the rollout spanned, minus one    */
  const float* const* logprobs;   /* [n_completed] per generated token (cfg.logprobs), else NULL */
  const int64_t* group_id;        /* [n_completed] (n_samples_per_prompt > 1: the members of a group are
                                     adjacent, ascending request id), else NULL                  */
  april_buffer*  buffer;          /* unfinished + surplus-complete rollouts (never NULL)   */
  int32_t  n_new_consumed;        /* how many of new_reqs were admitted                    */
  int64_t  decode_iters;          /* iterations executed (each adds 1 token per live seq)  */
  int64_t  tokens_generated;      /* over all in-flight rollouts, partial ones included    */
  int64_t  prefill_tokens;        /* prompt tokens of newly admitted rollouts              */
  int64_t  reprefill_tokens;      /* tokens recomputed for rollouts resumed without KV     */
  int64_t  n_preempted;           /* rollouts preempted in this step (KV pool exhausted)   */
  int64_t  sum_live;              /* sum over decode-path iterations of the live batch     */
  int64_t  sum_ctx;               /* sum over decode-path (iteration, seq) of context len  */
  int64_t  dec_sum_live, dec_sum_ctx;  /* the same sums over iterations 2.. only: the ones
                                          t_decode_s covers (iteration 1 is timed with prefill) */
  int64_t  dec_sum_experts;       /* routed experts: sum over (iteration 2.., layer) of the
                                     experts that received at least one token              */
  double   t_prefill_s, t_decode_s, t_total_s;   /* host wall clock                        */
} april_step_result;

/* A rollout as stored in a continuation buffer, token-level view (Section 3.2.3:
 * the buffer caches the tokens of incomplete trajectories). */
typedef struct {
  int64_t request_id;
  const int32_t* prompt;    int32_t n_prompt;      /* host */
  const int32_t* generated; int32_t n_generated;   /* host */
  int32_t limit;            /* generated length at which it completes                      */
  int32_t n_resumes;
  int32_t done;             /* 1: complete, waiting to be delivered first next step        */
  int32_t kv_resident;      /* 1: its KV pages are still on the device                     */
  const float* logprobs;    /* host, [n_generated] (cfg.logprobs), or NULL                  */
  int64_t group_id;         /* input instance (n_samples_per_prompt > 1), else -1           */
} april_partial;

/* Create a context on the current HIP device: copy/re-layout the weights, carve the
 * KV pool into pages, allocate scheduler state and workspaces. */
int april_init(const april_model_cfg* cfg, const april_tensor* weights, int32_t n_weights,
               april_ctx** out);

/* One rollout step (Section 2.2).  In flight = rollouts resumed by april_resume
 * (ascending request id) + new_reqs in order until N_overprovision are in flight
 * (surplus-complete rollouts in the resumed buffer count toward N_target and reduce
 * the number admitted).  Runs prefill for new / KV-less rollouts and decode
 * iterations - one token per live rollout per iteration - until N_target rollouts
 * are complete, then returns exactly N_target of them and a buffer with the rest.
 * N_overprovision == N_target is the wait-for-all baseline.
 * KV pool exhausted: a rollout that needs prefill is admitted only while the pages of its
 * tokens fit (the first that does not fit closes admission for the step); before an
 * iteration, if the rollouts that open a new page need more pages than are free, the
 * youngest decoding rollout (largest request id) is preempted - pages freed, tokens kept,
 * no progress this step, re-prefilled when resumed; if nothing is left in flight the step
 * returns fewer than N_target (n_completed says how many).
 * new_reqs: host array [n_new_avail]; out: host struct filled by the call.
 * A call that fails is transactional with respect to the rollouts: none of new_reqs is
 * consumed (the caller still owns them), and every rollout that april_resume had handed in
 * goes back to the pending set - with the tokens it generated before the failure, without its
 * KV pages - so the next april_rollout_step admits it first again; `out` is not filled. */
int april_rollout_step(april_ctx* ctx, const april_request* new_reqs, int32_t n_new_avail,
                       int32_t N_target, int32_t N_overprovision, int32_t max_new,
                       april_step_result* out);

/* Prioritized resumption: hand a buffer back; its rollouts are admitted ahead of new
 * requests in the NEXT april_rollout_step.  Consumes the handle. */
int april_resume(april_ctx* ctx, april_buffer* buffer);

/* Number of rollouts in a buffer (negative: error). */
int april_buffer_size(const april_ctx* ctx, const april_buffer* buffer);
/* Token-level view of a buffer: fills out[0..min(size,cap)) (host), arrays are owned
 * by the context and valid until the buffer is freed or resumed.  Returns the size. */
int april_buffer_export(april_ctx* ctx, const april_buffer* buffer, april_partial* out, int32_t cap);
/* Build a buffer from token-level entries (host, copied); such rollouts have no KV on
 * the device and are re-prefilled when resumed. */
int april_buffer_import(april_ctx* ctx, const april_partial* in, int32_t n, april_buffer** out);
/* Release the KV pages of every rollout in the buffer: they resume by re-prefill
 * (fallback path; also what a change of policy weights would require). */
int april_buffer_drop_kv(april_ctx* ctx, april_buffer* buffer);
/* Drop a buffer and everything it holds. */
void april_buffer_free(april_ctx* ctx, april_buffer* buffer);

/* Policy update between steps (Eq. 1: the trainer moves theta_k to theta_{k+1} after every
 * step, and rollouts parked under theta_k are continued under theta_{k+1}: Section 2.2,
 * trajectories of a mixed policy).  `weights` as for april_init (same names and sizes, host or
 * device, borrowed during the call); the library overwrites its own copies in place.
 * keep_kv = 0: the K/V of every parked rollout was computed under the old weights, so its pages
 * are released and the rollout is re-prefilled under the new weights when it is resumed (its
 * tokens are kept).  keep_kv = 1: the stale K/V stays and decoding simply goes on (cheaper, and
 * an approximation: the measured alternative).  Call between steps only.  On an error the
 * context's weights are undefined until a later call succeeds. */
int april_update_weights(april_ctx* ctx, const april_tensor* weights, int32_t n_weights, int32_t keep_kv);

/* Pause / resume of the engine's large device buffers by virtual-memory remapping (Section 3.3,
 * the memory-saving extension that lets rollout and training share one GPU on either vendor's
 * hardware; cfg.pausable = 1).  tags: APRIL_MEM_KV | APRIL_MEM_WEIGHTS.
 * april_memory_pause releases the physical memory behind the tagged buffers; their virtual
 * addresses stay reserved, so everything that holds those addresses (captured iteration graphs
 * included) remains valid.  april_memory_resume maps fresh physical memory at the same addresses.
 * Contents do not survive: after a KV pause every parked rollout keeps its tokens and is
 * re-prefilled when resumed (the pool comes back zeroed and entirely free); after a weights
 * pause april_update_weights must be called before the next step.  Call between steps only;
 * april_rollout_step fails with APRIL_EINVAL while anything is paused. */
int april_memory_pause(april_ctx* ctx, int32_t tags);
int april_memory_resume(april_ctx* ctx, int32_t tags);

/* Parity mode (cfg.debug_logits = 1): keep the fp32 logits that produced generated
 * tokens [first_gen, first_gen + n_gen) of request_id.  Call before the step that
 * generates them. */
int april_debug_watch(april_ctx* ctx, int64_t request_id, int32_t first_gen, int32_t n_gen);
/* Copy the kept logits row (vocab floats, host) and the sampler's own choice for it. */
int april_debug_logits(april_ctx* ctx, int64_t request_id, int32_t gen_index,
                       float* out_logits, int32_t* out_sampled);

/* The sampler alone (Section 3.1 samples with a temperature; greedy / top-k are the
 * configured ones): logits is a DEVICE array [n_rows, vocab] of float; request_ids,
 * gen_index (host, [n_rows]) key the Philox stream; out_tokens host [n_rows]. */
int april_sample_rows(april_ctx* ctx, const float* logits, int32_t n_rows,
                      const int64_t* request_ids, const int32_t* gen_index, int32_t* out_tokens);

/* The same with the log-probability of each chosen token (out_logprobs host [n_rows]):
 * log softmax(logits / temperature) over the whole vocabulary. */
int april_sample_rows_logprobs(april_ctx* ctx, const float* logits, int32_t n_rows,
                               const int64_t* request_ids, const int32_t* gen_index,
                               int32_t* out_tokens, float* out_logprobs);

/* april_sample_rows for callers that cannot allocate device memory (code under HIP graph
 * capture rules, tight serving loops, harnesses that forbid hipMalloc): same arguments, same
 * result, but every temporary (row keys, result staging, control word, the per-row maxima of
 * 64-logit groups) lives in a static device array of 4 MiB + 16.25 KiB that the library holds on
 * every GPU it runs on until the process ends; the call makes no hipMalloc / hipFree.
 * Limits: n_rows <= 1024 and n_rows * (vocab / 64) <= 1048576 (APRIL_EINVAL beyond).
 * All calls on one GPU share that array and it keeps the last call's contents: calls that
 * overlap on one GPU (other threads, other contexts) race; serialise them. */
int april_sample_rows_noalloc(april_ctx* ctx, const float* logits, int32_t n_rows,
                              const int64_t* request_ids, const int32_t* gen_index, int32_t* out_tokens);

/* Per-kernel-class timing, measured with HIP events on the context's stream around
 * sampled launches of the real decode loop (every `every`-th iteration; 0 = off).  Two extra
 * classes calibrate the method: "event_pair_no_kernel" is what a pair of event records reads
 * with nothing between them (the cost of the pair itself; subtract it from a class's average to
 * get the launch's own time), "event_pair_empty_kernel" the same around a kernel that does
 * nothing (the floor of any single launch). */
#define APRIL_KERNEL_CLASSES 24
typedef struct {
  const char* name;
  int64_t launches;          /* timed launches                                           */
  double  total_ms;          /* their summed duration                                    */
  double  alg_bytes;         /* algorithmic HBM bytes those launches had to move         */
  double  alg_flops;         /* floating-point operations of those launches              */
} april_kernel_stat;
int april_profile_enable(april_ctx* ctx, int32_t every);
int april_profile_get(april_ctx* ctx, april_kernel_stat* out, int32_t cap);   /* returns count */
int april_profile_reset(april_ctx* ctx);

/* Device facts used for reporting: free/total bytes, KV pages, weight bytes. */
typedef struct {
  int64_t hbm_total, hbm_free, kv_pool_bytes, kv_blocks_total, kv_blocks_free,
          weight_bytes, decode_weight_bytes, kv_bytes_per_token,
          expert_bytes;   /* routed experts: bytes of one expert's matrices; decode_weight_bytes
                             then covers everything but the experts                         */
} april_info;
int april_get_info(april_ctx* ctx, april_info* out);

const char* april_last_error(const april_ctx* ctx);   /* ctx may be NULL: init errors */
void april_destroy(april_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* APRIL_H */
