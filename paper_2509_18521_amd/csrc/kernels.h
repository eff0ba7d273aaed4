// Launcher prototypes of the HIP kernels (gfx950).  Every launcher enqueues on
// `st` and returns immediately; none allocates.
//
// Row model: a forward pass runs over "rows"; row r belongs to sequence slot
// row_slot[r] and sits at position row_pos[r].  For a decode iteration the rows are
// the live rollouts (written by the scheduler kernel), for prefill they are all
// prompt tokens of the admitted rollouts.  The row count lives in device memory next to
// the stop flag; kernels whose block index is beyond it exit, and a raised stop flag
// turns every kernel into a no-op once the scheduler has ended the step.
#pragma once
#include "common.h"

namespace april {

struct RowCtx {
  const int* row_slot;
  const int* row_pos;
  const int2* ctl;       // device: x = number of rows, y = stop flag (one 8-byte scalar load)
  int max_rows;          // host-known upper bound (grid size)
};

// Rows to process: 0 once the scheduler has ended the step.
__device__ inline int rows_or_zero(const RowCtx& rc) {
  const int2 v = *rc.ctl;
  return v.y ? 0 : v.x;
}
// Early exit of a one-workgroup-per-row kernel: step stopped, or row beyond the batch.
#define ROW_GUARD(rc, r) \
  if ((r) >= rows_or_zero(rc)) return;

// Rotary embedding of the pair (a, b) = (x[i], x[i + d/2]) with cos c and sin s, in one
// fixed operation order (no compiler-chosen contraction), so that every kernel that rotates
// produces the same bits.
__device__ inline float rope_first(float a, float b, float c, float s) { return __fmaf_rn(a, c, -__fmul_rn(b, s)); }
__device__ inline float rope_second(float a, float b, float c, float s) { return __fmaf_rn(b, c, __fmul_rn(a, s)); }

// silu(g) * u with the hardware reciprocal (1 ulp) instead of a full-precision division: the
// result is rounded to bf16 right after, and the division was most of the SwiGLU epilogue.
__device__ inline float silu_mul(float g, float u) { return g * u * __builtin_amdgcn_rcpf(1.0f + __expf(-g)); }

// --- scheduler / allocator -------------------------------------------------
// check_only = 1: only the "N complete => stop" test (end of a chunk of iterations).
// row_cap / ctx_cap: the bounds the host sized this iteration's launches for (live rows, longest
// context); exceeding one sets error bit 2 in the control block and stops the step.
// att_items (or null): work list for the decode attention, written when rows are rebuilt: entry 0
// = {count, 0, 0, 0}, entry 1 + i = {row, KV split, slot, position}, one per (row, split of
// att_split tokens the row's context reaches), full splits first, then the rows' last splits by
// descending length (classes of att_split / 32 tokens; the order inside a class is arbitrary).
// att_cap = entries the list holds beyond the first; more items than that raise error bit 2.
void launch_sched(hipStream_t st, Ctrl* ctrl, Slots s, int* row_slot, int* row_pos,
                  int* free_stack, int blk, int check_only, int row_cap, int ctx_cap,
                  int4* att_items = nullptr, int att_split = 0, int att_cap = 0);
void launch_alloc_prefill(hipStream_t st, Ctrl* ctrl, Slots s, const int* slot_list,
                          const int* n_blocks_needed, int n, int* free_stack);
void launch_free_slots(hipStream_t st, Ctrl* ctrl, Slots s, const int* slot_list, int n,
                       int* free_stack);
void launch_init_free_stack(hipStream_t st, int* free_stack, int n_blocks);
void launch_fill_i32(hipStream_t st, int* p, int v, size_t n);

// --- model ------------------------------------------------------------------
template <typename T>
void launch_embed(hipStream_t st, RowCtx rc, Slots s, const T* emb, float* x_res, int d);

// x_res += sum of partials (if any); h = rmsnorm(x_res) * gain.  gather (nullable):
// input row index of output row r.
// pos_of / wts (nullable, mixture-of-experts combine): partial p of row r is then the row
// pos_of[r * n_partials + p] of `partials` ([packed rows][d]) weighted by wts[r * n_partials + p].
template <typename T, bool XF>
void launch_add_rmsnorm(hipStream_t st, RowCtx rc, float* x_res, const float* partials,
                        int n_partials, size_t partial_stride, const float* gain, T* h,
                        int d, float eps, const int* gather, const int* pos_of = nullptr,
                        const float* wts = nullptr, T* h_rows = nullptr);

// --- routed experts (bf16) ---------------------------------------------------------
void launch_moe_route(hipStream_t st, RowCtx rc, const float* logits, int n_partials, size_t partial_stride,
                      int E, int top_k, int* ids, float* wts);
void launch_moe_dispatch(hipStream_t st, RowCtx rc, const int* ids, int E, int top_k, int* cnt, int* base,
                         int* pos_of, int* src_row, int p_cap, Ctrl* ctrl, int tall_rows, int* group_expert);
// upper bound on the row groups (of `align` rows) of a launch over at most max_rows rows
int moe_group_count(int max_rows, int top_k, int E, int align);
// tall_rows: row bound from which a GEMM workgroup takes 4 m-tiles of an expert instead of 2
// (the dispatch aligns the expert segments accordingly: pass the same value to all three)
// LDS-tiled expert GEMMs for prefill passes (kernels_gemm_tile.hip): row groups of moe_tile_rows()
// packed rows (the dispatch must have aligned the expert segments to that), one accumulator chain
// per output element.  Return false (nothing launched) for shapes they do not take.
int moe_tile_rows();
// (gate/up: h_rows is the plain [row][d] copy of the normalised activations that
// launch_add_rmsnorm writes on request; its rows are gathered through src_row)
bool launch_moe_tile_gateup(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                            const int* src_row, const bf16_t* h_rows, const bf16_t* Wg, const bf16_t* Wu, bf16_t* act,
                            int Fe, int d, int n_groups);
bool launch_moe_tile_down(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                          const bf16_t* act, const bf16_t* Wd, float* out, int Fe, int d, int n_groups);
void launch_moe_gateup(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                       const int* src_row, const bf16_t* h, const bf16_t* Wg, const bf16_t* Wu, bf16_t* act, int E,
                       int top_k, int Fe, int d, int tall_rows);
void launch_moe_down(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                     const bf16_t* act, const bf16_t* Wd, float* out, int E, int top_k, int Fe, int d, int tall_rows);

template <typename T>
void launch_rope_append(hipStream_t st, RowCtx rc, Slots s, const float* qkv, int n_partials,
                        size_t partial_stride, const float* rope_cos, const float* rope_sin,
                        float* q_rot, T* kv_pool, KVLayout kvl, int layer, int n_q_heads);

template <typename T, bool XF>
void launch_attn_ref(hipStream_t st, RowCtx rc, Slots s, const float* q_rot, const T* kv_pool,
                     KVLayout kvl, int layer, int n_q_heads, T* out);

// bf16 MFMA paged attention (KV layout mode 1).  Rows [row_base, row_base + rc.max_rows)
// of the row arrays.  A context longer than attn_split_tokens() is cut in KV splits of
// that fixed size, so a row's reduction order depends on its own length only; ws /
// counters: split workspace for rc.max_rows rows (counters zero on entry and on exit);
// max_splits <= 32.
int attn_split_tokens(int head_dim);
// fused_qkv != nullptr (decode iterations): the kernel also rotates q / the new key and
// appends the new key / value itself from the QKV GEMM's split-K partials (q_rot unused).
// items != nullptr (row_base 0, rows listed by launch_sched in this iteration): a 1-D launch of
// rc.max_rows * grid_splits * KV heads workgroups that takes its (row, split) from the work list.
void launch_attn_decode(hipStream_t st, RowCtx rc, int row_base, Slots s, const float* q_rot,
                        bf16_t* kv_pool, KVLayout kvl, int layer, int n_q_heads, bf16_t* out,
                        float* ws, int max_splits, int grid_splits,
                        const float* fused_qkv, int n_partials, size_t partial_stride,
                        const float* rope_cos, const float* rope_sin, const int4* items = nullptr);
// Causal attention over prefill rows, one workgroup per (item, KV head); an item = {slot, first
// row of the sequence in the row arrays, tokens of the sequence, first position of the tile},
// tiles of attn_prefill_tile(query heads per KV head) positions.  q_rot and the pages must hold
// the rotated queries / keys and the values of every row (launch_rope_append first).
int attn_prefill_tile(int group);
void launch_attn_prefill(hipStream_t st, const int4* items, int n_items, Slots s, const float* q_rot,
                         const bf16_t* kv_pool, KVLayout kvl, int layer, int n_q_heads, bf16_t* out);
// Merge of the KV-split partials (needed after launch_attn_decode whenever grid_splits > 1).
void launch_attn_merge(hipStream_t st, RowCtx rc, int row_base, KVLayout kvl, int n_q_heads, bf16_t* out,
                       const float* ws, int max_splits);

template <typename T, bool XF>
void launch_silu_mul(hipStream_t st, RowCtx rc, const float* gu, int F, T* act);

// out[m][n] = sum_k x[m][k] W[n][k]; plain row-major W; reference path.
template <typename T, bool XF>
void launch_gemm_ref(hipStream_t st, RowCtx rc, const T* x, const T* W, float* out, int N, int K);

// bf16 MFMA GEMM over fragment-tiled operands.  Wp: weights re-laid by
// launch_shuffle_weights.  out: fp32 [ksplit][m_cap][N] partial sums.
void launch_gemm_mfma(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out,
                      int N, int K, int ksplit, size_t partial_stride,
                      const float* ssq = nullptr, int ssq_stride = 0, float eps = 0.f);
// act[m][f] = silu(x.Wg[f]) * (x.Wu[f]) as fragment-tiled bf16.
// ssq != nullptr: the activations are residual * gain (not yet normalised); the kernel divides
// its accumulators by the row's RMS, from the sums of squares the producer left (see
// launch_gemm_mfma_resid).
void launch_gemm_mfma_swiglu(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg,
                             const bf16_t* Wu, bf16_t* act, int F, int K, const float* ssq = nullptr,
                             int ssq_stride = 0, float eps = 0.f);
void launch_gemm_mfma_resid(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* x_res,
                            const float* gain, bf16_t* act, float* ssq, int ssq_stride, int N, int K);
// LDS-tiled GEMM for tall activations (prefill); single pass over k, no partials.
void launch_gemm_tile(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K);
void launch_gemm_tile_swiglu(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                             bf16_t* act, int F, int K);
bool launch_gemm_tile_swiglu_chain(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                                   bf16_t* act, int F, int K, const float* ssq, int ssq_stride, float eps);
// Split-k partial-sum GEMM (qkv, down) for more than 128 rows on the LDS-tiled kernel with the skinny
// kernel's summation chains: out[slice][m][n], slices partial_stride floats apart.  Returns false
// (nothing launched) when the k slices do not fall on the kernel's stage boundaries.
bool launch_gemm_tile_chain_f32(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K,
                                int ksplit, size_t partial_stride);
void launch_gemm_tile_logits(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* logits,
                             float* group_max, int V, int K, int* group_idx = nullptr);
// LM head: logits fp32 [rows][V] plus, per row, the maximum of every group of
// lmhead_group_cols() consecutive logits (group_max [rows][V / group]); V % 64 == 0.
// group_idx (nullable, same shape): the column inside the group that holds the maximum, the
// lowest one on ties.  logits may be null: nothing but the group records is written then (all
// the greedy sampler needs).
int lmhead_group_cols();
void launch_gemm_mfma_logits(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* logits,
                             float* group_max, int V, int K, int* group_idx = nullptr);
void launch_shuffle_weights(hipStream_t st, const bf16_t* src, bf16_t* dst, int N, int K);

void launch_rope_table(hipStream_t st, float* cos_t, float* sin_t, int max_pos, int head_dim,
                       float theta);

// --- sampler + per-rollout state update ---------------------------------------
struct SamplerCfg {
  int kind, top_k;            // kind: 0 greedy, 1 top-k (+ nucleus), 2 categorical over the whole vocabulary
  float temperature;
  unsigned long long seed;
  float top_p;                // nucleus cut of the top-k candidates; >= 1: none
};
// Rows here are sampling rows: sample_row_slot / sample_row_pos give the slot and the
// position of the LAST fed token of each row.  update = 0: only write out_tokens
// (standalone sampler; req_ids/gen_idx arrays given explicitly).
// group_max (nullable): per row the maxima of groups of `group` consecutive logits, as
// written by launch_gemm_mfma_logits; lets the sampler look at a few groups only.
// out_logprobs (nullable, update = 0): log softmax(logits / temperature)[token]; with update = 1
// the log-probability goes to s.logprob when that array exists.
void launch_sample(hipStream_t st, RowCtx rc, Slots s, Ctrl* ctrl, const float* logits, int vocab,
                   SamplerCfg sc, Watch w, int update, const long long* req_ids,
                   const int* gen_idx, int* out_tokens, const float* group_max, int group,
                   float* out_logprobs = nullptr, const int* group_idx = nullptr);

void launch_group_max(hipStream_t st, const float* logits, int n_rows, int V, int group, float* out);

}  // namespace april
