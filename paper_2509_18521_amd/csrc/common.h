// Shared declarations of the APRIL rollout engine (device control block, slot
// table, layouts, launcher prototypes).  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace april {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Sequence slot states.
enum : int { SLOT_FREE = 0, SLOT_LIVE = 1, SLOT_DONE = 2, SLOT_PARKED = 3, SLOT_PREFILL = 4, SLOT_PREEMPTED = 5 };

// Device-resident control block of the early-termination scheduler (Section 2.2, second
// item of the method: the step ends as soon as N rollouts are complete; decided here, on device).
struct Ctrl {
  int n_rows;       // live rollouts of the current decode iteration   } read together by every
  int stop;         // 1: the step is over, every later kernel is a no-op } kernel as one int2
  int finished;     // rollouts complete in this step (surplus from the last step included)
  int n_target;     // N
  int iter;         // iterations executed so far in this step
  int stop_iter;    // iteration count at which stop was raised
  int free_top;     // free KV pages on the stack
  int error;        // 1: page stack underflow
  int n_slots;
  int eos_token;
  int n_watch;
  int inflight;     // rollouts in flight at the start of the step (bound on the page demand of an iteration)
  int n_preempted;  // rollouts preempted in this step because the KV pool ran out
  int pad1;
  long long sum_live;   // sum over iterations of n_rows
  long long sum_ctx;    // sum over (iteration, row) of context length
  long long iter_ctx;   // context-length sum of the current iteration alone
  long long sum_experts;  // sum over (iteration, layer) of the experts that received a token
};

// Per-slot state, structure of arrays in device memory.
struct Slots {
  long long* req_id;
  int* prompt_len;
  int* gen;           // generated tokens so far
  int* limit;         // completes when gen == limit
  int* state;
  int* kv_len;        // positions whose K/V are in the cache
  int* n_blocks;      // KV pages owned
  int* finish_iter;   // iteration of this step at which it completed
  int* block_table;   // [n_slots][max_blocks]
  int* tokens;        // [n_slots][max_ctx]: prompt, then generated tokens
  int* forced;        // [n_slots][max_ctx] teacher-forced generated tokens (-1: none), or null
  float* logprob;     // [n_slots][max_ctx] log-probability of generated token g at index g, or null
  int* group;         // [n_slots] index of the slot's group in grp_left for this step (-1: none), or null
  int* grp_left;      // [groups in flight] members of the group that are not complete yet
  int max_blocks;
  int max_ctx;
};

// Parity-mode capture of logits rows.
struct Watch {
  long long* req;     // [n_watch]
  int* first;         // [n_watch] first generated index kept
  int* count;         // [n_watch]
  int* row0;          // [n_watch] first row in `logits`
  float* logits;      // [rows][vocab]
  int* sampled;       // [rows] the sampler's own choice
  int* filled;        // [rows]
};

struct ModelDims {
  int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
  int n_experts, experts_per_tok, d_expert_ffn;
  float rope_theta, rms_eps;
  int blk;            // tokens per KV page
};

// ---------------------------------------------------------------------------
// Activation layouts.  Plain: row-major [row][K].  Fragment-tiled ("XF"): the
// operand layout of v_mfma_f32_32x32x16_bf16's 32(row) x 16(k) operand, so that one
// wavefront reads a whole fragment as 64 consecutive 16-byte pieces:
//   element (row, k) -> tile (row/32, k/16), lane = row%32 + 32*((k%16)/8), j = k%8
// ---------------------------------------------------------------------------
template <bool XF>
__host__ __device__ inline size_t act_index(int row, int k, int K) {
  if (XF) {
    size_t tile = (size_t)(row >> 5) * (size_t)(K >> 4) + (size_t)(k >> 4);
    int lane = (row & 31) + (((k & 15) >> 3) << 5);
    return (tile * 64 + lane) * 8 + (k & 7);
  } else {
    return (size_t)row * K + k;
  }
}

// KV cache addressing: pool[layer][k|v][page][kv_head][blk * head_dim elements].
// Inside one (page, head) block, mode 0 keeps [token][dim] for both K and V; mode 1
// (bf16 MFMA attention) keeps K in the A-operand order of v_mfma_f32_16x16x32_bf16
// ([dim/32][lane = token + 16*((dim%32)/8)][dim%8]) and V transposed ([dim][token]).
struct KVLayout {
  size_t layer_stride;   // elements between layers (covers k and v)
  size_t kv_stride;      // elements between the k part and the v part
  int n_kv_heads, head_dim, blk, mode;
  __host__ __device__ inline size_t at(int layer, int kv, int page, int head, int tok, int d) const {
    const size_t base = (size_t)layer * layer_stride + (size_t)kv * kv_stride +
                        ((size_t)page * n_kv_heads + head) * (size_t)(blk * head_dim);
    int inner;
    if (mode == 0) inner = tok * head_dim + d;
    else if (kv == 0) inner = ((((d >> 5) << 6) + tok + (((d & 31) >> 3) << 4)) << 3) + (d & 7);
    else inner = d * blk + tok;
    return base + inner;
  }
};

inline __host__ __device__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace april
