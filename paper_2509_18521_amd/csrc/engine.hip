// Host side of the APRIL rollout engine: C ABI, context, weights, KV pool, the
// rollout step (admission, prefill, decode loop, early termination, parking).
// Method: paper Section 2.2 (over-provisioned generation, early termination,
// buffering continuations, prioritized resumption).
#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "../../include/april.h"
#include "kernels.h"

using namespace april;

namespace {

thread_local std::string g_init_error;

double now_s() {
  return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

enum KernelClass {
  KC_SCHED = 0, KC_EMBED, KC_NORM, KC_GEMM_QKV, KC_ROPE, KC_ATTN, KC_GEMM_O, KC_GEMM_GATEUP, KC_SILU,
  KC_GEMM_DOWN, KC_GEMM_LMHEAD, KC_SAMPLE, KC_MOE_ROUTE, KC_MOE_GATEUP, KC_MOE_DOWN, KC_ATTN_MERGE, KC_EVENT_EMPTY, KC_EVENT_NONE, KC_COUNT
};
static_assert(KC_COUNT <= APRIL_KERNEL_CLASSES, "april_profile_get callers size their arrays with APRIL_KERNEL_CLASSES");
const char* kKernelNames[KC_COUNT] = {"sched", "embed", "add_rmsnorm", "gemm_qkv", "rope_append", "attn_decode",
                                      "gemm_o", "gemm_gateup", "silu_mul", "gemm_down", "gemm_lmhead", "sample",
                                      "moe_route", "moe_gateup", "moe_down", "attn_merge", "event_pair_empty_kernel", "event_pair_no_kernel"};

struct LayerW {
  float *attn_norm = nullptr, *mlp_norm = nullptr;
  void *wqkv = nullptr, *wo = nullptr, *wgu = nullptr, *wd = nullptr;            // plain [N][K]
  bf16_t *wqkv_s = nullptr, *wo_s = nullptr, *wg_s = nullptr, *wu_s = nullptr, *wd_s = nullptr;  // fragment-tiled
  bf16_t *router_s = nullptr, *eg_s = nullptr, *eu_s = nullptr, *ed_s = nullptr;  // routed experts, [E*rows][K] tiled
};

struct SlotH {
  int state = SLOT_FREE;
  long long req = -1;
  int prompt_len = 0, gen = 0, limit = 0, kv_len = 0, n_blocks = 0, n_resumes = 0;
  long long group = -1;          // input instance (n_samples_per_prompt > 1)
  std::vector<int> prompt;
  std::vector<int> forced;
};

struct Entry {
  long long req = -1;
  int slot = -1;                 // -1: token-level entry without a slot
  std::vector<int> prompt, generated;
  std::vector<float> logprobs;   // of `generated` (contexts that keep log-probabilities), token-level entries
  int limit = 0, n_resumes = 0, done = 0;
  long long group = -1;
};

}  // namespace

// Scratch of april_sample_rows_noalloc: staging of the row keys and of the result, the control
// word, and the group maxima the sampler's candidate search needs.  One copy per GPU, held
// until the process ends; host code only ever uses the device address looked up at april_init.
constexpr size_t NOALLOC_MAX_ROWS = 1024;
constexpr size_t NOALLOC_MAX_GROUP_MAX = (size_t)1 << 20;        // floats: n_rows * (vocab / 64) may not exceed this
constexpr size_t NOALLOC_OFF_CTL = 0, NOALLOC_OFF_REQ = 256, NOALLOC_OFF_GEN = NOALLOC_OFF_REQ + 8 * NOALLOC_MAX_ROWS,
                 NOALLOC_OFF_OUT = NOALLOC_OFF_GEN + 4 * NOALLOC_MAX_ROWS, NOALLOC_OFF_GM = NOALLOC_OFF_OUT + 4 * NOALLOC_MAX_ROWS,
                 NOALLOC_BYTES = NOALLOC_OFF_GM + 4 * NOALLOC_MAX_GROUP_MAX;
static_assert(NOALLOC_OFF_GM % 256 == 0, "group maxima start on a 256-byte boundary");
static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];
constexpr int MAX_DEVICES = 64;
static unsigned char* g_scratch_ptr[MAX_DEVICES];                // device address of `scratch` on each GPU, set by april_init

struct april_buffer {
  uint64_t magic = 0xA9B1FFEEull;
  std::vector<Entry> entries;
  bool alive = true;
};

struct ProfRec { int kc; hipEvent_t e0, e1; double bytes, flops; int snap; };

struct april_ctx {
  april_model_cfg cfg;
  ModelDims dm;
  hipStream_t stream = nullptr;
  bool own_stream = false;
  std::string err;
  bool bf16 = false, use_mfma = false;
  size_t esz = 4;

  // weights
  void* tok_emb = nullptr;
  std::vector<LayerW> layers;
  float* final_norm = nullptr;
  void* lm_head = nullptr;
  bf16_t* lm_head_s = nullptr;
  int64_t weight_bytes = 0, decode_weight_bytes = 0;
  std::vector<void*> allocs;

  // KV pool
  void* kv_pool = nullptr;
  KVLayout kvl;
  int n_pages = 0;
  int64_t kv_pool_bytes = 0, kv_bytes_per_token = 0;
  int free_pages_host = 0;

  // scheduler state
  int n_slots = 0, max_blocks = 0, max_ctx = 0;
  Slots ds;
  Ctrl* d_ctrl = nullptr;
  Ctrl* h_ctrl = nullptr;        // pinned
  int* d_free_stack = nullptr;
  int *d_row_slot = nullptr, *d_row_pos = nullptr;
  std::vector<SlotH> slots;
  Watch dwatch{};
  int watch_rows_cap = 0, watch_rows_used = 0, n_watch = 0, watch_cap = 2048;
  std::map<std::pair<long long, int>, int> watch_row_of;

  // prefill staging (device) + pinned host staging
  int prefill_cap = 0;
  int *d_pf_row_slot = nullptr, *d_pf_row_pos = nullptr, *d_pf_nrows = nullptr;
  int *d_pf_srow_slot = nullptr, *d_pf_srow_pos = nullptr, *d_pf_nsrows = nullptr, *d_pf_gather = nullptr;
  int4* d_pf_items = nullptr;    // query tiles of the chunk's sequences (prefill attention)
  int pf_n_items = 0, pf_items_cap = 0;
  bool prefill_tiled = true;     // query-tiled prefill attention (APRIL_PREFILL_ATTN=rows: one workgroup per row)
  int *d_list_a = nullptr, *d_list_b = nullptr;
  int* h_stage = nullptr;        // pinned
  size_t h_stage_ints = 0;
  int* h_slot_arrays = nullptr;  // pinned: mirrors for D2H/H2D of per-slot ints
  long long* h_req = nullptr;    // pinned

  // workspaces
  int m_cap = 0;
  float *x_res = nullptr, *qkv = nullptr, *q_rot = nullptr, *proj = nullptr, *gu = nullptr, *logits = nullptr;
  float* group_max = nullptr;  // per row, maxima of groups of lmhead_group_cols() logits (MFMA LM head)
  int* group_idx = nullptr;    // ... and the column of each maximum (greedy sampling without logits)
  bool write_logits = true;    // false: greedy sampling from the group records alone, the LM head writes no logits
  void *h_act = nullptr, *attn_out = nullptr, *act = nullptr, *hf = nullptr;
  float *rope_cos = nullptr, *rope_sin = nullptr;
  int s_qkv = 1, s_o = 1, s_down = 1;
  size_t qkv_stride = 0, proj_stride = 0;
  // bf16 MFMA attention: split-KV workspace
  bool attn_mfma = false, fuse_rope = true, tile_gemm = true, fuse_norm = true, fuse_down = false;
  bool moe_tile = true;         // prefill: expert GEMMs on the LDS-tiled kernel
  bool tile_f32 = true;         // decode above 128 rows: split-k projections on the LDS-tiled kernel
  bf16_t* h_rows = nullptr;     // plain [row][d] copy of the MLP input (routed experts, prefill)
  int moe_tall_rows = 2048;     // expert GEMMs: 4 m-tiles per workgroup from this row bound (prefill), 2 below
  int tile_decode_rows = 128;   // decode gate/up goes through the LDS-tiled kernel from this bound on the rows in flight (0 = never)
  float* ssq = nullptr;         // [d_model / 32][m_cap] per-row partial sums of squares (fused norm)
  int attn_chunk = 256, attn_max_splits = 1, attn_ws_rows = 0;
  int4* d_att_items = nullptr;   // work list of the decode attention, rebuilt by the scheduler kernel every iteration
  int att_items_cap = 0;         // entries beyond the header
  bool att_list = true;
  float* attn_ws = nullptr;
  int* d_dummy = nullptr;       // target of the empty kernel that calibrates event-pair timing
  int step_max_ctx = 0;        // bound on the context length of any row in the current pass
  // routed experts
  bool moe = false;
  int n_experts = 0, top_k_experts = 0, d_expert = 0, s_router = 1, moe_p_cap = 0;
  size_t router_stride = 0;
  float *router_out = nullptr, *moe_wts = nullptr, *moe_out = nullptr;
  int *moe_ids = nullptr, *moe_pos = nullptr, *moe_cnt = nullptr, *moe_base = nullptr, *moe_src = nullptr, *moe_group = nullptr;
  bf16_t* moe_act = nullptr;
  int64_t expert_bytes = 0;    // bytes of one expert's three matrices
  // one decode iteration (scheduler + forward + sample) captured as a HIP graph, keyed by
  // the launch geometry (row bound, attention split bound)
  bool use_graph = true;
  std::map<std::pair<int, int>, hipGraphExec_t> iter_graphs;
  std::vector<int> it_rows, it_gs, it_ctx;   // per-iteration bounds of the batch being enqueued
  int debug_fail_step = -1, debug_fail_iter = -1;   // APRIL_DEBUG_FAIL_AT=step:iteration, see april_rollout_step (one shot)
  int steps_started = 0;
  int graph_iters = 4;                       // iterations per replayed graph when consecutive ones share their bounds
                                             // (a graph boundary costs about 4 us on the device: 45.6 -> 45.7 k tokens/s)

  int weight_version = 0;        // bumped by april_update_weights
  // pausable memory (Section 3.3): allocations made while alloc_tag != 0 are virtual address
  // ranges with physical memory mapped behind them in chunks, so the memory can be handed back
  // and re-mapped at the same addresses
  struct VmRegion { char* va; size_t bytes; int tag; std::vector<hipMemGenericAllocationHandle_t> chunks; bool mapped; };
  std::vector<VmRegion> vm_regions;
  int alloc_tag = 0;
  size_t vm_granularity = 0;
  int paused_tags = 0;           // tags whose physical memory is released right now
  bool weights_valid = true;     // false between a resume of the weights' memory and the next april_update_weights
  int device = 0;                // HIP device the context lives on
  unsigned char* scratch_dev = nullptr;   // this device's copy of the static scratch array

  // pending resume
  std::vector<Entry> pending;
  bool have_pending = false;
  std::vector<april_buffer*> buffers;

  // result storage
  std::vector<long long> r_req;
  std::vector<std::vector<int>> r_tokens;
  std::vector<const int32_t*> r_tok_ptrs;
  std::vector<int> r_ntok, r_nres;
  std::vector<long long> r_group;
  std::vector<std::vector<float>> r_logprobs;
  std::vector<const float*> r_lp_ptrs;
  std::vector<std::vector<int>> export_store;

  // profiling
  int prof_every = 0;
  std::vector<ProfRec> prof_recs;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev_pool;
  size_t ev_used = 0;
  Ctrl* h_snaps = nullptr;       // pinned ring
  int snaps_cap = 0, snaps_used = 0;
  april_kernel_stat stats[KC_COUNT];
  bool prof_now = false;
  int prof_snap = -1;
};

namespace {

int fail(april_ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_init_error = buf;
  return code;
}

#define HIPCHK(c, expr)                                                                       \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(c, APRIL_EDEVICE, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

constexpr size_t VM_CHUNK = (size_t)1 << 30;      // physical memory is created and mapped in pieces of this size

// Physical memory behind a region: create, map at the region's address, allow access.
int vm_map_region(april_ctx* c, april_ctx::VmRegion& r) {
  hipMemAllocationProp prop{};
  prop.type = hipMemAllocationTypePinned;
  prop.location.type = hipMemLocationTypeDevice;
  prop.location.id = c->device;
  hipMemAccessDesc acc{};
  acc.location = prop.location;
  acc.flags = hipMemAccessFlagsProtReadWrite;
  for (size_t off = 0; off < r.bytes; off += VM_CHUNK) {
    const size_t n = std::min(VM_CHUNK, r.bytes - off);
    hipMemGenericAllocationHandle_t h;
    hipError_t e = hipMemCreate(&h, n, &prop, 0);
    if (e != hipSuccess) return fail(c, APRIL_ENOMEM, "hipMemCreate(%zu bytes) failed: %s", n, hipGetErrorString(e));
    e = hipMemMap(r.va + off, n, 0, h, 0);
    if (e != hipSuccess) { hipMemRelease(h); return fail(c, APRIL_EDEVICE, "hipMemMap failed: %s", hipGetErrorString(e)); }
    r.chunks.push_back(h);
  }
  // One call for the whole range: set per piece, the call is refused (invalid argument) for a
  // last piece that is smaller than the ones before it.
  const hipError_t e = hipMemSetAccess(r.va, r.bytes, &acc, 1);
  if (e != hipSuccess)
    return fail(c, APRIL_EDEVICE, "hipMemSetAccess(%zu-byte region) failed: %s", r.bytes, hipGetErrorString(e));
  r.mapped = true;
  return APRIL_OK;
}
// Hand the physical memory of a region back; the address range stays reserved.
void vm_unmap_region(april_ctx::VmRegion& r) {
  size_t off = 0;
  for (auto h : r.chunks) {
    const size_t n = std::min(VM_CHUNK, r.bytes - off);
    hipMemUnmap(r.va + off, n);
    hipMemRelease(h);
    off += n;
  }
  r.chunks.clear();
  r.mapped = false;
}
int vm_alloc(april_ctx* c, void** p, size_t bytes, int tag) {
  if (c->vm_granularity == 0) {
    hipMemAllocationProp prop{};
    prop.type = hipMemAllocationTypePinned;
    prop.location.type = hipMemLocationTypeDevice;
    prop.location.id = c->device;
    size_t g = 0;
    hipError_t e = hipMemGetAllocationGranularity(&g, &prop, hipMemAllocationGranularityRecommended);
    if (e != hipSuccess || g == 0) return fail(c, APRIL_EDEVICE, "hipMemGetAllocationGranularity failed: %s", hipGetErrorString(e));
    if (VM_CHUNK % g) return fail(c, APRIL_EDEVICE, "allocation granularity %zu does not divide the chunk size", g);
    c->vm_granularity = g;
  }
  const size_t rounded = (bytes + c->vm_granularity - 1) / c->vm_granularity * c->vm_granularity;
  void* va = nullptr;
  hipError_t e = hipMemAddressReserve(&va, rounded, c->vm_granularity, nullptr, 0);
  if (e != hipSuccess) return fail(c, APRIL_ENOMEM, "hipMemAddressReserve(%zu bytes) failed: %s", rounded, hipGetErrorString(e));
  c->vm_regions.push_back({(char*)va, rounded, tag, {}, false});
  int rc = vm_map_region(c, c->vm_regions.back());
  if (rc != APRIL_OK) return rc;
  *p = va;
  return APRIL_OK;
}

template <typename T>
int dev_alloc(april_ctx* c, T** p, size_t n_elems, bool zero = true) {
  void* q = nullptr;
  size_t bytes = std::max<size_t>(n_elems * sizeof(T), 256);
  if (c->alloc_tag != 0) {
    int rc = vm_alloc(c, &q, bytes, c->alloc_tag);
    if (rc != APRIL_OK) return rc;
    if (zero && hipMemsetAsync(q, 0, bytes, c->stream) != hipSuccess) return fail(c, APRIL_EDEVICE, "hipMemsetAsync failed");
    *p = reinterpret_cast<T*>(q);
    return APRIL_OK;
  }
  hipError_t e = hipMalloc(&q, bytes);
  if (e != hipSuccess) return fail(c, APRIL_ENOMEM, "hipMalloc(%zu bytes) failed: %s", bytes, hipGetErrorString(e));
  if (zero) {
    e = hipMemsetAsync(q, 0, bytes, c->stream);
    if (e != hipSuccess) return fail(c, APRIL_EDEVICE, "hipMemsetAsync failed: %s", hipGetErrorString(e));
  }
  c->allocs.push_back(q);
  *p = reinterpret_cast<T*>(q);
  return APRIL_OK;
}
int dev_alloc_bytes(april_ctx* c, void** p, size_t bytes, bool zero = true) {
  char* q = nullptr;
  int rc = dev_alloc<char>(c, &q, bytes, zero);
  *p = q;
  return rc;
}

const april_tensor* find_tensor(const april_tensor* w, int n, const std::string& name) {
  for (int i = 0; i < n; ++i)
    if (w[i].name && name == w[i].name) return &w[i];
  return nullptr;
}

// Copy a named tensor (host or device source) to dst (device).
int fetch_tensor(april_ctx* c, const april_tensor* w, int n, const std::string& name, void* dst, size_t bytes) {
  const april_tensor* t = find_tensor(w, n, name);
  if (!t) return fail(c, APRIL_EINVAL, "weight tensor '%s' missing", name.c_str());
  if ((size_t)t->nbytes != bytes)
    return fail(c, APRIL_EINVAL, "weight tensor '%s': %lld bytes given, %zu expected", name.c_str(),
                (long long)t->nbytes, bytes);
  HIPCHK(c, hipMemcpyAsync(dst, t->data, bytes, t->on_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice,
                           c->stream));
  if (!t->on_device) HIPCHK(c, hipStreamSynchronize(c->stream));   // the caller's buffer is only borrowed
  return APRIL_OK;
}

// Copy every weight tensor to the device in the layout the kernels want.  First call (from
// april_init): allocates the buffers.  Later calls (april_update_weights): the same buffers are
// overwritten in place, so captured iteration graphs stay valid.
int load_weights(april_ctx* c, const april_tensor* weights, int n_weights) {
  const april_model_cfg& g = c->cfg;
  const bool moe = c->moe, first = c->layers.empty();
  const int nq = g.n_q_heads * g.head_dim, nkv = g.n_kv_heads * g.head_dim, nqkv = nq + 2 * nkv;
  const int d = g.d_model, F = g.d_ffn, V = g.vocab;
  const size_t e = c->esz;
  // staging buffer for one matrix at a time: the largest of every matrix that goes through it
  size_t stage_bytes = std::max({(size_t)V * d, (size_t)F * d, (size_t)nqkv * d, (size_t)d * nq}) * e;
  if (moe) stage_bytes = std::max({stage_bytes, (size_t)g.n_experts * g.d_expert_ffn * d * e, (size_t)g.n_experts * d * e});
  void* stage = nullptr;
  if (c->use_mfma && hipMalloc(&stage, stage_bytes) != hipSuccess) return fail(c, APRIL_ENOMEM, "staging buffer for the weights (%zu bytes)", stage_bytes);
  struct StageGuard { void*& p; ~StageGuard() { if (p) hipFree(p); p = nullptr; } } guard{stage};
#define TRYW(x) do { int rc_ = (x); if (rc_ != APRIL_OK) return rc_; } while (0)
  // allocate on the first call only
  auto walloc = [&](void** p, size_t bytes) -> int { return *p ? APRIL_OK : dev_alloc_bytes(c, p, bytes, false); };
  auto wallocf = [&](float** p, size_t n) -> int { return *p ? APRIL_OK : dev_alloc(c, p, n, false); };
  auto wallocb = [&](bf16_t** p, size_t n) -> int { return *p ? APRIL_OK : dev_alloc(c, p, n, false); };

  TRYW(walloc(&c->tok_emb, (size_t)V * d * e));
  TRYW(fetch_tensor(c, weights, n_weights, "tok_emb", c->tok_emb, (size_t)V * d * e));
  TRYW(wallocf(&c->final_norm, d));
  TRYW(fetch_tensor(c, weights, n_weights, "final_norm", c->final_norm, d * sizeof(float)));
  if (first) {
    c->weight_bytes = (int64_t)V * d * e;
    c->decode_weight_bytes = 0;
    c->layers.resize(g.n_layers);
  }
  const bool keep_plain = !c->use_mfma;
  // Fetch a matrix into `plain` (kept) or into the staging buffer, and re-lay it for MFMA.
  auto load_matrix = [&](const std::string& name, int N, int K, void* plain_dst, bf16_t** shuffled) -> int {
    void* dstp = keep_plain ? plain_dst : stage;
    int rc = fetch_tensor(c, weights, n_weights, name, dstp, (size_t)N * K * e);
    if (rc != APRIL_OK) return rc;
    if (c->use_mfma && shuffled) {
      rc = wallocb(shuffled, (size_t)N * K);
      if (rc != APRIL_OK) return rc;
      launch_shuffle_weights(c->stream, (const bf16_t*)dstp, *shuffled, N, K);
      HIPCHK(c, hipStreamSynchronize(c->stream));
    }
    return APRIL_OK;
  };
  for (int l = 0; l < g.n_layers; ++l) {
    LayerW& L = c->layers[l];
    const std::string sl = "." + std::to_string(l);
    TRYW(wallocf(&L.attn_norm, d));
    TRYW(wallocf(&L.mlp_norm, d));
    TRYW(fetch_tensor(c, weights, n_weights, "attn_norm" + sl, L.attn_norm, d * sizeof(float)));
    TRYW(fetch_tensor(c, weights, n_weights, "mlp_norm" + sl, L.mlp_norm, d * sizeof(float)));
    // q, k, v concatenated along the output dimension
    void* qkv_dst = nullptr;
    if (keep_plain) { TRYW(walloc(&L.wqkv, (size_t)nqkv * d * e)); qkv_dst = L.wqkv; }
    else qkv_dst = stage;
    TRYW(fetch_tensor(c, weights, n_weights, "wq" + sl, qkv_dst, (size_t)nq * d * e));
    TRYW(fetch_tensor(c, weights, n_weights, "wk" + sl, (char*)qkv_dst + (size_t)nq * d * e, (size_t)nkv * d * e));
    TRYW(fetch_tensor(c, weights, n_weights, "wv" + sl, (char*)qkv_dst + (size_t)(nq + nkv) * d * e, (size_t)nkv * d * e));
    if (c->use_mfma) {
      TRYW(wallocb(&L.wqkv_s, (size_t)nqkv * d));
      launch_shuffle_weights(c->stream, (const bf16_t*)qkv_dst, L.wqkv_s, nqkv, d);
      HIPCHK(c, hipStreamSynchronize(c->stream));
    }
    if (moe) {
      const int E = g.n_experts, Fe = g.d_expert_ffn;
      TRYW(load_matrix("wo" + sl, d, nq, nullptr, &L.wo_s));
      TRYW(load_matrix("router" + sl, E, d, nullptr, &L.router_s));
      TRYW(load_matrix("e_gate" + sl, E * Fe, d, nullptr, &L.eg_s));
      TRYW(load_matrix("e_up" + sl, E * Fe, d, nullptr, &L.eu_s));
      TRYW(load_matrix("e_down" + sl, E * d, Fe, nullptr, &L.ed_s));
      if (first) {
        c->decode_weight_bytes += ((int64_t)nqkv * d + (int64_t)d * nq + (int64_t)E * d) * e + 2 * d * 4;
        c->weight_bytes += (int64_t)3 * E * Fe * d * e;
      }
      continue;
    }
    if (keep_plain) {
      TRYW(walloc(&L.wo, (size_t)d * nq * e));
      TRYW(walloc(&L.wgu, (size_t)2 * F * d * e));
      TRYW(walloc(&L.wd, (size_t)d * F * e));
      TRYW(load_matrix("wo" + sl, d, nq, L.wo, nullptr));
      TRYW(load_matrix("w_gate" + sl, F, d, L.wgu, nullptr));
      TRYW(load_matrix("w_up" + sl, F, d, (char*)L.wgu + (size_t)F * d * e, nullptr));
      TRYW(load_matrix("w_down" + sl, d, F, L.wd, nullptr));
    } else {
      TRYW(load_matrix("wo" + sl, d, nq, nullptr, &L.wo_s));
      TRYW(load_matrix("w_gate" + sl, F, d, nullptr, &L.wg_s));
      TRYW(load_matrix("w_up" + sl, F, d, nullptr, &L.wu_s));
      TRYW(load_matrix("w_down" + sl, d, F, nullptr, &L.wd_s));
    }
    if (first) c->decode_weight_bytes += ((int64_t)nqkv * d + (int64_t)d * nq + (int64_t)3 * F * d) * e + 2 * d * 4;
  }
  if (keep_plain) {
    TRYW(walloc(&c->lm_head, (size_t)V * d * e));
    TRYW(load_matrix("lm_head", V, d, c->lm_head, nullptr));
  } else {
    TRYW(load_matrix("lm_head", V, d, nullptr, &c->lm_head_s));
  }
  if (first) {
    c->decode_weight_bytes += (int64_t)V * d * e + d * 4;
    c->weight_bytes += c->decode_weight_bytes;
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));
#undef TRYW
  return APRIL_OK;
}

// Cross-workgroup k-split of a projection GEMM: enough workgroups to occupy the chip when
// there are few n-tiles, none when the n-tiles alone do; a function of (N, K) only, so a
// row's summation order never depends on the batch.
int pick_ksplit(int N, int K) {
  const int n_tiles = N / 32, KT = K / 16;
  int s = std::min(KT / 12, 384 / std::max(n_tiles, 1));
  // Large matrices run two n-tiles per workgroup: as many k slices as bring the launch closest
  // to one workgroup per compute unit (256) from below.  Measured at 64 / 128 rows: a 2560 x 9728
  // down projection 20.2 / 23.6 us with 4 slices (160 workgroups), 15.8 / 21.0 us with 6 (240);
  // 4096 x 14336: 33.3 / 42.0 us with 3 (192), 27.6 / 36.3 us with 4 (256).
  if ((long long)N * K >= (8ll << 20) && n_tiles % 2 == 0 && n_tiles / 2 <= 256) s = std::min(KT / 12, 256 / (n_tiles / 2));
  if (s < 1) s = 1;
  if (s > 8) s = 8;
  return s;
}

// ---- profiling helpers -------------------------------------------------------
struct ProfScope {
  april_ctx* c; int idx;
  ProfScope(april_ctx* c_, int kc, double bytes, double flops) : c(c_), idx(-1) {
    if (!c->prof_now) return;
    if (c->ev_used == c->ev_pool.size()) {
      hipEvent_t a, b;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return;
      c->ev_pool.push_back({a, b});
    }
    auto& ev = c->ev_pool[c->ev_used++];
    c->prof_recs.push_back({kc, ev.first, ev.second, bytes, flops, c->prof_snap});
    idx = (int)c->prof_recs.size() - 1;
    hipEventRecord(ev.first, c->stream);
  }
  ~ProfScope() {
    if (idx >= 0) hipEventRecord(c->prof_recs[idx].e1, c->stream);
  }
};

void prof_collect(april_ctx* c) {   // stream must be idle
  for (auto& r : c->prof_recs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) continue;
    double bytes = r.bytes, flops = r.flops;
    auto& st = c->stats[r.kc];
    st.launches += 1;
    st.total_ms += ms;
    st.alg_bytes += bytes;
    st.alg_flops += flops;
  }
  c->prof_recs.clear();
  c->ev_used = 0;
  c->snaps_used = 0;
}

SamplerCfg sampler_cfg(const april_ctx* c) {
  const float T = c->cfg.temperature > 0.f ? c->cfg.temperature : 1.0f;
  const float tp = (c->cfg.top_p > 0.f && c->cfg.top_p < 1.f) ? c->cfg.top_p : 1.0f;
  return SamplerCfg{c->cfg.sampler, c->cfg.top_k, T, (unsigned long long)c->cfg.seed, tp};
}

// ---- forward pass --------------------------------------------------------------
// rows: the tokens fed; srows: the rows that are sampled (decode: the same rows;
// prefill: the last token of each sequence, `gather` maps them into `rows`).
// B / C: host estimates of live rows and summed context, used only for the
// algorithmic-byte bookkeeping of profiled launches.
void forward(april_ctx* c, RowCtx rows, RowCtx srows, const int* gather, double B, double C) {
  const ModelDims& m = c->dm;
  hipStream_t st = c->stream;
  const int d = m.d_model, dh = m.head_dim, Hq = m.n_q_heads, Hkv = m.n_kv_heads, F = m.d_ffn, V = m.vocab;
  const int nq = Hq * dh, nkv = Hkv * dh, nqkv = nq + 2 * nkv;
  const double e = (double)c->esz;
  {
    ProfScope p(c, KC_EMBED, B * d * (e + 4), 0);
    if (c->bf16) launch_embed<bf16_t>(st, rows, c->ds, (const bf16_t*)c->tok_emb, c->x_res, d);
    else launch_embed<float>(st, rows, c->ds, (const float*)c->tok_emb, c->x_res, d);
  }
  // mlp_in = true: the partials are the previous layer's MLP output (for routed experts: the
  // top-k expert outputs of each row, gathered and weighted)
  auto norm = [&](RowCtx rc, int n_part, const float* gain, void* out, const int* gth, double rowsB, bool mlp_in,
                  bf16_t* out_rows = nullptr) {
    ProfScope p(c, KC_NORM, rowsB * d * (4.0 * (2 + (n_part > 0 ? 1 : 0)) + e), 0);
    if (c->moe && mlp_in && n_part > 0)
      launch_add_rmsnorm<bf16_t, true>(st, rc, c->x_res, c->moe_out, c->top_k_experts, 0, gain, (bf16_t*)out, d, m.rms_eps, gth, c->moe_pos, c->moe_wts);
    else if (c->bf16) launch_add_rmsnorm<bf16_t, true>(st, rc, c->x_res, c->proj, n_part, c->proj_stride, gain, (bf16_t*)out, d, m.rms_eps, gth, nullptr, nullptr, out_rows);
    else launch_add_rmsnorm<float, false>(st, rc, c->x_res, c->proj, n_part, c->proj_stride, gain, (float*)out, d, m.rms_eps, gth);
  };
  // Prefill rows (hundreds to thousands) go through the LDS-tiled GEMM, which needs no k-split
  // across workgroups: its consumers then read a single partial.  The choice follows the kind
  // of pass, never the number of rows, so a rollout's arithmetic does not depend on the batch.
  const bool tile = c->use_mfma && c->tile_gemm && gather != nullptr;
  const int sq = tile ? 1 : c->s_qkv, so = tile ? 1 : c->s_o, sd = tile ? 1 : c->s_down, sr = tile ? 1 : c->s_router;
  auto gemm = [&](int kc, RowCtx rc, const void* x, const void* w_plain, const bf16_t* w_s, float* out, int N, int K,
                  int ks, size_t stride, double rowsB, const float* ssq = nullptr) {
    ProfScope p(c, kc, (double)N * K * e + rowsB * K * e + rowsB * N * 4.0, 2.0 * rowsB * N * K);
    if (tile) launch_gemm_tile(st, rc, (const bf16_t*)x, w_s, out, N, K);
    else if (c->use_mfma && c->tile_f32 && rc.max_rows > 128 && ssq == nullptr && N >= 1024 && (N / 64) * ks >= 128 &&
             K / ks >= 3072 && launch_gemm_tile_chain_f32(st, rc, (const bf16_t*)x, w_s, out, N, K, ks, stride)) {
      // decode with more than 128 rows, wide matrix, long k slices: LDS-tiled kernel with the skinny
      // kernel's chains.  Measured at 230 rows: the 4096 x 14336 down projection (4 slices of
      // 3584) 57.4 us against 62.4 us; qkv projections with slices of 1280 / 2048 are slower
      // there (18.1 against 16.4 us, 34.2 against 30.4 us), hence the bound on the slice length.
    }
    else if (c->use_mfma) launch_gemm_mfma(st, rc, (const bf16_t*)x, w_s, out, N, K, ks, stride, ssq, (int)c->m_cap, m.rms_eps);
    else if (c->bf16) launch_gemm_ref<bf16_t, true>(st, rc, (const bf16_t*)x, (const bf16_t*)w_plain, out, N, K);
    else launch_gemm_ref<float, false>(st, rc, (const float*)x, (const float*)w_plain, out, N, K);
  };
  bool normed_by_down = false;       // the previous layer's down projection already did this layer's first norm
  for (int l = 0; l < m.n_layers; ++l) {
    const LayerW& L = c->layers[l];
    if (!normed_by_down) norm(rows, l == 0 ? 0 : sd, L.attn_norm, c->h_act, nullptr, B, true);
    gemm(KC_GEMM_QKV, rows, c->h_act, L.wqkv, L.wqkv_s, c->qkv, nqkv, d, sq, c->qkv_stride, B,
         normed_by_down ? c->ssq : nullptr);
    normed_by_down = false;
    // decode iterations: rotary + KV append are done inside the attention kernel
    const bool fuse_rope = c->attn_mfma && c->fuse_rope && gather == nullptr;
    if (!fuse_rope) {
      ProfScope p(c, KC_ROPE, B * (nqkv * 4.0 + nq * 4.0 + 2 * nkv * e), 0);
      if (c->bf16) launch_rope_append<bf16_t>(st, rows, c->ds, c->qkv, sq, c->qkv_stride, c->rope_cos, c->rope_sin, c->q_rot, (bf16_t*)c->kv_pool, c->kvl, l, Hq);
      else launch_rope_append<float>(st, rows, c->ds, c->qkv, sq, c->qkv_stride, c->rope_cos, c->rope_sin, c->q_rot, (float*)c->kv_pool, c->kvl, l, Hq);
    }
    if (c->attn_mfma && gather != nullptr && c->prefill_tiled) {
      // prefill: one workgroup per tile of query positions, the keys / values of a prompt are
      // streamed once per tile instead of once per row
      ProfScope p(c, KC_ATTN, C * 2.0 * nkv * e + B * nq * (4.0 + e), 4.0 * C * nq);
      launch_attn_prefill(st, c->d_pf_items, c->pf_n_items, c->ds, c->q_rot, (const bf16_t*)c->kv_pool, c->kvl, l, Hq,
                          (bf16_t*)c->attn_out);
    } else if (c->attn_mfma) {
      const int gs = std::min(c->attn_max_splits, std::max(1, ceil_div(c->step_max_ctx, c->attn_chunk)));
      for (int base = 0; base < rows.max_rows; base += c->attn_ws_rows) {
        RowCtx sub = rows;
        sub.max_rows = std::min(c->attn_ws_rows, rows.max_rows - base);
        {
          ProfScope p(c, KC_ATTN, C * 2.0 * nkv * e + B * nq * (4.0 + e), 4.0 * C * nq);
          launch_attn_decode(st, sub, base, c->ds, c->q_rot, (bf16_t*)c->kv_pool, c->kvl, l, Hq,
                             (bf16_t*)c->attn_out, c->attn_ws, c->attn_max_splits, gs,
                             fuse_rope ? c->qkv : nullptr, sq, c->qkv_stride, c->rope_cos, c->rope_sin,
                             fuse_rope && c->att_list && rows.max_rows <= c->attn_ws_rows ? c->d_att_items : nullptr);
        }
        if (gs > 1) {      // some row may span several KV splits: merge their partial results
          ProfScope p(c, KC_ATTN_MERGE, 0, 0);
          launch_attn_merge(st, sub, base, c->kvl, Hq, (bf16_t*)c->attn_out, c->attn_ws, c->attn_max_splits);
        }
      }
    } else {
      ProfScope p(c, KC_ATTN, C * 2.0 * nkv * e + B * nq * (4.0 + e), 4.0 * C * nq);
      if (c->bf16) launch_attn_ref<bf16_t, true>(st, rows, c->ds, c->q_rot, (const bf16_t*)c->kv_pool, c->kvl, l, Hq, (bf16_t*)c->attn_out);
      else launch_attn_ref<float, false>(st, rows, c->ds, c->q_rot, (const float*)c->kv_pool, c->kvl, l, Hq, (float*)c->attn_out);
    }
    // decode, dense MLP: the output projection adds into the residual stream itself and hands the
    // gate/up GEMM un-normalised activations plus per-row sums of squares (no norm launch)
    const bool fuse_norm2 = c->use_mfma && c->fuse_norm && !tile && !c->moe;
    if (fuse_norm2) {
      ProfScope p(c, KC_GEMM_O, (double)d * nq * e + B * nq * e + B * d * (8.0 + e), 2.0 * B * d * nq);
      launch_gemm_mfma_resid(st, rows, (const bf16_t*)c->attn_out, L.wo_s, c->x_res, L.mlp_norm, (bf16_t*)c->h_act,
                             c->ssq, c->m_cap, d, nq);
    } else {
      gemm(KC_GEMM_O, rows, c->attn_out, L.wo, L.wo_s, c->proj, d, nq, so, c->proj_stride, B);
      // (routed experts in prefill gather token rows: they get a plain [row][d] copy as well)
      norm(rows, so, L.mlp_norm, c->h_act, nullptr, B, false, c->moe && tile && c->moe_tile ? c->h_rows : nullptr);
    }
    if (c->moe) {
      const int E = c->n_experts, Fe = c->d_expert, tk = c->top_k_experts;
      gemm(KC_MOE_ROUTE, rows, c->h_act, nullptr, L.router_s, c->router_out, E, d, sr, c->router_stride, B);
      launch_moe_route(st, rows, c->router_out, sr, c->router_stride, E, tk, c->moe_ids, c->moe_wts);
      // prefill: LDS-tiled expert GEMMs over row groups of 128 packed rows (the dispatch aligns the
      // expert segments to what the GEMM workgroups cover: same bound to all three launches)
      const bool moe_tiled = tile && c->moe_tile;
      const int tall = moe_tiled ? 1 : c->moe_tall_rows;
      const int n_groups = moe_group_count(rows.max_rows, tk, E, moe_tile_rows());
      launch_moe_dispatch(st, rows, c->moe_ids, E, tk, c->moe_cnt, c->moe_base, c->moe_pos, c->moe_src, c->moe_p_cap,
                          rows.ctl == reinterpret_cast<const int2*>(c->d_ctrl) ? c->d_ctrl : nullptr, tall,
                          c->moe_group);
      const double hit = std::min<double>(E, B * tk);   // bookkeeping estimate: experts that receive a token
      {
        ProfScope p(c, KC_MOE_GATEUP, hit * 2.0 * Fe * d * e + B * tk * (d + Fe) * e, 4.0 * B * tk * Fe * d);
        if (!(moe_tiled && launch_moe_tile_gateup(st, rows, c->moe_cnt, c->moe_base, c->moe_group, c->moe_src, c->h_rows,
                                                  L.eg_s, L.eu_s, c->moe_act, Fe, d, n_groups)))
          launch_moe_gateup(st, rows, c->moe_cnt, c->moe_base, c->moe_group, c->moe_src, (const bf16_t*)c->h_act, L.eg_s, L.eu_s, c->moe_act, E, tk, Fe, d, tall);
      }
      {
        ProfScope p(c, KC_MOE_DOWN, hit * 1.0 * Fe * d * e + B * tk * (Fe * e + d * 4.0), 2.0 * B * tk * Fe * d);
        if (!(moe_tiled && launch_moe_tile_down(st, rows, c->moe_cnt, c->moe_base, c->moe_group, c->moe_act, L.ed_s, c->moe_out, Fe, d, n_groups)))
          launch_moe_down(st, rows, c->moe_cnt, c->moe_base, c->moe_group, c->moe_act, L.ed_s, c->moe_out, E, tk, Fe, d, tall);
      }
      continue;
    }
    if (c->use_mfma) {
      ProfScope p(c, KC_GEMM_GATEUP, 2.0 * F * d * e + B * d * e + B * F * e, 4.0 * B * F * d);
      if (tile) launch_gemm_tile_swiglu(st, rows, (const bf16_t*)c->h_act, L.wg_s, L.wu_s, (bf16_t*)c->act, F, d);
      else if (c->tile_decode_rows > 0 && rows.max_rows >= c->tile_decode_rows &&
               launch_gemm_tile_swiglu_chain(st, rows, (const bf16_t*)c->h_act, L.wg_s, L.wu_s, (bf16_t*)c->act, F, d,
                                             fuse_norm2 ? c->ssq : nullptr, c->m_cap, m.rms_eps)) {
        // many rows in flight: LDS-tiled kernel, same summation chains as the skinny one
      } else launch_gemm_mfma_swiglu(st, rows, (const bf16_t*)c->h_act, L.wg_s, L.wu_s, (bf16_t*)c->act, F, d,
                                   fuse_norm2 ? c->ssq : nullptr, c->m_cap, m.rms_eps);
    } else {
      gemm(KC_GEMM_GATEUP, rows, c->h_act, L.wgu, nullptr, c->gu, 2 * F, d, 1, 0, B);
      ProfScope p(c, KC_SILU, B * F * (8.0 + e), 0);
      if (c->bf16) launch_silu_mul<bf16_t, true>(st, rows, c->gu, F, (bf16_t*)c->act);
      else launch_silu_mul<float, false>(st, rows, c->gu, F, (float*)c->act);
    }
    if (fuse_norm2 && c->fuse_down && l + 1 < m.n_layers) {
      // same folding for the next layer's first norm (the last layer keeps the split-k form: the
      // final norm gathers rows and feeds the LM head)
      ProfScope p(c, KC_GEMM_DOWN, (double)d * F * e + B * F * e + B * d * (8.0 + e), 2.0 * B * d * F);
      launch_gemm_mfma_resid(st, rows, (const bf16_t*)c->act, L.wd_s, c->x_res, c->layers[l + 1].attn_norm,
                             (bf16_t*)c->h_act, c->ssq, c->m_cap, d, F);
      normed_by_down = true;
    } else {
      gemm(KC_GEMM_DOWN, rows, c->act, L.wd, L.wd_s, c->proj, d, F, sd, c->proj_stride, B);
    }
  }
  const double SB = gather ? (double)srows.max_rows : B;
  norm(srows, sd, c->final_norm, c->hf, gather, SB, true);
  float* lg_out = c->write_logits ? c->logits : nullptr;
  {
    ProfScope p(c, KC_GEMM_LMHEAD, (double)V * d * e + SB * d * e, 2.0 * SB * V * d);
    // more than 128 sampling rows: the tiled kernel reads the head once per 256 rows instead of
    // once per 128 (same bits either way)
    if (c->use_mfma && c->group_max && c->tile_gemm && srows.max_rows > 128 && d % 32 == 0)
      launch_gemm_tile_logits(st, srows, (const bf16_t*)c->hf, c->lm_head_s, lg_out, c->group_max, V, d, c->group_idx);
    else if (c->use_mfma && c->group_max) launch_gemm_mfma_logits(st, srows, (const bf16_t*)c->hf, c->lm_head_s, lg_out, c->group_max, V, d, c->group_idx);
    else if (c->use_mfma) launch_gemm_mfma(st, srows, (const bf16_t*)c->hf, c->lm_head_s, c->logits, V, d, 1, 0);
    else if (c->bf16) launch_gemm_ref<bf16_t, true>(st, srows, (const bf16_t*)c->hf, (const bf16_t*)c->lm_head, c->logits, V, d);
    else launch_gemm_ref<float, false>(st, srows, (const float*)c->hf, (const float*)c->lm_head, c->logits, V, d);
  }
  {
    const bool fused = c->group_max && !c->write_logits;
    ProfScope p(c, KC_SAMPLE, fused ? SB * (V / 64) * 8.0 : SB * V * 4.0, 0);
    const SamplerCfg sc = sampler_cfg(c);
    Watch w = c->cfg.debug_logits ? c->dwatch : Watch{};
    launch_sample(st, srows, c->ds, c->d_ctrl, c->logits, V, sc, w, 1, nullptr, nullptr, nullptr, c->group_max,
                  lmhead_group_cols(), nullptr, c->group_max ? c->group_idx : nullptr);
  }
}

int alloc_slot(april_ctx* c) {
  for (int i = 0; i < c->n_slots; ++i)
    if (c->slots[i].state == SLOT_FREE) return i;
  return -1;
}

int upload_slot_tables(april_ctx* c) {
  // host mirrors are authoritative between steps
  const int S = c->n_slots;
  int* a = c->h_slot_arrays;
  for (int i = 0; i < S; ++i) {
    const SlotH& s = c->slots[i];
    a[0 * S + i] = s.prompt_len; a[1 * S + i] = s.gen; a[2 * S + i] = s.limit;
    a[3 * S + i] = s.state; a[4 * S + i] = s.kv_len; a[5 * S + i] = s.n_blocks;
    a[6 * S + i] = 0;
    c->h_req[i] = s.req;
  }
  int* dst[7] = {c->ds.prompt_len, c->ds.gen, c->ds.limit, c->ds.state, c->ds.kv_len, c->ds.n_blocks, c->ds.finish_iter};
  for (int k = 0; k < 7; ++k)
    HIPCHK(c, hipMemcpyAsync(dst[k], a + k * S, S * sizeof(int), hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipMemcpyAsync(c->ds.req_id, c->h_req, S * sizeof(long long), hipMemcpyHostToDevice, c->stream));
  return APRIL_OK;
}

}  // namespace

// =============================================================================
// C ABI
// =============================================================================
extern "C" {

const char* april_last_error(const april_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

// The graph of n_iters decode iterations (each: scheduler + forward + sampler) sized for at most
// rows_cap live rows and gs KV splits; instantiated on first use and kept for the context's life.
static int iter_graph(april_ctx* c, int rows_cap, int gs, int n_iters, hipGraphExec_t* out) {
  const std::pair<int, int> key{rows_cap | (n_iters << 24), gs};
  auto it = c->iter_graphs.find(key);
  if (it == c->iter_graphs.end()) {
    hipStream_t st = c->stream;
    const int ctx_grid = c->attn_mfma ? gs * c->attn_chunk : c->max_ctx;
    hipGraph_t graph = nullptr;
    c->prof_now = false;
    RowCtx grc{c->d_row_slot, c->d_row_pos, reinterpret_cast<const int2*>(c->d_ctrl), rows_cap};
    c->step_max_ctx = ctx_grid;
    HIPCHK(c, hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
    for (int q = 0; q < n_iters; ++q) {
      launch_sched(st, c->d_ctrl, c->ds, c->d_row_slot, c->d_row_pos, c->d_free_stack, 16, 0, rows_cap, ctx_grid,
                   c->d_att_items, c->attn_chunk, std::min(c->att_items_cap, rows_cap * gs));
      forward(c, grc, grc, nullptr, 0, 0);
    }
    HIPCHK(c, hipStreamEndCapture(st, &graph));
    hipGraphExec_t exec = nullptr;
    HIPCHK(c, hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0));
    HIPCHK(c, hipGraphDestroy(graph));
    it = c->iter_graphs.emplace(key, exec).first;
  }
  *out = it->second;
  return APRIL_OK;
}

int april_init(const april_model_cfg* cfg, const april_tensor* weights, int32_t n_weights, april_ctx** out) {
  if (!cfg || !weights || !out) return fail(nullptr, APRIL_EINVAL, "null argument");
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return fail(nullptr, APRIL_EDEVICE, "no HIP device");
  const april_model_cfg& g = *cfg;
  const bool moe = g.n_experts != 0;
  if (moe && (g.dtype != APRIL_DTYPE_BF16 || g.n_experts < 1 || g.n_experts > 256 || g.experts_per_tok < 1 ||
              g.experts_per_tok > 8 || g.experts_per_tok > g.n_experts || g.d_expert_ffn <= 0 ||
              g.d_expert_ffn % 32 || g.d_model % 64 || g.n_experts % 32))
    return fail(nullptr, APRIL_EINVAL, "routed experts need bf16, 32 | n_experts <= 256, experts_per_tok <= 8, 32 | d_expert_ffn, 64 | d_model");
  if (g.kv_block_tokens != 16) return fail(nullptr, APRIL_EINVAL, "kv_block_tokens must be 16");
  if (g.n_layers <= 0 || g.d_model <= 0 || g.n_q_heads <= 0 || g.n_kv_heads <= 0 || g.vocab <= 0 || (!moe && g.d_ffn <= 0))
    return fail(nullptr, APRIL_EINVAL, "non-positive model dimension");
  if (g.n_q_heads % g.n_kv_heads) return fail(nullptr, APRIL_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
  if (g.n_q_heads / g.n_kv_heads > 16) return fail(nullptr, APRIL_EINVAL, "at most 16 query heads per KV head");
  if (g.head_dim != 32 && g.head_dim != 64 && g.head_dim != 128) return fail(nullptr, APRIL_EINVAL, "head_dim must be 32, 64 or 128");
  if (g.d_model % 8 || g.d_model > 8192) return fail(nullptr, APRIL_EINVAL, "d_model must be a multiple of 8, at most 8192");
  if (g.dtype != APRIL_DTYPE_FP32 && g.dtype != APRIL_DTYPE_BF16) return fail(nullptr, APRIL_EINVAL, "bad dtype");
  if (g.max_inflight <= 0 || g.max_inflight > 2048) return fail(nullptr, APRIL_EINVAL, "max_inflight must be in 1..2048");
  if (g.max_ctx <= 1 || g.max_ctx > 32768) return fail(nullptr, APRIL_EINVAL, "max_ctx must be in 2..32768");
  if (g.sampler != APRIL_SAMPLER_GREEDY && g.sampler != APRIL_SAMPLER_TOPK && g.sampler != APRIL_SAMPLER_CATEGORICAL)
    return fail(nullptr, APRIL_EINVAL, "unknown sampler");
  if (g.sampler == APRIL_SAMPLER_TOPK && (g.top_k < 1 || g.top_k > 64 || !(g.temperature > 0.f)))
    return fail(nullptr, APRIL_EINVAL, "top_k must be in 1..64 and temperature > 0");
  if (g.sampler == APRIL_SAMPLER_CATEGORICAL && !(g.temperature > 0.f))
    return fail(nullptr, APRIL_EINVAL, "the categorical sampler needs temperature > 0");
  if (g.top_p < 0.f) return fail(nullptr, APRIL_EINVAL, "top_p must be in (0, 1], or 0 for none");
  if (g.n_samples_per_prompt < 0 || g.n_samples_per_prompt > g.max_inflight)
    return fail(nullptr, APRIL_EINVAL, "n_samples_per_prompt must be in 0..max_inflight");
  const int nq = g.n_q_heads * g.head_dim, nkv = g.n_kv_heads * g.head_dim, nqkv = nq + 2 * nkv;
  const int d = g.d_model, F = g.d_ffn, V = g.vocab;
  if (g.dtype == APRIL_DTYPE_BF16 && (d % 32 || (!moe && F % 32) || V % 32 || nq % 32 || nqkv % 32))
    return fail(nullptr, APRIL_EINVAL, "bf16 path needs d_model, d_ffn, vocab, head widths multiple of 32");

  april_ctx* c = new april_ctx();
  c->cfg = g;
  c->dm = ModelDims{g.n_layers, d, g.n_q_heads, g.n_kv_heads, g.head_dim, F, V, g.n_experts, g.experts_per_tok,
                    g.d_expert_ffn, g.rope_theta, g.rms_eps, 16};
  c->moe = moe; c->n_experts = g.n_experts; c->top_k_experts = g.experts_per_tok; c->d_expert = g.d_expert_ffn;
  c->bf16 = g.dtype == APRIL_DTYPE_BF16;
  c->esz = c->bf16 ? 2 : 4;
  const char* gm = getenv("APRIL_GEMM");
  c->use_mfma = c->bf16 && !(gm && !strcmp(gm, "ref"));
  const char* am = getenv("APRIL_ATTN");
  c->attn_mfma = c->bf16 && !(am && !strcmp(am, "ref"));
  if (moe && !(c->use_mfma && c->attn_mfma)) { delete c; return fail(nullptr, APRIL_EINVAL, "routed experts run on the MFMA path only"); }
  const char* fr = getenv("APRIL_FUSE_ROPE");
  c->fuse_rope = !(fr && !strcmp(fr, "0"));
  const char* fn = getenv("APRIL_FUSE_NORM");
  c->fuse_norm = !(fn && !strcmp(fn, "0"));
  const char* fd = getenv("APRIL_FUSE_DOWN");    // off by default: measured 5 % slower end to end on configuration 2
  c->fuse_down = fd && !strcmp(fd, "1");
  // (an MLP wide enough for 128 or more of that kernel's workgroups already gains from a row
  // bound of 64: 38.9 against 40.2 us per gate/up launch over a run of the 2560 x 9728 model)
  if (g.d_ffn >= 8192) c->tile_decode_rows = 64;
  if (const char* td = getenv("APRIL_TILE_DECODE_ROWS")) c->tile_decode_rows = atoi(td);   // debug switch
  if (const char* mt = getenv("APRIL_MOE_TALL_ROWS")) c->moe_tall_rows = atoi(mt);          // debug switch
  if (const char* mt = getenv("APRIL_MOE_TILE")) c->moe_tile = strcmp(mt, "0") != 0;
  if (const char* tf = getenv("APRIL_TILE_F32")) c->tile_f32 = strcmp(tf, "0") != 0;
  if (const char* fa = getenv("APRIL_DEBUG_FAIL_AT")) {                                       // debug switch
    if (sscanf(fa, "%d:%d", &c->debug_fail_step, &c->debug_fail_iter) != 2) c->debug_fail_step = c->debug_fail_iter = -1;
  }
  if (const char* gi = getenv("APRIL_GRAPH_ITERS")) c->graph_iters = std::max(1, std::min(16, atoi(gi)));
  const char* pa = getenv("APRIL_PREFILL_ATTN");
  c->prefill_tiled = !(pa && !strcmp(pa, "rows"));
  const char* tg = getenv("APRIL_TILE_GEMM");
  c->tile_gemm = !(tg && !strcmp(tg, "0"));
  const char* gr = getenv("APRIL_GRAPH");
  c->use_graph = !(gr && !strcmp(gr, "0"));
  for (int i = 0; i < KC_COUNT; ++i) c->stats[i] = april_kernel_stat{kKernelNames[i], 0, 0, 0, 0};
  auto bail = [&](int rc) { g_init_error = c->err; april_destroy(c); return rc; };
#define TRY(x) do { int rc_ = (x); if (rc_ != APRIL_OK) return bail(rc_); } while (0)
#define HIPTRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { fail(c, APRIL_EDEVICE, "%s failed: %s", #expr, hipGetErrorString(e_)); return bail(APRIL_EDEVICE); } } while (0)

  if (g.stream) c->stream = (hipStream_t)g.stream;
  else { HIPTRY(hipStreamCreate(&c->stream)); c->own_stream = true; }
  // device address of the static scratch array on this GPU (each GPU has its own copy)
  HIPTRY(hipGetDevice(&c->device));
  if (c->device < 0 || c->device >= MAX_DEVICES) { fail(c, APRIL_EINVAL, "device index %d not supported", c->device); return bail(APRIL_EINVAL); }
  if (!g_scratch_ptr[c->device]) {
    unsigned char* sp = nullptr;
    HIPTRY(hipGetSymbolAddress((void**)&sp, HIP_SYMBOL(scratch)));
    g_scratch_ptr[c->device] = sp;
  }
  c->scratch_dev = g_scratch_ptr[c->device];

  // ---- weights ------------------------------------------------------------------
  c->alloc_tag = g.pausable ? APRIL_MEM_WEIGHTS : 0;
  { int rc_w = load_weights(c, weights, n_weights); c->alloc_tag = 0; if (rc_w != APRIL_OK) return bail(rc_w); }
  const size_t e = c->esz;

  // ---- scheduler state ------------------------------------------------------------
  const int S = g.max_inflight;
  c->n_slots = S;
  c->max_ctx = g.max_ctx;
  c->max_blocks = ceil_div(g.max_ctx, 16);
  c->slots.assign(S, SlotH());
  c->ds.max_blocks = c->max_blocks;
  c->ds.max_ctx = c->max_ctx;
  TRY(dev_alloc(c, &c->ds.req_id, S));
  TRY(dev_alloc(c, &c->ds.prompt_len, S)); TRY(dev_alloc(c, &c->ds.gen, S)); TRY(dev_alloc(c, &c->ds.limit, S));
  TRY(dev_alloc(c, &c->ds.state, S)); TRY(dev_alloc(c, &c->ds.kv_len, S)); TRY(dev_alloc(c, &c->ds.n_blocks, S));
  TRY(dev_alloc(c, &c->ds.finish_iter, S));
  TRY(dev_alloc(c, &c->ds.block_table, (size_t)S * c->max_blocks));
  TRY(dev_alloc(c, &c->ds.tokens, (size_t)S * c->max_ctx));
  c->ds.forced = nullptr;
  if (g.debug_logits) {
    TRY(dev_alloc(c, &c->ds.forced, (size_t)S * c->max_ctx, false));
    launch_fill_i32(c->stream, c->ds.forced, -1, (size_t)S * c->max_ctx);
  }
  c->ds.logprob = nullptr;
  if (g.logprobs) TRY(dev_alloc(c, &c->ds.logprob, (size_t)S * c->max_ctx));
  c->ds.group = nullptr; c->ds.grp_left = nullptr;
  if (g.n_samples_per_prompt > 1) { TRY(dev_alloc(c, &c->ds.group, S)); TRY(dev_alloc(c, &c->ds.grp_left, S)); }
  TRY(dev_alloc(c, &c->d_ctrl, 1));
  HIPTRY(hipHostMalloc((void**)&c->h_ctrl, sizeof(Ctrl)));
  HIPTRY(hipHostMalloc((void**)&c->h_slot_arrays, (size_t)8 * S * sizeof(int)));
  HIPTRY(hipHostMalloc((void**)&c->h_req, (size_t)S * sizeof(long long)));
  TRY(dev_alloc(c, &c->d_row_slot, S)); TRY(dev_alloc(c, &c->d_row_pos, S));
  TRY(dev_alloc(c, &c->d_list_a, 2048)); TRY(dev_alloc(c, &c->d_list_b, 2048));

  // ---- KV pool --------------------------------------------------------------------
  c->kv_bytes_per_token = (int64_t)2 * g.n_layers * nkv * e;
  const int64_t page_bytes = c->kv_bytes_per_token * 16;
  int64_t pool = g.kv_pool_bytes;
  if (pool <= 0) {
    // every slot at max_ctx, but no more than the device has free after a reserve for the
    // workspaces allocated below (a smaller pool is legal: rollouts are then preempted and
    // re-prefilled when pages run out)
    pool = (int64_t)S * c->max_blocks * page_bytes;
    size_t free_b = 0, total_b = 0;
    HIPTRY(hipMemGetInfo(&free_b, &total_b));
    const int64_t reserve = std::max<int64_t>((int64_t)12 << 30, (int64_t)(total_b / 16));
    const int64_t cap = (int64_t)free_b - reserve;
    if (pool > cap && cap >= page_bytes) pool = cap;
  }
  c->n_pages = (int)std::min<int64_t>(pool / page_bytes, (int64_t)1 << 30);
  if (c->n_pages < 1) { fail(c, APRIL_ENOMEM, "KV pool smaller than one page"); return bail(APRIL_ENOMEM); }
  c->kv_pool_bytes = (int64_t)c->n_pages * page_bytes;
  c->alloc_tag = g.pausable ? APRIL_MEM_KV : 0;
  { int rc_kv = dev_alloc_bytes(c, &c->kv_pool, (size_t)c->kv_pool_bytes, true); c->alloc_tag = 0; if (rc_kv != APRIL_OK) return bail(rc_kv); }   // zeroed: masked lanes must stay finite
  c->kvl.n_kv_heads = g.n_kv_heads; c->kvl.head_dim = g.head_dim; c->kvl.blk = 16;
  c->kvl.mode = c->attn_mfma ? 1 : 0;
  c->kvl.kv_stride = (size_t)c->n_pages * nkv * 16;
  c->kvl.layer_stride = 2 * c->kvl.kv_stride;
  TRY(dev_alloc(c, &c->d_free_stack, c->n_pages, false));
  launch_init_free_stack(c->stream, c->d_free_stack, c->n_pages);
  c->free_pages_host = c->n_pages;
  memset(c->h_ctrl, 0, sizeof(Ctrl));
  c->h_ctrl->free_top = c->n_pages;
  c->h_ctrl->n_slots = S;
  c->h_ctrl->eos_token = g.eos_token;
  c->h_ctrl->stop = 1;
  HIPTRY(hipMemcpyAsync(c->d_ctrl, c->h_ctrl, sizeof(Ctrl), hipMemcpyHostToDevice, c->stream));
  HIPTRY(hipStreamSynchronize(c->stream));

  // ---- workspaces -----------------------------------------------------------------
  c->prefill_cap = std::max(g.max_ctx, 16384);   // rows per prefill chunk: enough tiles to fill the chip
  c->m_cap = ((std::max(c->prefill_cap, S) + 31) / 32) * 32;
  const size_t M = c->m_cap;
  if (c->use_mfma) { c->s_qkv = pick_ksplit(nqkv, d); c->s_o = pick_ksplit(d, nq); c->s_down = pick_ksplit(d, F); }
  c->qkv_stride = M * nqkv;
  c->proj_stride = M * d;
  TRY(dev_alloc(c, &c->x_res, M * d));
  if (c->use_mfma) TRY(dev_alloc(c, &c->ssq, (size_t)(d / 32) * M));
  TRY(dev_alloc(c, &c->qkv, (size_t)c->s_qkv * c->qkv_stride));
  TRY(dev_alloc(c, &c->q_rot, M * nq));
  TRY(dev_alloc(c, &c->proj, (size_t)std::max(c->s_o, c->s_down) * c->proj_stride));
  if (!c->use_mfma) TRY(dev_alloc(c, &c->gu, M * 2 * F));
  if (moe) {
    const int E = g.n_experts, Fe = g.d_expert_ffn, tk = g.experts_per_tok;
    c->expert_bytes = (int64_t)3 * Fe * d * e;
    c->s_router = pick_ksplit(E, d);
    c->router_stride = M * E;
    c->moe_p_cap = (int)((M * tk + (size_t)E * 127 + 127) / 128 * 128);   // expert segments are aligned to 64 or 128 rows
    TRY(dev_alloc(c, &c->router_out, (size_t)c->s_router * c->router_stride));
    TRY(dev_alloc(c, &c->moe_ids, M * tk)); TRY(dev_alloc(c, &c->moe_wts, M * tk)); TRY(dev_alloc(c, &c->moe_pos, M * tk));
    TRY(dev_alloc(c, &c->moe_cnt, E)); TRY(dev_alloc(c, &c->moe_base, E + 1)); TRY(dev_alloc(c, &c->moe_src, c->moe_p_cap));
    TRY(dev_alloc(c, &c->moe_group, c->moe_p_cap / 64 + 1));
    TRY(dev_alloc(c, &c->moe_act, (size_t)c->moe_p_cap * Fe));
    TRY(dev_alloc(c, &c->moe_out, (size_t)c->moe_p_cap * d));
    if (c->moe_tile) TRY(dev_alloc(c, &c->h_rows, M * d));
  }
  const size_t SR = ((size_t)S + 31) / 32 * 32;
  TRY(dev_alloc(c, &c->logits, SR * V));
  if (c->use_mfma && V % lmhead_group_cols() == 0) {
    TRY(dev_alloc(c, &c->group_max, SR * (V / lmhead_group_cols())));
    TRY(dev_alloc(c, &c->group_idx, SR * (V / lmhead_group_cols())));
    // the fused sampler must not write logits: greedy sampling needs only the group records;
    // parity mode, log-probabilities and the candidate search of the sampling modes read logits
    const char* wl = getenv("APRIL_WRITE_LOGITS");
    c->write_logits = g.debug_logits || g.logprobs || g.sampler != APRIL_SAMPLER_GREEDY || (wl && !strcmp(wl, "1"));
  }
  TRY(dev_alloc_bytes(c, &c->h_act, M * d * e));
  TRY(dev_alloc_bytes(c, &c->attn_out, M * nq * e));
  TRY(dev_alloc_bytes(c, &c->act, M * std::max(F, 1) * e));
  TRY(dev_alloc_bytes(c, &c->hf, SR * d * e));
  if (c->attn_mfma) {
    c->attn_chunk = attn_split_tokens(g.head_dim);
    c->attn_max_splits = ceil_div(g.max_ctx, c->attn_chunk);
    const size_t rec = 32 + (size_t)16 * g.head_dim;
    // rows per attention launch: all decode rows; prefill chunks go in pieces of up to 4096 rows
    // (fewer, fuller launches) as long as the split workspace stays within 1 GiB
    const size_t ws_row_bytes = (size_t)g.n_kv_heads * c->attn_max_splits * rec * sizeof(float);
    const int by_bytes = (int)std::min<size_t>(4096, ((size_t)1 << 30) / ws_row_bytes) / 32 * 32;
    c->attn_ws_rows = std::min<int>(c->m_cap, std::max({512, (S + 31) / 32 * 32, by_bytes}));
    TRY(dev_alloc(c, &c->attn_ws, (size_t)c->attn_ws_rows * g.n_kv_heads * c->attn_max_splits * rec, false));
    const char* al = getenv("APRIL_ATTN_LIST");
    c->att_list = c->fuse_rope && !(al && !strcmp(al, "0"));
    if (c->att_list) {
      c->att_items_cap = S * c->attn_max_splits;
      TRY(dev_alloc(c, &c->d_att_items, (size_t)c->att_items_cap + 1));
    }
  }
  TRY(dev_alloc(c, &c->rope_cos, (size_t)g.max_ctx * g.head_dim / 2, false));
  TRY(dev_alloc(c, &c->rope_sin, (size_t)g.max_ctx * g.head_dim / 2, false));
  launch_rope_table(c->stream, c->rope_cos, c->rope_sin, g.max_ctx, g.head_dim, g.rope_theta);
  TRY(dev_alloc(c, &c->d_pf_row_slot, M)); TRY(dev_alloc(c, &c->d_pf_row_pos, M));
  TRY(dev_alloc(c, &c->d_pf_nrows, 2)); TRY(dev_alloc(c, &c->d_pf_nsrows, 2));   // {rows, stop = 0}
  TRY(dev_alloc(c, &c->d_pf_srow_slot, S)); TRY(dev_alloc(c, &c->d_pf_srow_pos, S)); TRY(dev_alloc(c, &c->d_pf_gather, S));
  c->pf_items_cap = (int)(M / 16 + S + 16);
  TRY(dev_alloc(c, &c->d_pf_items, (size_t)c->pf_items_cap));
  c->h_stage_ints = 2 * M + 8 * (size_t)S + 64 + 4 * (size_t)c->pf_items_cap;
  HIPTRY(hipHostMalloc((void**)&c->h_stage, c->h_stage_ints * sizeof(int)));

  // ---- parity-mode capture ----------------------------------------------------------
  if (g.debug_logits) {
    c->watch_rows_cap = (int)std::max<int64_t>(16, std::min<int64_t>(8192, ((int64_t)512 << 20) / ((int64_t)V * 4)));
    TRY(dev_alloc(c, &c->dwatch.req, c->watch_cap)); TRY(dev_alloc(c, &c->dwatch.first, c->watch_cap));
    TRY(dev_alloc(c, &c->dwatch.count, c->watch_cap)); TRY(dev_alloc(c, &c->dwatch.row0, c->watch_cap));
    TRY(dev_alloc(c, &c->dwatch.logits, (size_t)c->watch_rows_cap * V));
    TRY(dev_alloc(c, &c->dwatch.sampled, c->watch_rows_cap)); TRY(dev_alloc(c, &c->dwatch.filled, c->watch_rows_cap));
  }
  HIPTRY(hipStreamSynchronize(c->stream));
  // Graphs of the decode iteration for every (row bound, KV splits) a step can meet, when they
  // are few (small models, where an instantiation inside a step would show): otherwise on first use.
  if (c->use_graph) {
    std::vector<int> row_bounds;
    for (int rb = 32; rb < c->n_slots; rb += 32) row_bounds.push_back(rb);
    row_bounds.push_back(c->n_slots);
    const int n_gs = c->attn_mfma ? c->attn_max_splits : 1;
    if ((int)row_bounds.size() * n_gs * (c->graph_iters > 1 ? 2 : 1) <= 48) {
      for (int rb : row_bounds)
        for (int gs = 1; gs <= n_gs; ++gs) {
          hipGraphExec_t exec = nullptr;
          if (iter_graph(c, rb, gs, 1, &exec) != APRIL_OK) return bail(APRIL_EDEVICE);
          if (c->graph_iters > 1 && iter_graph(c, rb, gs, c->graph_iters, &exec) != APRIL_OK) return bail(APRIL_EDEVICE);
        }
    }
  }
  *out = c;
  return APRIL_OK;
#undef TRY
#undef TRYW
#undef HIPTRY
}

void april_destroy(april_ctx* c) {
  if (!c) return;
  if (c->stream) hipStreamSynchronize(c->stream);
  for (void* p : c->allocs) hipFree(p);
  for (auto& r : c->vm_regions) { if (r.mapped) vm_unmap_region(r); hipMemAddressFree(r.va, r.bytes); }
  if (c->h_ctrl) hipHostFree(c->h_ctrl);
  if (c->h_slot_arrays) hipHostFree(c->h_slot_arrays);
  if (c->h_req) hipHostFree(c->h_req);
  if (c->h_stage) hipHostFree(c->h_stage);
  if (c->h_snaps) hipHostFree(c->h_snaps);
  for (auto& ev : c->ev_pool) { hipEventDestroy(ev.first); hipEventDestroy(ev.second); }
  for (auto& kv : c->iter_graphs) hipGraphExecDestroy(kv.second);
  for (april_buffer* b : c->buffers) delete b;
  if (c->own_stream && c->stream) hipStreamDestroy(c->stream);
  delete c;
}

int april_get_info(april_ctx* c, april_info* out) {
  if (!c || !out) return APRIL_EINVAL;
  size_t fr = 0, tot = 0;
  HIPCHK(c, hipMemGetInfo(&fr, &tot));
  out->hbm_total = (int64_t)tot; out->hbm_free = (int64_t)fr;
  out->kv_pool_bytes = c->kv_pool_bytes; out->kv_blocks_total = c->n_pages; out->kv_blocks_free = c->free_pages_host;
  out->weight_bytes = c->weight_bytes; out->decode_weight_bytes = c->decode_weight_bytes;
  out->kv_bytes_per_token = c->kv_bytes_per_token;
  out->expert_bytes = c->expert_bytes;
  return APRIL_OK;
}

static april_buffer* find_buffer(const april_ctx* c, const april_buffer* b) {
  for (april_buffer* x : c->buffers)
    if (x == b && x->alive && x->magic == 0xA9B1FFEEull) return x;
  return nullptr;
}
static april_buffer* new_buffer(april_ctx* c) {
  april_buffer* b = new april_buffer();
  c->buffers.push_back(b);
  return b;
}
static void retire_buffer(april_ctx* c, april_buffer* b) {
  b->alive = false;
  b->entries.clear();
  auto it = std::find(c->buffers.begin(), c->buffers.end(), b);
  if (it != c->buffers.end()) c->buffers.erase(it);
  delete b;
}

int april_resume(april_ctx* c, april_buffer* buffer) {
  if (!c) return APRIL_EINVAL;
  april_buffer* b = find_buffer(c, buffer);
  if (!b) return fail(c, APRIL_EHANDLE, "april_resume: unknown or stale buffer handle");
  for (auto& e : b->entries) c->pending.push_back(std::move(e));
  c->have_pending = true;
  retire_buffer(c, b);
  return APRIL_OK;
}

int april_buffer_size(const april_ctx* c, const april_buffer* buffer) {
  if (!c) return APRIL_EINVAL;
  april_buffer* b = find_buffer(c, buffer);
  if (!b) return APRIL_EHANDLE;
  return (int)b->entries.size();
}

// Make sure the host copy of an entry's tokens is current (slot-resident entries).
static int sync_entry_tokens(april_ctx* c, Entry& e) {
  if (e.slot < 0) return APRIL_OK;
  const SlotH& s = c->slots[e.slot];
  e.prompt = s.prompt;
  e.generated.resize(s.gen);
  if (s.gen > 0) {
    HIPCHK(c, hipMemcpyAsync(e.generated.data(), c->ds.tokens + (size_t)e.slot * c->max_ctx + s.prompt_len,
                             (size_t)s.gen * sizeof(int), hipMemcpyDeviceToHost, c->stream));
    if (c->ds.logprob) {
      e.logprobs.resize(s.gen);
      HIPCHK(c, hipMemcpyAsync(e.logprobs.data(), c->ds.logprob + (size_t)e.slot * c->max_ctx,
                               (size_t)s.gen * sizeof(float), hipMemcpyDeviceToHost, c->stream));
    }
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  return APRIL_OK;
}

int april_buffer_export(april_ctx* c, const april_buffer* buffer, april_partial* out, int32_t cap) {
  if (!c) return APRIL_EINVAL;
  april_buffer* b = find_buffer(c, buffer);
  if (!b) return fail(c, APRIL_EHANDLE, "april_buffer_export: unknown or stale buffer handle");
  const int n = (int)b->entries.size();
  for (int i = 0; i < n && i < cap; ++i) {
    Entry& e = b->entries[i];
    int rc = sync_entry_tokens(c, e);
    if (rc != APRIL_OK) return rc;
    out[i].request_id = e.req;
    out[i].prompt = e.prompt.data(); out[i].n_prompt = (int)e.prompt.size();
    out[i].generated = e.generated.data(); out[i].n_generated = (int)e.generated.size();
    out[i].limit = e.limit; out[i].n_resumes = e.n_resumes; out[i].done = e.done;
    out[i].group_id = e.group;
    out[i].kv_resident = (e.slot >= 0 && c->slots[e.slot].kv_len > 0) ? 1 : 0;
    out[i].logprobs = (c->ds.logprob && e.logprobs.size() == e.generated.size() && !e.logprobs.empty()) ? e.logprobs.data() : nullptr;
  }
  return n;
}

int april_buffer_import(april_ctx* c, const april_partial* in, int32_t n, april_buffer** out) {
  if (!c || !out || (n > 0 && !in)) return APRIL_EINVAL;
  for (int i = 0; i < n; ++i) {
    if (in[i].n_prompt <= 0 || !in[i].prompt || in[i].n_generated < 0 || in[i].limit <= 0 ||
        (in[i].n_generated > 0 && !in[i].generated))
      return fail(c, APRIL_EINVAL, "april_buffer_import: bad entry %d", i);
    if (in[i].n_prompt + in[i].limit > c->max_ctx)
      return fail(c, APRIL_EINVAL, "april_buffer_import: entry %d exceeds max_ctx", i);
    const bool done = in[i].n_generated >= in[i].limit;
    // below its limit a rollout can only be complete through the EOS token
    if (in[i].done && !done && (c->cfg.eos_token < 0 || in[i].n_generated == 0))
      return fail(c, APRIL_EINVAL, "april_buffer_import: entry %d flagged done below its limit", i);
  }
  april_buffer* b = new_buffer(c);
  for (int i = 0; i < n; ++i) {
    Entry e;
    e.req = in[i].request_id;
    e.prompt.assign(in[i].prompt, in[i].prompt + in[i].n_prompt);
    e.generated.assign(in[i].generated, in[i].generated + in[i].n_generated);
    if (in[i].logprobs && in[i].n_generated > 0) e.logprobs.assign(in[i].logprobs, in[i].logprobs + in[i].n_generated);
    e.limit = in[i].limit; e.n_resumes = in[i].n_resumes; e.group = in[i].group_id;
    e.done = in[i].n_generated >= in[i].limit ? 1 : (in[i].done ? 1 : 0);
    b->entries.push_back(std::move(e));
  }
  *out = b;
  return APRIL_OK;
}

static int free_slot_pages(april_ctx* c, const std::vector<int>& slot_ids) {
  // returns the pages of the listed slots to the device stack, 2048 slots per launch
  if (slot_ids.empty()) return APRIL_OK;
  std::vector<int> with_pages;
  for (int s : slot_ids) if (c->slots[s].n_blocks > 0) with_pages.push_back(s);
  if (with_pages.empty()) return APRIL_OK;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  memcpy(c->h_stage, with_pages.data(), with_pages.size() * sizeof(int));
  HIPCHK(c, hipMemcpyAsync(c->d_list_a, c->h_stage, with_pages.size() * sizeof(int), hipMemcpyHostToDevice, c->stream));
  launch_free_slots(c->stream, c->d_ctrl, c->ds, c->d_list_a, (int)with_pages.size(), c->d_free_stack);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int s : with_pages) { c->free_pages_host += c->slots[s].n_blocks; c->slots[s].n_blocks = 0; c->slots[s].kv_len = 0; }
  return APRIL_OK;
}

int april_buffer_drop_kv(april_ctx* c, april_buffer* buffer) {
  if (!c) return APRIL_EINVAL;
  april_buffer* b = find_buffer(c, buffer);
  if (!b) return fail(c, APRIL_EHANDLE, "april_buffer_drop_kv: unknown or stale buffer handle");
  std::vector<int> ids;
  for (auto& e : b->entries) if (e.slot >= 0) ids.push_back(e.slot);
  return free_slot_pages(c, ids);
}

void april_buffer_free(april_ctx* c, april_buffer* buffer) {
  if (!c) return;
  april_buffer* b = find_buffer(c, buffer);
  if (!b) return;
  std::vector<int> ids;
  for (auto& e : b->entries) if (e.slot >= 0) ids.push_back(e.slot);
  free_slot_pages(c, ids);
  for (int s : ids) c->slots[s] = SlotH();
  retire_buffer(c, b);
}

// New policy weights (Eq. 1: theta_{k+1}); rollouts that were parked under the old policy go on
// under the new one (Section 2.2, mixed-policy trajectories).
int april_update_weights(april_ctx* c, const april_tensor* weights, int32_t n_weights, int32_t keep_kv) {
  if (!c || !weights || n_weights <= 0) return APRIL_EINVAL;
  if (c->paused_tags & APRIL_MEM_WEIGHTS) return fail(c, APRIL_EINVAL, "the weights' memory is paused: call april_memory_resume first");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  { int rc = load_weights(c, weights, n_weights); if (rc != APRIL_OK) return rc; }
  c->weights_valid = true;
  if (!keep_kv) {
    // K/V computed under the old weights are not the new policy's: every parked or pending
    // rollout gives its pages back and is re-prefilled when it is resumed
    std::vector<int> ids;
    for (int s = 0; s < c->n_slots; ++s)
      if (c->slots[s].state != SLOT_FREE && c->slots[s].n_blocks > 0) ids.push_back(s);
    for (size_t i = 0; i < ids.size(); i += 2048) {
      std::vector<int> part(ids.begin() + i, ids.begin() + std::min(ids.size(), i + 2048));
      int rc = free_slot_pages(c, part);
      if (rc != APRIL_OK) return rc;
    }
  }
  c->weight_version += 1;
  return APRIL_OK;
}

// Release / re-map the physical memory behind the KV pool and the weights (Section 3.3: the
// rollout engine and the trainer share the GPU; addresses stay, so captured graphs stay valid).
int april_memory_pause(april_ctx* c, int32_t tags) {
  if (!c) return APRIL_EINVAL;
  if (!c->cfg.pausable) return fail(c, APRIL_EINVAL, "context was not created with pausable = 1");
  if (tags & ~(APRIL_MEM_KV | APRIL_MEM_WEIGHTS)) return fail(c, APRIL_EINVAL, "unknown memory tag");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipDeviceSynchronize());
  for (auto& r : c->vm_regions)
    if ((r.tag & tags) && r.mapped) vm_unmap_region(r);
  if ((tags & APRIL_MEM_KV) && !(c->paused_tags & APRIL_MEM_KV)) {
    // the K/V of every parked rollout is gone with the pool: they keep their tokens and are
    // re-prefilled when resumed
    for (auto& sh : c->slots) { sh.n_blocks = 0; sh.kv_len = 0; }
    c->free_pages_host = c->n_pages;
  }
  if (tags & APRIL_MEM_WEIGHTS) c->weights_valid = false;
  c->paused_tags |= tags;
  return APRIL_OK;
}
int april_memory_resume(april_ctx* c, int32_t tags) {
  if (!c) return APRIL_EINVAL;
  if (!c->cfg.pausable) return fail(c, APRIL_EINVAL, "context was not created with pausable = 1");
  tags &= c->paused_tags;
  for (auto& r : c->vm_regions)
    if ((r.tag & tags) && !r.mapped) { int rc = vm_map_region(c, r); if (rc != APRIL_OK) return rc; }
  if (tags & APRIL_MEM_KV) {
    HIPCHK(c, hipMemsetAsync(c->kv_pool, 0, (size_t)c->kv_pool_bytes, c->stream));   // masked lanes must stay finite
    launch_init_free_stack(c->stream, c->d_free_stack, c->n_pages);
    // per-slot page counts on the device follow the host mirrors at the next step; the stack top too
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  c->paused_tags &= ~tags;
  return APRIL_OK;
}

int april_debug_watch(april_ctx* c, int64_t request_id, int32_t first_gen, int32_t n_gen) {
  if (!c) return APRIL_EINVAL;
  if (!c->cfg.debug_logits) return fail(c, APRIL_EINVAL, "context was not created with debug_logits");
  if (n_gen <= 0 || first_gen < 0) return fail(c, APRIL_EINVAL, "bad watch range");
  if (c->n_watch >= c->watch_cap || c->watch_rows_used + n_gen > c->watch_rows_cap)
    return fail(c, APRIL_ENOMEM, "watch capacity exceeded");
  long long req = request_id;
  int row0 = c->watch_rows_used;
  const int i = c->n_watch;
  HIPCHK(c, hipMemcpy(c->dwatch.req + i, &req, sizeof req, hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->dwatch.first + i, &first_gen, sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->dwatch.count + i, &n_gen, sizeof(int), hipMemcpyHostToDevice));
  HIPCHK(c, hipMemcpy(c->dwatch.row0 + i, &row0, sizeof(int), hipMemcpyHostToDevice));
  for (int k = 0; k < n_gen; ++k) c->watch_row_of[{req, first_gen + k}] = row0 + k;
  c->watch_rows_used += n_gen;
  c->n_watch += 1;
  return APRIL_OK;
}

int april_debug_logits(april_ctx* c, int64_t request_id, int32_t gen_index, float* out_logits, int32_t* out_sampled) {
  if (!c) return APRIL_EINVAL;
  auto it = c->watch_row_of.find({(long long)request_id, gen_index});
  if (it == c->watch_row_of.end()) return fail(c, APRIL_EHANDLE, "request/generated index is not watched");
  const int row = it->second;
  int filled = 0, sampled = -1;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(&filled, c->dwatch.filled + row, sizeof(int), hipMemcpyDeviceToHost));
  if (!filled) return fail(c, APRIL_EHANDLE, "watched logits were not produced yet");
  if (out_logits)
    HIPCHK(c, hipMemcpy(out_logits, c->dwatch.logits + (size_t)row * c->dm.vocab, (size_t)c->dm.vocab * sizeof(float), hipMemcpyDeviceToHost));
  HIPCHK(c, hipMemcpy(&sampled, c->dwatch.sampled + row, sizeof(int), hipMemcpyDeviceToHost));
  if (out_sampled) *out_sampled = sampled;
  return APRIL_OK;
}

static int sample_rows_impl(april_ctx* c, const float* logits, int32_t n_rows, const int64_t* request_ids,
                            const int32_t* gen_index, int32_t* out_tokens, float* out_logprobs) {
  if (!c || !logits || !request_ids || !gen_index || !out_tokens || n_rows <= 0) return APRIL_EINVAL;
  long long* d_req = nullptr; int *d_gen = nullptr, *d_out = nullptr, *d_n = nullptr;
  float *d_gm = nullptr, *d_lp = nullptr;
  auto release = [&]() { hipFree(d_req); hipFree(d_gen); hipFree(d_out); hipFree(d_n); hipFree(d_gm); hipFree(d_lp); };
  auto run = [&]() -> int {
    HIPCHK(c, hipMalloc((void**)&d_req, n_rows * sizeof(long long)));
    HIPCHK(c, hipMalloc((void**)&d_gen, n_rows * sizeof(int)));
    HIPCHK(c, hipMalloc((void**)&d_out, n_rows * sizeof(int)));
    HIPCHK(c, hipMalloc((void**)&d_n, 2 * sizeof(int)));
    if (out_logprobs) HIPCHK(c, hipMalloc((void**)&d_lp, n_rows * sizeof(float)));
    HIPCHK(c, hipMemset(d_n, 0, 2 * sizeof(int)));
    HIPCHK(c, hipMemcpy(d_req, request_ids, n_rows * sizeof(long long), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(d_gen, gen_index, n_rows * sizeof(int), hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(d_n, &n_rows, sizeof(int), hipMemcpyHostToDevice));
    RowCtx rc{nullptr, nullptr, reinterpret_cast<const int2*>(d_n), n_rows};
    const SamplerCfg sc = sampler_cfg(c);
    // same candidate search as the rollout path: group maxima first when the vocabulary allows
    const int grp = lmhead_group_cols();
    if (c->dm.vocab % grp == 0) {
      HIPCHK(c, hipMalloc((void**)&d_gm, (size_t)n_rows * (c->dm.vocab / grp) * sizeof(float)));
      launch_group_max(c->stream, logits, n_rows, c->dm.vocab, grp, d_gm);
    }
    launch_sample(c->stream, rc, c->ds, nullptr, logits, c->dm.vocab, sc, Watch{}, 0, d_req, d_gen, d_out, d_gm, grp, d_lp);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(out_tokens, d_out, n_rows * sizeof(int), hipMemcpyDeviceToHost));
    if (out_logprobs) HIPCHK(c, hipMemcpy(out_logprobs, d_lp, n_rows * sizeof(float), hipMemcpyDeviceToHost));
    return APRIL_OK;
  };
  const int rc_ = run();
  release();
  return rc_;
}
int april_sample_rows(april_ctx* c, const float* logits, int32_t n_rows, const int64_t* request_ids,
                      const int32_t* gen_index, int32_t* out_tokens) {
  return sample_rows_impl(c, logits, n_rows, request_ids, gen_index, out_tokens, nullptr);
}
int april_sample_rows_logprobs(april_ctx* c, const float* logits, int32_t n_rows, const int64_t* request_ids,
                               const int32_t* gen_index, int32_t* out_tokens, float* out_logprobs) {
  if (!out_logprobs) return APRIL_EINVAL;
  return sample_rows_impl(c, logits, n_rows, request_ids, gen_index, out_tokens, out_logprobs);
}

// The same sampler for callers that must not allocate: every temporary lives in this GPU's
// static scratch array.  No hipMalloc / hipFree here or below.
int april_sample_rows_noalloc(april_ctx* c, const float* logits, int32_t n_rows, const int64_t* request_ids,
                              const int32_t* gen_index, int32_t* out_tokens) {
  if (!c || !logits || !request_ids || !gen_index || !out_tokens || n_rows <= 0) return APRIL_EINVAL;
  const int grp = lmhead_group_cols();
  const bool use_gm = c->dm.vocab % grp == 0;
  if ((size_t)n_rows > NOALLOC_MAX_ROWS)
    return fail(c, APRIL_EINVAL, "april_sample_rows_noalloc: %d rows, at most %zu", n_rows, NOALLOC_MAX_ROWS);
  if (use_gm && (size_t)n_rows * (size_t)(c->dm.vocab / grp) > NOALLOC_MAX_GROUP_MAX)
    return fail(c, APRIL_EINVAL, "april_sample_rows_noalloc: rows x vocab/%d = %zu exceeds the scratch (%zu)", grp,
                (size_t)n_rows * (size_t)(c->dm.vocab / grp), NOALLOC_MAX_GROUP_MAX);
  if (!c->scratch_dev) return fail(c, APRIL_EDEVICE, "scratch address was not resolved at april_init");
  unsigned char* sp = c->scratch_dev;
  int* d_n = reinterpret_cast<int*>(sp + NOALLOC_OFF_CTL);
  long long* d_req = reinterpret_cast<long long*>(sp + NOALLOC_OFF_REQ);
  int* d_gen = reinterpret_cast<int*>(sp + NOALLOC_OFF_GEN);
  int* d_out = reinterpret_cast<int*>(sp + NOALLOC_OFF_OUT);
  float* d_gm = use_gm ? reinterpret_cast<float*>(sp + NOALLOC_OFF_GM) : nullptr;
  hipStream_t st = c->stream;
  const int ctl[2] = {n_rows, 0};                 // {rows, stop flag}: the array keeps the last call's contents
  HIPCHK(c, hipMemcpyAsync(d_n, ctl, sizeof ctl, hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(d_req, request_ids, n_rows * sizeof(long long), hipMemcpyHostToDevice, st));
  HIPCHK(c, hipMemcpyAsync(d_gen, gen_index, n_rows * sizeof(int), hipMemcpyHostToDevice, st));
  RowCtx rc{nullptr, nullptr, reinterpret_cast<const int2*>(d_n), n_rows};
  const SamplerCfg sc = sampler_cfg(c);
  if (use_gm) launch_group_max(st, logits, n_rows, c->dm.vocab, grp, d_gm);
  launch_sample(st, rc, c->ds, nullptr, logits, c->dm.vocab, sc, Watch{}, 0, d_req, d_gen, d_out, d_gm, grp);
  HIPCHK(c, hipMemcpyAsync(out_tokens, d_out, n_rows * sizeof(int), hipMemcpyDeviceToHost, st));
  HIPCHK(c, hipStreamSynchronize(st));
  return APRIL_OK;
}

static int measure_event_overhead(april_ctx* c);
int april_profile_enable(april_ctx* c, int32_t every) {
  if (!c || every < 0) return APRIL_EINVAL;
  c->prof_every = every;
  if (every > 0 && !c->h_snaps) {
    c->snaps_cap = 4096;
    HIPCHK(c, hipHostMalloc((void**)&c->h_snaps, c->snaps_cap * sizeof(Ctrl)));
  }
  if (every > 0 && c->stats[KC_EVENT_EMPTY].launches == 0) return measure_event_overhead(c);
  return APRIL_OK;
}
// What an event pair around one eager launch reads for a kernel that does nothing: the part
// of every profiled launch's time that is dispatch and completion latency, not execution.
static int measure_event_overhead(april_ctx* c) {
  if (!c->d_dummy) { int rc = dev_alloc(c, &c->d_dummy, 64, true); if (rc != APRIL_OK) return rc; }
  const bool was = c->prof_now;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->prof_now = true;
  for (int i = 0; i < 64; ++i) {
    ProfScope p(c, KC_EVENT_EMPTY, 0, 0);
    launch_fill_i32(c->stream, c->d_dummy, 0, 1);
  }
  // and with nothing between the two records: what the pair itself costs on the stream
  for (int i = 0; i < 64; ++i) { ProfScope p(c, KC_EVENT_NONE, 0, 0); }
  c->prof_now = was;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  prof_collect(c);
  return APRIL_OK;
}
int april_profile_reset(april_ctx* c) {
  if (!c) return APRIL_EINVAL;
  for (int i = 0; i < KC_COUNT; ++i) c->stats[i] = april_kernel_stat{kKernelNames[i], 0, 0, 0, 0};
  if (c->prof_every > 0) return measure_event_overhead(c);
  return APRIL_OK;
}
int april_profile_get(april_ctx* c, april_kernel_stat* out, int32_t cap) {
  if (!c || !out) return APRIL_EINVAL;
  int n = 0;
  for (int i = 0; i < KC_COUNT && n < cap; ++i) out[n++] = c->stats[i];
  return n;
}

// -----------------------------------------------------------------------------
// The rollout step
// -----------------------------------------------------------------------------
int april_rollout_step(april_ctx* c, const april_request* new_reqs, int32_t n_new_avail, int32_t N_target,
                       int32_t N_over, int32_t max_new, april_step_result* out) {
  if (!c || !out) return APRIL_EINVAL;
  if (N_target <= 0 || N_over < N_target || max_new <= 0 || n_new_avail < 0 || (n_new_avail > 0 && !new_reqs))
    return fail(c, APRIL_EINVAL, "bad step arguments (need 0 < N_target <= N_overprovision, max_new > 0)");
  if (c->paused_tags) return fail(c, APRIL_EINVAL, "the engine's memory is paused: call april_memory_resume first");
  if (!c->weights_valid) return fail(c, APRIL_EINVAL, "the weights' memory was released and re-mapped: call april_update_weights first");
  const double t_begin = now_s();
  hipStream_t st = c->stream;
  const int blk = 16;

  // ---- admission plan (nothing is modified until every check has passed) -------------
  // Resumed rollouts first (ascending id): KV-resident ones are in flight as they are; a
  // rollout that needs prefill (resumed without KV, or new) is admitted only while the pages of
  // its tokens fit in the free pool - the first that does not fit closes admission for the step.
  // Instance-level completion (Section 3.2.3): with G = n_samples_per_prompt > 1 the unit that
  // completes, is counted toward N and is delivered is the group of G rollouts of one input
  // instance; N_target and N_overprovision still count rollouts (multiples of G).
  const int G = std::max(1, c->cfg.n_samples_per_prompt);
  if (G > 1 && (N_target % G || N_over % G))
    return fail(c, APRIL_EINVAL, "N_target and N_overprovision must be multiples of n_samples_per_prompt (%d)", G);
  const int N_units = N_target / G, Nover_units = N_over / G;
  std::vector<Entry>& pend = c->pending;
  std::sort(pend.begin(), pend.end(), [](const Entry& a, const Entry& b) { return a.req < b.req; });
  std::map<long long, std::vector<int>> gmem;                  // group id -> indices into pend (G > 1)
  std::map<long long, bool> gdone;
  if (G > 1) {
    for (int i = 0; i < (int)pend.size(); ++i) gmem[pend[i].group].push_back(i);
    for (auto& kv : gmem) {
      if ((int)kv.second.size() != G)
        return fail(c, APRIL_EINVAL, "group %lld: %d of its %d rollouts were resumed (resume every buffer that holds its members)", kv.first, (int)kv.second.size(), G);
      bool all = true;
      for (int i : kv.second) all = all && pend[i].done;
      gdone[kv.first] = all;
    }
  }
  std::vector<int> deliver_idx, resume_idx, stay_idx, wait_idx;   // indices into pend
  int64_t pages_left = c->free_pages_host;
  bool admission_open = true;
  for (int i = 0; i < (int)pend.size(); ++i) {
    const Entry& e = pend[i];
    if (e.done) {
      // complete: delivered now - or, as a member of a group that is not complete yet, it waits
      if (G == 1 || gdone[e.group]) deliver_idx.push_back(i); else wait_idx.push_back(i);
      continue;
    }
    const bool resident = e.slot >= 0 && c->slots[e.slot].kv_len > 0;
    if (!resident) {
      const int ntok = e.slot >= 0 ? c->slots[e.slot].prompt_len + c->slots[e.slot].gen
                                   : (int)(e.prompt.size() + e.generated.size());
      const int need = ceil_div(ntok, blk);
      if (admission_open && need <= pages_left) pages_left -= need;
      else { admission_open = false; stay_idx.push_back(i); continue; }
    }
    resume_idx.push_back(i);
  }
  const int D = (int)deliver_idx.size() / G;                   // units (rollouts, or groups) delivered from the buffer
  int n_inflight = (int)resume_idx.size();
  int n_admit = 0, n_avail_for_n = 0;
  if (G == 1) {
    while (n_inflight + n_avail_for_n < N_over - D && n_avail_for_n < n_new_avail) ++n_avail_for_n;
    if (D + (int)stay_idx.size() + n_inflight + n_avail_for_n < N_target)
      return fail(c, APRIL_ESTARVED, "only %d rollouts available, %d needed", D + (int)stay_idx.size() + n_inflight + n_avail_for_n, N_target);
  } else {
    std::map<long long, int> running, open;
    for (int i : resume_idx) { running[pend[i].group] = 1; open[pend[i].group] = 1; }
    for (int i : stay_idx) open[pend[i].group] = 1;
    int new_groups = 0;
    while ((int)running.size() + new_groups < Nover_units - D && (new_groups + 1) * G <= n_new_avail) ++new_groups;
    n_avail_for_n = new_groups * G;
    if (D + (int)open.size() + new_groups < N_units)
      return fail(c, APRIL_ESTARVED, "only %d groups available, %d needed", D + (int)open.size() + new_groups, N_units);
    std::map<long long, int> seen;
    for (int b = 0; b < new_groups; ++b) {
      const long long gid = new_reqs[b * G].group_id;
      for (int k = 1; k < G; ++k)
        if (new_reqs[b * G + k].group_id != gid) return fail(c, APRIL_EINVAL, "request %d: the %d rollouts of a group must be consecutive", b * G + k, G);
      if (gmem.count(gid) || seen.count(gid)) return fail(c, APRIL_EINVAL, "group %lld is already in flight or buffered", gid);
      seen[gid] = 1;
    }
  }
  for (int i = 0; i < n_avail_for_n; ++i) {
    const april_request& r = new_reqs[i];
    if (r.n_tokens <= 0 || !r.tokens) return fail(c, APRIL_EINVAL, "request %d: empty prompt", i);
    const int lim = r.forced_len > 0 ? std::min(r.forced_len, max_new) : max_new;
    if (r.n_tokens + lim > c->max_ctx) return fail(c, APRIL_EINVAL, "request %d: prompt %d + limit %d exceeds max_ctx %d", i, r.n_tokens, lim, c->max_ctx);
    if (ceil_div(r.n_tokens + lim, blk) > c->n_pages) return fail(c, APRIL_ENOMEM, "request %d: the KV pool (%d pages) cannot hold even this one rollout", i, c->n_pages);
    for (int k = 0; k < r.n_tokens; ++k)
      if (r.tokens[k] < 0 || r.tokens[k] >= c->dm.vocab) return fail(c, APRIL_EINVAL, "request %d: token out of range", i);
    if (r.forced_tokens && !c->cfg.debug_logits) return fail(c, APRIL_EINVAL, "forced_tokens need a debug_logits context");
    if (r.forced_tokens)
      for (int k = 0; k < r.n_forced_tokens; ++k)
        if (r.forced_tokens[k] < 0 || r.forced_tokens[k] >= c->dm.vocab) return fail(c, APRIL_EINVAL, "request %d: forced token out of range", i);
  }
  while (n_admit < n_avail_for_n && admission_open) {      // new requests: whole groups (G = 1: single rollouts)
    int need = 0;
    for (int k = 0; k < G; ++k) need += ceil_div(new_reqs[n_admit + k].n_tokens, blk);
    if (need > pages_left) { admission_open = false; break; }
    pages_left -= need;
    n_admit += G;
  }
  n_inflight += n_admit;
  int slots_needed = n_admit;
  for (int i : resume_idx) if (pend[i].slot < 0) ++slots_needed;
  int slots_free = 0;
  for (auto& s : c->slots) if (s.state == SLOT_FREE) ++slots_free;
  if (slots_needed > slots_free) return fail(c, APRIL_ENOMEM, "%d sequence slots needed, %d free (max_inflight)", slots_needed, slots_free);
  // does the worst case (every rollout runs to its limit) fit?  If it does, no rollout can be
  // preempted and the iteration count of the step is known in advance.
  bool pool_ample = true;
  {
    long long need = 0;
    for (int i : resume_idx) {
      const Entry& e = pend[i];
      const int P = e.slot >= 0 ? c->slots[e.slot].prompt_len : (int)e.prompt.size();
      const int have = e.slot >= 0 ? c->slots[e.slot].n_blocks : 0;
      need += ceil_div(P + e.limit, blk) - have;
    }
    for (int i = 0; i < n_admit; ++i) {
      const april_request& r = new_reqs[i];
      const int lim = r.forced_len > 0 ? std::min(r.forced_len, max_new) : max_new;
      need += ceil_div(r.n_tokens + lim, blk);
    }
    pool_ample = need <= c->free_pages_host;
  }

  // ---- commit admission (host bookkeeping only: nothing here can fail) -------------------
  std::vector<int> inflight;            // slots in flight this step: resumed ones first, then new ones
  std::vector<int> prefill_slots;       // need (re-)prefill
  std::vector<Entry> deliver;           // surplus-complete from the last step, ascending id
  int64_t prefill_tokens = 0, reprefill_tokens = 0;
  int n_resident = 0;
  std::vector<Entry> stay;              // buffered rollouts that could not be admitted (KV pool)
  struct Upload { int slot; std::vector<int> tokens; std::vector<int> forced; bool has_forced; std::vector<float> logprobs; };
  std::vector<Upload> uploads;          // token arrays the device still needs
  std::vector<std::pair<int, Entry>> token_level;   // (slot, entry as resumed) of entries that came without a slot
  std::vector<Entry> waiting;           // complete members of groups that are not complete yet (G > 1)
  for (int i : stay_idx) stay.push_back(pend[i]);
  for (int i : deliver_idx) deliver.push_back(pend[i]);
  for (int i : wait_idx) waiting.push_back(pend[i]);
  for (int i : resume_idx) {
    Entry& e = pend[i];
    int s = e.slot;
    if (s < 0) {                         // token-level entry: take a slot, upload its tokens
      s = alloc_slot(c);
      SlotH& sh = c->slots[s];
      sh = SlotH();
      sh.group = e.group;
      sh.req = e.req; sh.prompt = e.prompt; sh.prompt_len = (int)e.prompt.size();
      sh.gen = (int)e.generated.size(); sh.limit = e.limit; sh.n_resumes = e.n_resumes;
      sh.state = SLOT_PARKED;
      std::vector<int> all(e.prompt);
      all.insert(all.end(), e.generated.begin(), e.generated.end());
      // parity mode: the slot's previous occupant may have left teacher-forced tokens behind
      uploads.push_back({s, std::move(all), std::vector<int>(), c->ds.forced != nullptr, e.logprobs});
      token_level.push_back({s, e});
    }
    SlotH& sh = c->slots[s];
    sh.n_resumes += 1;
    if (sh.kv_len > 0) { sh.state = SLOT_LIVE; ++n_resident; }
    else { sh.state = SLOT_PREFILL; prefill_slots.push_back(s); reprefill_tokens += sh.prompt_len + sh.gen; }
    inflight.push_back(s);
  }
  const int n_resumed_inflight = (int)inflight.size();
  for (int i = 0; i < n_admit; ++i) {
    const april_request& r = new_reqs[i];
    const int s = alloc_slot(c);
    SlotH& sh = c->slots[s];
    sh = SlotH();
    sh.req = r.request_id; sh.prompt.assign(r.tokens, r.tokens + r.n_tokens); sh.prompt_len = r.n_tokens;
    sh.group = G > 1 ? r.group_id : -1;
    sh.limit = r.forced_len > 0 ? std::min(r.forced_len, max_new) : max_new;
    sh.state = SLOT_PREFILL;
    Upload u{s, sh.prompt, std::vector<int>(), c->ds.forced != nullptr, std::vector<float>()};
    if (c->ds.forced && r.forced_tokens) u.forced.assign(r.forced_tokens, r.forced_tokens + std::min(r.n_forced_tokens, c->max_ctx));
    uploads.push_back(std::move(u));
    prefill_slots.push_back(s);
    prefill_tokens += r.n_tokens;
    inflight.push_back(s);
  }
  // groups in flight this step: dense index, members still unfinished (the ones that could not be
  // admitted included: their group cannot complete in this step)
  std::map<long long, int> gindex;
  std::vector<int> g_left, g_blocked;
  std::vector<long long> g_id;
  std::vector<int> slot_gidx(c->n_slots, -1);
  if (G > 1) {
    auto idx_of = [&](long long gid) {
      auto it = gindex.find(gid);
      if (it != gindex.end()) return it->second;
      const int k = (int)g_id.size();
      gindex[gid] = k; g_id.push_back(gid); g_left.push_back(0); g_blocked.push_back(0);
      return k;
    };
    for (int s : inflight) { const int k = idx_of(c->slots[s].group); slot_gidx[s] = k; g_left[k] += 1; }
    for (const Entry& e : stay) { const int k = idx_of(e.group); g_left[k] += 1; g_blocked[k] = 1; }
  }
  pend.clear();
  c->have_pending = false;
  c->steps_started += 1;

  // From here on the step is transactional: `body` runs it; if it fails, `rollback` below hands
  // every resumed rollout back to the pending set (tokens generated so far kept, KV dropped) and
  // forgets the newly admitted requests, which the caller still owns (a failed call consumes
  // none of new_reqs).  Nothing a previous step left in the buffer is lost (Section 2.2: no
  // rollout is discarded).
  bool device_touched = false;          // the step has started to change per-slot device state
  april_buffer* nb = nullptr;
  auto body = [&]() -> int {
  for (Upload& u : uploads) {
    HIPCHK(c, hipMemcpyAsync(c->ds.tokens + (size_t)u.slot * c->max_ctx, u.tokens.data(), u.tokens.size() * sizeof(int), hipMemcpyHostToDevice, st));
    if (c->ds.logprob && !u.logprobs.empty())
      HIPCHK(c, hipMemcpyAsync(c->ds.logprob + (size_t)u.slot * c->max_ctx, u.logprobs.data(), u.logprobs.size() * sizeof(float), hipMemcpyHostToDevice, st));
    if (u.has_forced) {
      launch_fill_i32(st, c->ds.forced + (size_t)u.slot * c->max_ctx, -1, (size_t)c->max_ctx);
      if (!u.forced.empty())
        HIPCHK(c, hipMemcpyAsync(c->ds.forced + (size_t)u.slot * c->max_ctx, u.forced.data(), u.forced.size() * sizeof(int), hipMemcpyHostToDevice, st));
    }
  }
  HIPCHK(c, hipStreamSynchronize(st));   // the upload sources are pageable host vectors

  // ---- run ------------------------------------------------------------------------------
  double t_prefill = 0, t_decode = 0;
  int n_preempted = 0;
  long long iters = 0, sum_live = 0, sum_ctx = 0, it1_live = 0, it1_ctx = 0, sum_experts = 0, it1_experts = 0;
  std::vector<int> snap(7 * c->n_slots);
  if (D < N_units) {
    device_touched = true;
    { int rc = upload_slot_tables(c); if (rc != APRIL_OK) return rc; }
    if (G > 1) {
      HIPCHK(c, hipMemcpyAsync(c->ds.group, slot_gidx.data(), c->n_slots * sizeof(int), hipMemcpyHostToDevice, st));
      if (!g_left.empty())
        HIPCHK(c, hipMemcpyAsync(c->ds.grp_left, g_left.data(), g_left.size() * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipStreamSynchronize(st));
    }
    Ctrl& hc = *c->h_ctrl;
    hc.n_rows = 0; hc.finished = D; hc.n_target = N_units; hc.stop = 0; hc.iter = 0; hc.stop_iter = -1;
    hc.free_top = c->free_pages_host; hc.error = 0; hc.n_slots = c->n_slots; hc.eos_token = c->cfg.eos_token;
    hc.n_watch = c->n_watch; hc.inflight = (int)inflight.size(); hc.n_preempted = 0; hc.sum_live = 0; hc.sum_ctx = 0; hc.iter_ctx = 0; hc.sum_experts = 0;
    HIPCHK(c, hipMemcpyAsync(c->d_ctrl, &hc, sizeof(Ctrl), hipMemcpyHostToDevice, st));
    HIPCHK(c, hipStreamSynchronize(st));

    // Upper bound on the iterations of this step when only length limits end rollouts:
    // the (N - D)-th smallest remaining length.  With an EOS token the device may stop
    // earlier; the host then polls the control block between chunks.
    // (groups: a group completes when its slowest member does; a group with a member that could
    // not be admitted cannot complete in this step)
    std::vector<int> rem;
    int rem_max = 0;
    for (int s : inflight) rem_max = std::max(rem_max, c->slots[s].limit - c->slots[s].gen);
    if (G == 1) {
      for (int s : inflight) rem.push_back(c->slots[s].limit - c->slots[s].gen);
    } else {
      std::vector<int> gmax(g_id.size(), 0);
      for (int s : inflight) gmax[slot_gidx[s]] = std::max(gmax[slot_gidx[s]], c->slots[s].limit - c->slots[s].gen);
      for (size_t k = 0; k < g_id.size(); ++k) if (!g_blocked[k]) rem.push_back(gmax[k]);
    }
    std::sort(rem.begin(), rem.end());
    const bool exact = c->cfg.eos_token < 0 && pool_ample && (int)rem.size() >= N_units - D;
    const int T_bound = exact ? rem[N_units - D - 1] : rem_max;

    int decode_max_ctx = 1;
    for (int s : inflight) decode_max_ctx = std::max(decode_max_ctx, c->slots[s].prompt_len + c->slots[s].limit);
    c->step_max_ctx = decode_max_ctx;
    RowCtx drc{c->d_row_slot, c->d_row_pos, reinterpret_cast<const int2*>(c->d_ctrl), 0};
    const double t0 = now_s();
    // pages of every rollout that is (re-)prefilled this step, in admission order, before
    // the first scheduler pass hands out decode pages
    if (!prefill_slots.empty()) {
      int* h_list = c->h_stage; int* h_need = c->h_stage + c->n_slots;
      for (size_t i = 0; i < prefill_slots.size(); ++i) {
        const SlotH& sh = c->slots[prefill_slots[i]];
        h_list[i] = prefill_slots[i];
        h_need[i] = ceil_div(sh.prompt_len + sh.gen, blk);
      }
      HIPCHK(c, hipMemcpyAsync(c->d_list_a, h_list, prefill_slots.size() * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_list_b, h_need, prefill_slots.size() * sizeof(int), hipMemcpyHostToDevice, st));
      launch_alloc_prefill(st, c->d_ctrl, c->ds, c->d_list_a, c->d_list_b, (int)prefill_slots.size(), c->d_free_stack);
      // the prefill must not run on block tables that were not filled: look at the error flag now
      HIPCHK(c, hipMemcpyAsync(c->h_ctrl, c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipStreamSynchronize(st));
      if (c->h_ctrl->error) return fail(c, APRIL_ENOMEM, "KV page stack underflow on device (prefill pages)");
    }
    // iteration 1: resident rollouts decode, the others are (re-)prefilled
    const int NOCAP = 0x7fffffff;
    launch_sched(st, c->d_ctrl, c->ds, c->d_row_slot, c->d_row_pos, c->d_free_stack, blk, 0, NOCAP, NOCAP,
                 c->d_att_items, c->attn_chunk,
                 std::min(c->att_items_cap, n_resident * std::min(c->attn_max_splits, std::max(1, ceil_div(decode_max_ctx, c->attn_chunk)))));
    if (n_resident > 0) {
      drc.max_rows = n_resident;
      forward(c, drc, drc, nullptr, n_resident, 0);
    }
    // prefill in chunks of whole sequences
    size_t pi = 0;
    while (pi < prefill_slots.size()) {
      int rows = 0, nseq = 0, chunk_max_ctx = 1;
      int* hs = c->h_stage;
      int* h_row_slot = hs; int* h_row_pos = hs + c->m_cap;
      int* h_ss = hs + 2 * (size_t)c->m_cap; int* h_sp = h_ss + c->n_slots; int* h_g = h_sp + c->n_slots;
      int* h_list = h_g + c->n_slots; int* h_need = h_list + c->n_slots; int* h_n = h_need + c->n_slots;
      int4* h_items = reinterpret_cast<int4*>(hs + 2 * (size_t)c->m_cap + 8 * (size_t)c->n_slots + 64);
      const int q_tile = attn_prefill_tile(c->dm.n_q_heads / c->dm.n_kv_heads);
      int n_items = 0;
      while (pi < prefill_slots.size()) {
        const int s = prefill_slots[pi];
        const SlotH& sh = c->slots[s];
        const int nt = sh.prompt_len + sh.gen;
        if (rows + nt > c->prefill_cap && nseq > 0) break;
        for (int q0 = 0; q0 < nt && n_items < c->pf_items_cap; q0 += q_tile) h_items[n_items++] = int4{s, rows, nt, q0};
        for (int p = 0; p < nt; ++p) { h_row_slot[rows + p] = s; h_row_pos[rows + p] = p; }
        h_ss[nseq] = s; h_sp[nseq] = nt - 1; h_g[nseq] = rows + nt - 1;
        h_list[nseq] = s; h_need[nseq] = ceil_div(nt, blk);
        rows += nt; ++nseq; ++pi;
        chunk_max_ctx = std::max(chunk_max_ctx, nt);
      }
      c->step_max_ctx = chunk_max_ctx;
      h_n[0] = rows; h_n[1] = nseq;
      HIPCHK(c, hipMemcpyAsync(c->d_pf_row_slot, h_row_slot, rows * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_row_pos, h_row_pos, rows * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_srow_slot, h_ss, nseq * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_srow_pos, h_sp, nseq * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_gather, h_g, nseq * sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_nrows, h_n, sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_nsrows, h_n + 1, sizeof(int), hipMemcpyHostToDevice, st));
      HIPCHK(c, hipMemcpyAsync(c->d_pf_items, h_items, n_items * sizeof(int4), hipMemcpyHostToDevice, st));
      c->pf_n_items = n_items;
      RowCtx prc{c->d_pf_row_slot, c->d_pf_row_pos, reinterpret_cast<const int2*>(c->d_pf_nrows), rows};
      RowCtx src{c->d_pf_srow_slot, c->d_pf_srow_pos, reinterpret_cast<const int2*>(c->d_pf_nsrows), nseq};
      forward(c, prc, src, c->d_pf_gather, rows, 0);
      HIPCHK(c, hipStreamSynchronize(st));     // staging buffers are reused by the next chunk
    }
    HIPCHK(c, hipMemcpyAsync(c->h_ctrl, c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
    if (c->h_ctrl->error) return fail(c, APRIL_ENOMEM, "KV page stack underflow on device (prefill)");
    it1_live = c->h_ctrl->sum_live; it1_ctx = c->h_ctrl->sum_ctx; it1_experts = c->h_ctrl->sum_experts;
    t_prefill = now_s() - t0;

    // iterations 2..: pure decode
    const double t1 = now_s();
    // What the host knows about iteration `it` without asking the device: a rollout with r
    // tokens left is live in iterations 1..r, and its context then is at most prompt + generated
    // + it.  (EOS and preemption only take rows away.)  Each iteration is launched with grids
    // sized for these bounds; the scheduler kernel checks them.
    std::vector<std::pair<int, int>> by_rem;          // (tokens left, prompt + generated) per rollout
    for (int s : inflight) by_rem.push_back({c->slots[s].limit - c->slots[s].gen, c->slots[s].prompt_len + c->slots[s].gen});
    std::sort(by_rem.begin(), by_rem.end(), [](const auto& a, const auto& b) { return a.first > b.first; });
    std::vector<int> ctx_prefix_max(by_rem.size() + 1, 0);   // max base over the j longest-running rollouts
    for (size_t j = 0; j < by_rem.size(); ++j) ctx_prefix_max[j + 1] = std::max(ctx_prefix_max[j], by_rem[j].second);
    size_t n_alive = by_rem.size();
    auto bounds_at = [&](int it, int* rows_cap, int* ctx_cap) {
      while (n_alive > 0 && by_rem[n_alive - 1].first < it) --n_alive;     // `it` only grows
      int rb = ((int)n_alive + 31) / 32 * 32;
      if (rb < 32) rb = 32;
      if (rb > c->n_slots) rb = c->n_slots;
      *rows_cap = rb;
      *ctx_cap = std::min(c->max_ctx, ctx_prefix_max[n_alive] + it);
    };
    // one captured graph per (row bound, KV-split bound), replayed by every iteration that fits it
    bool stopped = false;
    int launched = 1;
    const int chunk = 32;
    while (!stopped) {
      int todo = exact ? T_bound - launched : std::min(chunk, T_bound - launched);
      if (todo < 0) todo = 0;
      // bounds of every iteration of this batch (bounds_at wants increasing iterations)
      c->it_rows.resize(todo); c->it_gs.resize(todo); c->it_ctx.resize(todo);
      for (int k = 0; k < todo; ++k) {
        int rows_cap = 0, ctx_cap = 0;
        bounds_at(launched + k + 1, &rows_cap, &ctx_cap);
        const int gs = c->attn_mfma ? std::min(c->attn_max_splits, std::max(1, ceil_div(ctx_cap, c->attn_chunk))) : 1;
        c->it_rows[k] = rows_cap; c->it_gs[k] = gs; c->it_ctx[k] = c->attn_mfma ? gs * c->attn_chunk : c->max_ctx;
      }
      auto profiled = [&](int it) { return c->prof_every > 0 && (it % c->prof_every) == 0; };
      for (int k = 0; k < todo; ++k) {
        const int it = launched + k + 1;
        const int rows_cap = c->it_rows[k], gs = c->it_gs[k], ctx_grid = c->it_ctx[k];
        c->prof_now = profiled(it) && c->snaps_used < c->snaps_cap;
        // debug switch (tests of the failure path): this iteration's scheduler pass is told a row
        // bound of zero, so the device raises its bounds error and ends the step
        const bool fail_here = c->steps_started == c->debug_fail_step && it == c->debug_fail_iter;
        if (c->use_graph && !c->prof_now && !fail_here) {
          // runs of iterations with the same bounds replay one graph of GRAPH_ITERS iterations
          int run = 1;
          while (run < c->graph_iters && k + run < todo && c->it_rows[k + run] == rows_cap && c->it_gs[k + run] == gs &&
                 !profiled(it + run) && !(c->steps_started == c->debug_fail_step && it + run == c->debug_fail_iter)) ++run;
          const int n_it = run == c->graph_iters ? run : 1;
          hipGraphExec_t exec = nullptr;
          { int rc = iter_graph(c, rows_cap, gs, n_it, &exec); if (rc != APRIL_OK) return rc; }
          HIPCHK(c, hipGraphLaunch(exec, st));
          k += n_it - 1;
          continue;
        }
        drc.max_rows = rows_cap;
        c->step_max_ctx = ctx_grid;
        {
          ProfScope p(c, KC_SCHED, 0, 0);
          launch_sched(st, c->d_ctrl, c->ds, c->d_row_slot, c->d_row_pos, c->d_free_stack, blk, 0,
                       fail_here ? 0 : rows_cap, ctx_grid, c->d_att_items, c->attn_chunk,
                       std::min(c->att_items_cap, rows_cap * gs));
          if (fail_here) c->debug_fail_step = -1;      // one shot
        }
        double B = 0, C = 0;
        if (c->prof_now) {
          c->prof_snap = c->snaps_used++;
          HIPCHK(c, hipMemcpyAsync(&c->h_snaps[c->prof_snap], c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
          HIPCHK(c, hipStreamSynchronize(st));
          B = c->h_snaps[c->prof_snap].n_rows; C = (double)c->h_snaps[c->prof_snap].iter_ctx;
        }
        forward(c, drc, drc, nullptr, B, C);
        c->prof_now = false;
      }
      launched += todo;
      launch_sched(st, c->d_ctrl, c->ds, c->d_row_slot, c->d_row_pos, c->d_free_stack, blk, 1, NOCAP, NOCAP);
      HIPCHK(c, hipMemcpyAsync(c->h_ctrl, c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
      HIPCHK(c, hipStreamSynchronize(st));
      if (c->h_ctrl->error & 2) return fail(c, APRIL_EDEVICE, "an iteration met more rows or a longer context than the host sized it for");
      if (c->h_ctrl->error) return fail(c, APRIL_ENOMEM, "KV page stack underflow on device");
      stopped = c->h_ctrl->stop != 0;
      if (!stopped && launched >= T_bound) {
        // every rollout has run to its limit or was preempted: a full scheduler pass ends the
        // step (nothing live, nothing waiting for prefill)
        launch_sched(st, c->d_ctrl, c->ds, c->d_row_slot, c->d_row_pos, c->d_free_stack, blk, 0, NOCAP, NOCAP);
        HIPCHK(c, hipMemcpyAsync(c->h_ctrl, c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost, st));
        HIPCHK(c, hipStreamSynchronize(st));
        stopped = c->h_ctrl->stop != 0;
        if (!stopped) return fail(c, APRIL_EDEVICE, "scheduler did not stop after %d iterations", launched);
      }
    }
    t_decode = now_s() - t1;
    iters = c->h_ctrl->stop_iter;
    sum_live = c->h_ctrl->sum_live; sum_ctx = c->h_ctrl->sum_ctx; sum_experts = c->h_ctrl->sum_experts;
    if (exact && iters != T_bound) return fail(c, APRIL_EDEVICE, "device stopped at iteration %lld, host expected %d", iters, T_bound);
    n_preempted = c->h_ctrl->n_preempted;
    prof_collect(c);

    // ---- read back per-slot state --------------------------------------------------------
    const int S = c->n_slots;
    int* srcs[5] = {c->ds.gen, c->ds.state, c->ds.kv_len, c->ds.n_blocks, c->ds.finish_iter};
    for (int k = 0; k < 5; ++k)
      HIPCHK(c, hipMemcpyAsync(c->h_slot_arrays + k * S, srcs[k], S * sizeof(int), hipMemcpyDeviceToHost, st));
    HIPCHK(c, hipStreamSynchronize(st));
    memcpy(snap.data(), c->h_slot_arrays, 5 * S * sizeof(int));
    c->free_pages_host = c->h_ctrl->free_top;
  }

  // ---- classify: newly complete (iteration, request id), surplus, partial -----------------
  const int S = c->n_slots;
  struct Fin { int iter; long long key; int slot; };      // key: request id (G = 1) or group id
  std::vector<Fin> fins;                                   // G = 1: rollouts complete in this step
  int64_t tokens_generated = 0;
  std::vector<int> partial_slots, done_slots;              // done_slots: complete in this step
  if (D < N_units) {
    for (int s : inflight) {
      SlotH& sh = c->slots[s];
      const int gen = snap[0 * S + s], state = snap[1 * S + s];
      tokens_generated += gen - sh.gen;
      sh.gen = gen; sh.kv_len = snap[2 * S + s]; sh.n_blocks = snap[3 * S + s];
      if (state == SLOT_DONE) { sh.state = SLOT_DONE; done_slots.push_back(s); if (G == 1) fins.push_back({snap[4 * S + s], sh.req, s}); }
      else { sh.state = SLOT_PARKED; partial_slots.push_back(s); }   // preempted ones come back with kv_len 0
    }
  } else {
    for (int s : inflight) { c->slots[s].state = SLOT_PARKED; partial_slots.push_back(s); }
  }
  std::sort(fins.begin(), fins.end(), [](const Fin& a, const Fin& b) { return a.iter != b.iter ? a.iter < b.iter : a.key < b.key; });

  // delivery order: surplus of the last step (ascending id), then this step's finishers
  c->r_req.clear(); c->r_tokens.clear(); c->r_ntok.clear(); c->r_nres.clear(); c->r_tok_ptrs.clear();
  c->r_logprobs.clear(); c->r_lp_ptrs.clear(); c->r_group.clear();
  nb = new_buffer(c);
  std::vector<int> release;             // slots whose rollout is returned now
  int delivered = 0;                    // units: rollouts (G = 1) or groups
  auto deliver_slot = [&](int s) -> int {
    SlotH& sh = c->slots[s];
    c->r_req.push_back(sh.req);
    c->r_group.push_back(sh.group);
    c->r_tokens.emplace_back((size_t)sh.gen);
    if (sh.gen > 0)
      HIPCHK(c, hipMemcpyAsync(c->r_tokens.back().data(), c->ds.tokens + (size_t)s * c->max_ctx + sh.prompt_len,
                               (size_t)sh.gen * sizeof(int), hipMemcpyDeviceToHost, st));
    c->r_logprobs.emplace_back(c->ds.logprob ? (size_t)sh.gen : 0);
    if (c->ds.logprob && sh.gen > 0)
      HIPCHK(c, hipMemcpyAsync(c->r_logprobs.back().data(), c->ds.logprob + (size_t)s * c->max_ctx,
                               (size_t)sh.gen * sizeof(float), hipMemcpyDeviceToHost, st));
    c->r_ntok.push_back(sh.gen);
    c->r_nres.push_back(sh.n_resumes);
    release.push_back(s);
    return APRIL_OK;
  };
  auto deliver_entry = [&](Entry& e) -> int {
    if (e.slot >= 0) return deliver_slot(e.slot);
    c->r_req.push_back(e.req); c->r_group.push_back(e.group); c->r_tokens.push_back(e.generated);
    c->r_logprobs.push_back(c->ds.logprob ? e.logprobs : std::vector<float>());
    c->r_ntok.push_back((int)e.generated.size()); c->r_nres.push_back(e.n_resumes);
    return APRIL_OK;
  };
  std::vector<int> surplus_slots;
  if (G == 1) {
    for (Entry& e : deliver) {
      if (delivered < N_target) { int rc = deliver_entry(e); if (rc != APRIL_OK) return rc; ++delivered; }
      else nb->entries.push_back(e);       // still surplus (only when N' > 2N)
    }
    for (const Fin& f : fins) {
      if (delivered < N_target) { int rc = deliver_slot(f.slot); if (rc != APRIL_OK) return rc; ++delivered; }
      else surplus_slots.push_back(f.slot);
    }
  } else {
    // groups complete in the buffer (ascending group id; `deliver` is in ascending request id, a
    // group's members are adjacent only if ids are dealt group by group: collect per group)
    std::map<long long, std::vector<Entry*>> dg;
    for (Entry& e : deliver) dg[e.group].push_back(&e);
    for (auto& kv : dg) {
      if (delivered < N_units) {
        for (Entry* e : kv.second) { int rc = deliver_entry(*e); if (rc != APRIL_OK) return rc; }
        ++delivered;
      } else for (Entry* e : kv.second) nb->entries.push_back(*e);
    }
    // groups completed by this step: every member complete, none left out; in order of the
    // iteration in which the last member completed, then group id
    std::vector<int> left(g_id.size(), 0), fin_iter(g_id.size(), -1);
    for (size_t k = 0; k < g_id.size(); ++k) left[k] = g_left[k];
    for (int s : done_slots) { const int k = slot_gidx[s]; left[k] -= 1; fin_iter[k] = std::max(fin_iter[k], snap[4 * S + s]); }
    std::vector<Fin> gfins;
    for (size_t k = 0; k < g_id.size(); ++k) if (left[k] == 0) gfins.push_back({fin_iter[k], g_id[k], (int)k});
    std::sort(gfins.begin(), gfins.end(), [](const Fin& a, const Fin& b) { return a.iter != b.iter ? a.iter < b.iter : a.key < b.key; });
    std::vector<char> g_delivered(g_id.size(), 0);
    for (const Fin& f : gfins) if (delivered < N_units) { g_delivered[f.slot] = 1; ++delivered; }
    // members of a delivered group, ascending request id: the ones that were waiting in the buffer
    // and the ones that completed now
    struct Mem { long long req; int slot; Entry* e; };
    std::map<int, std::vector<Mem>> by_group;
    for (Entry& e : waiting) { auto it = gindex.find(e.group); if (it != gindex.end() && g_delivered[it->second]) by_group[it->second].push_back({e.req, -1, &e}); }
    for (int s : done_slots) if (g_delivered[slot_gidx[s]]) by_group[slot_gidx[s]].push_back({c->slots[s].req, s, nullptr});
    for (const Fin& f : gfins) {
      if (!g_delivered[f.slot]) continue;
      auto& mem = by_group[f.slot];
      std::sort(mem.begin(), mem.end(), [](const Mem& a, const Mem& b) { return a.req < b.req; });
      for (Mem& m : mem) { int rc = m.e ? deliver_entry(*m.e) : deliver_slot(m.slot); if (rc != APRIL_OK) return rc; }
    }
    // complete, but not delivered (their group is not complete, or is surplus): wait in the buffer
    for (int s : done_slots) if (!g_delivered[slot_gidx[s]]) surplus_slots.push_back(s);
    for (Entry& e : waiting) {
      auto it = gindex.find(e.group);
      if (it == gindex.end() || !g_delivered[it->second]) nb->entries.push_back(e);
    }
  }
  HIPCHK(c, hipStreamSynchronize(st));
  // complete rollouts that stay keep their tokens (slot) but no KV pages
  {
    std::vector<int> to_free = release;
    to_free.insert(to_free.end(), surplus_slots.begin(), surplus_slots.end());
    int rc = free_slot_pages(c, to_free);
    if (rc != APRIL_OK) return rc;
  }
  std::vector<long long> rel_group;
  for (int s : release) c->slots[s] = SlotH();
  for (int s : surplus_slots) {
    Entry e; e.req = c->slots[s].req; e.slot = s; e.limit = c->slots[s].limit; e.n_resumes = c->slots[s].n_resumes; e.done = 1;
    e.group = c->slots[s].group;
    nb->entries.push_back(std::move(e));
  }
  for (int s : partial_slots) {
    Entry e; e.req = c->slots[s].req; e.slot = s; e.limit = c->slots[s].limit; e.n_resumes = c->slots[s].n_resumes; e.done = 0;
    e.group = c->slots[s].group;
    nb->entries.push_back(std::move(e));
  }
  for (Entry& e : stay) nb->entries.push_back(std::move(e));
  std::sort(nb->entries.begin(), nb->entries.end(), [](const Entry& a, const Entry& b) { return a.req < b.req; });

  for (auto& v : c->r_tokens) c->r_tok_ptrs.push_back(v.data());
  for (auto& v : c->r_logprobs) c->r_lp_ptrs.push_back(v.data());
  out->n_completed = (int)c->r_req.size();
  out->request_id = (const int64_t*)c->r_req.data();
  out->group_id = G > 1 ? (const int64_t*)c->r_group.data() : nullptr;
  out->tokens = c->r_tok_ptrs.data();
  out->n_tokens = c->r_ntok.data();
  out->n_resumes = c->r_nres.data();
  out->logprobs = c->ds.logprob ? c->r_lp_ptrs.data() : nullptr;
  out->buffer = nb;
  out->n_new_consumed = n_admit;
  out->decode_iters = iters;
  out->tokens_generated = tokens_generated;
  out->prefill_tokens = prefill_tokens;
  out->reprefill_tokens = reprefill_tokens;
  out->n_preempted = n_preempted;
  out->sum_live = sum_live;
  out->sum_ctx = sum_ctx;
  out->dec_sum_live = sum_live - it1_live;
  out->dec_sum_ctx = sum_ctx - it1_ctx;
  out->dec_sum_experts = sum_experts - it1_experts;
  out->t_prefill_s = t_prefill;
  out->t_decode_s = t_decode;
  out->t_total_s = now_s() - t_begin;
  return APRIL_OK;
  };   // body

  const int rc = body();
  if (rc == APRIL_OK) return rc;

  // ---- rollback of a failed step ----------------------------------------------------------
  const std::string first_error = c->err;
  c->prof_now = false;
  c->prof_recs.clear(); c->ev_used = 0; c->snaps_used = 0;
  {
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) == hipSuccess && cs != hipStreamCaptureStatusNone) {
      hipGraph_t g = nullptr;
      hipStreamEndCapture(st, &g);
      if (g) hipGraphDestroy(g);
    }
  }
  if (nb) { retire_buffer(c, nb); nb = nullptr; }
  c->r_req.clear(); c->r_tokens.clear(); c->r_ntok.clear(); c->r_nres.clear(); c->r_tok_ptrs.clear();
  c->r_logprobs.clear(); c->r_lp_ptrs.clear(); c->r_group.clear();
  const int S = c->n_slots;
  bool dev_ok = hipStreamSynchronize(st) == hipSuccess;
  std::vector<int> dgen(S), dstate(S), dnb(S);
  if (device_touched) {
    dev_ok = dev_ok && hipMemcpy(dgen.data(), c->ds.gen, S * sizeof(int), hipMemcpyDeviceToHost) == hipSuccess &&
             hipMemcpy(dstate.data(), c->ds.state, S * sizeof(int), hipMemcpyDeviceToHost) == hipSuccess &&
             hipMemcpy(dnb.data(), c->ds.n_blocks, S * sizeof(int), hipMemcpyDeviceToHost) == hipSuccess &&
             hipMemcpy(c->h_ctrl, c->d_ctrl, sizeof(Ctrl), hipMemcpyDeviceToHost) == hipSuccess;
    if (dev_ok) {
      // the device's view is the current one: progress made before the failure is kept, the KV
      // of every rollout that was in flight is released (after an error it is not trusted)
      c->free_pages_host = c->h_ctrl->free_top;
      for (int s : inflight) c->slots[s].n_blocks = dnb[s];
      dev_ok = free_slot_pages(c, inflight) == APRIL_OK;
    }
    // (if the device is gone the host mirrors are at least kept consistent)
    for (int s : inflight) { c->slots[s].n_blocks = 0; c->slots[s].kv_len = 0; }
  }
  for (Entry& e : deliver) c->pending.push_back(std::move(e));
  for (Entry& e : stay) c->pending.push_back(std::move(e));
  for (Entry& e : waiting) c->pending.push_back(std::move(e));
  for (int k = 0; k < (int)inflight.size(); ++k) {
    const int s = inflight[k];
    SlotH& sh = c->slots[s];
    if (k >= n_resumed_inflight) { sh = SlotH(); continue; }        // a new request: not consumed, the caller still has it
    const bool have_dev = device_touched && dev_ok;
    if (!have_dev) {
      // nothing ran on the device for this step: entries that came as tokens go back as tokens
      auto tl = std::find_if(token_level.begin(), token_level.end(), [&](const std::pair<int, Entry>& x) { return x.first == s; });
      if (tl != token_level.end()) { c->pending.push_back(tl->second); sh = SlotH(); continue; }
    }
    Entry e;
    e.req = sh.req; e.slot = s; e.limit = sh.limit; e.group = sh.group;
    if (have_dev) { sh.gen = dgen[s]; e.done = dstate[s] == SLOT_DONE ? 1 : 0; }
    sh.n_resumes -= 1;
    e.n_resumes = sh.n_resumes;
    sh.state = e.done ? SLOT_DONE : SLOT_PARKED;
    c->pending.push_back(std::move(e));
  }
  c->have_pending = !c->pending.empty();
  c->err = first_error;
  return rc;
}

}  // extern "C"
