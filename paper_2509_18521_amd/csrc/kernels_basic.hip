// Scheduler, allocator, embedding, RMSNorm, rotary + KV append, reference attention,
// reference GEMM, SiLU*mul.  gfx950, wave64.
#include "kernels.h"

namespace april {

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ inline int wave_incl_scan(int v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int t = __shfl_up(v, off, 64);
    if (lane >= off) v += t;
  }
  return v;
}
template <typename T> __device__ inline float to_f32(T v) { return (float)v; }
template <typename T> __device__ inline T from_f32(float v) { return (T)v; }

// ---------------------------------------------------------------------------
// Scheduler: early termination, live-batch compaction, KV page allocation.
// One workgroup.  Runs at the start of every decode iteration:
//   - if the step already stopped: nothing;
//   - if finished >= N: raise stop, remember the iteration count (early termination,
//     Section 2.2, second item of the method);
//   - else rebuild the dense list of live rollouts (slot order) and give a fresh
//     KV page to every live rollout whose next position opens a new page.  If the
//     free pages do not cover that demand, the youngest live rollout (largest request
//     id) is preempted first, repeatedly: its pages return to the stack, it keeps its
//     tokens, stops for this step and is re-prefilled when resumed;
//   - if nothing is live and nothing waits for prefill, the step ends (fewer than N).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void sched_kernel(Ctrl* c, Slots s, int* row_slot, int* row_pos,
                                                     int* free_stack, int blk, int check_only, int row_cap,
                                                     int ctx_cap, int4* att_items, int att_split, int att_cap) {
  __shared__ int sh_a[16], sh_b[16], sh_err[16];
  __shared__ long long sh_ctx[16];
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const int stop = c->stop, finished = c->finished, n_target = c->n_target;
  const int n_slots = c->n_slots, iter = c->iter, inflight = c->inflight;
  int free_top = c->free_top;
  __shared__ int sh_need, sh_free, sh_pending;
  if (tid == 0) { sh_need = 0; sh_pending = 0; }
  __syncthreads();
  if (stop) return;
  if (finished >= n_target) {
    if (tid == 0) { c->stop = 1; c->stop_iter = iter; c->n_rows = 0; }
    return;
  }
  if (check_only) return;
  if (free_top < inflight) {
    // the pool may be short: count this iteration's page demand, preempt if it is
    int cnt = 0;
    for (int slot = tid; slot < n_slots; slot += 1024)
      if (s.state[slot] == SLOT_LIVE) {
        const int pos = s.kv_len[slot];
        cnt += (pos % blk == 0) && (pos / blk >= s.n_blocks[slot]);
      }
    if (cnt) atomicAdd(&sh_need, cnt);
    __syncthreads();
    if (tid == 0) {
      int need = sh_need, ft = free_top;
      while (need > ft) {
        int victim = -1;
        long long best = -1;
        for (int slot = 0; slot < n_slots; ++slot)
          if (s.state[slot] == SLOT_LIVE && s.req_id[slot] > best) { best = s.req_id[slot]; victim = slot; }
        if (victim < 0) break;
        const int pos = s.kv_len[victim], nb = s.n_blocks[victim];
        if ((pos % blk == 0) && (pos / blk >= nb)) --need;
        for (int j = 0; j < nb; ++j) free_stack[ft++] = s.block_table[(size_t)victim * s.max_blocks + j];
        s.n_blocks[victim] = 0;
        s.kv_len[victim] = 0;
        s.state[victim] = SLOT_PREEMPTED;
        s.finish_iter[victim] = c->n_preempted;      // order of preemption within the step
        c->n_preempted += 1;
      }
      sh_free = ft;
    }
    __syncthreads();
    free_top = sh_free;
  }
  int base_live = 0, base_need = 0, err = 0;
  long long ctx_sum = 0;
  for (int s0 = 0; s0 < n_slots; s0 += 1024) {
    const int slot = s0 + tid;
    int live = 0, need = 0, pos = 0;
    if (slot < n_slots) {
      const int stt = s.state[slot];
      if (stt == SLOT_LIVE) {
        live = 1;
        pos = s.kv_len[slot];
        need = (pos % blk == 0) && (pos / blk >= s.n_blocks[slot]);
      } else if (stt == SLOT_PREFILL) {
        sh_pending = 1;
      }
    }
    const int ia = wave_incl_scan(live), ib = wave_incl_scan(need);
    if (lane == 63) { sh_a[wid] = ia; sh_b[wid] = ib; }
    __syncthreads();
    int wa = 0, wb = 0, ta = 0, tb = 0;
    for (int w = 0; w < 16; ++w) {
      const int va = sh_a[w], vb = sh_b[w];
      if (w < wid) { wa += va; wb += vb; }
      ta += va; tb += vb;
    }
    __syncthreads();
    if (live) {
      const int r = base_live + wa + ia - 1;
      row_slot[r] = slot;
      row_pos[r] = pos;
      ctx_sum += pos + 1;
      if (pos + 1 > ctx_cap) err |= 2;       // the host sized this iteration's launches for shorter contexts
    }
    if (need) {
      const int idx = free_top - 1 - (base_need + wb + ib - 1);
      const int bi = pos / blk;
      if (idx < 0 || bi >= s.max_blocks) {
        err |= 1;
      } else {
        s.block_table[(size_t)slot * s.max_blocks + bi] = free_stack[idx];
        s.n_blocks[slot] = bi + 1;
      }
    }
    base_live += ta;
    base_need += tb;
  }
  // Work list of the decode attention: one item per (row, KV split), longest first.  Class 0 =
  // full splits, class 1 + j = last splits that are j 32nds of a split short of full; a
  // counting sort over the classes (shared-memory counters; the order inside a class does not
  // matter, every item's result is independent of where it runs).
  if (att_items != nullptr) {
    __shared__ int sh_hist[33], sh_cur[33];
    if (tid < 33) sh_hist[tid] = 0;
    __syncthreads();                                   // also: this workgroup's row_slot / row_pos stores are visible
    for (int r = tid; r < base_live; r += 1024) {
      const int ctx = row_pos[r] + 1;
      const int ns = (ctx + att_split - 1) / att_split, last = ctx - (ns - 1) * att_split;
      const int cl = 1 + (int)(((long long)(att_split - last) * 32) / att_split);
      if (ns > 1) atomicAdd(&sh_hist[0], ns - 1);
      atomicAdd(&sh_hist[cl], 1);
    }
    __syncthreads();
    if (tid == 0) {
      int acc = 0;
      for (int i = 0; i < 33; ++i) { sh_cur[i] = acc; acc += sh_hist[i]; }
      if (acc > att_cap) { acc = 0; err |= 2; }
      sh_hist[0] = acc;
      att_items[0] = make_int4(acc, 0, 0, 0);
    }
    __syncthreads();
    if (sh_hist[0] > 0) {
      for (int r = tid; r < base_live; r += 1024) {
        const int pos = row_pos[r], slot = row_slot[r], ctx = pos + 1;
        const int ns = (ctx + att_split - 1) / att_split, last = ctx - (ns - 1) * att_split;
        const int cl = 1 + (int)(((long long)(att_split - last) * 32) / att_split);
        if (ns > 1) {
          const int p0 = atomicAdd(&sh_cur[0], ns - 1);
          for (int j = 0; j < ns - 1; ++j) att_items[1 + p0 + j] = make_int4(r, j, slot, pos);
        }
        att_items[1 + atomicAdd(&sh_cur[cl], 1)] = make_int4(r, ns - 1, slot, pos);
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    ctx_sum += __shfl_xor(ctx_sum, off, 64);
    err |= __shfl_xor(err, off, 64);
  }
  if (lane == 0) { sh_ctx[wid] = ctx_sum; sh_err[wid] = err; }
  __syncthreads();
  if (tid == 0) {
    long long tot = 0; int e = 0;
    for (int w = 0; w < 16; ++w) { tot += sh_ctx[w]; e |= sh_err[w]; }
    c->n_rows = base_live;
    c->free_top = free_top - base_need < 0 ? 0 : free_top - base_need;
    if (base_live == 0 && !sh_pending) {
      c->stop = 1;                 // nothing left in flight: the step ends short of N
      c->stop_iter = iter;
    } else {
      c->iter = iter + 1;
      c->sum_live += base_live;
      c->sum_ctx += tot;
      c->iter_ctx = tot;
    }
    if (base_live > row_cap) e |= 2;         // ... or for fewer rows
    if (e) { c->error = e; c->stop = 1; c->stop_iter = iter; c->n_rows = 0; }
  }
}

void launch_sched(hipStream_t st, Ctrl* ctrl, Slots s, int* row_slot, int* row_pos, int* free_stack, int blk,
                  int check_only, int row_cap, int ctx_cap, int4* att_items, int att_split, int att_cap) {
  hipLaunchKernelGGL(sched_kernel, dim3(1), dim3(1024), 0, st, ctrl, s, row_slot, row_pos, free_stack, blk,
                     check_only, row_cap, ctx_cap, att_items, att_split, att_cap);
}

// Pages for freshly admitted rollouts (prefill): slot_list[i] gets need[i] pages.
__global__ __launch_bounds__(256) void alloc_prefill_kernel(Ctrl* c, Slots s, const int* slot_list,
                                                            const int* need, int n, int* free_stack) {
  __shared__ int s_off[2049];
  const int free_top = c->free_top;
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int i = 0; i < n; ++i) { s_off[i] = acc; acc += need[i]; }
    s_off[n] = acc;
  }
  __syncthreads();
  const int total = s_off[n];
  if (total > free_top) { if (threadIdx.x == 0) c->error = 1; return; }
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const int slot = slot_list[i], nb = need[i];
    if (nb > s.max_blocks) { c->error = 1; continue; }
    for (int j = 0; j < nb; ++j)
      s.block_table[(size_t)slot * s.max_blocks + j] = free_stack[free_top - 1 - (s_off[i] + j)];
    s.n_blocks[slot] = nb;
  }
  __syncthreads();
  if (threadIdx.x == 0) c->free_top = free_top - total;
}
void launch_alloc_prefill(hipStream_t st, Ctrl* ctrl, Slots s, const int* slot_list, const int* need, int n,
                          int* free_stack) {
  if (n <= 0) return;
  hipLaunchKernelGGL(alloc_prefill_kernel, dim3(1), dim3(256), 0, st, ctrl, s, slot_list, need, n, free_stack);
}

// Return every page of the listed slots to the stack.
__global__ __launch_bounds__(256) void free_slots_kernel(Ctrl* c, Slots s, const int* slot_list, int n,
                                                         int* free_stack) {
  __shared__ int s_off[2049];
  const int free_top = c->free_top;
  if (threadIdx.x == 0) {
    int acc = 0;
    for (int i = 0; i < n; ++i) { s_off[i] = acc; acc += s.n_blocks[slot_list[i]]; }
    s_off[n] = acc;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) {
    const int slot = slot_list[i], nb = s.n_blocks[slot];
    for (int j = 0; j < nb; ++j)
      free_stack[free_top + s_off[i] + j] = s.block_table[(size_t)slot * s.max_blocks + j];
  }
  __syncthreads();
  for (int i = threadIdx.x; i < n; i += blockDim.x) { s.n_blocks[slot_list[i]] = 0; s.kv_len[slot_list[i]] = 0; }
  if (threadIdx.x == 0) c->free_top = free_top + s_off[n];
}
void launch_free_slots(hipStream_t st, Ctrl* ctrl, Slots s, const int* slot_list, int n, int* free_stack) {
  if (n <= 0) return;
  hipLaunchKernelGGL(free_slots_kernel, dim3(1), dim3(256), 0, st, ctrl, s, slot_list, n, free_stack);
}

// The free stack starts as a permutation that puts successive pops far apart: pop j hands out
// page (j * stride) mod n with stride ~ 0.618 n, coprime to n.  A prompt takes its pages in
// one go, and a row whose pages are consecutive in memory streams slower (the attention's
// load pattern alone: 5.4 TB/s against 6.0-6.1 TB/s for scattered or interleaved pages).
__global__ void free_stack_init_kernel(int* p, int n, int stride) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = (int)(((long long)(n - 1 - i) * stride) % n);     // the top of the stack is popped first
}
void launch_init_free_stack(hipStream_t st, int* free_stack, int n_blocks) {
  int stride = (int)((double)n_blocks * 0.6180339887) | 1;
  auto gcd = [](int a, int b) { while (b) { const int t = a % b; a = b; b = t; } return a; };
  while (stride < n_blocks && gcd(stride, n_blocks) != 1) stride += 2;
  if (stride >= n_blocks) stride = 1;
  hipLaunchKernelGGL(free_stack_init_kernel, dim3(ceil_div(n_blocks, 256)), dim3(256), 0, st, free_stack, n_blocks, stride);
}
__global__ void fill_i32_kernel(int* p, int v, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
void launch_fill_i32(hipStream_t st, int* p, int v, size_t n) {
  if (n == 0) return;
  size_t blocks = (n + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, v, n);
}

// ---------------------------------------------------------------------------
// Embedding gather: x_res[r] = E[token at (slot, pos)]
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void embed_kernel(RowCtx rc, Slots s, const T* emb, float* x_res, int d) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int slot = rc.row_slot[r], pos = rc.row_pos[r];
  const int tok = s.tokens[(size_t)slot * s.max_ctx + pos];
  const T* e = emb + (size_t)tok * d;
  for (int i = threadIdx.x; i < d; i += blockDim.x) x_res[(size_t)r * d + i] = to_f32(e[i]);
}
template <typename T>
void launch_embed(hipStream_t st, RowCtx rc, Slots s, const T* emb, float* x_res, int d) {
  hipLaunchKernelGGL(embed_kernel<T>, dim3(rc.max_rows), dim3(256), 0, st, rc, s, emb, x_res, d);
}
template void launch_embed<float>(hipStream_t, RowCtx, Slots, const float*, float*, int);
template void launch_embed<bf16_t>(hipStream_t, RowCtx, Slots, const bf16_t*, float*, int);

// ---------------------------------------------------------------------------
// Residual add (deterministic sum of split-K partials) + RMSNorm.
// One workgroup per output row; each thread owns up to 4 chunks of 8 columns.
// ---------------------------------------------------------------------------
template <typename T, bool XF, int NP>
__global__ __launch_bounds__(256) void add_rmsnorm_kernel(RowCtx rc, float* x_res, const float* partials,
                                                          int n_partials_rt, size_t partial_stride,
                                                          const float* gain, T* h, int d, float eps,
                                                          const int* gather, const int* pos_of,
                                                          const float* wts, T* h_rows) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int rin = gather ? gather[r] : r;
  __shared__ float sh[4];
  float v[4][8];
  float ss = 0.f;
  const int nchunk = d >> 3;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int ch = threadIdx.x + c * 256;
    if (ch < nchunk) {
      float* xp = x_res + (size_t)rin * d + ch * 8;
      // NP >= 0: compile-time partial count, every load issued before the first add
      const int n_partials = NP >= 0 ? NP : n_partials_rt;
      f32x4 xv[2] = {*reinterpret_cast<const f32x4*>(xp), *reinterpret_cast<const f32x4*>(xp + 4)};
      if (NP >= 0) {
        f32x4 pv[NP > 0 ? NP : 1][2];
        float pw[NP > 0 ? NP : 1];
#pragma unroll
        for (int p = 0; p < NP; ++p) {
          const float* pp = pos_of ? partials + (size_t)pos_of[(size_t)rin * NP + p] * d + ch * 8
                                   : partials + p * partial_stride + (size_t)rin * d + ch * 8;
          pw[p] = wts ? wts[(size_t)rin * NP + p] : 1.0f;
          pv[p][0] = *reinterpret_cast<const f32x4*>(pp);
          pv[p][1] = *reinterpret_cast<const f32x4*>(pp + 4);
        }
#pragma unroll
        for (int p = 0; p < NP; ++p) { xv[0] += pv[p][0] * pw[p]; xv[1] += pv[p][1] * pw[p]; }
      } else {
        for (int p = 0; p < n_partials; ++p) {
          const float* pp = partials + p * partial_stride + (size_t)rin * d + ch * 8;
          xv[0] += *reinterpret_cast<const f32x4*>(pp);
          xv[1] += *reinterpret_cast<const f32x4*>(pp + 4);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) v[c][j] = xv[j >> 2][j & 3];
      if (n_partials > 0) {
#pragma unroll
        for (int j = 0; j < 8; ++j) xp[j] = v[c][j];
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) ss += v[c][j] * v[c][j];
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = sh[0] + sh[1] + sh[2] + sh[3];
  const float rinv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int ch = threadIdx.x + c * 256;
    if (ch < nchunk) {
      T* hp = h + act_index<XF>(r, ch * 8, d);
      T hv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) hv[j] = from_f32<T>(v[c][j] * rinv * gain[ch * 8 + j]);
#pragma unroll
      for (int j = 0; j < 8; ++j) hp[j] = hv[j];
      if (h_rows != nullptr) {           // second copy, plain [row][d]: rows that a later kernel gathers one by one
        T* rp = h_rows + (size_t)r * d + ch * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) rp[j] = hv[j];
      }
    }
  }
}
template <typename T, bool XF>
void launch_add_rmsnorm(hipStream_t st, RowCtx rc, float* x_res, const float* partials, int n_partials,
                        size_t partial_stride, const float* gain, T* h, int d, float eps, const int* gather,
                        const int* pos_of, const float* wts, T* h_rows) {
#define ARN_CASE(NP)                                                                                          \
  hipLaunchKernelGGL((add_rmsnorm_kernel<T, XF, NP>), dim3(rc.max_rows), dim3(256), 0, st, rc, x_res, partials, \
                     n_partials, partial_stride, gain, h, d, eps, gather, pos_of, wts, h_rows)
  switch (n_partials) {
    case 0: ARN_CASE(0); break;
    case 1: ARN_CASE(1); break;
    case 2: ARN_CASE(2); break;
    case 3: ARN_CASE(3); break;
    case 4: ARN_CASE(4); break;
    case 5: ARN_CASE(5); break;
    case 6: ARN_CASE(6); break;
    case 7: ARN_CASE(7); break;
    case 8: ARN_CASE(8); break;
    default: ARN_CASE(-1); break;
  }
#undef ARN_CASE
}
template void launch_add_rmsnorm<float, false>(hipStream_t, RowCtx, float*, const float*, int, size_t, const float*, float*, int, float, const int*, const int*, const float*, float*);
template void launch_add_rmsnorm<bf16_t, true>(hipStream_t, RowCtx, float*, const float*, int, size_t, const float*, bf16_t*, int, float, const int*, const int*, const float*, bf16_t*);

// ---------------------------------------------------------------------------
// Rotary tables, computed once in double precision: cos/sin[pos][i], i < head_dim/2,
// angle = pos * theta^(-2i/head_dim).
// ---------------------------------------------------------------------------
__global__ void rope_table_kernel(float* cos_t, float* sin_t, int max_pos, int head_dim, float theta) {
  const int half = head_dim / 2;
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)max_pos * half) return;
  const int pos = (int)(idx / half), i = (int)(idx % half);
  const double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)head_dim);
  cos_t[idx] = (float)cos(ang);
  sin_t[idx] = (float)sin(ang);
}
void launch_rope_table(hipStream_t st, float* cos_t, float* sin_t, int max_pos, int head_dim, float theta) {
  const size_t n = (size_t)max_pos * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, cos_t, sin_t,
                     max_pos, head_dim, theta);
}

// ---------------------------------------------------------------------------
// Rotary embedding of q and k, append of k and v to the paged cache.
// qkv: fp32 [n_partials][rows][(Hq + 2 Hkv) * dh]
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void rope_append_kernel(RowCtx rc, Slots s, const float* qkv, int n_partials,
                                                          size_t partial_stride, const float* rope_cos,
                                                          const float* rope_sin, float* q_rot, T* kv_pool,
                                                          KVLayout L, int layer, int Hq) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int slot = rc.row_slot[r], pos = rc.row_pos[r];
  const int dh = L.head_dim, half = dh >> 1, Hkv = L.n_kv_heads;
  const int nq = Hq * dh, nkv = Hkv * dh, ncol = nq + 2 * nkv;
  const int page = s.block_table[(size_t)slot * s.max_blocks + pos / L.blk], t = pos % L.blk;
  const float* src = qkv + (size_t)r * ncol;
  const float* cs = rope_cos + (size_t)pos * half;
  const float* sn = rope_sin + (size_t)pos * half;
  auto val = [&](int col) {
    float a = src[col];
    for (int p = 1; p < n_partials; ++p) a += src[p * partial_stride + col];
    return a;
  };
  // rotations: Hq + Hkv heads, `half` pairs each
  for (int e = threadIdx.x; e < (Hq + Hkv) * half; e += blockDim.x) {
    const int hd = e / half, i = e % half;
    const float a = val(hd * dh + i), b = val(hd * dh + i + half);
    const float c = cs[i], sI = sn[i];
    const float ra = rope_first(a, b, c, sI), rb = rope_second(a, b, c, sI);
    if (hd < Hq) {
      q_rot[(size_t)r * nq + hd * dh + i] = ra;
      q_rot[(size_t)r * nq + hd * dh + i + half] = rb;
    } else {
      const int kh = hd - Hq;
      kv_pool[L.at(layer, 0, page, kh, t, i)] = from_f32<T>(ra);
      kv_pool[L.at(layer, 0, page, kh, t, i + half)] = from_f32<T>(rb);
    }
  }
  for (int e = threadIdx.x; e < nkv; e += blockDim.x) {
    const int kh = e / dh, i = e % dh;
    kv_pool[L.at(layer, 1, page, kh, t, i)] = from_f32<T>(val(nq + nkv + e));
  }
}
template <typename T>
void launch_rope_append(hipStream_t st, RowCtx rc, Slots s, const float* qkv, int n_partials, size_t partial_stride,
                        const float* rope_cos, const float* rope_sin, float* q_rot, T* kv_pool, KVLayout kvl,
                        int layer, int n_q_heads) {
  hipLaunchKernelGGL(rope_append_kernel<T>, dim3(rc.max_rows), dim3(256), 0, st, rc, s, qkv, n_partials,
                     partial_stride, rope_cos, rope_sin, q_rot, kv_pool, kvl, layer, n_q_heads);
}
template void launch_rope_append<float>(hipStream_t, RowCtx, Slots, const float*, int, size_t, const float*, const float*, float*, float*, KVLayout, int, int);
template void launch_rope_append<bf16_t>(hipStream_t, RowCtx, Slots, const float*, int, size_t, const float*, const float*, float*, bf16_t*, KVLayout, int, int);

// ---------------------------------------------------------------------------
// Reference paged attention: one wavefront per (row, query head), one cached token
// per loop trip, online softmax.  Correctness path (fp32 configuration, bring-up).
// ---------------------------------------------------------------------------
template <typename T, bool XF>
__global__ __launch_bounds__(64) void attn_ref_kernel(RowCtx rc, Slots s, const float* q_rot, const T* kv_pool,
                                                      KVLayout L, int layer, int Hq, T* out) {
  const int r = blockIdx.x, a = blockIdx.y;
  ROW_GUARD(rc, r);
  const int slot = rc.row_slot[r], pos = rc.row_pos[r];
  const int ctx = pos + 1, dh = L.head_dim, lane = threadIdx.x;
  const int kvh = a / (Hq / L.n_kv_heads);
  const float* q = q_rot + (size_t)r * Hq * dh + a * dh;
  const bool has0 = lane < dh, has1 = lane + 64 < dh;
  const float q0 = has0 ? q[lane] : 0.f, q1 = has1 ? q[lane + 64] : 0.f;
  const float scale = 1.0f / sqrtf((float)dh);
  const int* bt = s.block_table + (size_t)slot * s.max_blocks;
  float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
  for (int j = 0; j < ctx; ++j) {
    const int page = bt[j / L.blk], t = j % L.blk;
    float part = 0.f;
    if (has0) part += q0 * to_f32(kv_pool[L.at(layer, 0, page, kvh, t, lane)]);
    if (has1) part += q1 * to_f32(kv_pool[L.at(layer, 0, page, kvh, t, lane + 64)]);
    const float sc = wave_sum(part) * scale;
    const float m_new = fmaxf(m, sc);
    const float corr = expf(m - m_new), p = expf(sc - m_new);
    l = l * corr + p;
    if (has0) o0 = o0 * corr + p * to_f32(kv_pool[L.at(layer, 1, page, kvh, t, lane)]);
    if (has1) o1 = o1 * corr + p * to_f32(kv_pool[L.at(layer, 1, page, kvh, t, lane + 64)]);
    m = m_new;
  }
  const int K = Hq * dh;
  if (has0) out[act_index<XF>(r, a * dh + lane, K)] = from_f32<T>(o0 / l);
  if (has1) out[act_index<XF>(r, a * dh + lane + 64, K)] = from_f32<T>(o1 / l);
}
template <typename T, bool XF>
void launch_attn_ref(hipStream_t st, RowCtx rc, Slots s, const float* q_rot, const T* kv_pool, KVLayout kvl,
                     int layer, int n_q_heads, T* out) {
  hipLaunchKernelGGL((attn_ref_kernel<T, XF>), dim3(rc.max_rows, n_q_heads), dim3(64), 0, st, rc, s, q_rot,
                     kv_pool, kvl, layer, n_q_heads, out);
}
template void launch_attn_ref<float, false>(hipStream_t, RowCtx, Slots, const float*, const float*, KVLayout, int, int, float*);
template void launch_attn_ref<bf16_t, true>(hipStream_t, RowCtx, Slots, const float*, const bf16_t*, KVLayout, int, int, bf16_t*);

// ---------------------------------------------------------------------------
// act = silu(gate) * up from gu fp32 [rows][2F] (gate columns first, then up).
// ---------------------------------------------------------------------------
template <typename T, bool XF>
__global__ __launch_bounds__(256) void silu_mul_kernel(RowCtx rc, const float* gu, int F, T* act) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const float* g = gu + (size_t)r * 2 * F;
  for (int f = threadIdx.x; f < F; f += blockDim.x) {
    const float x = g[f];
    act[act_index<XF>(r, f, F)] = from_f32<T>(x / (1.0f + expf(-x)) * g[F + f]);
  }
}
template <typename T, bool XF>
void launch_silu_mul(hipStream_t st, RowCtx rc, const float* gu, int F, T* act) {
  hipLaunchKernelGGL((silu_mul_kernel<T, XF>), dim3(rc.max_rows), dim3(256), 0, st, rc, gu, F, act);
}
template void launch_silu_mul<float, false>(hipStream_t, RowCtx, const float*, int, float*);
template void launch_silu_mul<bf16_t, true>(hipStream_t, RowCtx, const float*, int, bf16_t*);

// ---------------------------------------------------------------------------
// Reference GEMM: out[m][n] = sum_k x[m][k] W[n][k], fp32 accumulate.
// One wavefront per output column n and 8 rows; lanes stride over k.
// ---------------------------------------------------------------------------
template <typename T, bool XF>
__global__ __launch_bounds__(256) void gemm_ref_kernel(RowCtx rc, const T* x, const T* W, float* out, int N, int K) {
  const int rows = rows_or_zero(rc);
  const int r0 = blockIdx.y * 8;
  if (r0 >= rows) return;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= N) return;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const T* w = W + (size_t)n * K;
  for (int k = lane; k < K; k += 64) {
    const float wv = to_f32(w[k]);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (r0 + j < rows) acc[j] += wv * to_f32(x[act_index<XF>(r0 + j, k, K)]);
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float v = wave_sum(acc[j]);
    if (lane == 0 && r0 + j < rows) out[(size_t)(r0 + j) * N + n] = v;
  }
}
template <typename T, bool XF>
void launch_gemm_ref(hipStream_t st, RowCtx rc, const T* x, const T* W, float* out, int N, int K) {
  hipLaunchKernelGGL((gemm_ref_kernel<T, XF>), dim3(ceil_div(N, 4), ceil_div(rc.max_rows, 8)), dim3(256), 0, st,
                     rc, x, W, out, N, K);
}
template void launch_gemm_ref<float, false>(hipStream_t, RowCtx, const float*, const float*, float*, int, int);
template void launch_gemm_ref<bf16_t, true>(hipStream_t, RowCtx, const bf16_t*, const bf16_t*, float*, int, int);

}  // namespace april
