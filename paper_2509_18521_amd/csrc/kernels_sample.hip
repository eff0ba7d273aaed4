// Sampler (greedy arg-max / top-k with Philox4x32-10) fused with the per-rollout
// state update: append the token, advance the generated length, detect completion
// and count it for the early-termination scheduler (Section 2.2).  One workgroup
// per sampling row.  gfx950.
//
// Top-k is exact: the k largest logits, ties broken by lower index, in descending
// order.  When the LM-head GEMM has left the maximum of every group of 64 logits, the
// k-th largest group maximum is a lower bound of the k-th largest logit (each group
// maximum is a logit), so only the groups whose maximum reaches it are read again.
// Without group maxima (or if a candidate list overflows) a 4-pass radix select over
// the whole row is used.
#include "kernels.h"

namespace april {

#define SAMPLE_THREADS 1024
#define MAX_TOPK 64
#define MAX_HOT 1024
#define MAX_CAND 2048

// Order-preserving map float -> unsigned (larger float <=> larger key); -0 == +0.
__device__ inline unsigned f2key(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Philox4x32-10 (Salmon et al., SC'11): first output word.
__device__ inline unsigned philox4x32_10_word0(unsigned c0, unsigned c1, unsigned c2, unsigned c3,
                                               unsigned k0, unsigned k1) {
  const unsigned M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const unsigned hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const unsigned n0 = hi1 ^ c1 ^ k0, n1 = lo1, n2 = hi0 ^ c3 ^ k1, n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += W0; k1 += W1;
  }
  return c0;
}

struct SampleShared {
  unsigned hist[256];
  unsigned prefix, krem, ntie;
  int cnt, choice, watch_row, n_hot, overflow;
  unsigned cand_key[MAX_CAND];
  int cand_idx[MAX_CAND];
  int hot[MAX_HOT];
  float sort_logit[MAX_TOPK];
  int sort_idx[MAX_TOPK];
  unsigned red_key[16];
  int red_idx[16];
  double red_d[16];
  float red_f[16];
  double total_d;
  float max_f;
};

// Block-wide maximum of vals[0..n) (all threads call; result in every thread).
__device__ inline float block_max_f32(const float* vals, int n, SampleShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  float m = -INFINITY;
  for (int i = tid; i < n; i += SAMPLE_THREADS) m = fmaxf(m, vals[i]);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  __syncthreads();
  if (lane == 0) sh.red_f[wid] = m;
  __syncthreads();
  if (tid == 0) {
    for (int x = 1; x < SAMPLE_THREADS / 64; ++x) m = fmaxf(m, sh.red_f[x]);
    sh.max_f = m;
  }
  __syncthreads();
  return sh.max_f;
}
// Block-wide sum of one double per thread (all threads call; result in every thread), added
// in a fixed order: lanes by the shuffle tree, wavefronts in index order.
__device__ inline double block_sum_f64(double v, SampleShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  __syncthreads();
  if (lane == 0) sh.red_d[wid] = v;
  __syncthreads();
  if (tid == 0) {
    double t = sh.red_d[0];
    for (int x = 1; x < SAMPLE_THREADS / 64; ++x) t += sh.red_d[x];
    sh.total_d = t;
  }
  __syncthreads();
  return sh.total_d;
}

// Key of the k-th largest of vals[0..n) (k <= n): 4 radix passes of 8 bits.  On return
// sh.prefix = that key, sh.krem = how many entries equal to it belong to the top k,
// sh.ntie = how many entries equal it.  All threads must call.  Up to 4 keys per thread are
// kept in registers across the passes (n <= 4 * SAMPLE_THREADS reads memory once).
__device__ inline void block_kth_largest(const float* vals, int n, int k, SampleShared& sh) {
  const int tid = threadIdx.x;
  const bool cached = n <= 4 * SAMPLE_THREADS;
  unsigned ck[4] = {0u, 0u, 0u, 0u};
  if (cached) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int i = tid + q * SAMPLE_THREADS;
      if (i < n) ck[q] = f2key(vals[i]);
    }
  }
  if (tid == 0) { sh.prefix = 0u; sh.krem = (unsigned)k; }
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const unsigned mask_hi = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
    if (tid < 256) sh.hist[tid] = 0u;
    __syncthreads();
    const unsigned prefix = sh.prefix;
    if (cached) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (tid + q * SAMPLE_THREADS < n && (ck[q] & mask_hi) == prefix) atomicAdd(&sh.hist[(ck[q] >> shift) & 255u], 1u);
    } else {
      for (int i = tid; i < n; i += SAMPLE_THREADS) {
        const unsigned key = f2key(vals[i]);
        if ((key & mask_hi) == prefix) atomicAdd(&sh.hist[(key >> shift) & 255u], 1u);
      }
    }
    __syncthreads();
    if (tid < 64) {
      // Wavefront 0 walks the histogram from the top: lane l owns bins 4l..4l+3; `above` =
      // entries in higher bins.  The one lane with above < krem <= above + own holds the digit.
      const unsigned krem = sh.krem;
      const unsigned h0 = sh.hist[4 * tid], h1 = sh.hist[4 * tid + 1], h2 = sh.hist[4 * tid + 2], h3 = sh.hist[4 * tid + 3];
      const unsigned own = h0 + h1 + h2 + h3;
      unsigned suf = own;                                   // inclusive suffix sum over lanes >= tid
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const unsigned o = __shfl_down(suf, off, 64);
        if (tid + off < 64) suf += o;
      }
      const unsigned above = suf - own;
      if (above < krem && krem <= above + own) {
        unsigned cum = above;
        const unsigned hs[4] = {h3, h2, h1, h0};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          if (cum + hs[q] >= krem) {
            sh.prefix = prefix | ((unsigned)(4 * tid + 3 - q) << shift);
            sh.krem = krem - cum;
            sh.ntie = hs[q];
            break;
          }
          cum += hs[q];
        }
      }
    }
    __syncthreads();
  }
}

// Block arg-max with lowest index on ties over vals[idx0 + i*stride...]: generic helper.
__device__ inline int block_argmax(const float* vals, int n, SampleShared& sh) {
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  unsigned bk = 0u;
  int bi = 0x7fffffff;
  for (int i = tid; i < n; i += SAMPLE_THREADS) {
    const unsigned k = f2key(vals[i]);
    if (bi == 0x7fffffff || k > bk) { bk = k; bi = i; }     // ascending i: first maximum stays
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned ok = __shfl_xor(bk, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (ok > bk || (ok == bk && oi < bi)) { bk = ok; bi = oi; }
  }
  __syncthreads();
  if (lane == 0) { sh.red_key[wid] = bk; sh.red_idx[wid] = bi; }
  __syncthreads();
  if (tid == 0) {
    for (int x = 1; x < SAMPLE_THREADS / 64; ++x)
      if (sh.red_key[x] > bk || (sh.red_key[x] == bk && sh.red_idx[x] < bi)) { bk = sh.red_key[x]; bi = sh.red_idx[x]; }
    sh.choice = bi;
  }
  __syncthreads();
  return sh.choice;
}

__global__ __launch_bounds__(SAMPLE_THREADS) void sample_kernel(RowCtx rc, Slots s, Ctrl* ctrl,
                                                                const float* logits, int V, SamplerCfg sc,
                                                                Watch w, int update, const long long* req_ids,
                                                                const int* gen_idx, int* out_tokens,
                                                                const float* group_max, int group,
                                                                float* out_logprobs, const int* group_idx) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const float* lg = logits + (size_t)r * V;
  __shared__ SampleShared sh;

  int slot = -1, pos = 0, g = 0;
  long long req = 0;
  if (update) {
    slot = rc.row_slot[r];
    pos = rc.row_pos[r];
    g = s.gen[slot];
    req = s.req_id[slot];
  } else {
    req = req_ids[r];
    g = gen_idx[r];
  }
  const int n_groups = group_max ? V / group : 0;
  const float* gm = group_max ? group_max + (size_t)r * n_groups : nullptr;

  if (sc.kind == 0 || (sc.kind == 1 && sc.top_k <= 1)) {
    // ---- greedy: maximum, lowest index on ties --------------------------------------
    if (gm) {
      const int gi = block_argmax(gm, n_groups, sh);               // lowest group holding the maximum
      // the column inside the group: left by the LM head, else looked up in the logits
      const int li = group_idx ? group_idx[(size_t)r * n_groups + gi] : block_argmax(lg + (size_t)gi * group, group, sh);
      __syncthreads();
      if (tid == 0) sh.choice = gi * group + li;
      __syncthreads();
    } else {
      block_argmax(lg, V, sh);
    }
  } else if (sc.kind == 2) {
    // ---- temperature sampling over the whole vocabulary: inverse CDF in index order ----------
    // Thread t owns the indices [t * chunk, (t + 1) * chunk): its partial sum of exp((l - max) / T),
    // an exclusive scan over the threads (wavefront scans, then wavefront totals in order), and the
    // thread whose range holds the crossing of u * total walks its range.
    const float M = gm ? block_max_f32(gm, n_groups, sh) : block_max_f32(lg, V, sh);
    const double invT = 1.0 / (double)sc.temperature;
    const int chunk = (V + SAMPLE_THREADS - 1) / SAMPLE_THREADS;
    const int i0 = tid * chunk, i1 = (i0 + chunk < V) ? i0 + chunk : V;
    double part = 0.0;
    for (int i = i0; i < i1; ++i) part += exp(((double)lg[i] - (double)M) * invT);
    double incl = part;                                     // inclusive scan inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const double o = __shfl_up(incl, off, 64);
      if (lane >= off) incl += o;
    }
    __syncthreads();
    if (lane == 63) sh.red_d[wid] = incl;
    __syncthreads();
    double before = 0.0, total = 0.0;
    for (int x = 0; x < SAMPLE_THREADS / 64; ++x) {
      if (x < wid) before += sh.red_d[x];
      total += sh.red_d[x];
    }
    const unsigned long long rid = (unsigned long long)req;
    const unsigned w0 = philox4x32_10_word0((unsigned)(rid & 0xFFFFFFFFull), (unsigned)(rid >> 32),
                                            (unsigned)g, 0u, (unsigned)(sc.seed & 0xFFFFFFFFull),
                                            (unsigned)(sc.seed >> 32));
    const double u = (double)(w0 >> 8) * (1.0 / 16777216.0);
    const double target = u * total;                        // cumulative / total > u  <=>  cumulative > u * total
    const double lo = before + incl - part, hi = before + incl;
    if (tid == 0) sh.choice = V - 1;                        // rounding leaves no crossing: the last index
    __syncthreads();
    if (i0 < i1 && lo <= target && hi > target) {
      double c = lo;
      int pick = i1 - 1;
      for (int i = i0; i < i1; ++i) {
        c += exp(((double)lg[i] - (double)M) * invT);
        if (c > target) { pick = i; break; }
      }
      sh.choice = pick;
    }
    __syncthreads();
  } else {
    const int k = sc.top_k < V ? (sc.top_k < MAX_TOPK ? sc.top_k : MAX_TOPK) : (V < MAX_TOPK ? V : MAX_TOPK);
    bool have = false;
    if (gm && n_groups >= k) {
      // ---- candidates from the groups whose maximum reaches the k-th largest maximum ---
      block_kth_largest(gm, n_groups, k, sh);
      const unsigned tau = sh.prefix;
      if (tid == 0) { sh.n_hot = 0; sh.cnt = 0; sh.overflow = 0; }
      __syncthreads();
      for (int i = tid; i < n_groups; i += SAMPLE_THREADS)
        if (f2key(gm[i]) >= tau) {
          const int p = atomicAdd(&sh.n_hot, 1);
          if (p < MAX_HOT) sh.hot[p] = i; else sh.overflow = 1;
        }
      __syncthreads();
      if (!sh.overflow) {
        const int n_hot = sh.n_hot;
        for (int e = tid; e < n_hot * group; e += SAMPLE_THREADS) {
          const int idx = sh.hot[e / group] * group + e % group;
          const unsigned key = f2key(lg[idx]);
          if (key >= tau) {
            const int p = atomicAdd(&sh.cnt, 1);
            if (p < MAX_CAND) { sh.cand_key[p] = key; sh.cand_idx[p] = idx; } else sh.overflow = 1;
          }
        }
        __syncthreads();
        have = !sh.overflow;
      }
      __syncthreads();
    }
    if (!have) {
      // ---- radix select over the whole row ---------------------------------------------
      block_kth_largest(lg, V, k, sh);
      const unsigned thr = sh.prefix;
      const int krem = (int)sh.krem, ntie = (int)sh.ntie;
      if (tid == 0) sh.cnt = 0;
      __syncthreads();
      // everything above the threshold, plus the threshold ties with the lowest indices
      for (int i = tid; i < V; i += SAMPLE_THREADS) {
        const unsigned key = f2key(lg[i]);
        if (key > thr || (key == thr && ntie == krem)) {
          const int p = atomicAdd(&sh.cnt, 1);
          if (p < MAX_CAND) { sh.cand_key[p] = key; sh.cand_idx[p] = i; }
        }
      }
      __syncthreads();
      if (ntie != krem) {
        int last = -1;
        for (int t = 0; t < krem; ++t) {
          int best = 0x7fffffff;
          for (int i = tid; i < V; i += SAMPLE_THREADS)
            if (i > last && f2key(lg[i]) == thr) { best = i; break; }
#pragma unroll
          for (int off = 32; off > 0; off >>= 1) { const int o = __shfl_xor(best, off, 64); best = o < best ? o : best; }
          if (lane == 0) sh.red_idx[wid] = best;
          __syncthreads();
          if (tid == 0) {
            for (int x = 1; x < SAMPLE_THREADS / 64; ++x) best = sh.red_idx[x] < best ? sh.red_idx[x] : best;
            const int p = sh.cnt++;
            if (p < MAX_CAND) { sh.cand_key[p] = thr; sh.cand_idx[p] = best; }
            sh.red_idx[0] = best;
          }
          __syncthreads();
          last = sh.red_idx[0];
          __syncthreads();
        }
      }
    }
    // ---- exact top-k of the candidates: the rank of a candidate is its place in the
    // descending order (ties: lower index first) ------------------------------------------
    const int n_cand = sh.cnt < MAX_CAND ? sh.cnt : MAX_CAND;
    for (int c = tid; c < n_cand; c += SAMPLE_THREADS) {
      const unsigned mk = sh.cand_key[c];
      const int mi = sh.cand_idx[c];
      int rank = 0;
      for (int j = 0; j < n_cand; ++j) rank += (sh.cand_key[j] > mk) || (sh.cand_key[j] == mk && sh.cand_idx[j] < mi);
      if (rank < k) { sh.sort_logit[rank] = lg[mi]; sh.sort_idx[rank] = mi; }
    }
    __syncthreads();
    if (tid < 64) {
      // Wavefront 0: lane j holds candidate j (k <= 64).  fp64 softmax over the candidates and
      // its running sum; the token is the first candidate whose cumulative probability
      // exceeds the uniform draw, the last candidate if none does.
      const int n = n_cand < k ? n_cand : k;
      const unsigned long long rid = (unsigned long long)req;
      const unsigned w0 = philox4x32_10_word0((unsigned)(rid & 0xFFFFFFFFull), (unsigned)(rid >> 32),
                                              (unsigned)g, 0u, (unsigned)(sc.seed & 0xFFFFFFFFull),
                                              (unsigned)(sc.seed >> 32));
      const double u = (double)(w0 >> 8) * (1.0 / 16777216.0);
      const double T = (double)sc.temperature;
      const double z0 = (double)sh.sort_logit[0] / T;
      const double e = tid < n ? exp((double)sh.sort_logit[tid < n ? tid : 0] / T - z0) : 0.0;
      double sum = e;
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
      double c = e / sum;                                   // inclusive prefix sum over lanes <= tid
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const double o = __shfl_up(c, off, 64);
        if (tid >= off) c += o;
      }
      int keep = n;
      double tot = 1.0;
      if (sc.top_p > 0.f && sc.top_p < 1.f) {
        // nucleus: the shortest prefix whose cumulative probability reaches top_p
        const unsigned long long reach = __ballot(tid < n && c >= (double)sc.top_p);
        keep = reach ? __ffsll((long long)reach) : n;
        tot = __shfl(c, keep - 1, 64);                      // mass of the nucleus: renormalise by it
      }
      const unsigned long long hit = __ballot(tid < keep && c > u * tot);
      if (tid == 0) sh.choice = sh.sort_idx[hit ? __ffsll((long long)hit) - 1 : keep - 1];
    }
    __syncthreads();
  }

  const int sampled = sh.choice;

  // ---- parity-mode capture --------------------------------------------------------------
  if (w.req != nullptr && ctrl != nullptr) {
    if (tid == 0) {
      int row = -1;
      const int nw = ctrl->n_watch;
      for (int i = 0; i < nw; ++i)
        if (w.req[i] == req && g >= w.first[i] && g < w.first[i] + w.count[i]) row = w.row0[i] + (g - w.first[i]);
      sh.watch_row = row;
    }
    __syncthreads();
    const int row = sh.watch_row;
    if (row >= 0) {
      for (int i = tid; i < V; i += SAMPLE_THREADS) w.logits[(size_t)row * V + i] = lg[i];
      if (tid == 0) { w.sampled[row] = sampled; w.filled[row] = 1; }
    }
  }

  // the token that is appended: the sampler's choice, or the teacher-forced one (parity mode)
  int tok_final = sampled;
  if (update && s.forced != nullptr) {
    const int f = s.forced[(size_t)slot * s.max_ctx + g];
    if (f >= 0) tok_final = f;
  }
  // ---- log-probability of that token under softmax(logits / T) over the whole vocabulary ----
  float* lp_dst = update ? (s.logprob ? s.logprob + (size_t)slot * s.max_ctx + g : nullptr)
                         : (out_logprobs ? out_logprobs + r : nullptr);
  if (lp_dst != nullptr) {
    const float M = gm ? block_max_f32(gm, n_groups, sh) : block_max_f32(lg, V, sh);
    const float invT = 1.0f / sc.temperature;
    double part = 0.0;
    for (int i = tid; i < V; i += SAMPLE_THREADS) part += (double)__expf((lg[i] - M) * invT);
    const double Z = block_sum_f64(part, sh);
    if (tid == 0) *lp_dst = (float)((double)((lg[tok_final] - M) * invT) - log(Z));
  }

  if (tid == 0) {
    if (!update) {
      out_tokens[r] = sampled;
    } else {
      int tok = tok_final;
      s.tokens[(size_t)slot * s.max_ctx + pos + 1] = tok;
      s.gen[slot] = g + 1;
      s.kv_len[slot] = pos + 1;
      int stt = s.state[slot];
      if (stt == SLOT_PREFILL) stt = SLOT_LIVE;
      if (g + 1 >= s.limit[slot] || tok == ctrl->eos_token) {
        stt = SLOT_DONE;
        s.finish_iter[slot] = ctrl->iter;
        // what the scheduler counts toward N: the rollout, or (instance-level completion,
        // Section 3.2.3) its group once the last member is complete
        const int gi = s.group != nullptr ? s.group[slot] : -1;
        if (gi < 0) atomicAdd(&ctrl->finished, 1);
        else if (atomicSub(&s.grp_left[gi], 1) == 1) atomicAdd(&ctrl->finished, 1);
      }
      s.state[slot] = stt;
    }
  }
}

// Maxima of groups of `group` consecutive logits (what the LM-head GEMM epilogue leaves),
// for callers that bring their own logits.
__global__ __launch_bounds__(256) void group_max_kernel(const float* logits, int n_rows, int V, int group, float* out) {
  const int n_groups = V / group;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)n_rows * n_groups) return;
  const size_t r = i / n_groups, gi = i % n_groups;
  const float* p = logits + r * V + gi * group;
  float m = p[0];
  for (int j = 1; j < group; ++j) m = fmaxf(m, p[j]);
  out[i] = m;
}
void launch_group_max(hipStream_t st, const float* logits, int n_rows, int V, int group, float* out) {
  const size_t n = (size_t)n_rows * (V / group);
  hipLaunchKernelGGL(group_max_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, logits, n_rows, V, group, out);
}

void launch_sample(hipStream_t st, RowCtx rc, Slots s, Ctrl* ctrl, const float* logits, int vocab, SamplerCfg sc,
                   Watch w, int update, const long long* req_ids, const int* gen_idx, int* out_tokens,
                   const float* group_max, int group, float* out_logprobs, const int* group_idx) {
  hipLaunchKernelGGL(sample_kernel, dim3(rc.max_rows), dim3(SAMPLE_THREADS), 0, st, rc, s, ctrl, logits, vocab,
                     sc, w, update, req_ids, gen_idx, out_tokens, group_max, group, out_logprobs, group_idx);
}

}  // namespace april
