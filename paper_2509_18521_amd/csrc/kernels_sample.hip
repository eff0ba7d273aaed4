// Sampler (greedy arg-max / top-k with Philox4x32-10) fused with the per-rollout
// state update: append the token, advance the generated length, detect completion
// and count it for the early-termination scheduler (Section 2.2).  One workgroup
// per sampling row.  gfx950.
#include "kernels.h"

namespace april {

#define SAMPLE_THREADS 1024
#define MAX_TOPK 64

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

__global__ __launch_bounds__(SAMPLE_THREADS) void sample_kernel(RowCtx rc, Slots s, Ctrl* ctrl,
                                                                const float* logits, int V, SamplerCfg sc,
                                                                Watch w, int update, const long long* req_ids,
                                                                const int* gen_idx, int* out_tokens) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int tid = threadIdx.x, lane = tid & 63, wid = tid >> 6;
  const float* lg = logits + (size_t)r * V;

  __shared__ unsigned hist[256];
  __shared__ unsigned s_prefix, s_krem, s_ntie;
  __shared__ int s_cnt, s_choice, s_watch_row;
  __shared__ unsigned cand_key[MAX_TOPK];
  __shared__ int cand_idx[MAX_TOPK];
  __shared__ float sort_logit[MAX_TOPK];
  __shared__ int sort_idx[MAX_TOPK];
  __shared__ unsigned red_key[16];
  __shared__ int red_idx[16];

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

  if (sc.kind == 0 || sc.top_k <= 1) {
    // ---- greedy: maximum, lowest index on ties --------------------------------
    unsigned bk = 0u; int bi = 0x7fffffff;
    for (int i = tid; i < V; i += SAMPLE_THREADS) {
      const unsigned k = f2key(lg[i]);
      if (bi == 0x7fffffff || k > bk) { bk = k; bi = i; }     // ascending i: first maximum stays
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const unsigned ok = __shfl_xor(bk, off, 64);
      const int oi = __shfl_xor(bi, off, 64);
      if (ok > bk || (ok == bk && oi < bi)) { bk = ok; bi = oi; }
    }
    if (lane == 0) { red_key[wid] = bk; red_idx[wid] = bi; }
    __syncthreads();
    if (tid == 0) {
      for (int x = 1; x < SAMPLE_THREADS / 64; ++x)
        if (red_key[x] > bk || (red_key[x] == bk && red_idx[x] < bi)) { bk = red_key[x]; bi = red_idx[x]; }
      s_choice = bi;
    }
    __syncthreads();
  } else {
    // ---- top-k: radix select of the k-th largest key, gather, sort, sample ---
    const int k = sc.top_k < V ? (sc.top_k < MAX_TOPK ? sc.top_k : MAX_TOPK) : (V < MAX_TOPK ? V : MAX_TOPK);
    if (tid == 0) { s_prefix = 0u; s_krem = (unsigned)k; }
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      const unsigned mask_hi = pass == 0 ? 0u : (0xFFFFFFFFu << (shift + 8));
      if (tid < 256) hist[tid] = 0u;
      __syncthreads();
      const unsigned prefix = s_prefix;
      for (int i = tid; i < V; i += SAMPLE_THREADS) {
        const unsigned key = f2key(lg[i]);
        if ((key & mask_hi) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
      }
      __syncthreads();
      if (tid == 0) {
        unsigned cum = 0u, krem = s_krem;
        for (int b = 255; b >= 0; --b) {
          if (cum + hist[b] >= krem) {
            s_prefix = prefix | ((unsigned)b << shift);
            s_krem = krem - cum;
            s_ntie = hist[b];
            break;
          }
          cum += hist[b];
        }
      }
      __syncthreads();
    }
    const unsigned thr = s_prefix;            // key of the k-th largest logit
    const int krem = (int)s_krem;             // how many entries equal to it are kept
    const int ntie = (int)s_ntie;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    for (int i = tid; i < V; i += SAMPLE_THREADS) {
      const unsigned key = f2key(lg[i]);
      if (key > thr || (key == thr && ntie == krem)) {
        const int p = atomicAdd(&s_cnt, 1);
        if (p < MAX_TOPK) { cand_key[p] = key; cand_idx[p] = i; }
      }
    }
    __syncthreads();
    if (ntie != krem) {
      // more ties at the threshold than places left: keep the lowest indices
      int last = -1;
      for (int t = 0; t < krem; ++t) {
        int best = 0x7fffffff;
        for (int i = tid; i < V; i += SAMPLE_THREADS)
          if (i > last && f2key(lg[i]) == thr) { best = i; break; }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) { const int o = __shfl_xor(best, off, 64); best = o < best ? o : best; }
        if (lane == 0) red_idx[wid] = best;
        __syncthreads();
        if (tid == 0) {
          for (int x = 1; x < SAMPLE_THREADS / 64; ++x) best = red_idx[x] < best ? red_idx[x] : best;
          const int p = s_cnt++;
          if (p < MAX_TOPK) { cand_key[p] = thr; cand_idx[p] = best; }
          red_idx[0] = best;
        }
        __syncthreads();
        last = red_idx[0];
        __syncthreads();
      }
    }
    const int n = s_cnt < MAX_TOPK ? s_cnt : MAX_TOPK;      // == k
    if (tid < n) {
      const unsigned mk = cand_key[tid]; const int mi = cand_idx[tid];
      int rank = 0;
      for (int j = 0; j < n; ++j) rank += (cand_key[j] > mk) || (cand_key[j] == mk && cand_idx[j] < mi);
      sort_logit[rank] = lg[mi];
      sort_idx[rank] = mi;
    }
    __syncthreads();
    if (tid == 0) {
      const unsigned long long rid = (unsigned long long)req;
      const unsigned w0 = philox4x32_10_word0((unsigned)(rid & 0xFFFFFFFFull), (unsigned)(rid >> 32),
                                              (unsigned)g, 0u, (unsigned)(sc.seed & 0xFFFFFFFFull),
                                              (unsigned)(sc.seed >> 32));
      const double u = (double)(w0 >> 8) * (1.0 / 16777216.0);
      const double T = (double)sc.temperature;
      const double z0 = (double)sort_logit[0] / T;
      double sum = 0.0;
      for (int j = 0; j < n; ++j) sum += exp((double)sort_logit[j] / T - z0);
      double c = 0.0;
      int choice = sort_idx[n - 1];
      for (int j = 0; j < n; ++j) {
        c += exp((double)sort_logit[j] / T - z0) / sum;
        if (c > u) { choice = sort_idx[j]; break; }
      }
      s_choice = choice;
    }
    __syncthreads();
  }

  const int sampled = s_choice;

  // ---- parity-mode capture ----------------------------------------------------
  if (w.req != nullptr && ctrl != nullptr) {
    if (tid == 0) {
      int row = -1;
      const int nw = ctrl->n_watch;
      for (int i = 0; i < nw; ++i)
        if (w.req[i] == req && g >= w.first[i] && g < w.first[i] + w.count[i]) row = w.row0[i] + (g - w.first[i]);
      s_watch_row = row;
    }
    __syncthreads();
    const int row = s_watch_row;
    if (row >= 0) {
      for (int i = tid; i < V; i += SAMPLE_THREADS) w.logits[(size_t)row * V + i] = lg[i];
      if (tid == 0) { w.sampled[row] = sampled; w.filled[row] = 1; }
    }
  }

  if (tid == 0) {
    if (!update) {
      out_tokens[r] = sampled;
    } else {
      int tok = sampled;
      if (s.forced != nullptr) {
        const int f = s.forced[(size_t)slot * s.max_ctx + g];
        if (f >= 0) tok = f;
      }
      s.tokens[(size_t)slot * s.max_ctx + pos + 1] = tok;
      s.gen[slot] = g + 1;
      s.kv_len[slot] = pos + 1;
      int stt = s.state[slot];
      if (stt == SLOT_PREFILL) stt = SLOT_LIVE;
      if (g + 1 >= s.limit[slot] || tok == ctrl->eos_token) {
        stt = SLOT_DONE;
        s.finish_iter[slot] = ctrl->iter;
        atomicAdd(&ctrl->finished, 1);
      }
      s.state[slot] = stt;
    }
  }
}

void launch_sample(hipStream_t st, RowCtx rc, Slots s, Ctrl* ctrl, const float* logits, int vocab, SamplerCfg sc,
                   Watch w, int update, const long long* req_ids, const int* gen_idx, int* out_tokens) {
  hipLaunchKernelGGL(sample_kernel, dim3(rc.max_rows), dim3(SAMPLE_THREADS), 0, st, rc, s, ctrl, logits, vocab,
                     sc, w, update, req_ids, gen_idx, out_tokens);
}

}  // namespace april
