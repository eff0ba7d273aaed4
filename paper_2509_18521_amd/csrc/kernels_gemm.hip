// bf16 MFMA GEMM for skinny (decode) and tall (prefill) activations, gfx950.
//
// out[m][n] = sum_k x[m][k] * W[n][k].  Both operands are kept in the register
// layout of v_mfma_f32_32x32x16_bf16's 32x16 operand ("fragment-tiled"), so a
// wavefront fetches one fragment as 64 consecutive 16-byte pieces (1 KiB, fully
// coalesced) straight into VGPRs: the weight stream - the only HBM-sized traffic
// of a decode GEMM - is read exactly once, with no LDS staging.  The weight tile is
// the MFMA's A operand (rows = output features), the activation tile its B operand
// (columns = batch rows), so the accumulator holds out^T tiles:
//   lane l, register i  ->  n = 8*(i/4) + 4*(l/32) + i%4,  m = l%32.
#include "kernels.h"

namespace april {

__global__ __launch_bounds__(256) void shuffle_weights_kernel(const bf16_t* src, bf16x8* dst, int N, int K) {
  const size_t c = (size_t)blockIdx.x * blockDim.x + threadIdx.x;      // 16-byte piece index
  const size_t total = (size_t)N * K / 8;
  if (c >= total) return;
  const int KT = K >> 4;
  const size_t tile = c >> 6;
  const int lane = (int)(c & 63);
  const int nt = (int)(tile / KT), kt = (int)(tile % KT);
  const int row = nt * 32 + (lane & 31), k = kt * 16 + ((lane >> 5) << 3);
  dst[c] = *reinterpret_cast<const bf16x8*>(src + (size_t)row * K + k);
}
void launch_shuffle_weights(hipStream_t st, const bf16_t* src, bf16_t* dst, int N, int K) {
  const size_t total = (size_t)N * K / 8;
  hipLaunchKernelGGL(shuffle_weights_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, src,
                     reinterpret_cast<bf16x8*>(dst), N, K);
}

enum { EPI_F32 = 0, EPI_SWIGLU = 1, EPI_LOGITS = 2, EPI_RESID = 3 };

// RMSNorm folded into the GEMMs around it (decode).  The producer (EPI_RESID, the attention
// output projection) adds its result to the residual stream in place, writes the residual times
// the next norm's gain as the bf16 activations of the next GEMM, and leaves per row the sum of
// squares of its 32 columns (ssq[n_tile][row]).  The consumer (EPI_SWIGLU with ssq set) sums
// those partials in a fixed order and scales its accumulators by 1/sqrt(mean square + eps):
// W . (x g / rms) = (W . (x g)) / rms.  No separate normalisation launch in between.
struct NormFuse {
  const float* gain;     // producer: gain of the following norm [N]
  float* ssq;            // producer: out; consumer: in.  nullptr = not fused
  int ssq_stride;        // rows per n-tile slab
  int n_ssq;             // consumer: number of slabs (= d_model / 32)
  float inv_d, eps;      // consumer
};

constexpr int KW4 = 4;       // wavefronts of a workgroup (template parameter KW); they split the k range among themselves

// One workgroup: NT weight tiles x MTC activation tiles over k-tiles [k0, k1).  Each of
// the KW wavefronts accumulates a quarter of the k range, the partial accumulators are
// summed through LDS in a fixed tree order, wavefront 0 runs the epilogue.
template <int NT, int MTC, int EPI, bool INTRA, int KW>
__device__ inline void gemm_group(const bf16x8* __restrict__ w0, const bf16x8* __restrict__ w1,
                                  const bf16x8* __restrict__ x, int KT, int k0, int k1, int nt0, int mt0,
                                  int rows, int N, float* __restrict__ out, bf16_t* __restrict__ act,
                                  float* red, float* ssp, const NormFuse& nf) {
  // k-tiles per fetch group: two groups fill the register file (4 VGPRs per fragment).  The
  // next group is requested before the MFMAs of the current one, so a wavefront whose k range
  // fits in two groups has all of it in flight at once, and a longer range streams with one
  // group always in flight behind the arithmetic.
  constexpr int KH = (NT + MTC) <= 4 ? 8 : ((NT + MTC) == 5 ? 7 : ((NT + MTC) == 6 ? 5 : 3));
  // the wavefront index is uniform: keep it (and the k range derived from it) in scalar registers
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  f32x16 acc[NT][MTC];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MTC; ++j) acc[i][j] = f32x16{};

  const bf16x8* wp[NT];
  if (EPI == EPI_SWIGLU) {
    wp[0] = w0 + (size_t)nt0 * KT * 64 + lane;
    if (NT > 1) wp[NT - 1] = w1 + (size_t)nt0 * KT * 64 + lane;
  } else {
#pragma unroll
    for (int i = 0; i < NT; ++i) wp[i] = w0 + (size_t)(nt0 + i) * KT * 64 + lane;
  }
  const bf16x8* xp[MTC];
#pragma unroll
  for (int j = 0; j < MTC; ++j) xp[j] = x + (size_t)(mt0 + j) * KT * 64 + lane;

  const int len = k1 - k0;
  const int kb = INTRA ? k0 + (int)((long long)len * wave / KW) : k0;
  const int ke = INTRA ? k0 + (int)((long long)len * (wave + 1) / KW) : k1;
  // A group past the end re-reads the final k-tile (loads stay unconditional and in flight
  // together) and skips its MFMAs.
  bf16x8 a[2][KH][NT], b[2][KH][MTC];
  auto fetch = [&](int g, int kt) {
#pragma unroll
    for (int u = 0; u < KH; ++u) {
      const size_t k = (size_t)(kt + u < ke ? kt + u : ke - 1) * 64;
#pragma unroll
      for (int i = 0; i < NT; ++i) a[g][u][i] = wp[i][k];
#pragma unroll
      for (int j = 0; j < MTC; ++j) b[g][u][j] = xp[j][k];
    }
  };
  auto multiply = [&](int g, int kt) {
#pragma unroll
    for (int u = 0; u < KH; ++u) {
      if (kt + u < ke) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int j = 0; j < MTC; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[g][u][i], b[g][u][j], acc[i][j], 0, 0, 0);
      }
    }
  };
  // Fused norm (consumer side): wavefront w adds the slabs w, w + KW, ... of its rows, wavefront
  // 0 later adds the four sums.  The first 8 slabs per wavefront are requested here and summed
  // after the k loop, so their latency hides behind the operand stream.
  constexpr bool NORM_IN = (EPI == EPI_SWIGLU || EPI == EPI_F32) && INTRA;
  float sq[NORM_IN ? MTC : 1][8];
  if (NORM_IN && nf.ssq != nullptr) {
#pragma unroll
    for (int j = 0; j < MTC; ++j) {
      const float* col = nf.ssq + (mt0 + j) * 32 + (lane & 31);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int t = wave + u * KW;
        sq[j][u] = col[(size_t)(t < nf.n_ssq ? t : nf.n_ssq - 1) * nf.ssq_stride];
      }
    }
  }
  if (kb < ke) {
    fetch(0, kb);
    for (int kt = kb; kt < ke; kt += 2 * KH) {
      fetch(1, kt + KH);
      __builtin_amdgcn_sched_barrier(0);        // both groups requested before the first MFMA waits
      multiply(0, kt);
      if (kt + 2 * KH < ke) fetch(0, kt + 2 * KH);
      __builtin_amdgcn_sched_barrier(0);
      multiply(1, kt + KH);
    }
  }

  if (NORM_IN && nf.ssq != nullptr) {
#pragma unroll
    for (int j = 0; j < MTC; ++j) {
      float sacc = 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (wave + u * KW < nf.n_ssq) sacc += sq[j][u];
      const float* col = nf.ssq + (mt0 + j) * 32 + (lane & 31);
      // wide models have more than 8 slabs per wavefront: the rest in groups of 8 independent loads
      for (int t0 = wave + 8 * KW; t0 < nf.n_ssq; t0 += 8 * KW) {
        float more[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int t = t0 + u * KW;
          more[u] = col[(size_t)(t < nf.n_ssq ? t : nf.n_ssq - 1) * nf.ssq_stride];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (t0 + u * KW < nf.n_ssq) sacc += more[u];
      }
      if (lane < 32) ssp[(wave * MTC + j) * 32 + lane] = sacc;
    }
  }
  // Reduction over the KW wavefronts through LDS, and the split of the epilogue: every wavefront
  // publishes its partial tiles, then wavefront w adds the KW partials of activation tile j = w
  // in wavefront order (0 + 1 + 2 + 3) and runs the epilogue of that tile, so up to KW tiles are
  // finished in parallel.  One weight tile per round: the buffer holds KW x MTC accumulator tiles.
  constexpr int NREG = MTC * 16;
  constexpr int JT = INTRA ? 1 : MTC;           // activation tiles this wavefront finishes
  f32x16 res[NT][JT];
  if (INTRA) {
    static_assert(!INTRA || MTC <= KW, "one activation tile per wavefront");
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      if (i > 0) __syncthreads();               // everyone has read the previous round
      float* dst = red + (size_t)wave * NREG * 64 + lane;
#pragma unroll
      for (int jq = 0; jq < MTC; ++jq)
#pragma unroll
        for (int e = 0; e < 16; ++e) dst[(jq * 16 + e) * 64] = acc[i][jq][e];
      __syncthreads();
      if (wave < MTC) {
        const float* src = red + (size_t)wave * 16 * 64 + lane;      // tile j = wave of wavefront 0's slab
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float v = src[e * 64];
#pragma unroll
          for (int w = 1; w < KW; ++w) v += src[(size_t)w * NREG * 64 + e * 64];
          res[i][0][e] = v;
        }
      }
    }
    if (wave >= MTC) return;
  } else {
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int jq = 0; jq < JT; ++jq) res[i][jq] = acc[i][jq];
  }
  const int j0 = INTRA ? wave : 0;              // first (INTRA: only) activation tile of this wavefront

  const int mloc = lane & 31, nhalf = (lane >> 5) << 2;
  if (EPI == EPI_LOGITS) {
    // per row: the maximum over this wavefront's NT*32 output columns (a group of the sampler's
    // candidate search) and the column that holds it, the lowest one on ties: with those two the
    // greedy sampler needs no logits at all.  (nf.ssq carries the index array here, or null.)
    int* gidx = reinterpret_cast<int*>(nf.ssq);
#pragma unroll
    for (int jq = 0; jq < JT; ++jq) {
      const int j = j0 + jq;
      float bv = -INFINITY;
      int bn = 0;
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) {             // increasing column: a strict comparison keeps the first maximum
            const float v = res[i][jq][4 * q + e];
            if (v > bv) { bv = v; bn = i * 32 + 8 * q + nhalf + e; }
          }
      const float ov = __shfl_xor(bv, 32, 64);
      const int on = __shfl_xor(bn, 32, 64);
      if (ov > bv || (ov == bv && on < bn)) { bv = ov; bn = on; }
      const int m = (mt0 + j) * 32 + mloc;
      if (m < rows && lane < 32) {
        const size_t gi = (size_t)m * (N / (32 * NT)) + nt0 / NT;
        reinterpret_cast<float*>(act)[gi] = bv;
        if (gidx) gidx[gi] = bn;
      }
    }
  }
  if (EPI == EPI_F32 || (EPI == EPI_LOGITS && out != nullptr)) {
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int jq = 0; jq < JT; ++jq) {
      const int j = j0 + jq;
        const int m = (mt0 + j) * 32 + mloc;
        float inv = 1.0f;
        if (NORM_IN && nf.ssq != nullptr) {          // fused norm: a k-split partial scales like the sum
          float ssum = ssp[j * 32 + mloc];
#pragma unroll
          for (int w = 1; w < KW; ++w) ssum += ssp[(w * MTC + j) * 32 + mloc];
          inv = 1.0f / sqrtf(ssum * nf.inv_d + nf.eps);
        }
        if (m < rows) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = (nt0 + i) * 32 + 8 * q + nhalf;
            f32x4 v = {res[i][jq][4 * q] * inv, res[i][jq][4 * q + 1] * inv, res[i][jq][4 * q + 2] * inv, res[i][jq][4 * q + 3] * inv};
            *reinterpret_cast<f32x4*>(out + (size_t)m * N + n) = v;
          }
        }
      }
  } else if (EPI == EPI_RESID) {
    // out = residual stream (updated in place), act = gain-scaled bf16 copy for the next GEMM
#pragma unroll
    for (int jq = 0; jq < JT; ++jq) {
      const int j = j0 + jq;
      const int m = (mt0 + j) * 32 + mloc;
      float ss = 0.f;
      if (m < rows) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = nt0 * 32 + 8 * q + nhalf;
          float* xr = out + (size_t)m * N + n;
          f32x4 v = *reinterpret_cast<const f32x4*>(xr);
          const f32x4 gn = *reinterpret_cast<const f32x4*>(nf.gain + n);
          bf16x4 h;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] += res[0][jq][4 * q + e];
            ss += v[e] * v[e];
            h[e] = (bf16_t)(v[e] * gn[e]);
          }
          *reinterpret_cast<f32x4*>(xr) = v;
          *reinterpret_cast<bf16x4*>(act + act_index<true>(m, n, N)) = h;
        }
      }
      ss += __shfl_xor(ss, 32, 64);
      if (m < rows && lane < 32) nf.ssq[(size_t)nt0 * nf.ssq_stride + m] = ss;
    }
  } else if (EPI == EPI_SWIGLU) {
    // acc[0] = gate tile, acc[1] = up tile of features [nt0*32, nt0*32+32); N is F here.
#pragma unroll
    for (int jq = 0; jq < JT; ++jq) {
      const int j = j0 + jq;
      const int m = (mt0 + j) * 32 + mloc;
      float inv = 1.0f;
      if (INTRA && nf.ssq != nullptr) {
        float ssum = ssp[j * 32 + mloc];
#pragma unroll
        for (int w = 1; w < KW; ++w) ssum += ssp[(w * MTC + j) * 32 + mloc];
        inv = 1.0f / sqrtf(ssum * nf.inv_d + nf.eps);
      }
      if (m < rows) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = nt0 * 32 + 8 * q + nhalf;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = res[0][jq][4 * q + e] * inv, u = res[NT - 1][jq][4 * q + e] * inv;
            v[e] = (bf16_t)silu_mul(g, u);
          }
          *reinterpret_cast<bf16x4*>(act + act_index<true>(m, f, N)) = v;
        }
      }
    }
  }
}

// grid: x = n-tile group, y = k-split across workgroups, z = group of MT m-tiles.
// INTRA: the 4 wavefronts of a workgroup split the k range of one n-tile group (few
// n-tiles, or fused SwiGLU); otherwise each wavefront owns its own n-tile group.
template <int NT, int MT, int EPI, bool INTRA, int KW = KW4>
__global__ __launch_bounds__(64 * KW) void gemm_mfma_kernel(RowCtx rc, const bf16x8* __restrict__ x,
                                                           const bf16x8* __restrict__ w0,
                                                           const bf16x8* __restrict__ w1, float* __restrict__ out,
                                                           bf16_t* __restrict__ act, int N, int K, int ksplit,
                                                           size_t partial_stride, NormFuse nf) {
  __shared__ float red[INTRA ? KW * MT * 16 * 64 : 1];
  __shared__ float ssp[(INTRA && (EPI == EPI_SWIGLU || EPI == EPI_F32)) ? KW * MT * 32 : 1];
  const int rows = rows_or_zero(rc);
  // EPI_RESID: 1-D launch.  The m-groups of one weight tile re-read that tile, so they are
  // placed 8 workgroup ids apart: same XCD (ids are dealt to the 8 XCDs in turn), same moment,
  // one HBM read.  Id = ((tile / 8) * m_groups + m_group) * 8 + tile % 8.
  int bx = blockIdx.x, by = blockIdx.y, bz = blockIdx.z, ks = ksplit;
  if (EPI == EPI_RESID) {
    const int m_groups = ksplit;                  // (this launch has no k split: the field carries the m-group count)
    const int rem = bx % (8 * m_groups);
    by = (bx / (8 * m_groups)) * 8 + (rem & 7);
    bz = rem >> 3;
    bx = 0;
    ks = 1;
    if (by >= (N >> 5)) return;
  }
  const int mt0 = bz * MT;
  if (mt0 * 32 >= rows) return;
  const int KT = K >> 4;
  // Split-k launches put the k split in blockIdx.x: consecutive workgroups go to consecutive
  // XCDs, so with 8 (4) splits every XCD works on one (two) k slices and pulls only that slice
  // of the activations into its L2 instead of all of them.
  constexpr bool SPLIT_FIRST = INTRA && (EPI == EPI_F32 || EPI == EPI_RESID);
  const int bgrp = SPLIT_FIRST ? by : bx;
  const int grp = INTRA ? bgrp : bgrp * KW + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nt0 = (EPI == EPI_SWIGLU) ? grp : grp * NT;
  if (!INTRA && nt0 >= (N >> 5)) return;
  const int sidx = SPLIT_FIRST ? bx : by;
  const int k0 = (int)((long long)KT * sidx / ks), k1 = (int)((long long)KT * (sidx + 1) / ks);
  float* o = out ? out + (EPI == EPI_RESID ? (size_t)0 : sidx * partial_stride) : nullptr;
  int mtc = ceil_div(rows, 32) - mt0;
  if (mtc > MT) mtc = MT;
  switch (mtc) {
    case 1: gemm_group<NT, 1, EPI, INTRA, KW>(w0, w1, x, KT, k0, k1, nt0, mt0, rows, N, o, act, red, ssp, nf); break;
    case 2: gemm_group<NT, (MT >= 2 ? 2 : 1), EPI, INTRA, KW>(w0, w1, x, KT, k0, k1, nt0, mt0, rows, N, o, act, red, ssp, nf); break;
    case 3: gemm_group<NT, (MT >= 3 ? 3 : 1), EPI, INTRA, KW>(w0, w1, x, KT, k0, k1, nt0, mt0, rows, N, o, act, red, ssp, nf); break;
    default: gemm_group<NT, MT, EPI, INTRA, KW>(w0, w1, x, KT, k0, k1, nt0, mt0, rows, N, o, act, red, ssp, nf); break;
  }
}

void launch_gemm_mfma(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K,
                      int ksplit, size_t partial_stride, const float* ssq, int ssq_stride, float eps) {
  const NormFuse nf{nullptr, const_cast<float*>(ssq), ssq_stride, K >> 5, 1.0f / (float)K, eps};
  constexpr int MT = 4;
  const int n_tiles = N >> 5;
  const int m_groups = ceil_div(ceil_div(rc.max_rows, 32), MT);
  const bf16x8* xv = reinterpret_cast<const bf16x8*>(x);
  const bf16x8* wv = reinterpret_cast<const bf16x8*>(Wp);
  if (n_tiles >= 2048 && n_tiles % 2 == 0 && ssq == nullptr) {
    // plenty of n-tiles (LM head): one wavefront per pair of tiles, whole k range
    dim3 grid(ceil_div(n_tiles / 2, KW4), ksplit, m_groups);
    hipLaunchKernelGGL((gemm_mfma_kernel<2, MT, EPI_F32, false>), grid, dim3(64 * KW4), 0, st, rc, xv, wv, nullptr,
                       out, nullptr, N, K, ksplit, partial_stride, nf);
  } else if (n_tiles % 2 == 0 && (n_tiles / 2) * ksplit >= 128) {
    // wide matrices: two n-tiles per workgroup, so every activation fragment feeds two MFMAs
    // (the activation re-reads from L2 bound these shapes: 1.3-1.4x faster at 64-384 rows of
    // a 2560- or 4096-wide model).  Every output element keeps its summation chain.
    dim3 grid(ksplit, n_tiles / 2, m_groups);
    hipLaunchKernelGGL((gemm_mfma_kernel<2, MT, EPI_F32, true>), grid, dim3(64 * KW4), 0, st, rc, xv, wv, nullptr,
                       out, nullptr, N, K, ksplit, partial_stride, nf);
  } else {
    dim3 grid(ksplit, n_tiles, m_groups);
    hipLaunchKernelGGL((gemm_mfma_kernel<1, MT, EPI_F32, true>), grid, dim3(64 * KW4), 0, st, rc, xv, wv, nullptr,
                       out, nullptr, N, K, ksplit, partial_stride, nf);
  }
}

int lmhead_group_cols() { return 64; }

void launch_gemm_mfma_logits(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* logits,
                             float* group_max, int V, int K, int* group_idx) {
  constexpr int MT = 4;
  const int n_tiles = V >> 5;
  dim3 grid(ceil_div(n_tiles / 2, KW4), 1, ceil_div(ceil_div(rc.max_rows, 32), MT));
  hipLaunchKernelGGL((gemm_mfma_kernel<2, MT, EPI_LOGITS, false>), grid, dim3(64 * KW4), 0, st, rc,
                     reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wp), nullptr, logits,
                     reinterpret_cast<bf16_t*>(group_max), V, K, 1, (size_t)0,
                     NormFuse{nullptr, reinterpret_cast<float*>(group_idx), 0, 0, 0.f, 0.f});
}

void launch_gemm_mfma_swiglu(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                             bf16_t* act, int F, int K, const float* ssq, int ssq_stride, float eps) {
  constexpr int MT = 4;
  const int n_tiles = F >> 5;
  dim3 grid(n_tiles, 1, ceil_div(ceil_div(rc.max_rows, 32), MT));
  NormFuse nf{nullptr, const_cast<float*>(ssq), ssq_stride, K >> 5, 1.0f / (float)K, eps};
  hipLaunchKernelGGL((gemm_mfma_kernel<2, MT, EPI_SWIGLU, true>), grid, dim3(64 * KW4), 0, st, rc,
                     reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wg),
                     reinterpret_cast<const bf16x8*>(Wu), nullptr, act, F, K, 1, (size_t)0, nf);
}

// x_res += x . W^T (whole k range per workgroup, no partials); act = bf16(x_res * gain) in the
// fragment order of the next GEMM; ssq[n_tile][row] = sum of squares of the tile's 32 columns.
void launch_gemm_mfma_resid(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* x_res,
                            const float* gain, bf16_t* act, float* ssq, int ssq_stride, int N, int K) {
  const int n_tiles = N >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  const bf16x8* xv = reinterpret_cast<const bf16x8*>(x);
  const bf16x8* wv = reinterpret_cast<const bf16x8*>(Wp);
  NormFuse nf{gain, ssq, ssq_stride, 0, 0.f, 0.f};
  // few n-tiles: one m-tile per workgroup for more workgroups (the weights are small then);
  // also while that stays within 512 workgroups (2560 columns at 129-192 rows: 13.3 us
  // against 14.1 us on average over a run)
  const int tiles8 = ceil_div(n_tiles, 8) * 8;
  if (n_tiles * ceil_div(m_tiles, 4) < 128 || n_tiles * m_tiles <= 512) {
    // (8 wavefronts per workgroup for the long k range of the down projection were measured:
    // 14.0 us against 12.9 us)
    hipLaunchKernelGGL((gemm_mfma_kernel<1, 1, EPI_RESID, true>), dim3(tiles8 * m_tiles), dim3(64 * KW4), 0, st, rc,
                       xv, wv, nullptr, x_res, act, N, K, m_tiles, (size_t)0, nf);
  } else {
    const int mg = ceil_div(m_tiles, 4);
    hipLaunchKernelGGL((gemm_mfma_kernel<1, 4, EPI_RESID, true>), dim3(tiles8 * mg), dim3(64 * KW4), 0, st, rc, xv, wv,
                       nullptr, x_res, act, N, K, mg, (size_t)0, nf);
  }
}

}  // namespace april
