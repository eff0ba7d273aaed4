// Routed mixture of SwiGLU experts (bf16, gfx950): router soft-max + top-k, token ->
// expert dispatch lists, grouped expert GEMMs on v_mfma_f32_32x32x16_bf16.
//
// Per token: r = softmax over all E router logits; the top_k largest r (ties: lower
// expert index) are kept and renormalised to sum 1; y = sum_k w_k * expert_k(h), added to
// the residual stream in the fixed order k = 0..top_k-1 (descending r) by the following
// add/RMSNorm kernel, so the result does not depend on where a token lands in an expert's
// batch.
#include "kernels.h"

namespace april {

// ---------------------------------------------------------------------------
// Router: one wavefront per row.  logits = sum of split-K partials [n_partials][rows][E].
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(64) void moe_route_kernel(RowCtx rc, const float* logits, int n_partials,
                                                       size_t partial_stride, int E, int top_k, int* ids,
                                                       float* wts) {
  const int r = blockIdx.x;
  ROW_GUARD(rc, r);
  const int lane = threadIdx.x;
  // up to 256 experts: 4 per lane
  float v[4];
  float mx = -INFINITY;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int e = lane + 64 * j;
    float a = -INFINITY;
    if (e < E) {
      a = 0.f;
      for (int p = 0; p < n_partials; ++p) a += logits[p * partial_stride + (size_t)r * E + e];
    }
    v[j] = a;
    mx = fmaxf(mx, a);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j) { v[j] = lane + 64 * j < E ? expf(v[j] - mx) : 0.f; sum += v[j]; }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] /= sum;
  // top_k by repeated arg-max (value desc, index asc)
  float kept = 0.f;
  float myw = 0.f;
  int myid = -1;
  for (int k = 0; k < top_k; ++k) {
    float bv = -1.f;
    int bi = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int e = lane + 64 * j;
      if (e < E && v[j] > bv) { bv = v[j]; bi = e; }      // ascending e within the lane
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      const float ov = __shfl_xor(bv, off, 64);
      const int oi = __shfl_xor(bi, off, 64);
      if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    kept += bv;
    if (lane == k) { myw = bv; myid = bi; }
    if ((bi & 63) == lane) v[bi >> 6] = -2.f;               // remove the winner
  }
  if (lane < top_k) {
    ids[(size_t)r * top_k + lane] = myid;
    wts[(size_t)r * top_k + lane] = myw / kept;
  }
}

void launch_moe_route(hipStream_t st, RowCtx rc, const float* logits, int n_partials, size_t partial_stride,
                      int E, int top_k, int* ids, float* wts) {
  hipLaunchKernelGGL(moe_route_kernel, dim3(rc.max_rows), dim3(64), 0, st, rc, logits, n_partials, partial_stride,
                     E, top_k, ids, wts);
}

// ---------------------------------------------------------------------------
// Dispatch: one workgroup.  cnt[e] = tokens routed to expert e; base[e] = first packed row
// of expert e, aligned to `align` rows (the rows one GEMM workgroup covers: whole MFMA tiles, and
// no workgroup straddles two experts); pos_of[row*top_k + k] = packed row of that assignment;
// src_row[packed row] = token row (-1 in the padding); group_expert[g] = expert that owns packed
// rows [g*align, (g+1)*align), -1 past the end.  The GEMMs launch one workgroup per (n-tile
// group, row group) of that flat list: with a (expert, row group of the expert) grid sized for
// the worst case, five of six workgroups of a decode launch - and nearly all of a prefill
// launch - found nothing to do after a dependent load.
// Placement inside an expert's batch is arbitrary (LDS atomics); values never depend on it.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void moe_dispatch_kernel(RowCtx rc, const int* ids, int E, int top_k, int* cnt,
                                                            int* base, int* pos_of, int* src_row, int p_cap,
                                                            Ctrl* ctrl, int align, int* group_expert, int n_groups) {
  __shared__ int s_cnt[256], s_base[257];
  const int rows = rows_or_zero(rc), tid = threadIdx.x;
  if (rows == 0) return;
  if (tid < 256) s_cnt[tid] = 0;
  __syncthreads();
  const int n = rows * top_k;
  for (int a = tid; a < n; a += 1024) atomicAdd(&s_cnt[ids[a]], 1);
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    int hit = 0;
    for (int e = 0; e < E; ++e) { s_base[e] = acc; acc += (s_cnt[e] + align - 1) / align * align; hit += s_cnt[e] > 0; }
    s_base[E] = acc;
    if (ctrl != nullptr) ctrl->sum_experts += hit;
  }
  __syncthreads();
  const int total = s_base[E];
  for (int p = tid; p < total && p < p_cap; p += 1024) src_row[p] = -1;
  if (tid < E)
    for (int g = s_base[tid] / align; g < s_base[tid + 1] / align && g < n_groups; ++g) group_expert[g] = tid;
  for (int g = total / align + tid; g < n_groups; g += 1024) group_expert[g] = -1;
  if (tid < E) { cnt[tid] = s_cnt[tid]; base[tid] = s_base[tid]; s_cnt[tid] = 0; }
  if (tid == 0) base[E] = total;
  __syncthreads();
  for (int a = tid; a < n; a += 1024) {
    const int e = ids[a];
    const int p = s_base[e] + atomicAdd(&s_cnt[e], 1);
    pos_of[a] = p;
    if (p < p_cap) src_row[p] = a / top_k;
  }
}

// rows per GEMM workgroup (and alignment of the expert segments) for a launch over at most max_rows rows
int moe_group_rows(int max_rows, int tall_rows) { return max_rows >= tall_rows ? 128 : 64; }
// upper bound on the row groups of such a launch
int moe_group_count(int max_rows, int top_k, int E, int align) {
  return (int)(((long long)max_rows * top_k + (long long)E * (align - 1) + align - 1) / align);
}

void launch_moe_dispatch(hipStream_t st, RowCtx rc, const int* ids, int E, int top_k, int* cnt, int* base,
                         int* pos_of, int* src_row, int p_cap, Ctrl* ctrl, int tall_rows, int* group_expert) {
  const int align = moe_group_rows(rc.max_rows, tall_rows);
  hipLaunchKernelGGL(moe_dispatch_kernel, dim3(1), dim3(1024), 0, st, rc, ids, E, top_k, cnt, base, pos_of, src_row,
                     p_cap, ctrl, align, group_expert, moe_group_count(rc.max_rows, top_k, E, align));
}

// ---------------------------------------------------------------------------
// Grouped expert GEMMs.  grid: x = n-tile group inside the expert, y = row group of the flat
// packed list (MT m-tiles of one expert, see the dispatch kernel).  The 4 wavefronts of a
// workgroup split the k range (LDS reduction in wavefront order).
//   GATHER = true : the B operand rows are token rows looked up through src_row (gate/up);
//   GATHER = false: the B operand is the packed fragment-tiled activation (down).
// ---------------------------------------------------------------------------
constexpr int MOE_KW = 4;

template <int NT, int MT, bool SWIGLU>
__global__ __launch_bounds__(64 * MOE_KW) void moe_gemm_kernel(const int* stop, const int* cnt, const int* base,
                                                              const int* __restrict__ group_expert,
                                                              const int* src_row, const bf16x8* __restrict__ x,
                                                              const bf16x8* __restrict__ w0,
                                                              const bf16x8* __restrict__ w1, size_t w_expert_stride,
                                                              float* __restrict__ out, bf16_t* __restrict__ act,
                                                              int N, int K, int x_cols) {
  constexpr int KU = MT > 2 ? 4 : 8;            // k-tiles requested together (register budget)
  __shared__ float red[(MOE_KW - 1) * NT * MT * 16 * 64];
  if (stop != nullptr && *stop != 0) return;
  const int e = group_expert[blockIdx.y];
  if (e < 0) return;
  const int rows_e = cnt[e];
  const int p0 = base[e];                       // first packed row of this expert (multiple of MT * 32)
  const int mt0 = (int)blockIdx.y * MT - (p0 >> 5);   // first m-tile of this group inside the expert's batch
  if (mt0 * 32 >= rows_e) return;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KT = K >> 4;
  const int nt0 = SWIGLU ? blockIdx.x : blockIdx.x * NT;
  int mtc = ((rows_e + 31) >> 5) - mt0;
  if (mtc > MT) mtc = MT;

  f32x16 acc[NT][MT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[i][j] = f32x16{};
  const bf16x8* wp[NT];
  const bf16x8* we0 = w0 + (size_t)e * w_expert_stride;
  if (SWIGLU) {
    wp[0] = we0 + (size_t)nt0 * KT * 64 + lane;
    wp[NT - 1] = w1 + (size_t)e * w_expert_stride + (size_t)nt0 * KT * 64 + lane;
  } else {
#pragma unroll
    for (int i = 0; i < NT; ++i) wp[i] = we0 + (size_t)(nt0 + i) * KT * 64 + lane;
  }
  // B operand pointers: either a token row of the un-packed activation (gathered per lane)
  // or the packed tile
  const bf16x8* xp[MT];
  bool xok[MT];
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    xok[j] = j < mtc;
    xp[j] = x;
    if (SWIGLU) {
      int row = -1;
      if (j < mtc) row = src_row[p0 + (mt0 + j) * 32 + (lane & 31)];
      xok[j] = row >= 0;
      if (row < 0) row = 0;
      // fragment-tiled token activation [rows][x_cols]: element (row, k) -> act_index<true>
      xp[j] = x + ((size_t)(row >> 5) * (x_cols >> 4) * 64 + (row & 31) + ((lane >> 5) << 5));
    } else if (j < mtc) {
      xp[j] = x + ((size_t)((p0 >> 5) + mt0 + j) * KT * 64 + lane);
    }
  }
  const int len = KT;
  const int kb = (int)((long long)len * wave / MOE_KW), ke = (int)((long long)len * (wave + 1) / MOE_KW);
  for (int kt = kb; kt < ke; kt += KU) {
    bf16x8 a[KU][NT], b[KU][MT];
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      const size_t k = (size_t)(kt + u < ke ? kt + u : ke - 1) * 64;
#pragma unroll
      for (int i = 0; i < NT; ++i) a[u][i] = wp[i][k];
#pragma unroll
      for (int j = 0; j < MT; ++j) b[u][j] = xok[j] ? xp[j][k] : bf16x8{};
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < KU; ++u) {
      if (kt + u < ke) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int j = 0; j < MT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u][i], b[u][j], acc[i][j], 0, 0, 0);
      }
    }
  }
  constexpr int NREG = NT * MT * 16;
  if (wave != 0) {
    float* dst = red + (size_t)(wave - 1) * NREG * 64 + lane;
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) dst[((i * MT + j) * 16 + q) * 64] = acc[i][j][q];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int w = 0; w < MOE_KW - 1; ++w) {
    const float* src = red + (size_t)w * NREG * 64 + lane;
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MT; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][j][q] += src[((i * MT + j) * 16 + q) * 64];
  }
  const int mloc = lane & 31, nhalf = (lane >> 5) << 2;
#pragma unroll
  for (int j = 0; j < MT; ++j) {
    if (j >= mtc) continue;
    const int ml = (mt0 + j) * 32 + mloc;            // row inside the expert's batch
    if (ml >= rows_e) continue;
    const int p = p0 + ml;                           // packed row
    if (SWIGLU) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int f = nt0 * 32 + 8 * q + nhalf;
        bf16x4 v;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float g = acc[0][j][4 * q + t], u = acc[NT - 1][j][4 * q + t];
          v[t] = (bf16_t)silu_mul(g, u);
        }
        *reinterpret_cast<bf16x4*>(act + act_index<true>(p, f, N)) = v;
      }
    } else {
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = (nt0 + i) * 32 + 8 * q + nhalf;
          f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          *reinterpret_cast<f32x4*>(out + (size_t)p * N + n) = v;
        }
    }
  }
}

void launch_moe_gateup(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                       const int* src_row, const bf16_t* h, const bf16_t* Wg, const bf16_t* Wu, bf16_t* act, int E,
                       int top_k, int Fe, int d, int tall_rows) {
  // tall batches (prefill): 4 m-tiles per workgroup, so an expert's weight tile is fetched half as
  // often; the summation chain of an output element does not depend on the grouping
  const int align = moe_group_rows(rc.max_rows, tall_rows);
  dim3 grid(Fe >> 5, moe_group_count(rc.max_rows, top_k, E, align));
  const int* stop = reinterpret_cast<const int*>(rc.ctl) + 1;
  const bf16x8 *hv = reinterpret_cast<const bf16x8*>(h), *gv = reinterpret_cast<const bf16x8*>(Wg), *uv = reinterpret_cast<const bf16x8*>(Wu);
  if (align == 128)
    hipLaunchKernelGGL((moe_gemm_kernel<2, 4, true>), grid, dim3(64 * MOE_KW), 0, st, stop, cnt, base, group_expert, src_row,
                       hv, gv, uv, (size_t)Fe * d / 8, nullptr, act, Fe, d, d);
  else
    hipLaunchKernelGGL((moe_gemm_kernel<2, 2, true>), grid, dim3(64 * MOE_KW), 0, st, stop, cnt, base, group_expert, src_row,
                       hv, gv, uv, (size_t)Fe * d / 8, nullptr, act, Fe, d, d);
}

void launch_moe_down(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                     const bf16_t* act, const bf16_t* Wd, float* out, int E, int top_k, int Fe, int d, int tall_rows) {
  const int align = moe_group_rows(rc.max_rows, tall_rows);
  dim3 grid((d >> 5) / 2, moe_group_count(rc.max_rows, top_k, E, align));
  const int* stop = reinterpret_cast<const int*>(rc.ctl) + 1;
  const bf16x8 *av = reinterpret_cast<const bf16x8*>(act), *wv = reinterpret_cast<const bf16x8*>(Wd);
  if (align == 128)
    hipLaunchKernelGGL((moe_gemm_kernel<2, 4, false>), grid, dim3(64 * MOE_KW), 0, st, stop, cnt, base, group_expert, nullptr,
                       av, wv, nullptr, (size_t)d * Fe / 8, out, nullptr, d, Fe, Fe);
  else
    hipLaunchKernelGGL((moe_gemm_kernel<2, 2, false>), grid, dim3(64 * MOE_KW), 0, st, stop, cnt, base, group_expert, nullptr,
                       av, wv, nullptr, (size_t)d * Fe / 8, out, nullptr, d, Fe, Fe);
}

}  // namespace april
