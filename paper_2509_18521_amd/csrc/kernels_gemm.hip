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

enum { EPI_F32 = 0, EPI_SWIGLU = 1 };

// One wavefront: NT weight tiles x MTC activation tiles over k-tiles [kt0, kt1).
template <int NT, int MTC, int EPI>
__device__ inline void gemm_wave(const bf16x8* __restrict__ w0, const bf16x8* __restrict__ w1,
                                 const bf16x8* __restrict__ x, int KT, int kt0, int kt1, int nt0, int mt0,
                                 int rows, int N, float* __restrict__ out, bf16_t* __restrict__ act) {
  const int lane = threadIdx.x & 63;
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

#pragma unroll 4
  for (int kt = kt0; kt < kt1; ++kt) {
    bf16x8 a[NT], b[MTC];
#pragma unroll
    for (int i = 0; i < NT; ++i) a[i] = wp[i][(size_t)kt * 64];
#pragma unroll
    for (int j = 0; j < MTC; ++j) b[j] = xp[j][(size_t)kt * 64];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MTC; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }

  const int mloc = lane & 31, nhalf = (lane >> 5) << 2;
  if (EPI == EPI_F32) {
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < MTC; ++j) {
        const int m = (mt0 + j) * 32 + mloc;
        if (m < rows) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = (nt0 + i) * 32 + 8 * q + nhalf;
            f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            *reinterpret_cast<f32x4*>(out + (size_t)m * N + n) = v;
          }
        }
      }
  } else {
    // acc[0] = gate tile, acc[1] = up tile of features [nt0*32, nt0*32+32); N is F here.
#pragma unroll
    for (int j = 0; j < MTC; ++j) {
      const int m = (mt0 + j) * 32 + mloc;
      if (m < rows) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int f = nt0 * 32 + 8 * q + nhalf;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float g = acc[0][j][4 * q + e], u = acc[NT - 1][j][4 * q + e];
            v[e] = (bf16_t)(g / (1.0f + __expf(-g)) * u);
          }
          *reinterpret_cast<bf16x4*>(act + act_index<true>(m, f, N)) = v;
        }
      }
    }
  }
}

// grid: x = groups of 4 wavefronts over n-tile groups, y = k-split, z = group of MT m-tiles.
template <int NT, int MT, int EPI>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(RowCtx rc, const bf16x8* __restrict__ x,
                                                        const bf16x8* __restrict__ w0,
                                                        const bf16x8* __restrict__ w1, float* __restrict__ out,
                                                        bf16_t* __restrict__ act, int N, int K, int ksplit,
                                                        size_t partial_stride) {
  if (rc.stop != nullptr && *rc.stop != 0) return;
  const int rows = *rc.n_rows;
  const int mt0 = blockIdx.z * MT;
  if (mt0 * 32 >= rows) return;
  const int n_tiles = N >> 5, KT = K >> 4;
  const int gw = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int nt0 = (EPI == EPI_SWIGLU) ? gw : gw * NT;
  if (nt0 >= n_tiles) return;
  const int sidx = blockIdx.y;
  const int kt0 = (int)((long long)KT * sidx / ksplit), kt1 = (int)((long long)KT * (sidx + 1) / ksplit);
  float* o = out ? out + sidx * partial_stride : nullptr;
  int mtc = ceil_div(rows, 32) - mt0;
  if (mtc > MT) mtc = MT;
  switch (mtc) {
    case 1: gemm_wave<NT, 1, EPI>(w0, w1, x, KT, kt0, kt1, nt0, mt0, rows, N, o, act); break;
    case 2: gemm_wave<NT, (MT >= 2 ? 2 : 1), EPI>(w0, w1, x, KT, kt0, kt1, nt0, mt0, rows, N, o, act); break;
    case 3: gemm_wave<NT, (MT >= 3 ? 3 : 1), EPI>(w0, w1, x, KT, kt0, kt1, nt0, mt0, rows, N, o, act); break;
    default: gemm_wave<NT, MT, EPI>(w0, w1, x, KT, kt0, kt1, nt0, mt0, rows, N, o, act); break;
  }
}

void launch_gemm_mfma(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K,
                      int ksplit, size_t partial_stride) {
  constexpr int NT = 2, MT = 4;
  const int n_tiles = N >> 5;
  // N/32 may be odd: the kernel's last wavefront would read one tile past the end, so
  // fall back to NT = 1 in that case.
  const int m_groups = ceil_div(ceil_div(rc.max_rows, 32), MT);
  if (n_tiles % NT == 0) {
    dim3 grid(ceil_div(n_tiles / NT, 4), ksplit, m_groups);
    hipLaunchKernelGGL((gemm_mfma_kernel<NT, MT, EPI_F32>), grid, dim3(256), 0, st, rc,
                       reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wp), nullptr, out,
                       nullptr, N, K, ksplit, partial_stride);
  } else {
    dim3 grid(ceil_div(n_tiles, 4), ksplit, m_groups);
    hipLaunchKernelGGL((gemm_mfma_kernel<1, MT, EPI_F32>), grid, dim3(256), 0, st, rc,
                       reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wp), nullptr, out,
                       nullptr, N, K, ksplit, partial_stride);
  }
}

void launch_gemm_mfma_swiglu(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                             bf16_t* act, int F, int K) {
  constexpr int MT = 4;
  const int n_tiles = F >> 5;
  dim3 grid(ceil_div(n_tiles, 4), 1, ceil_div(ceil_div(rc.max_rows, 32), MT));
  hipLaunchKernelGGL((gemm_mfma_kernel<2, MT, EPI_SWIGLU>), grid, dim3(256), 0, st, rc,
                     reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wg),
                     reinterpret_cast<const bf16x8*>(Wu), nullptr, act, F, K, 1, (size_t)0);
}

}  // namespace april
