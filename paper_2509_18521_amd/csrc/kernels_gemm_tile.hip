// bf16 MFMA GEMM for tall activations (prefill: hundreds to thousands of rows), gfx950.
//
// out[m][n] = sum_k x[m][k] * W[n][k], same operand layouts as the skinny decode GEMM
// (both operands fragment-tiled for v_mfma_f32_32x32x16_bf16: one 32x16 fragment is 1 KiB of
// consecutive bytes), but compute-bound, so it is organised around operand reuse:
//   * a workgroup of WGM x WGN wavefronts owns a (WGM*MTW*32) x (WGN*NTW*32) output tile;
//     each wavefront keeps MTW x NTW accumulator tiles;
//   * the k loop advances in stages of BK k-tiles; the fragments of a stage go
//     global -> registers -> LDS once per workgroup (every fragment is one contiguous 1 KiB
//     piece; LDS reads are lane-consecutive 16-byte pieces, conflict-free) while the MFMAs of
//     the previous stage run from the other LDS buffer; one barrier per stage;
//   * every output element is one accumulator chain over k-tiles 0..K/16-1 in order, whatever
//     the tile shape or the number of rows: results do not depend on the batch.
#include "kernels.h"

namespace april {

enum { TEPI_F32 = 0, TEPI_SWIGLU = 1, TEPI_LOGITS = 2 };   // LOGITS: F32 + per-row maxima of 64-column groups

// Epilogue of one wavefront: accumulator tile = out^T (lane l, register e:
// n = 8*(e/4) + 4*(l/32) + e%4, m = l%32).  nt0: first weight tile (SwiGLU: first feature
// tile; acc[i] = gate, acc[i + NTW/2] = up), mt0: first activation tile.
template <int MTW, int NTW, int EPI>
__device__ inline void tile_epilogue(f32x16 (&acc)[NTW][MTW], int nt0, int mt0, int rows, int n_tiles, int N, int lane,
                                     float* __restrict__ out, bf16_t* __restrict__ act,
                                     const float* row_scale = nullptr, int scale_m0 = 0, int* gidx = nullptr) {
  const int mloc = lane & 31, nhalf = (lane >> 5) << 2;
  if (EPI == TEPI_LOGITS) {
    // act carries the group maxima (float [rows][N / 64]); a group is an aligned pair of weight
    // tiles, which is what one wavefront holds (NTW == 2, nt0 even)
    static_assert(EPI != TEPI_LOGITS || NTW == 2, "one 64-column group per wavefront");
    float* gmax = reinterpret_cast<float*>(act);
    if (nt0 < n_tiles) {
#pragma unroll
      for (int j = 0; j < MTW; ++j) {
        // maximum of the 64 columns and the column holding it (lowest on ties): see the skinny LM head
        float bv = -INFINITY;
        int bn = 0;
#pragma unroll
        for (int i = 0; i < NTW; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float v = acc[i][j][4 * q + e];
              if (v > bv) { bv = v; bn = i * 32 + 8 * q + nhalf + e; }
            }
        const float ov = __shfl_xor(bv, 32, 64);
        const int on = __shfl_xor(bn, 32, 64);
        if (ov > bv || (ov == bv && on < bn)) { bv = ov; bn = on; }
        const int m = (mt0 + j) * 32 + mloc;
        if (m < rows && lane < 32) {
          const size_t gi = (size_t)m * (N >> 6) + (nt0 >> 1);
          gmax[gi] = bv;
          if (gidx) gidx[gi] = bn;
        }
      }
    }
  }
  if (EPI == TEPI_F32 || (EPI == TEPI_LOGITS && out != nullptr)) {
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
      const int nt = nt0 + i;
      if (nt >= n_tiles) continue;
#pragma unroll
      for (int j = 0; j < MTW; ++j) {
        const int m = (mt0 + j) * 32 + mloc;
        if (m < rows) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = nt * 32 + 8 * q + nhalf;
            f32x4 v = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
            *reinterpret_cast<f32x4*>(out + (size_t)m * N + n) = v;
          }
        }
      }
    }
  } else if (EPI == TEPI_SWIGLU) {
    constexpr int H = NTW / 2;
#pragma unroll
    for (int i = 0; i < H; ++i) {
      const int ft = nt0 + i;
      if (ft >= n_tiles) continue;
#pragma unroll
      for (int j = 0; j < MTW; ++j) {
        const int m = (mt0 + j) * 32 + mloc;
        // folded RMSNorm (decode): the accumulators are scaled by the row's 1/rms first
        const float inv = row_scale ? row_scale[m - scale_m0] : 1.0f;
        if (m < rows) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int f = ft * 32 + 8 * q + nhalf;
            bf16x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float g = acc[i][j][4 * q + e] * inv, u = acc[i + H][j][4 * q + e] * inv;
              v[e] = (bf16_t)silu_mul(g, u);
            }
            *reinterpret_cast<bf16x4*>(act + act_index<true>(m, f, N)) = v;
          }
        }
      }
    }
  }
}

template <int WGM, int WGN, int MTW, int NTW, int BK, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(2)))
void gemm_tile_kernel(RowCtx rc, const bf16x8* __restrict__ x,
                                                                   const bf16x8* __restrict__ w0,
                                                                   const bf16x8* __restrict__ w1,
                                                                   float* __restrict__ out, bf16_t* __restrict__ act,
                                                                   int N, int K) {
  constexpr int NW = WGM * WGN, MT = WGM * MTW, NT = WGN * NTW, FR = MT + NT;
  constexpr int PER = FR * BK / NW;             // fragments one wavefront stages per stage
  static_assert(FR * BK % NW == 0 && NW % BK == 0, "staging split");
  static_assert(EPI != TEPI_SWIGLU || NTW % 2 == 0, "gate/up pairs");
  __shared__ bf16x8 lds[2][BK][FR][64];
  const int rows = rows_or_zero(rc);
  const int m0 = blockIdx.y * MT;
  if (m0 * 32 >= rows) return;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int KT = K >> 4;
  const int m_last = (rows - 1) >> 5;           // last activation tile that holds a live row
  const int n_tiles = N >> 5;                   // SwiGLU: feature tiles (N = F)

  // Fragment slot t of a stage: t < MT activation tile m0 + t, else weight slot t - MT.
  // Weight slot i belongs to wavefront column i / NTW; plain: tile n0 + i; SwiGLU: the first
  // half of a wavefront's slots are gate tiles, the second half the up tiles of the same
  // features.  Tiles past the end are clamped for the loads and never stored.
  auto slot_base = [&](int t) -> const bf16x8* {
    if (t < MT) {
      int mt = m0 + t;
      if (mt > m_last) mt = m_last;
      return x + (size_t)mt * KT * 64;
    }
    const int i = t - MT;
    if (EPI == TEPI_SWIGLU) {
      constexpr int H = NTW / 2;
      const int col = i / NTW, ii = i % NTW;
      int f = blockIdx.x * (NT / 2) + col * H + (ii < H ? ii : ii - H);
      if (f >= n_tiles) f = n_tiles - 1;
      return (ii < H ? w0 : w1) + (size_t)f * KT * 64;
    }
    int nt = blockIdx.x * NT + i;
    if (nt >= n_tiles) nt = n_tiles - 1;
    return w0 + (size_t)nt * KT * 64;
  };

  // staging: wavefront w moves k-tile (w % BK) of the slots t = w / BK + (NW / BK) * u
  const int skk = wave % BK, st0 = wave / BK;
  const bf16x8* src[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) src[u] = slot_base(st0 + (NW / BK) * u) + lane;
  bf16x8 stg[PER];
  auto stage_load = [&](int s) {
    const int kt = s * BK + skk;
    const bool live = kt < KT;                  // a k-tile past the end contributes zeros
    const size_t off = (size_t)(live ? kt : KT - 1) * 64;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const bf16x8 v = src[u][off];
      stg[u] = live ? v : bf16x8{};
    }
  };
  auto stage_store = [&](int buf) {
#pragma unroll
    for (int u = 0; u < PER; ++u) lds[buf][skk][st0 + (NW / BK) * u][lane] = stg[u];
  };

  f32x16 acc[NTW][MTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MTW; ++j) acc[i][j] = f32x16{};

  const int n_stages = (KT + BK - 1) / BK;
  stage_load(0);
  stage_store(0);
  __syncthreads();
  for (int s = 0; s < n_stages; ++s) {
    const int buf = s & 1;
    const bool more = s + 1 < n_stages;
    if (more) stage_load(s + 1);
    // operand fragments of k-tile kk+1 are read from LDS while the MFMAs of k-tile kk run
    bf16x8 a[2][NTW], b[2][MTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) a[0][i] = lds[buf][0][MT + wn * NTW + i][lane];
#pragma unroll
    for (int j = 0; j < MTW; ++j) b[0][j] = lds[buf][0][wm * MTW + j][lane];
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < BK) {
#pragma unroll
        for (int i = 0; i < NTW; ++i) a[nxt][i] = lds[buf][kk + 1][MT + wn * NTW + i][lane];
#pragma unroll
        for (int j = 0; j < MTW; ++j) b[nxt][j] = lds[buf][kk + 1][wm * MTW + j][lane];
      }
#pragma unroll
      for (int i = 0; i < NTW; ++i)
#pragma unroll
        for (int j = 0; j < MTW; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
    }
    if (more) stage_store(buf ^ 1);
    __syncthreads();
  }

  tile_epilogue<MTW, NTW, EPI>(acc, blockIdx.x * (EPI == TEPI_SWIGLU ? NT / 2 : NT) + wn * (EPI == TEPI_SWIGLU ? NTW / 2 : NTW),
                               m0 + wm * MTW, rows, n_tiles, N, lane, out, act);
}

// One wavefront-wide copy of 64 x 16 bytes from global memory (a per-lane address) to LDS
// (a wavefront-uniform base; lane l lands at base + 16*l).  Device pass only: the host pass
// has no such instruction to type-check.
__device__ inline void copy_fragment_to_lds(const bf16x8* src_lane, bf16x8* lds_base) {
#if defined(__HIP_DEVICE_COMPILE__)
  __builtin_amdgcn_global_load_lds(src_lane, lds_base, 16, 0, 0);
#else
  (void)src_lane; (void)lds_base;
#endif
}
template <int LEFT>
__device__ inline void wait_vector_memory() {   // until at most LEFT vector-memory operations are outstanding
#if defined(__HIP_DEVICE_COMPILE__)
  // s_waitcnt with the expcnt and lgkmcnt fields all-ones: only vmcnt is waited for
  __builtin_amdgcn_s_waitcnt(0x0f70 | (LEFT & 15) | ((LEFT >> 4) << 14));
#endif
}

// Same tiling with the stage fragments copied global -> LDS by the memory pipeline itself
// (global_load_lds_dwordx4: each lane's 16 bytes land at consecutive LDS addresses, which is
// exactly the fragment layout), through a ring of R stage buffers.  Nothing is staged in
// registers, so R - 1 stages of loads stay in flight behind the MFMAs.  Hand-placed waits:
// the copies of stage s are this wavefront's oldest outstanding vector-memory operations, so
// "at most (R - 2) stages still outstanding" means stage s has landed; the barrier that
// follows makes that true for every wavefront's share and also says everyone has finished
// reading the buffer that the next copies overwrite.  Requires K % (16 * BK) == 0.
//
// CHAIN (decode with many rows): the skinny decode kernel sums k in four quarters (its four
// wavefronts), each quarter its own accumulator chain, and adds them as ((q0 + q1) + q2) + q3.
// Here one wavefront walks all of k, so it closes a chain at every quarter boundary and adds
// it to a second accumulator set in that order: every output element gets the same bits from
// either kernel, and the choice between them can follow the row count.  The quarter
// boundaries must fall on stage boundaries (K % (64 * BK) == 0).  The second accumulator set
// needs the whole register file of a SIMD, hence the separate entry without the two-waves hint.
struct TileNorm {              // RMSNorm folded into the SwiGLU epilogue (CHAIN only)
  const float* ssq;            // [n_ssq][ssq_stride] per-row sums of squares of 32-column slabs; nullptr = none
  int ssq_stride, n_ssq;
  float inv_d, eps;
  int* gidx;                   // LM head: column of every 64-column group's maximum (nullptr = not wanted)
  int ksplit = 0;              // CHAIN, plain epilogue: blockIdx.z = k slice of ksplit (0: the whole k range)
  size_t partial_stride = 0;   // floats between the slices' partial outputs
};

// Routed experts (MOE): blockIdx.y is a row group of the dispatch kernel's packed list (MT m-tiles
// of one expert; the expert segments are aligned to MT * 32 rows), rows are packed-row indices,
// the weights are the expert's, and the activation rows are either the packed tiles (down
// projection) or token rows gathered through src_row from a plain [row][K] copy of the
// activations (gate/up: each lane copies its own 16 bytes, so a gathered fragment lands in LDS
// exactly like a dense one; gathering from the fragment-tiled layout would use 16 bytes of
// every 128-byte line it touches).
struct TileMoe {
  const int* cnt;              // [E] rows of every expert
  const int* base;             // [E] first packed row of every expert
  const int* group_expert;     // [row groups] expert of the group, -1 = none
  const int* src_row;          // [packed rows] token row, or nullptr (activations already packed)
  size_t w_expert_stride;      // bf16x8 units between the experts' matrices
};

template <int WGM, int WGN, int MTW, int NTW, int BK, int R, int EPI, bool CHAIN, bool MOE = false>
__device__ __forceinline__ void tile_dma_body(RowCtx rc, const bf16x8* __restrict__ x, const bf16x8* __restrict__ w0,
                                              const bf16x8* __restrict__ w1, float* __restrict__ out,
                                              bf16_t* __restrict__ act, int N, int K, const TileNorm& tn,
                                              const TileMoe& mo = TileMoe{}) {
  constexpr int NW = WGM * WGN, MT = WGM * MTW, NT = WGN * NTW, FR = MT + NT;
  constexpr int PER = FR * BK / NW;
  static_assert(FR * BK % NW == 0 && NW % BK == 0, "staging split");
  static_assert(EPI != TEPI_SWIGLU || NTW % 2 == 0, "gate/up pairs");
  static_assert(R >= 3 && (R - 2) * PER < 64, "ring depth");
  __shared__ bf16x8 lds[R][BK][FR][64];
  const int bx = blockIdx.x, by = blockIdx.y;
  int rows = rows_or_zero(rc);
  const int m0 = by * MT;
  if constexpr (MOE) {
    if (rows == 0) return;                       // step stopped, or nothing to do
    const int e = mo.group_expert[by];
    if (e < 0) return;
    const int rows_e = mo.cnt[e], p0 = mo.base[e];
    if (m0 * 32 < p0 || m0 * 32 - p0 >= rows_e) return;
    rows = p0 + rows_e;                          // one past the expert's last packed row
    w0 += (size_t)e * mo.w_expert_stride;
    if (w1 != nullptr) w1 += (size_t)e * mo.w_expert_stride;
  } else {
    if (m0 * 32 >= rows) return;
  }
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int KT = K >> 4;
  const int m_last = (rows - 1) >> 5;
  const int n_tiles = N >> 5;
  auto slot_base = [&](int t) -> const bf16x8* {        // this lane's piece of the slot's fragment at k-tile 0
    if (t < MT) {
      if constexpr (MOE) {
        if (mo.src_row != nullptr) {
          int p = (m0 + t) * 32 + (lane & 31);
          if (p > rows - 1) p = rows - 1;                 // rows beyond the expert's repeat its last one (never written)
          int row = mo.src_row[p];
          if (row < 0) row = 0;
          return x + ((size_t)row * KT * 2 + (lane >> 5));   // plain [row][K]: a k-tile of a row is two 16-byte pieces
        }
      }
      int mt = m0 + t;
      if (mt > m_last) mt = m_last;
      return x + (size_t)mt * KT * 64 + lane;
    }
    const int i = t - MT;
    if (EPI == TEPI_SWIGLU) {
      constexpr int H = NTW / 2;
      const int col = i / NTW, ii = i % NTW;
      int f = bx * (NT / 2) + col * H + (ii < H ? ii : ii - H);
      if (f >= n_tiles) f = n_tiles - 1;
      return (ii < H ? w0 : w1) + (size_t)f * KT * 64 + lane;
    }
    int nt = bx * NT + i;
    if (nt >= n_tiles) nt = n_tiles - 1;
    return w0 + (size_t)nt * KT * 64 + lane;
  };
  const int skk = wave % BK, st0 = wave / BK;
  const bf16x8* src[PER];
#pragma unroll
  for (int u = 0; u < PER; ++u) src[u] = slot_base(st0 + (NW / BK) * u);
  // k range of this workgroup: everything, or slice blockIdx.z of tn.ksplit (the skinny kernel's
  // slices; the launcher has checked that slices and their quarters fall on stage boundaries)
  int kt0 = 0, kt1 = KT;
  if (CHAIN && EPI == TEPI_F32 && tn.ksplit > 0) {
    kt0 = (int)((long long)KT * blockIdx.z / tn.ksplit);
    kt1 = (int)((long long)KT * (blockIdx.z + 1) / tn.ksplit);
    out += (size_t)blockIdx.z * tn.partial_stride;
  }
  const int klen = kt1 - kt0;
  const int n_stages = klen / BK;
  const bool gathered = MOE && mo.src_row != nullptr;
  auto issue = [&](int s) {
    const size_t off = (size_t)(kt0 + s * BK + skk) * 64;
    const size_t off_rows = (size_t)(kt0 + s * BK + skk) * 2;      // gathered activation rows advance 32 bytes per k-tile
    const int slot = s % R;
#pragma unroll
    for (int u = 0; u < PER; ++u) {
      const int t = st0 + (NW / BK) * u;
      copy_fragment_to_lds(src[u] + (gathered && t < MT ? off_rows : off), &lds[slot][skk][t][0]);
    }
  };

  f32x16 acc[NTW][MTW];
#pragma unroll
  for (int i = 0; i < NTW; ++i)
#pragma unroll
    for (int j = 0; j < MTW; ++j) acc[i][j] = f32x16{};
  f32x16 tot[CHAIN ? NTW : 1][CHAIN ? MTW : 1];
  int quarter = 1, next_close = CHAIN ? (klen / 4) / BK : -1;     // stage at which the next chain closes

#pragma unroll
  for (int r = 0; r < R - 1; ++r)
    if (r < n_stages) issue(r);

  // folded norm: 1/rms of this workgroup's rows, summed in the skinny kernel's order (wavefront w
  // of that kernel adds the slabs w, w + 4, ...; then ((s0 + s1) + s2) + s3)
  __shared__ float row_scale[CHAIN ? MT * 32 : 1];
  const bool scaled = CHAIN && EPI == TEPI_SWIGLU && tn.ssq != nullptr;
  if (scaled) {
    for (int rl = threadIdx.x; rl < MT * 32; rl += 64 * NW) {
      int m = m0 * 32 + rl;
      if (m > rows - 1) m = rows - 1;
      const float* col = tn.ssq + m;
      float sw[4] = {0.f, 0.f, 0.f, 0.f};
      // 32 slabs requested together (independent loads), then added in slab order: chain w sees
      // the slabs w, w + 4, ... in increasing order
      for (int t0 = 0; t0 < tn.n_ssq; t0 += 32) {
        float sl[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) {
          const int t = t0 + u < tn.n_ssq ? t0 + u : tn.n_ssq - 1;
          sl[u] = col[(size_t)t * tn.ssq_stride];
        }
#pragma unroll
        for (int u = 0; u < 32; ++u)
          if (t0 + u < tn.n_ssq) sw[u & 3] += sl[u];
      }
      float ssum = sw[0];
#pragma unroll
      for (int w = 1; w < 4; ++w) ssum += sw[w];
      row_scale[rl] = 1.0f / sqrtf(ssum * tn.inv_d + tn.eps);
    }
    __syncthreads();
  }

  for (int s = 0; s < n_stages; ++s) {
    if (CHAIN && s == next_close) {
#pragma unroll
      for (int i = 0; i < NTW; ++i)
#pragma unroll
        for (int j = 0; j < MTW; ++j) {
          if (quarter == 1) tot[CHAIN ? i : 0][CHAIN ? j : 0] = acc[i][j];
          else tot[CHAIN ? i : 0][CHAIN ? j : 0] += acc[i][j];
          acc[i][j] = f32x16{};
        }
      ++quarter;
      next_close = quarter < 4 ? (int)(((long long)klen * quarter / 4) / BK) : -1;
    }
    // wait for this wavefront's copies of stage s (s_waitcnt vmcnt only: expcnt/lgkmcnt fields all-ones)
    constexpr int LEFT = (R - 2) * PER;
    if (s + R - 2 < n_stages) wait_vector_memory<LEFT>();
    else wait_vector_memory<0>();
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (s + R - 1 < n_stages) issue(s + R - 1);
    const int slot = s % R;
    bf16x8 a[2][NTW], b[2][MTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) a[0][i] = lds[slot][0][MT + wn * NTW + i][lane];
#pragma unroll
    for (int j = 0; j < MTW; ++j) b[0][j] = lds[slot][0][wm * MTW + j][lane];
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < BK) {
#pragma unroll
        for (int i = 0; i < NTW; ++i) a[nxt][i] = lds[slot][kk + 1][MT + wn * NTW + i][lane];
#pragma unroll
        for (int j = 0; j < MTW; ++j) b[nxt][j] = lds[slot][kk + 1][wm * MTW + j][lane];
      }
#pragma unroll
      for (int i = 0; i < NTW; ++i)
#pragma unroll
        for (int j = 0; j < MTW; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      if (kk + 1 < BK) {          // issue order: the LDS reads of k-tile kk+1, then the MFMAs of kk
        __builtin_amdgcn_sched_group_barrier(0x100, NTW + MTW, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NTW * MTW, 0);
      }
    }
    asm volatile("" ::: "memory");
  }
  if (CHAIN) {
#pragma unroll
    for (int i = 0; i < NTW; ++i)
#pragma unroll
      for (int j = 0; j < MTW; ++j) acc[i][j] = tot[CHAIN ? i : 0][CHAIN ? j : 0] + acc[i][j];
  }
  tile_epilogue<MTW, NTW, EPI>(acc, bx * (EPI == TEPI_SWIGLU ? NT / 2 : NT) + wn * (EPI == TEPI_SWIGLU ? NTW / 2 : NTW),
                               m0 + wm * MTW, rows, n_tiles, N, lane, out, act, scaled ? row_scale : nullptr, m0 * 32, tn.gidx);
}

template <int WGM, int WGN, int MTW, int NTW, int BK, int R, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(2)))
void gemm_tile_dma_kernel(RowCtx rc, const bf16x8* __restrict__ x, const bf16x8* __restrict__ w0,
                          const bf16x8* __restrict__ w1, float* __restrict__ out, bf16_t* __restrict__ act, int N,
                          int K, int* gidx) {
  TileNorm tn{};
  tn.gidx = gidx;
  tile_dma_body<WGM, WGN, MTW, NTW, BK, R, EPI, false>(rc, x, w0, w1, out, act, N, K, tn);
}

template <int WGM, int WGN, int MTW, int NTW, int BK, int R, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN)
void gemm_tile_chain_kernel(RowCtx rc, const bf16x8* __restrict__ x, const bf16x8* __restrict__ w0,
                            const bf16x8* __restrict__ w1, float* __restrict__ out, bf16_t* __restrict__ act, int N,
                            int K, TileNorm tn) {
  tile_dma_body<WGM, WGN, MTW, NTW, BK, R, EPI, true>(rc, x, w0, w1, out, act, N, K, tn);
}

// Routed experts in prefill: 128 packed rows (one row group of the dispatch list) x 256 weight
// rows per workgroup, 4 wavefronts side by side (each 128 x 64), ring of 3 stages (72 KiB, two
// workgroups per CU).  One accumulator chain per output element, like every prefill GEMM.
template <int EPI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2)))
void moe_tile_kernel(RowCtx rc, const bf16x8* __restrict__ x, const bf16x8* __restrict__ w0,
                     const bf16x8* __restrict__ w1, float* __restrict__ out, bf16_t* __restrict__ act, int N, int K,
                     TileMoe mo) {
  tile_dma_body<1, 4, 4, 2, 2, 3, EPI, false, true>(rc, x, w0, w1, out, act, N, K, TileNorm{}, mo);
}

int moe_tile_rows() { return 128; }

bool launch_moe_tile_gateup(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                            const int* src_row, const bf16_t* h_rows, const bf16_t* Wg, const bf16_t* Wu, bf16_t* act,
                            int Fe, int d, int n_groups) {
  if (d % 32 != 0 || Fe % 32 != 0 || n_groups <= 0 || h_rows == nullptr) return false;
  const TileMoe mo{cnt, base, group_expert, src_row, (size_t)Fe * d / 8};
  dim3 grid(ceil_div(Fe >> 5, 4), n_groups);            // 4 feature tiles (gate + up: 8 weight tiles) per workgroup
  hipLaunchKernelGGL((moe_tile_kernel<TEPI_SWIGLU>), grid, dim3(256), 0, st, rc, reinterpret_cast<const bf16x8*>(h_rows),
                     reinterpret_cast<const bf16x8*>(Wg), reinterpret_cast<const bf16x8*>(Wu), nullptr, act, Fe, d, mo);
  return true;
}

bool launch_moe_tile_down(hipStream_t st, RowCtx rc, const int* cnt, const int* base, const int* group_expert,
                          const bf16_t* act, const bf16_t* Wd, float* out, int Fe, int d, int n_groups) {
  if (d % 32 != 0 || Fe % 32 != 0 || n_groups <= 0) return false;
  const TileMoe mo{cnt, base, group_expert, nullptr, (size_t)d * Fe / 8};
  dim3 grid(ceil_div(d >> 5, 8), n_groups);
  hipLaunchKernelGGL((moe_tile_kernel<TEPI_F32>), grid, dim3(256), 0, st, rc, reinterpret_cast<const bf16x8*>(act),
                     reinterpret_cast<const bf16x8*>(Wd), nullptr, out, nullptr, d, Fe, mo);
  return true;
}

// Tile shapes.  WIDE: 256 x 256 outputs on 8 wavefronts (2 per SIMD, each 128 x 64), ring of
// 4 stages of 32 values of k (128 KiB LDS).  NARROW: 256 x 128 on 4 wavefronts, ring of 3
// (72 KiB, two workgroups per CU) - for few or ragged weight tiles and for short batches.
// REGS: register-staged fallback for K not a multiple of 32.  Measured on MI355X, 8192 x
// (2 x 14336) x 4096 fused gate/up: REGS 0.84, NARROW 0.99, WIDE 1.03 PFLOP/s.  The choice
// changes no result (see the header comment).
#define TILE_WIDE(EPI) gemm_tile_dma_kernel<2, 4, 4, 2, 2, 4, EPI>
#define TILE_NARROW(EPI) gemm_tile_dma_kernel<2, 2, 4, 2, 2, 3, EPI>
#define TILE_REGS(EPI) gemm_tile_kernel<2, 2, 4, 2, 2, EPI>

// units: weight tiles (plain) or feature tiles (SwiGLU); per_wide: units per WIDE workgroup
static bool wide_tile(int units, int per_wide, int m_tiles) {
  const int wgs = ceil_div(units, per_wide) * ceil_div(m_tiles, 8);
  return wgs >= 128 && ceil_div(units, per_wide) * per_wide * 20 <= units * 23;   // <= 15 % padding
}

void launch_gemm_tile(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K) {
  const int n_tiles = N >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  const bf16x8* xv = reinterpret_cast<const bf16x8*>(x);
  const bf16x8* wv = reinterpret_cast<const bf16x8*>(Wp);
  if (K % 32 != 0) {
    dim3 grid(ceil_div(n_tiles, 4), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_REGS(TEPI_F32)), grid, dim3(256), 0, st, rc, xv, wv, nullptr, out, nullptr, N, K);
  } else if (wide_tile(n_tiles, 8, m_tiles)) {
    dim3 grid(ceil_div(n_tiles, 8), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_WIDE(TEPI_F32)), grid, dim3(512), 0, st, rc, xv, wv, nullptr, out, nullptr, N, K, (int*)nullptr);
  } else {
    dim3 grid(ceil_div(n_tiles, 4), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_NARROW(TEPI_F32)), grid, dim3(256), 0, st, rc, xv, wv, nullptr, out, nullptr, N, K, (int*)nullptr);
  }
}

void launch_gemm_tile_swiglu(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                             bf16_t* act, int F, int K) {
  const int f_tiles = F >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  const bf16x8* xv = reinterpret_cast<const bf16x8*>(x);
  const bf16x8* gv = reinterpret_cast<const bf16x8*>(Wg);
  const bf16x8* uv = reinterpret_cast<const bf16x8*>(Wu);
  if (K % 32 != 0) {
    dim3 grid(ceil_div(f_tiles, 2), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_REGS(TEPI_SWIGLU)), grid, dim3(256), 0, st, rc, xv, gv, uv, nullptr, act, F, K);
  } else if (wide_tile(f_tiles, 4, m_tiles)) {
    dim3 grid(ceil_div(f_tiles, 4), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_WIDE(TEPI_SWIGLU)), grid, dim3(512), 0, st, rc, xv, gv, uv, nullptr, act, F, K, (int*)nullptr);
  } else {
    dim3 grid(ceil_div(f_tiles, 2), ceil_div(m_tiles, 8));
    hipLaunchKernelGGL((TILE_NARROW(TEPI_SWIGLU)), grid, dim3(256), 0, st, rc, xv, gv, uv, nullptr, act, F, K, (int*)nullptr);
  }
}

// Decode with many rows in flight: fused gate/up + SiLU*mul with the skinny kernel's summation
// chains (see CHAIN above) and, when ssq is set, the folded RMSNorm of that kernel.  Returns
// false (nothing launched) when the shape does not allow it.
// Measured on MI355X, fused gate/up of a 4096 x 14336 (2560 x 9728) MLP, event pairs around eager
// launches: at a row bound of 128 the half-height tile takes 76 (43) us against 84 (53) us for the
// skinny kernel (tie at 96, slower at 64); at 256 the full tile 91 (60) us against 132 (67) us;
// beyond 256 rows (two row groups) it only pays where the weight tiles alone fill the chip.
// A ring deeper than 3 stages made these variants 1.8x slower (the plain kernel does not care).
bool launch_gemm_tile_swiglu_chain(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wg, const bf16_t* Wu,
                                   bf16_t* act, int F, int K, const float* ssq, int ssq_stride, float eps) {
  if (K % 128 != 0 || F % 32 != 0) return false;     // quarter boundaries on stage boundaries (BK = 2)
  if (rc.max_rows > 256 && F < 12288) return false;
  if (rc.max_rows <= 128) {
    // half-height tile (128 rows x 64 features, 2 x 2 accumulator tiles per wavefront)
    dim3 grid(ceil_div(F >> 5, 2), 1);
    hipLaunchKernelGGL((gemm_tile_chain_kernel<2, 2, 2, 2, 2, 3, TEPI_SWIGLU>), grid, dim3(256), 0, st, rc,
                       reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wg),
                       reinterpret_cast<const bf16x8*>(Wu), nullptr, act, F, K,
                       TileNorm{ssq, ssq_stride, K >> 5, 1.0f / (float)K, eps, nullptr});
    return true;
  }
  const int f_tiles = F >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  const TileNorm tn{ssq, ssq_stride, K >> 5, 1.0f / (float)K, eps, nullptr};
  if (rc.max_rows <= 192) {
    // 192-row tile (3 accumulator row tiles per wavefront): a quarter less matrix work and LDS
    // traffic than the full tile would spend on rows that are not there
    dim3 grid(ceil_div(f_tiles, 2), 1);
    hipLaunchKernelGGL((gemm_tile_chain_kernel<2, 2, 3, 2, 2, 3, TEPI_SWIGLU>), grid, dim3(256), 0, st, rc,
                       reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wg),
                       reinterpret_cast<const bf16x8*>(Wu), nullptr, act, F, K, tn);
    return true;
  }
  // 256 rows x 64 features on 8 wavefronts of 64 x 64: with both accumulator sets a wavefront
  // stays within 160 registers, so two or three run per SIMD (4 wavefronts of 128 x 64 need
  // the whole register file each: 105 against 97 us per launch on the 4096 x 14336 MLP)
  dim3 grid(ceil_div(f_tiles, 2), ceil_div(m_tiles, 8));
  hipLaunchKernelGGL((gemm_tile_chain_kernel<4, 2, 2, 2, 2, 3, TEPI_SWIGLU>), grid, dim3(512), 0, st, rc,
                     reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wg),
                     reinterpret_cast<const bf16x8*>(Wu), nullptr, act, F, K, tn);
  return true;
}

// Split-k projections (qkv, down) with more than 128 rows in flight: 256 rows x 64 columns per
// workgroup on 4 wavefronts of 64 x 64, one k slice per workgroup (grid.z), the skinny kernel's
// summation chains (four quarter chains per slice, added in order; the consumer adds the slices).
// Each weight tile is fetched once for all rows (the skinny kernel runs a second group of rows
// over the same weights).  Returns false (nothing launched) unless every slice and every quarter
// of a slice is a whole number of stages.
bool launch_gemm_tile_chain_f32(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* out, int N, int K,
                                int ksplit, size_t partial_stride) {
  const int KT = K >> 4, n_tiles = N >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  if (K % 16 != 0 || N % 32 != 0 || ksplit < 1 || KT % (ksplit * 4 * 2) != 0) return false;
  TileNorm tn{};
  tn.ksplit = ksplit;
  tn.partial_stride = partial_stride;
  dim3 grid(ceil_div(n_tiles, 2), ceil_div(m_tiles, 8), ksplit);
  hipLaunchKernelGGL((gemm_tile_chain_kernel<4, 1, 2, 2, 2, 3, TEPI_F32>), grid, dim3(256), 0, st, rc,
                     reinterpret_cast<const bf16x8*>(x), reinterpret_cast<const bf16x8*>(Wp), nullptr, out, nullptr, N, K,
                     tn);
  return true;
}

// LM head for many rows: logits plus the maxima of every 64 columns.  Same accumulation chain
// per element as the skinny LM-head kernel (k-tiles in order, one accumulator), so the choice
// between the two changes no bit.  Needs V % 64 == 0 and K % 32 == 0.
void launch_gemm_tile_logits(hipStream_t st, RowCtx rc, const bf16_t* x, const bf16_t* Wp, float* logits,
                             float* group_max, int V, int K, int* group_idx) {
  const int n_tiles = V >> 5, m_tiles = ceil_div(rc.max_rows, 32);
  dim3 grid(ceil_div(n_tiles, 8), ceil_div(m_tiles, 8));
  hipLaunchKernelGGL((TILE_WIDE(TEPI_LOGITS)), grid, dim3(512), 0, st, rc, reinterpret_cast<const bf16x8*>(x),
                     reinterpret_cast<const bf16x8*>(Wp), nullptr, logits, reinterpret_cast<bf16_t*>(group_max), V, K, group_idx);
}

}  // namespace april
