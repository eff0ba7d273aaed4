// Paged-attention decode for bf16 KV, gfx950.
//
// One workgroup (4 wavefronts) per (row, KV head, KV split of ATT_SPLIT tokens).  The
// wavefronts take the split's 32-token tiles round-robin, each keeps an online softmax
// in registers, the four partial results are merged through LDS in wavefront order;
// when a context spans several splits the merged partials go to a workspace and a small
// second kernel merges them in split order (deterministic: the order of every
// floating-point sum depends on the row's own length only).  The kernel boundary is the
// cheapest device-wide ordering on this chip: publishing the partials behind agent-scope
// fences and letting the last workgroup merge cost more than the extra launch.
//
// Both products run on v_mfma_f32_16x16x32_bf16, computed transposed so that no
// operand has to be re-laid between them:
//   S^T[token, head] = K[token, :] . Q[head, :]      A = K fragment, B = Q^T fragment
//   O^T[dim,  head]  = V^T[dim, token] . P^T[token, head]
// The accumulator of the first product (lane l: head l%16, tokens 4*(l/16)+i of a
// 16-token page) is, after exp(), directly the B operand of the second product: its
// k index runs over (page A tokens 4g..4g+3, page B tokens 4g..4g+3), and the V^T
// fragment is loaded with the same token order.
//
// FUSED (decode iterations): the kernel also does the rotary embedding and the KV append of
// the row's new token, so no separate kernel runs between the QKV GEMM and attention.  Every
// workgroup sums the split-K partials of its query heads and rotates them; the workgroup of
// the last KV split computes the new token's rotated key and its value, stores them in the
// page as bf16, and substitutes exactly those bf16 values into the fragments of the tile
// that holds the position, so the products are bit-identical to reading them back.
// (Prefill keeps the separate rope/append kernel: its rows attend to each other's new keys.)
//
// KV page layout (written by rope_append_kernel or here, mode 1), per (page, KV head):
//   K: MFMA A-fragment order  [d/32][lane = t + 16*((d%32)/8)][d%8]   -> 1 KiB coalesced loads
//   V: transposed             [d][t]                                 -> 8-byte loads, 512 B/wave coalesced
#include "kernels.h"

namespace april {

#ifndef ATT_SPLIT_64
#define ATT_SPLIT_64 1024
#endif
#ifndef ATT_SPLIT_128
#define ATT_SPLIT_128 4096
#endif
// tokens per KV split, a multiple of 1024 (a lane holds one page id per 1024 tokens of the split).
// head_dim 64 (small model, 2 KV heads): 2048 was 1.6 % slower end to end than 1024; 512: 7 % slower
// on long rows.  head_dim 128, launched over the length-sorted work list: the kernel itself is
// 1 % slower with 4096-token splits than with 1024 (160.8 against 158.7 us on the 4.4 B
// configuration), but few rows then need the merge kernel at all, and the run is 1 % faster end to
// end on each of the three wide configurations (before the work list, on a grid launch, 2048-token
// splits cost 4.5 % on a ragged batch).
constexpr int att_split(int dh) { return dh == 64 ? ATT_SPLIT_64 : (dh == 128 ? ATT_SPLIT_128 : 1024); }
// wavefronts per workgroup (8 for head_dim <= 64 was measured: 11.8 us against 10.6 us per launch)
#ifndef ATT_WAVES_128
#define ATT_WAVES_128 4
#endif
constexpr int att_waves(int dh, bool fused) { return dh == 128 ? ATT_WAVES_128 : 4; }

struct AttnFuse {              // inputs of the fused rotary + append (FUSED only)
  const float* qkv;            // fp32 [n_partials][rows][(Hq + 2 Hkv) * dh] split-K partials of the QKV GEMM
  int n_partials;
  size_t partial_stride;
  const float* rope_cos;       // [pos][dh/2]
  const float* rope_sin;
};

template <int DH, bool FUSED>
__global__ __launch_bounds__(64 * att_waves(DH, FUSED)) __attribute__((amdgpu_waves_per_eu(2))) void attn_decode_kernel(
    RowCtx rc, int row_base, Slots s, const float* __restrict__ q_rot, bf16_t* kv_pool, KVLayout L, int layer,
    int Hq, bf16_t* __restrict__ out, float* __restrict__ ws, int max_splits, AttnFuse fz,
    const int4* __restrict__ items) {
  constexpr int KC = DH / 32;      // k-chunks of the QK product
  constexpr int DT = DH / 16;      // dim tiles of the PV product
  constexpr int REC = 32 + 16 * DH;   // floats of one partial result: m[16], l[16], o[16][DH]
  constexpr int ATT_WAVES = att_waves(DH, FUSED);
  constexpr int RS = DH + 4;          // padded row stride of O in LDS
  constexpr int LREC = 32 + 16 * RS;
  __shared__ float lds[ATT_WAVES * LREC];
  __shared__ bf16_t s_knew[DH], s_vnew[DH];
  // Workgroup ids are dealt to the 8 XCDs in turn, so with a row count that is a multiple of 8 the
  // plain mapping would put every (KV head, split) of a row on one XCD and a long row would
  // overload it.  Rotating the row index by the other two coordinates spreads a row's
  // workgroups over the XCDs (a bijection of blockIdx.x for fixed y and z).
  //
  // With a work list (items != nullptr; 1-D launch) the scheduler kernel has listed this
  // iteration's (row, split) pairs longest first: entry 0 holds their number, entry 1 + i =
  // {row, split, slot, position}.  Workgroup id = item * n_kv_heads + KV head, so the long items
  // start first, the launch ends on the short ones, no workgroup is launched for a split its row
  // does not have, and the KV heads of one item go to different XCDs.
  int kvh, split, wr, slot, pos;
  if (items != nullptr) {
    const int nkv = L.n_kv_heads;
    const int item = (int)blockIdx.x / nkv;
    kvh = (int)blockIdx.x - item * nkv;
    const int4 head = items[0], it = items[1 + item];
    const int2 ctl = *rc.ctl;
    if (ctl.y || item >= head.x) return;
    wr = __builtin_amdgcn_readfirstlane(it.x);
    split = __builtin_amdgcn_readfirstlane(it.y);
    slot = __builtin_amdgcn_readfirstlane(it.z);
    pos = __builtin_amdgcn_readfirstlane(it.w);
  } else {
    kvh = blockIdx.y; split = blockIdx.z;
    wr = (int)((blockIdx.x + blockIdx.y + 3u * blockIdx.z) % gridDim.x);     // wr: workspace row
    // the row arrays hold max_rows entries: fetch them together with the control word
    const int slot_raw = rc.row_slot[row_base + wr], pos_raw = rc.row_pos[row_base + wr];
    ROW_GUARD(rc, row_base + wr);
    slot = slot_raw; pos = pos_raw;
  }
  const int r = row_base + wr;
  const int ctx = pos + 1;
  constexpr int ATT_SPLIT = att_split(DH), PR = ATT_SPLIT / 1024;
  static_assert(ATT_SPLIT % 1024 == 0 && PR >= 1, "split length");
  const int n_splits = (ctx + ATT_SPLIT - 1) / ATT_SPLIT;
  if (split >= n_splits) return;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), hh = lane & 15, g = lane >> 4;
  const int Hkv = L.n_kv_heads, G = Hq / Hkv;
  const int t_begin = split * ATT_SPLIT, t_end = min(ctx, t_begin + ATT_SPLIT);
  const int n_tiles = (t_end - t_begin + 31) >> 5;
  const int n_pages = (t_end - t_begin + 15) >> 4;
  const size_t blk_elems = (size_t)16 * DH;
  const bf16_t* kbase = kv_pool + (size_t)layer * L.layer_stride;
  const bf16_t* vbase = kbase + L.kv_stride;

  // page ids of this split: lane i holds page i (one vector load instead of a scalar
  // load per tile inside the loop)
  const int* bt = s.block_table + (size_t)slot * s.max_blocks + (t_begin >> 4);
  int my_page[PR];
#pragma unroll
  for (int q = 0; q < PR; ++q) { const int i = q * 64 + lane; my_page[q] = bt[i < n_pages ? i : n_pages - 1]; }

  // A wavefront takes tiles wave, wave + ATT_WAVES, ... of the split.  Every load inside load_tile
  // is unconditional (a missing second page is clamped), so the wait counts around it are static.
  auto load_tile = [&](int tile, bf16x8 (&kk)[2][KC], bf16x4 (&vv)[2][DT]) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      int pl = 2 * tile + p;                                   // page within the split
      pl = pl < n_pages ? pl : n_pages - 1;                    // a missing second page re-reads the last one
      const int pls = __builtin_amdgcn_readfirstlane(pl);
      int page = __builtin_amdgcn_readlane(my_page[0], pls & 63);
#pragma unroll
      for (int q = 1; q < PR; ++q)
        if ((pls >> 6) == q) page = __builtin_amdgcn_readlane(my_page[q], pls & 63);
      const size_t off = ((size_t)page * Hkv + kvh) * blk_elems;
      const bf16x8* kp = reinterpret_cast<const bf16x8*>(kbase + off);
      const bf16x4* vp = reinterpret_cast<const bf16x4*>(vbase + off);
#pragma unroll
      for (int c = 0; c < KC; ++c) kk[p][c] = kp[c * 64 + lane];
#pragma unroll
      for (int d = 0; d < DT; ++d) vv[p][d] = vp[(d * 16 + hh) * 4 + g];
    }
  };

  constexpr bool DEEP = DH <= 64;              // two tiles in flight behind the one being used
  bf16x8 kf[2][KC], km[DEEP ? 2 : 1][KC];
  bf16x4 vf[2][DT], vm[DEEP ? 2 : 1][DT];
  auto first_tiles = [&]() {
    load_tile(wave < n_tiles ? wave : n_tiles - 1, kf, vf);
    if constexpr (DEEP) {
      // (an array reference of the right shape for the lambda)
      auto& km2 = reinterpret_cast<bf16x8 (&)[2][KC]>(km);
      auto& vm2 = reinterpret_cast<bf16x4 (&)[2][DT]>(vm);
      load_tile(wave + ATT_WAVES < n_tiles ? wave + ATT_WAVES : n_tiles - 1, km2, vm2);
    }
  };

  // Q^T fragments: lane holds q[head hh][32c + 8g .. +7]; heads beyond the group read
  // the group's last head and are zeroed.
  constexpr int HALF = DH / 2;
  const bool last_split = split == n_splits - 1;
  bf16x8 qf[KC];
  if (FUSED) {
    // Order of requests: (1) the page ids (above), (2) everything that depends on the row only -
    // the q partials, the rotary table, for the owner of the new token also its k / v partials -
    // (3) the first KV tiles, which need the page ids.  Loads complete in order, so waiting for
    // (2) does not wait for (3), and the rotation arithmetic runs while the tiles arrive.
    // Narrow heads: (2) and (3) fit the register file together.  Wide heads: (2) for every k-chunk
    // at once fits only while the tile registers are still free, so the rotation runs before (3)
    // is requested - one round trip for all of (2) instead of one per k-chunk and partial.
    constexpr bool ALL = true;
    constexpr bool TILES_FIRST = DH <= 64;
    constexpr int QC = ALL ? KC : 1;
    constexpr int QB = DH <= 64 ? 4 : 2;        // partials requested together
    const int hq = hh < G ? hh : G - 1;
    const int ncol = (Hq + 2 * Hkv) * DH;
    const float* qsrc = fz.qkv + (size_t)r * ncol + (size_t)(kvh * G + hq) * DH;
    const float* ksrc = fz.qkv + (size_t)r * ncol + (size_t)(Hq + kvh) * DH;
    const float* vsrc = fz.qkv + (size_t)r * ncol + (size_t)(Hq + Hkv + kvh) * DH;
    const float* cs = fz.rope_cos + (size_t)pos * HALF;
    const float* sn = fz.rope_sin + (size_t)pos * HALF;
    const bool owner = last_split && wave == 0;         // computes and stores the new key / value
    f32x4 la[QC][QB][2], lb[QC][QB][2], c4[QC][2], s4[QC][2];
    float nka[QB], nkb[QB], nvv[QB], ncs = 0.f, nsn = 0.f;
    auto request_q = [&](int c, int slot_c, int p0) {
      const int d0 = 32 * c + 8 * g;            // 8 consecutive dims, all in the same half
      const int i0 = d0 < HALF ? d0 : d0 - HALF;
#pragma unroll
      for (int u = 0; u < QB; ++u) {
        const int p = p0 + u < fz.n_partials ? p0 + u : fz.n_partials - 1;
        const float* q = qsrc + p * fz.partial_stride;
        la[slot_c][u][0] = *reinterpret_cast<const f32x4*>(q + i0);
        la[slot_c][u][1] = *reinterpret_cast<const f32x4*>(q + i0 + 4);
        lb[slot_c][u][0] = *reinterpret_cast<const f32x4*>(q + i0 + HALF);
        lb[slot_c][u][1] = *reinterpret_cast<const f32x4*>(q + i0 + HALF + 4);
      }
      if (p0 == 0) {
        c4[slot_c][0] = *reinterpret_cast<const f32x4*>(cs + i0);
        c4[slot_c][1] = *reinterpret_cast<const f32x4*>(cs + i0 + 4);
        s4[slot_c][0] = *reinterpret_cast<const f32x4*>(sn + i0);
        s4[slot_c][1] = *reinterpret_cast<const f32x4*>(sn + i0 + 4);
      }
    };
    // new token, dim d = lane (+64 for the second pass of wide heads): pair index and partials
    auto request_kv = [&](int d, int p0) {
      const int i = d < HALF ? d : d - HALF;
#pragma unroll
      for (int u = 0; u < QB; ++u) {
        const size_t po = (size_t)(p0 + u < fz.n_partials ? p0 + u : fz.n_partials - 1) * fz.partial_stride;
        nka[u] = ksrc[po + i]; nkb[u] = ksrc[po + i + HALF]; nvv[u] = vsrc[po + d];
      }
      if (p0 == 0) { ncs = cs[i]; nsn = sn[i]; }
    };
    if constexpr (ALL) {
#pragma unroll
      for (int c = 0; c < KC; ++c) request_q(c, c, 0);
      if (owner && lane < DH) request_kv(lane, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (TILES_FIRST) {
      first_tiles();
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const int sc = ALL ? c : 0;
      const bool lo = 32 * c + 8 * g < HALF;
      f32x4 a[2] = {f32x4{}, f32x4{}}, b[2] = {f32x4{}, f32x4{}};
      // partials are added in the order p = 0, 1, ... (as rope_append_kernel does); four at a
      // time are requested together so that the additions do not serialise the loads
      for (int p0 = 0; p0 < fz.n_partials; p0 += QB) {
        if (!ALL || p0 > 0) request_q(c, sc, p0);
#pragma unroll
        for (int u = 0; u < QB; ++u)
          if (p0 + u < fz.n_partials) { a[0] += la[sc][u][0]; a[1] += la[sc][u][1]; b[0] += lb[sc][u][0]; b[1] += lb[sc][u][1]; }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float av = a[j >> 2][j & 3], bv = b[j >> 2][j & 3], cv = c4[sc][j >> 2][j & 3], sv2 = s4[sc][j >> 2][j & 3];
        const float rot = lo ? rope_first(av, bv, cv, sv2) : rope_second(av, bv, cv, sv2);
        qf[c][j] = hh < G ? (bf16_t)rot : (bf16_t)0.f;
      }
    }
    if constexpr (!TILES_FIRST) {
      __builtin_amdgcn_sched_barrier(0);
      first_tiles();
      __builtin_amdgcn_sched_barrier(0);
    }
    if (owner) {
      // the new token: rotated key and value of this KV head, to the page and to LDS
      const int page = s.block_table[(size_t)slot * s.max_blocks + (pos >> 4)], tin = pos & 15;
      for (int d = lane; d < DH; d += 64) {
        const bool lo = d < HALF;
        float av = 0.f, bv = 0.f, vv = 0.f;
        for (int p0 = 0; p0 < fz.n_partials; p0 += QB) {
          if (!ALL || p0 > 0 || d >= 64) request_kv(d, p0);
#pragma unroll
          for (int u = 0; u < QB; ++u)
            if (p0 + u < fz.n_partials) { av += nka[u]; bv += nkb[u]; vv += nvv[u]; }
        }
        const float rot = lo ? rope_first(av, bv, ncs, nsn) : rope_second(av, bv, ncs, nsn);
        const bf16_t kb = (bf16_t)rot, vb = (bf16_t)vv;
        s_knew[d] = kb;
        s_vnew[d] = vb;
        kv_pool[L.at(layer, 0, page, kvh, tin, d)] = kb;
        kv_pool[L.at(layer, 1, page, kvh, tin, d)] = vb;
      }
    }
    if (last_split) __syncthreads();
  } else {
    first_tiles();
    __builtin_amdgcn_sched_barrier(0);
    const int hq = hh < G ? hh : G - 1;
    const float* q = q_rot + (size_t)r * Hq * DH + (size_t)(kvh * G + hq) * DH + 8 * g;
    f32x4 qa[KC][2];
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      qa[c][0] = *reinterpret_cast<const f32x4*>(q + 32 * c);
      qa[c][1] = *reinterpret_cast<const f32x4*>(q + 32 * c + 4);
    }
#pragma unroll
    for (int c = 0; c < KC; ++c)
#pragma unroll
      for (int j = 0; j < 8; ++j) qf[c][j] = hh < G ? (bf16_t)qa[c][j >> 2][j & 3] : (bf16_t)0.f;
  }
  const float scale = 1.0f / sqrtf((float)DH);
  float m_run = -INFINITY, l_run = 0.f;
  f32x4 oacc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d) oacc[d] = f32x4{};

  // One tile: scores, online softmax, PV; reads kf / vf.
  auto compute_tile = [&](int tile) {
    const int t0 = t_begin + tile * 32;
    if (FUSED && last_split && tile == ((pos - t_begin) >> 5)) {
      // the tile that holds the new token: take its key / value from LDS (the page copy may
      // not be visible yet); same bf16 values as the page now holds
      const int pp = ((pos - t_begin) >> 4) & 1, tin = pos & 15;
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        if (p != pp) continue;
        if (hh == tin) {
#pragma unroll
          for (int c = 0; c < KC; ++c)
#pragma unroll
            for (int j = 0; j < 8; ++j) kf[p][c][j] = s_knew[32 * c + 8 * g + j];
        }
        if ((tin >> 2) == g) {
#pragma unroll
          for (int d = 0; d < DT; ++d) {
            const bf16_t nv = s_vnew[d * 16 + hh];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              if (j == (tin & 3)) vf[p][d][j] = nv;
          }
        }
      }
    }
    f32x4 sacc[2];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      sacc[p] = f32x4{};
#pragma unroll
      for (int c = 0; c < KC; ++c)
        sacc[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[p][c], qf[c], sacc[p], 0, 0, 0);
    }
    float sv[8];
    float mx = -INFINITY;
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int tok = t0 + p * 16 + 4 * g + i;
        const float v = tok < t_end ? sacc[p][i] * scale : -INFINITY;
        sv[p * 4 + i] = v;
        mx = fmaxf(mx, v);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float corr = __expf(m_run - m_new);
    float rs = 0.f;
    bf16x8 pf;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float pe = __expf(sv[e] - m_new);
      rs += pe;
      pf[e] = (bf16_t)pe;
    }
    rs += __shfl_xor(rs, 16, 64);
    rs += __shfl_xor(rs, 32, 64);
    l_run = l_run * corr + rs;
    m_run = m_new;
#pragma unroll
    for (int d = 0; d < DT; ++d) {
      oacc[d] *= corr;
      bf16x8 af;
#pragma unroll
      for (int j = 0; j < 4; ++j) { af[j] = vf[0][d][j]; af[4 + j] = vf[1][d][j]; }
      oacc[d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, pf, oacc[d], 0, 0, 0);
    }
  };
  // Steady state: the tile AHEAD tiles further on is requested before this one is used.  The
  // tiles that have no such successor are peeled off below, so no wavefront ends its loop
  // waiting for a load it will not use (that wait was a full memory latency per wavefront).
  if (wave < n_tiles) {
    constexpr int AHEAD = (DEEP ? 2 : 1) * ATT_WAVES;
    int tile = wave;
    for (; tile + AHEAD < n_tiles; tile += ATT_WAVES) {
      bf16x8 kn[2][KC];
      bf16x4 vn[2][DT];
      load_tile(tile + AHEAD, kn, vn);
      __builtin_amdgcn_sched_barrier(0);
      compute_tile(tile);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < 2; ++p) {
#pragma unroll
        for (int c = 0; c < KC; ++c) {
          if constexpr (DEEP) { kf[p][c] = km[p][c]; km[p][c] = kn[p][c]; } else kf[p][c] = kn[p][c];
        }
#pragma unroll
        for (int d = 0; d < DT; ++d) {
          if constexpr (DEEP) { vf[p][d] = vm[p][d]; vm[p][d] = vn[p][d]; } else vf[p][d] = vn[p][d];
        }
      }
    }
    compute_tile(tile);                          // tile < n_tiles here: the loop leaves at least one
    if constexpr (DEEP) {
      if (tile + ATT_WAVES < n_tiles) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
#pragma unroll
          for (int c = 0; c < KC; ++c) kf[p][c] = km[p][c];
#pragma unroll
          for (int d = 0; d < DT; ++d) vf[p][d] = vm[p][d];
        }
        compute_tile(tile + ATT_WAVES);
      }
    }
  }

  // ---- merge the wavefronts of this workgroup through LDS, in wavefront order -----------
  // Every wavefront publishes (m, l, O); then each merges its share of the dim tiles (tile d
  // goes to wavefront d % ATT_WAVES) and writes it out, so the tail of a workgroup's life is
  // shared by all of them.  Rows of O are padded by 4 floats in LDS: with a stride of DH floats
  // the 16 heads of a lane group would all hit the same banks.
  {
    float* my = lds + wave * LREC;
    if (g == 0) { my[hh] = m_run; my[16 + hh] = l_run; }
#pragma unroll
    for (int d = 0; d < DT; ++d) *reinterpret_cast<f32x4*>(my + 32 + hh * RS + d * 16 + 4 * g) = oacc[d];
  }
  __syncthreads();
  float M = lds[hh];
#pragma unroll
  for (int w = 1; w < ATT_WAVES; ++w) M = fmaxf(M, lds[w * LREC + hh]);
  float wgt[ATT_WAVES], lsum = 0.f;
#pragma unroll
  for (int w = 0; w < ATT_WAVES; ++w) {
    wgt[w] = __expf(lds[w * LREC + hh] - M);
    lsum += wgt[w] * lds[w * LREC + 16 + hh];
  }
  const int K = Hq * DH;
  const float inv = 1.0f / lsum;
  float* rec = ws + (((size_t)wr * Hkv + kvh) * max_splits + split) * REC;     // several splits: (m, l, O) for the merge kernel
  for (int d = wave; d < DT; d += ATT_WAVES) {
    f32x4 o = f32x4{};
#pragma unroll
    for (int w = 0; w < ATT_WAVES; ++w)
      o += *reinterpret_cast<const f32x4*>(lds + w * LREC + 32 + hh * RS + d * 16 + 4 * g) * wgt[w];
    if (n_splits == 1) {
      if (hh < G) {
        bf16x4 ob;
#pragma unroll
        for (int i = 0; i < 4; ++i) ob[i] = (bf16_t)(o[i] * inv);
        *reinterpret_cast<bf16x4*>(out + act_index<true>(r, (kvh * G + hh) * DH + d * 16 + 4 * g, K)) = ob;
      }
    } else if (hh < G) {
      // record layout [dim tile][head][16 dims]: the lanes of one store cover consecutive
      // addresses, and only the G heads of the group are written (and read back)
      *reinterpret_cast<f32x4*>(rec + 32 + (d * 16 + hh) * 16 + 4 * g) = o;
    }
  }
  if (n_splits > 1 && wave == 0 && g == 0) { rec[hh] = M; rec[16 + hh] = lsum; }
}

// Merge of the per-split partial results of the rows whose context spans several splits
// (one wavefront per (row, KV head); rows with a single split were finished by the main
// kernel).  Split order, so a row's result depends on its own length only.
template <int DH>
__global__ __launch_bounds__(64) void attn_merge_kernel(RowCtx rc, int row_base, int Hkv, int Hq,
                                                        bf16_t* __restrict__ out, const float* __restrict__ ws,
                                                        int max_splits) {
  constexpr int DT = DH / 16;
  constexpr int REC = 32 + 16 * DH;
  const int wr = blockIdx.x, r = row_base + wr, kvh = blockIdx.y;
  const int pos = rc.row_pos[r];
  ROW_GUARD(rc, r);
  constexpr int ATT_SPLIT = att_split(DH);
  const int n_splits = (pos + ATT_SPLIT) / ATT_SPLIT;          // ceil((pos + 1) / ATT_SPLIT)
  if (n_splits == 1) return;
  const int lane = threadIdx.x, hh = lane & 15, g = lane >> 4;
  const int G = Hq / Hkv, K = Hq * DH;
  const float* base = ws + ((size_t)wr * Hkv + kvh) * max_splits * REC;
  // every load of the merge is independent of the others: issue them in batches
  float M = -INFINITY;
#pragma unroll
  for (int k = 0; k < 8; ++k) {                      // max_splits <= 32: lane group g takes splits g, g+4, ...
    const int si = g + 4 * k;
    M = fmaxf(M, base[(size_t)(si < n_splits ? si : n_splits - 1) * REC + hh]);
  }
  M = fmaxf(M, __shfl_xor(M, 16, 64));
  M = fmaxf(M, __shfl_xor(M, 32, 64));
  float lsum = 0.f;
  f32x4 acc[DT];
#pragma unroll
  for (int d = 0; d < DT; ++d) acc[d] = f32x4{};
  for (int i0 = 0; i0 < n_splits; i0 += 2) {
    float mi[2], li[2];
    f32x4 o[2][DT];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const float* p = base + (size_t)(i0 + u < n_splits ? i0 + u : n_splits - 1) * REC;
      mi[u] = p[hh];
      li[u] = p[16 + hh];
#pragma unroll
      for (int d = 0; d < DT; ++d)
        o[u][d] = hh < G ? *reinterpret_cast<const f32x4*>(p + 32 + (d * 16 + hh) * 16 + 4 * g) : f32x4{};
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const float wgt = i0 + u < n_splits ? __expf(mi[u] - M) : 0.f;
      lsum += wgt * li[u];
#pragma unroll
      for (int d = 0; d < DT; ++d) acc[d] += o[u][d] * wgt;
    }
  }
  if (hh < G) {
    const float inv = 1.0f / lsum;
#pragma unroll
    for (int d = 0; d < DT; ++d) {
      bf16x4 o;
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = (bf16_t)(acc[d][i] * inv);
      *reinterpret_cast<bf16x4*>(out + act_index<true>(r, (kvh * G + hh) * DH + d * 16 + 4 * g, K)) = o;
    }
  }
}

// ---------------------------------------------------------------------------
// Causal attention of prefill rows, tiled over queries.
//
// The decode kernel serves one query position per workgroup; run over the rows of a prompt it
// reads the prompt's keys and values once per position.  Here a workgroup owns a tile of query
// positions of one (sequence, KV head) and streams the keys / values 0 .. last position of the
// tile once, for all of them and for all query heads of the KV head.
//
// Same transposed products as the decode kernel (S^T = K . Q^T, O^T = V^T . P^T on
// v_mfma_f32_16x16x32_bf16), with the 16 columns of a product holding (position, head) pairs:
// column = position_in_tile * GP + head, GP = heads per KV head rounded up to a power of two.
// A wavefront keeps CT = 4 column tiles (its own positions: 64 / GP of them), so a K / V tile
// fetched once feeds four products; the four wavefronts of a workgroup take consecutive groups
// of positions and walk the same K / V tiles (second and later readers hit the L1 / L2).
// Every column runs its own online softmax over the 32-token tiles in order; positions beyond
// the column's own are masked.  A sequence's result does not depend on what else is in the
// chunk.  (Its summation order differs from the decode kernel's; so does the prefill GEMM's.)
// Column tiles per wavefront, measured on 16384-row chunks of 512-token prompts, head_dim 128,
// 4 query heads per KV head: 4 tiles 452 us per launch, 2 tiles (two wavefronts per SIMD) 511 us,
// 1 tile 498 us.
// ---------------------------------------------------------------------------
#ifndef PF_CT
#define PF_CT 4
#endif
template <int DH, int GP>
__global__ __launch_bounds__(256) void attn_prefill_kernel(const int4* __restrict__ items, Slots s,
                                                           const float* __restrict__ q_rot,
                                                           const bf16_t* __restrict__ kv_pool, KVLayout L, int layer,
                                                           int Hq, bf16_t* __restrict__ out) {
  constexpr int KC = DH / 32, DT = DH / 16, CT = PF_CT;
  constexpr int PPT = 16 / GP;            // positions per column tile
  constexpr int PPW = CT * PPT;           // positions per wavefront
  const int4 it = items[blockIdx.x];      // {slot, first row of the sequence, tokens of the sequence, first position of the tile}
  const int slot = it.x, row0 = it.y, nt = it.z, q0 = it.w;
  const int kvh = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), hh = lane & 15, g = lane >> 4;
  const int Hkv = L.n_kv_heads, G = Hq / Hkv;
  const int wq0 = q0 + wave * PPW;        // this wavefront's first position
  if (wq0 >= nt) return;                  // (no workgroup barrier below)
  const int wlast = min(nt, wq0 + PPW) - 1;
  const size_t blk_elems = (size_t)16 * DH;
  const bf16_t* kbase = kv_pool + (size_t)layer * L.layer_stride;
  const bf16_t* vbase = kbase + L.kv_stride;
  const int* bt = s.block_table + (size_t)slot * s.max_blocks;
  const int last_page = wlast >> 4;

  // query fragments: column hh of tile ct = (position, head)
  int qpos[CT];
  bool qok[CT];
  bf16x8 qf[CT][KC];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    const int p = wq0 + ct * PPT + hh / GP, h = hh % GP;
    qok[ct] = p < nt && h < G;
    qpos[ct] = p < nt ? p : nt - 1;
    const int hc = h < G ? h : G - 1;
    const float* q = q_rot + (size_t)(row0 + qpos[ct]) * Hq * DH + (size_t)(kvh * G + hc) * DH + 8 * g;
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(q + 32 * c), b = *reinterpret_cast<const f32x4*>(q + 32 * c + 4);
#pragma unroll
      for (int j = 0; j < 4; ++j) { qf[ct][c][j] = qok[ct] ? (bf16_t)a[j] : (bf16_t)0.f; qf[ct][c][4 + j] = qok[ct] ? (bf16_t)b[j] : (bf16_t)0.f; }
    }
  }
  const float scale = 1.0f / sqrtf((float)DH);
  float m_run[CT], l_run[CT];
  f32x4 oacc[CT][DT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    m_run[ct] = -INFINITY; l_run[ct] = 0.f;
#pragma unroll
    for (int d = 0; d < DT; ++d) oacc[ct][d] = f32x4{};
  }

  const int n_tiles = (wlast >> 5) + 1;
  int my_page = bt[lane < last_page ? lane : last_page];     // page ids of tiles 0..31 (64 pages), one per lane
  auto load_tile = [&](int tile, bf16x8 (&kk)[2][KC], bf16x4 (&vv)[2][DT]) {
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      int pl = 2 * tile + p;
      pl = pl < last_page ? pl : last_page;                   // a missing second page re-reads the last one (masked)
      const int page = __builtin_amdgcn_readlane(my_page, __builtin_amdgcn_readfirstlane(pl) & 63);
      const size_t off = ((size_t)page * Hkv + kvh) * blk_elems;
      const bf16x8* kp = reinterpret_cast<const bf16x8*>(kbase + off);
      const bf16x4* vp = reinterpret_cast<const bf16x4*>(vbase + off);
#pragma unroll
      for (int c = 0; c < KC; ++c) kk[p][c] = kp[c * 64 + lane];
#pragma unroll
      for (int d = 0; d < DT; ++d) vv[p][d] = vp[(d * 16 + hh) * 4 + g];
    }
  };
  bf16x8 kf[2][KC];
  bf16x4 vf[2][DT];
  load_tile(0, kf, vf);
  for (int tile = 0; tile < n_tiles; ++tile) {
    bf16x8 kn[2][KC];
    bf16x4 vn[2][DT];
    const int nxt = tile + 1 < n_tiles ? tile + 1 : tile;
    if ((nxt & 31) == 0 && nxt != tile) {                     // the next tile opens a new group of 64 pages
      const int i = nxt * 2 + lane;
      my_page = bt[i < last_page ? i : last_page];
    }
    load_tile(nxt, kn, vn);
    __builtin_amdgcn_sched_barrier(0);
    const int t0 = tile * 32;
    bf16x8 af[DT];
#pragma unroll
    for (int d = 0; d < DT; ++d)
#pragma unroll
      for (int j = 0; j < 4; ++j) { af[d][j] = vf[0][d][j]; af[d][4 + j] = vf[1][d][j]; }
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      if (t0 > __builtin_amdgcn_readfirstlane(wq0 + ct * PPT + PPT - 1)) continue;   // the tile lies beyond every position of this column tile
      f32x4 sacc[2];
#pragma unroll
      for (int p = 0; p < 2; ++p) {
        sacc[p] = f32x4{};
#pragma unroll
        for (int c = 0; c < KC; ++c) sacc[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[p][c], qf[ct][c], sacc[p], 0, 0, 0);
      }
      float sv[8], mx = -INFINITY;
#pragma unroll
      for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int tok = t0 + p * 16 + 4 * g + i;
          const float v = tok <= qpos[ct] ? sacc[p][i] * scale : -INFINITY;
          sv[p * 4 + i] = v;
          mx = fmaxf(mx, v);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[ct], mx);               // finite from the first tile on: token 0 is visible to every position
      const float corr = __expf(m_run[ct] - m_new);
      float rs = 0.f;
      bf16x8 pf;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float pe = __expf(sv[e] - m_new);
        rs += pe;
        pf[e] = (bf16_t)pe;
      }
      rs += __shfl_xor(rs, 16, 64);
      rs += __shfl_xor(rs, 32, 64);
      l_run[ct] = l_run[ct] * corr + rs;
      m_run[ct] = m_new;
#pragma unroll
      for (int d = 0; d < DT; ++d) {
        oacc[ct][d] *= corr;
        oacc[ct][d] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[d], pf, oacc[ct][d], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int p = 0; p < 2; ++p) {
#pragma unroll
      for (int c = 0; c < KC; ++c) kf[p][c] = kn[p][c];
#pragma unroll
      for (int d = 0; d < DT; ++d) vf[p][d] = vn[p][d];
    }
  }
  const int K = Hq * DH;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
    if (!qok[ct]) continue;
    const float inv = 1.0f / l_run[ct];
    const int r = row0 + qpos[ct], h = hh % GP;
#pragma unroll
    for (int d = 0; d < DT; ++d) {
      bf16x4 ob;
#pragma unroll
      for (int i = 0; i < 4; ++i) ob[i] = (bf16_t)(oacc[ct][d][i] * inv);
      *reinterpret_cast<bf16x4*>(out + act_index<true>(r, (kvh * G + h) * DH + d * 16 + 4 * g, K)) = ob;
    }
  }
}

// positions per workgroup of the prefill attention for a model with `group` query heads per KV head
int attn_prefill_tile(int group) {
  int gp = 1;
  while (gp < group) gp <<= 1;
  return 4 * PF_CT * (16 / gp);
}

void launch_attn_prefill(hipStream_t st, const int4* items, int n_items, Slots s, const float* q_rot,
                         const bf16_t* kv_pool, KVLayout kvl, int layer, int n_q_heads, bf16_t* out) {
  if (n_items <= 0) return;
  dim3 grid(n_items, kvl.n_kv_heads);
  const int G = n_q_heads / kvl.n_kv_heads;
  int gp = 1;
  while (gp < G) gp <<= 1;
#define ATT_PF(DH, GP) hipLaunchKernelGGL((attn_prefill_kernel<DH, GP>), grid, dim3(256), 0, st, items, s, q_rot, kv_pool, kvl, layer, n_q_heads, out)
#define ATT_PF_G(DH) switch (gp) { case 1: ATT_PF(DH, 1); break; case 2: ATT_PF(DH, 2); break; case 4: ATT_PF(DH, 4); break; \
                                   case 8: ATT_PF(DH, 8); break; default: ATT_PF(DH, 16); break; }
  switch (kvl.head_dim) {
    case 32: ATT_PF_G(32); break;
    case 64: ATT_PF_G(64); break;
    default: ATT_PF_G(128); break;
  }
#undef ATT_PF_G
#undef ATT_PF
}

int attn_split_tokens(int head_dim) { return att_split(head_dim); }

void launch_attn_decode(hipStream_t st, RowCtx rc, int row_base, Slots s, const float* q_rot, bf16_t* kv_pool,
                        KVLayout kvl, int layer, int n_q_heads, bf16_t* out, float* ws,
                        int max_splits, int grid_splits, const float* fused_qkv, int n_partials,
                        size_t partial_stride, const float* rope_cos, const float* rope_sin, const int4* items) {
  // items: the scheduler's work list of this iteration (decode, row_base 0), or null
  dim3 grid(rc.max_rows, kvl.n_kv_heads, grid_splits);
  if (items != nullptr) grid = dim3((unsigned)rc.max_rows * grid_splits * kvl.n_kv_heads);
  AttnFuse fz{fused_qkv, n_partials, partial_stride, rope_cos, rope_sin};
#define ATT_LAUNCH(DH, F)                                                                                    \
  hipLaunchKernelGGL((attn_decode_kernel<DH, F>), grid, dim3(64 * att_waves(DH, F)), 0, st, rc, row_base, s, q_rot, kv_pool, kvl, layer, \
                     n_q_heads, out, ws, max_splits, fz, items)
  const bool fused = fused_qkv != nullptr;
  switch (kvl.head_dim) {
    case 32: if (fused) ATT_LAUNCH(32, true); else ATT_LAUNCH(32, false); break;
    case 64: if (fused) ATT_LAUNCH(64, true); else ATT_LAUNCH(64, false); break;
    default: if (fused) ATT_LAUNCH(128, true); else ATT_LAUNCH(128, false); break;
  }
#undef ATT_LAUNCH
}

// Second pass for iterations in which some row may span several KV splits.
void launch_attn_merge(hipStream_t st, RowCtx rc, int row_base, KVLayout kvl, int n_q_heads, bf16_t* out,
                       const float* ws, int max_splits) {
  dim3 mgrid(rc.max_rows, kvl.n_kv_heads);
#define ATT_MERGE(DH)                                                                                       \
  hipLaunchKernelGGL((attn_merge_kernel<DH>), mgrid, dim3(64), 0, st, rc, row_base, kvl.n_kv_heads, n_q_heads, out, \
                     ws, max_splits)
  switch (kvl.head_dim) {
    case 32: ATT_MERGE(32); break;
    case 64: ATT_MERGE(64); break;
    default: ATT_MERGE(128); break;
  }
#undef ATT_MERGE
}

}  // namespace april
