// Selective-refresh attention for MANY query rows (a long selected set, step 0, the
// isolated attention op with m = 256): the regime where the m x L x d_h contraction
// is at the matrix-core / HBM ridge rather than bound by streaming K and V once.
// Same mathematics as the few-row kernels (Sec. 4.2 of the d2Cache paper: the selected
// queries attend to all L cached keys without a mask, and A-bar is the head mean of the
// normalised rows), different blocking:
//
//   forward   one workgroup = 64*QT query rows of one head over one range of keys.
//             K and V blocks of 64 keys are staged through LDS once per workgroup, already
//             in matrix-core operand order (one 16-byte fragment per lane, read back with a
//             single conflict-free 16-byte LDS read), double-buffered with the next block's
//             global loads in flight during the arithmetic.  Scores are computed transposed
//             (S^T = K Q^T) so the accumulator of two 16-key tiles IS the 32-key B operand of
//             O^T += V^T P^T; V is transposed 4x4 in registers on its way INTO LDS, once per
//             workgroup instead of once per wave.  Both contractions use the 16x16x32 step.
//             When the grid would not fill the chip the key range is split; every split writes
//             an unnormalised fp32 partial with its running maximum and sum, and a merge
//             kernel combines them in a fixed order (bit-reproducible, no atomics).
//   A-bar     one workgroup = 64 query rows x 16*KA keys, looping over the heads with the K
//             block of each head staged through LDS; exp(s - lse) accumulates in registers.
#include <algorithm>
#include <cmath>

#include "common.h"
#include "internal.h"

namespace d2c {
namespace {

constexpr int kThreads = 256;
constexpr int kBlockKeys = 64;

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }
// two floats -> one register of two bf16 (round to nearest even): a single packed conversion
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

// Workgroup id -> (query block, head, key split).  Ids are dealt round-robin to the 8 XCDs; the query
// blocks that share one (head, split), i.e. the same K and V bytes, get consecutive slots of ONE XCD.
struct TileId {
  int qb, head, split;
  bool valid;
};
__device__ __forceinline__ TileId tile_of(int bid, int q_blocks, int n_heads, int n_splits) {
  const int xcd = bid & 7, slot = bid >> 3;
  const int tile = (slot / q_blocks) * 8 + xcd;
  TileId t;
  t.qb = slot % q_blocks;
  t.head = tile / n_splits;
  t.split = tile - t.head * n_splits;
  t.valid = tile < n_heads * n_splits;
  return t;
}

template <int DH, int QT>
__global__ __launch_bounds__(kThreads) void attn_tiled_fwd_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k_cache, const bf16* __restrict__ v_cache, int m, int L,
    int n_heads, int n_kv_heads, float scale, int keys_per_split, int n_splits, int q_blocks,
    bf16* __restrict__ out, float* __restrict__ lse, float* __restrict__ o_part, float* __restrict__ ml_part) {
  constexpr int NS = DH / 32;            // contraction steps of K Q^T
  constexpr int ND = DH / 16;            // head-dim tiles of O^T
  constexpr int NB = DH / 64;            // 64-wide head-dim blocks (one V staging unit covers 64)
  __shared__ u32x4 k_lds[2][4 * NS * 64];      // [key tile a][step s][lane]
  __shared__ u32x4 v_lds[2][ND * 2 * 64];      // [head-dim tile][32-key step][lane]

  const TileId id = tile_of(blockIdx.x, q_blocks, n_heads, n_splits);
  if (!id.valid) return;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int head = id.head;
  const int kvh = head / (n_heads / n_kv_heads);
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const bf16* kbase = k_cache + (size_t)kvh * DH;
  const bf16* vbase = v_cache + (size_t)kvh * DH;
  const int q0 = id.qb * (64 * QT) + wave * (16 * QT);
  const int key_lo = id.split * keys_per_split;
  const int key_hi = min(L, key_lo + keys_per_split);
  const int n_blocks = (key_hi - key_lo + kBlockKeys - 1) / kBlockKeys;      // >= 1 by the launch plan

  // this wave's queries as B operands of S^T = K Q^T (rows past m repeat row m-1 and are not stored)
  Frag<bf16> qf[QT][NS];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int row = min(q0 + t * 16 + r, m - 1);
    const bf16* qrow = q + (size_t)row * dq + head * DH + g * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[t][s].raw = ld16(qrow + s * 32);
  }

  // staging registers of the K/V block on its way from global memory to LDS: requested at the top of an
  // iteration, stored behind its arithmetic.  Wave w brings key tile w of K (its NS fragments) and one
  // 8-key x 4-value unit of V per lane (unit = 32-key step ks, 64-wide block b).
  struct Stage {
    u32x4 k[NS];
    u32x2 v[2][4];
  };
  Stage stg;
  const int v_b = wave % NB, v_ks = wave / NB;          // v_ks < 2 only for the waves that stage V
  const bool stages_v = NB == 2 || v_ks < 2;            // with two 64-wide blocks all four waves stage V
  const int last_block = n_blocks - 1;
  // Row addresses: a block that lies wholly inside [0, L) uses per-lane pointers fixed at launch plus a
  // uniform block offset; only a ragged last block pays for clamping every row to L-1.
  const bf16* const kfast = kbase + (size_t)(key_lo + wave * 16 + r) * kv_pitch + g * 8;
  const bf16* const vfast = vbase + (size_t)(key_lo + 2 * v_ks * 16 + 4 * g) * kv_pitch + v_b * 64 + 4 * r;
  auto load_block = [&](Stage& sg, int blk_req) {       // past the end: the last block again, never used
    const int blk = min(blk_req, last_block);
    const int key0 = key_lo + blk * kBlockKeys;
    if (key0 + kBlockKeys <= L) {
      const size_t boff = (size_t)blk * kBlockKeys * kv_pitch;
#pragma unroll
      for (int s = 0; s < NS; ++s) sg.k[s] = ld16(kfast + boff + s * 32);
      if (stages_v) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) sg.v[a][e] = ld8(vfast + boff + (size_t)(a * 16 + e) * kv_pitch);
      }
    } else {
      const int key = min(key0 + wave * 16 + r, L - 1);
      const bf16* krow = kbase + (size_t)key * kv_pitch + g * 8;
#pragma unroll
      for (int s = 0; s < NS; ++s) sg.k[s] = ld16(krow + s * 32);
      if (stages_v) {
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int vkey = min(key0 + (2 * v_ks + a) * 16 + 4 * g + e, L - 1);
            sg.v[a][e] = ld8(vbase + (size_t)vkey * kv_pitch + v_b * 64 + 4 * r);
          }
      }
    }
  };
  auto store_block = [&](const Stage& sg, int buf) {
#pragma unroll
    for (int s = 0; s < NS; ++s) k_lds[buf][(wave * NS + s) * 64 + lane] = sg.k[s];
    if (stages_v) {
      // 4x4 transposes: op[a][i] = keys 4g..4g+3 of tile 2ks+a for head-dim value 4r+i of block b
      u32x2 op[2][4];
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        op[a][0] = u32x2{pack_lo(sg.v[a][0].x, sg.v[a][1].x), pack_lo(sg.v[a][2].x, sg.v[a][3].x)};
        op[a][1] = u32x2{pack_hi(sg.v[a][0].x, sg.v[a][1].x), pack_hi(sg.v[a][2].x, sg.v[a][3].x)};
        op[a][2] = u32x2{pack_lo(sg.v[a][0].y, sg.v[a][1].y), pack_lo(sg.v[a][2].y, sg.v[a][3].y)};
        op[a][3] = u32x2{pack_hi(sg.v[a][0].y, sg.v[a][1].y), pack_hi(sg.v[a][2].y, sg.v[a][3].y)};
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        // head-dim value b*64 + 4r + i lives in tile dt at row 4(r%4)+i; the fragment's 8 keys are
        // this lane group's 4 keys of tile 2ks, then of tile 2ks+1: the order P is packed in below
        const int dtile = v_b * 4 + (r >> 2), drow = 4 * (r & 3) + i;
        v_lds[buf][(dtile * 2 + v_ks) * 64 + g * 16 + drow] = u32x4{op[0][i].x, op[0][i].y, op[1][i].x, op[1][i].y};
      }
    }
  };

  // Online softmax in the base-2 domain: p = 2^(s*c - ref) with c = scale*log2(e).  ref is a per-row
  // reference, not necessarily the running maximum: it is only raised (and O, l rescaled) when a block's
  // maximum exceeds it by more than kRaise, so p stays below 2^kRaise.  The result is the same softmax
  // (shift invariance); the decision depends on the data only.  The raise is rare after the first block,
  // and it is the only vector arithmetic on the O accumulators: it lives OUTSIDE the hot loop (the loop
  // leaves through a break, the raise is applied, the block is finished, the loop is entered again), so
  // inside the hot loop the accumulators are touched by matrix-core instructions only and never have to
  // be copied between the accumulator and the vector register files.
  constexpr float kRaise = 8.f;
  const float c2 = scale * 1.44269504088896341f;
  float ref[QT], l_run[QT];
  f32x4 acc[ND][QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    ref[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int d = 0; d < ND; ++d) acc[d][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  constexpr int FB = QT == 1 ? 8 : 16;         // LDS fragments read per batch (one latency per batch)
  f32x4 st[4][QT];
  float tmax2[QT];

  // scores of block blk (S^T = K Q^T, masked past key_hi) and their scaled row maxima; returns whether any
  // row of the wave needs its reference raised
  auto scores = [&](int blk) -> bool {
    const int buf = blk & 1;
    const int key0 = key_lo + blk * kBlockKeys;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int t = 0; t < QT; ++t) st[a][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int b0 = 0; b0 < 4 * NS; b0 += FB) {
      Frag<bf16> kf[FB];
#pragma unroll
      for (int i = 0; i < FB; ++i) kf[i].raw = k_lds[buf][(b0 + i) * 64 + lane];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int t = 0; t < QT; ++t) mfma16(st[(b0 + i) / NS][t], kf[i], qf[t][(b0 + i) % NS]);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (key0 + kBlockKeys > key_hi) {    // ragged last block of the range: keys past the end score -inf
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (key0 + a * 16 + 4 * g + j >= key_hi) {
#pragma unroll
            for (int t = 0; t < QT; ++t) st[a][t][j] = -INFINITY;
          }
    }
    bool need = false;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      float tmax = fmaxf(fmaxf(st[0][t][0], st[0][t][1]), fmaxf(st[0][t][2], st[0][t][3]));
#pragma unroll
      for (int a = 1; a < 4; ++a)
        tmax = fmaxf(tmax, fmaxf(fmaxf(st[a][t][0], st[a][t][1]), fmaxf(st[a][t][2], st[a][t][3])));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 16, kWave));
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
      tmax2[t] = tmax * c2;                            // finite: every block holds at least one key
      need = need || tmax2[t] > ref[t] + kRaise;
    }
    return __builtin_amdgcn_ballot_w64(need) != 0;
  };
  // probabilities of the block against the current references, O^T += V^T P^T, then the block that was
  // requested at the top of the iteration goes to the other LDS buffer
  auto finish = [&](int blk) {
    const int buf = blk & 1;
    Frag<bf16> pf[2][QT];
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const float nref = -ref[t];
      float psum = 0.f;
      float x[4][4];
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          x[a][j] = __builtin_amdgcn_exp2f(fmaf(st[a][t][j], c2, nref));
          psum += x[a][j];
        }
      l_run[t] += psum;                                // this lane's share; lanes are added at the end
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        pf[ks][t].raw = u32x4{pack_bf16(x[2 * ks][0], x[2 * ks][1]), pack_bf16(x[2 * ks][2], x[2 * ks][3]),
                              pack_bf16(x[2 * ks + 1][0], x[2 * ks + 1][1]),
                              pack_bf16(x[2 * ks + 1][2], x[2 * ks + 1][3])};
    }
#pragma unroll
    for (int b0 = 0; b0 < ND * 2; b0 += FB) {
      Frag<bf16> vf[FB];
#pragma unroll
      for (int i = 0; i < FB; ++i) vf[i].raw = v_lds[buf][(b0 + i) * 64 + lane];
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < FB; ++i)
#pragma unroll
        for (int t = 0; t < QT; ++t) mfma16(acc[(b0 + i) / 2][t], vf[i], pf[(b0 + i) % 2][t]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // the other buffer was last read one iteration ago, before the barrier every wave has passed
    store_block(stg, buf ^ 1);
    __syncthreads();
  };

  load_block(stg, 0);
  store_block(stg, 0);
  __syncthreads();
  int blk = 0;
  for (;;) {
    for (; blk < n_blocks; ++blk) {                    // hot loop
      load_block(stg, blk + 1);                        // flies during this block's arithmetic
      __builtin_amdgcn_sched_barrier(0);
      if (scores(blk)) break;
      finish(blk);
    }
    if (blk >= n_blocks) break;
    // a row's reference must go up: rescale its sums, then finish the block as usual
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      const float ref_new = fmaxf(ref[t], tmax2[t] > ref[t] + kRaise ? tmax2[t] : ref[t]);
      const float alpha = __builtin_amdgcn_exp2f(ref[t] - ref_new);        // 0 on the first block, 1 if unchanged
      l_run[t] *= alpha;
#pragma unroll
      for (int d = 0; d < ND; ++d) acc[d][t] *= alpha;
      ref[t] = ref_new;
    }
    finish(blk);
    ++blk;
  }

#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16, kWave);
    l += __shfl_xor(l, 32, kWave);
    const int row = q0 + t * 16 + r;
    if (row >= m) continue;
    if (n_splits == 1) {
      const float inv = 1.0f / l;
      bf16* dst = out + (size_t)row * dq + head * DH + 4 * g;
#pragma unroll
      for (int d = 0; d < ND; ++d) {
        const u32x2 v = {pack_bf16(acc[d][t][0] * inv, acc[d][t][1] * inv),
                         pack_bf16(acc[d][t][2] * inv, acc[d][t][3] * inv)};
        *reinterpret_cast<u32x2*>(dst + d * 16) = v;
      }
      if (g == 0) lse[(size_t)head * m + row] = ref[t] * 0.693147180559945309f + __logf(l);
    } else {
      const size_t prow = ((size_t)id.split * n_heads + head) * m + row;
      float* dst = o_part + prow * DH + 4 * g;
#pragma unroll
      for (int d = 0; d < ND; ++d) *reinterpret_cast<f32x4*>(dst + d * 16) = acc[d][t];
      if (g == 0) {
        ml_part[prow * 2] = ref[t] * 0.693147180559945309f;      // natural-log reference of this partial
        ml_part[prow * 2 + 1] = l;
      }
    }
  }
}

// out[row, head, :] = sum_s e^{m_s - M} O_s / sum_s e^{m_s - M} l_s over the key splits, in split order.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_merge_kernel(const float* __restrict__ o_part,
                                                              const float* __restrict__ ml_part, int m, int n_heads,
                                                              int n_splits, bf16* __restrict__ out,
                                                              float* __restrict__ lse) {
  constexpr int PER_ROW = DH / 4;                       // threads per (head, row): 4 values each
  const size_t item = (size_t)blockIdx.x * kThreads + threadIdx.x;
  const size_t hr = item / PER_ROW;                     // head * m + row
  const int c = (int)(item - hr * PER_ROW);
  if (hr >= (size_t)n_heads * m) return;
  const int head = (int)(hr / m), row = (int)(hr - (size_t)head * m);
  float mx = -INFINITY;
  for (int s = 0; s < n_splits; ++s) mx = fmaxf(mx, ml_part[((size_t)s * n_heads * m + hr) * 2]);
  float lsum = 0.f;
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < n_splits; ++s) {
    const size_t prow = (size_t)s * n_heads * m + hr;
    const float f = __expf(ml_part[prow * 2] - mx);
    lsum += ml_part[prow * 2 + 1] * f;
    o += *reinterpret_cast<const f32x4*>(o_part + prow * DH + 4 * c) * f;
  }
  const float inv = 1.0f / lsum;
  const u32x2 v = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv)};
  *reinterpret_cast<u32x2*>(out + (size_t)row * n_heads * DH + head * DH + 4 * c) = v;
  if (c == 0) lse[hr] = mx + __logf(lsum);
}

// A-bar tile of 64*QT queries x 16*KA keys: loop over the heads, K block of each head through LDS,
// exp2(s*c - lse*log2e) accumulated in registers.  Every iteration streams its Q and K pieces once
// (no reuse across heads), so the bytes per tile fall with the tile size: the plan takes the largest
// tile and restores the workgroup count by dealing the heads to several workgroups per tile.
template <int DH, int KA, int QT>
__global__ __launch_bounds__(kThreads) void attn_tiled_avg_kernel(const bf16* __restrict__ q,
                                                                  const bf16* __restrict__ k_cache,
                                                                  const float* __restrict__ lse, int m, int L,
                                                                  int n_heads, int n_kv_heads, float scale,
                                                                  int heads_per_group,
                                                                  float* __restrict__ attn_avg) {
  constexpr int NS = DH / 32;
  constexpr int NF = KA * NS;                    // K fragments per head
  constexpr int FW = (NF + 3) / 4;               // of which one wave stages this many
  __shared__ u32x4 k_lds[2][NF * 64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.x * (64 * QT) + wave * (16 * QT);
  const int key0 = blockIdx.y * (16 * KA);
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const int group = n_heads / n_kv_heads;
  int row[QT];
  const bf16* qrow[QT];
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    row[t] = min(q0 + t * 16 + r, m - 1);
    qrow[t] = q + (size_t)row[t] * dq + g * 8;
  }
  // blockIdx.z = head group; with several groups each writes its own [m, L] partial (already divided
  // by the head count) and a separate launch adds the partials in group order
  const int head_lo = blockIdx.z * heads_per_group;
  const int head_hi = min(n_heads, head_lo + heads_per_group);
  attn_avg += (size_t)blockIdx.z * m * L;
  const float c2 = scale * 1.44269504088896341f;

  u32x4 kst[FW];
  Frag<bf16> qf[2][QT][NS];
  float e[2][QT];                                // lse of the head in flight / in use (raw: any arithmetic on a
                                                 // value just loaded would wait for every outstanding load)
  auto load_head = [&](int head, int slot) {
    const int kvh = head / group;
#pragma unroll
    for (int i = 0; i < FW; ++i) {
      const int f = min(wave + 4 * i, NF - 1);    // fragment (key tile f / NS, step f % NS); surplus waves repeat the last
      const int key = min(key0 + (f / NS) * 16 + r, L - 1);
      kst[i] = ld16(k_cache + (size_t)key * kv_pitch + kvh * DH + (f % NS) * 32 + g * 8);
    }
#pragma unroll
    for (int t = 0; t < QT; ++t) {
#pragma unroll
      for (int s = 0; s < NS; ++s) qf[slot][t][s].raw = ld16(qrow[t] + head * DH + s * 32);
      e[slot][t] = lse[(size_t)head * m + row[t]];
    }
  };
  auto store_head = [&](int buf) {
#pragma unroll
    for (int i = 0; i < FW; ++i) k_lds[buf][min(wave + 4 * i, NF - 1) * 64 + lane] = kst[i];
  };

  f32x4 acc[KA][QT];
#pragma unroll
  for (int a = 0; a < KA; ++a)
#pragma unroll
    for (int t = 0; t < QT; ++t) acc[a][t] = f32x4{0.f, 0.f, 0.f, 0.f};
  load_head(head_lo, 0);
  store_head(0);
  __syncthreads();
  for (int h0 = head_lo; h0 < head_hi; h0 += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int head = h0 + u;                    // a head past the end repeats the last one with zero weight
      load_head(min(head + 1, head_hi - 1), u ^ 1);
      const float live = head < head_hi ? 1.f : 0.f;
#pragma unroll
      for (int a = 0; a < KA; ++a) {
        f32x4 st[QT];
#pragma unroll
        for (int t = 0; t < QT; ++t) st[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          Frag<bf16> kf;
          kf.raw = k_lds[u][(a * NS + s) * 64 + lane];
#pragma unroll
          for (int t = 0; t < QT; ++t) mfma16(st[t], kf, qf[u][t][s]);
        }
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          const float ne2 = -1.44269504088896341f * e[u][t];
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[a][t][j] += live * __builtin_amdgcn_exp2f(fmaf(st[t][j], c2, ne2));
        }
      }
      store_head(u ^ 1);
      __syncthreads();
      // nothing of the next head's arithmetic may move up here: anything that touches a value still in
      // flight would make this half wait for all of its own prefetch loads
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  const float inv_h = 1.0f / (float)n_heads;
#pragma unroll
  for (int t = 0; t < QT; ++t) {
    const int qr = q0 + t * 16 + r;
    if (qr >= m) continue;
#pragma unroll
    for (int a = 0; a < KA; ++a) {
      float* dst = attn_avg + (size_t)qr * L + key0 + a * 16 + 4 * g;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (key0 + a * 16 + 4 * g + j < L) dst[j] = acc[a][t][j] * inv_h;
    }
  }
}

constexpr int kTargetWgs = 256;       // one workgroup per compute unit before the key range is split

struct FwdPlan {
  int qt, q_blocks, n_splits, keys_per_split;
};
FwdPlan plan_fwd(const Tunables& t, int m, int L, int n_heads) {
  FwdPlan p;
  const int want_qt = t.attn_qt;
  p.qt = want_qt == 1 ? 1 : want_qt == 2 ? 2 : (m > 64 ? 2 : 1);
  p.q_blocks = (m + 64 * p.qt - 1) / (64 * p.qt);
  const int blocks = (L + kBlockKeys - 1) / kBlockKeys;
  int splits = 1;
  const int max_splits = std::max(1, std::min(8, t.attn_max_splits));
  while (splits < max_splits && p.q_blocks * n_heads * splits < t.attn_target_wgs && blocks / (splits * 2) >= 1) splits *= 2;
  const int blocks_per_split = (blocks + splits - 1) / splits;
  p.keys_per_split = blocks_per_split * kBlockKeys;
  p.n_splits = (L + p.keys_per_split - 1) / p.keys_per_split;     // every split holds at least one key
  return p;
}

template <int DH>
hipError_t launch_fwd(const Tunables& t, const void* q, const void* k_cache, const void* v_cache, int m, int L, int n_heads,
                      int n_kv_heads, void* out, float* lse, float* scratch, size_t scratch_floats, hipStream_t st) {
  const FwdPlan p = plan_fwd(t, m, L, n_heads);
  if (p.n_splits > 1 && (size_t)p.n_splits * n_heads * m * (DH + 2) > scratch_floats) return hipErrorInvalidValue;
  const float scale = 1.0f / sqrtf((float)DH);
  float* o_part = scratch;
  float* ml_part = scratch ? scratch + (size_t)p.n_splits * n_heads * m * DH : nullptr;
  if (p.n_splits > 1 && !scratch) return hipErrorInvalidValue;
  const int groups = (n_heads * p.n_splits + 7) / 8;
  const dim3 grid(groups * 8 * p.q_blocks);
  if (p.qt == 2)
    hipLaunchKernelGGL((attn_tiled_fwd_kernel<DH, 2>), grid, dim3(kThreads), 0, st, (const bf16*)q,
                       (const bf16*)k_cache, (const bf16*)v_cache, m, L, n_heads, n_kv_heads, scale, p.keys_per_split,
                       p.n_splits, p.q_blocks, (bf16*)out, lse, o_part, ml_part);
  else
    hipLaunchKernelGGL((attn_tiled_fwd_kernel<DH, 1>), grid, dim3(kThreads), 0, st, (const bf16*)q,
                       (const bf16*)k_cache, (const bf16*)v_cache, m, L, n_heads, n_kv_heads, scale, p.keys_per_split,
                       p.n_splits, p.q_blocks, (bf16*)out, lse, o_part, ml_part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.n_splits == 1) return e;
  const size_t items = (size_t)n_heads * m * (DH / 4);
  hipLaunchKernelGGL(attn_merge_kernel<DH>, dim3((unsigned)((items + kThreads - 1) / kThreads)), dim3(kThreads), 0, st,
                     o_part, ml_part, m, n_heads, p.n_splits, (bf16*)out, lse);
  return hipGetLastError();
}

struct AvgPlan {
  int ka, qt, key_blocks, q_blocks, groups, heads_per_group;
};
AvgPlan plan_avg(const Tunables& t, int m, int L, int n_heads, bool one_group = false) {
  AvgPlan p;
  // the largest tile the row and key counts fill: 128 x 128, 64 x 128 (m <= 64) or 64 x 32 (L <= 32)
  p.qt = m > 64 ? 2 : 1;
  p.ka = L > 32 ? 8 : 2;
  p.q_blocks = (m + 64 * p.qt - 1) / (64 * p.qt);
  p.key_blocks = (L + 16 * p.ka - 1) / (16 * p.ka);
  // The loop over the heads is a chain of dependent load latencies: when the tile grid alone leaves
  // most of the chip idle, the heads are dealt to several workgroups per tile.
  // one_group: the caller runs the launch beside other work and wants less total work rather than the
  // shortest launch: fewer head groups, fewer partials to add
  int groups = 1;
  const int max_groups = one_group ? std::max(1, std::min(8, t.attn_side_groups)) : 8;
  while (groups < max_groups && groups * 2 <= n_heads && (size_t)p.q_blocks * p.key_blocks * groups < 2 * kTargetWgs) groups *= 2;
  p.heads_per_group = (n_heads + groups - 1) / groups;
  p.groups = (n_heads + p.heads_per_group - 1) / p.heads_per_group;
  return p;
}

template <int DH>
hipError_t launch_avg(const Tunables& t, const void* q, const void* k_cache, const float* lse, int m, int L, int n_heads,
                      int n_kv_heads, float* attn_avg, float* scratch, size_t scratch_floats, hipStream_t st,
                      bool one_group) {
  const float scale = 1.0f / sqrtf((float)DH);
  const AvgPlan p = plan_avg(t, m, L, n_heads, one_group);
  if (p.groups > 1 && (!scratch || (size_t)p.groups * m * L > scratch_floats)) return hipErrorInvalidValue;
  float* dst = p.groups > 1 ? scratch : attn_avg;
  const dim3 grid(p.q_blocks, p.key_blocks, p.groups);
#define D2C_AVG(KA_, QT_)                                                                                      \
  hipLaunchKernelGGL((attn_tiled_avg_kernel<DH, KA_, QT_>), grid, dim3(kThreads), 0, st, (const bf16*)q,       \
                     (const bf16*)k_cache, lse, m, L, n_heads, n_kv_heads, scale, p.heads_per_group, dst)
  if (p.ka == 8 && p.qt == 2) D2C_AVG(8, 2);
  else if (p.ka == 8) D2C_AVG(8, 1);
  else if (p.qt == 2) D2C_AVG(2, 2);
  else D2C_AVG(2, 1);
#undef D2C_AVG
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.groups == 1) return e;
  return launch_sum_splits(attn_avg, scratch, p.groups, (size_t)m * L, (size_t)m * L, st);
}

}  // namespace

// Worst case over every (m <= max_m, L <= max_L): the split count depends on the number of 64-key blocks
// and shorter sequences can be split as often as longer ones, so both are scanned (L at block boundaries).
size_t attention_tiled_scratch_floats(const Tunables& t, int max_m, int max_L, int n_heads, int head_dim) {
  size_t worst = 0;
  for (int L = kBlockKeys;; L += kBlockKeys) {
    const int Lc = std::min(L, max_L);
    for (int m = 1; m <= max_m; ++m) {
      const FwdPlan p = plan_fwd(t, m, Lc, n_heads);
      if (p.n_splits > 1) worst = std::max(worst, (size_t)p.n_splits * n_heads * m * (head_dim + 2));
    }
    if (L >= max_L) break;
  }
  return worst;
}

hipError_t launch_attention_tiled_fwd(const Tunables& t, const void* q, const void* k_cache, const void* v_cache, int m, int L,
                                      int n_heads, int n_kv_heads, int head_dim, void* out, float* lse,
                                      float* scratch, size_t scratch_floats, hipStream_t st) {
  if (head_dim == 128)
    return launch_fwd<128>(t, q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, scratch, scratch_floats, st);
  if (head_dim == 64)
    return launch_fwd<64>(t, q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, scratch, scratch_floats, st);
  return hipErrorInvalidValue;
}

// Worst case over every (m <= max_m, L <= max_L): a short sequence has few key tiles and therefore more
// head groups, so the product groups * m * L does not peak at max_L; L is scanned at tile boundaries.
size_t attention_tiled_avg_scratch_floats(const Tunables& t, int max_m, int max_L, int n_heads) {
  size_t worst = 0;
  for (int L = 32;; L += 32) {
    const int Lc = std::min(L, max_L);
    for (int m = 1; m <= max_m; ++m) {
      const AvgPlan p = plan_avg(t, m, Lc, n_heads);
      if (p.groups > 1) worst = std::max(worst, (size_t)p.groups * m * Lc);
    }
    if (L >= max_L) break;
  }
  return worst;
}

hipError_t launch_attention_tiled_avg(const Tunables& t, const void* q, const void* k_cache, const float* lse, int m, int L,
                                      int n_heads, int n_kv_heads, int head_dim, float* attn_avg, float* scratch,
                                      size_t scratch_floats, hipStream_t st, bool one_group) {
  if (head_dim == 128)
    return launch_avg<128>(t, q, k_cache, lse, m, L, n_heads, n_kv_heads, attn_avg, scratch, scratch_floats, st,
                           one_group);
  if (head_dim == 64)
    return launch_avg<64>(t, q, k_cache, lse, m, L, n_heads, n_kv_heads, attn_avg, scratch, scratch_floats, st,
                          one_group);
  return hipErrorInvalidValue;
}

}  // namespace d2c
