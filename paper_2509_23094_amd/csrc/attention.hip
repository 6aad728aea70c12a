// Selective-refresh attention: the m selected query rows attend to ALL L cached
// keys without a mask, and the kernel also emits A-bar, the mean over the query
// heads of the normalised attention rows (A^(l) in R^{H x |y*| x L} averaged over
// heads, Sec. 4.2 of the d2Cache paper), which the rollout (Eq. 6-8) consumes.
//
// This file: the kernels for FEW query rows in bf16 and the fp32 path; the LDS-tiled kernels for many rows
// are in attention_tiled.hip.  No atomics anywhere (bit-reproducible).
//   forward   one workgroup per (16-query tile, head, part of the output columns), placed so that the
//             readers of one kv head share an L2; its 8 waves take 32-key pairs of tiles
//             round-robin (the next pair's loads in flight while one is consumed), run
//             an online softmax each and merge through LDS.  Scores are
//             computed transposed, S^T = K Q^T, so that the 16x16 accumulator layout
//             (4 consecutive keys per lane for one query), taken for both tiles of a
//             pair, IS the B operand of the 16x16x32 matrix-core step of
//             O^T = V^T P^T: P never leaves registers.
//             V rows are read straight from global memory (8 bytes = 4 head-dim
//             values per lane and key) and 4x4 in-register transposes turn them
//             into the A operand (4+4 keys per lane for one head-dim value).
//             Writes O (bf16), the log-sum-exp per (head, row) and, up to 1024 keys, the
//             normalised probability rows of its head in bf16 (the waves keep their scaled scores
//             in registers until the row's log-sum-exp is known).
//   head mean one launch per step: A-bar of every layer = mean over the heads of those rows.
//   second pass (more than 1024 keys and too few rows for the tiled kernels): one workgroup per
//             (16-query tile, 16-key tile); its 4 waves split the heads, recompute S^T and
//             accumulate exp(s - lse) in registers, then add their partial sums in a fixed
//             order through LDS.
// fp32 path (small test model only): forward and second pass, one workgroup per query row, plain FMA.
#include <algorithm>

#include "common.h"
#include "internal.h"

namespace d2c {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// Operands of one pair of 16-key tiles (32 keys), loaded ahead of their use: per tile the K rows for S^T
// (DH/32 fragments) and, per 64-wide head-dim block, four keys x four head-dim values of V.
template <int DH, int NBL>
struct KvPair {
  Frag<bf16> k[2][DH / 32];
  u32x2 v[2][NBL][4];           // NBL 64-wide head-dim blocks of V (the workgroup's share of the output columns)
};

// Unconditional: rows past the end are clamped to the last key (their scores are masked by the consumer).
template <int DH, int NBL>
__device__ __forceinline__ void load_kv_pair(KvPair<DH, NBL>& t, const bf16* __restrict__ kbase,
                                             const bf16* __restrict__ vbase, size_t pitch, int key0, int L, int r,
                                             int g) {
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const int key = min(key0 + a * 16 + r, L - 1);
    const bf16* krow = kbase + (size_t)key * pitch + g * 8;
#pragma unroll
    for (int s = 0; s < DH / 32; ++s) t.k[a][s].raw = ld16(krow + s * 32);
  }
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int vkey = min(key0 + a * 16 + 4 * g + e, L - 1);
      const bf16* vrow = vbase + (size_t)vkey * pitch + 4 * r;
#pragma unroll
      for (int b = 0; b < NBL; ++b) t.v[a][b][e] = ld8(vrow + b * 64);
    }
}

constexpr int kFwdWaves = 8;
constexpr int kFwdThreads = kFwdWaves * 64;
constexpr int kXcds = 8;          // workgroup i of a launch runs on XCD i % 8 (each XCD has its own L2)

// Which (query tile, head) a workgroup takes.  All workgroups that read the K/V of one kv head are placed
// on one XCD (or, with fewer than 8 kv heads, on 8 / n_kv_heads of them), so the rows of a kv head come
// from HBM once (resp. 8 / n_kv_heads times) and the other readers hit that XCD's L2.
struct FwdMap {
  int mode;          // 0: plain, 1: n_kv_heads % 8 == 0, 2: 8 % n_kv_heads == 0
  int n_qt, group;   // query tiles, query heads per kv head
  int dparts;        // workgroups that share a (query tile, head), each with its own part of the output columns
  int n_wgs;
};
__host__ __device__ inline FwdMap fwd_map(int m, int n_heads, int n_kv_heads, int dparts) {
  FwdMap f;
  f.n_qt = (m + 15) / 16;
  f.group = n_heads / n_kv_heads;
  f.dparts = dparts;
  const int items = f.group * f.n_qt * dparts;        // workgroups per kv head
  if (n_kv_heads % kXcds == 0) {
    f.mode = 1;
    f.n_wgs = n_kv_heads * items;
  } else if (kXcds % n_kv_heads == 0) {
    f.mode = 2;
    const int share = kXcds / n_kv_heads;             // XCDs per kv head
    f.n_wgs = kXcds * ((items + share - 1) / share);
  } else {
    f.mode = 0;
    f.n_wgs = n_kv_heads * items;
  }
  return f;
}
// false: this workgroup has nothing to do (padding of mode 2)
__device__ __forceinline__ bool fwd_map_decode(const FwdMap& f, int n_kv_heads, int wg, int& head, int& qt,
                                               int& dpart) {
  int kvh, item;
  const int items = f.group * f.n_qt * f.dparts;
  if (f.mode == 1) {
    const int xcd = wg % kXcds, j = wg / kXcds;
    kvh = xcd + kXcds * (j / items);
    item = j % items;
  } else if (f.mode == 2) {
    const int share = kXcds / n_kv_heads;
    const int xcd = wg % kXcds, j = wg / kXcds;
    kvh = xcd / share;
    item = xcd % share + share * j;
    if (item >= items) return false;
  } else {
    kvh = wg / items;
    item = wg % items;
  }
  dpart = item % f.dparts;
  item /= f.dparts;
  head = kvh * f.group + item / f.n_qt;
  qt = item % f.n_qt;
  return true;
}

// One workgroup per (16-query tile, head).  Its 8 waves take 32-key pairs of tiles round-robin, run an
// online softmax each and merge through LDS.
// KEEP > 0: the wave also keeps the scaled scores of its first 2*KEEP pairs (all of them when
// L <= 512*KEEP) and, once the workgroup knows the rows' log-sum-exp, writes the normalised probabilities
// of this head to probs [H, m, L]: the head average then needs no second pass over Q and K.
// DPARTS = 1 or DH / 64: with DPARTS > 1 a (query tile, head) is shared by DPARTS workgroups; each computes all
// scores (and the same softmax) but accumulates only its 64 output columns, so it pulls all of K and only its
// part of V through its compute unit: less per workgroup, more workgroups, nothing to merge.  Part 0 writes
// the log-sum-exp; the probability rows (every part holds all scores) are written in equal shares.
template <int DH, int KEEP, int DPARTS>
__global__ __launch_bounds__(kFwdThreads) void attn_fwd_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k_cache, const bf16* __restrict__ v_cache, int m, int L,
    int n_heads, int n_kv_heads, float scale, bf16* __restrict__ out, float* __restrict__ lse,
    bf16* __restrict__ probs) {
  constexpr int NS = DH / 32;     // contraction steps of Q K^T
  constexpr int NB = DH / 64 / DPARTS;     // 64-wide head-dim blocks of the output this workgroup owns
  constexpr int DW = NB * 64;              // its output columns
  __shared__ float o_lds[kFwdWaves][16][DW + 1];
  __shared__ float m_lds[kFwdWaves][16], l_lds[kFwdWaves][16], f_lds[kFwdWaves][16];
  __shared__ float lse_lds[16];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  int head, qt, dpart;
  if (!fwd_map_decode(fwd_map(m, n_heads, n_kv_heads, DPARTS), n_kv_heads, blockIdx.x, head, qt, dpart)) return;
  const int q0 = qt * 16;
  const int kvh = head / (n_heads / n_kv_heads);
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const bf16* kbase = k_cache + (size_t)kvh * DH;
  const bf16* vbase = v_cache + (size_t)kvh * DH + dpart * DW;

  Frag<bf16> qf[NS];
  {
    const int row = min(q0 + r, m - 1);
    const bf16* qrow = q + (size_t)row * dq + head * DH + g * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s].raw = ld16(qrow + s * 32);
  }

  float m_run = -INFINITY, l_run = 0.f;
  f32x4 acc[NB][4];
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[b][i] = f32x4{0.f, 0.f, 0.f, 0.f};

  // S^T of both tiles, one online-softmax update for the 32 keys, then O^T += V^T P^T with K = 32:
  // contraction slot (g, j) of the matrix-core step stands for key 16*(j/4) + 4g + j%4 of the pair, which
  // is how the two accumulators of S^T hold the probabilities, so P never leaves registers.
  auto consume = [&](const KvPair<DH, NB>& t, int key0, f32x4* keep) {
    float x[2][4];
    float tmax = -INFINITY;
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < NS; ++s) mfma16(st, t.k[a][s], qf[s]);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        x[a][j] = (key0 + a * 16 + 4 * g + j < L) ? st[j] * scale : -INFINITY;
        tmax = fmaxf(tmax, x[a][j]);
      }
      if (keep) keep[a] = f32x4{x[a][0], x[a][1], x[a][2], x[a][3]};
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, kWave));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);          // finite: a pair holds at least one key below L
    const float alpha = __expf(m_run - m_new);
    float p[2][4];
    float psum = 0.f;
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        p[a][j] = __expf(x[a][j] - m_new);
        psum += p[a][j];
      }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    Frag<bf16> pf;
    {
      bf16x4 p0 = {(bf16)p[0][0], (bf16)p[0][1], (bf16)p[0][2], (bf16)p[0][3]};
      bf16x4 p1 = {(bf16)p[1][0], (bf16)p[1][1], (bf16)p[1][2], (bf16)p[1][3]};
      const u32x2 a0 = __builtin_bit_cast(u32x2, p0), a1 = __builtin_bit_cast(u32x2, p1);
      pf.raw = u32x4{a0.x, a0.y, a1.x, a1.y};
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) {
      // in-register 4x4 transposes: operand i holds keys 4g..4g+3 of both tiles for head-dim value b*64 + 4r + i
      Frag<bf16> op[4];
      op[0].raw = u32x4{pack_lo(t.v[0][b][0].x, t.v[0][b][1].x), pack_lo(t.v[0][b][2].x, t.v[0][b][3].x),
                        pack_lo(t.v[1][b][0].x, t.v[1][b][1].x), pack_lo(t.v[1][b][2].x, t.v[1][b][3].x)};
      op[1].raw = u32x4{pack_hi(t.v[0][b][0].x, t.v[0][b][1].x), pack_hi(t.v[0][b][2].x, t.v[0][b][3].x),
                        pack_hi(t.v[1][b][0].x, t.v[1][b][1].x), pack_hi(t.v[1][b][2].x, t.v[1][b][3].x)};
      op[2].raw = u32x4{pack_lo(t.v[0][b][0].y, t.v[0][b][1].y), pack_lo(t.v[0][b][2].y, t.v[0][b][3].y),
                        pack_lo(t.v[1][b][0].y, t.v[1][b][1].y), pack_lo(t.v[1][b][2].y, t.v[1][b][3].y)};
      op[3].raw = u32x4{pack_hi(t.v[0][b][0].y, t.v[0][b][1].y), pack_hi(t.v[0][b][2].y, t.v[0][b][3].y),
                        pack_hi(t.v[1][b][0].y, t.v[1][b][1].y), pack_hi(t.v[1][b][2].y, t.v[1][b][3].y)};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[b][i] *= alpha;
        mfma16(acc[b][i], op[i], pf);
      }
    }
  };

  // waves take pairs round-robin; two pairs of a wave are in flight: a slot is refilled with the pair two
  // strides ahead as soon as it has been consumed.  Loads are unconditional (a pair past the end reads the
  // last key again and is never consumed), so no wait separates them.
  const int n_pairs = (L + 31) / 32;
  KvPair<DH, NB> ring[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) load_kv_pair<DH, NB>(ring[u], kbase, vbase, kv_pitch, (wave + u * kFwdWaves) * 32, L, r, g);
  f32x4 kept[KEEP > 0 ? 4 * KEEP : 1];
  if constexpr (KEEP > 0) {
    // all of the wave's pairs in 2*KEEP statically indexed slots (the launcher guarantees L <= 512*KEEP)
#pragma unroll
    for (int it = 0; it < KEEP; ++it)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int t = wave + (it * 2 + u) * kFwdWaves;
        if (t < n_pairs) consume(ring[u], t * 32, &kept[(it * 2 + u) * 2]);
        if (it + 1 < KEEP) load_kv_pair<DH, NB>(ring[u], kbase, vbase, kv_pitch, (t + 2 * kFwdWaves) * 32, L, r, g);
      }
  } else {
    for (int t0 = wave; t0 < n_pairs; t0 += 2 * kFwdWaves) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int t = t0 + u * kFwdWaves;
        if (t < n_pairs) consume(ring[u], t * 32, nullptr);
        load_kv_pair<DH, NB>(ring[u], kbase, vbase, kv_pitch, (t + 2 * kFwdWaves) * 32, L, r, g);
      }
    }
  }

  // merge the waves' partial softmaxes: the weights of the 8 partial results of a row first, then the sums
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (g == 0) {
    m_lds[wave][r] = m_run;              // -inf, l = 0 for a wave that had no pair
    l_lds[wave][r] = l_run;
  }
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) o_lds[wave][r][b * 64 + 16 * g + 4 * j + i] = acc[b][i][j];
  __syncthreads();
  if (tid < kFwdWaves * 16) {
    const int w = tid >> 4, qi = tid & 15;
    float mx = m_lds[0][qi];
#pragma unroll
    for (int u = 1; u < kFwdWaves; ++u) mx = fmaxf(mx, m_lds[u][qi]);
    float lsum = 0.f;
#pragma unroll
    for (int u = 0; u < kFwdWaves; ++u) lsum += l_lds[u][qi] * __expf(m_lds[u][qi] - mx);
    f_lds[w][qi] = __expf(m_lds[w][qi] - mx) / lsum;
    if (w == 0) {
      const float e = mx + __logf(lsum);
      lse_lds[qi] = e;
      if (q0 + qi < m && dpart == 0) lse[(size_t)head * m + q0 + qi] = e;
    }
  }
  __syncthreads();
  for (int o = tid; o < 16 * DW; o += kFwdThreads) {
    const int qi = o / DW, dcol = o - qi * DW;
    float osum = 0.f;
#pragma unroll
    for (int w = 0; w < kFwdWaves; ++w) osum += o_lds[w][qi][dcol] * f_lds[w][qi];
    if (q0 + qi < m) out[(size_t)(q0 + qi) * dq + head * DH + dpart * DW + dcol] = (bf16)osum;
  }
  if constexpr (KEEP > 0) {
    if (q0 + r >= m) return;
    const float e = lse_lds[r];
    bf16* prow = probs + ((size_t)head * m + q0 + r) * L;
#pragma unroll
    for (int o = 0; o < 4 * KEEP; ++o) {
      if (o % DPARTS != dpart) continue;        // the workgroups that share this (tile, head) share the rows' stores
      const int key0 = (wave + (o >> 1) * kFwdWaves) * 32 + (o & 1) * 16 + 4 * g;
      const bf16x4 pv = {(bf16)__expf(kept[o][0] - e), (bf16)__expf(kept[o][1] - e), (bf16)__expf(kept[o][2] - e),
                         (bf16)__expf(kept[o][3] - e)};
      if ((L & 3) == 0) {                       // rows start 8-byte aligned: one store per tile
        if (key0 < L) __builtin_nontemporal_store(__builtin_bit_cast(u32x2, pv), reinterpret_cast<u32x2*>(prow + key0));
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (key0 + j < L) prow[key0 + j] = pv[j];                     // masked scores are -inf: never stored
      }
    }
  }
}

// abar[l][i, j] = mean over the heads of probs[l][h][i, j], heads added in order.  The probability rows are kept
// in bf16, the precision in which the second contraction consumed them (and in which the tiled kernels keep
// theirs).  PIECE = 4: four consecutive elements per thread (element counts that are multiples of 4).
template <int PIECE>
__global__ __launch_bounds__(kThreads) void head_mean_kernel(const bf16* __restrict__ probs, size_t probs_layer_stride,
                                                             float* __restrict__ abar, size_t abar_layer_stride,
                                                             int n_heads, size_t n_elems) {
  const size_t i = ((size_t)blockIdx.x * kThreads + threadIdx.x) * PIECE;
  if (i >= n_elems) return;
  const bf16* p = probs + (size_t)blockIdx.y * probs_layer_stride + i;
  const float inv_h = 1.0f / (float)n_heads;
  if constexpr (PIECE == 4) {
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    auto add = [&](const u32x2 raw) {
      const bf16x4 v = __builtin_bit_cast(bf16x4, raw);
      sum += f32x4{(float)v[0], (float)v[1], (float)v[2], (float)v[3]};
    };
    int h = 0;
    for (; h + 8 <= n_heads; h += 8) {                     // eight heads' loads in flight; read once: past the L2
      u32x2 raw[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        raw[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p + (size_t)(h + u) * n_elems));
#pragma unroll
      for (int u = 0; u < 8; ++u) add(raw[u]);             // heads in order
    }
    for (; h < n_heads; ++h) add(__builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p + (size_t)h * n_elems)));
    *reinterpret_cast<f32x4*>(abar + (size_t)blockIdx.y * abar_layer_stride + i) = sum * inv_h;
  } else {
    float sum = 0.f;
    for (int h = 0; h < n_heads; ++h) sum += (float)p[(size_t)h * n_elems];
    abar[(size_t)blockIdx.y * abar_layer_stride + i] = sum * inv_h;
  }
}

// Pass 2: one workgroup per (16-query tile, 16-key tile); its 4 waves split the heads (wave w takes
// heads w, w+4, ..), each recomputes S^T for its heads and accumulates exp(s - lse); the four partial
// sums are added in a fixed order through LDS.
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_avg_bf16_kernel(const bf16* __restrict__ q,
                                                                 const bf16* __restrict__ k_cache,
                                                                 const float* __restrict__ lse, int m, int L,
                                                                 int n_heads, int n_kv_heads, float scale,
                                                                 float* __restrict__ attn_avg) {
  constexpr int NS = DH / 32;
  __shared__ f32x4 part[kWaves][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.x * 16;
  const int key0 = blockIdx.y * 16;
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const int group = n_heads / n_kv_heads;
  const int row = min(q0 + r, m - 1);
  const int key = min(key0 + r, L - 1);
  const bf16* qrow = q + (size_t)row * dq + g * 8;
  const bf16* krow = k_cache + (size_t)key * kv_pitch + g * 8;

  auto load_head = [&](Frag<bf16> (&qf)[NS], Frag<bf16> (&kf)[NS], float& e, int head) {
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      qf[s].raw = ld16(qrow + head * DH + s * 32);
      kf[s].raw = ld16(krow + (head / group) * DH + s * 32);
    }
    e = lse[(size_t)head * m + row];
  };
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  auto consume = [&](const Frag<bf16> (&qf)[NS], const Frag<bf16> (&kf)[NS], float e) {
    f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NS; ++s) mfma16(st, kf[s], qf[s]);
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] += __expf(st[j] * scale - e);
  };
  Frag<bf16> qa[NS], ka[NS], qb[NS], kb[NS];
  float ea = 0.f, eb = 0.f;
  int h = wave;
  if (h < n_heads) load_head(qa, ka, ea, h);
  while (h < n_heads) {
    const int h1 = h + kWaves;
    if (h1 < n_heads) load_head(qb, kb, eb, h1);
    consume(qa, ka, ea);
    if (h1 >= n_heads) break;
    const int h2 = h1 + kWaves;
    if (h2 < n_heads) load_head(qa, ka, ea, h2);
    consume(qb, kb, eb);
    h = h2;
  }
  part[wave][lane] = acc;
  __syncthreads();
  if (wave != 0 || q0 + r >= m) return;
  f32x4 sum = part[0][lane];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) sum += part[w][lane];
  const float inv_h = 1.0f / (float)n_heads;
  float* dst = attn_avg + (size_t)(q0 + r) * L + key0 + 4 * g;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (key0 + 4 * g + j < L) dst[j] = sum[j] * inv_h;
}

// fp32 path (small test model): one workgroup per query row, heads in sequence, plain FMA.
__global__ __launch_bounds__(kThreads) void attn_fwd_f32_kernel(const float* __restrict__ q,
                                                                const float* __restrict__ k_cache,
                                                                const float* __restrict__ v_cache, int m, int L,
                                                                int n_heads, int n_kv_heads, int head_dim,
                                                                float scale, float* __restrict__ out,
                                                                float* __restrict__ lse) {
  extern __shared__ float smem[];          // scores[L], red[8]
  float* scores = smem;
  float* red = smem + L;
  const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int dq = n_heads * head_dim, dkv = n_kv_heads * head_dim, group = n_heads / n_kv_heads;
  for (int head = 0; head < n_heads; ++head) {
    const float* qv = q + (size_t)row * dq + head * head_dim;
    const int kvh = head / group;
    float mx = -INFINITY;
    for (int j = tid; j < L; j += kThreads) {
      const float* kv = k_cache + (size_t)j * dkv + kvh * head_dim;
      float s = 0.f;
      for (int e = 0; e < head_dim; ++e) s = fmaf(qv[e], kv[e], s);
      s *= scale;
      scores[j] = s;
      mx = fmaxf(mx, s);
    }
    mx = wave_max(mx);
    __syncthreads();
    if (lane == 0) red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    float sum = 0.f;
    for (int j = tid; j < L; j += kThreads) {
      const float e = expf(scores[j] - mx);
      scores[j] = e;
      sum += e;
    }
    sum = wave_sum(sum);
    __syncthreads();
    if (lane == 0) red[4 + wave] = sum;
    __syncthreads();
    const float total = red[4] + red[5] + red[6] + red[7];
    const float inv = 1.0f / total;
    if (tid == 0) lse[(size_t)head * m + row] = mx + logf(total);
    for (int e = tid; e < head_dim; e += kThreads) {
      float o = 0.f;
      for (int j = 0; j < L; ++j) o = fmaf(scores[j], v_cache[(size_t)j * dkv + kvh * head_dim + e], o);
      out[(size_t)row * dq + head * head_dim + e] = o * inv;
    }
    __syncthreads();
  }
}

// A-bar row of one query: mean over heads of exp(s - lse).
__global__ __launch_bounds__(kThreads) void attn_avg_f32_kernel(const float* __restrict__ q,
                                                                const float* __restrict__ k_cache,
                                                                const float* __restrict__ lse, int m, int L,
                                                                int n_heads, int n_kv_heads, int head_dim,
                                                                float scale, float* __restrict__ attn_avg) {
  const int row = blockIdx.x;
  const int dq = n_heads * head_dim, dkv = n_kv_heads * head_dim, group = n_heads / n_kv_heads;
  const float inv_h = 1.0f / (float)n_heads;
  for (int j = threadIdx.x; j < L; j += kThreads) {
    float acc = 0.f;
    for (int head = 0; head < n_heads; ++head) {
      const float* qv = q + (size_t)row * dq + head * head_dim;
      const float* kv = k_cache + (size_t)j * dkv + (head / group) * head_dim;
      float s = 0.f;
      for (int e = 0; e < head_dim; ++e) s = fmaf(qv[e], kv[e], s);
      acc += expf(s * scale - lse[(size_t)head * m + row]);
    }
    attn_avg[(size_t)row * L + j] = acc * inv_h;
  }
}

template <int DH>
hipError_t launch_fwd_bf16(const void* q, const void* k_cache, const void* v_cache, int m, int L, int n_heads,
                           int n_kv_heads, void* out, float* lse, bf16* probs, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)DH);
  // split the output columns over two workgroups when that still fits one round of workgroups on the chip
  constexpr int kUnits = 256;
  const bool split = DH == 128 && fwd_map(m, n_heads, n_kv_heads, 2).n_wgs <= kUnits;
#define D2C_FWD(KEEP_, DP_)                                                                                     \
  hipLaunchKernelGGL((attn_fwd_bf16_kernel<DH, KEEP_, DP_>), dim3(fwd_map(m, n_heads, n_kv_heads, DP_).n_wgs),  \
                     dim3(kFwdThreads), 0, st, (const bf16*)q, (const bf16*)k_cache, (const bf16*)v_cache, m, L, \
                     n_heads, n_kv_heads, scale, (bf16*)out, lse, probs)
  if constexpr (DH == 128) {
    if (split) {
      if (!probs) D2C_FWD(0, 2);
      else if (L <= 512) D2C_FWD(1, 2);
      else if (L <= 1024) D2C_FWD(2, 2);
      else return hipErrorInvalidValue;
      return hipGetLastError();
    }
  }
  if (!probs) D2C_FWD(0, 1);
  else if (L <= 512) D2C_FWD(1, 1);
  else if (L <= 1024) D2C_FWD(2, 1);
  else return hipErrorInvalidValue;
#undef D2C_FWD
  return hipGetLastError();
}

template <int DH>
hipError_t launch_avg_bf16(const void* q, const void* k_cache, const float* lse, int m, int L, int n_heads,
                           int n_kv_heads, float* attn_avg, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)DH);
  const int key_blocks = (L + 15) / 16;
  hipLaunchKernelGGL(attn_avg_bf16_kernel<DH>, dim3((m + 15) / 16, key_blocks), dim3(kThreads), 0, st, (const bf16*)q,
                     (const bf16*)k_cache, lse, m, L, n_heads, n_kv_heads, scale, attn_avg);
  return hipGetLastError();
}

}  // namespace

constexpr int kProbsMaxM = 128, kProbsMaxL = 1024;

bool attention_fwd_emits_probs(const Tunables& t, int dtype, int m, int L) {
  return dtype == kBF16 && m > 0 && !attention_is_tiled(t, dtype, m, L) && m <= kProbsMaxM && L <= kProbsMaxL;
}

size_t attention_probs_elems(int dtype, int n_heads, int max_L) {
  return dtype == kBF16 ? (size_t)n_heads * kProbsMaxM * std::min(max_L, kProbsMaxL) : 0;
}

hipError_t launch_head_mean(const void* probs, size_t probs_layer_stride, float* abar, size_t abar_layer_stride,
                            int n_layers, int n_heads, int m, int L, hipStream_t st) {
  if (n_layers <= 0 || m <= 0) return hipSuccess;
  const size_t n = (size_t)m * L;
  // four elements per thread need 8-byte aligned pieces of the rows and 16-byte aligned pieces of A-bar
  if (n % 4 == 0 && probs_layer_stride % 4 == 0 && abar_layer_stride % 4 == 0 && (uintptr_t)probs % 8 == 0 &&
      (uintptr_t)abar % 16 == 0) {
    hipLaunchKernelGGL(head_mean_kernel<4>, dim3((unsigned)((n / 4 + kThreads - 1) / kThreads), n_layers), dim3(kThreads),
                       0, st, (const bf16*)probs, probs_layer_stride, abar, abar_layer_stride, n_heads, n);
  } else {
    hipLaunchKernelGGL(head_mean_kernel<1>, dim3((unsigned)((n + kThreads - 1) / kThreads), n_layers), dim3(kThreads), 0,
                       st, (const bf16*)probs, probs_layer_stride, abar, abar_layer_stride, n_heads, n);
  }
  return hipGetLastError();
}

// per sequence of a batch; a caller that batches n sequences provides n times as much
size_t attention_scratch_floats(const Tunables& t, int dtype, int max_m, int max_L, int n_heads, int head_dim) {
  return dtype == kBF16 ? attention_tiled_scratch_floats(t, max_m, max_L, n_heads, head_dim) : 0;
}

// From kLongMinM rows on the tiled kernels also take the key ranges too long for the per-head probability
// rows: there the few-row kernels would need their second Q K^T launch for the head average.
constexpr int kLongMinM = 48;
bool attention_is_tiled(const Tunables& t, int dtype, int m, int L) {
  return dtype == kBF16 && (m >= t.attn_tiled_min_m || (m >= std::min(kLongMinM, t.attn_tiled_min_m) && L > kProbsMaxL));
}

hipError_t launch_attention_fwd(const Tunables& t, int dtype, const void* q, const void* k_cache, const void* v_cache, int m, int L,
                                int n_heads, int n_kv_heads, int head_dim, void* out, float* lse, float* scratch,
                                size_t scratch_floats, hipStream_t st, void* probs, float* tiled_avg) {
  if (m <= 0) return hipSuccess;
  if (L <= 0 || n_heads % n_kv_heads) return hipErrorInvalidValue;
  if (probs && !attention_fwd_emits_probs(t, dtype, m, L)) return hipErrorInvalidValue;
  if (attention_is_tiled(t, dtype, m, L)) {
    const TiledCall call{q, k_cache, v_cache, m, L, out, lse, tiled_avg};
    return launch_attention_tiled(t, &call, 1, n_heads, n_kv_heads, head_dim, scratch, scratch_floats, st);
  }
  if (tiled_avg) return hipErrorInvalidValue;
  if (dtype == kBF16) {
    if (head_dim == 128)
      return launch_fwd_bf16<128>(q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, (bf16*)probs, st);
    if (head_dim == 64)
      return launch_fwd_bf16<64>(q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, (bf16*)probs, st);
    return hipErrorInvalidValue;
  }
  const size_t smem = ((size_t)L + 8) * sizeof(float);
  if (smem > 64 * 1024) return hipErrorInvalidValue;   // default dynamic LDS limit
  const float scale = 1.0f / sqrtf((float)head_dim);
  hipLaunchKernelGGL(attn_fwd_f32_kernel, dim3(m), dim3(kThreads), smem, st, (const float*)q, (const float*)k_cache,
                     (const float*)v_cache, m, L, n_heads, n_kv_heads, head_dim, scale, (float*)out, lse);
  return hipGetLastError();
}

hipError_t launch_attention_avg(const Tunables& t, int dtype, const void* q, const void* k_cache, const float* lse, int m, int L,
                                int n_heads, int n_kv_heads, int head_dim, float* attn_avg, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  if (L <= 0 || n_heads % n_kv_heads || attention_is_tiled(t, dtype, m, L)) return hipErrorInvalidValue;
  if (dtype == kBF16) {
    if (head_dim == 128) return launch_avg_bf16<128>(q, k_cache, lse, m, L, n_heads, n_kv_heads, attn_avg, st);
    if (head_dim == 64) return launch_avg_bf16<64>(q, k_cache, lse, m, L, n_heads, n_kv_heads, attn_avg, st);
    return hipErrorInvalidValue;
  }
  const float scale = 1.0f / sqrtf((float)head_dim);
  hipLaunchKernelGGL(attn_avg_f32_kernel, dim3(m), dim3(kThreads), 0, st, (const float*)q, (const float*)k_cache, lse,
                     m, L, n_heads, n_kv_heads, head_dim, scale, attn_avg);
  return hipGetLastError();
}

}  // namespace d2c
