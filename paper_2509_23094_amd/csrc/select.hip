// Selection side of the d2Cache step: Eq. 1 (prediction and confidence over the
// vocabulary), Eq. 3-4 (certainty density, stage-1 top-k), unmasking (Eq. 2),
// the rollout update on the compact |S| x L block (Eq. 6-8), influence scores
// (Eq. 9) and the stage-2 cumulative-mass selection (Sec. 4.2, last paragraph).
//
// Everything that decides an index is integer-exact and order-independent:
// top-k ranks 64-bit keys (float bits of the non-negative score, then lower
// index first); top-p sorts such keys with a bitonic network in LDS and scans
// fixed-point masses floor(c * 2^32) in uint64.  Ties always go to the lowest index.
#include <algorithm>
#include <cstring>

#include "common.h"
#include "internal.h"

namespace d2c {
namespace {

// ------------------------------------------------------------------ Eq. 1
// x-hat = argmax_v, s = 1 / sum_v exp(x_v - max).  A vocabulary row (0.5 MB at V = 126464) is cut into
// chunks, one workgroup each, so that a few dozen rows still fill the chip: per chunk (max, first index of
// the max, sum of exp(x - chunk max)); a second tiny launch merges the chunks of a row in ascending order
// (ties keep the lowest index) -- fixed order, bit-reproducible.
constexpr int kConfThreads = 256;
constexpr int kConfMaxChunks = 64;

__global__ __launch_bounds__(kConfThreads) void confidence_chunk_kernel(const float* __restrict__ logits, int vocab,
                                                                        int chunk, int n_chunks,
                                                                        float* __restrict__ part) {
  __shared__ float s_val[kConfThreads / 64];
  __shared__ int s_idx[kConfThreads / 64];
  __shared__ float s_sum[kConfThreads / 64];
  const int row = blockIdx.y, ck = blockIdx.x;
  const float* x = logits + (size_t)row * vocab;
  const int lo = ck * chunk, hi = min(vocab, lo + chunk);
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  float best = -INFINITY;
  int bidx = 0x7fffffff;
  for (int v = lo + tid; v < hi; v += kConfThreads) {       // ascending per thread: a tie keeps the lower index
    const float xv = x[v];
    if (xv > best) { best = xv; bidx = v; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bidx, o, kWave);
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  if (lane == 0) { s_val[wave] = best; s_idx[wave] = bidx; }
  __syncthreads();
  best = s_val[0]; bidx = s_idx[0];
  for (int w = 1; w < kConfThreads / 64; ++w) {
    const float ob = s_val[w];
    const int oi = s_idx[w];
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  float sum = 0.f;
  for (int v = lo + tid; v < hi; v += kConfThreads) sum += expf(x[v] - best);
  sum = wave_sum(sum);
  if (lane == 0) s_sum[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < kConfThreads / 64; ++w) t += s_sum[w];
    float* o = part + ((size_t)row * n_chunks + ck) * 3;
    o[0] = best;
    o[1] = __int_as_float(bidx);
    o[2] = t;
  }
}

// The same for chunks of exactly 8192 entries of 16-byte aligned rows (vocab % 4 == 0): a thread keeps its 32
// entries in registers (eight 16-byte loads issued together), so the row is read once and the kernel is one
// memory latency long.  Entry order per thread is ascending (piece, then element), as the tie rule needs.
__global__ __launch_bounds__(kConfThreads) void confidence_chunk_vec_kernel(const float* __restrict__ logits,
                                                                            int vocab, int n_chunks,
                                                                            float* __restrict__ part) {
  constexpr int kChunk = 8192, kPieces = kChunk / (4 * kConfThreads);
  __shared__ float s_val[kConfThreads / 64];
  __shared__ int s_idx[kConfThreads / 64];
  __shared__ float s_sum[kConfThreads / 64];
  const int row = blockIdx.y, ck = blockIdx.x;
  const float* x = logits + (size_t)row * vocab;
  const int lo = ck * kChunk;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  f32x4 val[kPieces];
#pragma unroll
  for (int p = 0; p < kPieces; ++p) {
    const int v = lo + (p * kConfThreads + tid) * 4;
    val[p] = *reinterpret_cast<const f32x4*>(x + min(v, vocab - 4));       // past the end: re-read, masked below
  }
  float best = -INFINITY;
  int bidx = 0x7fffffff;
#pragma unroll
  for (int p = 0; p < kPieces; ++p) {
    const int v = lo + (p * kConfThreads + tid) * 4;
    if (v >= vocab) val[p] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (val[p][e] > best) { best = val[p][e]; bidx = v + e; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ob = __shfl_xor(best, o, kWave);
    const int oi = __shfl_xor(bidx, o, kWave);
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  if (lane == 0) { s_val[wave] = best; s_idx[wave] = bidx; }
  __syncthreads();
  best = s_val[0]; bidx = s_idx[0];
  for (int w = 1; w < kConfThreads / 64; ++w) {
    const float ob = s_val[w];
    const int oi = s_idx[w];
    if (ob > best || (ob == best && oi < bidx)) { best = ob; bidx = oi; }
  }
  float sum = 0.f;
#pragma unroll
  for (int p = 0; p < kPieces; ++p)
#pragma unroll
    for (int e = 0; e < 4; ++e) sum += expf(val[p][e] - best);              // exp(-inf) = 0 past the end
  sum = wave_sum(sum);
  if (lane == 0) s_sum[wave] = sum;
  __syncthreads();
  if (tid == 0) {
    float t = 0.f;
    for (int w = 0; w < kConfThreads / 64; ++w) t += s_sum[w];
    float* o = part + ((size_t)row * n_chunks + ck) * 3;
    o[0] = best;
    o[1] = __int_as_float(bidx);
    o[2] = t;
  }
}

__global__ void confidence_merge_kernel(const float* __restrict__ part, int n_rows, int n_chunks,
                                        const int32_t* __restrict__ pos, const int32_t* __restrict__ via,
                                        float* __restrict__ conf, int32_t* __restrict__ pred) {
  const int row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n_rows) return;
  const float* p = part + (size_t)row * n_chunks * 3;
  float best = p[0];
  int bidx = __float_as_int(p[1]);
  for (int c = 1; c < n_chunks; ++c)
    if (p[3 * c] > best) { best = p[3 * c]; bidx = __float_as_int(p[3 * c + 1]); }   // ascending chunks: lowest index wins
  float sum = 0.f;
  for (int c = 0; c < n_chunks; ++c) sum += p[3 * c + 2] * expf(p[3 * c] - best);
  const int where = via ? via[pos[row]] : pos[row];            // row -> position, directly or through S
  conf[where] = 1.0f / sum;
  pred[where] = bidx;
}

// ------------------------------------------------------------------ Eq. 6-8 on the compact block
// c_out[i, c] = ( sum_r A[i, S_r] c_in[r, c] + A[i, c] [c not in S] + c_in[i, c] ) / 2
// Rows outside S stay one-hot under Eq. 6-7, so only these m rows ever change.
constexpr int kRollThreads = 256;

// First layer: C^(0) = I, so sum_r A[i,S_r][c == S_r] + A[i,c][c not in S] = A[i,c] and c_in[i,c] = [c == S_i].
__global__ __launch_bounds__(kRollThreads) void rollout_first_kernel(const float* __restrict__ A,
                                                                     float* __restrict__ c_out,
                                                                     const int32_t* __restrict__ idx, int m, int L) {
  const int col = blockIdx.x * kRollThreads + threadIdx.x;
  const int i = blockIdx.y;
  if (col >= L) return;
  c_out[(size_t)i * L + col] = 0.5f * (A[(size_t)i * L + col] + (idx[i] == col ? 1.f : 0.f));
}

// Later layers: the m x m by m x L product runs on the fp32 matrix cores, one wave per 16 x 16
// output tile (4 waves = 16 rows x 64 columns per workgroup).  Per 16-long step of the
// contraction a lane holds A[i0 + l%16][S[k0 + 4(l/16) + e]] and C[k0 + 4(l/16) + e][c0 + l%16],
// e = 0..3, one 16x16x4 instruction per e.
__global__ __launch_bounds__(kRollThreads) void rollout_kernel(const float* __restrict__ A,
                                                               const float* __restrict__ c_in,
                                                               float* __restrict__ c_out,
                                                               const int32_t* __restrict__ idx, int m, int L) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int r = lane & 15, g = lane >> 4;
  const int i0 = blockIdx.y * 16;
  const int c0 = (blockIdx.x * 4 + wave) * 16;
  if (c0 >= L) return;
  const int arow = min(i0 + r, m - 1);
  const int bcol = min(c0 + r, L - 1);
  const float* a_row = A + (size_t)arow * L;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k0 = 0; k0 < m; k0 += 16) {
    float av[4], bv[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int k = k0 + 4 * g + e;
      const bool ok = k < m;
      const int kk = ok ? k : m - 1;
      const float x = a_row[idx[kk]];
      av[e] = ok ? x : 0.f;
      bv[e] = c_in[(size_t)kk * L + bcol];
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(av[e], bv[e], acc, 0, 0, 0);
  }
  const int col = c0 + r;
  if (col >= L) return;
  const bool in_s = find_sorted(idx, m, col) >= 0;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = i0 + 4 * g + j;
    if (i >= m) break;
    const float direct = in_s ? 0.f : A[(size_t)i * L + col];
    c_out[(size_t)i * L + col] = 0.5f * (acc[j] + direct + c_in[(size_t)i * L + col]);
  }
}

// Eq. 9 on the compact block: c_j = [j not in S] + sum_i C_S[i, j]
__global__ void influence_kernel(const float* __restrict__ c_block, const int32_t* __restrict__ idx, int m, int L,
                                 float* __restrict__ influence) {
  const int col = blockIdx.x * blockDim.x + threadIdx.x;
  if (col >= L) return;
  float s = find_sorted(idx, m, col) < 0 ? 1.f : 0.f;
  for (int i = 0; i < m; ++i) s += c_block[(size_t)i * L + col];
  influence[col] = s;
}

// ------------------------------------------------------------------ Eq. 9 without the rollout matrix
// c = 1^T C^(N) = 1^T W^(N) W^(N-1) ... W^(1) (Eq. 8-9): multiplying from the LEFT keeps a length-L row
// vector v instead of the |S| x L block, O(m L) work per layer instead of O(m^2 L), at the price of needing
// the layers in reverse order, i.e. every layer's A-bar kept until the last one is done.  With rows outside
// S of W equal to unit vectors and rows i in S equal to (A-bar_i + e_i)/2 (Eq. 6-7):
//   (v W)_j = ( sum_{i in S} v_i A-bar_ij + ([j not in S] + 1) v_j ) / 2.
// Only the m entries u = v[S] feed back into later products; a column j outside S just accumulates:
//   u^(N) = ones;  u^(l-1)_k = ( sum_i u^(l)_i A-bar^(l)[i, S_k] + u^(l)_k ) / 2      (sequential, m x m per layer)
//   c_j = 1 + sum_l sum_i u^(l)_i A-bar^(l)[i, j] / 2   for j outside S,   c_{S_k} = u^(0)_k  (parallel)
// so the sequential part touches m^2 numbers per layer and the m L part is one fully parallel launch.
constexpr int kChainThreads = 1024;
constexpr int kChainMaxLen = 4096;           // = the selection kernel's length limit
constexpr int kChainFewRows = 128;           // up to this many rows a wave's share of a layer's block fits its registers
constexpr int kChainFewVals = 16;            // = kChainFewRows / (1024 / 128) rows per wave at most
constexpr int kChainSpreadMinRows = 129;     // from this many rows on the sequential part runs as a launch per layer

// The sequences one chain covers (independent: own A-bar slots, index set and influence vector); their dense
// blocks and per-layer vectors sit one after the other in the scratch buffers.
constexpr int kChainMaxSeqs = 8;
struct ChainSeq {
  const float* abar;
  const int32_t* idx;
  float* influence;
  int m, L;
  size_t g_off, u_off;          // in floats: n_layers * (sum of m^2, resp. of m, over the sequences before)
};
struct ChainSeqs {
  ChainSeq seq[kChainMaxSeqs];
};

// G[l][i, k] = abar[l][i, S_k]: the m x m blocks the sequential part reads, made dense first (all layers in
// one launch) so that the one workgroup that walks the layers reads consecutive floats.
__global__ __launch_bounds__(256) void chain_gather_kernel(const ChainSeqs seqs, size_t layer_stride,
                                                           float* __restrict__ g_scratch) {
  const ChainSeq& q = seqs.seq[blockIdx.z];
  const int m = q.m, L = q.L;
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t mm = (size_t)m * m;
  if (e >= mm) return;
  const int i = (int)(e / m), k = (int)(e - (size_t)i * m);
  g_scratch[q.g_off + (size_t)blockIdx.y * mm + e] = q.abar[(size_t)blockIdx.y * layer_stride + (size_t)i * L + q.idx[k]];
}

// Sequential part, one workgroup per sequence: u through the layers in reverse order; writes U[l][i] = u^(l)_i (the
// vector entering layer l) for the parallel part and c at the positions of S.  Items of 64 entries of S x
// one of RG row groups keep all 16 waves busy for short S; fixed summation order.
__global__ __launch_bounds__(kChainThreads) void chain_rows_kernel(const ChainSeqs seqs, int n_layers,
                                                                   const float* __restrict__ g_scratch,
                                                                   float* __restrict__ u_scratch) {
  const ChainSeq& q = seqs.seq[blockIdx.x];
  const float* __restrict__ G = g_scratch + q.g_off;
  float* __restrict__ U = u_scratch + q.u_off;
  const int32_t* __restrict__ idx = q.idx;
  float* __restrict__ influence = q.influence;
  const int m = q.m;
  __shared__ float u[2][kChainMaxLen];
  __shared__ float part[kChainMaxLen];                 // [RG][padded m], RG * padded m <= max(padded m, 1024)
  __shared__ int32_t s_idx[kChainMaxLen];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  for (int i = tid; i < m; i += kChainThreads) {
    u[0][i] = 1.f;
    s_idx[i] = idx[i];
  }
  __syncthreads();
  const int n_cb = (m + 63) / 64, mp = n_cb * 64;
  const int RG = mp < kChainThreads ? kChainThreads / mp : 1;
  const int n_items = n_cb * RG;
  int cur = 0;
  if (m <= kChainFewRows) {
    // Few rows (the decode steps): every wave has at most one item of at most kChainFewVals rows, so its
    // values of the NEXT layer's block are requested before this layer's sums are exchanged: the chain then
    // runs at one LDS round trip per layer instead of a memory latency.  Same sums in the same order as below.
    const bool has_item = wave < n_items;
    const int cb = wave % n_cb, rg = wave / n_cb;
    const int k = cb * 64 + lane;
    const float* acol = G + min(k, m - 1);
    auto load_layer = [&](float (&x)[kChainFewVals], int l) {
      const float* a = acol + (size_t)l * m * m;
#pragma unroll
      for (int t = 0; t < kChainFewVals; ++t) x[t] = a[(size_t)min(rg + t * RG, m - 1) * m];
    };
    float xs[kChainFewVals], xn[kChainFewVals];
    load_layer(xs, n_layers - 1);
    for (int l = n_layers - 1; l >= 0; --l) {
      const float* uin = u[cur];
      float* uout = u[cur ^ 1];
      load_layer(xn, max(l - 1, 0));                       // unconditional: the last one re-reads layer 0
      for (int i = tid; i < m; i += kChainThreads) U[(size_t)l * m + i] = uin[i];
      if (has_item) {
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < kChainFewVals; ++t) {
          const int i = rg + t * RG;
          if (i < m) acc = fmaf(uin[i], xs[t], acc);
        }
        part[rg * mp + k] = acc;
      }
      __syncthreads();
      for (int kk = tid; kk < m; kk += kChainThreads) {
        float sum = 0.f;
        for (int g2 = 0; g2 < RG; ++g2) sum += part[g2 * mp + kk];
        uout[kk] = 0.5f * (sum + uin[kk]);
      }
      __syncthreads();
#pragma unroll
      for (int t = 0; t < kChainFewVals; ++t) xs[t] = xn[t];
      cur ^= 1;
    }
    for (int kk = tid; kk < m; kk += kChainThreads) influence[s_idx[kk]] = u[cur][kk];
    return;
  }
  for (int l = n_layers - 1; l >= 0; --l) {
    const float* a = G + (size_t)l * m * m;
    const float* uin = u[cur];
    float* uout = u[cur ^ 1];
    for (int i = tid; i < m; i += kChainThreads) U[(size_t)l * m + i] = uin[i];
    for (int item = wave; item < n_items; item += kChainThreads / 64) {
      const int cb = item % n_cb, rg = item / n_cb;
      const int k = cb * 64 + lane;
      const float* acol = a + min(k, m - 1);
      float acc = 0.f;
      int i = rg;
      for (; i + 7 * RG < m; i += 8 * RG) {
        float x[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) x[t] = acol[(size_t)(i + t * RG) * m];
#pragma unroll
        for (int t = 0; t < 8; ++t) acc = fmaf(uin[i + t * RG], x[t], acc);
      }
      for (; i < m; i += RG) acc = fmaf(uin[i], acol[(size_t)i * m], acc);
      part[rg * mp + k] = acc;
    }
    __syncthreads();
    for (int k = tid; k < m; k += kChainThreads) {
      float sum = 0.f;
      for (int rg = 0; rg < RG; ++rg) sum += part[rg * mp + k];
      uout[k] = 0.5f * (sum + uin[k]);
    }
    __syncthreads();
    cur ^= 1;
  }
  for (int k = tid; k < m; k += kChainThreads) influence[s_idx[k]] = u[cur][k];
}

// The sequential part for long index sets (step 0, select-all): one launch per layer, 64 entries of S per
// workgroup, so that a layer's m x m product is spread over m / 64 compute units instead of one.  The vector
// entering layer l is U[l] (ones for the last layer, written here); the result goes to U[l - 1], or, after
// layer 0, to c at the positions of S.  A lane owns one entry k, the 16 waves split the rows i (wave w: rows
// w, w + 16, ..), the waves' sums are added in wave order: fixed summation order.
__global__ __launch_bounds__(kChainThreads) void chain_layer_kernel(const ChainSeqs seqs, int n_layers, int l,
                                                                    const float* __restrict__ g_scratch,
                                                                    float* __restrict__ u_scratch) {
  const ChainSeq& q = seqs.seq[blockIdx.y];
  const int m = q.m;
  if ((int)blockIdx.x * 64 >= m) return;                  // the grid follows the longest index set
  __shared__ float red[kChainThreads / 64][64];
  const float* __restrict__ G = g_scratch + q.g_off + (size_t)l * m * m;
  float* __restrict__ U = u_scratch + q.u_off;
  const float* __restrict__ uin = U + (size_t)l * m;
  const bool first = l == n_layers - 1;                   // u = ones
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int k = blockIdx.x * 64 + lane;
  const float* acol = G + min(k, m - 1);
  constexpr int NW = kChainThreads / 64;
  float acc = 0.f;
  int i = wave;
  for (; i + 7 * NW < m; i += 8 * NW) {
    float x[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] = acol[(size_t)(i + t * NW) * m];
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = fmaf(first ? 1.f : uin[i + t * NW], x[t], acc);
  }
  for (; i < m; i += NW) acc = fmaf(first ? 1.f : uin[i], acol[(size_t)i * m], acc);
  red[wave][lane] = acc;
  __syncthreads();
  if (wave != 0 || k >= m) return;
  float sum = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) sum += red[w][lane];
  const float uk = first ? 1.f : uin[k];
  const float out = 0.5f * (sum + uk);
  if (first) U[(size_t)l * m + k] = 1.f;
  if (l > 0) U[(size_t)(l - 1) * m + k] = out;
  else q.influence[q.idx[k]] = out;
}

// Parallel part: 64 columns per workgroup, its 16 waves take the layers round-robin (wave w: layers w,
// w + 16, ..), a lane owns one column and adds u^(l)_i A-bar^(l)[i, j] over the rows in order with eight
// loads in flight; the waves' sums are added in wave order.  Columns inside S are left alone.
__global__ __launch_bounds__(kChainThreads) void chain_cols_kernel(const ChainSeqs seqs, size_t layer_stride,
                                                                   int n_layers,
                                                                   const float* __restrict__ u_scratch) {
  const ChainSeq& q = seqs.seq[blockIdx.y];
  const float* __restrict__ abar = q.abar;
  const int32_t* __restrict__ idx = q.idx;
  const float* __restrict__ U = u_scratch + q.u_off;
  float* __restrict__ influence = q.influence;
  const int m = q.m, L = q.L;
  if ((int)blockIdx.x * 64 >= L) return;                  // the grid follows the longest sequence
  __shared__ float red[kChainThreads / 64][64];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int col = blockIdx.x * 64 + lane;
  const float* acol = abar + min(col, L - 1);
  float acc = 0.f;
  for (int l = wave; l < n_layers; l += kChainThreads / 64) {
    const float* a = acol + (size_t)l * layer_stride;
    const float* ul = U + (size_t)l * m;
    int i = 0;
    for (; i + 16 <= m; i += 16) {                          // sixteen rows' loads in flight
      float x[16];
#pragma unroll
      for (int t = 0; t < 16; ++t) x[t] = a[(size_t)(i + t) * L];
#pragma unroll
      for (int t = 0; t < 16; ++t) acc = fmaf(ul[i + t], x[t], acc);
    }
    for (; i < m; ++i) acc = fmaf(ul[i], a[(size_t)i * L], acc);
  }
  red[wave][lane] = acc;
  __syncthreads();
  if (wave != 0 || col >= L || find_sorted(idx, m, col) >= 0) return;
  float sum = 0.f;
#pragma unroll
  for (int w = 0; w < kChainThreads / 64; ++w) sum += red[w][lane];
  influence[col] = 1.f + 0.5f * sum;
}

__global__ void ones_kernel(float* __restrict__ x, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) x[i] = 1.f;
}

// ------------------------------------------------------------------ two-stage selection, one workgroup
constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kSelMaxL = 4096;

struct SelShared {
  int wcnt[kSelWaves];
  int scalar[8];
  unsigned long long total;
};

// Ordered compaction of {i in [0,n) : pred(i)} into out (ascending); returns the count (uniform).
template <typename Pred, typename Emit>
__device__ int block_compact(int n, Pred pred, Emit emit, SelShared* sh) {
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  int base = 0;
  for (int start = 0; start < n; start += kSelThreads) {
    const int i = start + tid;
    const bool f = i < n && pred(i);
    const unsigned long long ballot = __ballot(f);
    const int before = __popcll(ballot & ((1ull << lane) - 1ull));
    __syncthreads();
    if (lane == 0) sh->wcnt[wave] = __popcll(ballot);
    __syncthreads();
    int off = 0, total = 0;
    for (int w = 0; w < kSelWaves; ++w) {
      const int c = sh->wcnt[w];
      if (w < wave) off += c;
      total += c;
    }
    if (f) emit(base + off + before, i);
    base += total;
  }
  __syncthreads();
  return base;
}

__device__ __forceinline__ unsigned long long make_key(float score, int index) {
  return ((unsigned long long)__float_as_uint(score) << 32) | (unsigned long long)(0xFFFFFFFFu - (unsigned)index);
}
__device__ __forceinline__ int key_index(unsigned long long key) { return (int)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull)); }
__device__ __forceinline__ unsigned long long key_mass(unsigned long long key) {
  // floor(c * 2^32): the scaling is exact in float, the conversion truncates a non-negative value
  return (unsigned long long)(__uint_as_float((unsigned)(key >> 32)) * 4294967296.0f);
}

constexpr int kSelMaxBatch = 8;
struct SelectBatch {
  SelectArgs seq[kSelMaxBatch];
};

// One workgroup per sequence (blockIdx.x); the sequences are independent.
__global__ __launch_bounds__(kSelThreads) void select_kernel(const SelectBatch batch) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const SelectArgs& a = batch.seq[blockIdx.x];
  const int L = a.L;
  int NP = 2;
  while (NP < L) NP <<= 1;
  unsigned long long* keys = reinterpret_cast<unsigned long long*>(smem);            // [NP]
  unsigned long long* keys1 = keys + NP;                                             // [L]
  unsigned long long* scan_a = keys1 + L;                                            // [kSelThreads]
  unsigned long long* scan_b = scan_a + kSelThreads;                                 // [kSelThreads]
  SelShared* sh = reinterpret_cast<SelShared*>(scan_b + kSelThreads);                // 8-byte aligned
  float* phi = reinterpret_cast<float*>(sh + 1);                                     // [L]
  int* cand = reinterpret_cast<int*>(phi + L);                                       // [L]
  int* slist = cand + L;                                                             // [L]
  unsigned char* msk = reinterpret_cast<unsigned char*>(slist + L);                  // [L]
  unsigned char* sel = msk + L;                                                      // [L]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  // ---- phase 0: mask flags, first masked position, |M_t|
  if (tid == 0) { sh->scalar[0] = 0x7fffffff; sh->scalar[1] = 0; sh->scalar[2] = 0x7fffffff; sh->total = 0ull; }
  __syncthreads();
  {
    int first = 0x7fffffff, cnt = 0;
    for (int j = tid; j < L; j += kSelThreads) {
      const unsigned char f = a.is_masked[j] ? 1 : 0;
      msk[j] = f;
      sel[j] = 0;
      if (f) { cnt++; first = min(first, j); }
    }
    if (first != 0x7fffffff) atomicMin(&sh->scalar[0], first);
    if (cnt) atomicAdd(&sh->scalar[1], cnt);
  }
  __syncthreads();
  const int first_masked = sh->scalar[0];
  const int n_masked = sh->scalar[1];
  int lo = L, hi = L;
  if (n_masked > 0) {
    // blocks are counted from the end of the prompt in both directions (floor division): a masked
    // position inside the prompt -- nothing the decoding loop produces, but a legal input -- lies in a
    // block with a negative number, cut at position 0
    const int diff = first_masked - a.prompt_len;
    const int b = diff >= 0 ? diff / a.block_len : -((-diff + a.block_len - 1) / a.block_len);
    const int lo_raw = a.prompt_len + b * a.block_len;
    lo = max(0, lo_raw);
    hi = min(L, lo_raw + a.block_len);
  }

  // ---- phase 1: Eq. 3 on the masked tokens of the current block, score = D(i) * s^i
  const float inv2s2 = 1.0f / (2.0f * a.sigma * a.sigma);
  for (int d = tid; d < L; d += kSelThreads) {
    phi[d] = expf(-((float)d * (float)d) * inv2s2);
    if (a.score_out) a.score_out[d] = 0.f;
  }
  const int n1 = block_compact(hi - lo, [&](int t) { return msk[lo + t] != 0; },
                               [&](int slot, int t) { cand[slot] = lo + t; }, sh);
  for (int c = wave; c < n1; c += kSelWaves) {
    const int i = cand[c];
    float dsum = 0.f;
    for (int j = lane; j < L; j += kWave)
      if (!msk[j]) dsum += phi[abs(i - j)];
    dsum = wave_sum(dsum);
    if (lane == 0) {
      const float score = dsum * a.conf[i];
      keys1[c] = make_key(score, i);
      if (a.score_out) a.score_out[i] = score;
    }
  }
  __syncthreads();

  // ---- phase 2: Eq. 4 (top-k) and the decode set by rank counting.  The decode set ranks the same
  // scores, or the confidences alone (conf_decode), and with a threshold also takes every candidate
  // whose confidence exceeds it.
  if (a.conf_decode)
    for (int c = tid; c < n1; c += kSelThreads) keys[c] = make_key(a.conf[cand[c]], cand[c]);
  __syncthreads();
  const unsigned long long* dkeys = a.conf_decode ? keys : keys1;
  for (int c = tid; c < n1; c += kSelThreads) {
    const unsigned long long mine = keys1[c], dmine = dkeys[c];
    int rank = 0, drank = 0;
    for (int o = 0; o < n1; ++o) {
      rank += keys1[o] > mine ? 1 : 0;
      drank += dkeys[o] > dmine ? 1 : 0;
    }
    unsigned char f = 0;
    if (rank < a.k) f |= 1;
    if (drank < a.n_unmask) f |= 4;
    if (a.threshold > 0.f && a.conf[cand[c]] > a.threshold) f |= 4;
    sel[cand[c]] = f;
  }
  __syncthreads();
  const int n_mstar = block_compact(n1, [&](int c) { return (sel[cand[c]] & 1) != 0; },
                                    [&](int slot, int c) { a.mstar[slot] = cand[c]; }, sh);
  const int n_dec = block_compact(n1, [&](int c) { return (sel[cand[c]] & 4) != 0; },
                                  [&](int slot, int c) { a.decode_idx[slot] = cand[c]; }, sh);

  // ---- phase 3: stage-2 keys (influence bits, lower index first); non-candidates sort last as key 0
  {
    unsigned long long part = 0ull;
    for (int j = tid; j < NP; j += kSelThreads) {
      unsigned long long key = 0ull;
      if (j < L) {
        const bool is_cand = a.cand_mode == 0 ? (msk[j] == 0) : ((sel[j] & 1) == 0);
        if (is_cand) {
          key = make_key(a.influence[j], j);
          part += key_mass(key);
        }
      }
      keys[j] = key;
    }
    if (part) atomicAdd(&sh->total, part);      // integer sum: order does not matter
  }
  __syncthreads();
  const int n2 = block_compact(L, [&](int j) { return keys[j] != 0ull; }, [&](int, int) {}, sh);
  const unsigned long long total = sh->total;

  // bitonic network, descending
  for (int k = 2; k <= NP; k <<= 1) {
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int t = tid; t < (NP >> 1); t += kSelThreads) {
        const int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
        const int ixj = i | j;
        const unsigned long long x = keys[i], y = keys[ixj];
        const bool up = (i & k) == 0;
        if (up ? (x < y) : (x > y)) { keys[i] = y; keys[ixj] = x; }
      }
      __syncthreads();
    }
  }

  // ---- phase 4: smallest prefix whose mass exceeds floor(p * total)
  int take = n2;
  if (n2 > 0 && a.p < 1.0f) {
    const unsigned long long thr = (unsigned long long)floor((double)a.p * __ull2double_rn(total));
    const int per = (NP + kSelThreads - 1) / kSelThreads;
    const int begin = tid * per;
    unsigned long long local = 0ull;
    for (int e = 0; e < per; ++e) {
      const int rnk = begin + e;
      if (rnk < n2) local += key_mass(keys[rnk]);
    }
    scan_a[tid] = local;
    __syncthreads();
    unsigned long long* src = scan_a;
    unsigned long long* dst = scan_b;
    for (int o = 1; o < kSelThreads; o <<= 1) {            // inclusive Hillis-Steele scan
      dst[tid] = src[tid] + (tid >= o ? src[tid - o] : 0ull);
      __syncthreads();
      unsigned long long* t = src; src = dst; dst = t;
    }
    unsigned long long run = src[tid] - local;             // exclusive prefix of this thread's chunk
    int found = 0x7fffffff;
    for (int e = 0; e < per; ++e) {
      const int rnk = begin + e;
      if (rnk < n2) {
        run += key_mass(keys[rnk]);
        if (run > thr && found == 0x7fffffff) found = rnk;
      }
    }
    if (found != 0x7fffffff) atomicMin(&sh->scalar[2], found);
    __syncthreads();
    if (sh->scalar[2] != 0x7fffffff) take = sh->scalar[2] + 1;
  }
  for (int rnk = tid; rnk < take; rnk += kSelThreads) sel[key_index(keys[rnk])] |= 2;
  __syncthreads();

  // ---- phase 5: unmask (Eq. 2), emit U, S_{t+1} = M* u U and its still-masked rows
  for (int c = tid; c < n1; c += kSelThreads) {
    const int i = cand[c];
    if (sel[i] & 4) {
      a.tokens[i] = a.pred[i];
      a.is_masked[i] = 0;
      msk[i] = 0;
    }
  }
  const int n_u = block_compact(L, [&](int j) { return (sel[j] & 2) != 0; },
                                [&](int slot, int j) { a.u_set[slot] = j; }, sh);
  const int n_s = block_compact(L, [&](int j) { return sel[j] != 0; },
                                [&](int slot, int j) { a.s_next[slot] = j; slist[slot] = j; }, sh);
  const int n_rows = block_compact(n_s, [&](int rr) { return msk[slist[rr]] != 0; },
                                   [&](int slot, int rr) { a.s_rows_next[slot] = rr; }, sh);
  if (tid == 0) {
    a.counts[0] = n_mstar;
    a.counts[1] = n_u;
    a.counts[2] = n_s;
    a.counts[3] = n_dec;
    a.counts[4] = n_rows;
    a.counts[5] = n_masked - n_dec;
    a.counts[6] = lo;
    a.counts[7] = hi;
  }
}

size_t select_smem_bytes(int L, int NP) {
  return (size_t)NP * 8 + (size_t)L * 8 + 2 * (size_t)kSelThreads * 8 + (size_t)L * 12 + sizeof(SelShared) +
         2 * (size_t)L + 64;
}

// Step-0 state: S_0 = all rows, s_rows = masked rows, conf = 0, pred = 0.
__global__ __launch_bounds__(kSelThreads) void seq_reset_kernel(const uint8_t* __restrict__ is_masked, int L,
                                                                int32_t* __restrict__ s_idx,
                                                                int32_t* __restrict__ s_rows,
                                                                float* __restrict__ conf, int32_t* __restrict__ pred,
                                                                int32_t* __restrict__ counts) {
  __shared__ SelShared sh;
  for (int j = threadIdx.x; j < L; j += kSelThreads) {
    s_idx[j] = j;
    conf[j] = 0.f;
    pred[j] = 0;
  }
  const int n = block_compact(L, [&](int j) { return is_masked[j] != 0; },
                              [&](int slot, int j) { s_rows[slot] = j; }, &sh);
  if (threadIdx.x == 0) {
    for (int c = 0; c < 8; ++c) counts[c] = 0;
    counts[2] = L;
    counts[4] = n;
    counts[5] = n;
  }
}

}  // namespace

int select_max_len() { return kSelMaxL; }

size_t confidence_scratch_floats(int n_rows) { return (size_t)n_rows * kConfMaxChunks * 3; }

hipError_t launch_confidence(const float* logits, const int32_t* pos, const int32_t* via, int n_rows, int vocab,
                             float* conf, int32_t* pred, float* scratch, hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  if (vocab <= 0 || scratch == nullptr) return hipErrorInvalidValue;
  int chunk = 8192;
  while ((vocab + chunk - 1) / chunk > kConfMaxChunks) chunk *= 2;
  const int n_chunks = (vocab + chunk - 1) / chunk;
  if (chunk == 8192 && vocab % 4 == 0 && vocab >= 4 && (uintptr_t)logits % 16 == 0)
    hipLaunchKernelGGL(confidence_chunk_vec_kernel, dim3(n_chunks, n_rows), dim3(kConfThreads), 0, st, logits, vocab,
                       n_chunks, scratch);
  else
    hipLaunchKernelGGL(confidence_chunk_kernel, dim3(n_chunks, n_rows), dim3(kConfThreads), 0, st, logits, vocab, chunk,
                       n_chunks, scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(confidence_merge_kernel, dim3((n_rows + 63) / 64), dim3(64), 0, st, scratch, n_rows, n_chunks,
                     pos, via, conf, pred);
  return hipGetLastError();
}

hipError_t launch_rollout(const float* attn_avg, const float* c_in, float* c_out, const int32_t* idx, int m, int L,
                          bool first, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  if (first) {
    hipLaunchKernelGGL(rollout_first_kernel, dim3((L + kRollThreads - 1) / kRollThreads, m), dim3(kRollThreads), 0, st,
                       attn_avg, c_out, idx, m, L);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(rollout_kernel, dim3((L + 63) / 64, (m + 15) / 16), dim3(kRollThreads), 0, st, attn_avg, c_in,
                     c_out, idx, m, L);
  return hipGetLastError();
}

hipError_t launch_influence(const float* c_block, const int32_t* idx, int m, int L, float* influence,
                            hipStream_t st) {
  if (L <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(influence_kernel, dim3((L + 255) / 256), dim3(256), 0, st, c_block, idx, m, L, influence);
  return hipGetLastError();
}

int chain_max_batch() { return kChainMaxSeqs; }

hipError_t launch_influence_chain(const ChainCall* calls, int n_calls, size_t layer_stride, int n_layers,
                                  float* u_scratch, float* g_scratch, hipStream_t st) {
  if (n_calls <= 0) return hipSuccess;
  if (n_calls > kChainMaxSeqs || n_layers < 0) return hipErrorInvalidValue;
  ChainSeqs seqs;
  std::memset(&seqs, 0, sizeof(seqs));
  int n = 0, max_m = 0, max_L = 0;
  size_t g_off = 0, u_off = 0;
  for (int i = 0; i < n_calls; ++i) {
    const ChainCall& c = calls[i];
    if (c.L <= 0 || c.L > kChainMaxLen || c.m < 0 || c.m > c.L) return hipErrorInvalidValue;
    if (c.m == 0 || n_layers == 0) {         // nothing was refreshed: C = I, every c_j = 1
      hipLaunchKernelGGL(ones_kernel, dim3((c.L + 255) / 256), dim3(256), 0, st, c.influence, c.L);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      continue;
    }
    seqs.seq[n++] = ChainSeq{c.abar, c.idx, c.influence, c.m, c.L, g_off, u_off};
    g_off += (size_t)n_layers * c.m * c.m;
    u_off += (size_t)n_layers * c.m;
    max_m = std::max(max_m, c.m);
    max_L = std::max(max_L, c.L);
  }
  if (n == 0) return hipSuccess;
  const size_t mm = (size_t)max_m * max_m;
  hipLaunchKernelGGL(chain_gather_kernel, dim3((unsigned)((mm + 255) / 256), n_layers, n), dim3(256), 0, st, seqs,
                     layer_stride, g_scratch);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (max_m >= kChainSpreadMinRows) {
    // long index sets: a launch per layer over m / 64 workgroups beats one workgroup walking all layers
    for (int l = n_layers - 1; l >= 0; --l) {
      hipLaunchKernelGGL(chain_layer_kernel, dim3((max_m + 63) / 64, n), dim3(kChainThreads), 0, st, seqs, n_layers, l,
                         g_scratch, u_scratch);
      e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
  } else {
    hipLaunchKernelGGL(chain_rows_kernel, dim3(n), dim3(kChainThreads), 0, st, seqs, n_layers, g_scratch, u_scratch);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(chain_cols_kernel, dim3((max_L + 63) / 64, n), dim3(kChainThreads), 0, st, seqs, layer_stride,
                     n_layers, u_scratch);
  return hipGetLastError();
}

int select_max_batch() { return kSelMaxBatch; }

hipError_t launch_select(const SelectArgs* args, int n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n > kSelMaxBatch) return hipErrorInvalidValue;
  SelectBatch batch;
  size_t smem = 0;
  for (int i = 0; i < n; ++i) {
    const SelectArgs& a = args[i];
    if (a.L <= 0 || a.L > kSelMaxL || a.block_len <= 0 || a.prompt_len < 0 || a.prompt_len > a.L)
      return hipErrorInvalidValue;
    int NP = 2;
    while (NP < a.L) NP <<= 1;
    smem = std::max(smem, select_smem_bytes(a.L, NP));
    batch.seq[i] = a;
  }
  for (int i = n; i < kSelMaxBatch; ++i) batch.seq[i] = args[0];        // never read: the grid has n workgroups
  static int lds_limit = 0;
  if (lds_limit == 0) {
    int dev = 0, optin = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&optin, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(select_kernel),
                            hipFuncAttributeMaxDynamicSharedMemorySize, optin);
    if (e != hipSuccess) return e;
    lds_limit = optin;
  }
  if (smem > (size_t)lds_limit) return hipErrorInvalidValue;
  hipLaunchKernelGGL(select_kernel, dim3(n), dim3(kSelThreads), smem, st, batch);
  return hipGetLastError();
}

hipError_t launch_seq_reset(const uint8_t* is_masked, int L, int32_t* s_idx, int32_t* s_rows, float* conf,
                            int32_t* pred, int32_t* counts, hipStream_t st) {
  if (L <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(seq_reset_kernel, dim3(1), dim3(kSelThreads), 0, st, is_masked, L, s_idx, s_rows, conf, pred,
                     counts);
  return hipGetLastError();
}

}  // namespace d2c
