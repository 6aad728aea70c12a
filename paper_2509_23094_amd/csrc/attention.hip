// Selective-refresh attention: the m selected query rows attend to ALL L cached
// keys without a mask, and the kernel also emits A-bar, the mean over the query
// heads of the normalised attention rows (A^(l) in R^{H x |y*| x L} averaged over
// heads, Sec. 4.2 of the d2Cache paper), which the rollout (Eq. 6-8) consumes.
//
// bf16 path, two launches, no atomics (bit-reproducible):
//   pass 1  one workgroup per (16-query tile, head); its 4 waves take key tiles
//           round-robin, run an online softmax and merge through LDS.  Scores are
//           computed transposed, S^T = K Q^T, so that the 16x16 accumulator layout
//           (4 consecutive keys per lane for one query) IS the B operand of the
//           16x16x16 matrix-core step of O^T = V^T P^T: P never leaves registers.
//           V rows are read straight from global memory (8 bytes = 4 head-dim
//           values per lane and key) and a 4x4 in-register transpose turns them
//           into the A operand (4 keys per lane for one head-dim value).
//           Writes O (bf16) and the log-sum-exp per (head, row).
//   pass 2  one wave per (16-query tile, 16-key tile) loops over the heads,
//           recomputes S^T and accumulates exp(s - lse) in registers; one
//           16-byte store per lane writes A-bar.
// fp32 path (small test model only): one workgroup per query row, plain FMA.
#include "common.cuh"
#include "internal.h"

namespace d2c {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;

__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xffffu) | (b << 16); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xffff0000u); }

// S^T tile for 16 keys x 16 queries: acc[j] = <K[key0+4g+j], Q[q0+r]> (raw dot product)
template <int DH>
__device__ __forceinline__ f32x4 score_tile(const bf16* __restrict__ kbase, size_t k_pitch, int key0, int L,
                                            const Frag<bf16> (&qf)[DH / 32], int r, int g) {
  const int key = min(key0 + r, L - 1);
  const bf16* krow = kbase + (size_t)key * k_pitch + g * 8;
  Frag<bf16> kf[DH / 32];
#pragma unroll
  for (int s = 0; s < DH / 32; ++s) kf[s].raw = ld16(krow + s * 32);
  f32x4 st = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < DH / 32; ++s) mfma16(st, kf[s], qf[s]);
  return st;
}

template <int DH>
__global__ __launch_bounds__(kThreads) void attn_fwd_bf16_kernel(
    const bf16* __restrict__ q, const bf16* __restrict__ k_cache, const bf16* __restrict__ v_cache, int m, int L,
    int n_heads, int n_kv_heads, float scale, bf16* __restrict__ out, float* __restrict__ lse) {
  constexpr int NS = DH / 32;     // contraction steps of Q K^T
  constexpr int NB = DH / 64;     // 64-wide head-dim blocks of the output
  __shared__ float o_lds[kWaves][16][DH + 1];
  __shared__ float m_lds[kWaves][16], l_lds[kWaves][16];

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.x * 16;
  const int head = blockIdx.y;
  const int kvh = head / (n_heads / n_kv_heads);
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const bf16* kbase = k_cache + (size_t)kvh * DH;
  const bf16* vbase = v_cache + (size_t)kvh * DH;

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

  const int n_tiles = (L + 15) / 16;
  for (int t = wave; t < n_tiles; t += kWaves) {
    const int key0 = t * 16;
    f32x4 st = score_tile<DH>(kbase, kv_pitch, key0, L, qf, r, g);
    float x[4];
    float tmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      x[j] = (key0 + 4 * g + j < L) ? st[j] * scale : -INFINITY;
      tmax = fmaxf(tmax, x[j]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, kWave));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = __expf(m_run - m_new);
    float p[4];
    float psum = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = __expf(x[j] - m_new);
      psum += p[j];
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    bf16x4 pb = {(bf16)p[0], (bf16)p[1], (bf16)p[2], (bf16)p[3]};
    const s16x4 pfrag = __builtin_bit_cast(s16x4, pb);

#pragma unroll
    for (int b = 0; b < NB; ++b) {
      // four keys (4g+e) x four head-dim values (b*64 + 4r + i), then transpose in registers
      u32x2 v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int key = min(key0 + 4 * g + e, L - 1);
        v[e] = ld8(vbase + (size_t)key * kv_pitch + b * 64 + 4 * r);
      }
      u32x2 op[4];
      op[0] = u32x2{pack_lo(v[0].x, v[1].x), pack_lo(v[2].x, v[3].x)};
      op[1] = u32x2{pack_hi(v[0].x, v[1].x), pack_hi(v[2].x, v[3].x)};
      op[2] = u32x2{pack_lo(v[0].y, v[1].y), pack_lo(v[2].y, v[3].y)};
      op[3] = u32x2{pack_hi(v[0].y, v[1].y), pack_hi(v[2].y, v[3].y)};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[b][i] *= alpha;
        acc[b][i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, op[i]), pfrag, acc[b][i], 0,
                                                              0, 0);
      }
    }
  }

  // merge the four waves' partial softmaxes
  l_run += __shfl_xor(l_run, 16, kWave);
  l_run += __shfl_xor(l_run, 32, kWave);
  if (g == 0) {
    m_lds[wave][r] = m_run;
    l_lds[wave][r] = l_run;
  }
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) o_lds[wave][r][b * 64 + 16 * g + 4 * j + i] = acc[b][i][j];
  __syncthreads();

  for (int o = tid; o < 16 * DH; o += kThreads) {
    const int qi = o / DH, dcol = o - qi * DH;
    float mx = m_lds[0][qi];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) mx = fmaxf(mx, m_lds[w][qi]);
    float lsum = 0.f, osum = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = __expf(m_lds[w][qi] - mx);
      lsum += l_lds[w][qi] * f;
      osum += o_lds[w][qi][dcol] * f;
    }
    if (q0 + qi < m) {
      out[(size_t)(q0 + qi) * dq + head * DH + dcol] = (bf16)(osum / lsum);
      if (dcol == 0) lse[(size_t)head * m + q0 + qi] = mx + __logf(lsum);
    }
  }
}

template <int DH>
__global__ __launch_bounds__(kThreads) void attn_avg_bf16_kernel(const bf16* __restrict__ q,
                                                                 const bf16* __restrict__ k_cache,
                                                                 const float* __restrict__ lse, int m, int L,
                                                                 int n_heads, int n_kv_heads, float scale,
                                                                 float* __restrict__ attn_avg) {
  constexpr int NS = DH / 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int q0 = blockIdx.x * 16;
  const int key0 = (blockIdx.y * kWaves + wave) * 16;
  if (key0 >= L) return;
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const int group = n_heads / n_kv_heads;
  const int row = min(q0 + r, m - 1);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int head = 0; head < n_heads; ++head) {
    Frag<bf16> qf[NS];
    const bf16* qrow = q + (size_t)row * dq + head * DH + g * 8;
#pragma unroll
    for (int s = 0; s < NS; ++s) qf[s].raw = ld16(qrow + s * 32);
    const f32x4 st = score_tile<DH>(k_cache + (size_t)(head / group) * DH, kv_pitch, key0, L, qf, r, g);
    const float e = lse[(size_t)head * m + row];
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[j] += __expf(st[j] * scale - e);
  }
  if (q0 + r >= m) return;
  const float inv_h = 1.0f / (float)n_heads;
  float* dst = attn_avg + (size_t)(q0 + r) * L + key0 + 4 * g;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (key0 + 4 * g + j < L) dst[j] = acc[j] * inv_h;
}

// fp32 path: one workgroup per query row, heads in sequence.
__global__ __launch_bounds__(kThreads) void attn_f32_kernel(const float* __restrict__ q,
                                                            const float* __restrict__ k_cache,
                                                            const float* __restrict__ v_cache, int L, int n_heads,
                                                            int n_kv_heads, int head_dim, float scale,
                                                            float* __restrict__ out, float* __restrict__ attn_avg) {
  extern __shared__ float smem[];          // scores[L], abar[L], red[8]
  float* scores = smem;
  float* abar = smem + L;
  float* red = abar + L;
  const int row = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int dq = n_heads * head_dim, dkv = n_kv_heads * head_dim, group = n_heads / n_kv_heads;
  for (int j = tid; j < L; j += kThreads) abar[j] = 0.f;
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
    const float inv = 1.0f / (red[4] + red[5] + red[6] + red[7]);
    for (int j = tid; j < L; j += kThreads) abar[j] += scores[j] * inv;
    for (int e = tid; e < head_dim; e += kThreads) {
      float o = 0.f;
      for (int j = 0; j < L; ++j) o = fmaf(scores[j], v_cache[(size_t)j * dkv + kvh * head_dim + e], o);
      out[(size_t)row * dq + head * head_dim + e] = o * inv;
    }
    __syncthreads();
  }
  if (attn_avg != nullptr) {
    const float inv_h = 1.0f / (float)n_heads;
    for (int j = tid; j < L; j += kThreads) attn_avg[(size_t)row * L + j] = abar[j] * inv_h;
  }
}

template <int DH>
hipError_t launch_bf16(const void* q, const void* k_cache, const void* v_cache, int m, int L, int n_heads,
                       int n_kv_heads, void* out, float* lse, float* attn_avg, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)DH);
  const int q_tiles = (m + 15) / 16;
  hipLaunchKernelGGL(attn_fwd_bf16_kernel<DH>, dim3(q_tiles, n_heads), dim3(kThreads), 0, st, (const bf16*)q,
                     (const bf16*)k_cache, (const bf16*)v_cache, m, L, n_heads, n_kv_heads, scale, (bf16*)out, lse);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || attn_avg == nullptr) return e;
  const int key_blocks = (L + 16 * kWaves - 1) / (16 * kWaves);
  hipLaunchKernelGGL(attn_avg_bf16_kernel<DH>, dim3(q_tiles, key_blocks), dim3(kThreads), 0, st, (const bf16*)q,
                     (const bf16*)k_cache, lse, m, L, n_heads, n_kv_heads, scale, attn_avg);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attention(int dtype, const void* q, const void* k_cache, const void* v_cache, int m, int L,
                            int n_heads, int n_kv_heads, int head_dim, void* out, float* lse, float* attn_avg,
                            hipStream_t st) {
  if (m <= 0) return hipSuccess;
  if (L <= 0 || n_heads % n_kv_heads) return hipErrorInvalidValue;
  if (dtype == kBF16) {
    if (head_dim == 128) return launch_bf16<128>(q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, attn_avg, st);
    if (head_dim == 64) return launch_bf16<64>(q, k_cache, v_cache, m, L, n_heads, n_kv_heads, out, lse, attn_avg, st);
    return hipErrorInvalidValue;
  }
  const size_t smem = ((size_t)2 * L + 8) * sizeof(float);
  if (smem > 64 * 1024) return hipErrorInvalidValue;   // default dynamic LDS limit
  const float scale = 1.0f / sqrtf((float)head_dim);
  hipLaunchKernelGGL(attn_f32_kernel, dim3(m), dim3(kThreads), smem, st, (const float*)q, (const float*)k_cache,
                     (const float*)v_cache, L, n_heads, n_kv_heads, head_dim, scale, (float*)out, attn_avg);
  return hipGetLastError();
}

}  // namespace d2c
