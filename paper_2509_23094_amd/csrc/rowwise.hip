// Row-wise kernels around the projections of one block on the selected rows
// (Eq. 5 of the d2Cache paper): embedding gather, residual add + RMSNorm,
// RoPE + K/V cache update ("updates their KV states", Sec. 4 overview), SwiGLU.
// All of them are HBM/L2-bound copies with a little arithmetic: one workgroup
// per row, 16-byte coalesced accesses where the layout allows.
#include <cstring>

#include "common.h"
#include "internal.h"

namespace d2c {
namespace {

constexpr int kThreads = 256;
constexpr int kManyRows = 256;       // from this many rows on a launch is bound by throughput, not by one memory latency

// Sum over the workgroup, same value in every thread, fixed order.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  __syncthreads();
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += red[w];
  return t;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void embed_norm_kernel(const T* __restrict__ emb,
                                                              const int32_t* __restrict__ tokens,
                                                              const int32_t* __restrict__ idx, int d,
                                                              const float* __restrict__ gain, float eps,
                                                              float* __restrict__ h, T* __restrict__ a) {
  __shared__ float red[kThreads / 64];
  const int r = blockIdx.x;
  const T* src = emb + (size_t)tokens[idx[r]] * d;
  float* hr = h + (size_t)r * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    float v = to_f32(src[c]);
    hr[c] = v;
    ss += v * v;
  }
  const float inv = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
  T* ar = a + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += kThreads) ar[c] = from_f32<T>(hr[c] * inv * gain[c]);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_norm_kernel(float* __restrict__ h, const float* __restrict__ P,
                                                            int n_splits, size_t split_stride, int ldp, int d,
                                                            const float* __restrict__ gain, float eps,
                                                            T* __restrict__ a) {
  __shared__ float red[kThreads / 64];
  const int r = blockIdx.x;
  float* hr = h + (size_t)r * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    float v = hr[c];
    float add = 0.f;
    for (int s = 0; s < n_splits; ++s) add += P[(size_t)s * split_stride + (size_t)r * ldp + c];
    v += add;
    hr[c] = v;
    ss += v * v;
  }
  if (a == nullptr) return;
  const float inv = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
  T* ar = a + (size_t)r * d;
  for (int c = threadIdx.x; c < d; c += kThreads) ar[c] = from_f32<T>(hr[c] * inv * gain[c]);
}

__device__ __forceinline__ void store4(float* dst, const f32x4& v) { *reinterpret_cast<f32x4*>(dst) = v; }
__device__ __forceinline__ void store4(bf16* dst, const f32x4& v) {
  bf16x4 o = {(bf16)v.x, (bf16)v.y, (bf16)v.z, (bf16)v.w};
  *reinterpret_cast<bf16x4*>(dst) = o;
}

// Same as add_norm_kernel for d <= 4*THREADS*PIECES, d % 4 == 0: PIECES 16-byte pieces of the row per thread,
// kept in registers; a thread's loads (the row pieces and one piece per split) are all independent.  With one
// piece per thread a 4096-wide row is spread over 16 waves and the kernel is about one memory latency long (a
// handful of rows); with four pieces per thread more rows are resident per compute unit, which is what many
// rows need.
template <typename T, int THREADS, int PIECES>
__global__ __launch_bounds__(THREADS) void add_norm_vec_kernel(float* __restrict__ h, const float* __restrict__ P,
                                                               int n_splits, size_t split_stride, int ldp, int d,
                                                               const float* __restrict__ gain, float eps,
                                                               T* __restrict__ a) {
  __shared__ float red[THREADS / 64];
  const int r = blockIdx.x;
  float* hr = h + (size_t)r * d;
  const float* pr = P + (size_t)r * ldp;
  f32x4 v[PIECES];
#pragma unroll
  for (int p = 0; p < PIECES; ++p) {
    const int c = (threadIdx.x + p * THREADS) * 4;
    v[p] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (c < d) v[p] = *reinterpret_cast<const f32x4*>(hr + c);
  }
  if (n_splits > 0) {
#pragma unroll
    for (int p = 0; p < PIECES; ++p) {
      const int c = (threadIdx.x + p * THREADS) * 4;
      if (c >= d) continue;
      f32x4 add = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
      for (int s = 0; s < n_splits; ++s) add += *reinterpret_cast<const f32x4*>(pr + (size_t)s * split_stride + c);
      v[p] += add;
      store4(hr + c, v[p]);
    }
  }
  if (a == nullptr) return;
  float ss = 0.f;
#pragma unroll
  for (int p = 0; p < PIECES; ++p) ss += v[p].x * v[p].x + v[p].y * v[p].y + v[p].z * v[p].z + v[p].w * v[p].w;
  const float inv = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
#pragma unroll
  for (int p = 0; p < PIECES; ++p) {
    const int c = (threadIdx.x + p * THREADS) * 4;
    if (c < d) store4(a + (size_t)r * d + c, v[p] * inv * *reinterpret_cast<const f32x4*>(gain + c));
  }
}

// Four consecutive elements of a row of T as floats (the row start and c are multiples of 4 elements).
__device__ __forceinline__ f32x4 load4(const float* p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ f32x4 load4(const bf16* p) {
  const bf16x4 v = *reinterpret_cast<const bf16x4*>(p);
  return f32x4{(float)v.x, (float)v.y, (float)v.z, (float)v.w};
}

// embed_norm_kernel / gather_norm_kernel for d <= 4*THREADS, d % 4 == 0: the row stays in registers, one
// 4-element piece per thread (src: the embedding row of T, or the fp32 hidden row; h_out may be null).
template <typename T, typename S, int THREADS>
__global__ __launch_bounds__(THREADS) void row_norm_vec_kernel(const S* __restrict__ src_base,
                                                               const int32_t* __restrict__ tokens,
                                                               const int32_t* __restrict__ rows, int d,
                                                               const float* __restrict__ gain, float eps,
                                                               float* __restrict__ h_out, T* __restrict__ a) {
  __shared__ float red[THREADS / 64];
  const int r = blockIdx.x;
  const int src_row = tokens ? tokens[rows[r]] : rows[r];
  const int c = threadIdx.x * 4;
  const bool live = c < d;
  f32x4 v = {0.f, 0.f, 0.f, 0.f};
  if (live) {
    v = load4(src_base + (size_t)src_row * d + c);
    if (h_out) store4(h_out + (size_t)r * d + c, v);
  }
  const float ss = v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  const float inv = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
  if (live) store4(a + (size_t)r * d + c, v * inv * *reinterpret_cast<const f32x4*>(gain + c));
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gather_norm_kernel(const float* __restrict__ h,
                                                               const int32_t* __restrict__ rows, int d,
                                                               const float* __restrict__ gain, float eps,
                                                               T* __restrict__ a) {
  __shared__ float red[kThreads / 64];
  const float* hr = h + (size_t)rows[blockIdx.x] * d;
  float ss = 0.f;
  for (int c = threadIdx.x; c < d; c += kThreads) {
    float v = hr[c];
    ss += v * v;
  }
  const float inv = 1.0f / sqrtf(block_sum(ss, red) / (float)d + eps);
  T* ar = a + (size_t)blockIdx.x * d;
  for (int c = threadIdx.x; c < d; c += kThreads) ar[c] = from_f32<T>(hr[c] * inv * gain[c]);
}

// The sequences whose rows one RoPE / cache-update launch covers: rows off .. off+m of the compact buffers
// belong to a sequence with its own index set and caches.
constexpr int kRopeMaxSeqs = 8;
struct RopeSeqs {
  const int32_t* idx[kRopeMaxSeqs];
  void* k_cache[kRopeMaxSeqs];
  void* v_cache[kRopeMaxSeqs];
  int off[kRopeMaxSeqs + 1];          // off[n] = total rows
  int n;
};
__device__ __forceinline__ int rope_seq_of(const RopeSeqs& sq, int r) {
  int s = 0;
  while (s + 1 < sq.n && r >= sq.off[s + 1]) ++s;
  return s;
}

// One workgroup per selected row.  Columns of the fused projection: n_heads
// query heads, then n_kv_heads key heads, then n_kv_heads value heads.
// Rotate-half RoPE pairs element i with i + head_dim/2 inside a head.
template <typename T>
__global__ __launch_bounds__(kThreads) void qkv_rope_scatter_kernel(
    const float* __restrict__ P, int n_splits, size_t split_stride, int ldp, const float* __restrict__ bias,
    const RopeSeqs seqs, int n_heads, int n_kv_heads, int head_dim, const float* __restrict__ rope_cos,
    const float* __restrict__ rope_sin, T* __restrict__ q_out) {
  const int r = blockIdx.x;
  const int sq = rope_seq_of(seqs, r);
  const int pos = seqs.idx[sq][r - seqs.off[sq]];
  T* __restrict__ k_cache = static_cast<T*>(seqs.k_cache[sq]);
  T* __restrict__ v_cache = static_cast<T*>(seqs.v_cache[sq]);
  const int half = head_dim >> 1;
  const int dq = n_heads * head_dim, dkv = n_kv_heads * head_dim;
  const float* pr = P + (size_t)r * ldp;
  auto col = [&](int c) {
    float v = bias ? bias[c] : 0.f;
    for (int s = 0; s < n_splits; ++s) v += pr[(size_t)s * split_stride + c];
    return v;
  };
  const float* cs = rope_cos + (size_t)pos * half;
  const float* sn = rope_sin + (size_t)pos * half;
  // rotated pairs of q and k
  const int n_pairs = (n_heads + n_kv_heads) * half;
  for (int t = threadIdx.x; t < n_pairs; t += kThreads) {
    const int head = t / half, i = t - head * half;
    const int c1 = head * head_dim + i, c2 = c1 + half;      // columns in the fused projection
    const float x1 = col(c1), x2 = col(c2);
    const float c = cs[i], s = sn[i];
    const float o1 = x1 * c - x2 * s, o2 = x2 * c + x1 * s;
    if (head < n_heads) {
      q_out[(size_t)r * dq + c1] = from_f32<T>(o1);
      q_out[(size_t)r * dq + c2] = from_f32<T>(o2);
    } else {
      k_cache[(size_t)pos * dkv + (c1 - dq)] = from_f32<T>(o1);
      k_cache[(size_t)pos * dkv + (c2 - dq)] = from_f32<T>(o2);
    }
  }
  for (int c = threadIdx.x; c < dkv; c += kThreads)
    v_cache[(size_t)pos * dkv + c] = from_f32<T>(col(dq + dkv + c));
}

// Vector form for head_dim % 8 == 0: a work item is four consecutive rotation pairs of one head
// (two 16-byte loads per split) or four consecutive value columns; blockIdx.y strides over items.
template <typename T>
__global__ __launch_bounds__(kThreads) void qkv_rope_scatter_vec_kernel(
    const float* __restrict__ P, int n_splits, size_t split_stride, int ldp, const float* __restrict__ bias,
    const RopeSeqs seqs, int n_heads, int n_kv_heads, int head_dim, const float* __restrict__ rope_cos,
    const float* __restrict__ rope_sin, T* __restrict__ q_out) {
  const int r = blockIdx.x;
  const int sq = rope_seq_of(seqs, r);
  const int pos = seqs.idx[sq][r - seqs.off[sq]];
  T* __restrict__ k_cache = static_cast<T*>(seqs.k_cache[sq]);
  T* __restrict__ v_cache = static_cast<T*>(seqs.v_cache[sq]);
  const int half = head_dim >> 1, q4 = half >> 2;            // 4-wide items per half head
  const int dq = n_heads * head_dim, dkv = n_kv_heads * head_dim;
  const float* pr = P + (size_t)r * ldp;
  auto col4 = [&](int c) {
    f32x4 v = bias ? *reinterpret_cast<const f32x4*>(bias + c) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int s = 0; s < n_splits; ++s) v += *reinterpret_cast<const f32x4*>(pr + (size_t)s * split_stride + c);
    return v;
  };
  const int n_rot = (n_heads + n_kv_heads) * q4;
  const int n_items = n_rot + (dkv >> 2);
  for (int t = blockIdx.y * kThreads + threadIdx.x; t < n_items; t += gridDim.y * kThreads) {
    if (t < n_rot) {
      const int head = t / q4, i = (t - head * q4) * 4;
      const int c1 = head * head_dim + i, c2 = c1 + half;
      const f32x4 x1 = col4(c1), x2 = col4(c2);
      const f32x4 c = *reinterpret_cast<const f32x4*>(rope_cos + (size_t)pos * half + i);
      const f32x4 sn = *reinterpret_cast<const f32x4*>(rope_sin + (size_t)pos * half + i);
      const f32x4 o1 = x1 * c - x2 * sn, o2 = x2 * c + x1 * sn;
      if (head < n_heads) {
        store4(q_out + (size_t)r * dq + c1, o1);
        store4(q_out + (size_t)r * dq + c2, o2);
      } else {
        store4(k_cache + (size_t)pos * dkv + (c1 - dq), o1);
        store4(k_cache + (size_t)pos * dkv + (c2 - dq), o2);
      }
    } else {
      const int c = (t - n_rot) * 4;
      store4(v_cache + (size_t)pos * dkv + c, col4(dq + dkv + c));
    }
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void swiglu_kernel(const float* __restrict__ P, int n_splits,
                                                          size_t split_stride, int ldp, int F, T* __restrict__ act) {
  const int r = blockIdx.y;
  const int f = blockIdx.x * kThreads + threadIdx.x;
  if (f >= F) return;
  float g = 0.f, u = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float* pr = P + (size_t)s * split_stride + (size_t)r * ldp;
    g += pr[f];
    u += pr[F + f];
  }
  act[(size_t)r * F + f] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}

// blockIdx.y picks one of two (rows, cache) pairs that share idx and width: new K rows and new V rows go
// out in one launch
template <typename T>
__global__ __launch_bounds__(kThreads) void scatter_rows_kernel(const T* __restrict__ rows_a, T* __restrict__ cache_a,
                                                                const T* __restrict__ rows_b, T* __restrict__ cache_b,
                                                                const int32_t* __restrict__ idx, int width, int wide) {
  const int r = blockIdx.x;
  const T* src = (blockIdx.y ? rows_b : rows_a) + (size_t)r * width;
  T* dst = (blockIdx.y ? cache_b : cache_a) + (size_t)idx[r] * width;
  if (wide) {                              // rows are whole, aligned 16-byte pieces
    const int n16 = (int)(sizeof(T) * width / 16);
    for (int c = threadIdx.x; c < n16; c += kThreads)
      reinterpret_cast<u32x4*>(dst)[c] = reinterpret_cast<const u32x4*>(src)[c];
  } else {
    for (int c = threadIdx.x; c < width; c += kThreads) dst[c] = src[c];
  }
}

__global__ void copy_f32_kernel(float* __restrict__ dst, const float* __restrict__ src, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = src[i];
}

__global__ void sum_splits_kernel(float* __restrict__ dst, const float* __restrict__ P, int n_splits,
                                  size_t split_stride, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    float v = 0.f;
    for (int s = 0; s < n_splits; ++s) v += P[(size_t)s * split_stride + i];
    dst[i] = v;
  }
}

// Angles in fp64 so that the table is the correctly rounded cos/sin of
// pos * theta^(-2i/head_dim) at every position the cache can hold.
__global__ void rope_table_kernel(float* __restrict__ cos_t, float* __restrict__ sin_t, int max_pos, int half,
                                  double theta) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= max_pos * half) return;
  const int pos = t / half, i = t - pos * half;
  const double ang = (double)pos * pow(theta, -(double)i / (double)half);
  cos_t[t] = (float)cos(ang);
  sin_t[t] = (float)sin(ang);
}

}  // namespace

#define D2C_DISPATCH(dtype, EXPR_BF16, EXPR_F32) \
  do {                                           \
    if ((dtype) == kBF16) { EXPR_BF16; } else { EXPR_F32; } \
  } while (0)

hipError_t launch_embed_norm(int dtype, const void* emb, const int32_t* tokens, const int32_t* idx, int m, int d,
                             const float* gain, float eps, float* h, void* a, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  if (d % 4 == 0 && d <= 4096) {                  // whole 4-element pieces, the row in one workgroup's registers
    D2C_DISPATCH(dtype,
                 hipLaunchKernelGGL((row_norm_vec_kernel<bf16, bf16, 1024>), dim3(m), dim3(1024), 0, st,
                                    (const bf16*)emb, tokens, idx, d, gain, eps, h, (bf16*)a),
                 hipLaunchKernelGGL((row_norm_vec_kernel<float, float, 1024>), dim3(m), dim3(1024), 0, st,
                                    (const float*)emb, tokens, idx, d, gain, eps, h, (float*)a));
    return hipGetLastError();
  }
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(embed_norm_kernel<bf16>, dim3(m), dim3(kThreads), 0, st, (const bf16*)emb, tokens,
                                  idx, d, gain, eps, h, (bf16*)a),
               hipLaunchKernelGGL(embed_norm_kernel<float>, dim3(m), dim3(kThreads), 0, st, (const float*)emb, tokens,
                                  idx, d, gain, eps, h, (float*)a));
  return hipGetLastError();
}

hipError_t launch_add_norm(int dtype, float* h, const float* P, int n_splits, size_t split_stride, int ldp, int m,
                           int d, const float* gain, float eps, void* a, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  if (d % 4 == 0 && d <= 4096 && ldp % 4 == 0 && split_stride % 4 == 0) {
#define D2C_ADD_NORM_VEC(THREADS, PIECES)                                                                          \
  D2C_DISPATCH(dtype,                                                                                             \
               hipLaunchKernelGGL((add_norm_vec_kernel<bf16, THREADS, PIECES>), dim3(m), dim3(THREADS), 0, st, h, P,   \
                                  n_splits, split_stride, ldp, d, gain, eps, (bf16*)a),                           \
               hipLaunchKernelGGL((add_norm_vec_kernel<float, THREADS, PIECES>), dim3(m), dim3(THREADS), 0, st, h, P,  \
                                  n_splits, split_stride, ldp, d, gain, eps, (float*)a))
    if (d <= 1024) {
      D2C_ADD_NORM_VEC(256, 1);
    } else if (m >= kManyRows) {
      D2C_ADD_NORM_VEC(256, 4);
    } else {
      D2C_ADD_NORM_VEC(1024, 1);
    }
#undef D2C_ADD_NORM_VEC
    return hipGetLastError();
  }
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(add_norm_kernel<bf16>, dim3(m), dim3(kThreads), 0, st, h, P, n_splits, split_stride,
                                  ldp, d, gain, eps, (bf16*)a),
               hipLaunchKernelGGL(add_norm_kernel<float>, dim3(m), dim3(kThreads), 0, st, h, P, n_splits,
                                  split_stride, ldp, d, gain, eps, (float*)a));
  return hipGetLastError();
}

hipError_t launch_gather_norm(int dtype, const float* h, const int32_t* rows, int n_rows, int d, const float* gain,
                              float eps, void* a, hipStream_t st) {
  if (n_rows <= 0) return hipSuccess;
  if (d % 4 == 0 && d <= 4096) {
    D2C_DISPATCH(dtype,
                 hipLaunchKernelGGL((row_norm_vec_kernel<bf16, float, 1024>), dim3(n_rows), dim3(1024), 0, st, h,
                                    (const int32_t*)nullptr, rows, d, gain, eps, (float*)nullptr, (bf16*)a),
                 hipLaunchKernelGGL((row_norm_vec_kernel<float, float, 1024>), dim3(n_rows), dim3(1024), 0, st, h,
                                    (const int32_t*)nullptr, rows, d, gain, eps, (float*)nullptr, (float*)a));
    return hipGetLastError();
  }
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(gather_norm_kernel<bf16>, dim3(n_rows), dim3(kThreads), 0, st, h, rows, d, gain,
                                  eps, (bf16*)a),
               hipLaunchKernelGGL(gather_norm_kernel<float>, dim3(n_rows), dim3(kThreads), 0, st, h, rows, d, gain,
                                  eps, (float*)a));
  return hipGetLastError();
}

hipError_t launch_qkv_rope_scatter(int dtype, const float* P, int n_splits, size_t split_stride, int ldp,
                                   const float* bias, const RopeCall* calls, int n_calls, int n_heads, int n_kv_heads,
                                   int head_dim, const float* rope_cos, const float* rope_sin, void* q_out,
                                   hipStream_t st) {
  if (n_calls <= 0) return hipSuccess;
  if (n_calls > kRopeMaxSeqs || head_dim % 2) return hipErrorInvalidValue;
  RopeSeqs sq;
  memset(&sq, 0, sizeof(sq));
  int m = 0;
  for (int i = 0; i < n_calls; ++i) {
    if (calls[i].m <= 0 || calls[i].off != m) return hipErrorInvalidValue;      // consecutive, non-empty slices
    sq.idx[i] = calls[i].idx;
    sq.k_cache[i] = calls[i].k_cache;
    sq.v_cache[i] = calls[i].v_cache;
    sq.off[i] = m;
    m += calls[i].m;
  }
  sq.off[n_calls] = m;
  sq.n = n_calls;
  // the vector kernel reads P, the bias and the RoPE table in 16-byte pieces
  if (head_dim % 8 == 0 && ldp % 4 == 0 && split_stride % 4 == 0 && (uintptr_t)P % 16 == 0 &&
      (bias == nullptr || (uintptr_t)bias % 16 == 0)) {
    const int items = ((n_heads + n_kv_heads) * (head_dim / 8) + n_kv_heads * head_dim / 4);
    const dim3 grid(m, (items + 2 * kThreads - 1) / (2 * kThreads));
    D2C_DISPATCH(dtype,
                 hipLaunchKernelGGL(qkv_rope_scatter_vec_kernel<bf16>, grid, dim3(kThreads), 0, st, P, n_splits,
                                    split_stride, ldp, bias, sq, n_heads, n_kv_heads, head_dim, rope_cos, rope_sin,
                                    (bf16*)q_out),
                 hipLaunchKernelGGL(qkv_rope_scatter_vec_kernel<float>, grid, dim3(kThreads), 0, st, P, n_splits,
                                    split_stride, ldp, bias, sq, n_heads, n_kv_heads, head_dim, rope_cos, rope_sin,
                                    (float*)q_out));
    return hipGetLastError();
  }
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(qkv_rope_scatter_kernel<bf16>, dim3(m), dim3(kThreads), 0, st, P, n_splits,
                                  split_stride, ldp, bias, sq, n_heads, n_kv_heads, head_dim, rope_cos, rope_sin,
                                  (bf16*)q_out),
               hipLaunchKernelGGL(qkv_rope_scatter_kernel<float>, dim3(m), dim3(kThreads), 0, st, P, n_splits,
                                  split_stride, ldp, bias, sq, n_heads, n_kv_heads, head_dim, rope_cos, rope_sin,
                                  (float*)q_out));
  return hipGetLastError();
}

int rope_max_batch() { return kRopeMaxSeqs; }

hipError_t launch_swiglu(int dtype, const float* P, int n_splits, size_t split_stride, int ldp, int m, int F,
                         void* act, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  dim3 grid((F + kThreads - 1) / kThreads, m);
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(swiglu_kernel<bf16>, grid, dim3(kThreads), 0, st, P, n_splits, split_stride, ldp, F,
                                  (bf16*)act),
               hipLaunchKernelGGL(swiglu_kernel<float>, grid, dim3(kThreads), 0, st, P, n_splits, split_stride, ldp,
                                  F, (float*)act));
  return hipGetLastError();
}

hipError_t launch_scatter_rows(int dtype, const void* rows_a, void* cache_a, const void* rows_b, void* cache_b,
                               const int32_t* idx, int m, int width, hipStream_t st) {
  if (m <= 0) return hipSuccess;
  const dim3 grid(m, rows_b ? 2 : 1);
  const uintptr_t bits = (uintptr_t)rows_a | (uintptr_t)cache_a | (uintptr_t)rows_b | (uintptr_t)cache_b;
  const int wide = (bits % 16 == 0) && (dtype_size(dtype) * (size_t)width % 16 == 0);
  D2C_DISPATCH(dtype,
               hipLaunchKernelGGL(scatter_rows_kernel<bf16>, grid, dim3(kThreads), 0, st, (const bf16*)rows_a,
                                  (bf16*)cache_a, (const bf16*)rows_b, (bf16*)cache_b, idx, width, wide),
               hipLaunchKernelGGL(scatter_rows_kernel<float>, grid, dim3(kThreads), 0, st, (const float*)rows_a,
                                  (float*)cache_a, (const float*)rows_b, (float*)cache_b, idx, width, wide));
  return hipGetLastError();
}

hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048);
  hipLaunchKernelGGL(copy_f32_kernel, dim3(blocks), dim3(256), 0, st, dst, src, n);
  return hipGetLastError();
}

hipError_t launch_sum_splits(float* dst, const float* P, int n_splits, size_t split_stride, size_t n, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const int blocks = (int)((n + 1023) / 1024 < 2048 ? (n + 1023) / 1024 : 2048);
  hipLaunchKernelGGL(sum_splits_kernel, dim3(blocks), dim3(256), 0, st, dst, P, n_splits, split_stride, n);
  return hipGetLastError();
}

hipError_t launch_rope_table(float* cos_t, float* sin_t, int max_pos, int head_dim, float theta, hipStream_t st) {
  const int half = head_dim / 2;
  const int n = max_pos * half;
  if (n <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, cos_t, sin_t, max_pos, half,
                     (double)theta);
  return hipGetLastError();
}

}  // namespace d2c
