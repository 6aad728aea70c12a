// Weight-streaming GEMM for the ragged handful of selected rows (Eq. 5 of the
// d2Cache paper feeds only the rows M* u U through the model, so every
// projection is  P = A[m,K] * W[N,K]^T  with m of the order of 100 or less).
//
// At such m the arithmetic intensity is about m FLOP per weight byte, far below
// the chip's ridge: the kernel is bound by streaming W from HBM once.  Design:
//   * each wave owns 16*NT weight rows (output columns) and reads them straight
//     from global memory into matrix-core operand registers, 16 bytes per lane,
//     256 contiguous bytes per weight row and chunk, through a register ring that
//     keeps RING-1 chunks in flight ahead of the one being consumed;
//   * the activation rows (shared by all waves of the workgroup) are staged
//     through LDS in 256-byte-per-row chunks, double-buffered, one barrier per chunk;
//     a chunk is requested two iterations before it is needed in LDS, so its
//     latency never sits between two barriers;
//   * the contraction axis can be split over blockIdx.y; every split writes its
//     own fp32 partial and the consumer kernel sums the partials in a fixed order
//     (deterministic, no atomics);
//   * more than 128 rows are covered by blockIdx.z (step 0 and select-all mode).
#include "common.cuh"
#include "internal.h"

namespace d2c {

Tunables& tunables() {
  static Tunables t;
  return t;
}

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kChunkBytes = 256;                 // bytes of one row in one chunk
constexpr int kRowStride = kChunkBytes + 16;     // LDS row pitch: 16-byte skew, conflict-free 16-byte reads
constexpr int kSteps = 4;                        // matrix-core steps per chunk

// RING = number of weight chunks a wave keeps in registers (one being consumed, RING-1 in flight).
template <typename T, int MT, int NT, int RING>
__global__ __launch_bounds__(kThreads) void gemm_rows_kernel(
    const T* __restrict__ A, int lda, const T* __restrict__ W, int ldw, float* __restrict__ P, int ldp,
    size_t split_stride, int m, int N, int K, int k_per_split) {
  static_assert(RING == 2 || RING == 4, "the ring index and the A register parity must stay compile-time");
  constexpr int E = Frag<T>::kElems;
  constexpr int KS = Frag<T>::kStep;
  constexpr int KC = kSteps * KS;                // elements per chunk (= 256 bytes)
  constexpr int PB = RING - 1;                   // prefetch distance of the weight stream, in chunks
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][MT * 16 * kRowStride];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int row0 = blockIdx.z * (MT * 16);
  const int k_begin = blockIdx.y * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_base = (blockIdx.x * kWaves + wave) * (16 * NT);
  const int n_chunks = (k_end - k_begin + KC - 1) / KC;

  // this lane's weight rows (clamped: out-of-range columns are computed on a valid row and dropped)
  const T* wrow[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    int n = min(n_base + nt * 16 + r, N - 1);
    wrow[nt] = W + (size_t)n * ldw;
  }

  Frag<T> areg[2][MT];                 // areg[c & 1]: activation chunk c on its way from global memory to LDS
  Frag<T> breg[RING][NT][kSteps];      // breg[c % RING]: weight chunk c
  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto load_a = [&](Frag<T> (&a)[MT], int chunk) {
    const int kc = k_begin + chunk * KC;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int f = tid + i * kThreads;          // fragment id in the chunk: row f/16, 16-byte column f%16
      const int row = row0 + (f >> 4);
      const int k = kc + (f & 15) * E;
      if (row < m && k < k_end) a[i].raw = ld16(A + (size_t)row * lda + k);
      else a[i].raw = u32x4{0u, 0u, 0u, 0u};
    }
  };
  auto store_a = [&](const Frag<T> (&a)[MT], int buf) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int f = tid + i * kThreads;
      *reinterpret_cast<u32x4*>(&lds[buf][(f >> 4) * kRowStride + (f & 15) * 16]) = a[i].raw;
    }
  };
  auto load_b = [&](Frag<T> (&b)[NT][kSteps], int chunk) {
    const int kc = k_begin + chunk * KC;
#pragma unroll
    for (int s = 0; s < kSteps; ++s) {
      const int k = kc + s * KS + g * E;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (k < k_end) b[nt][s].raw = ld16(wrow[nt] + k);
        else b[nt][s].raw = u32x4{0u, 0u, 0u, 0u};
      }
    }
  };

  // prologue: weight chunks 0..PB-1 and activation chunks 0, 1 are requested; chunk 0 reaches LDS
#pragma unroll
  for (int u = 0; u < PB; ++u)
    if (u < n_chunks) load_b(breg[u], u);
  if (n_chunks > 0) {
    load_a(areg[0], 0);
    if (n_chunks > 1) load_a(areg[1], 1);
    store_a(areg[0], 0);
  }
  __syncthreads();

  for (int base = 0; base < n_chunks; base += RING) {
#pragma unroll
    for (int u = 0; u < RING; ++u) {
      const int c = base + u;
      if (c >= n_chunks) break;
      // requests first: activation chunk c+2 (its registers were emptied into LDS one iteration ago)
      // and weight chunk c+PB
      if (c + 2 < n_chunks) load_a(areg[u & 1], c + 2);
      if (c + PB < n_chunks) load_b(breg[(u + PB) % RING], c + PB);
      const unsigned char* abuf = lds[u & 1];
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          Frag<T> af;
          af.raw = *reinterpret_cast<const u32x4*>(&abuf[(mt * 16 + r) * kRowStride + (s * 4 + g) * 16]);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) mfma16(acc[mt][nt], af, breg[u][nt][s]);
        }
      }
      // activation chunk c+1 was requested one iteration ago: its latency is behind us
      if (c + 1 < n_chunks) store_a(areg[(u + 1) & 1], (u + 1) & 1);
      __syncthreads();
    }
  }

  float* out = P + (size_t)blockIdx.y * split_stride;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int col = n_base + nt * 16 + r;
      if (col >= N) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = row0 + mt * 16 + g * 4 + j;
        if (row < m) out[(size_t)row * ldp + col] = acc[mt][nt][j];
      }
    }
}

template <typename T, int MT, int NT, int RING>
hipError_t launch_t(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                    size_t split_stride, int m, int N, int K, hipStream_t st) {
  dim3 grid((N + 64 * NT - 1) / (64 * NT), pl.splits, pl.row_chunks);
  hipLaunchKernelGGL((gemm_rows_kernel<T, MT, NT, RING>), grid, dim3(kThreads), 0, st, (const T*)A, lda, (const T*)W,
                     ldw, P, ldp, split_stride, m, N, K, pl.k_per_split);
  return hipGetLastError();
}

template <typename T, int NT, int RING>
hipError_t launch_mt(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                     size_t ss, int m, int N, int K, hipStream_t st) {
  switch (pl.mt) {
    case 1: return launch_t<T, 1, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 2: return launch_t<T, 2, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 3: return launch_t<T, 3, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 4: return launch_t<T, 4, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 5: return launch_t<T, 5, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 6: return launch_t<T, 6, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 7: return launch_t<T, 7, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    case 8: return launch_t<T, 8, NT, RING>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
  }
  return hipErrorInvalidValue;
}

template <typename T>
hipError_t launch_nt(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                     size_t ss, int m, int N, int K, hipStream_t st) {
  if (pl.nt == 1) {
    if (pl.ring == 4) return launch_mt<T, 1, 4>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
    return launch_mt<T, 1, 2>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
  }
  if (pl.ring == 4) return launch_mt<T, 2, 4>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
  return launch_mt<T, 2, 2>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st);
}

}  // namespace

GemmPlan plan_gemm(int dtype, int m, int N, int K, bool single_split) {
  const Tunables& t = tunables();
  GemmPlan pl;
  const int tiles = (m + 15) / 16;
  pl.mt = tiles <= 8 ? (tiles < 1 ? 1 : tiles) : 8;
  pl.row_chunks = tiles <= 8 ? 1 : (tiles + 7) / 8;
  pl.nt = N > t.gemm_nt_big_n ? 2 : 1;
  pl.ring = t.gemm_ring == 4 ? 4 : 2;
  const int kc = dtype == kBF16 ? 128 : 64;                       // elements per 256-byte chunk
  const int n_blocks = (N + 64 * pl.nt - 1) / (64 * pl.nt);
  const int chunks = (K + kc - 1) / kc;
  int splits = 1;
  while (!single_split && splits < t.gemm_max_splits && n_blocks * pl.row_chunks * splits < t.gemm_target_wgs &&
         chunks / (splits * 2) >= 2)
    splits *= 2;
  const int chunks_per_split = (chunks + splits - 1) / splits;
  pl.k_per_split = chunks_per_split * kc;
  pl.splits = (K + pl.k_per_split - 1) / pl.k_per_split;
  return pl;
}

hipError_t launch_gemm(int dtype, const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P,
                       int ldp, size_t split_stride, int m, int N, int K, hipStream_t st) {
  if (m <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  const int e = dtype == kBF16 ? 8 : 4;
  // 16-byte fragments: the contraction length and both pitches must be whole fragments
  if (K % e || lda % e || ldw % e) return hipErrorInvalidValue;
  if (pl.mt * 16 * pl.row_chunks < m || (size_t)pl.k_per_split * pl.splits < (size_t)K) return hipErrorInvalidValue;
  if (split_stride < (size_t)m * ldp || ldp < N) return hipErrorInvalidValue;
  if (dtype == kBF16) return launch_nt<bf16>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st);
  return launch_nt<float>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st);
}

}  // namespace d2c
