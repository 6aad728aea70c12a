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
//   * the contraction axis can be split over several workgroups; every split writes
//     its own fp32 partial and the consumer kernel sums the partials in a fixed order
//     (deterministic, no atomics);
//   * more than 128 rows (step 0, select-all mode) are covered by several row chunks.
//     The grid is one-dimensional and workgroup ids are dealt round-robin to the 8
//     XCDs, each with its own L2: the mapping below gives the row chunks of one weight
//     tile consecutive slots of the SAME XCD, so the tile comes from HBM once and the
//     other chunks hit it in L2.
#include "common.h"
#include "internal.h"

namespace d2c {

namespace {

constexpr int kChunkBytes = 256;                 // bytes of one row in one chunk
constexpr int kRowStride = kChunkBytes + 16;     // LDS row pitch: 16-byte skew, conflict-free 16-byte reads
constexpr int kSteps = 4;                        // matrix-core steps per chunk
constexpr int kSuperRows = 8, kSuperCols = 4;    // many rows: block of workgroups that share an XCD's L2

// RING = number of weight chunks a wave keeps in registers (one being consumed, RING-1 in flight).
// MODE: 0 = W row-major [N, K]; 1 = W pre-tiled; 2 = W pre-tiled with gate and up tiles interleaved and the
// SwiGLU applied in the epilogue (single k split, one column tile per wave): act[m, N/2] = T(silu(g) * u).
enum { kRowMajor = 0, kPre = 1, kPreSwiglu = 2 };

template <typename T, int MT, int NT, int WAVES, int MODE>
__global__ __launch_bounds__(WAVES * 64) void gemm_rows_kernel(
    const T* __restrict__ A, int lda, const T* __restrict__ W, int ldw, float* __restrict__ P, int ldp,
    size_t split_stride, int m, int N, int K, int k_per_split, int n_blocks, int n_splits, int row_chunks, int rot_mul,
    T* __restrict__ act) {
  constexpr bool PRE = MODE != kRowMajor;
  static_assert(MODE != kPreSwiglu || NT % 2 == 0 || WAVES % 2 == 0, "the SwiGLU epilogue pairs neighbouring waves");
  constexpr int RING = 2;
  constexpr int kThreads = WAVES * 64;
  constexpr int kAFrags = MT * 256;                              // 16-byte fragments of one activation chunk
  constexpr int AI = (kAFrags + kThreads - 1) / kThreads;        // of which one thread moves this many
  // workgroup id -> (weight tile, row chunk): id % 8 is the XCD, within an XCD the row chunk varies fastest
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  int tile, bz;
  if constexpr (NT >= 4) {
    // Many rows: the 32 workgroups that run on an XCD at one time form a block of kSuperRows row chunks x
    // kSuperCols weight tiles, so that what its L2 has to bring in per k-step (8 x 128 activation rows +
    // 4 x 256 weight rows) is less than half of that of 32 row chunks of one weight tile.
    const int n_row_st = (row_chunks + kSuperRows - 1) / kSuperRows;
    const int st = slot / (kSuperRows * kSuperCols), w = slot % (kSuperRows * kSuperCols);
    bz = (st % n_row_st) * kSuperRows + w % kSuperRows;
    tile = ((st / n_row_st) * kSuperCols + w / kSuperRows) * 8 + xcd;
    if (bz >= row_chunks) return;
  } else {
    tile = (slot / row_chunks) * 8 + xcd;
    bz = slot % row_chunks;
  }
  if (tile >= n_blocks * n_splits) return;       // padding (whole workgroup leaves)
  const int by = tile / n_blocks, bx = tile - by * n_blocks;
  constexpr int E = Frag<T>::kElems;
  constexpr int KS = Frag<T>::kStep;
  constexpr int KC = kSteps * KS;                // elements per chunk (= 256 bytes)
  constexpr int PB = RING - 1;                   // prefetch distance of the weight stream, in chunks
  __shared__ __attribute__((aligned(16))) unsigned char lds[2][MT * 16 * kRowStride];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int row0 = bz * (MT * 16);
  const int k_begin = by * k_per_split;
  const int k_end = min(K, k_begin + k_per_split);
  const int n_base = (bx * WAVES + wave) * (16 * NT);
  const int n_chunks = (k_end - k_begin + KC - 1) / KC;

  // this lane's weight rows (clamped: out-of-range columns are computed on a valid row and dropped).
  // PRE: W is the pre-tiled copy (see preshuffle_kernel): [16-row tile][256-byte chunk][step][lane][16 B],
  // ldw = chunks per tile; wrow then points at this lane's 16 bytes of step 0 of the tile's chunk 0.
  constexpr int kBlockElems = 16 * KC;           // elements of one 16-row x 256-byte block (4 KB)
  const T* wrow[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (PRE) {
      const int t16 = min((n_base + nt * 16) / 16, (N + 15) / 16 - 1);
      wrow[nt] = W + (size_t)t16 * ldw * kBlockElems + lane * E;
    } else {
      int n = min(n_base + nt * 16 + r, N - 1);
      wrow[nt] = W + (size_t)n * ldw;
    }
  }

  Frag<T> areg[2][AI];                 // areg[c & 1]: activation chunk c on its way from global memory to LDS
  Frag<T> breg[RING][NT][kSteps];      // breg[c % RING]: weight chunk c
  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // The loop below has no conditional loads or stores.  A load under a branch makes the compiler wait
  // for ALL outstanding loads before the next use, which would drain the prefetch ring every iteration;
  // so addresses are clamped instead: rows >= m read row m-1 (their accumulators are never stored),
  // chunks past the end re-read the last chunk (an L2 hit, never used), and the weight fragments of the
  // last chunk's tail are masked to zero where they are consumed.
  const int last_row = m - 1;
  const int last_chunk = n_chunks - 1;
  // Workgroups walk their k-range from different starting chunks (a rotation by a multiple of the
  // column-block index), so that at one moment they do not all ask for the same offsets within a row.
  const int rot = n_chunks > 0 ? (int)(((unsigned)bx * (unsigned)rot_mul) % (unsigned)n_chunks) : 0;
  auto chunk_k = [&](int chunk) {
    int p = min(chunk, last_chunk) + rot;
    if (p >= n_chunks) p -= n_chunks;
    return k_begin + p * KC;
  };
  auto load_a = [&](Frag<T> (&a)[AI], int chunk) {
    const int kc = chunk_k(chunk);
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      // fragment id in the chunk: row f/16, 16-byte column f%16; ids past the end repeat the last one
      const int f = min(tid + i * kThreads, kAFrags - 1);
      const int row = min(row0 + (f >> 4), last_row);
      const int k = min(kc + (f & 15) * E, k_end - E);
      a[i].raw = ld16(A + (size_t)row * lda + k);
    }
  };
  auto store_a = [&](const Frag<T> (&a)[AI], int buf) {
#pragma unroll
    for (int i = 0; i < AI; ++i) {
      const int f = min(tid + i * kThreads, kAFrags - 1);
      *reinterpret_cast<u32x4*>(&lds[buf][(f >> 4) * kRowStride + (f & 15) * 16]) = a[i].raw;
    }
  };
  // One column tile per wave means one row chunk: every weight byte is read by exactly one workgroup of the
  // launch, so its loads carry the streaming hint and leave the L2 to the activations and partial sums.
  auto ldw16 = [](const T* p) {
    if constexpr (NT == 1) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    else return ld16(p);
  };
  auto load_b = [&](Frag<T> (&b)[NT][kSteps], int chunk) {
    const int kc = chunk_k(chunk);
    if (PRE) {
      // one instruction = 1 KB contiguous: whole cache lines, no clamping (the copy is zero-padded)
      const size_t off = (size_t)(kc / KC) * kBlockElems;
#pragma unroll
      for (int s = 0; s < kSteps; ++s)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[nt][s].raw = ldw16(wrow[nt] + off + s * 64 * E);
    } else {
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const int k = min(kc + s * KS + g * E, k_end - E);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) b[nt][s].raw = ldw16(wrow[nt] + k);
      }
    }
  };

  if (n_chunks <= 0) return;
  if constexpr (NT >= 4) {
    // Many rows: 128 x 64 outputs per wave, one wave per SIMD.  Nothing else hides latencies here, so the
    // loop is pipelined by hand and the scheduler is told to keep the interleaving:
    //   * the activation fragments are read from LDS three matrix-core groups ahead of their use;
    //   * the weight registers of a k-step are refilled as soon as that step is done, with the same step
    //     of the chunk two ahead (two chunks of flight time: an L2 miss costs more than one);
    //   * the next activation chunk is requested at the top of an iteration and stored behind it.
    // The launcher guarantees whole chunks and an even number of them per split: nothing to mask.
    static_assert(RING == 2, "the wide loop keeps two weight chunks");
    constexpr int NI = kSteps * MT;
    auto load_b_step = [&](Frag<T> (&b)[NT][kSteps], int chunk, int step) {
      const size_t off = PRE ? (size_t)(chunk_k(chunk) / KC) * kBlockElems + step * 64 * E
                             : (size_t)(chunk_k(chunk) + step * KS + g * E);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) b[nt][step].raw = ld16(wrow[nt] + off);
    };
    load_a(areg[0], 0);
    load_b(breg[0], 0);
    load_b(breg[1], 1);
    store_a(areg[0], 0);
    __syncthreads();
    for (int base = 0; base < n_chunks; base += 2) {
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int c = base + u;
        load_a(areg[0], c + 1);
        __builtin_amdgcn_sched_barrier(0);
        const unsigned char* abuf = lds[u];
        auto read_af = [&](int i) {
          Frag<T> f;
          f.raw = *reinterpret_cast<const u32x4*>(&abuf[((i % MT) * 16 + r) * kRowStride + ((i / MT) * 4 + g) * 16]);
          return f;
        };
        Frag<T> af[4];
        af[0] = read_af(0);
        af[1] = read_af(1);
        af[2] = read_af(2);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) mfma16(acc[i % MT][nt], af[i % 4], breg[u][nt][i / MT]);
          if (i + 3 < NI) af[(i + 3) % 4] = read_af(i + 3);
          if (i % MT == MT - 1) load_b_step(breg[u], c + 2, i / MT);
        }
        __builtin_amdgcn_sched_group_barrier(0x100, 3, 0);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, NT, 0);                          // NT matrix-core instructions
          if (i + 3 < NI) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);           // one LDS read
          if (i % MT == MT - 1) __builtin_amdgcn_sched_group_barrier(0x020, NT, 0);    // the k-step's refill
        }
        __builtin_amdgcn_sched_barrier(0);
        store_a(areg[0], u ^ 1);
        __syncthreads();
      }
    }
  } else {
  // prologue: weight chunks 0..PB-1 and activation chunks 0, 1 are requested; chunk 0 reaches LDS
#pragma unroll
  for (int u = 0; u < PB; ++u) load_b(breg[u], u);
  load_a(areg[0], 0);
  load_a(areg[1], 1);
  store_a(areg[0], 0);
  __syncthreads();

  for (int base = 0; base < n_chunks; base += RING) {
#pragma unroll
    for (int u = 0; u < RING; ++u) {
      // no early exit: iterations past the last chunk (at most RING-1) re-read it and contribute zero,
      // which keeps the RING iterations one basic block that the scheduler can interleave freely
      const int c = base + u;
      // requests first: activation chunk c+2 (its registers were emptied into LDS one iteration ago)
      // and weight chunk c+PB
      load_a(areg[u & 1], c + 2);
      load_b(breg[(u + PB) % RING], c + PB);
      __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of this iteration's arithmetic
      const unsigned char* abuf = lds[u & 1];
      const int kc = chunk_k(c);
#pragma unroll
      for (int s = 0; s < kSteps; ++s) {
        const unsigned keep = (c < n_chunks && kc + s * KS + g * E < k_end) ? 0xffffffffu : 0u;   // zero in the tail of the last chunk and past it
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          Frag<T> af;
          af.raw = *reinterpret_cast<const u32x4*>(&abuf[(mt * 16 + r) * kRowStride + (s * 4 + g) * 16]);
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
            Frag<T> bf;
            bf.raw = breg[u][nt][s].raw & u32x4{keep, keep, keep, keep};
            mfma16(acc[mt][nt], af, bf);
          }
        }
      }
      // activation chunk c+1 was requested one iteration ago: its latency is behind us
      store_a(areg[(u + 1) & 1], (u + 1) & 1);
      __syncthreads();
    }
  }

  }   // narrow loop

  if (MODE == kPreSwiglu && NT % 2 == 0) {
    // Column tiles alternate gate, up, gate, up ..: with an even number of tiles per wave each pair sits in one wave
    const int F = N >> 1;
#pragma unroll
    for (int p = 0; p < NT / 2; ++p) {
      const int col = ((n_base >> 5) + p) * 16 + r;             // n_base = 32 * (first hidden tile of the wave)
      if (col >= F) continue;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int row = row0 + mt * 16 + g * 4 + j;
          const float gv = acc[mt][2 * p][j];
          if (row < m)
            act[(size_t)row * F + col] = from_f32<T>(gv / (1.0f + expf(-gv)) * acc[mt][NT > 1 ? 2 * p + 1 : 0][j]);
        }
    }
    return;
  }
  if (MODE == kPreSwiglu) {
    // Column tiles alternate gate, up, gate, up ..: wave 2p holds the gate values and wave 2p+1 the up
    // values of the same 16 hidden columns.  The odd wave hands its accumulators over through LDS (the
    // activation buffers are idle: the loop ended on a barrier), the even wave applies the gate.
    f32x4* xch = reinterpret_cast<f32x4*>(&lds[0][0]);          // [WAVES/2][MT][64]
    const int pair = wave >> 1;
    if (wave & 1) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) xch[(pair * MT + mt) * 64 + lane] = acc[mt][0];
    }
    __syncthreads();
    if (wave & 1) return;
    const int F = N >> 1;
    const int col = (n_base >> 5) * 16 + r;                     // n_base = 32 * (hidden tile)
    if (col >= F) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const f32x4 u = xch[(pair * MT + mt) * 64 + lane];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int row = row0 + mt * 16 + g * 4 + j;
        const float gv = acc[mt][0][j];
        if (row < m) act[(size_t)row * F + col] = from_f32<T>(gv / (1.0f + expf(-gv)) * u[j]);
      }
    }
    return;
  }
  float* out = P + (size_t)by * split_stride;
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

template <typename T, int MT, int NT, int WAVES, int MODE>
hipError_t launch_t(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                    size_t split_stride, int m, int N, int K, hipStream_t st, void* act) {
  const int cols = 16 * NT * WAVES;
  const int n_blocks = (N + cols - 1) / cols;
  const int groups = (n_blocks * pl.splits + 7) / 8;            // weight tiles are dealt to the XCDs in groups of 8
  dim3 grid(groups * 8 * pl.row_chunks);
  if (NT >= 4)
    grid.x = 8 * ((groups + kSuperCols - 1) / kSuperCols) * ((pl.row_chunks + kSuperRows - 1) / kSuperRows) *
             (kSuperRows * kSuperCols);
  hipLaunchKernelGGL((gemm_rows_kernel<T, MT, NT, WAVES, MODE>), grid, dim3(WAVES * 64), 0, st, (const T*)A, lda,
                     (const T*)W, ldw, P, ldp, split_stride, m, N, K, pl.k_per_split, n_blocks, pl.splits,
                     pl.row_chunks, pl.rot, (T*)act);
  return hipGetLastError();
}

template <typename T, int NT, int WAVES, int MODE>
hipError_t launch_mt(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                     size_t ss, int m, int N, int K, hipStream_t st, void* act) {
  switch (pl.mt) {
    case 1: return launch_t<T, 1, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 2: return launch_t<T, 2, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 3: return launch_t<T, 3, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 4: return launch_t<T, 4, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 5: return launch_t<T, 5, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 6: return launch_t<T, 6, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 7: return launch_t<T, 7, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    case 8: return launch_t<T, 8, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    default: break;
  }
  // 129-192 rows in one row chunk (bf16, one column tile per wave, 8 waves): even tile counts only
  if constexpr (sizeof(T) == 2 && NT == 1 && WAVES == 8) {
    switch (pl.mt) {
      case 10: return launch_t<T, 10, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
      case 12: return launch_t<T, 12, NT, WAVES, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
      default: break;
    }
  }
  return hipErrorInvalidValue;
}

template <typename T, int MODE>
hipError_t launch_nt(const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P, int ldp,
                     size_t ss, int m, int N, int K, hipStream_t st, void* act) {
  if (pl.nt == 1) {
    if (pl.waves == 8) return launch_mt<T, 1, 8, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    if (pl.waves == 6) return launch_mt<T, 1, 6, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    if (pl.waves == 10) return launch_mt<T, 1, 10, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
    if (pl.waves == 7) {
      if constexpr (MODE != kPreSwiglu) return launch_mt<T, 1, 7, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
      return hipErrorInvalidValue;
    }
    return launch_mt<T, 1, 4, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
  }
  if (pl.nt == 4) {
    // 128 rows x 64 columns per wave, one wave per SIMD: only for full row chunks in bf16
    if constexpr (sizeof(T) == 2) {
      const int kc = 256 / (int)sizeof(T);
      if (pl.waves == 4 && K % kc == 0 && pl.k_per_split % (2 * kc) == 0 && K % (2 * kc) == 0) {
        if (pl.mt == 8) return launch_t<T, 8, 4, 4, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
        if (pl.mt == 7) return launch_t<T, 7, 4, 4, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
        if (pl.mt == 6) return launch_t<T, 6, 4, 4, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
      }
    }
    return hipErrorInvalidValue;
  }
  if (pl.waves == 8) return launch_mt<T, 2, 8, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
  return launch_mt<T, 2, 4, MODE>(pl, A, lda, W, ldw, P, ldp, ss, m, N, K, st, act);
}

// One 16-byte fragment per thread: dst block (tile t, chunk c) slot (step s, lane) <- src row
// row_of(t) + lane%16, bytes c*256 + s*64 + (lane/16)*16; rows >= N and bytes >= the row length read as zero.
// half > 0 (gate/up interleave, half % 16 == 0): dst tile 2j is src tile j, dst tile 2j+1 is the tile
// that starts at src row half + 16j.
__global__ __launch_bounds__(256) void preshuffle_kernel(const unsigned char* __restrict__ src, size_t src_pitch_bytes,
                                                         int N, size_t row_bytes, int chunks, int half,
                                                         unsigned char* __restrict__ dst, size_t n_frags) {
  const size_t f = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (f >= n_frags) return;
  const int lane = (int)(f & 63), s = (int)((f >> 6) & 3);
  const size_t block = f >> 8;
  const int c = (int)(block % chunks);
  const size_t t = block / chunks;
  const size_t row0 = half > 0 ? (t >> 1) * 16 + ((t & 1) ? (size_t)half : 0) : t * 16;
  const size_t row = row0 + (lane & 15);
  const size_t byte = (size_t)c * 256 + s * 64 + (lane >> 4) * 16;
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row < (size_t)N && byte + 16 <= row_bytes) v = ld16(src + row * src_pitch_bytes + byte);
  *reinterpret_cast<u32x4*>(dst + f * 16) = v;
}

}  // namespace

GemmPlan plan_gemm(const Tunables& t, int dtype, int m, int N, int K, bool single_split) {
  GemmPlan pl;
  const int tiles = (m + 15) / 16;
  pl.mt = tiles <= 8 ? (tiles < 1 ? 1 : tiles) : 8;
  pl.row_chunks = tiles <= 8 ? 1 : (tiles + 7) / 8;
  // 129-192 rows in bf16: still one row chunk (10 or 12 row tiles).  Two row chunks pull every weight tile
  // through the L1 of two compute units, and that pull rate, not HBM, is what bounds the kernel; beyond 12
  // row tiles the LDS reads of one column tile per wave cost more than the second pull (measured per layer
  // at the LLaDA shape: 140 rows 170 vs 196 us, 166 rows 192 vs 200 us, 200 rows 214 vs 200 us).
  if (tiles > 8 && tiles <= 12 && dtype == kBF16 && t.gemm_tall_chunk && (t.gemm_waves == 0 || t.gemm_waves == 8)) {
    pl.mt = tiles + (tiles & 1);
    pl.row_chunks = 1;
  }
  // two column tiles per wave halve the LDS reads per matrix-core step: a gain once there are several
  // row chunks (the kernel is LDS- and L2-bound there), a loss for a handful of rows (fewer waves in flight)
  pl.nt = (N > t.gemm_nt_big_n || pl.row_chunks > 1) ? 2 : 1;
  // several row chunks in bf16: four column tiles per wave and one wave per SIMD (128 x 64 outputs per wave)
  // halve the LDS reads per matrix-core step once more
  const bool wide = pl.row_chunks > 1 && m >= t.gemm_wide_min_rows && dtype == kBF16 && t.gemm_wide_tiles &&
                    K % 256 == 0;                       // needs an even number of whole chunks
  if (wide) pl.nt = 4;
  pl.rot = t.gemm_rot;
  // 8 waves share one activation chunk in LDS: fewer, fatter workgroups (about 1.5 per compute unit) with
  // fewer k splits measured faster than 4-wave groups at every projection shape of the two models
  // (7 waves only where no gated epilogue can follow: it pairs neighbouring waves)
  pl.waves = wide ? 4
             : (t.gemm_waves == 4 || t.gemm_waves == 6 || t.gemm_waves == 10 || (t.gemm_waves == 7 && !single_split))
                 ? t.gemm_waves
                 : 8;
  const int kc = dtype == kBF16 ? 128 : 64;                       // elements per 256-byte chunk
  const int chunks = (K + kc - 1) / kc;
  const int max_splits = single_split ? 1 : t.gemm_max_splits;
  auto blocks_of = [&](int waves) { return (N + 16 * pl.nt * waves - 1) / (16 * pl.nt * waves); };
  auto splits_for = [&](int waves) {
    int s = 1;
    while (s < max_splits && blocks_of(waves) * (waves / 4) * pl.row_chunks * s < t.gemm_target_wgs && chunks / (s * 2) >= 2)
      s *= 2;
    return s;
  };
  int splits = splits_for(pl.waves);
  // Few rows (one row chunk, one column tile per wave): the kernel streams fastest when every compute unit
  // holds one workgroup of equal size, so the waves per workgroup and the split count are chosen together.
  // Cost of a shape = rounds of workgroups over the 256 units x (waves x chunks per split), +4 % per
  // additional split (its partial is written and read again).  Measured at 48-69 rows: LLaDA QKV 25.1 ->
  // 22.5 us (6 waves x 2 splits = 256 workgroups instead of 8 x 2 = 192), Dream gate/up 68.6 -> 51.5 us
  // (10 waves = 237 workgroups in one round instead of 296 in two); 4-wave workgroups were slower at every
  // shape and are not searched.
  constexpr int kUnits = 256;
  if (pl.nt == 1 && pl.row_chunks == 1) {
    double best = 1e30;
    for (int w : {8, 6, 10, 7}) {                                 // 8 first: ties keep the 8-wave shape
      if (t.gemm_waves != 0 && w != pl.waves) continue;
      if (w == 7 && single_split) continue;
      if (pl.mt > 8 && w != 8) continue;                          // the tall chunk fits the registers of 8 waves only
      for (int s = 1; s <= max_splits; s *= 2) {
        const int cps = (chunks + s - 1) / s;
        if (s > 1 && cps < 2) break;
        const int eff = (chunks + cps - 1) / cps;
        const int wgs = blocks_of(w) * eff;
        const int rounds = (wgs + kUnits - 1) / kUnits;
        const double cost = (double)rounds * w * cps * (1.0 + 0.04 * (eff - 1));
        if (cost < best * 0.999) {
          best = cost;
          pl.waves = w;
          splits = s;
        }
      }
    }
  }
  if (wide) {
    // Rows per workgroup: 8 row tiles unless fewer do the same job better.  Measured at the LLaDA widths,
    // 288-2048 rows: (a) fewer tiles in the SAME number of row chunks are always a gain (less matrix-core and
    // LDS work per weight pull: 288 rows as 3 x 6 tiles -14 %); (b) MORE row chunks gain only when their count
    // becomes a multiple of 8, the rows of the block of workgroups that shares an XCD's L2 (700 rows as
    // 8 x 6 tiles instead of 6 x 8: -16 %; 856 rows as 8 x 7 instead of 7 x 8: -7 %; 1500 rows as 16 x 6
    // instead of 12 x 8: -7 %), every other count lost 10-40 %.
    const int rc8 = (tiles + 7) / 8;
    int mt = 8;
    if (t.gemm_wide_mt != 0) {
      mt = t.gemm_wide_mt;
    } else {
      if (rc8 % kSuperRows != 0)
        for (int c : {7, 6})
          if (mt == 8 && ((tiles + c - 1) / c) % kSuperRows == 0) mt = c;
      if (mt == 8)
        for (int c : {6, 7})
          if (mt == 8 && (tiles + c - 1) / c == rc8) mt = c;
    }
    pl.mt = mt;
    pl.row_chunks = (tiles + mt - 1) / mt;
  }
  if (wide && !single_split) {
    // the same count of rounds, with +7 % per additional split (the partials are as large as the output and
    // there are hundreds of rows of them)
    double best = 1e30;
    for (int s = 1; s <= max_splits; s *= 2) {
      int cps = (chunks + s - 1) / s;
      cps += cps & 1;                                             // the wide loop takes chunks in pairs
      if (s > 1 && cps < 4) break;
      const int eff = (chunks + cps - 1) / cps;
      const int wgs = blocks_of(pl.waves) * pl.row_chunks * eff;
      const double cost = (double)((wgs + kUnits - 1) / kUnits) * cps * (1.0 + 0.07 * (eff - 1));
      if (cost < best * 0.999) {
        best = cost;
        splits = s;
      }
    }
  }
  int chunks_per_split = (chunks + splits - 1) / splits;
  if (wide) chunks_per_split += chunks_per_split & 1;
  pl.k_per_split = chunks_per_split * kc;
  pl.splits = (K + pl.k_per_split - 1) / pl.k_per_split;
  return pl;
}

hipError_t launch_gemm(int dtype, const GemmPlan& pl, const void* A, int lda, const void* W, int ldw, float* P,
                       int ldp, size_t split_stride, int m, int N, int K, hipStream_t st, bool pre) {
  if (m <= 0 || N <= 0 || K <= 0) return hipErrorInvalidValue;
  const int e = dtype == kBF16 ? 8 : 4;
  // 16-byte fragments: the contraction length and both pitches must be whole fragments
  if (K % e || lda % e || (!pre && ldw % e)) return hipErrorInvalidValue;
  if (pl.mt * 16 * pl.row_chunks < m || (size_t)pl.k_per_split * pl.splits < (size_t)K) return hipErrorInvalidValue;
  if (split_stride < (size_t)m * ldp || ldp < N) return hipErrorInvalidValue;
  if (pre) {
    // ldw = chunks per tile of the pre-tiled copy; every split must start on a chunk boundary
    const int kc = dtype == kBF16 ? 128 : 64;
    if (ldw != (K + kc - 1) / kc || pl.k_per_split % kc) return hipErrorInvalidValue;
    if (dtype == kBF16)
      return launch_nt<bf16, kPre>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st, nullptr);
    return launch_nt<float, kPre>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st, nullptr);
  }
  if (dtype == kBF16)
    return launch_nt<bf16, kRowMajor>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st, nullptr);
  return launch_nt<float, kRowMajor>(pl, A, lda, W, ldw, P, ldp, split_stride, m, N, K, st, nullptr);
}

hipError_t launch_gemm_swiglu(int dtype, const GemmPlan& pl, const void* A, int lda, const void* W, int ldw,
                              void* act, int F, int m, int K, hipStream_t st) {
  if (m <= 0 || F <= 0 || K <= 0 || F % 16) return hipErrorInvalidValue;
  const int e = dtype == kBF16 ? 8 : 4, kc = dtype == kBF16 ? 128 : 64;
  if (K % e || lda % e || ldw != (K + kc - 1) / kc) return hipErrorInvalidValue;
  if (pl.splits != 1 || pl.mt * 16 * pl.row_chunks < m || pl.k_per_split < K)
    return hipErrorInvalidValue;
  if (dtype == kBF16)
    return launch_nt<bf16, kPreSwiglu>(pl, A, lda, W, ldw, nullptr, 0, 0, m, 2 * F, K, st, act);
  return launch_nt<float, kPreSwiglu>(pl, A, lda, W, ldw, nullptr, 0, 0, m, 2 * F, K, st, act);
}

size_t preshuffled_bytes(int N, int K, int dtype) {
  const size_t row_bytes = (size_t)K * dtype_size(dtype);
  return (size_t)((N + 15) / 16) * ((row_bytes + 255) / 256) * 4096;
}

hipError_t launch_preshuffle(int dtype, const void* W, int ldw, int N, int K, void* dst, hipStream_t st,
                             int interleave_half) {
  if (N <= 0 || K <= 0 || ldw < K) return hipErrorInvalidValue;
  if (interleave_half < 0 || interleave_half % 16 || (interleave_half && N != 2 * interleave_half))
    return hipErrorInvalidValue;
  const size_t ts = dtype_size(dtype);
  if ((size_t)K * ts % 16 || (size_t)ldw * ts % 16) return hipErrorInvalidValue;
  const size_t n_frags = preshuffled_bytes(N, K, dtype) / 16;
  const int chunks = (int)(((size_t)K * ts + 255) / 256);
  hipLaunchKernelGGL(preshuffle_kernel, dim3((unsigned)((n_frags + 255) / 256)), dim3(256), 0, st,
                     (const unsigned char*)W, (size_t)ldw * ts, N, (size_t)K * ts, chunks, interleave_half,
                     (unsigned char*)dst, n_frags);
  return hipGetLastError();
}

}  // namespace d2c
