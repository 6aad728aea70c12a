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
#include <cstring>

#include "common.h"
#include "internal.h"

namespace d2c {
namespace {

constexpr int kThreads = 256;
constexpr int kBlockKeys = 64;
// rows of the unnormalised probabilities are padded by one block: the pitch between heads and rows is then no
// power of two (the head average reads the same piece of every head at once)
constexpr int kPtildePad = 64;

// low halves of (a, b) / high halves of (a, b) in one register: one byte-permute instruction each
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }
// two floats -> one register of two bf16 (round to nearest even): a single packed conversion
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{a, b}, bf16x2));
}

// One sequence of a batched launch (blockIdx.y picks it): its tensors, sizes, launch plan and scratch pieces.
struct SeqArgs {
  const bf16 *q, *k_cache, *v_cache;
  bf16* out;
  float *lse, *attn_avg, *o_part, *ml_part, *refblk;
  bf16* ptilde;
  int m, L, keys_per_split, n_splits, q_blocks, avg_blocks;
};
constexpr int kMaxBatch = 8;             // sequences per launch (the arguments travel by value)
struct BatchArgs {
  SeqArgs seq[kMaxBatch];
};

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

// EMIT: the kernel also writes what the head average needs, so that no second pass over Q and K is run:
// the unnormalised probabilities of every block exactly as they enter the matrix cores (bf16,
// ptilde [H, m, Lp], Lp = L rounded up to whole blocks; inside a block of 64 keys the values of a row sit in
// operand order: 16-byte piece (ks, g) holds keys 32ks + 4g .. +3, then 32ks + 16 + 4g .. +3) and the base-2
// reference each block was taken against (refblk [H, blocks, m]).  The head-average kernel turns them into normalised rows once the rows'
// log-sum-exp is known: p = ptilde * 2^(refblk - lse2).
//
// WAVES = 4 or 8 waves per workgroup, each owning 16*QT queries; with 8 waves two waves share a SIMD, so that
// one wave's matrix-core phase runs beside the other's vector phase (a single wave runs its phases one after
// the other), and a K/V block staged once serves twice as many queries.
template <int DH, int QT, int WAVES, bool EMIT>
__global__ __launch_bounds__(WAVES * 64) void attn_tiled_fwd_kernel(const BatchArgs batch, int n_heads, int n_kv_heads,
                                                                    float scale) {
  static_assert(WAVES == 4 || WAVES == 8, "4 or 8 waves");
  constexpr int NS = DH / 32;            // contraction steps of K Q^T
  constexpr int ND = DH / 16;            // head-dim tiles of O^T
  constexpr int NB = DH / 64;            // 64-wide head-dim blocks (one V staging unit covers 64)
  constexpr int WH = WAVES / 4;          // waves that share the staging of one key tile
  constexpr int KF = NS / WH;            // K fragments a lane stages per block
  constexpr int VA = 2 / WH;             // 16-key tiles of its V unit a lane stages
  __shared__ u32x4 k_lds[2][4 * NS * 64];      // [key tile a][step s][lane]
  __shared__ u32x4 v_lds[2][ND * 2 * 64];      // [head-dim tile][32-key step][slot]; slot = lane ^ (tile & 3)

  const SeqArgs& sq = batch.seq[blockIdx.y];
  const bf16* __restrict__ q = sq.q;
  const bf16* __restrict__ k_cache = sq.k_cache;
  const bf16* __restrict__ v_cache = sq.v_cache;
  bf16* __restrict__ out = sq.out;
  float* __restrict__ lse = sq.lse;
  float* __restrict__ o_part = sq.o_part;
  float* __restrict__ ml_part = sq.ml_part;
  bf16* __restrict__ ptilde = sq.ptilde;
  float* __restrict__ refblk = sq.refblk;
  const int m = sq.m, L = sq.L, keys_per_split = sq.keys_per_split, n_splits = sq.n_splits, q_blocks = sq.q_blocks;
  const TileId id = tile_of(blockIdx.x, q_blocks, n_heads, n_splits);
  if (!id.valid || id.qb >= q_blocks) return;          // the grid is sized for the largest sequence of the batch
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int r = lane & 15, g = lane >> 4;
  const int head = id.head;
  const int kvh = head / (n_heads / n_kv_heads);
  const int dq = n_heads * DH;
  const size_t kv_pitch = (size_t)n_kv_heads * DH;
  const bf16* kbase = k_cache + (size_t)kvh * DH;
  const bf16* vbase = v_cache + (size_t)kvh * DH;
  const int q0 = id.qb * (16 * QT * WAVES) + wave * (16 * QT);
  const int key_lo = id.split * keys_per_split;
  const int key_hi = min(L, key_lo + keys_per_split);
  const int n_blocks = (key_hi - key_lo + kBlockKeys - 1) / kBlockKeys;      // >= 1 by the launch plan
  const int n_blk_total = (L + kBlockKeys - 1) / kBlockKeys;
  const int Lp = n_blk_total * kBlockKeys + kPtildePad;                      // row pitch of ptilde

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
  // iteration, stored behind its arithmetic.  Key tile kt = wave % 4 of K: its NS fragments (with 8 waves,
  // wave / 4 picks which half of them); of V one 8-key x 4-value unit per lane (unit = 32-key step ks,
  // 64-wide block b; with 8 waves, wave / 4 picks which 16-key tile of the unit).
  struct Stage {
    u32x4 k[KF];
    u32x2 v[VA][4];
  };
  Stage stg;
  const int kt = wave & 3, wh = wave >> 2;
  const int v_b = kt % NB, v_ks = kt / NB;              // v_ks < 2 only for the waves that stage V
  const bool stages_v = NB == 2 || v_ks < 2;            // with two 64-wide blocks every wave stages V
  const int last_block = n_blocks - 1;
  // Row addresses: a block that lies wholly inside [0, L) uses per-lane byte offsets fixed at launch on top
  // of a uniform block base; only a ragged last block pays for clamping every row to L-1.
  const unsigned koff = (unsigned)(((size_t)(kt * 16 + r) * kv_pitch + g * 8 + wh * KF * 32) * sizeof(bf16));
  const unsigned voff =
      (unsigned)(((size_t)((2 * v_ks + wh * VA) * 16 + 4 * g) * kv_pitch + v_b * 64 + 4 * r) * sizeof(bf16));
  const unsigned vrow_bytes = (unsigned)(kv_pitch * sizeof(bf16));
  auto load_block = [&](Stage& sg, int blk_req) {       // past the end: the last block again, never used
    const int blk = min(blk_req, last_block);
    const int key0 = key_lo + blk * kBlockKeys;
    if (key0 + kBlockKeys <= L) {
      const char* kblk = reinterpret_cast<const char*>(kbase + (size_t)key0 * kv_pitch);     // uniform
      const char* vblk = reinterpret_cast<const char*>(vbase + (size_t)key0 * kv_pitch);
#pragma unroll
      for (int s = 0; s < KF; ++s) sg.k[s] = ld16(kblk + koff + s * 64);
      if (stages_v) {
#pragma unroll
        for (int a = 0; a < VA; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) sg.v[a][e] = ld8(vblk + voff + (unsigned)(a * 16 + e) * vrow_bytes);
      }
    } else {
      const int key = min(key0 + kt * 16 + r, L - 1);
      const bf16* krow = kbase + (size_t)key * kv_pitch + g * 8 + wh * KF * 32;
#pragma unroll
      for (int s = 0; s < KF; ++s) sg.k[s] = ld16(krow + s * 32);
      if (stages_v) {
#pragma unroll
        for (int a = 0; a < VA; ++a)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int vkey = min(key0 + (2 * v_ks + wh * VA + a) * 16 + 4 * g + e, L - 1);
            sg.v[a][e] = ld8(vbase + (size_t)vkey * kv_pitch + v_b * 64 + 4 * r);
          }
      }
    }
  };
  // Slots of V in LDS.  The value of head-dim index b*64 + 4r + i lives in head-dim tile dt = 4b + r/4 at row
  // 4(r%4) + i; a fragment's 8 keys are lane group g's 4 keys of tile 2ks, then of tile 2ks+1 (the order P is
  // packed in).  Reader lane l of tile dt reads slot l ^ (dt & 3): the same 64 slots, so reads stay
  // conflict-free, while the 64 writers of one store instruction (16 values of r for each g) now spread over
  // all banks instead of piling 16 deep on a quarter of them.
  const int v_dt = v_b * 4 + (r >> 2);
  auto store_block = [&](const Stage& sg, int buf) {
#pragma unroll
    for (int s = 0; s < KF; ++s) k_lds[buf][(kt * NS + wh * KF + s) * 64 + lane] = sg.k[s];
    if (stages_v) {
      // 4x4 transposes: op[a][i] = keys 4g..4g+3 of tile 2ks+a for head-dim value 4r+i of block b
      u32x2 op[VA][4];
#pragma unroll
      for (int a = 0; a < VA; ++a) {
        op[a][0] = u32x2{pack_lo(sg.v[a][0].x, sg.v[a][1].x), pack_lo(sg.v[a][2].x, sg.v[a][3].x)};
        op[a][1] = u32x2{pack_hi(sg.v[a][0].x, sg.v[a][1].x), pack_hi(sg.v[a][2].x, sg.v[a][3].x)};
        op[a][2] = u32x2{pack_lo(sg.v[a][0].y, sg.v[a][1].y), pack_lo(sg.v[a][2].y, sg.v[a][3].y)};
        op[a][3] = u32x2{pack_hi(sg.v[a][0].y, sg.v[a][1].y), pack_hi(sg.v[a][2].y, sg.v[a][3].y)};
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int slot = (g * 16 + 4 * (r & 3) + i) ^ (r >> 2);
        u32x4* dst = &v_lds[buf][(v_dt * 2 + v_ks) * 64 + slot];
        if constexpr (VA == 2) *dst = u32x4{op[0][i].x, op[0][i].y, op[1][i].x, op[1][i].y};
        else reinterpret_cast<u32x2*>(dst)[wh] = op[0][i];
      }
    }
  };

  // Online softmax in the base-2 domain: p = 2^(s*c - ref) with c = scale*log2(e).  ref is a per-row
  // reference, not necessarily the running maximum: it is only raised (and O, l rescaled) when a score
  // exceeds it by more than kRaise, so p stays below 2^kRaise.  The result is the same softmax (shift
  // invariance); the decision depends on the data only.  Every lane checks its own 16 scores of a row
  // against the row's reference; only when some lane of the wave finds one too large do the four lanes that
  // share a row exchange their maxima and raise the reference (rare after the first block).
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
  constexpr int kRing = 4;                     // LDS fragments in flight ahead of the matrix-core step that uses them
  f32x4 st[4][QT];
  const int vlane[4] = {lane, lane ^ 1, lane ^ 2, lane ^ 3};

  auto block = [&](int blk) {
    const int buf = blk & 1;
    const int key0 = key_lo + blk * kBlockKeys;
    // ---- scores S^T = K Q^T; the first step of every tile starts from a zero accumulator operand.
    // The K fragments come from LDS through a ring of kRing registers: fragment i + kRing is requested right
    // behind the matrix-core steps of fragment i, so one LDS latency is paid per block, not one per fragment
    // (the scheduler is told to keep this order; left alone it waits for every pair of reads).
    {
      constexpr int NF = 4 * NS;
      Frag<bf16> kf[kRing];
#pragma unroll
      for (int i = 0; i < kRing; ++i) kf[i].raw = k_lds[buf][i * 64 + lane];
#pragma unroll
      for (int i = 0; i < NF; ++i) {
#pragma unroll
        for (int t = 0; t < QT; ++t) {
          if (i % NS == 0)
            st[i / NS][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, kf[i % kRing].raw), __builtin_bit_cast(bf16x8, qf[t][0].raw),
                f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
          else
            mfma16(st[i / NS][t], kf[i % kRing], qf[t][i % NS]);
        }
        if (i + kRing < NF) kf[i % kRing].raw = k_lds[buf][(i + kRing) * 64 + lane];
      }
      __builtin_amdgcn_sched_group_barrier(0x100, kRing, 0);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, QT, 0);
        if (i + kRing < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
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
    // ---- this lane's maxima against the rows' references
    float tmax[QT];
    bool need = false;
#pragma unroll
    for (int t = 0; t < QT; ++t) {
      tmax[t] = fmaxf(fmaxf(st[0][t][0], st[0][t][1]), fmaxf(st[0][t][2], st[0][t][3]));
#pragma unroll
      for (int a = 1; a < 4; ++a)
        tmax[t] = fmaxf(tmax[t], fmaxf(fmaxf(st[a][t][0], st[a][t][1]), fmaxf(st[a][t][2], st[a][t][3])));
      need = need || tmax[t] * c2 > ref[t] + kRaise;
    }
    if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
      for (int t = 0; t < QT; ++t) {
        float rmax = fmaxf(tmax[t], __shfl_xor(tmax[t], 16, kWave));
        rmax = fmaxf(rmax, __shfl_xor(rmax, 32, kWave)) * c2;       // the row's maximum; -inf only if it has no key yet
        const float ref_new = rmax > ref[t] + kRaise ? rmax : ref[t];
        const float alpha = ref_new == ref[t] ? 1.f : __builtin_amdgcn_exp2f(ref[t] - ref_new);   // 0 on the first block
        l_run[t] *= alpha;
#pragma unroll
        for (int d = 0; d < ND; ++d) acc[d][t] *= alpha;
        ref[t] = ref_new;
      }
    }
    // ---- probabilities against the references, packed as the B operand of O^T += V^T P^T
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
      if constexpr (EMIT) {
        // this lane holds 4 consecutive keys of each of the block's 4 key tiles for query row r of tile t
        const int row = q0 + t * 16 + r;
        if (row < m && ptilde != nullptr) {      // null: a sequence of the batch whose average is not wanted
          const int gblk = (key_lo >> 6) + blk;                     // key_lo is a multiple of the block length
          // stored as packed: the 64 values of (row, block) in the order [32-key step][lane group][tile, key]
          bf16* prow = ptilde + ((size_t)head * m + row) * Lp + (size_t)gblk * kBlockKeys + 8 * g;
#pragma unroll
          for (int ks = 0; ks < 2; ++ks) *reinterpret_cast<u32x4*>(prow + ks * 32) = pf[ks][t].raw;
          if (g == 0) refblk[((size_t)head * n_blk_total + gblk) * m + row] = ref[t];
        }
      }
    }
    // ---- O^T += V^T P^T, the V fragments through the same kind of ring
    {
      constexpr int NF = ND * 2;
      Frag<bf16> vf[kRing];
#pragma unroll
      for (int i = 0; i < kRing; ++i) vf[i].raw = v_lds[buf][i * 64 + vlane[(i / 2) & 3]];
#pragma unroll
      for (int i = 0; i < NF; ++i) {
#pragma unroll
        for (int t = 0; t < QT; ++t) mfma16(acc[i / 2][t], vf[i % kRing], pf[i % 2][t]);
        if (i + kRing < NF) vf[i % kRing].raw = v_lds[buf][(i + kRing) * 64 + vlane[((i + kRing) / 2) & 3]];
      }
      __builtin_amdgcn_sched_group_barrier(0x100, kRing, 0);
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, QT, 0);
        if (i + kRing < NF) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }
  };

  load_block(stg, 0);
  store_block(stg, 0);
  __syncthreads();
  for (int blk = 0; blk < n_blocks; ++blk) {
    load_block(stg, blk + 1);                          // flies during this block's arithmetic
    block(blk);
    // the other buffer was last read one iteration ago, before the barrier every wave has passed
    store_block(stg, (blk & 1) ^ 1);
    __syncthreads();
  }

#pragma unroll
  for (int t = 0; t < QT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16, kWave);
    l += __shfl_xor(l, 32, kWave);
    const int row = q0 + t * 16 + r;
    if (row >= m) continue;
    const size_t prow = ((size_t)id.split * n_heads + head) * m + row;
    if (g == 0 && ml_part != nullptr && (EMIT || n_splits > 1)) {
      ml_part[prow * 2] = ref[t];                        // base-2 reference of this partial
      ml_part[prow * 2 + 1] = l;
    }
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
      float* dst = o_part + prow * DH + 4 * g;
#pragma unroll
      for (int d = 0; d < ND; ++d) *reinterpret_cast<f32x4*>(dst + d * 16) = acc[d][t];
    }
  }
}

// Everything that has to wait for all key splits of a row, in one launch with two kinds of workgroups.
//   merge (the workgroups behind the first avg_blocks, only with several key splits):
//     out[row, head, :] = sum_s 2^{ref_s - M} O_s / sum_s 2^{ref_s - M} l_s in split order, and the row's log-sum-exp;
//   head average (the first avg_blocks workgroups): A-bar[i, j] = (1/H) sum_h ptilde[h, i, j] 2^{refblk[h, j / 64, i] - lse2[h, i]}, heads in
//     order, with lse2[h, i] = M + log2 sum_s l_s 2^{ref_s - M} (M = max_s ref_s) recomputed from the splits' (ref, l).
//     A workgroup takes kFinRows rows x kFinKeys keys; a thread owns 8 consecutive keys of one row.
constexpr int kFinRows = 2, kFinKeys = 1024, kFinHeads = 64;
template <int DH>
__global__ __launch_bounds__(kThreads) void attn_finish_kernel(const BatchArgs batch, int n_heads) {
  const SeqArgs& sq = batch.seq[blockIdx.y];
  const float* __restrict__ o_part = sq.o_part;
  const float* __restrict__ ml_part = sq.ml_part;
  const bf16* __restrict__ ptilde = sq.ptilde;
  const float* __restrict__ refblk = sq.refblk;
  bf16* __restrict__ out = sq.out;
  float* __restrict__ lse = sq.lse;
  float* __restrict__ attn_avg = sq.attn_avg;
  const int m = sq.m, L = sq.L, n_splits = sq.n_splits, avg_blocks = sq.avg_blocks;
  if ((int)blockIdx.x >= avg_blocks) {                    // the head-average workgroups run longest and go first
    if (n_splits <= 1) return;                            // nothing to merge (the grid is sized for the whole batch)
    constexpr int PER_ROW = DH / 4;                       // threads per (head, row): 4 values each
    const size_t item = (size_t)((int)blockIdx.x - avg_blocks) * kThreads + threadIdx.x;
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
      const float f = __builtin_amdgcn_exp2f(ml_part[prow * 2] - mx);
      lsum += ml_part[prow * 2 + 1] * f;
      o += *reinterpret_cast<const f32x4*>(o_part + prow * DH + 4 * c) * f;
    }
    const float inv = 1.0f / lsum;
    const u32x2 v = {pack_bf16(o[0] * inv, o[1] * inv), pack_bf16(o[2] * inv, o[3] * inv)};
    *reinterpret_cast<u32x2*>(out + (size_t)row * n_heads * DH + head * DH + 4 * c) = v;
    if (c == 0) lse[hr] = mx * 0.693147180559945309f + __logf(lsum);
    return;
  }
  __shared__ float lse2_s[kFinHeads][kFinRows];
  const int n_blk = (L + kBlockKeys - 1) / kBlockKeys, Lk = n_blk * kBlockKeys, Lp = Lk + kPtildePad;
  const int key_tiles = (Lk + kFinKeys - 1) / kFinKeys;
  const int b = (int)blockIdx.x;
  const int rb = b / key_tiles, kb = b - rb * key_tiles;
  const int tid = threadIdx.x, rr = tid / (kFinKeys / 8), c = tid % (kFinKeys / 8);
  const int row = rb * kFinRows + rr;
  const int j0 = kb * kFinKeys + c * 8;                    // this thread's 16-byte piece of the row
  const bool live = row < m && j0 < Lk;
  const int rowc = min(row, m - 1), j0c = min(j0, Lk - 8);
  const bf16* pbase = ptilde + (size_t)rowc * Lp + j0c;
  const float* rbase = refblk + (size_t)(j0c >> 6) * m + rowc;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  constexpr int U = 32;                                    // heads per trip: their loads are issued together
  for (int h0 = 0; h0 < n_heads; h0 += kFinHeads) {
    const int nh = min(kFinHeads, n_heads - h0);
    // the first trip's loads are requested before the rows' log-sum-exp is put together, so that the two
    // latencies overlap (heads past the end repeat the last one and are not added)
    u32x4 pv[U];
    float rf[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t h = (size_t)(h0 + min(u, nh - 1));
      pv[u] = ld16(pbase + h * m * Lp);
      rf[u] = rbase[h * n_blk * m];
    }
    __syncthreads();
    for (int item = tid; item < kFinHeads * kFinRows; item += kThreads) {
      const int hh = item / kFinRows, r2 = item - hh * kFinRows;
      const int row2 = min(rb * kFinRows + r2, m - 1);
      if (hh < nh) {
        const size_t hr = (size_t)(h0 + hh) * m + row2;
        float ms[8], ls[8];                                  // at most 8 key splits
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          const size_t prow = (size_t)min(s, n_splits - 1) * n_heads * m + hr;
          ms[s] = ml_part[prow * 2];
          ls[s] = ml_part[prow * 2 + 1];
        }
        float mx = ms[0];
#pragma unroll
        for (int s = 1; s < 8; ++s) mx = fmaxf(mx, ms[s]);
        float lsum = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s)
          if (s < n_splits) lsum += ls[s] * __builtin_amdgcn_exp2f(ms[s] - mx);
        lse2_s[hh][r2] = mx + __builtin_amdgcn_logf(lsum);      // v_log_f32 is a base-2 logarithm
      }
    }
    __syncthreads();
    for (int hh = 0; hh < nh; hh += U) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (hh + u < nh) {
          const float f = __builtin_amdgcn_exp2f(rf[u] - lse2_s[hh + u][rr]);
          const bf16x8 pb = __builtin_bit_cast(bf16x8, pv[u]);
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] = fmaf((float)pb[e], f, acc[e]);
        }
      }
      if (hh + U < nh) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const size_t h = (size_t)(h0 + min(hh + U + u, nh - 1));
          pv[u] = ld16(pbase + h * m * Lp);
          rf[u] = rbase[h * n_blk * m];
        }
      }
    }
  }
  if (!live) return;
  // piece (ks, g) of block blk holds keys 64 blk + 32 ks + 4 g .. +3 and the same 16 keys further on
  const float inv_h = 1.0f / (float)n_heads;
  const int piece = (j0 >> 3) & 7, ks = piece >> 2, g = piece & 3;
  const int key_a = (j0 & ~63) + 32 * ks + 4 * g, key_b = key_a + 16;
  float* dst = attn_avg + (size_t)row * L;
  if ((L & 3) == 0) {                                      // rows start 16-byte aligned
    if (key_a < L) *reinterpret_cast<f32x4*>(dst + key_a) = f32x4{acc[0] * inv_h, acc[1] * inv_h, acc[2] * inv_h, acc[3] * inv_h};
    if (key_b < L) *reinterpret_cast<f32x4*>(dst + key_b) = f32x4{acc[4] * inv_h, acc[5] * inv_h, acc[6] * inv_h, acc[7] * inv_h};
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (key_a + e < L) dst[key_a + e] = acc[e] * inv_h;
      if (key_b + e < L) dst[key_b + e] = acc[4 + e] * inv_h;
    }
  }
}

struct FwdPlan {
  int qt, waves, q_blocks, n_splits, keys_per_split;
};
FwdPlan plan_fwd(const Tunables& t, int m, int L, int n_heads) {
  FwdPlan p;
  const int want_qt = t.attn_qt;
  p.qt = want_qt == 1 ? 1 : want_qt == 2 ? 2 : (m > 64 ? 2 : 1);
  // more than 128 rows: 8 waves (two per SIMD) on 256 queries per workgroup
  p.waves = t.attn_waves == 4 || t.attn_waves == 8 ? t.attn_waves : (p.qt == 2 && m > 128 ? 8 : 4);
  const int q_per_wg = 16 * p.qt * p.waves;
  p.q_blocks = (m + q_per_wg - 1) / q_per_wg;
  const int blocks = (L + kBlockKeys - 1) / kBlockKeys;
  int splits = 1;
  const int max_splits = std::max(1, std::min(8, t.attn_max_splits));
  while (splits < max_splits && p.q_blocks * n_heads * splits < t.attn_target_wgs && blocks / (splits * 2) >= 1) splits *= 2;
  const int blocks_per_split = (blocks + splits - 1) / splits;
  p.keys_per_split = blocks_per_split * kBlockKeys;
  p.n_splits = (L + p.keys_per_split - 1) / p.keys_per_split;     // every split holds at least one key
  return p;
}

// Scratch of one call, in floats: partial outputs of the key splits, their (reference, sum) pairs, the
// unnormalised probabilities (bf16, two per float) and the per-block references.
struct Scratch {
  size_t o_part, ml, ptilde, refblk, total;
};
Scratch scratch_of(const FwdPlan& p, int m, int L, int n_heads, int head_dim, bool emit) {
  Scratch s;
  const size_t hm = (size_t)n_heads * m;
  const size_t n_blk = (size_t)(L + kBlockKeys - 1) / kBlockKeys;
  s.o_part = p.n_splits > 1 ? (size_t)p.n_splits * hm * head_dim : 0;
  s.ml = (size_t)p.n_splits * hm * 2;
  s.ptilde = emit ? (hm * (n_blk * kBlockKeys + kPtildePad) + 1) / 2 : 0;
  s.ptilde = (s.ptilde + 3) & ~(size_t)3;                          // keep what follows 16-byte aligned
  s.refblk = emit ? hm * n_blk : 0;
  s.total = s.o_part + s.ml + s.ptilde + s.refblk;
  return s;
}

template <int DH>
hipError_t launch_tiled(const Tunables& t, const TiledCall* calls, int n_calls, int n_heads, int n_kv_heads,
                        float* scratch, size_t scratch_floats, hipStream_t st) {
  // one plan for the batch: tile shape by the largest row count, key splits so that all sequences together
  // give every compute unit a workgroup
  int max_m = 0, max_L = 0;
  bool emit = false;
  for (int i = 0; i < n_calls; ++i) {
    max_m = std::max(max_m, calls[i].m);
    max_L = std::max(max_L, calls[i].L);
    emit = emit || calls[i].attn_avg != nullptr;
  }
  FwdPlan shape = plan_fwd(t, max_m, max_L, n_heads);
  const int max_splits = std::max(1, std::min(8, t.attn_max_splits));
  const int min_blocks = (std::max(1, max_L) + kBlockKeys - 1) / kBlockKeys;
  auto splits_for = [&](int q_per_wg) {
    int wgs_unsplit = 0;
    for (int i = 0; i < n_calls; ++i) wgs_unsplit += ((calls[i].m + q_per_wg - 1) / q_per_wg) * n_heads;
    int sp = 1;
    while (sp < max_splits && wgs_unsplit * sp < t.attn_target_wgs && min_blocks / (sp * 2) >= 1) sp *= 2;
    return sp;
  };
  int splits = splits_for(16 * shape.qt * shape.waves);
  // 8-wave workgroups halve the K/V traffic per query and overlap two waves per SIMD, but also halve the
  // workgroup count, i.e. double the key splits a small problem needs; with fewer than 8 blocks left per
  // split the partial outputs (written, then merged) cost more than the loop gains (measured at 256 rows x
  // 2048 keys x 32 heads: 43 vs 47 us per call)
  if (shape.waves == 8 && t.attn_waves == 0 && min_blocks / splits < 8) {
    shape.waves = 4;
    splits = splits_for(16 * shape.qt * shape.waves);
  }
  const int q_per_wg = 16 * shape.qt * shape.waves;
  const float scale = 1.0f / sqrtf((float)DH);
  BatchArgs args;
  memset(&args, 0, sizeof(args));
  size_t used = 0;
  int max_tiles = 0, max_fin = 0;
  for (int i = 0; i < n_calls; ++i) {
    const TiledCall& c = calls[i];
    FwdPlan p = shape;
    p.q_blocks = (c.m + q_per_wg - 1) / q_per_wg;
    const int blocks = (c.L + kBlockKeys - 1) / kBlockKeys;
    const int s_i = std::max(1, std::min(splits, blocks));
    p.keys_per_split = ((blocks + s_i - 1) / s_i) * kBlockKeys;
    p.n_splits = (c.L + p.keys_per_split - 1) / p.keys_per_split;
    const bool emit_i = c.attn_avg != nullptr;
    const Scratch sc = scratch_of(p, c.m, c.L, n_heads, DH, emit_i);
    if (sc.total > 0 && (!scratch || used + sc.total > scratch_floats)) return hipErrorInvalidValue;
    float* base = scratch ? scratch + used : nullptr;
    used += (sc.total + 3) & ~(size_t)3;
    SeqArgs& a = args.seq[i];
    a.q = (const bf16*)c.q; a.k_cache = (const bf16*)c.k_cache; a.v_cache = (const bf16*)c.v_cache;
    a.out = (bf16*)c.out; a.lse = c.lse; a.attn_avg = c.attn_avg;
    a.o_part = base;                                               // 16-byte aligned pieces, in this order
    a.ptilde = reinterpret_cast<bf16*>(base && emit_i ? base + sc.o_part : nullptr);
    a.ml_part = base ? base + sc.o_part + sc.ptilde : nullptr;
    a.refblk = base && emit_i ? a.ml_part + sc.ml : nullptr;
    a.m = c.m; a.L = c.L; a.keys_per_split = p.keys_per_split; a.n_splits = p.n_splits; a.q_blocks = p.q_blocks;
    a.avg_blocks = emit_i ? ((c.m + kFinRows - 1) / kFinRows) * ((blocks * kBlockKeys + kFinKeys - 1) / kFinKeys) : 0;
    const int groups = (n_heads * p.n_splits + 7) / 8;
    max_tiles = std::max(max_tiles, groups * 8 * p.q_blocks);
    const size_t items = (size_t)n_heads * c.m * (DH / 4);
    const int merge_blocks = p.n_splits > 1 ? (int)((items + kThreads - 1) / kThreads) : 0;
    max_fin = std::max(max_fin, a.avg_blocks + merge_blocks);
  }
  const dim3 grid(max_tiles, n_calls);
#define D2C_TILED_FWD(QT_, WAVES_, EMIT_)                                                                         \
  hipLaunchKernelGGL((attn_tiled_fwd_kernel<DH, QT_, WAVES_, EMIT_>), grid, dim3(WAVES_ * 64), 0, st, args, n_heads, \
                     n_kv_heads, scale)
  if (shape.qt == 2 && shape.waves == 8 && emit) D2C_TILED_FWD(2, 8, true);
  else if (shape.qt == 2 && shape.waves == 8) D2C_TILED_FWD(2, 8, false);
  else if (shape.qt == 2 && emit) D2C_TILED_FWD(2, 4, true);
  else if (shape.qt == 2) D2C_TILED_FWD(2, 4, false);
  else if (shape.waves == 8) return hipErrorInvalidValue;
  else if (emit) D2C_TILED_FWD(1, 4, true);
  else D2C_TILED_FWD(1, 4, false);
#undef D2C_TILED_FWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || max_fin == 0) return e;
  hipLaunchKernelGGL(attn_finish_kernel<DH>, dim3((unsigned)max_fin, n_calls), dim3(kThreads), 0, st, args, n_heads);
  return hipGetLastError();
}

}  // namespace

// Most scratch ONE sequence of a batch can need, over every (m <= max_m, L <= max_L), with the head average
// wanted.  Inside a batch the tile shape follows the largest sequence and the split count the whole batch, so
// a sequence can be split whenever its workgroups in the largest tile shape alone would not fill the chip.
size_t attention_tiled_scratch_floats(const Tunables& t, int max_m, int max_L, int n_heads, int head_dim) {
  size_t worst = 0;
  const int max_splits = std::max(1, std::min(8, t.attn_max_splits));
  for (int L = kBlockKeys;; L += kBlockKeys) {
    const int Lc = std::min(L, max_L);
    const int blocks = (Lc + kBlockKeys - 1) / kBlockKeys;
    for (int m = 1; m <= max_m; ++m) {
      FwdPlan p = plan_fwd(t, m, Lc, n_heads);
      const bool can_split = ((m + 255) / 256) * n_heads < t.attn_target_wgs;
      p.n_splits = can_split ? std::min(max_splits, blocks) : 1;
      worst = std::max(worst, (scratch_of(p, m, Lc, n_heads, head_dim, true).total + 3) & ~(size_t)3);
    }
    if (L >= max_L) break;
  }
  return worst;
}

hipError_t launch_attention_tiled(const Tunables& t, const TiledCall* calls, int n_calls, int n_heads, int n_kv_heads,
                                  int head_dim, float* scratch, size_t scratch_floats, hipStream_t st) {
  if (n_calls <= 0) return hipSuccess;
  if (n_calls > kMaxBatch) return hipErrorInvalidValue;
  if (head_dim == 128) return launch_tiled<128>(t, calls, n_calls, n_heads, n_kv_heads, scratch, scratch_floats, st);
  if (head_dim == 64) return launch_tiled<64>(t, calls, n_calls, n_heads, n_kv_heads, scratch, scratch_floats, st);
  return hipErrorInvalidValue;
}

int attention_tiled_max_batch() { return kMaxBatch; }

}  // namespace d2c
