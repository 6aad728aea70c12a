/*
 * d2c_tools.h -- tooling around the d2Cache step library (include/d2c.h): per-kernel timing, launch-shape
 * tunables and the host-side launch planner.  None of these calls is part of the method; the tests use them to
 * force every kernel path, the benchmark to time kernel classes.  Same conventions as d2c.h (0 or a negative
 * error code, never throws).
 */
#ifndef D2C_TOOLS_H
#define D2C_TOOLS_H

#include <stdint.h>

#include "d2c.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Per-launch timing with HIP events on the stream the kernels run on, by kernel class.
 * Between d2c_profile_begin and d2c_profile_end every launch of the calls of d2c.h is
 * bracketed by an event pair (this perturbs the stream: do not time end-to-end while
 * it is on).  d2c_profile_end waits for the events and returns, per class, the summed
 * kernel time in milliseconds, the number of launches and the summed algorithmic
 * bytes (projection: the weight matrix once; attention: the K and V cache once). */
#define D2C_PROF_GEMM      0
#define D2C_PROF_ATTENTION 1
#define D2C_PROF_ROLLOUT   2
#define D2C_PROF_ROWWISE   3
#define D2C_PROF_SELECT    4
#define D2C_PROF_ATTN_AVG  5
#define D2C_PROF_CLASSES   6
int d2c_profile_begin(d2c_ctx* ctx);
int d2c_profile_end(d2c_ctx* ctx, double* ms, int64_t* launches, double* bytes);

/* Launch-shape tunables.  Every context has its own set; two contexts may differ.  Names:
 * projection kernel: "gemm_waves" (waves per workgroup: 4, 6, 7, 8, 10; 0 = chosen by shape together with the
 * split count), "gemm_max_splits" (1..8), "gemm_target_wgs" (workgroups aimed at where the shape search does
 * not apply), "gemm_nt_big_n", "gemm_wide_tiles" (0/1: 128 x 64 outputs per wave for many bf16 rows),
 * "gemm_wide_mt" (6, 7, 8 row tiles per workgroup of that shape; 0 = by shape),
 * "gemm_wide_min_rows" (that instantiation from this many rows on), "gemm_tall_chunk" (0/1: 129-192 bf16 rows
 * as one row chunk), "gemm_preshuffle" (0/1: pre-tiled weight copies; only at d2c_init_tuned), "gemm_rot";
 * attention: "attn_tiled_min_m" (bf16 attention switches to the LDS-tiled kernels from this many query rows
 * on), "attn_max_splits" (1..8, key-range splits of one attention launch), "attn_qt", "attn_waves" (4, 8),
 * "attn_target_wgs",
 * "side_stream" (0/1, default 0: whether d2c_step runs the head average and the rollout on a second
 * stream). */
typedef struct {
  const char* name;
  int32_t     value;
} d2c_tunable;

/* d2c_init with tunables in force from the start (the workspace is sized for them).  D2C_EINVAL for an
 * unknown name. */
int d2c_init_tuned(const d2c_dims* dims, const d2c_weights* weights, const d2c_tunable* tunables,
                   int32_t n_tunables, d2c_ctx** out);

/* Changes one tunable of a live context; takes effect from the next call on.  "gemm_preshuffle" cannot be
 * changed after init (D2C_EINVAL); a value whose launch shapes would need more workspace than the context
 * allocated is refused with D2C_ESHAPE and changes nothing. */
int d2c_ctx_set_tunable(d2c_ctx* ctx, const char* name, int32_t value);

/* The launch shape the projection kernel would take for P = A[m, K] W[N, K]^T under the default tunables
 * (host-side arithmetic only: no context, no GPU).  single_split != 0: the projection must not split the
 * contraction (the gate/up projection with the gated epilogue).  Writes
 * shape[0..6] = row tiles per workgroup (16 rows each), column tiles per wave, waves per workgroup, splits of
 * the contraction, contraction elements per split, row chunks, workgroups of the launch.
 * Returns D2C_EINVAL for a null pointer, a dtype other than D2C_F32 / D2C_BF16 or non-positive sizes. */
int d2c_plan_projection(int32_t dtype, int32_t m, int32_t N, int32_t K, int32_t single_split, int32_t shape[7]);

/* Device memory the context holds, in bytes: bytes[0] everything, bytes[1] of which the pre-tiled weight
 * copies, bytes[2] head averages / per-head probability rows / rollout scratch, bytes[3] attention partials. */
int d2c_memory_info(const d2c_ctx* ctx, int64_t bytes[4]);

#ifdef __cplusplus
}
#endif
#endif /* D2C_TOOLS_H */
