/*
 * bild_bench.h - measurement, probe and host-logic entry points of the MI355X Big Little Decoder library.
 *
 * None of these take part in decoding and none changes a result: they time passes and the dominant kernel,
 * run plain kernels of known size against which hardware counters are scaled, and expose host-side layout and
 * launch-shape logic to CPU tests.  The method's own boundary is bild.h.  Conventions as in bild.h (error
 * codes, host pointers owned by the caller).
 */
#ifndef BILD_BENCH_H
#define BILD_BENCH_H

#include "bild.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement helpers (no effect on results).
 * bild_bench_pass: brings model `which` up to y_len - rows consumed tokens (needs
 * y_len - len >= rows), then runs `reps` identical passes over the last `rows`
 * tokens of y, LM head and statistics included, WITHOUT committing anything, and
 * returns the mean time of one pass in milliseconds from HIP events on the
 * state's stream.
 * bild_profile_begin/end: between the two calls every weight-streaming GEMM launch
 * is bracketed by HIP events (at most max_records launches are recorded);
 * end() waits for the stream and sums, per model [0 small, 1 large] and per
 * class [0 layer GEMMs, 1 LM head]: launches, milliseconds and algorithmic bytes
 * (bytes of the weight matrix each launch streams). */
typedef struct bild_profile {
    int64_t launches[2][2];
    int64_t bytes[2][2];
    double  ms[2][2];
    int32_t dropped;        /* launches not recorded because max_records was reached */
} bild_profile;
int bild_bench_pass(bild_state* s, int which, int rows, int reps, float* ms_per_pass);
/* Like bild_bench_pass, but each pass launches ONLY its weight-streaming GEMM kernels (the
 * dominant kernel), back to back in pass order, so that ms_per_pass / launches is the mean
 * duration of one GEMM launch (including the gap to the next launch) and bytes the
 * algorithmic weight bytes the launches of one pass stream.  The activations the GEMMs read
 * are stale; only the timing is meaningful. */
int bild_bench_gemm(bild_state* s, int which, int rows, int reps, float* ms_per_pass, int64_t* launches,
                    int64_t* bytes);
/* Runs `reps` launches of a plain device-to-device copy kernel (bild::probe_copy_kernel) of
 * `bytes` bytes (a multiple of 16) on temporary buffers: it reads `bytes` and writes `bytes`,
 * the known quantity against which hardware byte counters are scaled. */
int bild_probe_copy(bild_state* s, int64_t bytes, int reps);
/* Mean time of `reps` back-to-back launches of a kernel that does nothing (one workgroup per CU) on the state's
 * stream, in microseconds: the cost of a dependent stage by itself, against which the stage count of a pass is read. */
int bild_probe_launch(bild_state* s, int reps, float* us_per_launch);
/* Mean time (microseconds, launch included) of a kernel in which `groups` workgroups of 8 waves each stream a private
 * contiguous region of kib_per_group KiB that no earlier launch touched: the streaming rate of one compute unit
 * (groups = 1) and how the total grows with the number of workgroups.  reps <= 64; the probe allocates
 * groups * kib_per_group KiB * (reps + 1) for its own use (at most 16 GiB, else BILD_EINVAL) and frees it. */
int bild_probe_stream(bild_state* s, int groups, int kib_per_group, int reps, float* us_per_launch);
/* GEMM launches ISSUED by the host since the last reset and the algorithmic weight bytes they stream
 * (replays of captured graphs are not counted: meaningful when graph replay is disabled). */
int bild_gemm_tally(bild_state* s, int64_t* launches, int64_t* bytes, int reset);
/* Kernel launches (dependent stages) of the pass the host issued last - the one bild_bench_gemm issues to count its
 * GEMM launches counts here too; replays of captured graphs do not change it. */
int bild_pass_stages(bild_state* s, int32_t* stages);
int bild_profile_begin(bild_state* s, int max_records);
int bild_profile_end(bild_state* s, bild_profile* out);

/* Algorithmic bytes one pass of model `which` must read at cache length t_cache
 * with `rows` new rows (weights + LM head + self K/V + cross K/V). */
int64_t bild_pass_bytes(const bild_state* s, int which, int t_cache, int rows);

/* Host logic exposed for tests (no device work).
 * bild_debug_tile_matrix: re-lays a row-major matrix into the streaming tile order the kernels read
 * (1 KiB tiles of 16 features x 32 inputs for bf16, x 16 for fp32; inside a tile the 16 bytes of lane l hold
 * feature l % 16, inputs (l / 16) * KT/4 .. +KT/4-1; tiles of a feature block contiguous along the inputs; features
 * beyond n are zero).  src is [k][n] if src_is_k_by_n else [n][k]; dst has bild_debug_tiled_bytes(n, k, dtype) bytes.
 * bild_debug_gemm_shape: the launch shape the library would choose for a projection of n features x k inputs over
 * `rows` rows: out = {input slices per workgroup, waves per workgroup, feature tiles per wave, inputs per LDS chunk,
 * feature-group workgroups, row blocks, dynamic LDS bytes, LDS limit}. */
int64_t bild_debug_tiled_bytes(int n, int k, int dtype);
int bild_debug_tile_matrix(const float* src, int src_is_k_by_n, int n, int k, int dtype, void* dst);
int bild_debug_gemm_shape(int n, int k, int rows, int gated, int lm_head, int dtype, int32_t out[8]);
/* The launch shape of attention for `rows` query rows over nkeys cached keys: out = {key splits, 1 if the consumer
 * projection merges the split partials (no merge kernel), waves per workgroup, dynamic LDS bytes}. */
int bild_debug_attn_shape(int heads, int d_head, int rows, int nkeys, int max_splits, int dtype, int32_t out[4]);

#ifdef __cplusplus
}
#endif
#endif /* BILD_BENCH_H */
