/*
 * spd_testing.h - test and benchmark aids of the SPD library.  Nothing here is part of the
 * product boundary (spd.h); the symbols live in the same shared library so that benchmarks and
 * tests can look inside a forward call without a second build.
 *
 * Nothing in this header keeps process-wide state: stage selection and timing are arguments of
 * the call they apply to.
 */
#ifndef SPD_TESTING_H
#define SPD_TESTING_H

#include "spd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---------------------------------------------------------------- stages of a block
 * The stages of a decoder block as the library launches them (Sec. 3 / Sec. 4.1.1 name the
 * operations; the cut into launches is the library's). */
#define SPD_STAGE_PREP 0    /* rank-sum + first-norm elementwise work */
#define SPD_STAGE_QKV 1     /* QKV projection + rotary + cache append */
#define SPD_STAGE_ATTN 2    /* attention over the KV cache (all its kernels) */
#define SPD_STAGE_O 3       /* O projection + residual fold */
#define SPD_STAGE_GATEUP 4  /* gate/up projection + SwiGLU */
#define SPD_STAGE_DOWN 5    /* down projection + partial-sum fold */
#define SPD_N_STAGES 6
#define SPD_ALL_STAGES ((1u << SPD_N_STAGES) - 1u)
#define SPD_STAGE_EMPTY 6   /* timers only: a pair of events with nothing between them, once per block (what the
                               bracket itself adds to a measured stage) */

/* A timer for one stage: every launch of that stage inside a call it is handed to is bracketed by
 * a pair of HIP events on the call's stream (so that call must not be under stream capture).
 * Holds room for max_records launches; further launches go untimed.  One timer serves one call at
 * a time.  `stage` is one of the stages above or SPD_STAGE_EMPTY.  SPD_EINVAL: unknown stage,
 * max_records <= 0, NULL; SPD_EHIP: event creation failed. */
typedef struct spd_stage_timer spd_stage_timer;
int spd_stage_timer_create(int32_t stage, int32_t max_records, spd_stage_timer **out);
/* Waits for the recorded events, returns the number of launches timed and their mean and minimum
 * duration in microseconds (any pointer may be NULL), and resets the record count. */
int spd_stage_timer_read(spd_stage_timer *timer, int32_t *n_records, double *mean_us, double *min_us);
void spd_stage_timer_destroy(spd_stage_timer *timer);

/* spd_model_forward() with three more arguments:
 *   stage_mask  bit s set = the kernels of stage s are launched.  SPD_ALL_STAGES is the ordinary
 *               call.  With a single bit a whole-model call becomes a train of launches of one
 *               stage's kernel over every layer's distinct weights (its inputs are whatever an
 *               earlier full call left in the workspace, its outputs are meaningless): the way to
 *               time a kernel on its own without the whole layer fitting a cache.
 *   timer       NULL, or a timer whose stage's launches are to be bracketed by events.
 *   layer_out   NULL, or device fp32 [n_layers][batch*q_len, hidden]: receives every block's output (a
 *               device-to-device copy after each block), so that a test can check a deep model block by block.
 * SPD_EINVAL for bits beyond SPD_ALL_STAGES; otherwise as spd_model_forward(). */
int spd_model_forward_staged(const spd_ctx *ctx, const uint8_t *spd_mask, int32_t rank,
                             const void *const *layer_weights, void *const *layer_kv,
                             const int32_t *positions, int32_t batch, int32_t q_len,
                             const float *x_in, float *slots, float *x_out, void *workspace,
                             void *stream, int64_t *n_rank_sums, uint32_t stage_mask,
                             spd_stage_timer *timer, float *layer_out);

/* ---------------------------------------------------------------- what the matrix cores sustain
 * A grid of one workgroup of 8 waves per compute unit (256 workgroups) in which every wave runs `iters`
 * rounds of 32 independent 16x16x32 fp16 MFMAs on operands it holds in registers: no LDS, no memory
 * traffic inside the loop.  With random_data != 0 the operands are pseudo-random values in (-2, 2), else
 * all ones (the chip's clock under load depends on how many bits toggle).  Returns the rate over the
 * whole launch (HIP events on `stream`) and the shader clock seen by one workgroup in the middle of the
 * grid (its cycle counter against the 100 MHz real-time counter).  `scratch` is device memory of at least
 * SPD_MFMA_PROBE_SCRATCH_BYTES that the kernel writes its sums to (so that the loop is not optimised
 * away).  Synchronises the stream.  SPD_EINVAL: iters <= 0 or NULL pointers; SPD_EHIP as elsewhere. */
#define SPD_MFMA_PROBE_SCRATCH_BYTES (256 * 512 * 4 + 16)
int spd_mfma_probe(int32_t iters, int32_t random_data, void *scratch, void *stream, double *tflops, double *mhz);

/* ---------------------------------------------------------------- what a plain read sustains
 * `reps` launches of a kernel that only reads: launch i reads the `chunk_bytes` bytes at buf + (i % n_chunks) *
 * chunk_bytes (so that with n_chunks * chunk_bytes well above the 256 MB Infinity Cache every launch reads from
 * HBM), 256 workgroups of 16 waves, every wave a contiguous share with four 1 KiB non-temporal loads in flight:
 * the access pattern of the decode projections without their arithmetic, activations, reduction and epilogue.
 * Returns the mean time per launch in microseconds (HIP events on `stream` around all launches, which follow each
 * other on the stream).  `sink` is device memory of at least 4 bytes (never written unless the data read is a
 * particular pattern; it keeps the loads alive).  Synchronises the stream.
 * SPD_EINVAL: NULL pointers, chunk_bytes not a multiple of 4 MiB, n_chunks or reps <= 0. */
int spd_read_probe(const void *buf, size_t chunk_bytes, int32_t n_chunks, int32_t reps, void *sink, void *stream,
                   double *us_per_launch);

/* ---------------------------------------------------------------- launch order of the GEMM tiles
 * The LDS-tiled GEMM of a long call runs its TN x TM tiles (of rn x rm rows) in an order that keeps the tiles
 * an XCD has in flight close together.  For a launch of n_tiles tiles of that order starting at tile number
 * tile0, spd_gemm_launch_size() is the number of workgroups launched and spd_gemm_tile_of() tells which tile
 * workgroup b takes: 0 and (*tn, *tm), or 1 when b is a spare workgroup that takes none; SPD_EINVAL for
 * arguments out of range or NULL pointers.  Host only; exists so that the order can be checked exhaustively
 * without a GPU. */
int spd_gemm_launch_size(int32_t n_tiles);
int spd_gemm_tile_of(int32_t TN, int32_t TM, int32_t rn, int32_t rm, int32_t tile0, int32_t n_tiles, int32_t b,
                     int32_t *tn, int32_t *tm);

#ifdef __cplusplus
}
#endif
#endif /* SPD_TESTING_H */
