/*
 * normtest.h -- C ABI of libnormtest.so: the per-step statistics pass of the norm-test adaptive
 * batch-size schedules (DDP-Norm / FSDP-Norm) fused with the AdamW update, for one MI355X (gfx950).
 *
 * Given J gradient vectors g_1..g_J of length d (the workers' minibatch gradients of Sec. 3.2, the
 * micro-batch gradients of a parameter shard of Sec. 3.3, or per-sample gradients of Sec. 3.1), one
 * streaming pass over HBM computes
 *
 *     gbar = (1/J) sum_j g_j                                   (Sec. 3.2; Alg. 1 "batch gradient")
 *     A = sum_j ||g_j||^2,  B = ||sum_j g_j||^2,  C = sum_j ||g_j - gbar||^2
 *     ||gbar||^2 = B/J^2,   ||Var||_1 = C/(J - ddof)           (variance estimator of Sec. 3.2 / Alg. 1)
 *     T = ||Var||_1 / (eta^2 ||gbar||^2)                       (Alg. 1, test statistic)
 *     pass = !(T > b_k), next_b by Alg. 1's rounding chain     (Alg. 1, If-branch)
 *     AdamW on gbar, in place on w, m, v                       (Alg. 1, last five update lines)
 *
 * Dynamic range: squares are formed in fp32, so |g| beyond ~1.8e19 overflows (reported as NT_STATUS_NONFINITE)
 * and sums of squares lose precision for |g| below ~1e-19; where (1 - beta2) gbar^2 falls below fp32's normal
 * range (|gbar| below ~1e-18) the stored second moment keeps few or no significant bits, as in any AdamW with
 * fp32 state.  Between those limits results are scale-invariant to the stated tolerances.
 *
 * All pointers named "device" must be dereferenceable by the GPU (device memory; result may also be
 * pinned host memory).  The library allocates nothing, keeps no state between calls, never
 * synchronises the device and never touches host copies of the data: it validates, enqueues kernels
 * on the caller's stream and returns.  No C++ types or exceptions cross this boundary.
 */
#ifndef NORMTEST_H
#define NORMTEST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element type of the gradient rows */
typedef enum { NT_F32 = 0, NT_BF16 = 1 } nt_dtype;

/* nt_hyper.flags */
enum {
  NT_DO_STATS = 1u,   /* compute A, B, C (and, unless NT_PARTIAL, the test)                      */
  NT_DO_ADAMW = 2u,   /* update w, m, v in place with AdamW on gbar                              */
  NT_PARTIAL = 4u,    /* FSDP shard: stop at the additive sums A, B, C; decide in normtest_combine */
  NT_WRITE_GBAR = 8u, /* also store gbar (fp32[d]) to gbar_out                                   */
  NT_COORD_TEST = 16u, /* also the coordinate-wise form of the test: count of failing coordinates, largest ratio */
  NT_ONE_PASS = 32u   /* accepted and without effect: the step is always one fused pass (the flag once kept       */
                      /* many-row steps from being split into statistics + gbar and AdamW from gbar)               */
};

/* nt_result.status bits */
enum {
  NT_STATUS_NONFINITE = 1u,      /* a sum is NaN/Inf (NaN/Inf gradient, or |g| beyond ~1.8e19): batch size kept  */
  NT_STATUS_ZERO_GRAD_NORM = 2u, /* ||gbar||^2 == 0: T is NaN (C == 0, passes) or +inf (fails; next_b = b_max, or  */
                                 /* b_k when b_max is 0 or below b_k: an infinite T names no finite batch size)   */
  NT_STATUS_CLAMPED = 4u,        /* the rounded batch size exceeded b_max and was cut to it                      */
  NT_STATUS_PARTIAL_ONLY = 8u,   /* NT_PARTIAL: only A, B, C (and their low parts) are meaningful                */
  NT_STATUS_T_SATURATED = 16u,   /* T >= 2^62: treated as infinite (same next_b rule as for +inf)                */
  NT_STATUS_NO_STATS = 32u,      /* NT_DO_STATS was clear: sums are NaN, pass = 1, next_b = b_k                  */
  NT_STATUS_BAD_RANGE = 64u      /* nt_layer_stats only: the layer's offsets were descending or outside [0, d]   */
};

/* return codes; values <= NT_ERR_HIP_BASE carry a HIP error: code = NT_ERR_HIP_BASE - hipError_t */
enum {
  NT_OK = 0,
  NT_ERR_BAD_ARG = -1,
  NT_ERR_UNSUPPORTED = -2,
  NT_ERR_WORKSPACE_TOO_SMALL = -3,
  NT_ERR_TOO_LARGE = -4,
  NT_ERR_HIP_BASE = -1000
};

/*
 * Scalars of one step.  AdamW symbols as in Alg. 1's Require line; eta, b_k and the rounding as in
 * Alg. 1's test; b_max as in Sec. 5 ("maximum global batch size").
 */
typedef struct {
  double lr, beta1, beta2, eps, weight_decay; /* alpha >= 0, 0 <= beta < 1, epsilon >= 0, lambda >= 0          */
  double eta;                                 /* eta > 0                                                       */
  int64_t step;                               /* k >= 1, used for the bias corrections 1 - beta^k              */
  int64_t b_k;                                /* current global batch size, >= 1                               */
  int64_t b_max;                              /* cap on next_b, 0 = none; never pulls next_b below b_k         */
  int64_t round_to;                           /* J*M (workers x accumulation steps): next_b is a multiple;     */
                                              /* 1 = the plain ceiling rule of Sec. 3.1; 1 <= round_to <= 2^31 */
  int32_t ddof;                               /* 0: variance / J (Alg. 1);  1: / (J-1) (sample variance)       */
  uint32_t flags;                             /* NT_DO_* | NT_PARTIAL | NT_WRITE_GBAR | NT_COORD_TEST | NT_ONE_PASS */
} nt_hyper;

/* Where this call's coordinates sit in the full parameter vector (Sec. 3.3).  The sums are additive over
 * coordinates, so a shard needs nothing from the others; the record is checked for consistency, and d_global
 * has one effect: long vectors are cut into larger tiles than short ones (steps that write per coordinate,
 * with 7 to 16 fp32 or 14 to 16 bf16 rows: from 2^26 coordinates; 17 to 32 rows: from 2^24; more rows: from
 * 3 * 2^21; a step with AdamW only, which forms no sums, also from 5 fp32 and 10 bf16 rows; read-only
 * statistics of up to 16 rows: from 2^21), and a call with a shard record is cut the way a vector of d_global
 * coordinates is (a call without one: the way a vector of d is). */
typedef struct {
  int32_t shard_id, num_shards;
  int64_t shard_offset, d_global;
} nt_shard_info;

typedef struct {
  double A, B, C;          /* sum_j||g_j||^2, ||sum_j g_j||^2, sum_j||g_j - gbar||^2 over this call's coordinates  */
  double A_lo, B_lo, C_lo; /* low-order parts: each sum is X + X_lo to ~1e-30 relative, so shards add up exactly   */
  double gbar_sq;          /* ||gbar||^2 = B/J^2                         (NaN if NT_PARTIAL or no stats)           */
  double var_l1;           /* C/(J - ddof)                                                                        */
  double T;                /* var_l1 / (eta^2 gbar_sq)                                                            */
  double clip_coef;        /* factor applied to gbar before AdamW: 1 unless normtest_step_clipped cut the norm    */
  int64_t next_b;          /* b_{k+1}                                                                             */
  int64_t coord_fail;      /* NT_COORD_TEST: number of coordinates i with Var_i / b_k > eta^2 gbar_i^2, the          */
                           /* coordinate-wise condition of Sec. 4 / Prop. 1 with the estimators of the aggregate     */
                           /* test, decided per coordinate in fp32; additive over shards; -1 if not requested        */
  int32_t pass;            /* 1 iff not (T > b_k)                                                                 */
  uint32_t status;         /* NT_STATUS_* bits                                                                    */
  double coord_max_ratio;  /* NT_COORD_TEST: largest Var_i / (eta^2 b_k gbar_i^2) over the coordinates (a coordinate */
                           /* fails iff its ratio exceeds 1), formed per coordinate in fp32; 0 for a coordinate       */
                           /* without spread, +inf for spread around a zero mean (the rows cancel exactly); the       */
                           /* largest over shards is the largest of the shards' values; -1 if not requested           */
} nt_result;

/* One layer (a block of consecutive coordinates) of normtest_layer_stats. */
typedef struct {
  double A, B, C;        /* the three sums over the layer's coordinates                                          */
  double gbar_sq;        /* B/J^2: squared norm of the layer's slice of gbar                                     */
  double var_l1;         /* C/(J - ddof)                                                                         */
  double T;              /* var_l1 / (eta^2 gbar_sq): Alg. 1's statistic evaluated on the layer alone            */
  int64_t n;             /* coordinates counted (after clamping the offsets into [0, d])                         */
  int64_t coord_fail;    /* failing coordinates in the layer if the step ran with NT_COORD_TEST, else -1         */
  int32_t pass;          /* 1 iff not (T > b_k)                                                                  */
  uint32_t status;       /* NT_STATUS_NONFINITE | ZERO_GRAD_NORM | T_SATURATED | NO_STATS | BAD_RANGE            */
  double coord_max_ratio; /* largest coordinate-wise ratio in the layer (see nt_result), else -1                 */
} nt_layer_stats;

/* Alignment, in coordinates, of the partial-sum tiles for J rows (every tile size divides it).  Results are
 * bit-identical for any split of a vector into calls whose boundaries are multiples of this, for the
 * same J, dtype and flags, when each call names the vector's full length in shard->d_global (without shard
 * records: when the parts and the whole are all on one side of the length named at nt_shard_info for that
 * row count, or the row count has none).  The updated w, m, v and a stored gbar never depend on how a vector
 * is cut. */
int64_t normtest_tile_coords(int64_t J);

/* Bytes of device workspace normtest_step needs for J rows of d coordinates (0 if J or d is invalid): a 256-byte
 * record of the step and a few doubles per tile of coordinates (about 0.01 byte per coordinate). */
size_t normtest_workspace_bytes(int64_t J, int64_t d);

/* The same for a known gradient dtype and nt_hyper.flags: what normtest_step (and the other step entry points)
 * check for exactly that call.  Equal to normtest_workspace_bytes(J, d) for every valid dtype and flag word (the
 * two differed while many-row steps kept gbar in the workspace); 0 if an argument is invalid. */
size_t normtest_workspace_bytes_for(nt_dtype gdtype, int64_t J, int64_t d, uint32_t flags);

/*
 * One step.  Row j of the gradients starts at element j*ld of `grads` (device; ld >= d; elements of
 * type gdtype).  w, m, v: device fp32[d], updated in place when NT_DO_ADAMW (may be NULL otherwise).
 * gbar_out: device fp32[d], written when NT_WRITE_GBAR, else ignored.  hyper, shard: host pointers,
 * read before returning (shard may be NULL).  workspace: device scratch of at least
 * normtest_workspace_bytes_for(gdtype, J, d, hyper->flags) bytes, 8-byte aligned; contents irrelevant before; afterwards it holds the
 * call's per-tile partial sums in a private format, which only normtest_layer_stats reads.
 * result_dev: device or pinned-host nt_result, 8-byte aligned, written by the last kernel.
 * hip_stream: a hipStream_t (NULL = the default stream).
 *
 * Everything is enqueued on the stream; the result and the updated state are valid once the caller
 * has synchronised it.  A call enqueues kernel launches only (no memsets, copies or allocations): a long vector
 * is walked by several launches of the same kernel over consecutive runs of tiles (about one per 1.3e8
 * coordinates up to 16 rows, one per 8e6 beyond; the memory system serves blocks that start together faster),
 * followed by one or two small reduction kernels; results do not depend on how many launches there were.  Any pointer alignment is accepted: rows, w, m, v (and gbar_out) that are not
 * all 16-byte aligned take a slower path with bit-identical results.  d == 0 succeeds (sums are 0).
 * AdamW is fused into the same pass: it has been applied even if status reports NONFINITE.
 * Returns NT_OK or a negative code; on any error nothing was enqueued and no buffer was touched,
 * except that a failing launch (HIP code returned) may follow launches that already succeeded.
 */
int normtest_step(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld,
                  float* w, float* m, float* v, float* gbar_out,
                  const nt_hyper* hyper, const nt_shard_info* shard,
                  void* workspace, size_t workspace_bytes,
                  nt_result* result_dev, void* hip_stream);

/*
 * The same step for gradient rows that are separate allocations (one buffer per worker or micro-batch,
 * Sec. 3.2): grad_rows_dev is a device-resident array of J device pointers (8-byte aligned), row j
 * holding at least d elements of type gdtype.  The table is read by the kernels, never by the host; rows
 * that are not all 16-byte aligned take the slower path, with bit-identical results.  Everything else
 * as in normtest_step; for the same rows the two calls return the same bits.
 */
int normtest_step_rows(const void* const* grad_rows_dev, nt_dtype gdtype, int64_t J, int64_t d,
                       float* w, float* m, float* v, float* gbar_out,
                       const nt_hyper* hyper, const nt_shard_info* shard,
                       void* workspace, size_t workspace_bytes,
                       nt_result* result_dev, void* hip_stream);

/*
 * normtest_step for callers that cannot allocate or hand over a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels and results (bit for bit) as
 * normtest_step, without `workspace`: the tile partial sums and the record of the step go to a 16 MiB array that
 * the library holds in each GPU's memory (a static __device__ array; no hipMalloc, hipFree or other allocating
 * call is made here, on any path).  Limits: d <= normtest_static_max_coords(J) (about 1.7e9 coordinates up to
 * 16 rows, 0.86e9 beyond), else NT_ERR_TOO_LARGE and nothing is enqueued.  The array keeps the last call's contents;
 * nothing in it has to be cleared between calls.  All calls on one GPU share it: two calls that overlap in time
 * on the same GPU (different streams, or graphs replayed concurrently) race and give wrong statistics; calls on
 * one stream, or ordered by events, are fine.  normtest_layer_stats cannot follow this call (it needs the
 * caller's workspace).
 */
int normtest_step_static(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld,
                         float* w, float* m, float* v, float* gbar_out,
                         const nt_hyper* hyper, const nt_shard_info* shard,
                         nt_result* result_dev, void* hip_stream);

/* Largest d that normtest_step_static accepts for J rows (0 if J is invalid). */
int64_t normtest_static_max_coords(int64_t J);

/*
 * Host-side combination of n per-shard partial results (all host memory), Sec. 3.3 / Appendix A:
 * gradients of the shards are concatenated, so A, B, C add.  Sums (with their low parts) are added in
 * shard order in double-double arithmetic, then the same decision as in normtest_step is taken in
 * fp64 with `hyper` (eta, b_k, b_max, round_to, ddof; flags ignored).  Status bits of the parts are
 * OR-ed (minus PARTIAL_ONLY); coord_fail adds up and coord_max_ratio is the largest of the parts (both -1 if a part
 * lacks them).  Returns NT_OK or NT_ERR_BAD_ARG.
 */
int normtest_combine(const nt_result* partials, int32_t n, int64_t J, const nt_hyper* hyper,
                     nt_result* out);

/*
 * Gradient-clipped step in two phases.  The paper's runs clip the global gradient norm (Sec. 5, training
 * specifications; hyper-parameter tables: "gradient clipping 1.0"); Alg. 1 omits it and the paper gives no
 * formula, so the usual convention is taken: gbar is scaled by c = min(1, max_norm / (||gbar|| + 1e-6)).
 * ||gbar|| is only known after the whole statistics pass, so this cannot be one pass:
 *   phase 1  statistics as in normtest_step, and gbar (fp32) stored to gbar_buf;
 *   phase 2  AdamW on c * gbar, with c read from result_dev on the device (no host round trip).
 * Arguments as in normtest_step; gbar_buf: device fp32[d], required; max_norm > 0 (<= 0: no clipping,
 * c = 1, and w, m, v come out bit-identical to normtest_step).  hyper->flags must contain NT_DO_STATS and
 * NT_DO_ADAMW and not NT_PARTIAL (a shard cannot know the global norm: see normtest_adamw_gbar).
 * The test statistic uses the unclipped gbar.  result_dev->clip_coef reports c.
 */
int normtest_step_clipped(const void* grads, nt_dtype gdtype, int64_t J, int64_t d, int64_t ld,
                          float* w, float* m, float* v, float* gbar_buf, double max_norm,
                          const nt_hyper* hyper, const nt_shard_info* shard,
                          void* workspace, size_t workspace_bytes,
                          nt_result* result_dev, void* hip_stream);

/*
 * Phase 2 on its own: AdamW (Alg. 1's update lines) on scale * gbar for a mean gradient that is already in
 * device memory (gbar: fp32[d], e.g. written by an earlier NT_WRITE_GBAR call).  scale = grad_scale, times
 * result_dev->clip_coef if result_dev (device or pinned host) is not NULL.  FSDP use: each shard runs
 * normtest_step with NT_DO_STATS | NT_PARTIAL | NT_WRITE_GBAR, the host combines the partial sums, computes
 * normtest_clip_coef and passes it here as grad_scale.  Only the AdamW fields and the step of hyper are read.
 */
int normtest_adamw_gbar(const float* gbar, int64_t d, float* w, float* m, float* v,
                        const nt_hyper* hyper, double grad_scale, const nt_result* result_dev,
                        void* hip_stream);

/*
 * Per-layer table of the statistics: A, B, C of Sec. 3.2 / Alg. 1 and the resulting T, each restricted to a
 * block of consecutive coordinates (a parameter tensor).  The paper tests the whole vector only; nothing here
 * feeds the batch-size decision.  Call it after normtest_step, normtest_step_rows or normtest_step_clipped,
 * on the same stream, with the same gradients (unchanged since), gdtype, J, d, ld and workspace: the tile
 * partial sums which that step left in the workspace are regrouped, and only the pieces of a layer that cover
 * part of a tile are recomputed from the rows (at most two tiles' worth per layer).  eta, b_k, ddof and the
 * coordinate-wise threshold are those of that step.
 *   grads            as in normtest_step, or (rows_are_table != 0) the pointer table of normtest_step_rows
 *   layer_offsets_dev  device int64[L+1], ascending, layer l = coordinates [offsets[l], offsets[l+1]);
 *                    layers need not cover the vector and may be empty.  Read by the kernel only: offsets
 *                    outside [0, d] or descending are clamped and the layer is flagged NT_STATUS_BAD_RANGE.
 *   layers_dev       device or pinned-host nt_layer_stats[L], 8-byte aligned
 * If the workspace does not hold the partial sums of a statistics step with the same gdtype, J and d, every
 * layer comes back with NaN sums and NT_STATUS_NO_STATS.  After an NT_PARTIAL step the sums cover this
 * shard's part of each layer (they add over shards); T is then that part's own.
 * Returns NT_OK or a negative code; on error nothing was enqueued.
 */
int normtest_layer_stats(const void* grads, int rows_are_table, nt_dtype gdtype, int64_t J, int64_t d,
                         int64_t ld, const int64_t* layer_offsets_dev, int32_t L, const void* workspace,
                         nt_layer_stats* layers_dev, void* hip_stream);

/* Host helper: min(1, max_norm / (sqrt(gbar_sq) + 1e-6)); 1 if max_norm <= 0. */
double normtest_clip_coef(double gbar_sq, double max_norm);

/*
 * Host helper: split a global batch size b (for instance nt_result.next_b) over J workers, accumulation
 * steps and a bounded micro-batch (the hyper-parameter tables list a base and a maximum micro-batch size
 * and a base number of accumulation steps; Alg. 1 itself keeps the number of steps fixed).  Keeps
 * accum_base steps while the micro-batch fits under micro_max, otherwise uses the fewest steps for which
 * it fits:  accum = max(accum_base, ceil(b / (J micro_max))),  micro = ceil(b / (J accum)),
 * global_batch = J accum micro >= b.  Returns NT_OK or NT_ERR_BAD_ARG.
 */
int normtest_resplit(int64_t b, int64_t J, int64_t accum_base, int64_t micro_max,
                     int64_t* micro, int64_t* accum, int64_t* global_batch);

/*
 * Host helper: the flags for step `step` (k >= 1) under the two scheduling rules of Sec. 5 (training
 * specifications; "Test interval" in the hyper-parameter tables): the test runs at a fixed interval of steps,
 * and not at all once the global batch size has reached its maximum.  Returns `flags` unchanged when step k
 * tests, i.e. when (k - 1) % test_interval == 0 and not (b_max > 0 and b_k >= b_max); otherwise `flags` without
 * NT_DO_STATS, NT_PARTIAL and NT_COORD_TEST, so that normtest_step runs the mean + AdamW pass only (0 if nothing
 * is left to do).  Invalid arguments (step < 1, test_interval < 1, b_k < 1, b_max < 0) return `flags` unchanged.
 */
uint32_t normtest_schedule_flags(int64_t step, int64_t test_interval, int64_t b_k, int64_t b_max,
                                 uint32_t flags);

/* Plain streaming copy of `bytes` bytes (device to device, 16-byte aligned, bytes % 16 == 0) with the
 * same load/store instructions as the step kernel: a yardstick for achievable HBM bandwidth and for
 * scaling hardware byte counters.  Enqueued on the stream. */
int normtest_calib_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * Yardstick for mixes of streams.  Walks, in step, `row_reads` read streams of 2 bytes per coordinate (8 bytes
 * per lane, like the bfloat16 gradient rows), `reads` read streams and `writes` written streams of 4 bytes per
 * coordinate (16 bytes per lane, like w, m, v; rmw != 0: each written stream is read first, as an in-place
 * update does), over `coords` coordinates (a multiple of 4) with the step kernel's load/store instructions and
 * block shape and no arithmetic.  Time it to see what HBM gives for a given mix, e.g. 8 row reads + 3 in-place
 * streams (the fused step at J = 8), or R reads x W writes.  buf: device scratch, 16-byte aligned, of at least
 * row_reads * r2 + (reads + writes) * r4 + 16 bytes, r2 = coords * 2 and r4 = coords * 4 each rounded up to a
 * multiple of 256; contents are irrelevant and are overwritten.  Supported mixes (else NT_ERR_UNSUPPORTED):
 * row_reads = 0 with reads in {0, 1, 2, 4, 8, 11} and writes in {0..3} (not both 0), rmw = 0; 1 or 3 in-place
 * streams alone; row_reads in {4, 8, 16} alone or with 3 in-place streams; 8 row reads + 1 write; 8 row reads +
 * 3 reads + 3 writes.  launch_coords > 0 (a multiple of 4): the walk is split into kernel launches of that many
 * coordinates each (rounded down to whole 4096-coordinate blocks), the way normtest_step walks a long vector;
 * 0: one launch.  Enqueued on the stream.
 */
int normtest_calib_streams(void* buf, size_t buf_bytes, int64_t coords, int row_reads, int reads, int writes,
                           int rmw, int64_t launch_coords, void* hip_stream);

/* Static, human-readable text for a return code. */
const char* normtest_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* NORMTEST_H */
