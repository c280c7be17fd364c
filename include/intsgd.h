/*
 * intsgd.h -- C ABI of the IntSGD compression hot path for AMD MI355X (gfx950).
 *
 * One IntSGD step (arXiv 2102.08374, Algorithm 1; block form: Algorithm 2 of
 * Appendix A.1) for n workers whose fp32 gradients live in ONE device memory:
 *
 *   a1 scale      t = alpha_k * g_i^k[j]                 (Algorithm 1, "scale and round")
 *   a2 round      Int(t), randomized (Section 2) or nearest-even (Section 5.1)
 *   a3 clip       saturate to [-L, L] and count          (Section 5.1)
 *   a4 aggregate  S[j] = sum_i q_i[j]                     (Algorithm 1, aggregation line;
 *                                                         stands in for the integer all-reduce)
 *   a5 decode     g~[j] = S[j] / (n alpha_k)              (Algorithm 1, estimator line)
 *   a6 update     x[j] <- x[j] - eta_k g~[j]              (Algorithm 1, update line)
 *   a7 norm       ||x^{k+1} - x^k||^2 (per block)         (Algorithm 1 / 2, moving-average line)
 *   a8 next alpha r <- beta r + (1-beta)||.||^2, alpha    (Section 4.1, Proposition 2; Algorithm 2)
 *
 * Conventions that hold for every entry point
 *   - "DEVICE" pointers address memory of the current HIP device; "HOST" pointers
 *     address ordinary host memory.  The caller owns every buffer; the library
 *     never frees or keeps a caller's pointer after the call returns.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and is asynchronous: results are in device memory once
 *     the stream reaches that point.  Nothing synchronises with the host.
 *   - Arguments are validated BEFORE anything is enqueued; on any error status
 *     nothing was launched and no output was touched.
 *   - Vectors of d coordinates must be 16-byte aligned (int8 vectors too).
 *   - Saturation and non-finite gradients are data conditions: they are counted
 *     in sat_count, never turned into an error.
 *   - The only library-owned device memory is a small per-partition tile table
 *     that is built the first time a descriptor with num_blocks > 1 is used (or
 *     by intsgd_prepare) and freed by intsgd_release().  Descriptors with
 *     num_blocks == 1 need none.
 *   - A workspace needs no initialisation and holds nothing between calls.  Calls
 *     on different streams that share a workspace race; give each concurrent call
 *     its own workspace.
 *   - For full bandwidth give every vector a 128-byte aligned start (only 16 is
 *     required).
 *   - The library keeps no tuning or profiling state of its own: what a call launches
 *     depends on its arguments only (the descriptor's optional `launch` options
 *     included), so callers in one process cannot disturb each other.
 */
#ifndef INTSGD_H_
#define INTSGD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility: the functions marked INTSGD_API are its
 * whole dynamic symbol table. */
#define INTSGD_API __attribute__((visibility("default")))

typedef enum {
  INTSGD_OK = 0,
  INTSGD_EINVAL = -1,     /* null pointer, zero size, bad enum, eta/beta/eps out of range */
  INTSGD_EALIGN = -2,     /* a vector pointer is not 16-byte aligned */
  INTSGD_ERANGE = -3,     /* clip bound or worker count outside what the wire / int32 sum can hold */
  INTSGD_EHIP = -4,       /* a HIP runtime call failed (see intsgd_last_hip_error) */
  INTSGD_EWORKSPACE = -5, /* workspace missing, misaligned or smaller than intsgd_workspace_bytes */
  INTSGD_ENOPLAN = -6     /* a call that must not allocate met a partition (num_blocks > 1) whose
                             tile table intsgd_prepare has not built on this device */
} intsgd_status;

typedef enum {
  INTSGD_ROUND_NEAREST_EVEN = 0, /* Section 5.1: deterministic rounding, ties to even */
  INTSGD_ROUND_STOCHASTIC = 1    /* Section 2: Int(t) = floor(t)+1 w.p. t-floor(t) */
} intsgd_rounding;

typedef enum {
  INTSGD_WIRE_INT8 = 8,  /* per-worker integer vectors are int8_t  (clip <= 127) */
  INTSGD_WIRE_INT32 = 32 /* per-worker integer vectors are int32_t */
} intsgd_wire;

#define INTSGD_MAX_WORKERS 128u

/*
 * Optional launch options of the calls made with a descriptor (intsgd_desc.launch; NULL or a
 * zero field = automatic: the library picks per call what measured best on MI355X).  They
 * are not part of the numerical contract: results do not depend on them except for the
 * summation order of the norm.  Read during the call only.
 *   tile_coords        coordinates per work tile, a multiple of 1024 in [1024, 65536]
 *                      (automatic: per kernel, 1024 to 16384; the sweeps over the n gradient
 *                      streams take 8192 at n = 1, 4096 up to n = 5, else 2048)
 *   max_workgroups     cap of the launch grid, in [1, 1048576]; tiles beyond it are
 *                      taken by striding
 *   workgroups_per_cu  residency cap of the streaming kernels, 2..8 (8 = no cap)
 *   two_phase          form of the sweeps that have one (intsgd_step_fused, .._next_alpha,
 *                      intsgd_step_momentum, intsgd_compress_sum; one block, d >= 2^22):
 *                      1 = always the tile sweep, 2 = always the two-phase sweep (gradient
 *                      reads, then the write-back, with the integer sums held in registers
 *                      in between), 0 = automatic (the tile sweep: it measured as fast or
 *                      faster for every worker count).
 *                      intsgd_int_sum follows it too: automatic = two-phase for any wire
 *                      (d >= 2^22), 1 = its tile form
 *   start_event, stop_event   profiling aid: hipEvent_t handles passed as void*, both set or
 *                      both NULL.  When set, the call attaches them to the dispatch of its
 *                      streaming kernel on the call's stream (not to the small final-sum
 *                      kernel behind it), so that hipEventElapsedTime(start, stop) is that
 *                      kernel's duration.
 * An out-of-range field makes every call with the descriptor return INTSGD_EINVAL.
 */
typedef struct intsgd_launch_opts {
  uint32_t tile_coords;
  uint32_t max_workgroups;
  uint32_t workgroups_per_cu;
  uint32_t two_phase;
  void* start_event;
  void* stop_event;
} intsgd_launch_opts;

/*
 * Problem statement shared by all calls.
 *   d, n        model dimension and number of workers (Section 1, eq. (1)); d > 0,
 *               1 <= n <= INTSGD_MAX_WORKERS.
 *   num_blocks  B >= 1.  B == 1 is Algorithm 1 (one alpha for the whole vector);
 *               B > 1 is Algorithm 2 (one alpha per block).
 *   block_offsets  HOST array of B+1 coordinate offsets, [0] = 0, [B] = d, strictly
 *               increasing; may be NULL when B == 1.  Read during the call only.
 *   rounding    a2.  wire: storage type of the per-worker integer vectors (a3).
 *   clip        L >= 1: rounded values saturate to [-L, L].  Required:
 *               n * L <= INT32_MAX so the int32 aggregate is the exact sum, and
 *               L <= 127 when wire is INT8.
 *   seed, step  randomized rounding draws, for worker i and GLOBAL coordinate j,
 *               word (j mod 4) of Philox4x32-10 at counter
 *               (lo32(j/4), hi32(j/4), i, step) with key (lo32(seed), hi32(seed));
 *               the top 24 bits u of the word decide: round up iff u 2^-24 < t - floor(t).
 *   launch      HOST pointer to launch options, or NULL (automatic).
 */
typedef struct intsgd_desc {
  uint64_t d;
  uint32_t n;
  uint32_t num_blocks;
  const uint64_t* block_offsets;
  int32_t rounding; /* intsgd_rounding */
  int32_t wire;     /* intsgd_wire */
  int32_t clip;
  uint32_t step;
  uint64_t seed;
  const intsgd_launch_opts* launch;
  /* Optional output, DEVICE uint32_t[B] (4-byte aligned) or NULL.  The calls whose sweep forms
   * the aggregate S (intsgd_compress_sum, intsgd_step_fused, intsgd_step_fused_next_alpha,
   * intsgd_step_fused_static, intsgd_step_momentum, intsgd_diana_step) overwrite it with
   * max_j |S_j| over each block's coordinates: the largest integer in the aggregated vector,
   * which Appendix A.2 reports per iteration.  Every other call ignores it. */
  uint32_t* largest_sum;
} intsgd_desc;

/* Bytes of DEVICE scratch (256-byte aligned) that any entry point taking a
 * workspace needs for this descriptor; 0 if the descriptor is invalid. */
INTSGD_API size_t intsgd_workspace_bytes(const intsgd_desc* desc);

/* Validates the descriptor and builds the library's tile table for its partition
 * now (the only call that may allocate device memory), so that later calls on
 * this partition only enqueue kernels.  Optional. */
INTSGD_API intsgd_status intsgd_prepare(const intsgd_desc* desc);

/* Frees every cached tile table on every device.  Must not run concurrently with
 * other calls. */
INTSGD_API void intsgd_release(void);

/*
 * a1-a3 (Algorithm 1 "scale and round the local gradient"; Algorithm 2 with B > 1).
 *   grads     HOST array of n DEVICE pointers, each d floats (read only).
 *   alpha     DEVICE float[B], alpha_k (per block).
 *   q_out     HOST array of n DEVICE pointers, each d int8_t or int32_t per desc->wire.
 *   sat_count DEVICE uint64_t[n], overwritten: clipped or non-finite coordinates per worker.
 */
INTSGD_API intsgd_status intsgd_compress(const intsgd_desc* desc, const float* const* grads,
                              const float* alpha, void* const* q_out, uint64_t* sat_count,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * a4 (Algorithm 1 aggregation line, on one device): sum_out[j] = sum_i q[i][j].
 *   q        HOST array of n DEVICE pointers to int8_t or int32_t vectors (desc->wire).
 *   sum_out  DEVICE int32_t[d].  Exact whenever |q| <= desc->clip.
 */
INTSGD_API intsgd_status intsgd_int_sum(const intsgd_desc* desc, const void* const* q, int32_t* sum_out,
                             void* hip_stream);

/*
 * a5-a6 (Algorithm 1 estimator and update lines): in fp64 per coordinate,
 * c = eta / (n alpha), x <- fl32(x - c S).
 *   sum         DEVICE int32_t[d];  alpha DEVICE float[B];  eta > 0 finite.
 *   x           DEVICE float[d], updated in place.
 *   gtilde_out  DEVICE float[d] or NULL: g~ = fl32(S / (n alpha)).
 */
INTSGD_API intsgd_status intsgd_decode_update(const intsgd_desc* desc, const int32_t* sum,
                                   const float* alpha, double eta, float* x, float* gtilde_out,
                                   void* hip_stream);

/*
 * a7 (Algorithm 1 / 2 moving-average line's norm): norm_sq_out[l] =
 * sum over block l of (x_new[j] - x_old[j])^2, fp64 accumulation of the stored
 * fp32 iterates.  norm_sq_out: DEVICE double[B], overwritten.
 */
INTSGD_API intsgd_status intsgd_update_norm(const intsgd_desc* desc, const float* x_new, const float* x_old,
                                 double* norm_sq_out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream);

/*
 * a8 (Section 4.1, Proposition 2; Algorithm 2 for B > 1), fp64:
 *   r[l] <- beta r[l] + (1-beta) norm_sq[l]
 *   B == 1: alpha = sqrt(d) / sqrt(2 n r / eta^2 + eps^2)
 *   B  > 1: alpha_l = eta sqrt(d_l) / sqrt(2 n r_l + eta^2 (d_l/d) eps^2)
 *   norm_sq DEVICE double[B]; r DEVICE double[B] in/out; alpha_out DEVICE float[B].
 *   0 <= beta < 1, eps >= 0, eta > 0.  A zero denominator (r = 0 and eps = 0)
 *   yields alpha = +Inf on the device: every coordinate then saturates and is counted.
 */
INTSGD_API intsgd_status intsgd_next_alpha(const intsgd_desc* desc, const double* norm_sq, double* r,
                                double beta, double eps, double eta, float* alpha_out,
                                void* hip_stream);

/* Host twin of intsgd_next_alpha: same arithmetic on HOST arrays, no device
 * involved.  Returns INTSGD_ERANGE (and still writes +Inf) on a zero denominator. */
INTSGD_API intsgd_status intsgd_next_alpha_host(const intsgd_desc* desc, const double* norm_sq, double* r,
                                     double beta, double eps, double eta, float* alpha_out);

/*
 * F1 = a1-a4 in one pass over the n gradient streams: sum_out DEVICE int32_t[d],
 * sat_count DEVICE uint64_t[n].  Bit-identical to intsgd_compress + intsgd_int_sum.
 */
INTSGD_API intsgd_status intsgd_compress_sum(const intsgd_desc* desc, const float* const* grads,
                                  const float* alpha, int32_t* sum_out, uint64_t* sat_count,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * F2 = a5-a7 in one pass over S and x: x updated in place, norm_sq_out DEVICE
 * double[B] = ||x_new - x_old||^2 per block.  Same x as intsgd_decode_update.
 */
INTSGD_API intsgd_status intsgd_decode_update_norm(const intsgd_desc* desc, const int32_t* sum,
                                        const float* alpha, double eta, float* x,
                                        double* norm_sq_out, void* workspace,
                                        size_t workspace_bytes, void* hip_stream);

/*
 * F3 = a1-a7 in a single sweep (the aggregate never leaves registers; legal on one
 * device because no real all-reduce separates a4 from a5).  Same x, norms and
 * counts as F1 followed by F2.
 */
INTSGD_API intsgd_status intsgd_step_fused(const intsgd_desc* desc, const float* const* grads,
                                const float* alpha, double eta, float* x, double* norm_sq_out,
                                uint64_t* sat_count, void* workspace, size_t workspace_bytes,
                                void* hip_stream);

/*
 * The whole step in one call: F3, whose small final-sum kernel also applies a8
 * (Section 4.1 / Algorithm 2).  alpha: DEVICE float[B], read as alpha_k during the
 * sweep and overwritten with alpha_{k+1} afterwards; r: DEVICE double[B] in/out;
 * norm_sq_out, sat_count as in intsgd_step_fused.  eta is eta_k, the stepsize of this
 * step's update; eta_next is eta_{k+1}, the stepsize that Algorithm 1's scaling-factor
 * line pairs with alpha_{k+1} (equal to eta under a constant stepsize).  Same results as
 * intsgd_step_fused(eta) followed by intsgd_next_alpha(eta_next).
 */
INTSGD_API intsgd_status intsgd_step_fused_next_alpha(const intsgd_desc* desc,
                                                      const float* const* grads, float* alpha,
                                                      double eta, double eta_next, float* x,
                                                      double* r, double beta, double eps,
                                                      double* norm_sq_out, uint64_t* sat_count,
                                                      void* workspace, size_t workspace_bytes,
                                                      void* hip_stream);

/*
 * For callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): intsgd_step_fused_next_alpha
 * with its scratch in a static device array of INTSGD_STATIC_SCRATCH_BYTES that every GPU
 * running the library holds until the process ends.  Same arguments (minus the workspace)
 * and the same results.  It calls no hipMalloc / hipFree and no allocating routine.
 *   - The scratch must hold 16 + 8 n bytes per work tile (the automatic tile of the sweep, or
 *     desc->launch->tile_coords), or per compute unit when the call takes the two-phase
 *     form, plus 1 KiB; a larger problem is refused with INTSGD_EWORKSPACE and nothing is
 *     launched.  32 MiB covers d = 8.5e8 at n = 8 (d = 1.3e9 with tile_coords = 4096),
 *     d = 6.6e7 at n = 128 in the tile form, and any d in the two-phase form.
 *   - num_blocks > 1 needs the partition's tile table, which only intsgd_prepare builds:
 *     without it the call returns INTSGD_ENOPLAN.  Calling intsgd_prepare(desc) once per
 *     device beforehand (with the launch options the later calls use) also resolves the
 *     array's address, after which this call only enqueues kernels.
 *   - The array keeps the previous call's contents; nothing in it needs clearing (flags and
 *     the clip hint are tagged per launch).  All calls on one GPU share it: calls that
 *     overlap in time on one GPU (different streams or threads) race; serialise them.
 */
#define INTSGD_STATIC_SCRATCH_BYTES (32u << 20)
INTSGD_API intsgd_status intsgd_step_fused_static(const intsgd_desc* desc, const float* const* grads,
                                                  float* alpha, double eta, double eta_next,
                                                  float* x, double* r, double beta, double eps,
                                                  double* norm_sq_out, uint64_t* sat_count,
                                                  void* hip_stream);

/*
 * Momentum / weight-decay form of the update (the optimizer of the paper's experiments,
 * Appendix C.1: SGD with momentum 0.9 and weight decay 1e-4; PyTorch's SGD rule).  Per
 * coordinate in fp64, every operation rounded on its own, both state vectors in fp32:
 *   g~ = S (1/(n alpha));  dd = g~ + weight_decay x;  m <- fl32(mu m + dd);  x <- fl32(x - eta m).
 * m: DEVICE float[d] in/out (16-byte aligned); 0 <= mu < 1; weight_decay >= 0.
 * norm_sq_out is ||x_new - x_old||^2 per block as everywhere else (it now contains the
 * momentum term).
 *
 * intsgd_decode_update_momentum: F2 with this update (a5-a7 on a given aggregate).
 * intsgd_step_momentum: F3 with this update in one sweep; if r is not NULL, a8 is applied
 * as in intsgd_step_fused_next_alpha (alpha in/out, with eta_next), otherwise alpha is only
 * read and eta_next is ignored.
 */
INTSGD_API intsgd_status intsgd_decode_update_momentum(const intsgd_desc* desc, const int32_t* sum,
                                            const float* alpha, double eta, double mu,
                                            double weight_decay, float* x, float* m,
                                            double* norm_sq_out, void* workspace,
                                            size_t workspace_bytes, void* hip_stream);
INTSGD_API intsgd_status intsgd_step_momentum(const intsgd_desc* desc, const float* const* grads,
                                              float* alpha, double eta, double eta_next, double mu,
                                              double weight_decay, float* x, float* m, double* r,
                                              double beta, double eps, double* norm_sq_out,
                                              uint64_t* sat_count, void* workspace,
                                              size_t workspace_bytes, void* hip_stream);

/*
 * IntDIANA (Appendix A.2, Algorithm 3) in one sweep, for heterogeneous workers: every
 * worker compresses the difference to its local shift and moves the shift by the decoded
 * message; the aggregate is decoded on top of the global shift.
 *   Q_i = Int(alpha (g_i - h_i)) clipped to [-L, L] (counted in sat_count[i]),
 *   h_i <- fl32(h_i + Q_i (1/alpha)),   S = sum_i Q_i,
 *   g~ = h + S (1/(n alpha)),   x <- fl32(x - eta g~),   h <- fl32(g~).
 * fp32 for the difference and the scale, fp64 with every operation rounded on its own for
 * the rest.  (The algorithm box writes h_i + Q(g_i); its analysis uses g = (1/n) sum (h_i +
 * Q(g_i)), i.e. Q carries the 1/alpha there.)
 *   grads    HOST array of n DEVICE pointers (d floats each, read only)
 *   h_local  HOST array of n DEVICE pointers (d floats each, in/out), 16-byte aligned
 *   h        DEVICE float[d], global shift, in/out;  x DEVICE float[d], in/out
 *   r        DEVICE double[B] or NULL.  Not NULL: a8 is applied afterwards (alpha in/out) with
 *            eta_next (the next step's stepsize, which Algorithm 3's scaling-factor line
 *            uses) and the given beta, eps; Algorithm 3's own rule is beta = 0, eps = 0.
 */
INTSGD_API intsgd_status intsgd_diana_step(const intsgd_desc* desc, const float* const* grads,
                                           float* const* h_local, float* alpha, double eta,
                                           double eta_next, float* x, float* h, double* r,
                                           double beta, double eps, double* norm_sq_out,
                                           uint64_t* sat_count, void* workspace,
                                           size_t workspace_bytes, void* hip_stream);

/*
 * Heuristic IntSGD scaling (Section 5.2: the SwitchML rule the paper compares with), which
 * needs a profiling pass over all gradients before they can be compressed:
 *   alpha_l = (2^nb - 1) / (n 2^max_exp),  2^max_exp = smallest power of two >= the largest
 *   finite |g_i[j]| over all n workers and all coordinates j of block l,
 * so that |alpha g| <= (2^nb - 1)/n.  nb in [1, 31] is the number of magnitude bits (7 for
 * an int8 aggregate, 31 for int32).  An all-zero block gets alpha = 1; alpha is capped at
 * the largest finite fp32.  alpha_out: DEVICE float[B].  The result can be passed to any
 * of the compress / step calls in place of the adaptive alpha.
 */
INTSGD_API intsgd_status intsgd_heuristic_alpha(const intsgd_desc* desc, const float* const* grads,
                                     uint32_t nb, float* alpha_out, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);

/* Which form the fused step (intsgd_step_fused, .._next_alpha, intsgd_step_momentum) and
 * intsgd_compress_sum take for this descriptor (its launch options included): 1 = tile
 * sweep, 2 = two-phase sweep; 0 if the descriptor is invalid.  Host-only, launches nothing. */
INTSGD_API int intsgd_fused_step_form(const intsgd_desc* desc);

/* Text of a status code; takes a plain int so that any value is a defined argument
 * ("unknown status" for codes that are not an intsgd_status). */
INTSGD_API const char* intsgd_status_string(int status);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
INTSGD_API const char* intsgd_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* INTSGD_H_ */
