/*
 * apms.h -- C ABI of libapms: the per-step data-parallel hot path of the
 * compression stage of APMSqueeze (error-compensated 1-bit compressed
 * momentum SGD with the Adam variance frozen after a warm-up) for one
 * AMD MI355X (gfx950), n workers simulated as n state slices in HBM.
 *
 * Notation follows the paper (Algorithm 1; Section 3.3; supplement "Proof to
 * the Updating Form"): x model, m momentum, v variance, g^(i) worker i's
 * stochastic gradient, delta^(i) worker i's compression error, deltabar the
 * server's compression error, C[.] the compression operator (here the 1-bit
 * operator of Section 5.1: signs + one l2 scale per chunk).
 *
 * Conventions for every entry point
 *   - Every array argument is a DEVICE pointer owned by the caller, 16-byte
 *     aligned, on the device the context was created for.  The library never
 *     allocates, frees or keeps them (it remembers the ADDRESS of a buffer
 *     left in deferred form, see apms_set_deferral).  Distinct array
 *     arguments of one call must not overlap.
 *   - "[n][d]" is worker-major: worker i's slice starts at element i*d.
 *     d is the (padded) vector length, a multiple of chunk_elems; chunk_elems
 *     is a multiple of 32; C = d / chunk_elems chunks; chunk k is elements
 *     [k*chunk_elems, (k+1)*chunk_elems).  A chunk is the unit that has its own
 *     scale and its own server (Algorithm 1 line 7: the paper uses C = n).
 *   - Sign words: element j of a vector is bit (j & 31) of 32-bit word (j >> 5);
 *     bit 1 means +scale, bit 0 means -scale; sign(+-0) = +1.
 *   - All floating point is IEEE binary32, one rounding per operation, no fused
 *     multiply-add, in the operation order stated per call.  Squared norms are
 *     accumulated in binary64 (exact squares, tree order fixed by the launch
 *     plan) and each scale is rounded to binary32 once.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is queued asynchronously; no compute call allocates, frees or
 *     synchronises the host (the set-up calls apms_create, apms_destroy and
 *     apms_topk_reserve do).  A context serves one stream at a time.  Results are deterministic for a given
 *     context geometry (no floating-point atomics).
 *   - Return value: APMS_OK or a negative apms_status.  Arguments are validated
 *     on the host before anything is launched; on a validation error nothing
 *     was queued.  After APMS_EHIP from a compute call (a launch failed part
 *     way) the call's output buffers are undefined and the context keeps the
 *     deferred state it had before the call.
 *     d == 0 is a valid empty problem: calls validate and return APMS_OK.
 *   - There is no CPU fallback.  A context created with APMS_DEVICE_NONE only
 *     validates: every compute call returns APMS_ENODEV once its arguments
 *     have passed validation.
 */
#ifndef APMS_H
#define APMS_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct apms_ctx apms_ctx;

typedef enum apms_status {
    APMS_OK = 0,
    APMS_EINVAL = -1,  /* null pointer, bad scalar (n < 1, beta outside [0,1), t < 1, ...) */
    APMS_EALIGN = -2,  /* an array pointer is not 16-byte aligned */
    APMS_ESHAPE = -3,  /* chunk_elems not a positive multiple of 32, or d not a multiple of it; n > 4096;
                          a launch grid or a top-k list position that does not fit 31 bits */
    APMS_ENOMEM = -4,  /* host or device allocation of the context's scratch failed */
    APMS_EHIP = -5,    /* a HIP call failed; see apms_last_hip_error */
    APMS_ENODEV = -6,  /* validation-only context: arguments are fine, nothing can run */
    APMS_EALIAS = -7,  /* two array arguments overlap */
    APMS_ESTATE = -8,  /* the call would lose or read state that is pending in deferred form, or a top-k
                          call found no scratch reserved for its K (apms_topk_reserve) */
    APMS_ELIMIT = -9   /* the problem is larger than a fixed-size resource of the call (apms_server_reduce_static) */
} apms_status;

#define APMS_DEVICE_NONE (-1)

/* Element type of 16-bit gradient inputs (apms_compress_g16, apms_warmup_step_g16). */
#define APMS_GRAD_F16 1  /* IEEE binary16 */
#define APMS_GRAD_BF16 2 /* bfloat16: the upper 16 bits of a binary32 */

/* Deferral flags for apms_set_deferral (0 = everything eager, the default). */
#define APMS_DEFER_ERRORS 1 /* error buffers hold the compensated vector u; delta = u - C[u] is formed on next read */
#define APMS_DEFER_GATHER 2 /* apms_apply leaves m untouched; the next apms_compress writes the gathered momentum */
#define APMS_IMPLICIT_MOMENTUM 4 /* with APMS_DEFER_GATHER: that apms_compress does not write m either */

/* Launch geometry of a context (read-only report; see apms_get_plan). */
typedef struct apms_plan {
    int64_t d;
    int32_t n;
    int64_t chunk_elems;
    int64_t chunks;                     /* C */
    /* A tile is the run of consecutive elements of one chunk a workgroup handles per iteration;
       a chunk has ceil(chunk_elems / tile) tiles, the last one possibly ragged. */
    int32_t compress_tile_elems;
    int32_t compress_tiles_per_block;
    int32_t compress_blocks_per_chunk;
    int64_t compress_grid;              /* n * C * compress_blocks_per_chunk workgroups */
    int32_t server_tile_elems;
    int32_t server_tiles_per_block;
    int32_t server_blocks_per_chunk;
    int64_t server_grid;                /* C * server_blocks_per_chunk */
    int32_t apply_tile_elems;
    int64_t apply_grid;                 /* n * C * ceil(chunk_elems / apply_tile_elems) */
    int64_t scratch_bytes;              /* device memory owned by the context */
    int32_t occupancy_pad[8];           /* bytes of unused dynamic LDS per workgroup, by APMS_KERNEL_*;
                                           entries past APMS_KERNEL_COUNT are 0 */
    int64_t topk_scratch_bytes;         /* further device memory apms_topk_reserve has allocated */
    int32_t gather_mode;                /* APMS_GATHER_*, see apms_set_gather_mode */
    int32_t gather_choice;              /* the form in use: APMS_GATHER_SPLIT / _FUSED, or -1 while
                                           APMS_GATHER_AUTO has not decided yet */
    int32_t gather_uncapped;            /* 1 if APMS_GATHER_AUTO chose the fused form without the occupancy cap */
    float gather_ms[3];                 /* APMS_GATHER_AUTO: best time it measured for [split, fused with the worker
                                           kernel capped at two workgroups per CU, fused uncapped] (0 until decided) */
} apms_plan;

/*
 * Create a context for vectors of d elements, n workers and chunks of
 * chunk_elems elements on HIP device `device` (or APMS_DEVICE_NONE).  The
 * context owns its device scratch (binary64 norm partials, pending scales: a few MB,
 * see apms_plan.scratch_bytes; apms_topk_reserve adds the top-k selection's, see below).
 * Errors: EINVAL (out NULL, n < 1, d < 0), ESHAPE (also n > 4096, or so many chunks or tiles that a
 * launch grid would pass 2^31 - 1), ENOMEM, EHIP.
 */
int apms_create(apms_ctx **out, int64_t d, int32_t n, int64_t chunk_elems, int device);

/* Free the context and its scratch.  NULL is accepted. */
int apms_destroy(apms_ctx *ctx);

/* Static English text for a status code. */
const char *apms_strerror(int status);

/* The raw hipError_t behind the last APMS_EHIP of this context (0 if none). */
int apms_last_hip_error(const apms_ctx *ctx);

/* Copy the launch geometry into *plan. */
int apms_get_plan(const apms_ctx *ctx, apms_plan *plan);

/*
 * Tuning knob: how many tiles one workgroup streams in apms_compress and in
 * apms_server_reduce (each >= 1; 0 keeps the current
 * value).  Changes the reduction tree of the norms, hence possibly the last
 * bit of a scale; results stay deterministic for a fixed setting.
 */
int apms_set_tiles_per_block(apms_ctx *ctx, int32_t compress_tiles, int32_t server_tiles);

/*
 * Tuning knob: ask for lds_bytes of dynamic LDS per workgroup of one kernel without using it.  LDS is
 * what caps the number of workgroups a compute unit holds at once at no other cost, and these
 * streaming kernels reach their best HBM efficiency with few workgroups in flight per CU.
 * 0 <= lds_bytes <= 128 KB, or APMS_PAD_AUTO for APMS_KERNEL_COMPRESS (its default: the library
 * picks by variant of the worker kernel).  Does not change any result.
 */
#define APMS_KERNEL_COMPRESS 0
#define APMS_KERNEL_SERVER 1
#define APMS_KERNEL_APPLY 2
#define APMS_KERNEL_FINALIZE 3
#define APMS_KERNEL_WARMUP 4
#define APMS_KERNEL_COUNT 5
#define APMS_PAD_AUTO (-1)
int apms_set_occupancy_pad(apms_ctx *ctx, int kernel, int32_t lds_bytes);

/*
 * Tuning knob: how the apms_compress that finds a gather pending on m (APMS_DEFER_GATHER) writes the n
 * momentum slices.  Same bytes moved, same results, bit for bit.
 *   APMS_GATHER_SPLIT   a fill of its own writes m[n][d], then the worker kernel runs without touching m.
 *                       Its speed does not depend on where the caller's buffers lie.
 *   APMS_GATHER_FUSED   the worker kernel writes m itself, next to the error buffer: two write streams in one
 *                       kernel.  On MI355X about 6 % faster than the split form when m lies in a different
 *                       third of the HBM address range than worker_err and g, and about 8 % slower when they
 *                       share one (which is where successive allocations of a new process land).
 *   APMS_GATHER_AUTO    (default) the context finds out which is faster for the buffers it is given: its
 *                       first gather runs split, the next six cycle through split / fused / fused without
 *                       the worker kernel's occupancy cap and are timed with events on the caller's stream,
 *                       and the first later call that finds those events complete (it never waits) fixes
 *                       the fastest form for the rest of the context's life; until then, and on a stream
 *                       under graph capture, the split form is used.
 *                       apms_plan.gather_choice and gather_ms report the outcome.  Setting a mode again
 *                       starts this over.
 */
#define APMS_GATHER_SPLIT 0
#define APMS_GATHER_FUSED 1
#define APMS_GATHER_AUTO 2
int apms_set_gather_mode(apms_ctx *ctx, int mode);

/*
 * Deferral: software pipelining of two writes across the step boundary.  Results are bit-identical to
 * the eager ones; what changes is WHEN a caller-owned buffer holds its final value.
 *
 * APMS_DEFER_ERRORS.  The new error delta' = u - C[u] (Section 3.1; supplement steps 1-2) needs the
 * scale of the WHOLE chunk, known only after the chunk has been streamed once.  Eagerly, a second pass
 * over the error buffer forms delta' before the call's work ends.  Deferred, the call stores the
 * compensated vector u in the error buffer and the context keeps the chunk scales; the next
 * apms_compress / apms_server_reduce on the SAME buffer forms delta' = u - (u >= 0 ? +s : -s) while
 * reading it (one binary32 subtraction of the same operands), saving one read and one write of the
 * buffer per step.
 *
 * APMS_DEFER_GATHER.  Eagerly, apms_apply writes the decoded server message to all n momentum slices
 * (Algorithm 1 line 10) and the next apms_compress reads them back.  Deferred, apms_apply only takes
 * the model step and remembers `spacked` (by address) and the server scales (by value); the next
 * apms_compress on the SAME m decodes the sign words itself, WRITES the n momentum slices and uses the
 * decoded values in place of reading m: the momentum state is still materialised in m[n][d] every step,
 * it is just not read back.  Until then `spacked` must stay untouched (apms_server_reduce with that
 * address is refused).
 *
 * APMS_IMPLICIT_MOMENTUM (only together with APMS_DEFER_GATHER; EINVAL otherwise).  The momentum is
 * kept ONLY as the server's sign words and scales: the apms_compress that consumes a pending gather
 * decodes them and writes nothing to m, so m[n][d] is never touched by a step (4n fewer bytes written
 * per parameter).  This departs from a state model in which every worker holds its fp32 momentum in memory:
 * m is defined only if apms_finalize(m) is called between apms_apply and the next apms_compress.
 *
 * While a buffer is pending its contents are not final: call apms_finalize before reading it
 * (checkpoint, test) or before handing a different buffer to the same context; a call that would lose
 * or read pending state returns APMS_ESTATE.
 */
int apms_set_deferral(apms_ctx *ctx, int flags);

/*
 * Bring pending buffers to their final contents: the paper's delta in worker_err / server_err, the
 * gathered momentum in m.  Any pointer may be NULL (skip).  A buffer that is not pending is untouched.
 *   worker_err [n][d], server_err [d], m [n][d].
 */
int apms_finalize(apms_ctx *ctx, float *worker_err, float *server_err, float *m, void *stream);

/*
 * Warm-up: one step of the original Adam (Section 3.2; Algorithm 1 line 2)
 * on the full-precision average of the n workers' gradients.
 *   gbar = (sum_{i=0}^{n-1} g_i) * fl(1/n)                (worker order)
 *   m <- fl(beta1*m) + fl(fl(1-beta1)*gbar)
 *   v <- fl(beta2*v) + fl(fl(1-beta2)*fl(gbar*gbar))
 *   x <- x - lr * (m / bc1) / (sqrt(v / bc2) + eps),  bc = 1 - beta^t formed in
 *        binary64 on the host and rounded to binary32
 *   x, m, v [d] in/out;  g [n][d] in;  t >= 1 is the 1-based step index.
 * Errors: EINVAL (beta1, beta2 outside [0,1), t < 1, null), EALIGN, EALIAS.
 */
int apms_warmup_step(apms_ctx *ctx, float *x, float *m, float *v, const float *g,
                     float lr, float beta1, float beta2, float eps, int64_t t, void *stream);

/*
 * The same step with 16-bit gradients (Section 5.1 trains with 16-bit floating-point values): g is [n][d]
 * binary16 or bfloat16 values (grad_format = APMS_GRAD_F16 / APMS_GRAD_BF16).  Every value is widened
 * to binary32 exactly, then the arithmetic is that of apms_warmup_step.  EINVAL for another format.
 */
int apms_warmup_step_g16(apms_ctx *ctx, float *x, float *m, float *v, const uint16_t *g, int grad_format,
                         float lr, float beta1, float beta2, float eps, int64_t t, void *stream);

/*
 * Hand-over from warm-up to the compression stage (Algorithm 1, line 1
 * initial errors = 0, and line 3): replicate worker 0's momentum slice to all
 * n slices and zero both error buffers; v is frozen simply by no longer
 * calling apms_warmup_step.  Clears any pending deferred state.
 *   m [n][d]: slice 0 in, all slices out;  worker_err [n][d], server_err [d] out.
 */
int apms_freeze(apms_ctx *ctx, float *m, float *worker_err, float *server_err, void *stream);

/*
 * Worker side of one compressed step (Algorithm 1 lines 6-7; supplement
 * step 1), for all n workers and all C chunks:
 *   u      = (fl(beta*m_i) + fl(fl(1-beta)*g_i)) + delta_i
 *   scale  = fl32( sqrt( sum_chunk u^2 / chunk_elems ) )        (Section 5.1)
 *   bit    = (u >= 0)
 *   delta_i <- u - (bit ? +scale : -scale)
 *   m           [n][d] in (written only when a deferred gather is pending on it)
 *   g           [n][d] in (the local momentum m_t^(i) is not stored: the gather overwrites m)
 *   worker_err  [n][d] in/out
 *   packed      [n][d/32] out, sign words
 *   scales      [n][C] out
 * With a gather pending on m (APMS_DEFER_GATHER) the kernel decodes the pending server message,
 * writes it to m and uses it as m_i; otherwise m is read only.
 * Errors: EINVAL (beta outside [0,1), null), EALIGN, EALIAS, ESTATE, EHIP.
 */
int apms_compress(apms_ctx *ctx, float *m, const float *g, float *worker_err,
                  uint32_t *packed, float *scales, float beta, void *stream);

/*
 * apms_compress with 16-bit gradients: g is [n][d] binary16 or bfloat16 values, widened to binary32
 * exactly before the same arithmetic; everything else as apms_compress (2n fewer bytes read per
 * parameter).  EINVAL for another format.
 */
int apms_compress_g16(apms_ctx *ctx, float *m, const uint16_t *g, int grad_format, float *worker_err,
                      uint32_t *packed, float *scales, float beta, void *stream);

/*
 * Server side (Algorithm 1 line 9; supplement step 2), for all C chunks:
 *   a      = (sum_{i=0}^{n-1} (bit_i ? +scale_i : -scale_i)) * fl(1/n)
 *   ubar   = a + deltabar
 *   sscale = fl32( sqrt( sum_chunk ubar^2 / chunk_elems ) );  sbit = (ubar >= 0)
 *   deltabar <- ubar - (sbit ? +sscale : -sscale)
 *   packed [n][d/32], scales [n][C] in (as written by apms_compress)
 *   server_err [d] in/out;  spacked [d/32] out;  sscales [C] out.
 */
int apms_server_reduce(apms_ctx *ctx, const uint32_t *packed, const float *scales,
                       float *server_err, uint32_t *spacked, float *sscales, void *stream);

/*
 * apms_server_reduce for callers that cannot allocate device memory or hold a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (plus the geometry a
 * context would carry), same kernels and same results, bit for bit, as apms_server_reduce on a newly
 * created context in eager mode: server_err, spacked and sscales are final when the queued work ends.
 * The binary64 norm partials go to a fixed array of APMS_STATIC_SCRATCH_BYTES that is part of the library's
 * device image (each GPU the library runs on holds its own copy until the process ends); nothing is
 * allocated, freed or synchronised by the call.
 *   - Runs on the calling thread's CURRENT HIP device; every array must live on it.
 *   - APMS_ELIMIT if the partials do not fit: ceil(chunk_elems / 16384) * (d / chunk_elems) * 8 bytes
 *     must not exceed APMS_STATIC_SCRATCH_BYTES (d up to 2^31 elements with chunks of 16384 and more).
 *   - The address of the array is looked up once per device, by apms_create on that device or else by the
 *     first call of this function there: under graph capture, make sure one of the two has happened before.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap in time on one GPU (different
 *     streams, no ordering between them) race.  Calls ordered on one stream are fine.
 * Errors: EINVAL, ESHAPE, EALIGN, EALIAS as for apms_create + apms_server_reduce; ELIMIT; EHIP.
 */
#define APMS_STATIC_SCRATCH_BYTES (1 << 20)
int apms_server_reduce_static(int64_t d, int32_t n, int64_t chunk_elems, const uint32_t *packed,
                              const float *scales, float *server_err, uint32_t *spacked, float *sscales,
                              void *stream);

/*
 * Gather + model update (Algorithm 1 lines 10-11; supplement step 3):
 *   m_i <- (sbit ? +sscale : -sscale)   for every worker i  (a copy: bit-exact)
 *   x   <- x - lr * ( m / (sqrt(v) + eps) )        v frozen, no bias correction;
 *          eps = 0 gives the paper's literal division by sqrt(v)
 *   spacked [d/32], sscales [C], v [d] in;  x [d] in/out;  m [n][d] out.
 */
int apms_apply(apms_ctx *ctx, const uint32_t *spacked, const float *sscales, const float *v,
               float *x, float *m, float lr, float eps, void *stream);

/*
 * APGSqueeze variant (Section 5.3, item 4: "instead of communicating the momentum, use the
 * error-compensated compression strategy for communicating the gradient").  The paper gives it one
 * sentence; this reading keeps everything else of the compression stage: the worker compensates and
 * compresses its gradient, the server step is apms_server_reduce unchanged, and every worker forms the
 * momentum from the decoded averaged gradient before the frozen-variance model step.
 *
 * apms_compress_gradient, for all n workers and C chunks:
 *   u = g_i + delta_i;  scale, bit as in apms_compress;  delta_i <- u - (bit ? +scale : -scale)
 *   g [n][d] in, of type grad_format (0 = binary32, APMS_GRAD_F16, APMS_GRAD_BF16);
 *   worker_err [n][d] in/out;  packed [n][d/32], scales [n][C] out.  APMS_DEFER_ERRORS applies.
 *
 * apms_apply_gradient:
 *   ghat = (sbit ? +sscale : -sscale)
 *   m_i <- fl(beta*m_i) + fl(fl(1-beta)*ghat)      for every worker i
 *   x   <- x - lr * ( m_0 / (sqrt(v) + eps) )
 *   spacked [d/32], sscales [C], v [d] in;  x [d], m [n][d] in/out.  ESTATE if a deferred gather is
 *   pending on m.
 */
int apms_compress_gradient(apms_ctx *ctx, const void *g, int grad_format, float *worker_err, uint32_t *packed,
                           float *scales, void *stream);
int apms_apply_gradient(apms_ctx *ctx, const uint32_t *spacked, const float *sscales, const float *v, float *x,
                        float *m, float lr, float beta, float eps, void *stream);

/*
 * Top-k compressor (Section 5.1, second bullet) under the same error-compensated worker / server /
 * gather structure: C[u] keeps the K elements of largest |u| of every chunk (K is the paper's percentage
 * of chunk_elems, chosen by the caller) and zeroes the rest.  Between equal magnitudes the lower
 * index is kept first (the paper is silent; this makes the result unique).  The wire form of a chunk is
 * K (index, value) pairs, indices local to the chunk and ascending; the selection is exact.
 * The deferral flags apply as in the 1-bit path.  APMS_DEFER_ERRORS: eagerly, a call zeroes the kept positions
 * of its error buffer before its work ends (scattered stores); deferred, it leaves the compensated vector in the
 * buffer whole and the context remembers each chunk's threshold, and the next apms_topk_compress /
 * apms_topk_server_reduce on the SAME buffer (or apms_finalize) reads the kept positions as zero - the same
 * values.  APMS_DEFER_GATHER: apms_topk_apply takes the model step and leaves m untouched; the next
 * apms_topk_compress on the SAME m (or apms_finalize) decodes the server's list, uses it as the momentum and
 * writes it to m (with APMS_IMPLICIT_MOMENTUM it does not write m: m is then defined only by apms_finalize
 * between apms_topk_apply and that call).  Until then the context reads sidx and sval where the caller passed
 * them: they must stay unchanged, and an apms_topk_server_reduce that would write over them returns ESTATE.
 * A buffer left pending by a top-k call and one left by a 1-bit call are different forms: each path returns
 * ESTATE for a buffer the other left pending, and for a pending buffer other than the one it is given
 * (apms_apply and apms_topk_apply supersede a gather pending on the m they are given).
 * EINVAL unless 1 <= K <= chunk_elems; ESHAPE if chunk_elems > 2^31 or K > 2^31 - 1.
 *
 * apms_topk_reserve(ctx, K_max) is the set-up call that allocates the selection's scratch, sized for calls
 * with K <= K_max: histograms, per-tile counts and, per 4096-element tile, 64 to 512 slots of 8 bytes for the
 * elements near or above the threshold (256 slots, n*d/2 bytes in all, when K_max is 1 % of chunk_elems).
 * It allocates (ENOMEM if that fails) and synchronises the device; calling it again with a K_max the scratch
 * already covers does nothing, with a larger one it frees and allocates the slots again.
 * apms_plan.topk_scratch_bytes is what is allocated at the moment.  The three compute calls allocate
 * nothing and do not synchronise: they return ESTATE if the scratch was not reserved for their K.
 *
 * apms_topk_compress:       u = (fl(beta*m_i) + fl(fl(1-beta)*g_i)) + delta_i ;  (idx, val) <- C[u] ;
 *                           delta_i <- u - C[u]  (zero where kept, u elsewhere)
 *     m [n][d] in (out, or untouched, while a gather is pending on it);  g [n][d] in;  worker_err [n][d]
 *     in/out;  idx, val [n][C][K] out.
 * apms_topk_server_reduce:  ubar = (sum_{i=0}^{n-1} C[u_i]) * fl(1/n) + deltabar  (decoded lists summed in
 *                           worker order) ;  (sidx, sval) <- C[ubar] ;  deltabar <- ubar - C[ubar]
 *     idx, val [n][C][K] in, as written by apms_topk_compress;  server_err [d] in/out;  sidx, sval [C][K] out.
 * apms_topk_apply:          m_i <- C[ubar] (dense: zero outside the kept positions) for every worker ;
 *                           x <- x - lr * ( m / (sqrt(v) + eps) )
 *     sidx, sval [C][K], v [d] in;  x [d] in/out;  m [n][d] out (untouched with APMS_DEFER_GATHER).
 */
int apms_topk_reserve(apms_ctx *ctx, int64_t K_max);
int apms_topk_compress(apms_ctx *ctx, float *m, const float *g, float *worker_err, uint32_t *idx,
                       float *val, int64_t K, float beta, void *stream);
int apms_topk_server_reduce(apms_ctx *ctx, const uint32_t *idx, const float *val, int64_t K, float *server_err,
                            uint32_t *sidx, float *sval, void *stream);
int apms_topk_apply(apms_ctx *ctx, const uint32_t *sidx, const float *sval, int64_t K, const float *v, float *x,
                    float *m, float lr, float eps, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* APMS_H */
