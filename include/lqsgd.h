/*
 * lqsgd.h -- C ABI of the MI355X (gfx950) LQ-SGD gradient compressor.
 *
 * One context holds, for a fixed list of layer tensors and W simulated
 * workers, the state the method carries between iterations (Algorithm 1):
 * the error-feedback residual E of every worker and layer (Section 4.2,
 * Eq. (8)-(9)) and the warm-start factor Q of every layer (Algorithm 1,
 * "Warm-start from previous Q").  A step runs the loop body of Algorithm 1
 * for every layer at once, with the All-Reduce of the quantised factors
 * replaced by an on-device mean over the W workers (Section 3.1, Eq. (1)).
 *
 * Conventions
 *   - A 2-D layer gradient is rows x cols, fp32, row-major.  P is rows x r,
 *     Q is cols x r, both row-major (r contiguous), r = min(rank, rows, cols).
 *     (The paper calls the two dimensions n, m in Section 4 and m, n in
 *     Section 3.2; neither letter is used here.)
 *   - "device pointer" = memory of the GPU that was current at lqsgd_create;
 *     "host pointer" = ordinary process memory.  Every pointer says which.
 *     The caller keeps that GPU current in every later call on the context
 *     (the library never switches devices).
 *   - Every function returns LQSGD_OK (0) or a negative lqsgd_status; nothing
 *     throws or aborts.  Arguments are validated on the host before any
 *     kernel is launched.  lqsgd_last_error() gives a text for the last
 *     failure on that context.
 *   - Device work is enqueued on the HIP stream given at creation and does
 *     not synchronise, except where a function copies to or from host memory
 *     (those say "synchronises").
 *   - The caller owns the gradient (and optional G-hat) buffers; the context
 *     owns everything else and frees it in lqsgd_destroy.  Gradient buffers
 *     are never written.
 *   - Non-finite gradients are not detected; results are then undefined.
 *   - A context is not thread-safe; calls that overlap on one context race.
 */
#ifndef LQSGD_H
#define LQSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lqsgd_ctx lqsgd_ctx;

typedef enum {
  LQSGD_OK = 0,
  LQSGD_EINVAL = -1,        /* NULL pointer, value out of range                 */
  LQSGD_ESHAPE = -2,        /* bad layer shape or index                         */
  LQSGD_EUNSUPPORTED = -3,  /* valid request this build does not implement      */
  LQSGD_ENOMEM = -4,        /* host or device allocation failed                 */
  LQSGD_EHIP = -5,          /* a HIP call failed; text in lqsgd_last_error      */
  LQSGD_ESTATE = -6         /* phases called out of order                       */
} lqsgd_status;

/* Layer flags. */
#define LQSGD_LAYER_MATRIX 0u   /* compressed: rows x cols                                        */
#define LQSGD_LAYER_VECTOR 1u   /* 1-D tensor of `rows` elements (cols must be 1): sent            */
                                /* uncompressed, the step only averages it over the workers        */

typedef struct {
  int32_t rows;
  int32_t cols;
  uint32_t flags;
} lqsgd_layer;

/* Config flags. */
#define LQSGD_FLAG_NONE 0u
/* By default the residual update E = G' - G-hat (Eq. (8)) that ends an
 * iteration is deferred: the context keeps G' and the two aggregated factors,
 * and the next iteration's first sweep forms E on the fly while it adds the new
 * gradient (one pass over the data fewer; bit-identical results).
 * lqsgd_get_state / lqsgd_set_state apply a deferred update first, so callers
 * always see E.  With this flag the update runs at the end of every iteration. */
#define LQSGD_FLAG_EAGER_RESIDUAL 1u
/* The PowerSGD order of Section 3.2 instead of Algorithm 1's: the workers'
 * raw P_w = M_w Q are quantised and aggregated first, and the aggregate is
 * orthonormalised once (Gram-Schmidt) before Q_w = M_w^T P-hat.  With
 * bits_p = bits_q = 0 this is PowerSGD itself: W workers then act exactly like
 * one worker holding the mean gradient.  In this order LQSGD_FACTOR_P_ORTH does
 * not exist (EINVAL), LQSGD_FACTOR_P_MEAN is the aggregate before Gram-Schmidt
 * and LQSGD_FACTOR_P_BAR the orthonormalised aggregate that Q_w, G-hat and E use. */
#define LQSGD_FLAG_AGGREGATE_FIRST 2u
/* The gradient tensors (matrix and VECTOR layers alike) hold bfloat16 values
 * instead of fp32: grads[w * n_layers + l] then points to rows x cols 2-byte
 * elements, row-major, still 16-byte aligned.  Each value is widened exactly
 * (a bfloat16 is the upper half of a float) when G' = G + E is formed;
 * everything after that, the state and the outputs are fp32 as always.  The
 * first sweep then reads 2 bytes per element less. */
#define LQSGD_FLAG_BF16_GRADIENTS 4u
/* Never launch a kernel cooperatively.  The Gram-Schmidt of tall factors with few
 * (layer, worker) pairs normally runs as one cooperative launch whose workgroups
 * exchange partial sums while it runs; with this flag it takes its form of
 * several ordinary launches (same bits, slower: 0.2 ms instead of 0.1 ms at
 * 8192 rows, rank 32, 16 workers).  For processes in which cooperative launches
 * are unwelcome -- e.g. under rocprofv3, whose exit handler has been seen to
 * crash after the process has made one. */
#define LQSGD_FLAG_NO_COOPERATIVE_LAUNCH 8u

/* The "Require" line of Algorithm 1, plus the number of simulated workers. */
typedef struct {
  int32_t rank;      /* r, 1..LQSGD_MAX_RANK                                                     */
  int32_t bits_p;    /* b_p: 1..8, or 0 = factors exchanged as fp32 (PowerSGD, Section 3.2)      */
  int32_t bits_q;    /* b_q: as bits_p                                                           */
  int32_t workers;   /* W >= 1                                                                   */
  float alpha;       /* log scale of Eq. (5), > 0; the paper gives no value, 255 is the default  */
  uint32_t flags;
} lqsgd_config;

#define LQSGD_MAX_RANK 64
#define LQSGD_MAX_WORKERS 64

/* Phases of the staged interface: the P exchange (Algorithm 1, statements
 * "P <- G'Q" ... "P <- LogDequantize") and the Q exchange ("Q <- G'^T P" ...
 * "E <- G' - G-hat"). */
#define LQSGD_PHASE_P 0
#define LQSGD_PHASE_Q 1

/* Tensors readable with lqsgd_get_factor. */
#define LQSGD_FACTOR_P_PRE 0   /* P_w = M_w Q before orthonormalisation, rows x r  (per worker) */
#define LQSGD_FACTOR_P_ORTH 1  /* P_w after Gram-Schmidt, rows x r                 (per worker) */
#define LQSGD_FACTOR_P_BAR 2   /* mean over workers of the dequantised P_w, rows x r (shared)   */
#define LQSGD_FACTOR_Q_W 3     /* Q_w = M_w^T P-bar, cols x r                      (per worker) */
#define LQSGD_FACTOR_Q_BAR 4   /* mean of the dequantised Q_w = next warm-start Q, cols x r     */
#define LQSGD_FACTOR_VMEAN 5   /* mean over workers of a VECTOR layer, rows elements            */
#define LQSGD_FACTOR_P_MEAN 6  /* LQSGD_FLAG_AGGREGATE_FIRST only: mean of the dequantised raw   */
                               /* P_w before Gram-Schmidt, rows x r (shared)                      */

/* ---- lifetime ----------------------------------------------------------- */

/* Creates a context on the current HIP device.
 *   cfg, layers : host pointers; layers[n_layers] in the order the caller
 *                 will list gradient tensors.
 *   hip_stream  : a hipStream_t (NULL = the default stream); all device work
 *                 of this context runs on it.
 *   out         : host pointer receiving the context.
 * Allocates all device state; E = 0 (Algorithm 1, "Initialize error matrix")
 * and Q = 0 until lqsgd_set_q is called for each matrix layer.
 * Errors: EINVAL (NULL, rank/bits/workers/alpha out of range), ESHAPE
 * (rows or cols < 1, rows*cols >= 2^31, VECTOR with cols != 1), ENOMEM, EHIP. */
int lqsgd_create(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers,
                 void* hip_stream, lqsgd_ctx** out);

/* Frees everything; NULL is accepted.  Synchronises the stream first. */
int lqsgd_destroy(lqsgd_ctx* ctx);

/* Waits until all work enqueued by this context has finished.
 * One kernel (Gram-Schmidt of tall factors, launched cooperatively) has
 * workgroups wait for each other on the device; those waits are bounded, and if
 * one ever expires the kernel still runs to its end but the context's results
 * are invalid from then on: this call, and every other call that synchronises,
 * then returns LQSGD_EHIP with a text saying so. */
int lqsgd_synchronize(lqsgd_ctx* ctx);

/* Text for the most recent error on ctx (or for a failed lqsgd_create when
 * ctx is NULL).  The pointer stays valid until the next call on that context. */
const char* lqsgd_last_error(const lqsgd_ctx* ctx);

/* ---- state: what the method carries between iterations ------------------ */

/* Q_0 of one matrix layer (Algorithm 1, "Initialize Q_0 ~ N(0,1)": the random
 * draw is the caller's).  host_q: host pointer, cols x r floats.  Synchronises. */
int lqsgd_set_q(lqsgd_ctx* ctx, int32_t layer, const float* host_q);

/* Copies out / in the residual E of (layer, worker) (rows x cols floats) and
 * the warm-start Q of `layer` (cols x r floats).  Either host pointer may be
 * NULL to skip that tensor.  Synchronises.  For a VECTOR layer: ESHAPE.
 * Between iterations this pair is all the state the method carries (Section 4.2;
 * Algorithm 1, "Warm-start from previous Q"): saving it for every layer and
 * worker and loading it into a fresh context of the same configuration resumes
 * the run bit for bit.
 * In the middle of a staged iteration -- after lqsgd_compress(PHASE_P) and before
 * lqsgd_decompress(PHASE_Q) has run -- the residual buffer holds G' = G + E
 * (Eq. (9)) of the iteration in progress, and that is what host_e receives;
 * host_q still receives the Q this iteration started from.  lqsgd_set_state is
 * meant for the time between iterations: in the middle of one it overwrites G'
 * (or Q) under the iteration in progress. */
int lqsgd_get_state(lqsgd_ctx* ctx, int32_t layer, int32_t worker, float* host_e, float* host_q);
int lqsgd_set_state(lqsgd_ctx* ctx, int32_t layer, int32_t worker, const float* host_e,
                    const float* host_q);

/* ---- the compressor ----------------------------------------------------- */

/* grads: host array of workers * n_layers device pointers,
 * grads[w * n_layers + l] -> fp32 tensor of layer l on worker w, 16-byte
 * aligned, read-only.  The pointer values are copied; the array itself need
 * not outlive the call.  The context keeps a device copy of the list: a call
 * whose list (or G-hat / parameter list) differs from the previous call's waits
 * for the context's stream, then copies the new list to the device
 * (synchronously); a call that repeats the previous lists only enqueues kernels.
 *
 * lqsgd_compress(PHASE_P, grads): for every matrix layer and worker
 *     M_w = G_w + E_w (kept in the context, Eq. (9)); P_w = M_w Q;
 *     P_w <- Gram-Schmidt(P_w); packet_P[w] = LogQuantize(P_w, b_p, alpha).
 * lqsgd_decompress(PHASE_P): P-bar = mean_w LogDequantize(packet_P[w]).
 * lqsgd_compress(PHASE_Q, NULL): Q_w = M_w^T P-bar; packet_Q[w] =
 *     LogQuantize(Q_w, b_q, alpha).  (grads is ignored and may be NULL.)
 * lqsgd_decompress(PHASE_Q): Q-bar = mean_w LogDequantize(packet_Q[w]);
 *     E_w = M_w - P-bar Q-bar^T (Eq. (7), (8)); Q-bar becomes the warm-start Q.
 * The four calls in that order are one iteration for the matrix layers;
 * any other order returns ESTATE.  VECTOR layers are handled by lqsgd_step only.
 * With bits = 0 the packet is the fp32 factor itself. */
int lqsgd_compress(lqsgd_ctx* ctx, int32_t phase, const float* const* grads);
int lqsgd_decompress(lqsgd_ctx* ctx, int32_t phase);

/* One whole iteration (Algorithm 1, from "G' <- G + E" to "E <- G' - G-hat")
 * for all layers, with quantise / dequantise / mean fused, plus the plain
 * mean of every VECTOR layer.
 *   ghat : NULL, or host array of n_layers device pointers; a non-NULL entry
 *          receives G-hat = P-bar Q-bar^T (rows x cols, written once, the
 *          quantity Algorithm 1 applies in "w <- w - eta G-hat") or, for a
 *          VECTOR layer, the mean over workers.  Must not alias any gradient. */
int lqsgd_step(lqsgd_ctx* ctx, const float* const* grads, float* const* ghat);
/* Stream capture: once the same grads / ghat pointer lists have been used in an
 * ordinary call (so that their device copies exist) and at least one iteration
 * has run (so that the deferred residual is in its steady state), lqsgd_step
 * and lqsgd_step_update enqueue kernels only -- no copies, no memsets, no
 * synchronisation -- and may be recorded into a HIP graph on the context's
 * stream.  Every replay is then one iteration on whatever the recorded buffers
 * hold at that time.  Per-kernel timing must be off while recording.  A
 * recorded iteration continues from the state the previous one left (with the
 * residual update still deferred): calls that read or write E or the factors
 * from the host (lqsgd_get_state with host_e, lqsgd_set_state, lqsgd_set_factor,
 * lqsgd_set_q) apply that update, so after one of them run an ordinary
 * iteration and record again before replaying. */

/* The same iteration followed by Algorithm 1's last statement, fused into the
 * pass that would write G-hat: w <- w - eta G-hat (Eq. (2)) for every matrix
 * layer, w <- w - eta mean_w(g_w) for every VECTOR layer.
 *   params : host array of n_layers device pointers to the fp32 parameters
 *            (same shapes as the gradients, 16-byte aligned, updated in
 *            place); a NULL entry leaves that tensor alone.  Must not alias
 *            any gradient.  G-hat itself is not stored.
 *   eta    : learning rate, finite. */
int lqsgd_step_update(lqsgd_ctx* ctx, const float* const* grads, float* const* params, float eta);

/* One whole iteration, as lqsgd_step, for callers that cannot allocate device
 * memory or keep a context: code that runs under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  It takes the configuration
 * and the state with every call, keeps nothing between calls that the caller
 * must free, and calls no hipMalloc, hipFree or any other allocating routine:
 * everything lqsgd_create would allocate besides the state -- partial products,
 * factors, packets, quantiser tables, work lists -- lies in one static block of
 * device memory inside the library (LQSGD_STATIC_SCRATCH_BYTES, 32 MiB, per GPU,
 * held until the process ends).  A configuration that needs more returns
 * EUNSUPPORTED and launches nothing (fc 256 x 128 needs under 0.1 MiB, the small
 * CNN 1 MiB, the ResNet-18 set with 8 workers 9 MiB at rank 4 and 17 MiB at rank 8).
 *   cfg, layers, n_layers : as for lqsgd_create (host pointers).
 *   hip_stream : all work is enqueued here.
 *   grads, ghat: as for lqsgd_step.
 *   residual   : device pointer, workers x residual_stride floats (see
 *                lqsgd_plan_query), 16-byte aligned.  Worker w's E of the i-th
 *                matrix layer starts at w * residual_stride + off_i, where off_i
 *                adds up rows x cols of the matrix layers before it in list order,
 *                each rounded up to a multiple of 64 floats.  Holds E_{t-1} on
 *                entry (Algorithm 1 starts from zeros) and E_t once the enqueued
 *                work has run.
 *   warm_q     : device pointer, warm_q_floats floats, 16-byte aligned.  The Q of
 *                the i-th matrix layer (cols x r, row-major) starts where the
 *                cols x r of the layers before it add up to, each rounded up to 64
 *                floats; the floats after the last layer are slack that the
 *                kernels may read.  Holds the warm-start Q on entry and the
 *                aggregated Q of this iteration afterwards.
 *                Either may be NULL when there is no matrix layer.
 * The residual update runs at the end of the call's work (never deferred).
 * Results are bit-identical to lqsgd_step on a context holding the same state.
 * The first call with a configuration (or stream) other than the previous
 * call's on that GPU waits for the previous call's stream, lays the block out
 * anew and copies its tables in with synchronous copies; calls that repeat the
 * previous configuration only enqueue kernels (plus one small copy when the
 * pointer lists change).  All calls on a GPU share that GPU's block: two calls
 * whose work overlaps in time -- different streams, or different threads --
 * race; a caller that uses more than one stream orders them itself.  The
 * Gram-Schmidt of tall factors takes its form of several ordinary launches here.
 * Errors: as lqsgd_create and lqsgd_step; text from lqsgd_last_error(NULL). */
int lqsgd_step_static(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers,
                      void* hip_stream, const float* const* grads, float* residual, float* warm_q,
                      float* const* ghat);

/* ---- taps for parity checks and for a transport layer ------------------- */

/* Packet of (phase, layer, worker) as unpacked codes: mag_codes[i] in
 * [0, 2^b - 1], sign_bits[i] in {0, 1}, i over rows*r (P) or cols*r (Q)
 * elements in row-major factor order; *scale = absmax of the factor.  Any of
 * the three host pointers may be NULL.  Synchronises.  bits == 0:
 * EUNSUPPORTED. */
int lqsgd_get_packet(lqsgd_ctx* ctx, int32_t phase, int32_t layer, int32_t worker,
                     uint8_t* mag_codes, uint8_t* sign_bits, float* scale);
/* Overwrites a packet (to inject another worker's or another
 * implementation's codes before lqsgd_decompress).  Synchronises. */
int lqsgd_set_packet(lqsgd_ctx* ctx, int32_t phase, int32_t layer, int32_t worker,
                     const uint8_t* mag_codes, const uint8_t* sign_bits, float scale);
/* The same packet as it lies in device memory: magnitude plane (element e in
 * stream bits [e*b, (e+1)*b), least significant bit first, padded to groups of
 * 8 elements: b * ceil(n/8) bytes) and sign plane (1 bit per element, LSB
 * first: ceil(n/8) bytes).  *mag_len / *sign_len receive the byte counts; the
 * buffers (host pointers) may be NULL to query sizes only.  Synchronises. */
int lqsgd_get_packet_raw(lqsgd_ctx* ctx, int32_t phase, int32_t layer, int32_t worker,
                         uint8_t* mag_plane, int64_t* mag_len, uint8_t* sign_plane,
                         int64_t* sign_len);
/* Where that packet lies: device pointers to its magnitude plane, its sign
 * plane and its scale (one float), with the planes' byte counts, so that a
 * caller can hand a worker's packet to a collective, or have one written into a
 * worker's slot, without a trip through host memory -- the exchange of
 * Algorithm 1's "All-Reduce" statements (Section 3.1), which this one-GPU
 * build replaces by the on-device mean.  The memory belongs to the context and
 * stays valid until lqsgd_destroy; it is written by lqsgd_compress / lqsgd_step
 * and read by lqsgd_decompress, in stream order on the context's stream.  Any
 * output pointer may be NULL.  Does not synchronise.  bits == 0: EUNSUPPORTED
 * (the packet is then the fp32 factor, see lqsgd_get_factor). */
int lqsgd_packet_device(lqsgd_ctx* ctx, int32_t phase, int32_t layer, int32_t worker,
                        uint8_t** mag_plane, int64_t* mag_len, uint8_t** sign_plane,
                        int64_t* sign_len, float** scale);

/* Copies one of the LQSGD_FACTOR_* tensors to host memory.  `worker` is
 * ignored for shared tensors.  Synchronises. */
int lqsgd_get_factor(lqsgd_ctx* ctx, int32_t which, int32_t layer, int32_t worker, float* host);
/* Overwrites P-bar or Q-bar (LQSGD_FACTOR_P_BAR / _Q_BAR) from host memory. */
int lqsgd_set_factor(lqsgd_ctx* ctx, int32_t which, int32_t layer, const float* host);

/* Bytes one worker sends per iteration for the matrix layers: per factor
 * ceil(n*b/8) magnitude + ceil(n/8) sign + 4 scale bytes (4n bytes at b = 0).
 * Section 4.3 counts the magnitude bits only: r(n+m)b per layer. */
int64_t lqsgd_wire_bytes(const lqsgd_ctx* ctx);

/* ---- planning, without a GPU -------------------------------------------- */

typedef struct {
  int64_t device_bytes;      /* what lqsgd_create would allocate                        */
  int64_t wire_bytes;        /* as lqsgd_wire_bytes                                      */
  int64_t matrix_elements;   /* sum rows*cols over matrix layers (one worker)            */
  int32_t n_matrix, n_vector;
  int32_t rank_pad;          /* register rank the kernels are instantiated for           */
  int32_t tiles[3];          /* work items of the three streaming sweeps                 */
  int32_t reserved;
  int64_t residual_stride;   /* floats between two workers' residual slabs (lqsgd_step_static) */
  int64_t warm_q_floats;     /* floats of the warm-start buffer of lqsgd_step_static      */
} lqsgd_plan_info;

/* Pure host computation: validates cfg / layers exactly as lqsgd_create does
 * and reports sizes.  Usable on a machine with no GPU. */
int lqsgd_plan_query(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers,
                     lqsgd_plan_info* out);

/* Lists the work items of streaming sweep `sweep` (0: add + P product,
 * 1: Q product, 2: residual, 3: the G-hat-only pass that runs when the
 * residual is deferred; worker 0's shapes only) as 6 int32 each: layer, worker, row0, nrows,
 * col0, ncols.  out: host pointer with room for cap items; returns the number
 * of items (or a negative status).  Pure host computation. */
int64_t lqsgd_plan_tiles(const lqsgd_config* cfg, const lqsgd_layer* layers, int32_t n_layers,
                         int32_t sweep, int32_t* out, int64_t cap);

/* ---- per-kernel timing with HIP events on the context's stream ---------- */

#define LQSGD_KERNEL_ADD_PROJECT 0   /* M = G + E (+ deferred residual), P partials */
#define LQSGD_KERNEL_ORTH 1          /* reduce partials, Gram-Schmidt, absmax */
#define LQSGD_KERNEL_EXCHANGE_P 2    /* quantise / dequantise / mean of P */
#define LQSGD_KERNEL_BACK_PROJECT 3  /* Q partials = M^T P-bar, and the mean of the VECTOR layers */
#define LQSGD_KERNEL_REDUCE_Q 4      /* reduce partials, absmax           */
#define LQSGD_KERNEL_EXCHANGE_Q 5    /* quantise / dequantise / mean of Q */
#define LQSGD_KERNEL_RESIDUAL 6      /* E = M - P-bar Q-bar^T and / or G-hat */
#define LQSGD_KERNEL_REDUCE_P 7      /* aggregate-first order: reduce of the P partials, absmax */
#define LQSGD_KERNEL_COUNT 8

/* on != 0: every kernel launched from now on is bracketed by a pair of HIP
 * events on the context's stream (this adds a little time between kernels).
 * on == 0: stop.  Either way the accumulated figures are cleared. */
int lqsgd_timing_enable(lqsgd_ctx* ctx, int32_t on);
/* Synchronises, then adds up the event pairs recorded since the last
 * lqsgd_timing_enable: total_ms[k] and launches[k] for k < LQSGD_KERNEL_COUNT
 * (host pointers to arrays of that length). */
int lqsgd_timing_read(lqsgd_ctx* ctx, double* total_ms, int64_t* launches);
/* Name of a LQSGD_KERNEL_* timing slot: the stage of the iteration, not a device
 * function (which function serves a stage depends on rank, shapes and flags). */
const char* lqsgd_kernel_name(int32_t kernel);
/* The device function this context launched last for that slot, with its template
 * arguments, as a profiler's kernel list names it (namespaces and the parameter
 * list left out), e.g. "add_project_kernel<4, true, false, false>"; "" before
 * the first launch.  Valid until the next launch for that slot. */
const char* lqsgd_launched_kernel(const lqsgd_ctx* ctx, int32_t kernel);

#ifdef __cplusplus
}
#endif
#endif /* LQSGD_H */
