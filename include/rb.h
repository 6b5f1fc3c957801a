/*
 * rb.h -- C ABI of the per-GPU rehearsal buffer (gfx950 / MI355X).
 *
 * One process's local rehearsal buffer B_n of the paper "Efficient
 * Data-Parallel Continual Learning with Asynchronous Distributed Rehearsal
 * Buffers": one sub-buffer R^i_n per class, all of equal capacity (Sec. IV-A),
 * populated by Algorithm 1 (Sec. IV-B) and read by uniform sampling without
 * replacement to augment the next mini-batch (Sec. IV-C, Listing 1).  The
 * paper keeps the buffer in pinned host memory and hides its management on
 * background threads (Sec. IV-D, Sec. V); here the buffer lives in HBM and the
 * two hot calls only enqueue kernels on a caller-supplied HIP stream.
 *
 * Conventions
 *   - "device" pointers are HIP device memory of the current device, "host"
 *     pointers ordinary host memory.  The library never allocates or frees
 *     device memory: buffer storage, workspace, mini-batches and outputs are
 *     all owned by the caller and only borrowed for the duration stated.
 *   - Samples are opaque rows of row_bytes = prod(sample_shape) * sizeof(dtype)
 *     bytes; row_bytes must be a multiple of 16 and every sample pointer
 *     16-byte aligned.  Slot s of class k is row k*slots_per_class + s of
 *     buf_x / element k*slots_per_class + s of buf_y.
 *   - Labels are int64.  A never-written slot has buf_y = -1 and unspecified
 *     sample bytes.
 *   - Every random choice is a pure function of (seed, step, purpose, index)
 *     through Philox4x32-10, so a (seed, step) pair always reproduces the same
 *     decisions; the caller advances step once per training iteration.
 *   - rb_update and rb_sample_augment validate what the host can see, enqueue
 *     on the bound stream and return without synchronising.  Work is ordered
 *     by that stream: update(t), sample(t), update(t+1), ...  Calls on one
 *     handle must not be issued from two host threads at once.
 *   - All functions return RB_OK (0) or a negative rb_status; nothing aborts
 *     or throws.  On an error no kernel was enqueued by that call.
 */
#ifndef RB_H
#define RB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rb_buffer rb_buffer;   /* opaque host-side handle */

enum rb_dtype { RB_F32 = 0, RB_BF16 = 1 };   /* only fixes the element size: 4 or 2 bytes */

enum rb_status {
    RB_OK = 0,
    RB_EINVAL = -1,   /* an argument is out of range, null or misaligned          */
    RB_ENOMEM = -2,   /* host allocation of the handle failed                     */
    RB_ESTATE = -3,   /* hot call before rb_bind                                  */
    RB_EHIP = -4,     /* a HIP call (launch, copy, synchronise) reported an error */
    RB_ELIMIT = -5    /* rb_bind_static: the buffer's workspace exceeds the library's own scratch */
};

#define RB_MAX_BATCH 4096          /* largest b, c and r accepted                          */
#define RB_MAX_CLASSES (1 << 20)   /* largest number of classes                            */
#define RB_MAX_SLOTS 2147483647LL  /* classes * slots_per_class must not exceed this       */
#define RB_FLAG_BAD_LABEL 1u       /* state flag: a candidate's label was outside [0, K)   */
#define RB_FLAG_PLAN_TIMEOUT 2u    /* state flag: the workgroups that plan a several-steps launch for large counts
                                      did not hear from each other within 2 s; that launch moved nothing and the
                                      buffer's state is no longer defined (bind again) */

/*
 * Describe a buffer of `classes` sub-buffers of `slots_per_class` samples each
 * (Sec. IV-A: the per-process space is divided evenly between the classes; the
 * capacity |R^i_n|max is given directly, in samples).  sample_shape: host
 * array of ndim >= 1 positive extents.  Host-only: touches no device.
 * RB_EINVAL: null out/shape, classes < 1 or > RB_MAX_CLASSES, slots < 1,
 * classes*slots > RB_MAX_SLOTS, ndim < 1, non-positive extent, unknown dtype,
 * row_bytes not a multiple of 16.
 */
int rb_create(rb_buffer **out, int64_t classes, int64_t slots_per_class,
              const int64_t *sample_shape, int32_t ndim, int32_t dtype);

/* Bytes the caller must provide to rb_bind: sample storage, label storage,
 * workspace (per-class fill counts and their partial sums, state words).  Any
 * of the three out pointers may be null. */
int rb_query_sizes(const rb_buffer *rb, size_t *x_bytes, size_t *y_bytes, size_t *workspace_bytes);

/*
 * Attach device storage and a stream (hipStream_t, null = the default stream)
 * and enqueue the reset of the buffer to "empty": fill counts 0, buf_y = -1;
 * buf_x is not touched.  buf_x (16-byte aligned), buf_y and workspace (256-byte
 * aligned) are device pointers of at least the rb_query_sizes sizes and stay
 * borrowed until rb_destroy or the next rb_bind.  Binding again resets again.
 */
int rb_bind(rb_buffer *rb, void *buf_x, int64_t *buf_y, void *workspace, void *hip_stream);

/*
 * Reduced-precision storage (Sec. VII notes that data reduction can be applied
 * to the stored representatives; this is the plainest form for floating-point
 * samples).  RB_STORE_SAME (default): a stored row is the sample's bytes.
 * RB_STORE_BF16: samples are binary32 (dtype RB_F32); every element is stored
 * as the bfloat16 nearest to it (ties to even; NaN keeps its sign and upper
 * payload bits and is made quiet) by rb_update, and handed out widened back to
 * binary32, which is exact, by rb_sample_augment.  Mini-batches and outputs
 * keep the full row size; buf_x rows shrink to half: call this BEFORE
 * rb_query_sizes / rb_bind (RB_ESTATE once bound).  The sample's byte size
 * must be a multiple of 32.  Served by the general kernels (two launches per
 * step), by the plan-ahead forms of the single launch (rb_announce_next) and
 * by the several-steps launch (rb_update_sample_many).
 * RB_STORE_U8: samples are binary32 with values meant to lie in [0, 1] (image
 * tensors); an element x is stored as the byte nearest to 255 * x - product
 * and rounding in binary32, ties to even; x <= 0 and NaN give 0, 255 * x >= 255
 * gives 255 - and handed out as byte / 255 (binary32 division, correctly
 * rounded): a quarter of the memory, an absolute error of at most 1/510 for
 * values in [0, 1].  The sample's byte size must be a multiple of 64.  Served
 * by the general kernels, by the plan-ahead forms of the single launch and by
 * the several-steps launches of rb_update_sample_many; every call form gives
 * the same bytes.
 */
enum rb_storage { RB_STORE_SAME = 0, RB_STORE_BF16 = 1, RB_STORE_U8 = 2 };
int rb_set_storage(rb_buffer *rb, int32_t storage);

/*
 * Policy variants of Algorithm 1.  The defaults are what Algorithm 1 prints.
 * Selection: RB_SELECT_EXACT - the first step of Algorithm 1, a uniform subset
 * of exactly c positions; RB_SELECT_BERNOULLI - the wording of Sec. IV-B, where
 * each sample of the mini-batch is inserted with probability c/b: an independent
 * coin per sample (any number of candidates from 0 to b).
 * Eviction (Sec. IV-A allows strategies other than random replacement):
 * RB_EVICT_UNIFORM - overwrite a uniformly drawn slot of the class;
 * RB_EVICT_FIFO - overwrite the oldest sample of the class;
 * RB_EVICT_RESERVOIR - reservoir sampling per class: the n-th sample ever
 * offered to a full class replaces a uniformly drawn slot with probability
 * slots_per_class / n and is dropped otherwise (exact while a class has been
 * offered fewer than 2^31 - 1 samples).
 * With a variant selected a plain rb_update_sample enqueues the two general
 * kernels.  The plan-ahead forms of the single launch (rb_announce_next) serve
 * every variant (the Bernoulli selection for b <= 1024), and so do the
 * several-steps launches of rb_update_sample_many (the form for small counts
 * with the exact selection only; the form for large counts takes over for the
 * Bernoulli selection, again for b <= 1024).  RB_EINVAL: unknown value.  RB_ESTATE: an rb_update was already
 * enqueued since the last rb_bind.
 */
enum rb_selection { RB_SELECT_EXACT = 0, RB_SELECT_BERNOULLI = 1 };
enum rb_eviction { RB_EVICT_UNIFORM = 0, RB_EVICT_FIFO = 1, RB_EVICT_RESERVOIR = 2 };
int rb_set_policy(rb_buffer *rb, int32_t selection, int32_t eviction);

/*
 * rb_bind for callers that cannot allocate device memory at this point (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same call, but the workspace is a scratch array of
 * RB_STATIC_WORKSPACE_BYTES that the library itself holds in device memory
 * (a file-scope array of the loaded code object: one copy per GPU, from the
 * moment the library is loaded on that GPU until the process ends).  The call
 * allocates nothing, on the device or through any library; buf_x, buf_y and
 * every later input and output are still the caller's.  All later calls on the
 * handle work as after rb_bind.
 * Every handle bound this way on one GPU uses that GPU's one array, which keeps
 * whatever the last user left: the call clears the part it uses (fill counts,
 * state words, plan tables) on the stream, like rb_bind, and takes the array
 * away from the handle that held it before (that handle is unbound: its hot
 * calls return RB_ESTATE until it is bound again).  Work of the previous
 * holder that is still running on another stream when this call's clearing
 * runs would race with it: the caller orders the two (one handle at a time per
 * GPU, or a synchronisation in between).
 * RB_ELIMIT: the handle needs more workspace than RB_STATIC_WORKSPACE_BYTES
 * (rb_query_sizes tells how much: about 16 bytes per class plus 3.2 MB);
 * otherwise the errors of rb_bind.
 */
#define RB_STATIC_WORKSPACE_BYTES (4u << 20)
int rb_bind_static(rb_buffer *rb, void *buf_x, int64_t *buf_y, void *hip_stream);

/* Replace the stream later calls enqueue on.  The caller orders the old and
 * the new stream itself (events) if work is still pending on the old one. */
int rb_set_stream(rb_buffer *rb, void *hip_stream);

/*
 * Algorithm 1, update_buffer(m), for the mini-batch m = (batch_x, batch_y) of
 * b samples (device pointers; batch_x 16-byte aligned, b rows of row_bytes):
 *   1. C <- a uniformly random subset of exactly c of the b positions;
 *   2. for every candidate of C in ascending mini-batch position, with class
 *      k = batch_y[pos]: if R^k_n holds fewer than slots_per_class samples,
 *      append; otherwise overwrite a slot of R^k_n drawn uniformly from all
 *      its slots.  If several candidates of one step end on the same slot, the
 *      one latest in the mini-batch is what the slot holds afterwards.
 * A candidate whose label is outside [0, classes) is dropped and sets
 * RB_FLAG_BAD_LABEL.  c = 0 is a no-op.  batch_x / batch_y must stay valid and
 * unchanged until the enqueued work has run.
 * RB_EINVAL: null pointers, b < 1, b > RB_MAX_BATCH, c < 0, c > b,
 * misaligned batch_x / batch_y.  RB_ESTATE: not bound.
 */
int rb_update(rb_buffer *rb, const void *batch_x, const int64_t *batch_y,
              int64_t b, int64_t c, uint64_t seed, uint64_t step);

/*
 * Mini-batch augmentation (Sec. IV-C; what the training loop of Listing 1
 * concatenates to the mini-batch): draw n = min(r, F) representatives uniformly without
 * replacement from the F samples currently stored (every stored sample equally
 * likely, whatever its class) and copy sample j to row j of out_x and its
 * label to out_y[j]; out_y[j] = -1 for n <= j < r and those out_x rows are not
 * written.  out_x (16-byte aligned, r rows) and out_y (r labels) are device
 * pointers; pointing out_x at row b of a (b+r)-row tensor whose first b rows
 * hold the mini-batch yields the augmented mini-batch without another copy.
 * r = 0 is a no-op.  RB_EINVAL: r < 0, r > RB_MAX_BATCH, null or misaligned
 * outputs with r > 0.  RB_ESTATE: not bound.
 */
int rb_sample_augment(rb_buffer *rb, int64_t r, uint64_t seed, uint64_t step,
                      void *out_x, int64_t *out_y);

/*
 * The paper's single primitive (the update call of Listing 1; Sec. IV-D
 * step 2: update the buffer with the mini-batch, then sample the next
 * representatives): rb_update(rb, batch_x, batch_y, b, c, seed, step) followed
 * by rb_sample_augment(rb, r, seed, step, out_x, out_y), as one call with the
 * same arguments, meaning, errors and, bit for bit, the same results.  When
 * 1 <= c <= 64, 1 <= r <= 64 and classes <= 1024 both halves run as ONE kernel
 * launch (a representative whose slot is being written in this very step is
 * copied from the mini-batch row stored there); otherwise the two kernels are
 * enqueued one after the other.  out_x must not overlap batch_x.
 */
int rb_update_sample(rb_buffer *rb, const void *batch_x, const int64_t *batch_y, int64_t b, int64_t c,
                     int64_t r, uint64_t seed, uint64_t step, void *out_x, int64_t *out_y);

/*
 * Plan-ahead form of the single-launch step, for callers that already hold the
 * NEXT mini-batch's labels (a prefetching data pipeline): announce them, then
 * call rb_update_sample (or rb_pipeline_step) as usual.  The launch of that
 * step then also works out, in one extra workgroup and concurrently with the
 * row movement, the whole plan of the following step (its b, c, r and seed are
 * taken to be the same, its step number one higher) and leaves it in the
 * workspace; the following rb_update_sample call, if it comes with exactly
 * those labels (the same pointer) and arguments, only moves rows by that plan.
 * Results are bit for bit those of the plain calls.  An announcement serves the
 * one next rb_update_sample call and is forgotten if any other call on the
 * handle (rb_update, rb_sample_augment, rb_read_state, ...) comes first; if
 * the call after the announcing step does not match what was planned, or any
 * other call comes first, the plan is dropped and nothing is lost but the time
 * it took.  The match is by address: memory that held announced labels must
 * not be given other contents and passed as the next step's labels.  Used when the step is
 * eligible for the single launch (see rb_update_sample), and also for up to
 * 1024 candidates and representatives, b <= 4096 (b <= 1024 with the Bernoulli
 * selection) and up to 10240 classes (the step is then one launch that moves
 * rows by the plan, instead of two kernels); ignored otherwise.
 * next_batch_y: device, b int64 labels that must be in place, as far as the
 * bound stream is concerned, when the announcing step is enqueued, and stay
 * unchanged until the step they belong to has run; null withdraws an
 * announcement.  rb_update_sample_many announces for itself.
 */
int rb_announce_next(rb_buffer *rb, const int64_t *next_batch_y);

/*
 * n consecutive rb_update_sample steps (Sec. IV-D step 2: update the buffer
 * with the mini-batch, then sample the next representatives) from one call,
 * for callers that have several mini-batches ready (e.g. a prefetching data
 * pipeline).  When 1 <= c <= 64, 1 <= r <= 64, classes <= 1024, b <= 2048 and
 * the selection is the exact one (any replacement strategy, either storage
 * form), up to 32 of the steps
 * - as many as 1280 / (c + r) and 640 / max(c, r) allow, see
 * rb_query_steps_per_launch - share ONE launch: the rows of all of them are
 * moved at once, by a plan that one workgroup of the launch before made.  What
 * the order of separate launches would settle between steps (a representative
 * read from a slot that another step of the same launch writes, a slot written
 * twice) the plan settles, so the cost of a launch is paid once per that many
 * steps.  Beyond those limits - and within them when a step's rows are so
 * short that they are moved sooner than one workgroup plans a step
 * (RB_OPT_PLANNERS) -, for up to 1024 candidates and representatives,
 * b <= 4096 (b <= 1024 with the Bernoulli selection) and up to 10240 classes,
 * up to 16 steps share one launch in the same way; their plan is made by two
 * workgroups per step of the launch before, which work side by side (should
 * they ever fail to hear from each other within 2 s, that launch moves nothing
 * and raises RB_FLAG_PLAN_TIMEOUT).  Otherwise the steps are enqueued one
 * after the other, each
 * announcing the next one's labels (rb_announce_next) for itself.  Step i uses
 * batch_x[i], batch_y[i], step number first_step + i and writes to out_x[i],
 * out_y[i]; b, c, r and seed are common.  The four pointer arrays are HOST
 * arrays of n device pointers, read before the call returns.  All n steps are
 * validated first; on an error nothing was enqueued.  Results are those of n
 * separate calls, bit for bit.
 * The outputs and mini-batches of any 32 consecutive steps must not overlap.
 * The workspace behind the handle is used by the launches of this call while
 * they run: one stream of calls per handle.
 */
int rb_update_sample_many(rb_buffer *rb, int64_t n, const void *const *batch_x, const int64_t *const *batch_y,
                          int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t first_step,
                          void *const *out_x, int64_t *const *out_y);

/*
 * rb_announce_next for rb_update_sample_many: the labels of the first n steps
 * of the call AFTER the next rb_update_sample_many call (the data pipeline has
 * them already).  The last launch of the next call then also plans those steps
 * (at most 32, and at most what one launch covers), so that the call after it
 * starts moving rows at once instead of planning its first steps in a launch
 * of its own.  The plan is used if that later call comes with the same b, c,
 * r and seed, with first_step continuing where the call before ended, with at
 * least the planned number of steps, and with exactly the announced label
 * pointers for them; otherwise (or if any other call on the handle comes
 * first) it is dropped and nothing is lost but the time it took.  Results are
 * bit for bit those of the plain calls.  When the steps go out one by one
 * (see rb_update_sample_many) the first announced labels serve as
 * rb_announce_next for the call's last step.  The announcement serves the one
 * next rb_update_sample_many call and is forgotten by any other call.
 * next_batch_y: HOST array of n device pointers (read before the call
 * returns; only the first 32 are kept), each to b int64 labels that must be in
 * place, as far as the bound stream is concerned, when the next call is
 * enqueued, and stay unchanged until their steps have run.  n = 0 withdraws.
 * RB_EINVAL: null rb, n < 0, null or misaligned label pointers.
 */
int rb_announce_next_many(rb_buffer *rb, int64_t n, const int64_t *const *next_batch_y);

/*
 * How many steps of this shape rb_update_sample_many puts into one launch at
 * most, with the handle's present policy, storage and options (1: every step
 * gets a launch, or two, of its own).  A stream of calls that are announced to
 * each other (rb_announce_next_many) consists of launches of exactly this
 * size, apart from a call's remainder.  Host only.
 * RB_EINVAL: null pointers, b, c or r out of range (as in rb_update_sample).
 */
int rb_query_steps_per_launch(const rb_buffer *rb, int64_t b, int64_t c, int64_t r, int64_t *steps);

/*
 * The asynchronous form of that primitive (Sec. IV-D, Fig. 4, Listing 1): the
 * training loop calls it once per iteration with the iteration's mini-batch;
 * the call (1) makes `train_stream` wait until the representatives that the
 * PREVIOUS call started to collect are complete, and reports in *ready_rows
 * how many rows that call asked for (0 on the first call: the buffer was
 * empty, so the first iteration trains on the plain mini-batch); (2) enqueues,
 * on the buffer's bound stream, rb_update_sample with this mini-batch, whose
 * representatives go to next_x / next_y: the place where the caller wants the
 * NEXT iteration's representatives, usually the tail rows of the next
 * augmented mini-batch (or one of two alternating buffers).  Work the caller
 * then enqueues on train_stream (forward and backward pass on the augmented
 * mini-batch) runs concurrently with (2).
 *
 * Ordering set up by the call, with events and no host synchronisation: the
 * bound stream waits for everything enqueued on train_stream so far (the
 * mini-batch has been produced, and whatever read the memory behind next_x /
 * next_y in earlier iterations is done); train_stream waits for the previous
 * call's work as said in (1).  The mini-batch must stay unchanged until that
 * work is complete, i.e. until train_stream has passed the wait of the next
 * rb_pipeline_step or rb_pipeline_drain.  If train_stream is the bound stream
 * itself the call degenerates to rb_update_sample.
 *
 * rb_pipeline_create makes the two events (no device memory); the pipeline
 * borrows `rb`, which must outlive it.  rb_pipeline_drain only does (1): it
 * makes train_stream wait for the last step's representatives (end of
 * training, or before the caller touches the buffer's state).  Arguments,
 * limits and errors of rb_pipeline_step are those of rb_update_sample;
 * ready_rows may be null.  On an error nothing was enqueued and the pipeline
 * is unchanged.
 */
typedef struct rb_pipeline rb_pipeline;
int rb_pipeline_create(rb_pipeline **out, rb_buffer *rb);
int rb_pipeline_step(rb_pipeline *p, const void *batch_x, const int64_t *batch_y, int64_t b, int64_t c,
                     int64_t r, uint64_t seed, uint64_t step, void *next_x, int64_t *next_y,
                     void *train_stream, int64_t *ready_rows);
int rb_pipeline_drain(rb_pipeline *p, void *train_stream, int64_t *ready_rows);

/*
 * rb_pipeline_step for a training loop whose data pipeline holds the next n
 * mini-batches already (Sec. IV-D, Fig. 4, with a prefetching loader): one call
 * every n iterations, at the start of iteration first_step.  (1) train_stream
 * is made to wait for the representatives that the previous call (of either
 * kind) started to collect; (2) the buffer's stream is made to wait for
 * train_stream and then runs rb_update_sample_many with these n mini-batches:
 * step i updates the buffer with mini-batch i and writes the representatives
 * for iteration first_step + i + 1 to next_x[i] / next_y[i].  When the shape
 * is eligible, several of the steps share one launch (see
 * rb_update_sample_many), and an rb_announce_next_many before this call lets
 * its last launch plan the first steps of the following call.  The training
 * computation of iteration first_step, enqueued on train_stream afterwards,
 * overlaps (2); before iteration first_step + 1 the caller makes train_stream
 * wait for this call's representatives with rb_pipeline_drain (they are all
 * complete then), and trains the remaining n - 1 iterations of the group.
 * Every iteration thus trains on exactly the representatives that
 * rb_pipeline_step would have given it.  Arguments, limits and errors are those
 * of rb_update_sample_many; *ready_rows as in rb_pipeline_step.  n = 0 does
 * nothing.  On an error nothing was enqueued and the pipeline is unchanged.
 */
int rb_pipeline_step_many(rb_pipeline *p, int64_t n, const void *const *batch_x, const int64_t *const *batch_y,
                          int64_t b, int64_t c, int64_t r, uint64_t seed, uint64_t first_step,
                          void *const *next_x, int64_t *const *next_y, void *train_stream, int64_t *ready_rows);
int rb_pipeline_destroy(rb_pipeline *p);

/*
 * Synchronise the bound stream and copy state to the host: fill_host[classes]
 * (samples held per class), *last_n_host (n of the latest rb_sample_augment),
 * *flags_host (RB_FLAG_*).  Any pointer may be null.  Not for the hot path.
 */
int rb_read_state(rb_buffer *rb, int32_t *fill_host, int64_t *last_n_host, uint32_t *flags_host);

/*
 * Synchronise the bound stream and report how many sample rows the kernels have
 * moved since the last bind: every candidate that was actually stored (one that
 * loses its slot to a later candidate is not moved) and every representative
 * that was handed out.  2 * row_bytes times the difference between two readings
 * is the sample traffic of the steps in between.  Not for the hot path.
 */
int rb_read_moved_rows(rb_buffer *rb, uint64_t *rows_host);

/* Launch-shape knobs for measurement sweeps.  RB_OPT_UNROLL: 16-byte vectors a
 * thread keeps in flight while moving a row (0 = automatic, else 1, 2, 4 or 8).
 * RB_OPT_NONTEMPORAL: 1 (default) moves rows with streaming loads/stores, 0
 * with plain ones.  RB_OPT_ROWS_PER_BLOCK: rows one workgroup moves one after
 * the other when a row fits a single tile (0 = automatic, else 1..16).
 * RB_OPT_FUSE: 1 (default) lets rb_update_sample use its single-launch form,
 * 0 makes it always enqueue the two kernels.  RB_OPT_WINDOW: most steps that
 * rb_update_sample_many puts into one launch (1..32, default 32; 1 = one
 * launch per step).  RB_OPT_PLANNERS: which of its two several-steps forms
 * rb_update_sample_many uses for a shape that both can serve (at most 64
 * candidates and representatives, at most 1024 classes, exact selection):
 * 0 (default) = the library chooses by the time a step's rows take to move,
 * 1 = one workgroup per launch plans the next launch's steps one after the
 * other (up to 32 steps per launch), 2 = two workgroups per step plan them
 * side by side (up to 16 steps per launch).  Results do not depend on it. */
enum rb_option { RB_OPT_UNROLL = 0, RB_OPT_NONTEMPORAL = 1, RB_OPT_ROWS_PER_BLOCK = 2, RB_OPT_FUSE = 3, RB_OPT_WINDOW = 4,
                 RB_OPT_PLANNERS = 5 };
int rb_set_option(rb_buffer *rb, int32_t option, int64_t value);

/* Free the host handle.  Device memory stays the caller's. */
int rb_destroy(rb_buffer *rb);

/* Static description of an rb_status. */
const char *rb_strerror(int status);

/* ---- measurement helpers (not part of the method) ----------------------- */

/*
 * Stand-in for the training computation that buffer management overlaps with
 * (Sec. IV-D): a register-only multiply-add loop of `iters` iterations on
 * `blocks` workgroups of 256 threads; every thread writes one float to
 * sink[blocks*256] (device) so the loop is not optimised away.
 */
int rb_standin_compute(void *hip_stream, float *sink, int64_t blocks, int64_t iters);

/*
 * Plain contiguous device-to-device copy of `bytes` (multiple of 16, both
 * pointers 16-byte aligned) with the same per-thread inner loop the row mover
 * uses: the practical ceiling of that loop, and an HBM-bound stand-in load.
 * unroll: 1, 2, 4 or 8 vectors per thread.  nontemporal: 0 - plain loads and
 * stores; 1 - streaming ones, every store waited for before the next (the
 * one-step kernels' form); 2 - streaming ones, the stores of a tile in one
 * burst (the several-steps kernel's form).
 */
int rb_copy_bytes(void *hip_stream, void *dst, const void *src, size_t bytes, int32_t unroll, int32_t nontemporal);

#ifdef __cplusplus
}
#endif
#endif /* RB_H */
