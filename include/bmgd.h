/*
 * bmgd.h -- C ABI of the buffered mini-batch gradient descent (BMGD) library
 * for one AMD Instinct MI355X (gfx950).
 *
 * The library implements the *computation step* of the paper's Algorithm 1
 * (Section 2.2): a buffer of rows (X_i, Y_i) that already sits in GPU memory
 * is swept for T passes; each pass starts with a fresh random partition of the
 * buffer into mini-batches and then applies, strictly in order, the update of
 * eq. (2.1)
 *
 *      theta <- theta - alpha * (1/n_b) * sum_{i in mini-batch} grad l(X_i, Y_i; theta)
 *
 * for least squares (Section 3.1, eq. (3.1)), logistic regression (Section
 * 3.2.3 with b' = sigmoid, Section 4.1) or softmax regression (the C-class
 * member of the same family).  The estimate left by one buffer is the start of
 * the next (Section 2.2).  While one buffer is being computed on, the next one
 * is copied host -> device into a second slot on another stream: the paper's
 * "buffering step", which it wants executed fully in parallel (Section 2.1).
 *
 * The caller owns the loops over iterations r = 1..R and buffers k = 1..K of
 * Algorithm 1: per buffer it calls bmgd_load_buffer_async() and then
 * bmgd_run_buffer().  All work is enqueued on the caller's HIP streams (plus,
 * in BMGD_CHAIN_GRAM mode, one stream of the library's own, see below); the
 * calls that block the host are bmgd_get_theta(), bmgd_set_theta(),
 * bmgd_get_perm(), bmgd_get_stats(), bmgd_sync(), bmgd_eval_loss(), bmgd_get_swa(),
 * bmgd_set_lr_schedule(), bmgd_reset_optimizer(), bmgd_destroy() and (for
 * part of its passes) bmgd_run_buffer_adaptive().
 * The run calls keep a few events per buffer for the statistics; once 4096
 * runs have been enqueued since the last blocking call, the next run call
 * waits until the older half of them has finished and folds their timings,
 * so a caller that never synchronises is at most some thousand buffers ahead
 * of the device and holds a bounded number of events.
 *
 * General rules
 *   - Every function is extern "C", never throws and never aborts.  Except for
 *     bmgd_create(), bmgd_workspace_bytes() and bmgd_last_error() they return a
 *     status code; on failure bmgd_last_error() holds a message.
 *   - A context belongs to one host thread at a time (no internal locking) and
 *     to the HIP device that was current when it was created.
 *   - "host" pointers are ordinary or pinned host memory, "device" pointers are
 *     HIP device memory on the context's device.  Streams are hipStream_t
 *     values passed as void* (NULL = the default stream).  Keep all streams at
 *     the default priority.  HIP spreads a process's streams over a few
 *     hardware queues (four by default) and work on streams that share a queue
 *     runs one after the other, copies included: a process that wants the copy
 *     of one buffer to overlap the computation on another keeps the number of
 *     streams it uses small (default stream, one copy stream, one compute
 *     stream, the library's chain stream) and reuses them.
 *   - If no usable GPU is present every call that needs one fails with
 *     BMGD_EHIP; there is no CPU fallback.
 *   - A run that fails after part of its work has been enqueued, a device-side wait that exceeds
 *     barrier_timeout_us (the persistent kernels need all their workgroups resident at once: work of
 *     other streams that holds compute units for longer than the limit makes a run give up; it exits by
 *     itself and the next blocking call returns BMGD_EHIP) and a row subset with an index outside its
 *     buffer leave theta undefined.  From then on every run call returns BMGD_ESTATE until theta has been
 *     set again with bmgd_set_theta() (bmgd_set_position() and bmgd_reset_optimizer() restore the rest of
 *     a checkpoint); nothing is retried automatically, because runs enqueued behind the failed one have
 *     already used its result.
 */
#ifndef BMGD_H
#define BMGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bmgd_ctx bmgd_ctx;

/* In BMGD_CHAIN_GRAM mode the sequential chain runs on a stream the library creates (default priority) while
 * everything that reads the caller's buffer stays on compute_stream, so that the pre-pass over buffer k + 1
 * overlaps the chain of buffer k.  The blocking calls listed above wait for that stream too; a caller that
 * synchronises compute_stream by itself has waited for the reads of its buffers, not for the updates. */

/* status codes */
enum {
    BMGD_OK = 0,
    BMGD_EINVAL = 1,    /* bad argument (also: a shape outside the supported range) */
    BMGD_ESTATE = 2,    /* call out of order, e.g. run with nothing loaded */
    BMGD_EHIP = 3,      /* a HIP call failed, no GPU, or a kernel reported a time-out */
    BMGD_ENOMEM = 4     /* device or host allocation failed / workspace too small */
};

/* per-sample loss l (what grad l is) */
enum {
    BMGD_LINEAR = 0,    /* (x'theta - y) x            -- eq. (3.1) */
    BMGD_LOGISTIC = 1,  /* (sigmoid(x'theta) - y) x   -- Section 3.2.3, y in {0,1} */
    BMGD_SOFTMAX = 2    /* x (softmax(x'W) - onehot(y))', W is p x C row-major */
};

/* storage type of X */
enum { BMGD_F32 = 0, BMGD_BF16 = 1 };

/* how mini-batch partitions are drawn */
enum {
    BMGD_RESHUFFLE_PER_PASS = 0, /* Algorithm 1: a new partition for every pass of every buffer */
    BMGD_RESHUFFLE_FIXED = 1     /* Section 3.1.1: one partition per buffer index k, reused for all r, t */
};

/* how the sequential chain of mini-batch steps is driven */
enum {
    BMGD_CHAIN_AUTO = 0,
    BMGD_CHAIN_PERSISTENT = 1,   /* one persistent kernel per buffer; workgroups exchange sums once per step */
    BMGD_CHAIN_LAUNCH = 2,       /* kernel launches per step, in stream order */
    BMGD_CHAIN_GRAM = 3,         /* least squares with p <= 128 only: the update in the form of eq. (3.1),
                                    theta <- (I - alpha Sxx_m) theta + alpha Sxy_m.  The moment matrices of every
                                    mini-batch of a pass are formed first, in parallel over the buffer (each row
                                    read once), and the sequential chain then runs inside one workgroup at p^2
                                    multiply-adds per step.  Same result as the row form up to the order of
                                    summation.  BMGD_CHAIN_AUTO picks the moment form when it applies and batch_n >= 2 p: this
                                    mode, or BMGD_CHAIN_PRODUCT (see there). */
    BMGD_CHAIN_GRAPH = 4,        /* softmax only (its BMGD_CHAIN_AUTO): the launches of one pass over one buffer - the transpose of
                                    its mini-batches, then logits, residual and gradient + update per mini-batch - are captured
                                    once into a HIP graph per (buffer address, rows, partition slot) and replayed; learning
                                    rate and update counts are read from device memory, so a replay needs no new capture.
                                    BMGD_CHAIN_LAUNCH issues the same launches one by one. */
    BMGD_CHAIN_PRODUCT = 5       /* least squares with p <= 128 and plain steps (BMGD_OPT_SGD) only: the moment form of
                                    BMGD_CHAIN_GRAM with steps multiplied together.  A step of eq. (3.1) is the affine map
                                    [theta; 1] <- A_m [theta; 1], A_m = [[I - alpha Sxx_m, alpha Sxy_m], [0, 1]], and no A_m
                                    depends on theta, so products of steps can be formed in parallel on the matrix cores (the
                                    products of eq. (3.2)).  Neighbouring steps are multiplied in pairs behind the kernel that
                                    forms the moment matrices, and the sequential chain runs over half as many steps.  With
                                    cache_moments (fixed partitions) the whole product of a run over a buffer is formed, in
                                    log2 rounds, and kept per buffer index as long as the learning rate and the number of
                                    passes stay the same (no table of rates): every later run over that buffer is one
                                    matrix-vector product.  Same result as the chain up to the order of the fp32 operations;
                                    intermediate estimates are not formed.  Needs scratch of about 3/4 N matrices of
                                    (p + 1 rounded up to 16)^2 floats, twice, for the N steps of up to four passes; rejected
                                    if that exceeds 1 GiB.  BMGD_CHAIN_AUTO picks it, in place of BMGD_CHAIN_GRAM, for plain
                                    steps without cache_moments when a launch has at least 64 steps (bmgd_get_stats reports
                                    the mode in use). */
};

/* update rule fed with the mini-batch gradient g of eq. (2.1) (Section 4.3 combines the buffering idea with NAG and
 * Adam: "BNAG", "BAdam").  State (v; m and s) starts at zero and is carried across buffers like theta.
 *   BMGD_OPT_SGD       theta <- theta - alpha g                                                 (Algorithm 1)
 *   BMGD_OPT_MOMENTUM  v <- mu v - alpha g;  theta <- theta + v
 *   BMGD_OPT_NAG       v <- mu v - alpha g;  theta <- theta + mu v - alpha g
 *   BMGD_OPT_ADAM      m <- b1 m + (1 - b1) g;  s <- b2 s + (1 - b2) g^2;  k <- k + 1;
 *                      theta <- theta - alpha (m / (1 - b1^k)) / (sqrt(s / (1 - b2^k)) + eps) */
enum { BMGD_OPT_SGD = 0, BMGD_OPT_MOMENTUM = 1, BMGD_OPT_NAG = 2, BMGD_OPT_ADAM = 3 };

typedef struct bmgd_config {
    int64_t  p;            /* features per row (> 0) */
    int64_t  buffer_n;     /* N0: rows a slot can hold (> 0, < 2^30) */
    int64_t  batch_n;      /* n: rows per mini-batch (1 <= n <= buffer_n); a short last batch is averaged
                              over its own size */
    double   lr;           /* alpha: finite, > 0 */
    int32_t  passes;       /* T >= 1 */
    int32_t  model;        /* BMGD_LINEAR / BMGD_LOGISTIC / BMGD_SOFTMAX */
    int32_t  n_classes;    /* C >= 2 for softmax; ignored (treated as 1) otherwise */
    int32_t  x_dtype;      /* BMGD_F32 (linear, logistic) or BMGD_BF16 (softmax) */
    uint64_t seed;         /* seed of the partition generator */
    int32_t  reshuffle;    /* BMGD_RESHUFFLE_* */
    int32_t  n_buffers;    /* K; used only by BMGD_RESHUFFLE_FIXED (partition index = buffer counter mod K);
                              0 = use the buffer counter itself */
    int32_t  chain;        /* BMGD_CHAIN_* */
    int32_t  n_workgroups; /* workgroups taking part in each step; 0 = chosen from the shape.  At most one per compute unit;
                              two of the persistent kernels take multiples of 8 (a request is rounded down; bmgd_get_stats
                              reports what is used) */
    int64_t  barrier_timeout_us; /* upper bound on any single device-side wait; 0 = default (2 s).
                              A wait that exceeds it makes the kernel exit and the next blocking call
                              return BMGD_EHIP. */
    void*    workspace;    /* optional device memory for everything the context needs on the device;
                              NULL = the library allocates (and frees) it.  Must be 256-byte aligned and
                              stay valid until bmgd_destroy(). */
    size_t   workspace_bytes;
    int32_t  optimizer;    /* BMGD_OPT_*; anything but BMGD_OPT_SGD adds one or two theta-sized state arrays */
    int32_t  cache_moments; /* 0 / 1: with BMGD_RESHUFFLE_FIXED in the moment form, keep the moment matrices of each of
                              the n_buffers buffer indices on the device once formed (see bmgd_run_cached_buffer) */
    double   momentum;     /* mu of MOMENTUM / NAG, in [0, 1) */
    double   beta1;        /* Adam, in [0, 1) */
    double   beta2;        /* Adam, in [0, 1) */
    double   eps;          /* Adam, >= 0 */
} bmgd_config;

typedef struct bmgd_stats {
    int64_t buffers_run;       /* completed bmgd_run_* enqueues (= the buffer counter b) */
    int64_t steps;             /* mini-batch updates enqueued so far */
    int64_t sample_gradients;  /* rows visited, summed over steps */
    int64_t h2d_bytes;         /* bytes handed to host->device copies by bmgd_load_buffer_async */
    double  copy_ms;           /* device time spent in those copies (event-timed, completed ones) */
    double  compute_ms;        /* device time spent in bmgd_run_* work (event-timed, completed ones) */
    double  wait_ms;           /* part of copy_ms that was not overlapped by compute: sum over runs of the part of
                                  the run's copy that came after every earlier run had finished.
                                  1 - wait_ms / copy_ms = fraction of the host->device time that was hidden */
    int32_t n_workgroups;      /* launch shape in use */
    int32_t threads_per_group;
    int32_t chain;             /* resolved BMGD_CHAIN_* */
    int32_t reserved;
    double  chain_ms;          /* device time inside the chain kernels alone (events around each launch of the
                                  persistent kernel; in step-per-launch mode: around each pass-chunk of launches) */
    int64_t chain_launches;    /* number of such timed launches */
    double  prep_ms;           /* BMGD_CHAIN_GRAM only: device time inside the kernels that form the moment matrices
                                  (they run on the compute stream and overlap the chain of the buffer before) */
    int64_t prep_launches;     /* number of those launches */
} bmgd_stats;

/* Fill *cfg with defaults: linear model, fp32, 1 class, seed 0, per-pass reshuffle, automatic launch
 * shape, library-owned memory, plain gradient steps (momentum 0.9, beta1 0.9, beta2 0.999, eps 1e-8 if another
 * optimizer is chosen).  p, buffer_n, batch_n, lr, passes are left 0 for the caller to set. */
void bmgd_default_config(bmgd_config* cfg);

/* Algorithm 1's inputs (alpha, M via batch_n, T) plus the buffer capacity.  Defaults as above, theta = 0.
 * Returns NULL on failure (invalid argument, no GPU, out of memory). */
bmgd_ctx* bmgd_create(int64_t p, int64_t buffer_n, int64_t batch_n, double lr, int passes);

/* Full form.  *out receives the context.  Errors: BMGD_EINVAL (see field comments; also p above the
 * supported maximum: 4096 if p % 4 == 0, 2048 if p % 2 == 0, else 1024 for the GLM models),
 * BMGD_EHIP, BMGD_ENOMEM.  Also BMGD_EINVAL from the run calls when min(passes, 4) * ceil(rows / batch_n)
 * reaches 2^23 (step indices inside one kernel launch are kept below that). */
int bmgd_create_ex(const bmgd_config* cfg, bmgd_ctx** out);

/* Device bytes a context with this configuration needs (two buffer slots, partitions, theta and its running
 * average, optimizer state, scratch; in BMGD_CHAIN_GRAM mode also two sets of moment matrices of
 * 4 * ceil(buffer_n / batch_n) * (p + 1) * roundup(p, 4) floats each, and with cache_moments n_buffers more of a
 * quarter of that size); 0 if the configuration is invalid.  Needs no GPU. */
size_t bmgd_workspace_bytes(const bmgd_config* cfg);

/* Buffering step (Section 2.1; Algorithm 1's "start preparing buffered data"): enqueue on copy_stream the
 * copy of `rows` rows into the slot that is not being computed on.
 *   host_x  host, row-major [rows][p], fp32 or bf16 per x_dtype.  Pinned memory is needed for the copy
 *           to overlap with compute.
 *   host_y  host, [rows]: fp32 responses (0/1 for logistic) or int32 class ids for softmax.  Class ids must lie in
 *           [0, C): they are not checked, and an id outside that range makes its row count as belonging to no class.
 * The memory must stay valid and unchanged until the copy has completed (bmgd_sync, or a
 * synchronisation of copy_stream by the caller).  The copy waits, on the device, for the run that last
 * read the target slot.  At most one loaded-but-not-run buffer may exist: a second load without a run in
 * between returns BMGD_ESTATE.  rows must satisfy 1 <= rows <= buffer_n. */
int bmgd_load_buffer_async(bmgd_ctx* ctx, const void* host_x, const void* host_y, int64_t rows,
                           void* copy_stream);

/* Computation step on the most recently loaded buffer: enqueue on compute_stream T passes of sequential
 * mini-batch updates (eq. (2.1)), after a device-side wait for that buffer's copy.  Partitions are
 * PERM(seed, b, t, rows) for pass t = 1..T with b the number of buffers run before this one (or
 * PERM(seed, b mod K, 0, rows) in fixed mode).  Returns BMGD_ESTATE if nothing is loaded. */
int bmgd_run_buffer(bmgd_ctx* ctx, void* compute_stream);

/* Computation step with as many passes as the buffering step leaves time for (Section 2.1: the updates on the
 * buffer in hand go on until the next buffer has been prepared).  Starts the copy of the next buffer
 * (next_host_x, next_host_y, next_rows: as for bmgd_load_buffer_async, on copy_stream) and makes passes
 * t = 1, 2, ... over the loaded buffer on compute_stream, one launch per pass, until that copy has completed, but
 * never fewer than min_passes nor more than max_passes (1 <= min_passes <= max_passes <= 2^20); the passes value
 * of the context is not used.  The copy's completion is looked at before each pass is enqueued, with at most two
 * passes enqueued and unfinished, so the last pass starts at most two passes after the copy has ended.
 * *passes_done (may be NULL) receives the number of passes made: it depends on timing, and so does theta; a run
 * of bmgd_run_buffer with that many passes gives the same theta.  On return the next buffer is the loaded one.
 * next_host_x = next_host_y = NULL: there is no next buffer, min_passes passes are made.
 * Blocks the host while it waits for passes to finish (all but the last two); returns BMGD_ESTATE if nothing is
 * loaded. */
int bmgd_run_buffer_adaptive(bmgd_ctx* ctx, void* compute_stream, const void* next_host_x, const void* next_host_y,
                             int64_t next_rows, void* copy_stream, int min_passes, int max_passes, int* passes_done);

/* ---- Fixed partitions: moment matrices formed once (Section 3.1.1 fixes the buffers and their partitions for all
 * iterations, and eq. (3.1) then needs of a mini-batch only its two moment matrices) --------------------------------
 * With cache_moments = 1 (least squares in the moment form, BMGD_RESHUFFLE_FIXED, n_buffers = K >= 1) the first run over
 * buffer index k = b mod K forms the moment matrices of its M mini-batches and keeps them (K * M * (p + 1) * roundup(p, 4)
 * floats of device memory); every later run over index k is the chain of updates alone and reads no row.  The caller
 * promises that index k holds the same rows in every iteration.  Such later runs may be made with any run call (the
 * rows passed are then ignored) or with bmgd_run_cached_buffer, which needs no rows at all: no copy, no slot.
 * bmgd_run_cached_buffer returns BMGD_ESTATE if the next index is not cached yet.  A run with a row subset set does
 * not use the cache.  bmgd_clear_moment_cache (blocks) forgets all cached matrices, e.g. before new data. */
int bmgd_run_cached_buffer(bmgd_ctx* ctx, void* compute_stream);
int bmgd_clear_moment_cache(bmgd_ctx* ctx);

/* ---- Running on part of a buffer (Section 4.2: for data with few positive responses the negative instances of
 * each buffer are undersampled, so that mini-batches are roughly balanced) ---------------------------------------
 * The next run call (any of them; one run only) works on the rows dev_idx[0 .. count) of its buffer instead of all
 * of them: it partitions those count rows, M = ceil(count / batch_n), PERM(seed, b, t, count), and a row may be
 * listed more than once.  Which rows to keep is the caller's choice (e.g. all positives and as many negatives drawn
 * at random).  dev_idx: device memory, int32, valid until the run has completed; count <= rows of the buffer
 * (checked when the run is enqueued); count = 0 cancels.  Entries outside the buffer are not followed: row 0 is used
 * in their place and the next blocking call returns BMGD_EINVAL. */
int bmgd_set_row_subset(bmgd_ctx* ctx, const int32_t* dev_idx, int64_t count);

/* ---- Averaging of estimates (Section 4.4: the buffering idea combined with stochastic weight averaging, which
 * averages the weights after every so many epochs) --------------------------------------------------------------
 * bmgd_swa_update folds the estimate as it stands after all runs enqueued so far into a running average kept on
 * the device: avg <- avg + (theta - avg) / k for the k-th call (the first call copies theta).  The caller decides
 * when (say after every five buffers).  Asynchronous: one small kernel, enqueued behind the last update of theta;
 * compute_stream must be the stream of the run calls.  bmgd_get_swa copies the average to host_out (layout and len
 * as bmgd_get_theta; blocks) and stores the number of snapshots in *count (may be NULL); BMGD_ESTATE before the
 * first update.  bmgd_swa_reset makes the next update start a new average. */
int bmgd_swa_update(bmgd_ctx* ctx, void* compute_stream);
int bmgd_get_swa(bmgd_ctx* ctx, float* host_out, int64_t len, int64_t* count);
int bmgd_swa_reset(bmgd_ctx* ctx);

/* ---- Reading buffers from storage (the first of the two transfers of Section 2.1) -----------------------------
 * A reader owns a host thread that reads consecutive buffers of a data set from two flat files into a ring of
 * pinned host buffers, ahead of the consumer, so that bmgd_load_buffer_async() always finds its next buffer in
 * memory and the copy to the device can overlap both the reading and the computation.
 *   x_path   row-major [n_rows][p] fp32 or bf16 (x_dtype), no header
 *   y_path   [n_rows] 4-byte items (fp32 responses or int32 class ids), no header
 * Buffer k is rows [k buffer_n, min((k + 1) buffer_n, n_rows)); buffers are delivered in file order, and again from
 * the start after the last one if loop != 0 (iterations r = 1, 2, ... of Algorithm 1).  ring_slots in [2, 64] pinned
 * buffers of buffer_n rows are allocated.  Must be called with the device current on which the contexts it feeds
 * live.  Errors: BMGD_EINVAL (arguments, missing or short file), BMGD_EHIP, BMGD_ENOMEM; message from
 * bmgd_reader_last_error(NULL) for a failed open (per calling thread), else from the reader. */
typedef struct bmgd_reader bmgd_reader;
int bmgd_reader_open(const char* x_path, const char* y_path, int64_t p, int32_t x_dtype, int64_t n_rows,
                     int64_t buffer_n, int32_t ring_slots, int32_t loop, bmgd_reader** out);

/* Blocks until the next buffer is in memory and hands it out: *host_x, *host_y point into the ring (pinned; owned by
 * the reader), *rows is its row count.  *rows = 0 with BMGD_OK: the data set has been delivered completely
 * (loop = 0).  BMGD_ESTATE if every slot is handed out; BMGD_EINVAL if reading failed (see bmgd_reader_last_error). */
int bmgd_reader_acquire(bmgd_reader* r, const void** host_x, const void** host_y, int64_t* rows);

/* Hands back the oldest buffer that is handed out.  after_stream != 0: the reader refills it only once everything
 * enqueued on copy_stream up to now has completed (call it right after enqueueing the copy out of the buffer);
 * after_stream = 0: it may be refilled at once. */
int bmgd_reader_release(bmgd_reader* r, void* copy_stream, int32_t after_stream);

/* bmgd_reader_acquire + bmgd_load_buffer_async + bmgd_reader_release(after the copy) in one call.  *rows_out = rows
 * of the buffer now loaded, 0 at the end of the data (then nothing was loaded). */
int bmgd_load_from_reader(bmgd_ctx* ctx, bmgd_reader* r, void* copy_stream, int64_t* rows_out);

/* bmgd_run_buffer_adaptive with the next buffer taken from a reader: before every pass the reader is asked (without
 * blocking) whether its next buffer is in host memory; as soon as it is, its copy to the device starts (and the ring
 * slot is handed back behind that copy), and the passes go on until the copy has completed.  So the device keeps
 * working through both transfers of Section 2.1.  *next_rows (may be NULL) receives the rows of the buffer that is
 * loaded on return, 0 if the data set has been delivered completely (loop = 0): then nothing is loaded.  If
 * max_passes is reached before the reader has the buffer, the call waits for it and starts its copy before returning. */
int bmgd_run_buffer_adaptive_reader(bmgd_ctx* ctx, void* compute_stream, bmgd_reader* reader, void* copy_stream,
                                    int min_passes, int max_passes, int* passes_done, int64_t* next_rows);

/* Bytes read from the files so far and the time the reading thread spent inside read calls. */
int bmgd_reader_stats(bmgd_reader* r, int64_t* bytes_read, double* read_seconds);
const char* bmgd_reader_last_error(bmgd_reader* r);
/* Stops the thread, waits for copies out of the ring that the reader was told about, frees the ring. */
void bmgd_reader_close(bmgd_reader* r);

/* Same computation step on a buffer that is already resident in device memory and owned by the caller
 * (no copy, no slot): dev_x [rows][p], dev_y [rows], 256-byte aligned, valid until the work completes. */
int bmgd_run_device_buffer(bmgd_ctx* ctx, const void* dev_x, const void* dev_y, int64_t rows,
                           void* compute_stream);

/* Wait for all enqueued work, then copy theta to host_out (fp32, p values; p*C row-major [p][C] for
 * softmax).  len must equal that count.  This is Algorithm 1's output when called after the last buffer. */
int bmgd_get_theta(bmgd_ctx* ctx, float* host_out, int64_t len);

/* Wait for all enqueued work, then overwrite theta (the initial value of Algorithm 1, or a checkpoint).  The state
 * of the optimizer is left as it is; bmgd_reset_optimizer() zeroes it.  Also the way back after a failed or
 * abandoned run (see the general rules): the failure, if not reported yet, is not reported by this call. */
int bmgd_set_theta(bmgd_ctx* ctx, const float* host_in, int64_t len);

/* Wait for all enqueued work, then set the optimizer's state (v; m, s and the update count k) back to zero. */
int bmgd_reset_optimizer(bmgd_ctx* ctx);

/* Schedules (Theorem 4 lets the learning rate alpha_r and the number of passes T_r change with the iteration r;
 * Section 4 uses stage-wise T): both take effect for buffers run after the call, need no synchronisation and
 * leave theta and the buffer counter alone.  lr: finite, > 0; passes >= 1. */
int bmgd_set_lr(bmgd_ctx* ctx, double lr);
int bmgd_set_passes(bmgd_ctx* ctx, int passes);

/* A learning rate per mini-batch update (Theorem 4 lets alpha vary over the run; Section 4.4 trains with a cosine
 * schedule): the u-th update enqueued after this call (u = 0, 1, ...) uses host_alphas[min(u, len - 1)], whatever
 * buffer and pass it belongs to; lr and bmgd_set_lr are ignored while a schedule is set.  len = 0 (host_alphas may
 * then be NULL) removes the schedule.  Every value must be finite and > 0.  The table is copied: to device memory
 * that the library allocates for it (this call is the only one besides bmgd_create* that allocates), and to the
 * host.  Waits for all enqueued work first. */
int bmgd_set_lr_schedule(bmgd_ctx* ctx, const float* host_alphas, int64_t len);

/* Set the buffer counter b (wait-free); with bmgd_set_theta this resumes a run exactly. */
int bmgd_set_position(bmgd_ctx* ctx, int64_t buffer_counter);

/* Parity hook: compute on the device, and copy to host_out, the partition PERM(seed, buffer_counter,
 * pass, len) exactly as a run would use it (pass 0 = the fixed-mode partition).  Blocks. */
int bmgd_get_perm(bmgd_ctx* ctx, int64_t buffer_counter, int pass, int32_t* host_out, int64_t len);

/* Evaluation (the experiments of Section 4 report the loss / mean squared error along the run): wait for all
 * enqueued work, then compute on `stream` the mean over the rows of a device-resident buffer of the per-sample
 * loss at the current theta -- (x'theta - y)^2 / 2, log(1 + e^u) - y u with u = x'theta, or the softmax
 * cross-entropy (logits from the bf16 copy of W, as in the updates) -- and return it in *host_out.  fp32 per row,
 * fp64 sums in a fixed order.  dev_x, dev_y, rows as for bmgd_run_device_buffer (rows may exceed buffer_n).  Blocks. */
int bmgd_eval_loss(bmgd_ctx* ctx, const void* dev_x, const void* dev_y, int64_t rows, void* stream, double* host_out);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the mean loss of bmgd_eval_loss for the least-squares and logistic models, without a context.
 * The per-workgroup partial sums go to a static device array of the library (1024 doubles = 8 KiB on every device the
 * library runs on, held until the process ends) instead of a context's workspace, and the result is left in device
 * memory: the call enqueues two kernels on `stream` and nothing else - no allocation, no copy, no synchronisation.
 *   model      BMGD_LINEAR or BMGD_LOGISTIC (BMGD_SOFTMAX: BMGD_EINVAL, its logits scratch exceeds the static array)
 *   dev_x      device, row-major [rows][p] fp32, 16-byte aligned;  dev_y  device, [rows] fp32
 *   dev_theta  device, [p] fp32: the point at which the loss is evaluated (read in stream order)
 *   rows       in [1, 2^30);  p in [1, 4096]: larger sizes are rejected with BMGD_EINVAL
 *   dev_out    device, one double: receives the mean loss when the work on `stream` has run
 * fp32 per row, fp64 sums in the fixed order of bmgd_eval_loss (same value bit for bit).  The device that is current
 * at the call is used; `stream` must belong to it.  Every call on one device shares that device's array: calls that
 * overlap on one device (two streams, two threads) race and must be ordered by the caller; calls in stream order are
 * safe, and nothing needs clearing between them.  Message of a failure: bmgd_last_error(NULL), per calling thread. */
int bmgd_eval_loss_static(int32_t model, const float* dev_x, const float* dev_y, const float* dev_theta, int64_t rows,
                          int64_t p, void* stream, double* dev_out);

/* Wait for all enqueued work (both streams last used) and report a device-side time-out if one happened. */
int bmgd_sync(bmgd_ctx* ctx);

/* Counters and event timings; blocks like bmgd_sync. */
int bmgd_get_stats(bmgd_ctx* ctx, bmgd_stats* out);

/* Message for the last failure on this context; with ctx == NULL, for the last failed bmgd_create*. */
const char* bmgd_last_error(const bmgd_ctx* ctx);

/* Wait for enqueued work and release everything the library allocated.  NULL is ignored. */
void bmgd_destroy(bmgd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* BMGD_H */
