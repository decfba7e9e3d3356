/*
 * clockwork_exec.h -- C ABI of the MI355X worker hot path: the steps of an INFER
 * action on one GPU (INPUT -> EXEC -> OUTPUT) plus LOAD / UNLOAD of weights and a
 * measured EXEC-latency profile per (model, batch size).
 *
 * The call set follows the action model of the paper (section 4.4 "Predictable DNN
 * Worker", section 5.1 "Models", section 5.2 "DNN Workers"):
 *   - a model is weights + kernels per batch size + static memory metadata + a
 *     seed latency profile (section 5.1);
 *   - all device memory is allocated once and split into a workspace for
 *     intermediates, an IO cache for inputs/outputs and a pool for weights
 *     (section 5.2, "Managing model weights in memory");
 *   - INFER = INPUT, EXEC, OUTPUT; EXEC checks that weights and input are present
 *     and runs the kernels; one EXEC at a time per GPU (sections 4.4, 5.2);
 *   - every action reports a status and its on-device duration (section 5.2,
 *     "Results").
 *
 * Conventions
 *   - Every call returns an int32_t status: CW_OK (0) or a negative CW_ERR_*.
 *     No exception crosses this boundary.  cw_strerror() names a status;
 *     cw_last_error() gives detail for the last failing call on a context.
 *   - Pointers marked [host] are host memory owned by the caller; the library owns
 *     all device memory.  The device pools (workspace, IO cache, weight pool, LOAD
 *     staging) are allocated once, by cw_create(), and nothing is taken from or returned
 *     to the device allocator afterwards.  Host-side runtime objects are still created
 *     later: one event per model in cw_model_define(), and one recorded HIP graph per
 *     (model, batch size) in cw_load_weights() (recording executes nothing).
 *   - `stream` is a raw hipStream_t (passed as void*; NULL = the default stream).
 *     Calls that take a stream only enqueue work; the caller must keep [host]
 *     buffers alive and unmodified until that stream has been synchronised.  Host
 *     buffers should be pinned for the copies to be asynchronous.
 *   - A context is bound to one GPU and is not thread safe: serialise calls on
 *     one context (the paper's executors are one thread per action type; here the
 *     caller provides that discipline).
 *   - Storage type of weights and activations: fp16 or bf16 (per model);
 *     accumulation is always fp32; biases, logits and probabilities are fp32.
 */
#ifndef CLOCKWORK_EXEC_H
#define CLOCKWORK_EXEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct cw_ctx cw_ctx; /* one per GPU: the paper's "worker-GPU" */

enum {
    CW_OK = 0,
    CW_ERR_INVALID = -1,        /* bad argument (null pointer, unknown id, bad size) */
    CW_ERR_HIP = -2,            /* a HIP runtime call failed; see cw_last_error() */
    CW_ERR_NO_MEMORY = -3,      /* a pre-allocated pool cannot hold the request */
    CW_ERR_NOT_LOADED = -4,     /* EXEC on a model whose weights are not resident */
    CW_ERR_ALREADY_LOADED = -5, /* LOAD of a model that is resident */
    CW_ERR_NO_INPUT = -6,       /* EXEC/OUTPUT on a slot that holds no input / no result */
    CW_ERR_BAD_BATCH = -7,      /* batch size the model has no plan for */
    CW_ERR_BUSY = -8,           /* an EXEC is still in flight on another stream */
    CW_ERR_UNSUPPORTED = -9,    /* topology the kernels cannot run (see cw_model_define) */
    CW_ERR_NO_SLOT = -10,       /* every IO slot is in use */
    CW_ERR_TOO_LATE = -11,      /* an action's executor reached it after its `latest`: not executed */
    CW_ERR_TIMEOUT = -12        /* cw_worker_next_result: no result within the time given */
};

enum { CW_OP_CONV = 0, CW_OP_MAXPOOL = 1, CW_OP_GAVGPOOL = 2, CW_OP_FC = 3, CW_OP_SOFTMAX = 4, CW_OP_CONCAT = 5 };
enum { CW_ACT_NONE = 0, CW_ACT_RELU = 1, CW_ACT_HSWISH = 2 };   /* values of cw_op.relu */
enum { CW_DTYPE_FP16 = 0, CW_DTYPE_BF16 = 1 };

/* One operator of a model.  Ops form a DAG over earlier ops' outputs.
 * CONV:     cross-correlation, kh x kw, `stride`, zero padding, + bias[cout], then (if
 *           residual_from >= 0) + output of that op, then the activation `relu` (CW_ACT_*: none,
 *           ReLU, or hard swish x * min(max(x + 3, 0), 6) / 6).  A square filter is padded by
 *           `pad` on every side; a rectangular one (kh != kw, e.g. 1x7 and 7x1) by `pad` rows and
 *           `pad_w` columns.  groups <= 1: dense; groups == cin == cout: depthwise (one kh x kw
 *           filter per channel, weights W[cout][1][kh][kw]).
 * MAXPOOL:  kh x kw window, `stride`, `pad`; padded taps are ignored.
 * GAVGPOOL: mean over all spatial positions.
 * FC:       cin -> cout, + bias; its fp32 output is the model's logits.
 * SOFTMAX:  over the cout values of each sample; its output is the probabilities.
 * CONCAT:   the channels of op input_from followed by those of op residual_from (same spatial
 *           size; cin = channels of the first, cout = of both).  Where the producers allow it
 *           they write straight into their channel range of the result and nothing is copied.
 * The operators beyond the ResNet set serve the other model families of the paper's Table 1
 * (DenseNet: concatenation; Inception v3: rectangular filters; MobileNet: depthwise, hard swish). */
typedef struct {
    int32_t op;            /* CW_OP_* */
    int32_t cin, cout;     /* channels in / out (MAXPOOL, GAVGPOOL, SOFTMAX: cin == cout) */
    int32_t kh, kw;        /* filter or window size (0 where unused) */
    int32_t stride, pad;
    int32_t relu;          /* CONV only: CW_ACT_* */
    int32_t residual_from; /* CONV: -1 or index of an earlier op to add; CONCAT: the second source */
    int32_t input_from;    /* -1 = the network input, else index of an earlier op */
    int32_t pad_w;         /* CONV with kh != kw: padding in width (`pad` is then the padding in height) */
    int32_t groups;        /* CONV: 0 or 1 = dense, cin = depthwise */
} cw_op;

typedef struct {
    int32_t device;             /* HIP device ordinal */
    size_t workspace_bytes;     /* intermediates of the one EXEC in flight (paper: 512 MB) */
    size_t io_bytes;            /* IO cache: inputs and outputs of in-flight INFERs (paper: 512 MB) */
    size_t weight_pool_bytes;   /* packed weights of all resident models, handed out in pages */
    size_t load_staging_bytes;  /* device landing zone of one canonical blob during LOAD;
                                   must be >= the largest blob that will be loaded */
    size_t weight_page_bytes;   /* page size of the weight pool; 0 = 16 MiB (the paper's, section 5.1);
                                   a multiple of 256, and no weight tensor may be larger */
} cw_config;

/* Section 5.2, "Managing model weights in memory": a worker takes all the device memory it
 * will use when it starts and manages it itself, so that no allocation happens on the path of
 * an action.  cw_create makes one allocation per region of cw_config (+ the streams and events
 * the context needs); cfg [host].  CW_ERR_NO_MEMORY when the device cannot give a region,
 * CW_ERR_UNSUPPORTED on a GPU other than gfx950, CW_ERR_INVALID for a bad ordinal or page
 * size.  device == -1 makes a planning-only context: models and plans can be defined and
 * inspected, every call that would touch a GPU returns CW_ERR_INVALID. */
int32_t cw_create(cw_ctx **out, const cw_config *cfg);
/* The worker shuts down: waits for all work the context enqueued, then frees every region,
 * graph, stream and event.  The handle is invalid afterwards. */
int32_t cw_destroy(cw_ctx *ctx);

/* ---- models (section 5.1: kernels per batch size + memory metadata) ----------
 * Defines a topology and compiles one fixed launch plan per batch size: kernel
 * variant, grid, split-K factor and workspace offsets are functions of (ops, input
 * size, batch) only.  Nothing is tuned or chosen at run time.
 * ops, batch_sizes: [host], copied.  The first op must read the network input
 * (in_c x in_h x in_w, NCHW fp32 at the boundary); the list must end FC, SOFTMAX.
 * Supported: CONV with cin % 32 == 0, cout % 32 == 0 and kh == kw <= 5 anywhere,
 * plus a first CONV with cin <= 4 and kh == kw <= 8; GAVGPOOL over a multiple of 64
 * channels; FC with cin % 256 == 0 reading the GAVGPOOL.  Returns CW_ERR_UNSUPPORTED otherwise,
 * CW_ERR_NO_MEMORY if a plan's workspace exceeds workspace_bytes. */
int32_t cw_model_define(cw_ctx *ctx, const cw_op *ops, int32_t n_ops,
                        int32_t in_c, int32_t in_h, int32_t in_w,
                        const int32_t *batch_sizes, int32_t n_batch,
                        int32_t dtype, int32_t *model_id);
/* ResNet-18 / 50 / 152 (depth) with batch sizes 1,2,4,8,16 (section 5.1 default). */
int32_t cw_model_define_resnet(cw_ctx *ctx, int32_t depth, int32_t in_h, int32_t in_w,
                               int32_t dtype, int32_t *model_id);
/* Copies the model's op list to ops_out[0..cap) [host]; *n_ops = its length. */
int32_t cw_model_get_ops(cw_ctx *ctx, int32_t model_id, cw_op *ops_out, int32_t cap,
                         int32_t *n_ops);
/* Size in bytes of the canonical weight blob LOAD expects (0 for a bad id). */
size_t cw_model_weight_bytes(cw_ctx *ctx, int32_t model_id);
/* Workspace bytes the plan for (model, batch) uses (0 for a bad id / batch). */
size_t cw_model_workspace_bytes(cw_ctx *ctx, int32_t model_id, int32_t batch);

/* ---- LOAD / UNLOAD (section 5.2) ----------------------------------------------
 * Canonical blob [host]: for every op that owns weights (CONV, FC), in op order,
 * W[cout][cin][kh][kw] in the model's storage type, back to back; zero padding to
 * a multiple of 4 bytes; then every bias[cout] as fp32 in the same op order.
 * The weight pool is a set of equal pages (section 5.1; cw_config.weight_page_bytes).  A
 * model's packed tensors were given places in cw_model_weight_pages() pages of its own when it
 * was defined, none straddling a page boundary; LOAD takes that many free pages of the pool,
 * whichever they are (lowest-numbered first; CW_ERR_NO_MEMORY when fewer are free: the
 * paper's LOAD aborts when no pages are free), copies the blob to the device on `stream`
 * and re-lays it out there, tensor by tensor, for the MFMA kernels, which receive each
 * tensor's address as a kernel argument.  The same packed weights serve every batch size.
 * `bytes` must equal cw_model_weight_bytes(). */
int32_t cw_load_weights(cw_ctx *ctx, int32_t model_id, const void *host_blob,
                        size_t bytes, void *stream);
/* The same LOAD in steps, for a caller whose threads share one context under a lock of their
 * own (the worker's executors, section 5.2: LOAD runs beside EXEC), so that the lock is held
 * only while work is enqueued:
 *   cw_load_weights_begin    takes the pages and enqueues the copy and the re-layout on `stream`;
 *                            the model counts as resident from here on (an EXEC waits for the
 *                            copy on its own stream) and runs with plain launches until the end
 *                            step.  Serialise with the other calls on the context.
 *   cw_load_weights_record   records the plans' HIP graphs for the pages taken.  Host work of a few
 *                            milliseconds, nothing executes.  May run while other threads call
 *                            into the same context; only one recording at a time per context.
 *   cw_load_weights_end      installs the recorded graphs (nothing if the model has been unloaded
 *                            meanwhile).  Serialise with the other calls on the context.
 *   cw_load_weights_release  destroys `pending` and the graphs the new ones displaced.  Needs no
 *                            serialisation.  Always call it once for a `pending` that begin returned.
 * cw_load_weights() is these four in a row.  `*pending` is NULL when begin fails. */
typedef struct cw_load_pending cw_load_pending;
int32_t cw_load_weights_begin(cw_ctx *ctx, int32_t model_id, const void *host_blob, size_t bytes,
                              void *stream, cw_load_pending **pending);
int32_t cw_load_weights_record(cw_ctx *ctx, cw_load_pending *pending);
int32_t cw_load_weights_end(cw_ctx *ctx, cw_load_pending *pending);
void    cw_load_weights_release(cw_load_pending *pending);
/* Metadata only; succeeds whether or not the model is resident (section 5.2).  The pages go
 * back to the free list at once; an EXEC of the model that is still queued or running keeps
 * reading them safely, because the next LOAD that takes one of them makes its stream wait for
 * that EXEC's end before it writes. */
int32_t cw_unload_weights(cw_ctx *ctx, int32_t model_id);
/* Free pages of the weight pool: the only memory state a controller needs (section 5.1);
 * in bytes (free pages x page size), and as a count.  cw_model_weight_pages: the pages one
 * LOAD of the model takes (negative: unknown id). */
size_t cw_weight_pool_free(cw_ctx *ctx);
int32_t cw_weight_pages_free(cw_ctx *ctx);
int32_t cw_model_weight_pages(cw_ctx *ctx, int32_t model_id);

/* ---- INFER = INPUT, EXEC, OUTPUT (section 5.2) --------------------------------
 * INPUT: takes an IO slot and copies host_nchw [host], fp32 [batch][in_c][in_h][in_w],
 * to it on `stream`.  *slot receives the slot id.  CW_ERR_NO_SLOT / CW_ERR_NO_MEMORY
 * when the IO cache is full, CW_ERR_BAD_BATCH for a batch without a plan. */
int32_t cw_input(cw_ctx *ctx, int32_t model_id, int32_t batch, const float *host_nchw,
                 int32_t *slot, void *stream);
/* EXEC: checks that the model's weights are resident (else CW_ERR_NOT_LOADED) and
 * that `slot` holds an input of this (model, batch) (else CW_ERR_NO_INPUT /
 * CW_ERR_BAD_BATCH), then enqueues the plan's kernels on `stream`, bracketed by
 * two events.  The stream is made to wait for the slot's INPUT copy and the
 * model's LOAD, so they may have been issued on other streams.  A second EXEC
 * issued on a different stream while one is in flight returns CW_ERR_BUSY; on
 * the same stream EXECs simply run back to back.  EXEC may be repeated on a slot. */
int32_t cw_exec(cw_ctx *ctx, int32_t model_id, int32_t batch, int32_t slot, void *stream);
/* EXEC for callers that cannot allocate: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same plan, same kernels and same results as cw_exec, but
 *   - the input, the logits and the probabilities are the caller's own device buffers:
 *     dev_input_nchw [device] fp32 [batch][in_c][in_h][in_w], dev_logits and dev_probs [device]
 *     fp32 [batch][classes]; the caller orders their producers and consumers on `stream`;
 *   - the intermediates (activations, split-K partial sums and arrival counters) live in an array
 *     built into the library, cw_exec_static_capacity() bytes (80 MiB) per GPU, instead of the
 *     context's workspace: a plan whose intermediates need more returns CW_ERR_NO_MEMORY (see
 *     cw_model_workspace_bytes; ResNet-50 and ResNet-152 at 224x224 fit up to batch 16);
 *   - the call allocates nothing, creates no event or graph and records nothing but kernel
 *     launches (plus one wait for the model's LOAD if that has not finished yet).
 * Every call on a GPU uses that GPU's one array, whatever the context: calls that overlap in time
 * on one GPU (two streams, two contexts) race; on one stream they simply run in order.  The EXEC
 * is not timed and does not take part in cw_exec's one-at-a-time check.
 * CW_ERR_NOT_LOADED / CW_ERR_BAD_BATCH / CW_ERR_INVALID as for cw_exec. */
int32_t cw_exec_static(cw_ctx *ctx, int32_t model_id, int32_t batch, const float *dev_input_nchw,
                       float *dev_logits, float *dev_probs, void *stream);
/* Bytes of intermediates a plan may need to run through cw_exec_static. */
size_t cw_exec_static_capacity(void);
/* OUTPUT: enqueues the copies of the slot's results to host_probs [host]
 * [batch][classes] and, if not NULL, host_logits [host] [batch][classes] on
 * `stream` (after the slot's EXEC), then releases the slot; its memory is reused
 * only after these copies have completed.  CW_ERR_NO_INPUT if no EXEC ran. */
int32_t cw_output(cw_ctx *ctx, int32_t slot, float *host_probs, float *host_logits,
                  void *stream);
/* Section 5.2, INFER: an action that is rejected after its INPUT (its window passed, its EXEC
 * failed) must give its IO-cache entry back without an OUTPUT.  Releases the slot without
 * copying anything out; the memory is reused only after the slot's last EXEC has finished.
 * Succeeds on a slot that is already free. */
int32_t cw_release(cw_ctx *ctx, int32_t slot);
/* On-device duration of the slot's last EXEC (the "timing" field of a result).
 * Blocks until that EXEC has finished. */
int32_t cw_exec_duration_ns(cw_ctx *ctx, int32_t slot, uint64_t *on_device_ns);

/* ---- measured latency profile per (model, batch) (section 5.1 "Profiling data") */
typedef struct {
    uint32_t n;
    float p50_us, p99_us, p999_us, min_us, max_us, mean_us;
    float p9999_us;   /* nearest rank like the others: the maximum for n < 10000 */
} cw_profile;
/* Runs `repeats` EXECs of (model, batch) back to back on an internal stream, each timed on
 * the device, and stores and returns nearest-rank percentiles.  The EXECs read the input held
 * by `slot` (an IO slot of this (model, batch) filled by cw_input; it stays the caller's), or,
 * with slot == -1, a zero-filled input of the library's own.  EXEC time depends slightly on the
 * operand values through power and clocks, so a profile meant to predict real requests should
 * be measured over a representative input.  The EXECs are submitted in bursts of 128; one
 * untimed EXEC leads each burst so that every timed one starts behind queued work.
 * Synchronous.  samples_us [host] may be NULL, else receives the `repeats` individual
 * durations in microseconds. */
int32_t cw_profile_measure(cw_ctx *ctx, int32_t model_id, int32_t batch, int32_t slot,
                           uint32_t repeats, cw_profile *out, float *samples_us);
/* Last measured profile; n == 0 if none was measured. */
int32_t cw_profile_get(cw_ctx *ctx, int32_t model_id, int32_t batch, cw_profile *out);

/* Device ordinal the context was created on (-1: planning only). */
int32_t cw_context_device(cw_ctx *ctx);

/* ---- the worker's executors (section 5.2: actions with `earliest` / `latest`, results) ---------
 * A cw_worker runs one executor thread per action type over one context: LOAD, UNLOAD, and for
 * INFER the three steps INPUT (runs on receipt), EXEC (inherits the action's window; one at a
 * time) and OUTPUT (follows EXEC at once), each with a stream of its own (default priority).  An
 * executor takes its actions in order of `earliest` (arrival order among equals), waits until
 * `earliest`, and does not execute an action it reaches after `latest` (CW_ERR_TOO_LATE; an
 * INFER's IO slot is released).  Every action yields exactly one result.  While a worker exists,
 * the context's own calls must not be used from other threads. */
typedef struct cw_worker cw_worker;
enum { CW_ACTION_LOAD = 1, CW_ACTION_UNLOAD = 2, CW_ACTION_INFER = 3 };
typedef struct {
    int64_t id;                 /* the caller's; returned in the result */
    int32_t type;               /* CW_ACTION_* */
    int32_t model_id;
    int32_t batch;              /* INFER */
    uint64_t earliest_ns;       /* the action may begin from this time on ... */
    uint64_t latest_ns;         /* ... and is rejected when it has not begun by this time; both on the
                                   clock of cw_worker_now_ns() */
    const void *host_in;        /* [host] LOAD: canonical blob; INFER: fp32 [batch][in_c][in_h][in_w];
                                   the caller keeps it alive and unchanged until the result arrives */
    size_t host_in_bytes;       /* LOAD: size of the blob */
    float *host_probs;          /* [host] INFER: [batch][classes], written before the result arrives */
    float *host_logits;         /* [host] INFER: same shape, or NULL */
} cw_action;
typedef struct {
    int64_t id;
    int32_t type;
    int32_t status;             /* CW_OK or the error of the step that failed */
    uint64_t begin_ns, end_ns;  /* host clock: the executor began LOAD / UNLOAD / EXEC (or rejected
                                   the action); the action was complete (INFER: outputs on the host) */
    uint64_t device_ns;         /* on-device duration: EXEC of an INFER, copy and packing of a LOAD; else 0 */
} cw_result;
/* cores [host]: NULL, or 5 CPU numbers (-1 = unpinned) for the LOAD, UNLOAD, INPUT, EXEC and
 * OUTPUT executors; the threads also ask for real-time priority (silently kept at normal
 * priority where the process may not). */
int32_t cw_worker_create(cw_ctx *ctx, const int32_t *cores, cw_worker **out);
/* Stops the executors (actions not yet begun yield no result), waits for the GPU work they
 * issued and frees the worker; the context stays. */
int32_t cw_worker_destroy(cw_worker *w);
/* Monotonic clock of the action windows and result times, in nanoseconds. */
uint64_t cw_worker_now_ns(void);
/* Copies the action [host] and queues it; returns at once.  CW_ERR_INVALID for a malformed one. */
int32_t cw_worker_submit(cw_worker *w, const cw_action *action);
/* Next finished action, in order of completion; waits up to timeout_ns (CW_ERR_TIMEOUT). */
int32_t cw_worker_next_result(cw_worker *w, cw_result *out, uint64_t timeout_ns);
/* Action profile (section 5.3): over the last 10 successful actions of (type, model, batch;
 * batch ignored unless INFER), their count, mean and largest duration (device_ns where the
 * action has one, else end - begin). */
int32_t cw_worker_profile(cw_worker *w, int32_t type, int32_t model_id, int32_t batch, uint32_t *n,
                          uint64_t *mean_ns, uint64_t *max_ns);

/* Section 5.2, "Results": a result carries success or an error code.  cw_strerror names a
 * status (static string, never NULL); cw_last_error gives the detail of the last failing call
 * on a context (NULL context: of the last failing cw_create on this thread); the string is
 * owned by the library and valid until the next call on that context. */
const char *cw_strerror(int32_t status);
const char *cw_last_error(cw_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* CLOCKWORK_EXEC_H */
