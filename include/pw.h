/* pw.h - C boundary of the MI355X (gfx950) build of the Pathways hot path.
 *
 * What is behind it.  The paper's unit of work is the "compiled function": a
 * computation whose input/output types and shapes are known before its inputs
 * exist (Section 3; Appendix B).  Executors enqueue such functions "with buffer
 * futures as inputs" and hand back futures for the outputs at once (Section
 * 4.4); because shapes are static, all host-side work for a chain of functions
 * can run before the first of them has produced anything ("parallel
 * asynchronous dispatch", Section 4.5); buffers live in a device object store
 * and are named by opaque handles (Section 4.6).  The dominant compiled
 * function of the paper's workloads is one accelerator's share of a
 * decoder-only Transformer LM train step (Section 5.3).
 *
 * Here a future is (device buffer, HIP event, status, refcount), the executor
 * is one HIP stream (FIFO, as in Section 4.4), a chain may be replayed as a
 * HIP graph, and the train step is a static list of hand-written gfx950
 * kernels over a static buffer plan.
 *
 * Conventions for every call:
 *  - returns a pw_status; never throws; outputs go through pointer arguments;
 *  - "host" pointers are ordinary process memory, "device" pointers are HIP
 *    device memory on the context's GPU; the caller owns what it passes in;
 *  - the context, function, future, chain, pipeline, program, await, scheduler and model-state calls (pw_model_*,
 *    pw_encdec_*) of one pw_ctx are serialised inside the library, so threads may share a context; the
 *    single-kernel calls (pw_op_*) and pw_profile_* take no lock and must come from one thread at a time;
 *  - on error nothing is enqueued unless the text says otherwise, and
 *    pw_last_error() gives a message.
 * There is no CPU fallback: without a usable GPU pw_ctx_create fails.
 */
#ifndef PW_H_
#define PW_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PW_OK = 0,
  PW_ERR_INVALID = 1,     /* bad handle, null pointer, bad enum value */
  PW_ERR_SHAPE = 2,       /* tensor rank/dims do not match the compiled signature */
  PW_ERR_DTYPE = 3,       /* element type does not match the compiled signature */
  PW_ERR_OOM = 4,         /* device allocation failed */
  PW_ERR_DEVICE = 5,      /* a HIP call failed; see pw_last_error */
  PW_ERR_NOT_READY = 6,   /* pw_future_query: producer has not finished */
  PW_ERR_POISONED = 7,    /* the future, or one it depends on, failed or timed out */
  PW_ERR_UNSUPPORTED = 8
} pw_status;

typedef enum { PW_F32 = 0, PW_BF16 = 1, PW_I32 = 2 } pw_dtype;

typedef struct pw_ctx pw_ctx;       /* device, executor stream, buffer/event pools, handle tables */
typedef struct pw_model pw_model;   /* LM parameters, optimiser state, activation plan; owned by its ctx */
typedef struct pw_encdec pw_encdec; /* the same for the encoder-decoder model */
typedef uint64_t pw_fn;             /* compiled function handle; 0 is never valid */
typedef uint64_t pw_future;         /* buffer-future handle; 0 is never valid */

typedef struct {
  int32_t dtype;                    /* pw_dtype */
  int32_t rank;                     /* 0..4 */
  int64_t dims[4];
} pw_tensor_spec;

/* Kinds of compiled function. */
typedef enum {
  PW_FN_ADD_CONST = 1,   /* y = x + c, fp32; params: one float c.  The trivial computation of the
                            dispatch micro-benchmark (Section 5.1) and "b" of Figure 2. */
  PW_FN_MUL_CONST = 2,   /* y = x * c ("a" of Figure 2) */
  PW_FN_DIV_CONST = 3,   /* y = x / c ("c" of Figure 2) */
  PW_FN_BUSY = 4,        /* y = x + c after spinning params[1] microseconds on the device: a computation
                            of tunable duration for the overhead-masking sweep (Section 5.1) */
  PW_FN_BUSY_CHAIN = 5,  /* params {c, microseconds, count}: PW_FN_BUSY applied count times in a row inside ONE
                            launch - a chain of computations fused into a single node (the "Fused" case of
                            Section 5.1); the result equals count separate PW_FN_BUSY functions bit for bit */
  PW_FN_ADD2 = 6,        /* two inputs of one shape: y = a + b (no params): the fan-in node of dataflow programs */
  PW_FN_LM_TRAIN_STEP = 16, /* in: tokens i32 [B, T+1]; out: loss f32 [1].  params: pw_model*. */
  PW_FN_STAGE_FWD = 17,  /* in: X [N, d]; out: Y [N, d].  params: pw_stage_params */
  PW_FN_STAGE_BWD = 18,  /* in: dY [N, d]; out: dX [N, d]; adds into the stage's weight gradients.  A bf16 stage with
                            several micro-batches may hold the weight-gradient GEMMs back and run them once over all
                            micro-batches whose backward pass has run; pw_model_export, pw_model_import,
                            pw_model_apply_optimizer, pw_model_zero_grads and any call that would overwrite an operand
                            account for what is held back, so the gradients read through this API are always the
                            full sums.  Under HIP-graph capture nothing is held back. */
  PW_FN_ENCDEC_TRAIN_STEP = 19 /* in: source tokens i32 [B, Ts], target tokens i32 [B, Tt+1]; out: loss f32 [1].
                            params: pw_encdec*. */
} pw_fn_kind;

typedef struct {
  int32_t kind;                     /* pw_fn_kind */
  int32_t n_in, n_out;              /* at most 8 each */
  pw_tensor_spec in[8], out[8];
  const void* params;               /* host pointer, copied by pw_compile_fn */
  size_t params_bytes;
} pw_fn_desc;

typedef struct {
  pw_model* model;
  int32_t microbatch;               /* which activation slot the call stashes into / reads from */
} pw_stage_params;

typedef enum {
  PW_STREAM = 0,      /* enqueue every function of the chain at once on the executor stream */
  PW_GRAPH = 1,       /* the same launches, captured once into a HIP graph and replayed (chains of fewer than 8
                         single-kernel functions are enqueued as stream launches: a graph launch costs more) */
  PW_SEQUENTIAL = 2   /* wait for each function to complete before enqueuing the next: the
                         sequential-dispatch baseline of Section 5.1, for comparison only.  Its inputs must not
                         depend on an unresolved pending future: PW_ERR_NOT_READY, nothing enqueued */
} pw_chain_mode;

typedef enum {
  PW_DISPATCH_PARALLEL = 0,   /* every node is handed to its executor at once (parallel asynchronous dispatch,
                                 Section 4.5, Figure 4b) */
  PW_DISPATCH_SEQUENTIAL = 1  /* node i+1 is handed out only after node i's executor has reported it enqueued
                                 (Figure 4a; the comparison of Section 5.1, Figure 7) */
} pw_dispatch_mode;

typedef enum {
  PW_SCHED_FIFO = 0,          /* programs reach the executor in arrival order (the paper's current policy) */
  PW_SCHED_PROPORTIONAL = 1   /* among clients with work queued, the one with the least weighted device time goes
                                 next (the proportional-share multi-tenancy of Section 5.2) */
} pw_sched_policy;

/* A traced dataflow program (Section 3: the program tracer, Figure 2): a DAG of compiled functions.  Values are
 * numbered: the program's inputs are values 0 .. n_inputs-1, then every node's outputs in node order. */
typedef struct pw_program pw_program;   /* owned by its context; destroyed with it at the latest */
typedef struct {
  pw_fn fn;
  int32_t n_in;      /* must equal the function's input count */
  int32_t in[8];     /* value ids consumed; each must be defined before this node (nodes come in tracing order) */
} pw_node;

typedef struct pw_sched pw_sched;   /* owned by its context; destroyed with it at the latest */
typedef struct {
  int32_t client;
  int32_t computations;     /* computations the program contained */
  float start_ms, end_ms;   /* on the device, relative to the scheduler's creation */
} pw_sched_slice;

/* ---- context -------------------------------------------------------------------------------- */

/* Create a context on `device`.  `hip_stream` (a hipStream_t created by the caller, e.g. PyTorch's
 * current stream) becomes the executor stream when non-null; otherwise the context creates its own
 * non-blocking stream.  Fails with PW_ERR_DEVICE when no gfx950 GPU is usable. */
pw_status pw_ctx_create(int device, void* hip_stream, pw_ctx** out);
/* Cancels unresolved pending futures, drains the stream, frees everything the context owns
 * (models, functions, futures, pools). */
pw_status pw_ctx_destroy(pw_ctx* ctx);
/* Message of the last failing call on this context (valid until the next call); "" if none. */
const char* pw_last_error(pw_ctx* ctx);
/* The executor stream (a hipStream_t) so that callers can order their own work against it. */
void* pw_ctx_stream(pw_ctx* ctx);
/* Blocks until everything enqueued so far has run. */
pw_status pw_ctx_synchronize(pw_ctx* ctx);
/* Upper bound, in milliseconds, that a device-side wait on an unresolved future may spin before
 * it gives up and poisons the future (default 20000). */
pw_status pw_ctx_set_gate_timeout_ms(pw_ctx* ctx, int ms);

/* ---- compiled functions (Section 3, Appendix B) ---------------------------------------------- */

/* "Compile": validate the signature, copy params, choose kernels and launch shapes.  PW_ERR_SHAPE /
 * PW_ERR_DTYPE when the signature is impossible for the kind. */
pw_status pw_compile_fn(pw_ctx* ctx, const pw_fn_desc* desc, pw_fn* out);
pw_status pw_fn_release(pw_ctx* ctx, pw_fn fn);

/* Enqueue one function with futures as inputs (Section 4.4 (i)).  Returns as soon as the launches
 * are enqueued - before the inputs are ready - with new futures for the outputs (refcount 1, owned
 * by the caller).  Inputs are checked against the compiled signature first: on PW_ERR_SHAPE /
 * PW_ERR_DTYPE / PW_ERR_INVALID nothing is enqueued.  Inputs stay valid and may feed any number of
 * later calls (fan-out, Figure 2); outputs are always fresh buffers, never updated in place.
 * A poisoned input yields poisoned outputs. */
pw_status pw_run_fn(pw_ctx* ctx, pw_fn fn, const pw_future* in, int n_in, pw_future* out, int n_out);

/* Enqueue a chain: fns[0] consumes `in`, fns[i] consumes the outputs of fns[i-1] (so their
 * signatures must match), `out` receives the outputs of the last function (Section 4.5; the
 * "Chained" mode of Section 5.1).  Intermediate buffers never surface as futures.  All signature
 * checks for the whole chain happen before the first launch. */
pw_status pw_chain(pw_ctx* ctx, const pw_fn* fns, int n_fns, const pw_future* in, int n_in,
                   pw_future* out, int n_out, int mode /* pw_chain_mode */);

/* Executors (Section 4.4: one FIFO per set of devices).  Sets up n of them: executor 0 is the context's own
 * stream; each further one is a HIP stream of its own served by a host thread of its own - on one GPU the
 * stand-in for "a different set of cores attached to a different host".  n in [1, 64]; once per context. */
pw_status pw_ctx_set_executors(pw_ctx* ctx, int n);
/* Measurement aid: every node handed to an executor first costs its host thread `us` microseconds of busy work
 * (0 by default, at most 100000) - a stand-in for the buffer allocation, scheduling and coordination that a
 * node's host performs in a multi-host deployment and that does not depend on the node's predecessor.  With
 * parallel dispatch these overlap across executors; with sequential dispatch they add up (Section 4.5). */
pw_status pw_ctx_set_executor_prep_us(pw_ctx* ctx, int us);
/* A chain whose node i runs on executor executor_of[i] (host array of n_fns ids): fns[0] consumes `in`, node i+1
 * consumes node i's output.  Only elementwise kinds (one fp32 input, one output of the same shape).  Where
 * consecutive nodes sit on different executors the consumer's input buffer is allocated up front and the
 * producer's stream copies its output into it (Section 4.5: shapes are static, so every buffer is planned
 * before anything runs); the dependency is a HIP event.  Everything is validated first: on any error nothing
 * is enqueued.  Returns when every node has been enqueued (not run); `out` receives the last node's output
 * (refcount 1).  dispatch: a pw_dispatch_mode. */
pw_status pw_pipeline(pw_ctx* ctx, const pw_fn* fns, const int32_t* executor_of, int n_fns, pw_future in,
                      pw_future* out, int dispatch);

/* ---- dataflow programs (Section 3, Figure 2; "a single message describing the entire subgraph", Section 4.5) */
/* Trace -> program: checks every edge against the compiled signatures (PW_ERR_SHAPE / PW_ERR_DTYPE name the node in
 * pw_last_error), computes each value's last use so that intermediates are recycled as soon as their last consumer
 * has been enqueued, and snapshots the functions (they may be released afterwards).  outputs: value ids returned. */
pw_status pw_program_create(pw_ctx* ctx, const pw_tensor_spec* input_specs, int n_inputs, const pw_node* nodes,
                            int n_nodes, const int32_t* outputs, int n_outputs, pw_program** out);
/* One client call runs the whole DAG: inputs are checked against the traced specs first (nothing is enqueued on a
 * mismatch), then every node is enqueued in tracing order before any input needs to exist.  mode: PW_STREAM, or
 * PW_GRAPH (captured once per buffer pattern, then replayed).  A value may feed any number of nodes (fan-out) and
 * may be returned as well; outputs are fresh futures (refcount 1); a poisoned input poisons all outputs. */
pw_status pw_program_run(pw_ctx* ctx, pw_program* program, const pw_future* in, int n_in, pw_future* out, int n_out, int mode);
pw_status pw_program_destroy(pw_program* program);

/* ---- several clients, one executor: the centralized scheduler (Section 4.4 "gang-scheduled dynamic dispatch",
 * measured in Section 5.2).  pw_sched_submit / _wait / _client_stats / _drain / _trace may be called from any
 * thread at any time; so may the function / future / chain / await calls of the context while a scheduler exists
 * (they are serialised inside, like the model-state calls).  pw_op_* calls stay single-threaded. */
/* max_in_flight: programs the scheduler keeps enqueued on the device at once (1..1024); the rest wait in the
 * clients' queues, where the policy still has a say. */
pw_status pw_sched_create(pw_ctx* ctx, int policy, int max_in_flight, pw_sched** out);
/* Stops the scheduler thread after the queued programs have been enqueued and have run; results that were never
 * collected are released. */
pw_status pw_sched_destroy(pw_sched* sched);
/* weight > 0: share of device time under PW_SCHED_PROPORTIONAL (ignored by FIFO).  *client: id for the calls below. */
pw_status pw_sched_add_client(pw_sched* sched, double weight, int* client);
/* The client has failed: its queued programs are dropped (their tickets report PW_ERR_POISONED), every object it
 * owns - results it has not collected included - is garbage-collected, further submissions are refused. */
pw_status pw_sched_client_fail(pw_sched* sched, int client, int64_t* objects_released);
/* How many programs had to wait for memory (see pw_ctx_set_memory_limit) and for how long altogether. */
pw_status pw_sched_stalls(pw_sched* sched, int64_t* programs_stalled, double* stalled_ms);
/* Queue a program: the chain fns[0..n_fns) applied to `in` (one input, one output; validated when it is enqueued).
 * Returns at once with a ticket.  `in` must stay alive until the ticket has been waited for. */
pw_status pw_sched_submit(pw_sched* sched, int client, const pw_fn* fns, int n_fns, pw_future in, uint64_t* ticket);
/* Blocks until the program has run; copies `bytes` of its output to host_dst (may be null / 0); the output
 * future is released.  A ticket can be waited for once.  Returns the program's status. */
pw_status pw_sched_wait(pw_sched* sched, uint64_t ticket, void* host_dst, size_t bytes);
/* Blocks until every queued program has been enqueued, has run and has been accounted for. */
pw_status pw_sched_drain(pw_sched* sched);
/* Programs and computations enqueued for the client so far, and the device time (HIP events around each program)
 * of those that have been retired. */
pw_status pw_sched_client_stats(pw_sched* sched, int client, int64_t* programs, int64_t* computations, double* device_ms);
/* Device-time slices of retired programs in execution order (at most the first 65536): copies min(capacity, n)
 * of them, *n = how many there are. */
pw_status pw_sched_trace(pw_sched* sched, pw_sched_slice* out, int capacity, int* n);

/* One LM train step: pw_run_fn on a function of kind PW_FN_LM_TRAIN_STEP.  The model's parameters
 * and optimiser state are updated in place on the device (they are the function's private state). */
pw_status pw_train_step(pw_ctx* ctx, pw_fn step_fn, pw_future tokens, pw_future* loss_out);

/* ---- futures (Sections 4.4, 4.6) -------------------------------------------------------------- */

/* Blocks until the future is ready; then copies `bytes` (<= its size) to host_dst if non-null.
 * PW_ERR_POISONED if it or a dependency failed.  With nothing to copy out (host_dst NULL or bytes 0) the call only
 * establishes readiness; for the output of a one-workgroup elementwise function enqueued as a stream launch
 * (pw_run_fn, pw_chain outside a HIP graph) that is learnt from a completion word the kernel itself writes to pinned
 * host memory, a few microseconds before the stream's event reaches the host (pw_future_query consults it too). */
pw_status pw_await(pw_ctx* ctx, pw_future f, void* host_dst, size_t bytes);
/* New future whose library-owned device buffer is filled from host memory (asynchronous copy). */
pw_status pw_future_from_host(pw_ctx* ctx, const void* host_src, const pw_tensor_spec* spec, pw_future* out);
/* New future over caller-owned device memory (not freed by the library); ready with respect to
 * work already enqueued on the executor stream. */
pw_status pw_future_wrap_device(pw_ctx* ctx, void* dev_ptr, const pw_tensor_spec* spec, pw_future* out);
/* New future that is NOT ready: consumers enqueued on it wait on the device until
 * pw_future_resolve supplies the data.  This is how "enqueued before its inputs are ready" is made
 * real on one GPU. */
pw_status pw_future_pending(pw_ctx* ctx, const pw_tensor_spec* spec, pw_future* out);
/* Supplies the bytes of a pending future from host memory and releases its waiters.  With
 * host_src == NULL the future is poisoned instead (its producer "failed"). */
pw_status pw_future_resolve(pw_ctx* ctx, pw_future f, const void* host_src);
/* PW_OK (ready) | PW_ERR_NOT_READY | PW_ERR_POISONED; never blocks. */
pw_status pw_future_query(pw_ctx* ctx, pw_future f);
pw_status pw_future_spec(pw_ctx* ctx, pw_future f, pw_tensor_spec* out);
/* Device address of the buffer (valid while the caller holds a reference). */
pw_status pw_future_device_ptr(pw_ctx* ctx, pw_future f, void** out);
pw_status pw_future_retain(pw_ctx* ctx, pw_future f);
/* Drops one reference; at zero the buffer returns to the pool (stream-ordered, so work already
 * enqueued on it stays correct). */
pw_status pw_future_release(pw_ctx* ctx, pw_future f);
/* ---- object store: ownership labels and back-pressure (Section 4.6) ----
 * Every future carries the label that was current when it was created (0 until set).  pw_owner_collect drops
 * every live future with that label whatever its reference count - the garbage collection after a client or a
 * program has failed; their buffers return to the pool, unresolved pending futures are cancelled, the handles
 * become invalid.  *released: how many there were (may be null). */
pw_status pw_ctx_set_owner(pw_ctx* ctx, uint64_t owner);
pw_status pw_owner_collect(pw_ctx* ctx, uint64_t owner, int64_t* released);
/* Budget, in bytes, for what the buffer pool may have handed out at one time (0: none).  A call that would exceed
 * it enqueues nothing and returns PW_ERR_OOM; the scheduler (pw_sched) stalls such a program instead until
 * memory has come back. */
pw_status pw_ctx_set_memory_limit(pw_ctx* ctx, int64_t bytes);
/* Number of live futures / bytes currently handed out by the buffer pool (for leak tests). */
pw_status pw_ctx_stats(pw_ctx* ctx, int64_t* live_futures, int64_t* pool_bytes_in_use);

/* ---- the LM (Section 5.3) --------------------------------------------------------------------- */

typedef struct {
  int32_t n_layer, d_model, n_head, d_ff, vocab, seq, batch;
  int32_t bf16;          /* 0: fp32 throughout; 1: bf16 GEMM/attention operands, fp32 accumulation,
                            fp32 residual stream, statistics, master weights and optimiser state */
  int32_t optimizer;     /* 1 SGD, 2 Adam */
  float lr, beta1, beta2, eps;
  int32_t has_embed;     /* 0 for a pipeline stage fed with activations */
  int32_t has_head;      /* 0 for a pipeline stage returning activations */
  int32_t n_microbatch;  /* activation slots kept for a GPipe-like fwd-all / bwd-all schedule */
  int32_t fused_update;  /* 1 (full LM, bf16, Adam): every weight whose gradient is one full-tile GEMM is updated by
                            Adam inside that GEMM's epilogue - 26 instead of 30 bytes of optimizer traffic per
                            parameter.  Those gradients are never stored: pw_model_export of PW_GRADS returns
                            PW_ERR_UNSUPPORTED for them (their Adam moments are there).  0: one optimizer launch */
  int32_t fused_head_loss; /* 1 (full LM, bf16, head on full tiles): the LM-head GEMM is fused with the softmax
                            cross-entropy - logits are never stored; a first pass over the product keeps softmax
                            statistics only, a second writes the gradient of the logits in bf16 once.  0: logits are
                            stored and the loss kernel turns them into their gradient in place */
} pw_lm_config;

/* Allocates parameters (zero), gradients, optimiser state and every activation buffer of the step
 * up front (static buffer plan).  d_model % n_head == 0, head_dim in {64, 128}; with bf16 = 1 the number of
 * tokens batch * seq must be a multiple of 8; PW_ERR_UNSUPPORTED otherwise. */
pw_status pw_model_create(pw_ctx* ctx, const pw_lm_config* cfg, pw_model** out);
pw_status pw_model_destroy(pw_model* m);
/* Parameter tensors in the model's own order; weights are [in, out] row-major fp32. */
int64_t pw_model_param_count(pw_model* m);
pw_status pw_model_param_info(pw_model* m, int64_t idx, char* name, int name_cap, int64_t* numel);
typedef enum { PW_PARAMS = 0, PW_GRADS = 1, PW_ADAM_M = 2, PW_ADAM_V = 3 } pw_model_part;
/* Copy one tensor in (fp32; src may be host or device memory).  For PW_PARAMS in bf16 mode the
 * bf16 compute copy is refreshed too.  Synchronous with respect to the executor stream. */
pw_status pw_model_import(pw_model* m, int part, int64_t idx, const float* src, int src_on_device);
/* Copy one tensor out to host memory (fp32), after draining the executor stream. */
pw_status pw_model_export(pw_model* m, int part, int64_t idx, float* host_dst);
/* Zero the weight gradients (a pipeline stage does this before its first micro-batch). */
pw_status pw_model_zero_grads(pw_model* m);
/* Apply the optimiser to the current gradients (used by the pipeline stage after the last backward;
 * pw_train_step does it as part of the step). */
pw_status pw_model_apply_optimizer(pw_model* m);
/* Read back an activation of the most recent step for inspection: "logits" [N, V] as fp32. */
pw_status pw_model_export_activation(pw_model* m, const char* name, int microbatch, float* host_dst, int64_t numel);
/* Model FLOPs of one step (2 m n k per GEMM, forward + backward; causal attention at half the dense
 * T^2), the figure the throughput is priced against. */
double pw_model_step_flops(const pw_lm_config* cfg);

/* ---- the encoder-decoder model (the text-to-text Transformers of Table 1) -----------------------
 * The paper gives neither the layer recipe nor the sizes of these models; this one keeps what defines the
 * family and builds it from the LM's pieces: encoder layers x += SelfAttn_unmasked(LN x), x += FFN(LN x);
 * decoder layers y += SelfAttn_causal(LN y), y += Attn(LN y over mem), y += FFN(LN y); mem = LN(encoder
 * output); logits = LN(decoder output) Wh; mean next-token cross-entropy over the B*Tt target positions.
 * Encoder and decoder have their own token and position tables. */
typedef struct {
  int32_t n_enc_layer, n_dec_layer, d_model, n_head, d_ff, vocab, src_len, tgt_len, batch;
  int32_t bf16;          /* as in pw_lm_config */
  int32_t optimizer;     /* 1 SGD, 2 Adam */
  float lr, beta1, beta2, eps;
  int32_t fused_update;  /* as in pw_lm_config: with bf16 and Adam, and every weight-gradient GEMM of the step on full
                            tiles, all GEMM weights are updated inside those GEMMs; ignored (0) otherwise */
} pw_encdec_config;

/* Allocates parameters (zero), gradients, optimiser state and every activation buffer of the step up front.
 * d_model % n_head == 0, head_dim in {64, 128}, and with bf16 = 1 batch * src_len and batch * tgt_len multiples
 * of 8; PW_ERR_UNSUPPORTED otherwise, PW_ERR_OOM if HBM runs out. */
pw_status pw_encdec_create(pw_ctx* ctx, const pw_encdec_config* cfg, pw_encdec** out);
pw_status pw_encdec_destroy(pw_encdec* m);
/* Parameter tensors in the model's own order ("enc.wte", "e0.wqkv", ..., "d0.wkv", ..., "wh"); weights are
 * [in, out] row-major fp32; wqkv columns are [Q|K|V], wkv columns [K|V]. */
int64_t pw_encdec_param_count(pw_encdec* m);
pw_status pw_encdec_param_info(pw_encdec* m, int64_t idx, char* name, int name_cap, int64_t* numel);
/* As pw_model_import / pw_model_export (part: pw_model_part). */
pw_status pw_encdec_import(pw_encdec* m, int part, int64_t idx, const float* src, int src_on_device);
pw_status pw_encdec_export(pw_encdec* m, int part, int64_t idx, float* host_dst);
/* "dlogits" [B*Tt, V] of the most recent step, as fp32. */
pw_status pw_encdec_export_activation(pw_encdec* m, const char* name, float* host_dst, int64_t numel);
/* Model FLOPs of one step (2 m n k per GEMM, forward + backward; attention at the visible part of Tq x Tk). */
double pw_encdec_step_flops(const pw_encdec_config* cfg);
/* One train step: pw_run_fn on a function of kind PW_FN_ENCDEC_TRAIN_STEP with the two token arrays. */

/* ---- single kernels, for parity tests and profiling --------------------------------------------
 * All pointers are device pointers; work is enqueued on the executor stream and not waited for.
 * `dtype` is the element type of activations: PW_F32 or PW_BF16. */

typedef enum {
  PW_EPI_STORE = 0,          /* C = acc */
  PW_EPI_BIAS = 1,           /* C = acc + bias[n] */
  PW_EPI_BIAS_RESIDUAL = 2,  /* C(f32) = aux(f32)[m,n] + acc + bias[n] */
  PW_EPI_BIAS_GELU = 3,      /* C = u = acc + bias[n];  C2 = gelu(u) */
  PW_EPI_GELU_BWD = 4,       /* C = acc * gelu'(aux[m,n]),  aux in the activation dtype */
  PW_EPI_ADAM = 5,           /* acc is the gradient of a weight: Adam updates args->adam's w, m, v in the epilogue; the
                                gradient goes to C only if C is non-null (fp32).  bf16, both operands k-major, full
                                256 x 256 tiles (at least 150 of them, or any number in a shared group launch) */
  PW_EPI_XENT_STATS = 6,     /* acc is a tile of logits (rows: token positions, columns: vocabulary): only softmax
                                statistics leave the kernel (args->xent); C unused.  bf16, A row-major, B k-major,
                                at least 150 full tiles */
  PW_EPI_XENT_GRAD = 7       /* the same product: C (bf16) = (exp(acc - lse[row]) - [column == target]) * inv_n */
} pw_epilogue;

/* Adam in a weight-gradient epilogue: w, m, v (fp32 device arrays) and w_bf16 (optional bf16 copy of w) are laid out
 * like the product, [M, N] with leading dimension ldc; t >= 1 is the step number of the bias correction. */
typedef struct {
  float* w;
  float* m;
  float* v;
  void* w_bf16;
  float lr, beta1, beta2, eps;
  int32_t t;
} pw_adam_epilogue;
/* Loss epilogues of the LM head (Section 5.3: "a softmax layer at the end"): row r = b*T + t of the product has the
 * target tokens[b*(T+1) + t + 1] (device, int32 [B, T+1]).  PW_EPI_XENT_STATS writes part[r][N/64][2] = (max, sum of
 * exp(z - max)) of every 64-column group of row r and zt[r] = the target's logit; pw_op_xent_from_stats turns them
 * into lse[r] and the loss.  PW_EPI_XENT_GRAD reads lse[r]; inv_n = 1 / (number of rows). */
typedef struct {
  const int32_t* tokens;
  int32_t T;
  float* part;
  float* zt;
  const float* lse;
  float inv_n;
} pw_xent_epilogue;

typedef struct {
  int32_t dtype;             /* operand element type (A and B) */
  int32_t a_kmajor;          /* 0: A stored [M][K] (lda >= K); 1: A stored [K][M] (lda >= M) */
  int32_t b_kmajor;          /* 0: B stored [N][K] (ldb >= K); 1: B stored [K][N] (ldb >= N) */
  int64_t M, N, K, lda, ldb, ldc;
  int32_t epilogue;          /* pw_epilogue */
  int32_t out_dtype;         /* PW_F32 or PW_BF16 (bf16 only with bf16 operands) */
  int32_t accumulate;        /* 1: C += result (fp32 output, PW_EPI_STORE only) */
  const void* A;
  const void* B;
  const float* bias;         /* [N] or null */
  const void* aux;           /* [M, ldc] or null */
  void* C;
  void* C2;                  /* second output of PW_EPI_BIAS_GELU, else null */
  float* b_colsum;           /* optional, fp32 [N]: sum over k of op(B)[k, n] (overwritten, or added into when
                                accumulate = 1) - the bias gradient that goes with a weight gradient dW = x^T . dy.
                                Served only where it is free: bf16, both operands k-major, M, N multiples of 256, K of
                                64, fp32 PW_EPI_STORE output and at least 150 tiles of 256 x 256 (alone or as a pair);
                                PW_ERR_DEVICE otherwise.  Null: not wanted. */
  const pw_adam_epilogue* adam;  /* host pointer, read during the call; PW_EPI_ADAM only, else null */
  const pw_xent_epilogue* xent;  /* host pointer, read during the call; PW_EPI_XENT_* only, else null */
} pw_gemm_args;

/* C[M,N] = op(A)[M,K] . op(B)[K,N] with fp32 accumulation and a fused epilogue.  bf16 operands run on
 * MFMA; they need K, lda, ldb multiples of 8 and 16-byte aligned pointers. */
pw_status pw_op_gemm(pw_ctx* ctx, const pw_gemm_args* args);
/* Two independent GEMMs (their outputs must not overlap each other or any operand).  Same results as two
 * pw_op_gemm calls; when both are full-tile bf16 problems of one operand layout that would each leave
 * compute units idle - the attention weight gradients of one layer, section 5.3's Transformer layers - their
 * tiles run side by side in one launch.  Nothing is enqueued if either argument set is invalid. */
pw_status pw_op_gemm_pair(pw_ctx* ctx, const pw_gemm_args* args0, const pw_gemm_args* args1);
/* The same for n = 1..3 GEMMs given as an array (the three weight gradients of a decoder's attention over the
 * encoder output: query, key/value and output projections). */
pw_status pw_op_gemm_group(pw_ctx* ctx, const pw_gemm_args* args, int n);
/* x[b*T+t,:] = wte[tok[b*(T+1)+t],:] + wpe[t,:]  (fp32 in, fp32 out; exact). */
pw_status pw_op_embedding_fwd(pw_ctx* ctx, const int32_t* tokens, const float* wte, const float* wpe,
                              float* x, int B, int T, int d, int V);
/* dwte[id,:] = sum over positions holding id of dx (fixed ascending-position order: deterministic);
 * rows of unused ids are zeroed;  dwpe[t,:] = sum_b dx[b*T+t,:]. */
pw_status pw_op_embedding_bwd(pw_ctx* ctx, const int32_t* tokens, const float* dx, float* dwte, float* dwpe,
                              int B, int T, int d, int V);
/* y = (x - mean) rstd * g + b per row; x fp32 [N,d]; y in `dtype`; mean, rstd fp32 [N]. */
pw_status pw_op_layernorm_fwd(pw_ctx* ctx, int dtype, const float* x, const float* g, const float* b,
                              void* y, float* mean, float* rstd, int N, int d);
/* dx(f32) = (dres ? dres : 0) + LayerNorm-backward(dy); dx_lp (optional) receives dx in `dtype`;
 * dg, db fp32 [d] (overwritten, or added into when accumulate = 1); dxsum (optional, fp32 [d], same
 * accumulate rule) receives the column sums of dx: dx is the output gradient of the linear layer that feeds
 * the residual stream here, so this is that layer's bias gradient.  ws: fp32 workspace of
 * pw_layernorm_bwd_ws_floats(N, d) floats. */
pw_status pw_op_layernorm_bwd(pw_ctx* ctx, int dtype, const void* dy, const float* x, const float* g,
                              const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                              float* dg, float* db, float* dxsum, float* ws, int N, int d, int accumulate);
int64_t pw_layernorm_bwd_ws_floats(int N, int d);
/* pw_op_layernorm_bwd for callers that cannot allocate device memory - code under HIP-graph capture, tight serving
 * loops, harnesses that forbid hipMalloc: same arguments without `ws`, same kernels, same bits.  The block sums go
 * to a fixed 12 MiB array inside the library's code object (every GPU the library runs on holds its copy until the
 * process ends; its address is looked up once per device by pw_ctx_create), and the call itself allocates nothing,
 * frees nothing and calls no routine that does.  Limit: pw_layernorm_bwd_ws_floats(N, d) <= 3 * 512 * 2048
 * (any N for d <= 2048; wider rows only with N < 512 * 2048 / d); beyond it PW_ERR_UNSUPPORTED, nothing enqueued.
 * All calls on one GPU share the array and nothing in it has to survive or be cleared between calls, but two calls
 * in flight at once on one GPU (different streams or contexts) race on it: keep them in one stream's order. */
pw_status pw_op_layernorm_bwd_noalloc(pw_ctx* ctx, int dtype, const void* dy, const float* x, const float* g,
                                      const float* mean, const float* rstd, const float* dres, float* dx, void* dx_lp,
                                      float* dg, float* db, float* dxsum, int N, int d, int accumulate);
/* Causal multi-head attention over qkv [B*T, 3d] in `dtype` (columns [Q|K|V], head h at h*hd):
 * o [B*T, d] in `dtype`, lse fp32 [B, H, T] (log-sum-exp of the scaled scores of each row). */
pw_status pw_op_attention_fwd(pw_ctx* ctx, int dtype, const void* qkv, void* o, float* lse, int B, int T, int H, int hd);
/* dqkv [B*T, 3d] from qkv, o, dout and lse.  delta: fp32 workspace [B, H, T]. */
pw_status pw_op_attention_bwd(pw_ctx* ctx, int dtype, const void* qkv, const void* o, const void* dout,
                              const float* lse, float* delta, void* dqkv, int B, int T, int H, int hd);
/* Multi-head attention of Tq queries over Tk keys per (batch, head), scale 1/sqrt(hd): the encoder's unmasked
 * self-attention and the decoder's attention over the encoder output of an encoder-decoder model (the
 * text-to-text Transformers of the paper's Table 1), and - with causal = 1 and the packed layout - the call
 * above.  q, k, v: device pointers to element (batch 0, row 0, feature 0) of arrays in `dtype`; rows are ldq
 * (q) and ldkv (k and v) elements apart, batch b starts at row b*Tq (q) or b*Tk (k, v), head h owns features
 * h*hd .. (h+1)*hd of a row; hd in {64, 128}.  causal = 1: query i sees keys j <= i and Tq must equal Tk.
 * Nothing is owned or kept; PW_ERR_INVALID on a rejected shape or null pointer. */
typedef struct {
  int32_t dtype;
  const void* q;
  const void* k;
  const void* v;
  int64_t ldq, ldkv;
  int32_t B, Tq, Tk, H, hd;
  int32_t causal;
} pw_mha_args;
/* o: dense [B*Tq, H*hd] in `dtype`; lse: fp32 [B, H, Tq].  o_lo: null, or an array like o that receives what
 * the rounding of O to `dtype` left over (O ~ o + o_lo).  Passed on to pw_op_mha_bwd it removes the one rounding
 * the gradients of queries and keys are sensitive to: delta = rowsum(dO * O) is a common offset on a whole row of
 * the score gradient, and keys with a large common component amplify an error in it to several per cent. */
pw_status pw_op_mha_fwd(pw_ctx* ctx, const pw_mha_args* args, void* o, void* o_lo, float* lse);
/* Gradients from o, dout [B*Tq, H*hd] and lse: dq rows lddq elements apart, dk and dv rows lddkv (the H*hd
 * features of every row are overwritten; packed outputs are pointers into one array).  o_lo: what the forward
 * call wrote there, or null.  delta: fp32 workspace [B, H, Tq]. */
pw_status pw_op_mha_bwd(pw_ctx* ctx, const pw_mha_args* args, const void* o, const void* o_lo, const void* dout,
                        const float* lse, float* delta, void* dq, int64_t lddq, void* dk, void* dv, int64_t lddkv);
/* Mean softmax cross-entropy over N rows of logits z [N, V] in `dtype` against tokens[b*(T+1)+t+1];
 * z is overwritten by dz = (softmax(z) - onehot)/N; loss: one fp32; row_loss: fp32 workspace [N]. */
pw_status pw_op_softmax_xent(pw_ctx* ctx, int dtype, void* z, const int32_t* tokens, float* loss, float* row_loss,
                             int B, int T, int V);
/* From what a PW_EPI_XENT_STATS GEMM left: lse[r] = log sum exp of row r over its `groups` 64-column groups,
 * row_loss[r] = lse[r] - zt[r] (both fp32 [N], overwritten), loss = their mean. */
pw_status pw_op_xent_from_stats(pw_ctx* ctx, const float* part, const float* zt, float* lse, float* row_loss,
                                float* loss, int N, int groups);
/* out[c] (=|+=) sum_r in[r, c]; `in` is [rows, cols] in `dtype`; ws: fp32 workspace of
 * pw_colsum_ws_floats(rows, cols) floats. */
pw_status pw_op_colsum(pw_ctx* ctx, int dtype, const void* in, float* out, float* ws, int64_t rows, int64_t cols,
                       int accumulate);
int64_t pw_colsum_ws_floats(int64_t rows, int64_t cols);
/* w -= lr g */
pw_status pw_op_sgd(pw_ctx* ctx, float* w, const float* g, int64_t n, float lr);
/* Adam with bias correction at step t (>= 1); w_bf16 (optional) receives round-to-nearest-even(w). */
pw_status pw_op_adam(pw_ctx* ctx, float* w, float* m, float* v, const float* g, void* w_bf16, int64_t n,
                     float lr, float beta1, float beta2, float eps, int t);

/* ---- measurement aid ----------------------------------------------------------------------------
 * Between pw_profile_begin and pw_profile_end every MFMA GEMM launched on the executor stream (by a train
 * step or by pw_op_gemm) is bracketed by a pair of timing HIP events on that stream.  pw_profile_end
 * drains the stream and returns the number of such launches, the sum of their durations in
 * milliseconds and the sum of their algorithmic FLOPs (2 M N K each).  Not for use inside PW_GRAPH. */
pw_status pw_profile_begin(pw_ctx* ctx);
/* Stops bracketing further launches without waiting for anything (each pair of events costs a few microseconds of
 * stream time: a caller that times many steps brackets only the first few); the launches recorded so far are
 * still returned by pw_profile_end. */
pw_status pw_profile_pause(pw_ctx* ctx);
pw_status pw_profile_end(pw_ctx* ctx, int64_t* launches, double* total_ms, double* total_flops);
/* GEMM launches that carried the Adam epilogue (PW_EPI_ADAM) also do the optimizer's memory traffic - 26 bytes per
 * output element - so pw_profile_end leaves them out of its three figures; this call returns theirs, as of the last
 * pw_profile_end. */
pw_status pw_profile_fused_update(pw_ctx* ctx, int64_t* launches, double* total_ms, double* total_flops);
/* The launches of the last pw_profile_end (with and without the Adam epilogue) by problem shape, largest total time
 * first.  One launch shared by several GEMMs (pw_op_gemm_group, the weight-gradient pairs of a train step) is one
 * row entry under its largest member's shape, with members > 1 and total_flops covering all members.  rows (host,
 * caller-owned, may be NULL when cap is 0) receives at most cap rows; *n_rows the number there are. */
typedef struct pw_gemm_shape_row {
  int64_t M, N, K;
  int32_t a_kmajor, b_kmajor, epilogue, members;
  int64_t launches;
  double total_ms, total_flops;
} pw_gemm_shape_row;
pw_status pw_profile_gemm_shapes(pw_ctx* ctx, pw_gemm_shape_row* rows, int32_t cap, int32_t* n_rows);

#ifdef __cplusplus
}
#endif
#endif /* PW_H_ */
