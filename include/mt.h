/*
 * mt.h - C ABI of the multi-tenant inference worker runtime for one AMD MI355X.
 *
 * The library is the internal model-execution runtime of one worker of the
 * shared inference system the paper proposes: tenants upload a DNN, then send
 * inference requests (paper, section 3); a worker hosts the DNNs of many
 * tenants at once and multiplexes their requests (section 3); models come as a
 * description of structure plus parameters and are built only from a closed set
 * of supported layer types, never from user code (section 3.1); a DNN is a
 * fixed sequence of layers applied in turn, and the answer to a request is a
 * vector of class probabilities (section 1.1).
 *
 * One mt_run serves every pending request of every tenant: requests are grouped
 * by tenant on the device, then each layer index is executed as one grouped
 * launch over all tenants (tenant-specific weights, per-tenant batch sizes), and
 * predictions come back in submission order.
 *
 * Conventions
 *   - Every call returns an mt_status; nothing aborts or throws across the ABI.
 *     mt_last_error() gives a text for the last failing call on a context.
 *   - "HOST" pointers are ordinary process memory; "DEVICE" pointers are HIP
 *     device memory on the context's GPU (e.g. a torch tensor's data_ptr()).
 *   - A context is not thread-safe.  One mt_run may be in flight per context, or
 *     cfg.run_slots of them when they are enqueued on different streams: a run
 *     takes the slot (batch descriptors, activation buffers) that its stream used
 *     last, else a slot not used yet, else the one used longest ago, whose run its
 *     stream then waits for on the device.  Result queries (mt_last_counts) refer
 *     to the run enqueued last.
 *   - Element type of weights, inputs and hidden activations is the context's
 *     dtype: MT_F32 (4 bytes) or MT_BF16 (2 bytes, bfloat16 bit patterns).
 *     Biases, logits and probabilities are always fp32.  With MT_BF16 every
 *     hidden activation is rounded to bfloat16 (nearest even) after bias and
 *     activation; accumulation over the fan-in is fp32 throughout.
 */
#ifndef MT_H
#define MT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mt_ctx mt_ctx;

typedef enum {
    MT_OK = 0,
    MT_EINVAL = 1,       /* null pointer, zero size, value out of range            */
    MT_ENOMEM = 2,       /* weight arena or a device allocation exhausted          */
    MT_ENOTFOUND = 3,    /* tenant has no registered model                         */
    MT_EEXIST = 4,       /* tenant already has a model                             */
    MT_EUNSUPPORTED = 5, /* layer kind / activation / geometry outside the closed set */
    MT_EFULL = 6,        /* more than max_requests rows pending                    */
    MT_ESTATE = 7,       /* call not valid in this state (e.g. host-only context)  */
    MT_EDEVICE = 8       /* a HIP call failed; text in mt_last_error               */
} mt_status;

typedef enum { MT_FC = 0, MT_CONV2D = 1, MT_GAP = 2, MT_MAXPOOL = 3, MT_ADD = 4 } mt_kind;
typedef enum { MT_ACT_NONE = 0, MT_ACT_RELU = 1, MT_ACT_GELU = 2 } mt_act;
typedef enum { MT_F32 = 0, MT_BF16 = 1 } mt_dtype;

#define MT_MAX_LAYERS 48
#define MT_SEG_SLOTS 8      /* runs made of several submissions that may be in flight at once */

/* One layer of a model (closed set, paper section 3.1; section 1.1: DNNs are built from a few
 * dozen layer types).
 *   MT_FC:      y[n] = act(b[n] + sum_k W[n][k] x[k]); in_features = K, out_features = N.
 *   MT_CONV2D:  kh x kw cross-correlation (kh = kw = 1, 3 or 7) over an NHWC image of
 *               in_h x in_w x in_features, zero padding pad = (kh - 1) / 2, stride 1 or 2,
 *               out_features output channels (a multiple of 8; in_features too, except in a
 *               model's first layer), bias per channel, then act.  Output size
 *               floor((in + 2 pad - kh) / stride) + 1 each way.
 *   MT_GAP:     mean over in_h x in_w of every one of in_features channels
 *               (out_features must equal in_features, act must be MT_ACT_NONE).
 *   MT_MAXPOOL: maximum over a kh x kw window (kh = kw = 2 or 3), stride 1 or 2, pad 0 or 1
 *               (below kh); positions outside the image never win.  out_features = in_features,
 *               act MT_ACT_NONE.
 *   MT_ADD:     act(a + b) elementwise, a residual connection: a and b are the outputs of two
 *               earlier layers of the same shape in_h x in_w x in_features (out_features =
 *               in_features).
 * A layer reads the output of the layer before it (layer 0: the request), unless src says
 * otherwise: src = j + 1 reads the output of layer j (j below this layer's index), src = 0 the
 * previous layer.  MT_ADD takes its second operand from src2 the same way (src2 must be given).
 * Image layers (convolution, max-pool, add) pass NHWC images on; MT_FC reads a vector, so it
 * follows MT_FC or MT_GAP (or is the first layer).  The activation of a model's last layer,
 * which must be MT_FC, must be MT_ACT_NONE: its outputs are the logits.  At most four layer
 * outputs may be alive at once (a chain needs two; a residual block with a projection three). */
typedef struct {
    uint32_t kind, act;
    uint32_t in_features, out_features;
    uint32_t in_h, in_w, kh, kw, stride, pad;
    uint32_t src, src2;
} mt_layer_spec;

typedef struct {
    uint32_t max_tenants;   /* tenant ids are 0 .. max_tenants-1                         */
    uint32_t max_requests;  /* most rows that may be pending for one mt_run              */
    uint32_t max_width;     /* most elements any request occupies at any layer boundary  */
    uint32_t max_classes;   /* most outputs of any model's last layer                    */
    uint64_t arena_bytes;   /* size of the packed weight arena in device memory          */
    uint32_t dtype;         /* mt_dtype of weights / inputs / hidden activations         */
    int32_t  device;        /* HIP device ordinal; -1 = host-only context: registration,
                               validation and accounting work, mt_run returns MT_ESTATE  */
    uint32_t run_slots;     /* runs that may be in flight at once, each on a stream of its
                               own (batch interleaving, footnote of paper section 1.3): 0
                               or 1 = one; at most 4.  Every slot has its own batch
                               descriptors and activation buffers; the weights are shared */
    uint32_t cache;         /* 1: the arena is a cache of the registered models (paper
                               section 3.3): every model's packed weights stay in pinned
                               host memory, registering or prefetching a model when the
                               arena is full evicts the models used least recently, and
                               evicted models are reloaded on demand (mt_prefetch).
                               0: every registered model stays resident; a full arena
                               is MT_ENOMEM                                              */
} mt_config;

/* Where mt_run writes predictions.  All DEVICE memory owned by the caller, valid
 * until the stream work of that mt_run has completed.  Row i belongs to the i-th
 * submitted row.  logits and probs have row_stride floats per row; columns at and
 * past n_classes[i] are written as 0.  A row whose tenant id was out of range or
 * had no model gets label -1, n_classes 0 and zero rows.  logits, probs and
 * n_classes may each be NULL to skip that output. */
typedef struct {
    int32_t*  labels;      /* [capacity]                                  */
    float*    probs;       /* [capacity * row_stride]                     */
    float*    logits;      /* [capacity * row_stride]                     */
    int32_t*  n_classes;   /* [capacity]                                  */
    uint32_t  capacity;    /* rows the buffers can hold, >= pending rows  */
    uint32_t  row_stride;  /* floats per row, >= max_classes              */
} mt_outputs;

typedef struct {
    uint32_t n_tenants;          /* models registered                                  */
    uint64_t arena_used;         /* bytes of the arena in use (padded layouts)         */
    uint64_t arena_bytes;
    uint32_t last_run_rows;      /* rows consumed by the last mt_run                   */
    uint32_t last_run_launches;  /* kernels the last mt_run enqueued                   */
} mt_stats;

/* Create a worker context (paper section 3: a worker is a long-lived process that hosts the
 * DNNs of many tenants at once; section 3.3: their weights stay in device memory): allocates
 * the weight arena, the tenant table, and per run slot the batch descriptors and two
 * activation buffers of max_requests * max_width elements on cfg->device.  Serving calls
 * (submit, run, prefetch) allocate no device memory; registering a model with skip connections
 * adds the third or fourth activation buffer its layer graph needs.
 * Errors: MT_EINVAL (null / zero sizes), MT_ENOMEM, MT_EDEVICE. */
mt_status mt_create(mt_ctx** out, const mt_config* cfg);

/* Free everything the context owns (synchronises the device first). */
mt_status mt_destroy(mt_ctx* ctx);

/* Upload a tenant's DNN (paper section 3: a tenant hands over its model before it sends requests).
 *   specs[n_layers]: layer chain; out length of layer l must equal in length of l+1.
 *   weights[l]: HOST, context dtype; FC [N][K] row-major, CONV [C_out][C_in][kh][kw];
 *               ignored (may be NULL) for the kinds without parameters.
 *   biases[l]:  HOST fp32 [N] or [C_out]; NULL means zeros.
 * Weights are copied and repacked into the arena before the call returns; the caller
 * keeps ownership of its buffers.  Nothing is allocated when the call fails.
 * Errors: MT_EINVAL, MT_EEXIST, MT_EUNSUPPORTED (kind/act/geometry outside the closed
 * set, dims that do not chain, more than MT_MAX_LAYERS layers, widths beyond
 * max_width / max_classes), MT_ENOMEM (arena full), MT_EDEVICE. */
mt_status mt_register_model(mt_ctx* ctx, uint32_t tenant, const mt_layer_spec* specs, uint32_t n_layers,
                            const void* const* weights, const void* const* biases);

/* mt_register_model for models whose convolutions are followed by batch normalisation, which the
 * library folds into the convolution (the models of paper section 1.1 are built that way; the
 * runtime executes the folded form).  bn[l]: HOST fp32 [4][C_out] = gamma, beta, running mean,
 * running variance of the normalisation behind convolution l, or NULL for none (must be NULL for
 * other kinds); bn itself may be NULL.  With s = gamma / sqrt(var + bn_eps) per output channel the
 * layer becomes W' = round(W * s), b' = float((b - mean) * s + beta), computed in double
 * precision from the given values and rounded once, W' to the context's element type (nearest
 * even) and b' to fp32; the layer's act applies after it.  Errors: as mt_register_model, and
 * MT_EINVAL for a variance + eps that is not positive. */
mt_status mt_register_model_bn(mt_ctx* ctx, uint32_t tenant, const mt_layer_spec* specs, uint32_t n_layers,
                               const void* const* weights, const void* const* biases, const float* const* bn, float bn_eps);

/* Remove a tenant's model and return its arena slice.  Must not be called while an
 * mt_run that may serve the tenant is still executing.  Errors: MT_ENOTFOUND. */
mt_status mt_unregister_model(mt_ctx* ctx, uint32_t tenant);

/* Queue n_rows requests of ONE tenant for the next mt_run (paper section 3: once its
 * model is in place a tenant sends inference requests).  inputs: DEVICE, n_rows rows of the model's
 * input length, contiguous, context dtype; borrowed until the next mt_run's stream
 * work has completed.  *first_index (optional) receives the submission index of the
 * first row.  Errors: MT_EINVAL, MT_ENOTFOUND, MT_EFULL. */
mt_status mt_submit(mt_ctx* ctx, uint32_t tenant, const void* inputs, uint32_t n_rows, uint32_t* first_index);

/* Queue n_rows requests of MIXED tenants in arrival order (paper section 3: a worker receives
 * the incoming requests of all the tenants it hosts and multiplexes them), with the tenant id of
 * every row already in device memory (what a request front-end that lands ids and
 * payloads in GPU memory would hand over).  tenant_ids: DEVICE int32 [n_rows];
 * inputs: DEVICE, row i at inputs + i*row_stride elements, each row holding its
 * tenant's input length; row_stride must be at least the longest input of any
 * registered model (else MT_EINVAL), so that no row read can leave the buffer.  Ids are validated on the device: rows of
 * unknown tenants are answered with label -1 and never touch any model's weights.
 * Both buffers are borrowed like in mt_submit.  Errors: MT_EINVAL, MT_EFULL. */
mt_status mt_submit_batch(mt_ctx* ctx, const int32_t* tenant_ids, const void* inputs, uint32_t n_rows,
                          uint32_t row_stride, uint32_t* first_index);

/* Serve everything pending (paper section 3: the worker multiplexes the requests of many
 * models; section 1.1: a model is evaluated by applying its layers in turn, and the answer to
 * a request is a vector of class probabilities): enqueue, on hip_stream (a hipStream_t, NULL =
 * default stream), tenant segmentation, the gather into tenant-contiguous rows, one grouped
 * launch per layer index and kind, and the softmax/argmax head; write predictions to *out in
 * submission order.  Never waits for the GPU and allocates nothing; clears the pending list
 * (also when it fails after part of the run has been enqueued: those rows are lost and their
 * outputs undefined).  *n_rows (optional) receives the number of rows served.  With nothing
 * pending it returns MT_OK and serves 0 rows.  Errors: MT_EINVAL (out too small), MT_ESTATE,
 * MT_EFULL (the run is made of several submissions and the tables of MT_SEG_SLOTS earlier
 * such runs are all still being read by the GPU: nothing was enqueued, the pending list is
 * kept, call again later), MT_EDEVICE. */
mt_status mt_run(mt_ctx* ctx, void* hip_stream, const mt_outputs* out, uint32_t* n_rows);

/* What a model needs of a context, from its description alone (no context, no device): the
 * bytes its packed weights occupy in the arena (padded layouts, what mt_register_model takes
 * from cfg.arena_bytes and what an upload moves: the fixed footprint of paper section 3.3),
 * the max_width and max_classes a context must have to accept it, and the length of one
 * request's input.  dtype: mt_dtype.  Errors: MT_EINVAL (null), MT_EUNSUPPORTED (a chain that
 * mt_register_model would reject for its kinds, activations or geometry). */
typedef struct {
    uint64_t arena_bytes;
    uint32_t min_width;      /* smallest cfg.max_width that accepts the model   */
    uint32_t n_classes;      /* smallest cfg.max_classes that accepts the model */
    uint32_t in_len;         /* elements of one request's input                 */
    uint32_t reserved;
} mt_model_footprint;
mt_status mt_model_footprint_get(const mt_layer_spec* specs, uint32_t n_layers, uint32_t dtype, mt_model_footprint* out);

/* mt_run for callers that may not allocate device memory around the call and want a run that
 * touches no allocation of the context besides its weights and tables: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  It does what mt_run does,
 * with the same kernels, but the run's scratch (batch descriptors, both activation buffers,
 * logits) lives in one array of MT_STATIC_SCRATCH_BYTES that the library holds in device
 * memory for the life of the process (one per GPU).  A run whose scratch does not fit (the
 * need grows with the pending rows, the context's max_width, max_classes and max_tenants) is
 * refused with MT_EINVAL and nothing is enqueued; the pending list is kept, so mt_run can
 * serve it.  The call allocates nothing, on the device or through any allocating routine.
 * Every call on a GPU shares that GPU's array: the descriptors a run starts from are cleared
 * on the stream first, and runs enqueued through this call on different streams (or from
 * different contexts) that overlap on one GPU race; runs of one context are ordered by the
 * library (a later one waits for the earlier one on the device).  Other errors as mt_run. */
#define MT_STATIC_SCRATCH_BYTES (16u << 20)
mt_status mt_run_static(mt_ctx* ctx, void* hip_stream, const mt_outputs* out, uint32_t* n_rows);

/* The per-tenant batch sizes of the last mt_run (paper section 3.2: the cost of a run varies
 * with the batch size of every model in it, which the device-side segmentation computes):
 * copies the counts to HOST counts[max_tenants] after synchronising the stream the run was
 * enqueued on.  For tests and accounting. */
mt_status mt_last_counts(mt_ctx* ctx, uint32_t* counts);

/* Model cache (cfg.cache; paper section 3.3: a worker alternates between many tenants'
 * models, most requests find their model cached, and the cost of a miss is predictable
 * because a model's footprint is fixed).  mt_prefetch makes the n named models resident:
 * models that are not are copied from their pinned host images to the arena on `stream`
 * without waiting, after the least recently used other models have given way (a model
 * named in this call never gives way to another one of it).  The copies queue up behind
 * every run in flight, and a later mt_run on any stream waits for them on the device;
 * nothing blocks the host.  mt_run itself prefetches the tenants of pending mt_submit
 * calls; tenants that appear only in mt_submit_batch id arrays have to be prefetched by the
 * caller (the router knows them), else their rows are answered like rows of a tenant without
 * a model.  "Used" means registered or named in a prefetch.  Outside cache mode the call only
 * checks its arguments.  Errors: MT_EINVAL, MT_ENOTFOUND (a tenant without a model),
 * MT_ENOMEM (the named models do not fit the arena together; those named first may have
 * been brought in), MT_EDEVICE. */
mt_status mt_prefetch(mt_ctx* ctx, const uint32_t* tenants, uint32_t n, void* hip_stream);

typedef struct {
    uint32_t resident_models;
    uint64_t uploads, upload_bytes;   /* models copied to the arena so far (registration included) */
    uint64_t evictions;               /* models that gave way                                       */
} mt_cache_stats;
mt_status mt_cache_stats_get(const mt_ctx* ctx, mt_cache_stats* out);

/* Per-tenant accounting.  A request's cost follows from the model description alone
 * (paper section 3.2: the flops of every layer are known a priori), so billing by work
 * done (section 1.3) needs only a count of the requests served, which the batcher keeps
 * on the device.  flops_per_request = 2 x multiply-accumulates over all layers with the
 * true dimensions (convolutions count all nine taps at every output pixel);
 * weight_bytes = the parameters (true dimensions, the context's element type) and fp32
 * biases; io_bytes_per_request = the request's input, every hidden activation written
 * once and read once, logits, probabilities and label.
 * requests / runs count what every mt_run enqueued so far has served of this tenant and
 * in how many runs it had at least one request (the call synchronises the device; 0 for a
 * host-only context).  Errors: MT_EINVAL, MT_ENOTFOUND (no model), MT_EDEVICE. */
typedef struct {
    uint64_t requests, runs;
    uint64_t flops_per_request, weight_bytes, io_bytes_per_request;
    uint64_t resident;      /* 1: the model is in the device arena now                    */
    uint64_t arena_bytes;   /* bytes it occupies there (padded layouts): what an upload moves */
} mt_tenant_account;
mt_status mt_tenant_account_get(mt_ctx* ctx, uint32_t tenant, mt_tenant_account* out);

/* Predicted cost of one mt_run that serves counts[t] requests of tenant t (HOST array of
 * max_tenants entries; tenants without a model must have 0), from the registered
 * descriptors alone, before anything is enqueued (section 3.2: inference is a fixed
 * sequence of operations, so its cost is predictable; an admission controller picks
 * what enters the next run from this).  flops and hbm_bytes are the algorithmic work
 * (weights of active tenants read once, activations written once and read once);
 * launches is the number of kernels mt_run will enqueue; device_ms is the predicted
 * time of the run alone on the GPU, from a per-kernel model (fixed cost per launch +
 * bytes through HBM + bytes re-read through L2, or tile rounds for compute-bound
 * launches) whose constants were fitted on one MI355X.  Works on a host-only context.
 * Errors: MT_EINVAL (null, or more rows than max_requests), MT_ENOTFOUND (rows for a
 * tenant without a model). */
typedef struct {
    double flops, hbm_bytes, device_ms;
    uint32_t rows, launches;
    double upload_bytes, upload_ms;   /* models with requests that are not resident now: bytes to
                                         bring in first, and the predicted time of that copy  */
} mt_run_estimate;
mt_status mt_estimate_run(mt_ctx* ctx, const uint32_t* counts, mt_run_estimate* out);

/* Admission (paper section 3.2: because a run's cost is predictable before it runs, the
 * system can decide what to admit so that latency targets hold and no tenant starves the
 * others).  pending[t] = requests of tenant t waiting (HOST, max_tenants entries);
 * budget_ms = the device time the next run may take (uploads of models that are not
 * resident count towards it).  admitted[t] receives a max-min fair share: every tenant gets
 * min(pending[t], level) requests, with the highest level whose predicted run
 * (mt_estimate_run) fits the budget and max_requests; est (optional) receives the prediction
 * for the admitted mix.  A budget that not even one request per waiting tenant fits admits
 * nothing (level 0).  Works on a host-only context.  Errors: MT_EINVAL (null, budget <= 0),
 * MT_ENOTFOUND (requests pending for a tenant without a model). */
mt_status mt_admit(mt_ctx* ctx, const uint32_t* pending, double budget_ms, uint32_t* admitted, mt_run_estimate* est);

mt_status mt_get_stats(const mt_ctx* ctx, mt_stats* out);

/* Text of the last error on this context ("" if none); valid until the next call. */
const char* mt_last_error(const mt_ctx* ctx);

/* Library version string, e.g. "mt 0.1 gfx950". */
const char* mt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MT_H */
