/*
 * slp -- segment-wise training with synthetic intermediate labels on one AMD
 * MI355X (gfx950).  C ABI of the hot path of "Partitioned Neural Network
 * Training via Synthetic Intermediate Labels" (arXiv 2403.11204): the independent
 * training step of one network segment.
 *
 * Conventions
 *   - every function returns SLP_OK (0) or a negative slp_status; nothing throws
 *     across this boundary; slp_last_error() gives a thread-local message;
 *   - "device" pointers are HIP device addresses on the current device, "host"
 *     pointers are ordinary host memory; the library allocates NO device memory:
 *     every device byte it uses is handed in by the caller (slp_segment_bind);
 *   - slp_stream is a hipStream_t passed as void* (NULL = the default stream);
 *     calls that take a stream are asynchronous on it unless stated otherwise;
 *   - matrices are row-major; a weight matrix is [out][in] as in the paper's
 *     parameter count (in+1)*out (Sec. 3);
 *   - a label table is stored [classes][dim]: row j is the synthetic intermediate
 *     label of class j (the paper's SIL is the transpose, one column per class).
 *   - argument validation happens on the host before any device work is queued: a call
 *     that returns an error has launched nothing;
 *   - calls on ONE handle must not overlap in time (they share its workspace); different
 *     handles are independent and may run concurrently on different streams (Sec. 2.1:
 *     partitions are independent jobs).  A training step also uses a second stream that
 *     the handle owns (default priority) for parameter updates; it is forked from and
 *     joined back into `stream` inside the call, so `stream` alone orders everything.
 */
#ifndef SLP_H
#define SLP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct slp_segment slp_segment;
typedef void* slp_stream;

typedef enum {
  SLP_OK = 0,
  SLP_ERR_ARG = -1,    /* null pointer, unknown enum value, non-positive size */
  SLP_ERR_SHAPE = -2,  /* sizes that do not fit each other or the handle's limits */
  SLP_ERR_ALLOC = -3,  /* a caller-provided buffer is too small or misaligned */
  SLP_ERR_DEVICE = -4, /* the HIP runtime reported an error */
  SLP_ERR_STATE = -5   /* call made before the state it needs exists */
} slp_status;

/* label distributions: Eq. 1 of the paper is SLP_UNIFORM01 (kappa * U[0,1)) */
typedef enum { SLP_UNIFORM01 = 0, SLP_UNIFORM_PM1 = 1, SLP_NORMAL = 2, SLP_BINARY_PM1 = 3 } slp_dist;
typedef enum { SLP_F32 = 0, SLP_BF16 = 1 } slp_dtype;
/* Sec. 3: ReLU after every layer except the network's last one.  A non-final
 * segment ends at a cut and keeps its ReLU (SLP_RELU_ALL); the final segment
 * ends in the identity (SLP_RELU_HIDDEN_IDENTITY_LAST). */
typedef enum { SLP_RELU_ALL = 0, SLP_RELU_HIDDEN_IDENTITY_LAST = 1 } slp_act;
/* Sec. 2: a non-final segment regresses on the synthetic label of the sample's
 * class (mean squared error over batch x width); the final segment is trained on
 * the true classes (softmax cross-entropy, mean over the batch). */
typedef enum { SLP_MSE_SIL = 0, SLP_SOFTMAX_XENT = 1 } slp_loss;

typedef struct {
  int dtype;      /* slp_dtype: SLP_F32 = everything float32; SLP_BF16 = bf16 weights copy,
                     activations and dZ with float32 accumulation, float32 master weights,
                     gradients, momentum and biases */
  int max_batch;  /* largest batch a step or forward call may pass */
  float lr;       /* SGD learning rate (Sec. 3 uses 0.01) */
  float momentum; /* SGD momentum (Sec. 3 uses 0.9); 0 = plain SGD */
  int input_grad; /* 1: the segment can also return d loss / d input (slp_segment_input_grad); costs a
                     transposed copy of the first layer's weights and one input-sized buffer */
} slp_opts;

const char* slp_last_error(void);

/* ---- synthetic intermediate labels (Sec. 2, Eq. 1) --------------------------------
 * Writes T[classes][dim] (dense, row-major, dtype dt) to the caller-owned device
 * buffer `table`.  Entry (j,i) is a pure function of (seed, j, i, dist, kappa):
 * Philox4x32-10 with key = seed and counter (i, j, 0, 0), then a fixed float32
 * transform; kappa only scales SLP_UNIFORM01.  Bit-exact against the CPU
 * definition.  A bf16 table is the float32 value rounded to nearest even. */
int slp_make_synthetic_labels(uint64_t seed, int classes, int dim, int dist, float kappa,
                              void* table /*device*/, int dt, slp_stream stream);

/* ---- inputs of an interior segment in the simultaneous variant (Sec. 2, the
 * variant that trains every partition at once, where an interior partition takes
 * synthetic labels as its inputs as well as its targets) ----------------------------
 * out[n][i] = table[y[n]][i] + sigma * N(0,1), noise counter = global sample index
 * first_sample + n (Philox stream 2).  table: float32 [classes][dim] device;
 * y: int32 [batch] device, each in [0,classes) (clamped into range on the device);
 * out: [batch][dim] of dtype dt, device, caller-owned. */
int slp_make_segment_inputs(uint64_t seed, const float* table /*device*/, int classes, const int32_t* y /*device*/,
                            int64_t first_sample, int batch, int dim, float sigma,
                            void* out /*device*/, int dt, slp_stream stream);

/* ---- segment handle (Sec. 2: one partition; Sec. 2.1: its own hyper-parameters) ----
 * widths[0..n_widths-1] = input width then the width of every layer, n_widths >= 2.
 * The handle is host memory owned by the library until slp_segment_destroy.
 * Errors: SLP_ERR_ARG (null pointers, n_widths < 2 or > 65, a width outside [1, 2^20], unknown enum, max_batch
 * outside [1, 2^24], lr < 0, momentum outside [0,1)); SLP_ERR_SHAPE when a matrix cannot be
 * addressed with 32-bit byte offsets: a weight matrix (float32) or an activation matrix (max_batch x width
 * in the handle's dtype, and its transposed copy) of 2 GiB or more, counted with the library's leading
 * dimensions: the row length rounded up to a multiple of 64 elements, plus 192 elements where that row would
 * be a multiple of 4 KB in the handle's dtype. */
int slp_segment_create(const int* widths /*host*/, int n_widths, int act, int loss, const slp_opts* opts /*host*/,
                       slp_segment** out);
void slp_segment_destroy(slp_segment* seg);

/* Bytes of device memory the segment needs: parameters + optimiser state +
 * gradients ("params"), and activations / per-step temporaries ("workspace"). */
size_t slp_segment_param_bytes(const slp_segment* seg);
size_t slp_segment_workspace_bytes(const slp_segment* seg);

/* Hands the two caller-owned device buffers (256-byte aligned, at least the sizes
 * above) to the segment and zero-fills them on `stream`.  They must outlive every
 * later call on the handle; the library never frees them.  Parameters are undefined
 * (zero) until slp_segment_init or slp_segment_set_params on every layer.
 * Errors: SLP_ERR_ARG (null), SLP_ERR_ALLOC (misaligned or too small), SLP_ERR_DEVICE. */
int slp_segment_bind(slp_segment* seg, void* params /*device*/, size_t params_bytes, void* workspace /*device*/,
                     size_t workspace_bytes, slp_stream stream);

/* Initial parameters U(-1/sqrt(fan_in), 1/sqrt(fan_in)) for weights and biases (the
 * default of the framework named in Sec. 2), drawn from Philox stream 1 with
 * counter (in, out, 1, layer), bias at in = fan_in; momentum is reset to zero. */
int slp_segment_init(slp_segment* seg, uint64_t seed, slp_stream stream);

/* Parameter / gradient / momentum exchange, always as dense float32 W[out][in] and
 * b[out] whatever the internal layout; layer in [0, n_widths-2]; on_device selects
 * host or device pointers for W and b; either pointer may be NULL to skip it.  The
 * calls synchronise `stream` before returning when a host pointer is involved.
 * set_params also rebuilds the derived weight copies and leaves momentum alone.
 * Errors: SLP_ERR_ARG (layer out of range), SLP_ERR_STATE (not bound; get_* before any
 * parameters exist), SLP_ERR_DEVICE. */
int slp_segment_set_params(slp_segment* seg, int layer, const float* W, const float* b, int on_device, slp_stream stream);
int slp_segment_get_params(slp_segment* seg, int layer, float* W, float* b, int on_device, slp_stream stream);
int slp_segment_get_grads(slp_segment* seg, int layer, float* dW, float* db, int on_device, slp_stream stream);
int slp_segment_get_momentum(slp_segment* seg, int layer, float* vW, float* vb, int on_device, slp_stream stream);
/* Copies the stored activation A_layer (layer 0 = the ingested input, layer L =
 * the segment's output) of the last step, rows [0,batch), to out[batch][width],
 * dense, in the handle's dtype (device pointer). kind 0 = activation, 1 = dZ (layers 1..L). */
int slp_segment_get_activation(slp_segment* seg, int layer, int kind, int batch, void* out /*device*/, slp_stream stream);

int slp_segment_set_lr(slp_segment* seg, float lr, float momentum);

/* Label table for a SLP_MSE_SIL segment (Sec. 2, first training phase: the left partition is trained against the
 * synthetic intermediate label of each sample's class): float32 [classes][dim] on the device with
 * dim == the segment's last width; caller-owned, must outlive the steps.
 * Errors: SLP_ERR_STATE (the segment's loss is not SLP_MSE_SIL), SLP_ERR_ARG (null table,
 * classes <= 0), SLP_ERR_SHAPE (dim != last width). */
int slp_segment_set_labels(slp_segment* seg, const float* table /*device*/, int classes, int dim);

/* ---- the training step (Sec. 2: first and second training phase; Sec. 3:
 * optimiser and activations) -------------------------------------------------------
 * One pass of forward, loss, backward confined to the segment, and the SGD update
 * for the batch X[batch][widths[0]] (dense, handle dtype, device) with class ids
 * targets[batch] (int32, device).  For SLP_MSE_SIL the ids select rows of the bound
 * label table; for SLP_SOFTMAX_XENT they are the classes (< last width).  Ids are
 * clamped into range on the device and counted (slp_segment_target_errors).  If loss_out is not NULL the mean loss of the
 * batch (before the update) is written there (float32, device).  No host
 * synchronisation; X and targets are only read.  batch may be any value in
 * [1, max_batch]; the means run over the batch actually passed.
 * Errors: SLP_ERR_ARG (null X or targets), SLP_ERR_SHAPE (batch outside [1, max_batch]),
 * SLP_ERR_STATE (not bound, no parameters, SLP_MSE_SIL without a label table),
 * SLP_ERR_DEVICE (a launch failed). */
int slp_segment_step(slp_segment* seg, const void* X /*device*/, const int32_t* targets /*device*/, int batch,
                     float* loss_out /*device, may be NULL*/, slp_stream stream);

/* Class ids are the caller's data: an id outside its range (rows of the label table for SLP_MSE_SIL, the last width
 * for SLP_SOFTMAX_XENT) is clamped into range on the device so that nothing is read out of bounds, and the row is
 * COUNTED: *count_out (host) receives the number of such rows seen by the handle's loss kernels since slp_segment_bind.
 * A non-zero count means steps trained on wrong targets.  Synchronises `stream`.  Errors: SLP_ERR_ARG (null),
 * SLP_ERR_STATE (not bound), SLP_ERR_DEVICE. */
int slp_segment_target_errors(slp_segment* seg, int64_t* count_out /*host*/, slp_stream stream);

/* Forward only (Sec. 2: the stored response of the left partition; joining the
 * partitions): out[batch][last width], dense, handle dtype, device.  Parameters
 * are not changed; the activation workspace is overwritten (X and out themselves are
 * used in place of its first and last entries when their rows are aligned: X with a
 * width that is a multiple of 64 on a 128-byte boundary, out with a width that is a
 * multiple of 8 on a 16-byte boundary).  Errors as for the step. */
int slp_segment_forward(slp_segment* seg, const void* X /*device*/, int batch, void* out /*device*/, slp_stream stream);

/* ---- recovery phase (Sec. 5: the left partition is trained some more while the
 * right partition's weights are frozen) ------------------------------------------------
 * slp_segment_input_grad runs forward, the segment's own loss against `targets` and
 * the data gradients of EVERY layer, and writes d loss / d X to dX[batch][widths[0]]
 * (dense, handle dtype, device).  No parameter, momentum or gradient buffer changes:
 * this is the frozen partition.  Needs opts.input_grad = 1 (else SLP_ERR_STATE).
 * slp_segment_step_external is a training step whose output gradient comes from
 * outside: dA_out[batch][last width] (dense, handle dtype, device) = d loss / d (segment
 * output).  dZ_L = dA_out where the last layer's ReLU is active (or everywhere on an
 * identity-last segment), then the usual backward pass and SGD update.  Chaining
 * left.forward -> right.input_grad -> left.step_external is one recovery step. */
int slp_segment_input_grad(slp_segment* seg, const void* X /*device*/, const int32_t* targets /*device*/, int batch,
                           void* dX /*device*/, float* loss_out /*device, may be NULL*/, slp_stream stream);
int slp_segment_step_external(slp_segment* seg, const void* X /*device*/, const void* dA_out /*device*/, int batch,
                              slp_stream stream);

/* ---- launch-bound segments ----------------------------------------------------------
 * A step of a small segment (the paper's own network is 784-80-60 | 60-60-60-47, Sec. 3) is a
 * few dozen kernels of a few microseconds each: the host's launch rate, not the GPU, bounds
 * it.  With graphs on, slp_segment_step captures its launch sequence into a HIP graph the
 * first time it sees a combination (X, targets, batch, loss_out) -- the only arguments the
 * sequence depends on -- and replays that graph, one launch, on every later call with the
 * same combination (up to 16 are kept, least recently used evicted).  Results are those of
 * the eager launches, bit for bit: the same kernels with the same arguments in the same order.
 * Eager launches are used regardless while launches are being timed (profile hooks on), on the
 * null stream, for the first step of a handle, and when `stream` is already being captured by
 * the caller (the launches then become part of the caller's graph).  slp_segment_set_lr,
 * slp_segment_set_labels and slp_segment_bind drop the captured graphs (after a device
 * synchronisation), because those hold their values.  A caller that keeps passing new
 * combinations would pay a capture per step: after 32 misses in a row the handle returns to
 * eager launches until this function is called again (copy each batch into one fixed buffer
 * and step on that to have a single combination).  Off by default. */
int slp_segment_set_graph(slp_segment* seg, int on);

/* ---- optimiser step inside the weight-gradient product (Sec. 3: SGD with momentum) ----------------------
 * With the fused update on, the matrix product that forms dW_l applies v = mu v + dW; w = w - lr v to the tile of the
 * weight matrix it holds and rewrites the bf16 and transposed copies from there: the gradient is never written to
 * memory and never read back (20 instead of 28 bytes per parameter and step in bf16 mode), and a step of a small
 * segment ends with its last product instead of a tail of update launches (the paper's own network, Sec. 3: 0.20 ->
 * 0.14 ms per step of both partitions).  It pays where a layer's products are short; for very wide layers the separate
 * update, which streams beside the next products, is faster.  on = 0: off (default); 1: every layer; 2: the layers
 * where it measured faster, those with at most 4,194,304 weights; on > 2: the layers with at most `on` weights.
 * Results equal the separate update's to float32 rounding (the same expressions on the same values).  For a layer
 * that is fused, slp_segment_get_grads returns the bias gradient only (a request for dW fails with SLP_ERR_STATE).
 * Drops captured graphs.  Errors: SLP_ERR_ARG (null handle, on < 0). */
int slp_segment_set_fused_update(slp_segment* seg, int on);

/* ---- several segments trained side by side (end of Sec. 2: partitions are independent jobs) ----
 * The last thing a step does is stream every parameter once (the SGD update); it runs on a stream of the handle
 * beside the matrix products that are still to come, and the step normally ends by making `stream` wait for it.
 * With overlap on, slp_segment_step (and slp_segment_step_external) returns without that wait, and the update of
 * the first layer moves to the side stream too: whatever the caller enqueues next on `stream` -- typically the
 * step of another segment -- runs beside the tail of this one.  Until the handle's next step, every call on the
 * handle that takes a stream first makes that stream wait for the pending updates (whichever stream it is), so calls
 * through this interface see the same values as without overlap (bit for bit).  A caller that reads or frees the
 * parameter or workspace buffers directly must call slp_segment_join first (slp_segment_destroy and slp_segment_bind
 * wait on the host).  No effect on steps that are captured into a graph; a stream that is being captured cannot wait
 * for updates left pending outside the capture: such a call fails with SLP_ERR_STATE.  With overlap on, the weight updates of
 * large layers are also paced (each of their workgroups pauses between tiles, by an amount that grows with the batch), which
 * roughly doubles their duration and keeps their memory traffic from stalling the matrix products beside them; the caller is
 * expected to keep the device busy behind the step, as a loop over segments does.  Turning overlap off waits on
 * the host for pending updates, after which the handle is back to plain stream order.  Off by default.
 * slp_segment_join: makes `stream` wait for updates a previous step left running; a no-op when none are pending. */
int slp_segment_set_overlap(slp_segment* seg, int on);
int slp_segment_join(slp_segment* seg, slp_stream stream);

/* ---- the joined network at inference (Sec. 2: the partitions can be joined after training; Sec. 4 reports the
 * joined network's test accuracy) and the epoch figures of the training curves ----------------------------
 * slp_count_correct: number of rows n of logits[batch][classes] (dense, row-major, dtype dt, device) whose arg-max
 * column -- the lowest index among equal maxima -- equals targets[n] (int32, device; an id outside [0, classes) never
 * matches).  Logits must not be NaN.  The count goes to *correct_out (int64, device): written when accumulate is 0,
 * added to when it is not (so a loop over the batches of a dataset ends with the dataset's count).  scratch: device
 * memory of at least 4 * ceil(batch / 4) bytes, 4-byte aligned, caller-owned, overwritten (per-block partial counts;
 * they are summed in a fixed order, no atomics).  Asynchronous on `stream`.
 * Errors: SLP_ERR_ARG (null pointer, batch or classes <= 0, unknown dtype), SLP_ERR_ALLOC (scratch too small or
 * misaligned), SLP_ERR_DEVICE.
 * slp_mean_loss: *mean_out = (1/n) sum of losses[0..n) (float32, device; summed in float64 in a fixed order): the
 * epoch mean of the per-step losses that slp_segment_step wrote.  Errors: SLP_ERR_ARG (null, n <= 0), SLP_ERR_DEVICE. */
int slp_count_correct(const void* logits /*device*/, const int32_t* targets /*device*/, int batch, int classes, int dt,
                      void* scratch /*device*/, size_t scratch_bytes, int accumulate, int64_t* correct_out /*device*/,
                      slp_stream stream);
int slp_mean_loss(const float* losses /*device*/, int n, float* mean_out /*device*/, slp_stream stream);

/* slp_count_correct for callers that cannot allocate or hand over scratch memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same result as slp_count_correct, bit for bit; the per-block
 * partial counts live in a 64 KiB array inside the library's code object (one copy per GPU the library runs on, held
 * until the process ends) instead of caller memory, and the call allocates nothing and frees nothing.
 * Limit: batch <= SLP_COUNT_STATIC_MAX_BATCH (65536 rows), else SLP_ERR_SHAPE.  Every call on a GPU uses that GPU's one
 * array (each call overwrites the entries it reads; nothing has to be cleared): calls that overlap in time on the
 * same GPU -- different streams, or different host threads -- race and must be serialised by the caller; calls that
 * follow each other on one stream are safe.  Other errors as for slp_count_correct. */
#define SLP_COUNT_STATIC_MAX_BATCH 65536
int slp_count_correct_static(const void* logits /*device*/, const int32_t* targets /*device*/, int batch, int classes,
                             int dt, int accumulate, int64_t* correct_out /*device*/, slp_stream stream);

/* ---- measurement hooks -------------------------------------------------------------
 * When enabled, every matrix-product launch of the segment is bracketed by HIP
 * events on its stream.  slp_segment_profile_read synchronises the recorded events,
 * returns the accumulated device time of those launches (milliseconds), their count
 * and their algorithmic FLOPs (2*M*N*K with unpadded sizes), then clears the log.
 * on > 1 additionally creates `on` event pairs up front so that none has to be
 * created between timed launches. */
int slp_segment_profile_enable(slp_segment* seg, int on);
int slp_segment_profile_read(slp_segment* seg, double* gemm_ms, int64_t* gemm_launches, double* gemm_flops);

/* Sustained matrix-pipe rate of the device the caller has made current: a register-only
 * loop of the MFMA instructions the matrix products use (bf16 16x16x32 or float32
 * 32x32x2, 8 wavefronts per compute unit, one workgroup per compute unit, pseudo-random
 * operands), `iters` iterations of 16 MFMA groups per wavefront, timed with HIP events
 * on `stream` after a short warm-up launch.  Synchronous.  It is the rate the chip holds
 * under its power limit with no memory traffic at all: the practical ceiling to read a
 * measured matrix-product rate against, beside the published peak.
 * scratch: device buffer of at least 2048 bytes per compute unit (caller-owned, overwritten).
 * tflops_out (host) receives the rate in TFLOP/s, ms_out (host, may be NULL) the duration.
 * Errors: SLP_ERR_ARG (dtype, iters outside [1, 2^24], null pointers), SLP_ERR_SHAPE
 * (scratch too small), SLP_ERR_DEVICE. */
int slp_probe_mfma_rate(int dtype, int iters, void* scratch /*device*/, size_t scratch_bytes, double* tflops_out /*host*/,
                        double* ms_out /*host, may be NULL*/, slp_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SLP_H */
