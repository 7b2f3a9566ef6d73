// C ABI of the segment-training library (see include/slp.h for the contract).
// Host code only: argument validation, the device-memory carve-up of the two
// caller-provided buffers, and the launch sequence of one training step
// (paper Sec. 2: a segment is trained on its own inputs and targets, nothing
// flows to or from another segment).
#include "../../include/slp.h"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "slp_kernels.h"

using namespace slp;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                             \
  do {                                                                                            \
    hipError_t e__ = (expr);                                                                      \
    if (e__ != hipSuccess) return fail(SLP_ERR_DEVICE, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layer {
  int K, N;        // fan-in, fan-out
  int ldk, ldn;    // padded leading dimensions of [N][ldk] and [K][ldn] matrices
  // offsets into the parameter buffer
  size_t oW32, ovW, odW, ob, ovb, odb, oW16, oWT;
  // bound pointers
  float *W32, *vW, *dW, *b, *vb, *db;
  void *Wop;       // forward operand: W16 (bf16 mode) or W32
  void *W16;       // bf16 copy or null
  void *WT;        // [K][ldn] transposed copy for the data gradient, null for the first layer
};

struct ProfRec { hipEvent_t a, b; double flops; };

// One captured training step: the launch sequence depends on these arguments only
// (every other kernel argument is fixed once the handle is bound).
struct StepGraph {
  const void* X;
  const int32_t* targets;
  int batch;
  float* loss_out;
  hipGraphExec_t exec;
  uint64_t used;
};
constexpr size_t kMaxStepGraphs = 16;

}  // namespace

struct slp_segment {
  int L, act, loss, dtype, max_batch, ldb;   // ldb: leading dimension of batch-contiguous buffers
  float lr, mu;
  std::vector<int> widths, ldw;              // ldw[l] = padded width l
  std::vector<Layer> layers;
  size_t param_bytes, work_bytes;
  // workspace offsets / pointers, index = layer 0..L
  std::vector<size_t> oA, oAT, odZ, odZT, oBits;
  std::vector<void*> A, AT, dZ, dZT;
  std::vector<uint32_t*> bits;   // bf16 mode: [A_l > 0] of the hidden activations, one bit per element (GemmArgs::bits)
  int ldbits;
  size_t oPartials, oLoss, oBadIds;
  int n_partials;
  float *partials, *loss_dev;
  unsigned* bad_ids;                         // rows whose class id was out of range, counted by the loss kernels
  bool bound, have_params;
  bool input_grad;                           // keeps W_1^T and a dZ_0 buffer so that d loss / d input can be formed
  const float* table;
  int classes;
  int last_batch;
  bool prof;
  std::vector<ProfRec> prof_log;
  std::vector<hipEvent_t> ev_pool;
  // The parameter update of layer l is memory-bound and independent of the matrix products of the
  // layers below it, so it runs on a side stream next to them (fork after the weight gradient of
  // layer l, join at the end of the step: the caller's stream still orders everything).
  hipStream_t side;
  std::vector<hipEvent_t> ev_fork;   // one per layer
  hipEvent_t ev_join;
  // slp_segment_set_overlap: every layer's update goes to the side stream and slp_segment_step leaves the join to the
  // handle's next call that takes a stream (settle), so that the optimiser tail of one segment runs beside whatever
  // the caller enqueues next -- typically the step of another segment.
  bool defer_join, join_pending;
  // slp_segment_set_fused_update: the weight-gradient product applies the optimiser step in its epilogue; the weight
  // gradient itself is never stored.
  bool fused_update;
  long fused_max_params;                     // layers with more weights than this keep the separate update
  // Small segments are bound by launch latency, not by the GPU: with graphs on, the launch sequence of a step
  // is captured once per (X, targets, batch, loss_out) and replayed as one graph launch afterwards.
  bool use_graph, graph_warm;
  int graph_misses;                          // consecutive steps that found no captured graph
  std::vector<StepGraph> graphs;
  uint64_t graph_tick;
};

namespace {

int esize(const slp_segment* s) { return s->dtype == SLP_BF16 ? 2 : 4; }

// captured steps hold lr, momentum, the label table and the buffer addresses by value
void drop_graphs(slp_segment* s) {
  if (!s->graphs.empty()) (void)hipDeviceSynchronize();   // a replay may still be running; rare (set-up calls only)
  for (auto& g : s->graphs) (void)hipGraphExecDestroy(g.exec);
  s->graphs.clear();
}
bool relu_on(const slp_segment* s, int l) { return l < s->L || s->act == SLP_RELU_ALL; }

hipEvent_t get_event(slp_segment* s) {
  if (!s->ev_pool.empty()) {
    hipEvent_t e = s->ev_pool.back();
    s->ev_pool.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

int run_gemm(slp_segment* s, int epi, const GemmArgs& g, hipStream_t st) {
  ProfRec rec{nullptr, nullptr, 2.0 * g.M * (double)g.N * g.K};
  if (s->prof) {
    rec.a = get_event(s);
    rec.b = get_event(s);
    if (!rec.a || !rec.b) return fail(SLP_ERR_DEVICE, "hipEventCreate failed");
    HIP_TRY(hipEventRecord(rec.a, st));
  }
  HIP_TRY(launch_gemm(s->dtype, epi, g, st));
  if (s->prof) {
    HIP_TRY(hipEventRecord(rec.b, st));
    s->prof_log.push_back(rec);
  }
  return SLP_OK;
}

int check_seg(const slp_segment* s, bool need_bound, bool need_params) {
  if (!s) return fail(SLP_ERR_ARG, "segment handle is NULL");
  if (need_bound && !s->bound) return fail(SLP_ERR_STATE, "segment has no device buffers: call slp_segment_bind first");
  if (need_params && !s->have_params)
    return fail(SLP_ERR_STATE, "segment has no parameters: call slp_segment_init or slp_segment_set_params first");
  return SLP_OK;
}

// X[batch][w0] -> A[0] (padded rows) and, for training, its transpose
int ingest(slp_segment* s, const void* X, int batch, bool with_transpose, hipStream_t st) {
  HIP_TRY(launch_copy_transpose(s->dtype, X, s->widths[0], batch, s->widths[0], s->A[0], s->ldw[0],
                                with_transpose ? s->AT[0] : nullptr, s->ldb, 1, nullptr, 0, st));
  return SLP_OK;
}

// x_direct / out_direct (forward-only passes): the caller's dense input is the first layer's operand and the caller's
// dense output buffer the last layer's result, when their rows are 16-byte aligned; the workspace copies are skipped.
int forward_layers(slp_segment* s, int batch, bool training, hipStream_t st, const void* x_direct = nullptr,
                   void* out_direct = nullptr) {
  for (int l = 1; l <= s->L; ++l) {
    const Layer& ly = s->layers[l - 1];
    GemmArgs g{};
    g.A = s->A[l - 1]; g.lda = s->ldw[l - 1];
    if (l == 1 && x_direct) { g.A = x_direct; g.lda = s->widths[0]; }
    g.B = ly.Wop;      g.ldb = ly.ldk;
    g.M = batch; g.N = ly.N; g.K = ly.K;
    g.C = s->A[l]; g.ldc = s->ldw[l];
    if (l == s->L && out_direct) { g.C = out_direct; g.ldc = s->widths[l]; }
    g.CT = (training && l < s->L) ? s->AT[l] : nullptr; g.ldct = s->ldb;
    g.bits_out = (training && l < s->L) ? s->bits[l] : nullptr; g.ldbits = s->ldbits;
    g.bias = ly.b; g.relu = relu_on(s, l) ? 1 : 0;
    int rc = run_gemm(s, EPI_FWD, g, st);
    if (rc) return rc;
  }
  return SLP_OK;
}

// loss and dZ_L (row-major for the data gradient, transposed for the weight gradient)
int loss_and_output_grad(slp_segment* seg, const int32_t* targets, int batch, float* loss_out, hipStream_t st) {
  const int L = seg->L, D = seg->widths[L];
  if (seg->loss == SLP_MSE_SIL) {
    HIP_TRY(launch_mse_loss_grad(seg->dtype, seg->A[L], seg->ldw[L], targets, seg->table, seg->classes, batch, D,
                                 relu_on(seg, L) ? 1 : 0, seg->dZ[L], seg->dZT[L], seg->ldb, seg->partials, seg->bad_ids, st));
    HIP_TRY(launch_reduce_loss(seg->partials, mse_partial_count(batch, D), 1.0 / ((double)batch * D), seg->loss_dev, loss_out, st));
  } else {
    HIP_TRY(launch_xent_loss_grad(seg->dtype, seg->A[L], seg->ldw[L], targets, batch, D, relu_on(seg, L) ? 1 : 0,
                                  seg->dZ[L], seg->partials, seg->bad_ids, st));
    HIP_TRY(launch_copy_transpose(seg->dtype, seg->dZ[L], seg->ldw[L], batch, D, nullptr, 0, seg->dZT[L], seg->ldb, 1,
                                  nullptr, 0, st));
    HIP_TRY(launch_reduce_loss(seg->partials, batch, 1.0 / (double)batch, seg->loss_dev, loss_out, st));
  }
  return SLP_OK;
}

// dZ_{l-1} = (dZ_l W_l) * [A_{l-1} > 0]; for l = 1 the result is the gradient w.r.t. the segment input (no mask)
int data_gradient(slp_segment* seg, int l, int batch, hipStream_t st) {
  Layer& ly = seg->layers[l - 1];
  GemmArgs g{};
  g.A = seg->dZ[l]; g.lda = seg->ldw[l];
  g.B = ly.WT;      g.ldb = ly.ldn;
  g.M = batch; g.N = ly.K; g.K = ly.N;
  g.C = seg->dZ[l - 1]; g.ldc = seg->ldw[l - 1];
  g.CT = l > 1 ? seg->dZT[l - 1] : nullptr; g.ldct = seg->ldb;
  g.maskT = l > 1 ? seg->AT[l - 1] : nullptr; g.ldmask = seg->ldb;
  g.bits = l > 1 ? seg->bits[l - 1] : nullptr; g.ldbits = seg->ldbits;
  return run_gemm(seg, EPI_DGRAD, g, st);
}

// backward + update, last layer first; the data gradient of layer l reads W_l before it is updated
// Makes `st` wait for updates a previous step left running on the side stream (deferred join).  The flag stays set
// until the next step replaces the event (or the host has waited): every stream that touches the handle in between
// gets the wait, not only the first one.
int settle(slp_segment* seg, hipStream_t st) {
  if (!seg->join_pending) return SLP_OK;
  if (st) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(st, &cap));
    if (cap != hipStreamCaptureStatusNone)
      return fail(SLP_ERR_STATE, "updates of an overlapped step are still pending and a stream that is being captured cannot "
                                 "wait for them: call slp_segment_set_overlap(seg, 0) before the capture");
  }
  HIP_TRY(hipStreamWaitEvent(st, seg->ev_join, 0));
  return SLP_OK;
}

// Weight updates of large layers that run on the side stream, beside the next matrix products, are held to one workgroup
// per compute unit (256, 512 and 128 were tried: 256 is best, -2 % per step on the comparison and deep configurations).
constexpr int kSideUpdateWorkgroups = 256;
// slp_segment_set_fused_update(seg, 2): layers up to this many weights take the update inside their weight-gradient product.
// Measured on the wide configuration (784-4096-4096-2048 | 2048-4096-4096-47, batch 1024): fusing the layers up to 1 M
// or 4 M weights is 1-2 % faster than fusing none, fusing the 8 M and 16 M layers as well 2 % and 9 % slower (their
// epilogues wait on weight and momentum loads that the separate, massively parallel update kernel streams).
constexpr long kFusedAutoMaxWeights = 1L << 22;
int backward_and_update(slp_segment* seg, int batch, hipStream_t st) {
  // a join cannot be left to a later call while the launches are being captured into a graph
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (seg->defer_join && st) HIP_TRY(hipStreamIsCapturing(st, &cap));
  const bool defer = seg->defer_join && cap == hipStreamCaptureStatusNone;
  bool forked = false;           // whether anything of this step went to the side stream
  // With the join left to a later call the update's tail has the caller's next work to hide behind, and the update can
  // be paced so that its loads fit beside the products' (see sgd_update_strided_kernel).  How long it may take scales
  // with the batch (the products beside it do): nothing up to 2048 rows, 8 units at 4096, capped at 14 from 5632 on --
  // measured: comparison configuration (8192 rows) best at 10-16 units, deep configuration run serially (4096) at 8-14,
  // wide configuration (1024) 18 % slower with any pause.
  const int pause = defer ? std::min(14, std::max(0, (batch - 2048) / 256)) : 0;
  for (int l = seg->L; l >= 1; --l) {
    Layer& ly = seg->layers[l - 1];
    if (l > 1) {
      int rc = data_gradient(seg, l, batch, st);
      if (rc) return rc;
    }
    GemmArgs g{};
    g.A = seg->dZT[l];    g.lda = seg->ldb;
    g.B = seg->AT[l - 1]; g.ldb = seg->ldb;
    g.M = ly.N; g.N = ly.K; g.K = batch;
    g.Cf = ly.dW; g.ldc = ly.ldk;
    const bool fused = seg->fused_update && (long)ly.N * ly.K <= seg->fused_max_params;
    if (fused) {     // weights, momentum and the derived copies are rewritten by the product's epilogue
      g.uW = ly.W32; g.uV = ly.vW; g.uW16 = ly.W16; g.uWT = ly.WT; g.ldwt = ly.ldn;
      g.lr = seg->lr; g.mu = seg->mu;
    }
    int rc = run_gemm(seg, fused ? EPI_WGRAD_UPDATE : EPI_WGRAD, g, st);
    if (rc) return rc;
    if (fused) {
      // The data gradient of layer l read W_l^T before this product was queued (same stream).  What is left of the
      // layer is its bias: one small launch, on the caller's stream (nothing worth a second stream).
      HIP_TRY(launch_layer_update(seg->dtype, nullptr, nullptr, nullptr, ly.N, 0, ly.ldk, nullptr, nullptr, ly.ldn, seg->dZT[l],
                                  seg->ldb, batch, ly.db, ly.b, ly.vb, seg->lr, seg->mu, 0, 0, 0, st));
      continue;
    }
    // fork: everything layer l still needs (bias gradient, both updates) reads dZ_l^T / dW_l, which are
    // complete here, and writes only layer l's parameters, which nothing below reads in this step
    // without a deferred join the first layer has nothing left in this step to overlap with
    hipStream_t us = (l > 1 || defer) ? seg->side : st;
    if (us != st) {
      HIP_TRY(hipEventRecord(seg->ev_fork[l - 1], st));
      HIP_TRY(hipStreamWaitEvent(us, seg->ev_fork[l - 1], 0));
      forked = true;
    }
    // small layers are bound by launch latency: weights and bias in one launch.  Large ones run the bias part as a launch
    // of its own first: inside one launch its long reads of dZ^T slowed the matrix products beside it (measured 1 %).
    if ((size_t)ly.N * ly.K <= ((size_t)1 << 22)) {
      HIP_TRY(launch_layer_update(seg->dtype, ly.W32, ly.vW, ly.dW, ly.N, ly.K, ly.ldk, ly.W16, ly.WT, ly.ldn, seg->dZT[l],
                                  seg->ldb, batch, ly.db, ly.b, ly.vb, seg->lr, seg->mu, 0, 0, 0, us));
    } else {
      HIP_TRY(launch_layer_update(seg->dtype, nullptr, nullptr, nullptr, ly.N, 0, ly.ldk, nullptr, nullptr, ly.ldn, seg->dZT[l],
                                  seg->ldb, batch, ly.db, ly.b, ly.vb, seg->lr, seg->mu, 0, 0, 0, us));
      HIP_TRY(launch_layer_update(seg->dtype, ly.W32, ly.vW, ly.dW, ly.N, ly.K, ly.ldk, ly.W16, ly.WT, ly.ldn, nullptr, 0, 0,
                                  nullptr, nullptr, nullptr, seg->lr, seg->mu, 0, us != st ? kSideUpdateWorkgroups : 0, us != st ? pause : 0, us));
    }
  }
  if (forked) {     // join: later work on the caller's stream sees every update
    HIP_TRY(hipEventRecord(seg->ev_join, seg->side));
    if (!defer) HIP_TRY(hipStreamWaitEvent(st, seg->ev_join, 0));
  }
  seg->join_pending = defer && forked;
  return SLP_OK;
}

int refresh_copies(slp_segment* s, int layer, hipStream_t st) {
  Layer& ly = s->layers[layer];
  if (!ly.W16 && !ly.WT) return SLP_OK;
  HIP_TRY(launch_layer_update(s->dtype, ly.W32, ly.vW, ly.dW, ly.N, ly.K, ly.ldk, ly.W16, ly.WT, ly.ldn, nullptr, 0, 0, nullptr,
                              nullptr, nullptr, 0.0f, 0.0f, 1, 0, 0, st));
  return SLP_OK;
}

int copy_matrix(float* dense, float* padded, int rows, int cols, int ld, bool to_padded, int on_device, hipStream_t st) {
  const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : (to_padded ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost);
  if (to_padded)
    HIP_TRY(hipMemcpy2DAsync(padded, (size_t)ld * 4, dense, (size_t)cols * 4, (size_t)cols * 4, rows, kind, st));
  else
    HIP_TRY(hipMemcpy2DAsync(dense, (size_t)cols * 4, padded, (size_t)ld * 4, (size_t)cols * 4, rows, kind, st));
  return SLP_OK;
}

int exchange(slp_segment* s, int layer, float* W, float* b, int which, bool set, int on_device, hipStream_t st) {
  int rc = check_seg(s, true, !set);
  if (rc) return rc;
  if (layer < 0 || layer >= s->L) return fail(SLP_ERR_ARG, "layer %d out of range [0,%d)", layer, s->L);
  rc = settle(s, st);
  if (rc) return rc;
  Layer& ly = s->layers[layer];
  float* mats[3] = {ly.W32, ly.dW, ly.vW};
  float* vecs[3] = {ly.b, ly.db, ly.vb};
  if (W && which == 1 && s->fused_update && (long)ly.N * ly.K <= s->fused_max_params)
    return fail(SLP_ERR_STATE, "the weight gradient of layer %d is not stored: its update is fused into the product (slp_segment_set_fused_update)", layer);
  if (W) {
    rc = copy_matrix(W, mats[which], ly.N, ly.K, ly.ldk, set, on_device, st);
    if (rc) return rc;
  }
  if (b) {
    const hipMemcpyKind kind = on_device ? hipMemcpyDeviceToDevice : (set ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost);
    if (set) HIP_TRY(hipMemcpyAsync(vecs[which], b, (size_t)ly.N * 4, kind, st));
    else HIP_TRY(hipMemcpyAsync(b, vecs[which], (size_t)ly.N * 4, kind, st));
  }
  if (set && W) {
    rc = refresh_copies(s, layer, st);
    if (rc) return rc;
  }
  if (!on_device) HIP_TRY(hipStreamSynchronize(st));
  return SLP_OK;
}

}  // namespace

extern "C" {

const char* slp_last_error(void) { return g_err; }

int slp_make_synthetic_labels(uint64_t seed, int classes, int dim, int dist, float kappa, void* table, int dt,
                              slp_stream stream) {
  if (!table) return fail(SLP_ERR_ARG, "table is NULL");
  if (classes <= 0 || dim <= 0) return fail(SLP_ERR_ARG, "classes and dim must be positive (got %d, %d)", classes, dim);
  if (dist < SLP_UNIFORM01 || dist > SLP_BINARY_PM1) return fail(SLP_ERR_ARG, "unknown distribution %d", dist);
  if (dt != SLP_F32 && dt != SLP_BF16) return fail(SLP_ERR_ARG, "unknown dtype %d", dt);
  HIP_TRY(launch_make_labels(seed, classes, dim, dist, kappa, table, dt, (hipStream_t)stream));
  return SLP_OK;
}

int slp_make_segment_inputs(uint64_t seed, const float* table, int classes, const int32_t* y, int64_t first_sample,
                            int batch, int dim, float sigma, void* out, int dt, slp_stream stream) {
  if (!table || !y || !out) return fail(SLP_ERR_ARG, "table, y and out must not be NULL");
  if (classes <= 0 || dim <= 0 || batch <= 0 || first_sample < 0)
    return fail(SLP_ERR_ARG, "classes, dim, batch must be positive and first_sample non-negative");
  if (dt != SLP_F32 && dt != SLP_BF16) return fail(SLP_ERR_ARG, "unknown dtype %d", dt);
  HIP_TRY(launch_make_inputs(seed, table, classes, y, first_sample, batch, dim, sigma, out, dt, (hipStream_t)stream));
  return SLP_OK;
}

int slp_segment_create(const int* widths, int n_widths, int act, int loss, const slp_opts* opts, slp_segment** out) {
  if (!widths || !opts || !out) return fail(SLP_ERR_ARG, "widths, opts and out must not be NULL");
  *out = nullptr;
  if (n_widths < 2) return fail(SLP_ERR_ARG, "a segment needs at least one layer (n_widths = %d)", n_widths);
  if (n_widths > 65) return fail(SLP_ERR_ARG, "too many layers (%d)", n_widths - 1);
  for (int i = 0; i < n_widths; ++i)
    if (widths[i] <= 0 || widths[i] > (1 << 20)) return fail(SLP_ERR_ARG, "widths[%d] = %d is not in [1, 2^20]", i, widths[i]);
  if (act != SLP_RELU_ALL && act != SLP_RELU_HIDDEN_IDENTITY_LAST) return fail(SLP_ERR_ARG, "unknown activation rule %d", act);
  if (loss != SLP_MSE_SIL && loss != SLP_SOFTMAX_XENT) return fail(SLP_ERR_ARG, "unknown loss %d", loss);
  if (opts->dtype != SLP_F32 && opts->dtype != SLP_BF16) return fail(SLP_ERR_ARG, "unknown dtype %d", opts->dtype);
  if (opts->max_batch <= 0 || opts->max_batch > (1 << 24)) return fail(SLP_ERR_ARG, "max_batch = %d is not in [1, 2^24]", opts->max_batch);
  if (!(opts->lr >= 0.0f) || !(opts->momentum >= 0.0f && opts->momentum < 1.0f))
    return fail(SLP_ERR_ARG, "lr must be >= 0 and momentum in [0,1)");

  slp_segment* s = new slp_segment();
  s->L = n_widths - 1; s->act = act; s->loss = loss; s->dtype = opts->dtype; s->max_batch = opts->max_batch;
  s->ldb = internal_ld(opts->max_batch, opts->dtype == SLP_BF16 ? 2 : 4);
  s->lr = opts->lr; s->mu = opts->momentum;
  s->input_grad = opts->input_grad != 0;
  s->widths.assign(widths, widths + n_widths);
  for (int w : s->widths) s->ldw.push_back(internal_ld(w, opts->dtype == SLP_BF16 ? 2 : 4));
  const size_t es = esize(s);

  // every operand is addressed with 32-bit byte offsets below 2 GiB
  for (int l = 0; l <= s->L; ++l) {
    const size_t act_bytes = (size_t)std::max(s->ldb * (size_t)s->widths[l], (size_t)s->max_batch * s->ldw[l]) * es;
    if (act_bytes >= 0x80000000ull) {
      delete s;
      return fail(SLP_ERR_SHAPE, "activation of layer %d (%zu bytes) exceeds the 2 GiB operand limit", l, act_bytes);
    }
  }

  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  for (int l = 0; l < s->L; ++l) {
    Layer ly{};
    ly.K = widths[l]; ly.N = widths[l + 1];
    ly.ldk = s->ldw[l]; ly.ldn = s->ldw[l + 1];
    const size_t wbytes = (size_t)ly.N * ly.ldk * 4;
    if (wbytes >= 0x80000000ull || (size_t)ly.K * ly.ldn * 4 >= 0x80000000ull) {
      delete s;
      return fail(SLP_ERR_SHAPE, "weight matrix of layer %d exceeds the 2 GiB operand limit", l);
    }
    ly.oW32 = take(wbytes); ly.ovW = take(wbytes); ly.odW = take(wbytes);
    ly.ob = take((size_t)ly.N * 4); ly.ovb = take((size_t)ly.N * 4); ly.odb = take((size_t)ly.N * 4);
    ly.oW16 = s->dtype == SLP_BF16 ? take((size_t)ly.N * ly.ldk * 2) : (size_t)-1;
    ly.oWT = (l > 0 || s->input_grad) ? take((size_t)ly.K * ly.ldn * es) : (size_t)-1;
    s->layers.push_back(ly);
  }
  s->param_bytes = off;

  off = 0;
  s->oA.assign(s->L + 1, (size_t)-1); s->oAT = s->oA; s->odZ = s->oA; s->odZT = s->oA; s->oBits = s->oA;
  s->ldbits = (s->max_batch + 127) / 128 * 4;
  for (int l = 0; l <= s->L; ++l) {
    s->oA[l] = take((size_t)s->max_batch * s->ldw[l] * es);
    if (l < s->L) s->oAT[l] = take((size_t)s->widths[l] * s->ldb * es);
    if (l >= 1 && l < s->L && s->dtype == SLP_BF16) s->oBits[l] = take((size_t)s->widths[l] * s->ldbits * 4);
    if (l == 0 && s->input_grad) s->odZ[0] = take((size_t)s->max_batch * s->ldw[0] * es);
    if (l >= 1) {
      // row-major dZ_l is the A operand of layer l's data gradient: needed for l >= 2, for the loss
      // kernels' output (l = L), and for l = 1 when the gradient w.r.t. the input is wanted
      if (l >= 2 || l == s->L || s->input_grad) s->odZ[l] = take((size_t)s->max_batch * s->ldw[l] * es);
      s->odZT[l] = take((size_t)s->widths[l] * s->ldb * es);
    }
  }
  s->n_partials = loss == SLP_MSE_SIL ? mse_partial_count(s->max_batch, s->widths[s->L]) : s->max_batch;
  s->oPartials = take((size_t)s->n_partials * 4);
  s->oLoss = take(4);
  s->oBadIds = take(4);
  s->work_bytes = off;

  s->side = nullptr; s->ev_join = nullptr;
  s->defer_join = false; s->join_pending = false; s->fused_update = false; s->fused_max_params = 0;
  s->bound = false; s->have_params = false; s->table = nullptr; s->classes = 0; s->last_batch = 0; s->prof = false;
  s->use_graph = false; s->graph_warm = false; s->graph_tick = 0; s->graph_misses = 0;
  s->partials = nullptr; s->loss_dev = nullptr; s->bad_ids = nullptr;
  *out = s;
  return SLP_OK;
}

void slp_segment_destroy(slp_segment* seg) {
  if (!seg) return;
  for (auto& r : seg->prof_log) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : seg->ev_pool) (void)hipEventDestroy(e);
  for (auto e : seg->ev_fork) (void)hipEventDestroy(e);
  if (seg->ev_join) (void)hipEventDestroy(seg->ev_join);
  drop_graphs(seg);
  if (seg->side) {
    (void)hipStreamSynchronize(seg->side);   // updates of a step with a deferred join may still be writing the caller's buffers
    (void)hipStreamDestroy(seg->side);
  }
  delete seg;
}

size_t slp_segment_param_bytes(const slp_segment* seg) { return seg ? seg->param_bytes : 0; }
size_t slp_segment_workspace_bytes(const slp_segment* seg) { return seg ? seg->work_bytes : 0; }

int slp_segment_bind(slp_segment* seg, void* params, size_t params_bytes, void* workspace, size_t workspace_bytes,
                     slp_stream stream) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  if (seg->join_pending) {     // the old buffers are still being written
    HIP_TRY(hipStreamSynchronize(seg->side));
    seg->join_pending = false;
  }
  if (!params || !workspace) return fail(SLP_ERR_ARG, "params and workspace must not be NULL");
  if (((uintptr_t)params | (uintptr_t)workspace) & (kAlign - 1)) return fail(SLP_ERR_ALLOC, "buffers must be 256-byte aligned");
  if (params_bytes < seg->param_bytes) return fail(SLP_ERR_ALLOC, "params buffer has %zu bytes, %zu needed", params_bytes, seg->param_bytes);
  if (workspace_bytes < seg->work_bytes) return fail(SLP_ERR_ALLOC, "workspace has %zu bytes, %zu needed", workspace_bytes, seg->work_bytes);
  hipStream_t st = (hipStream_t)stream;
  drop_graphs(seg);      // captured steps hold the old buffers' addresses
  seg->graph_warm = false;
  HIP_TRY(hipMemsetAsync(params, 0, seg->param_bytes, st));
  HIP_TRY(hipMemsetAsync(workspace, 0, seg->work_bytes, st));
  char* p = (char*)params;
  for (auto& ly : seg->layers) {
    ly.W32 = (float*)(p + ly.oW32); ly.vW = (float*)(p + ly.ovW); ly.dW = (float*)(p + ly.odW);
    ly.b = (float*)(p + ly.ob); ly.vb = (float*)(p + ly.ovb); ly.db = (float*)(p + ly.odb);
    ly.W16 = ly.oW16 == (size_t)-1 ? nullptr : (void*)(p + ly.oW16);
    ly.WT = ly.oWT == (size_t)-1 ? nullptr : (void*)(p + ly.oWT);
    ly.Wop = ly.W16 ? ly.W16 : (void*)ly.W32;
  }
  char* w = (char*)workspace;
  auto at = [&](size_t o) -> void* { return o == (size_t)-1 ? nullptr : (void*)(w + o); };
  seg->A.clear(); seg->AT.clear(); seg->dZ.clear(); seg->dZT.clear(); seg->bits.clear();
  for (int l = 0; l <= seg->L; ++l) {
    seg->A.push_back(at(seg->oA[l])); seg->AT.push_back(at(seg->oAT[l]));
    seg->dZ.push_back(at(seg->odZ[l])); seg->dZT.push_back(at(seg->odZT[l]));
    seg->bits.push_back((uint32_t*)at(seg->oBits[l]));
  }
  seg->partials = (float*)at(seg->oPartials);
  seg->loss_dev = (float*)at(seg->oLoss);
  seg->bad_ids = (unsigned*)at(seg->oBadIds);
  if (!seg->side) {     // host-side objects only; default priority
    HIP_TRY(hipStreamCreateWithFlags(&seg->side, hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&seg->ev_join, hipEventDisableTiming));
    for (int l = 0; l < seg->L; ++l) {
      hipEvent_t e = nullptr;
      HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      seg->ev_fork.push_back(e);
    }
  }
  seg->bound = true;
  seg->have_params = false;
  return SLP_OK;
}

int slp_segment_init(slp_segment* seg, uint64_t seed, slp_stream stream) {
  int rc = check_seg(seg, true, false);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  rc = settle(seg, st);
  if (rc) return rc;
  for (int l = 0; l < seg->L; ++l) {
    Layer& ly = seg->layers[l];
    HIP_TRY(launch_init_weights(seed, l, ly.W32, ly.N, ly.K, ly.ldk, ly.b, st));
    HIP_TRY(hipMemsetAsync(ly.vW, 0, (size_t)ly.N * ly.ldk * 4, st));
    HIP_TRY(hipMemsetAsync(ly.vb, 0, (size_t)ly.N * 4, st));
    rc = refresh_copies(seg, l, st);
    if (rc) return rc;
  }
  seg->have_params = true;
  return SLP_OK;
}

int slp_segment_set_params(slp_segment* seg, int layer, const float* W, const float* b, int on_device, slp_stream stream) {
  int rc = exchange(seg, layer, const_cast<float*>(W), const_cast<float*>(b), 0, true, on_device, (hipStream_t)stream);
  if (rc == SLP_OK) seg->have_params = true;
  return rc;
}
int slp_segment_get_params(slp_segment* seg, int layer, float* W, float* b, int on_device, slp_stream stream) {
  return exchange(seg, layer, W, b, 0, false, on_device, (hipStream_t)stream);
}
int slp_segment_get_grads(slp_segment* seg, int layer, float* dW, float* db, int on_device, slp_stream stream) {
  return exchange(seg, layer, dW, db, 1, false, on_device, (hipStream_t)stream);
}
int slp_segment_get_momentum(slp_segment* seg, int layer, float* vW, float* vb, int on_device, slp_stream stream) {
  return exchange(seg, layer, vW, vb, 2, false, on_device, (hipStream_t)stream);
}

int slp_segment_get_activation(slp_segment* seg, int layer, int kind, int batch, void* out, slp_stream stream) {
  int rc = check_seg(seg, true, false);
  if (rc) return rc;
  if (!out) return fail(SLP_ERR_ARG, "out is NULL");
  if (layer < 0 || layer > seg->L || (kind != 0 && kind != 1)) return fail(SLP_ERR_ARG, "layer %d / kind %d out of range", layer, kind);
  if (batch <= 0 || batch > seg->max_batch) return fail(SLP_ERR_SHAPE, "batch %d not in [1,%d]", batch, seg->max_batch);
  hipStream_t st = (hipStream_t)stream;
  rc = settle(seg, st);
  if (rc) return rc;
  const int w = seg->widths[layer];
  if (kind == 0) {
    HIP_TRY(launch_copy_transpose(seg->dtype, seg->A[layer], seg->ldw[layer], batch, w, out, w, nullptr, 0, 0, nullptr, 0, st));
  } else {
    if (layer < 1) return fail(SLP_ERR_ARG, "no gradient is formed for the segment input");
    if (seg->dZ[layer]) {
      HIP_TRY(launch_copy_transpose(seg->dtype, seg->dZ[layer], seg->ldw[layer], batch, w, out, w, nullptr, 0, 0, nullptr, 0, st));
    } else {   // only the transposed copy exists: transpose it back
      HIP_TRY(launch_copy_transpose(seg->dtype, seg->dZT[layer], seg->ldb, w, batch, nullptr, 0, out, w, 0, nullptr, 0, st));
    }
  }
  return SLP_OK;
}

int slp_segment_set_lr(slp_segment* seg, float lr, float momentum) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  if (!(lr >= 0.0f) || !(momentum >= 0.0f && momentum < 1.0f)) return fail(SLP_ERR_ARG, "lr must be >= 0 and momentum in [0,1)");
  seg->lr = lr; seg->mu = momentum;
  drop_graphs(seg);
  return SLP_OK;
}

int slp_segment_set_labels(slp_segment* seg, const float* table, int classes, int dim) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  if (seg->loss != SLP_MSE_SIL) return fail(SLP_ERR_STATE, "only a segment with the label-regression loss takes a label table");
  if (!table || classes <= 0) return fail(SLP_ERR_ARG, "table must not be NULL and classes positive");
  if (dim != seg->widths[seg->L]) return fail(SLP_ERR_SHAPE, "label dim %d != last width %d", dim, seg->widths[seg->L]);
  seg->table = table; seg->classes = classes;
  drop_graphs(seg);
  return SLP_OK;
}

int slp_segment_forward(slp_segment* seg, const void* X, int batch, void* out, slp_stream stream) {
  int rc = check_seg(seg, true, true);
  if (rc) return rc;
  if (!X || !out) return fail(SLP_ERR_ARG, "X and out must not be NULL");
  if (batch <= 0 || batch > seg->max_batch) return fail(SLP_ERR_SHAPE, "batch %d not in [1,%d]", batch, seg->max_batch);
  hipStream_t st = (hipStream_t)stream;
  rc = settle(seg, st);
  if (rc) return rc;
  // the stored-response pass over a whole dataset (Sec. 2) is this call in a loop: no activation is kept for a
  // backward pass, and dense caller buffers whose rows start on 16-byte boundaries are used in place
  const int w0 = seg->widths[0], w = seg->widths[seg->L];
  const bool x_direct = w0 % kLdRows == 0 && ((uintptr_t)X & 127) == 0;      // rows on cache-line boundaries, else the copy pays
  const bool out_direct = w % kLdAlign == 0 && ((uintptr_t)out & 15) == 0;
  if (!x_direct) {
    rc = ingest(seg, X, batch, false, st);
    if (rc) return rc;
  }
  rc = forward_layers(seg, batch, false, st, x_direct ? X : nullptr, out_direct ? out : nullptr);
  if (rc) return rc;
  if (!out_direct)
    HIP_TRY(launch_copy_transpose(seg->dtype, seg->A[seg->L], seg->ldw[seg->L], batch, w, out, w, nullptr, 0, 0, nullptr, 0, st));
  seg->last_batch = batch;
  return SLP_OK;
}

int slp_segment_step(slp_segment* seg, const void* X, const int32_t* targets, int batch, float* loss_out, slp_stream stream) {
  int rc = check_seg(seg, true, true);
  if (rc) return rc;
  if (!X || !targets) return fail(SLP_ERR_ARG, "X and targets must not be NULL");
  if (batch <= 0 || batch > seg->max_batch) return fail(SLP_ERR_SHAPE, "batch %d not in [1,%d]", batch, seg->max_batch);
  if (seg->loss == SLP_MSE_SIL && !seg->table) return fail(SLP_ERR_STATE, "no label table bound: call slp_segment_set_labels first");
  hipStream_t st = (hipStream_t)stream;
  seg->last_batch = batch;
  rc = settle(seg, st);
  if (rc) return rc;

  auto launch_all = [&]() -> int {
    int r = ingest(seg, X, batch, true, st);
    if (!r) r = forward_layers(seg, batch, true, st);
    if (!r) r = loss_and_output_grad(seg, targets, batch, loss_out, st);
    if (!r) r = backward_and_update(seg, batch, st);
    return r;
  };
  // Eager launches when graphs are off, when launches are being timed one by one, on the null stream (it
  // cannot be captured), and when the caller is capturing this stream already (the launches then go into
  // the caller's graph).  The first step of a handle is eager too, so that one-time kernel set-up is over
  // before anything is captured.
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (seg->use_graph && st) HIP_TRY(hipStreamIsCapturing(st, &cap));
  // A caller that never repeats a combination (a loop over more distinct batch buffers than the cache holds) would
  // pay a capture per step: after 2 x cache size misses in a row the handle goes back to eager launches until
  // slp_segment_set_graph is called again.
  const bool thrashing = seg->graph_misses > 2 * (int)kMaxStepGraphs;
  if (!seg->use_graph || thrashing || seg->prof || !st || cap != hipStreamCaptureStatusNone || !seg->graph_warm) {
    seg->graph_warm = true;
    return launch_all();
  }
  ++seg->graph_tick;
  for (auto& g : seg->graphs)
    if (g.X == X && g.targets == targets && g.batch == batch && g.loss_out == loss_out) {
      g.used = seg->graph_tick;
      seg->graph_misses = 0;
      HIP_TRY(hipGraphLaunch(g.exec, st));
      return SLP_OK;
    }
  ++seg->graph_misses;
  HIP_TRY(hipStreamBeginCapture(st, hipStreamCaptureModeThreadLocal));
  rc = launch_all();
  hipGraph_t graph = nullptr;
  hipError_t e = hipStreamEndCapture(st, &graph);      // always ended, so that the stream is usable after an error
  if (rc || e != hipSuccess) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc ? rc : fail(SLP_ERR_DEVICE, "hipStreamEndCapture: %s", hipGetErrorString(e));
  }
  StepGraph sg{X, targets, batch, loss_out, nullptr, seg->graph_tick};
  e = hipGraphInstantiate(&sg.exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e != hipSuccess) return fail(SLP_ERR_DEVICE, "hipGraphInstantiate: %s", hipGetErrorString(e));
  if (seg->graphs.size() >= kMaxStepGraphs) {          // evict the least recently used
    size_t v = 0;
    for (size_t i = 1; i < seg->graphs.size(); ++i)
      if (seg->graphs[i].used < seg->graphs[v].used) v = i;
    HIP_TRY(hipDeviceSynchronize());                   // its last replay may still be running
    (void)hipGraphExecDestroy(seg->graphs[v].exec);
    seg->graphs[v] = sg;
  } else {
    seg->graphs.push_back(sg);
  }
  HIP_TRY(hipGraphLaunch(sg.exec, st));
  return SLP_OK;
}

int slp_segment_target_errors(slp_segment* seg, int64_t* count_out, slp_stream stream) {
  int rc = check_seg(seg, true, false);
  if (rc) return rc;
  if (!count_out) return fail(SLP_ERR_ARG, "count_out is NULL");
  hipStream_t st = (hipStream_t)stream;
  unsigned n = 0;
  HIP_TRY(hipMemcpyAsync(&n, seg->bad_ids, sizeof(n), hipMemcpyDeviceToHost, st));
  HIP_TRY(hipStreamSynchronize(st));
  *count_out = (int64_t)n;
  return SLP_OK;
}

int slp_segment_set_graph(slp_segment* seg, int on) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  if (on) HIP_TRY(gemm_configure_all());
  seg->use_graph = on != 0;
  seg->graph_misses = 0;
  if (!seg->use_graph) drop_graphs(seg);
  return SLP_OK;
}

int slp_segment_set_overlap(slp_segment* seg, int on) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  seg->defer_join = on != 0;
  if (!on && seg->join_pending) {      // back to ordinary stream order: nothing is left running
    HIP_TRY(hipStreamSynchronize(seg->side));
    seg->join_pending = false;
  }
  return SLP_OK;
}

int slp_segment_set_fused_update(slp_segment* seg, int on) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  if (on < 0) return fail(SLP_ERR_ARG, "slp_segment_set_fused_update: on must be >= 0 (got %d)", on);
  if (seg->join_pending) {             // updates of the other kind may still be running on the side stream
    HIP_TRY(hipStreamSynchronize(seg->side));
    seg->join_pending = false;
  }
  seg->fused_update = on != 0;
  seg->fused_max_params = on == 1 ? (1L << 62) : (on == 2 ? kFusedAutoMaxWeights : (long)on);
  drop_graphs(seg);                    // captured steps hold the other launch sequence
  return SLP_OK;
}

int slp_segment_join(slp_segment* seg, slp_stream stream) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  return settle(seg, (hipStream_t)stream);
}

int slp_segment_input_grad(slp_segment* seg, const void* X, const int32_t* targets, int batch, void* dX, float* loss_out,
                           slp_stream stream) {
  int rc = check_seg(seg, true, true);
  if (rc) return rc;
  if (!seg->input_grad) return fail(SLP_ERR_STATE, "segment was created without input_grad");
  if (!X || !targets || !dX) return fail(SLP_ERR_ARG, "X, targets and dX must not be NULL");
  if (batch <= 0 || batch > seg->max_batch) return fail(SLP_ERR_SHAPE, "batch %d not in [1,%d]", batch, seg->max_batch);
  if (seg->loss == SLP_MSE_SIL && !seg->table) return fail(SLP_ERR_STATE, "no label table bound: call slp_segment_set_labels first");
  hipStream_t st = (hipStream_t)stream;
  rc = settle(seg, st);
  if (rc) return rc;
  rc = ingest(seg, X, batch, true, st);
  if (rc) return rc;
  rc = forward_layers(seg, batch, true, st);
  if (rc) return rc;
  rc = loss_and_output_grad(seg, targets, batch, loss_out, st);
  if (rc) return rc;
  for (int l = seg->L; l >= 1; --l) {       // data gradients only, down to the input; parameters untouched
    rc = data_gradient(seg, l, batch, st);
    if (rc) return rc;
  }
  const int w0 = seg->widths[0];
  HIP_TRY(launch_copy_transpose(seg->dtype, seg->dZ[0], seg->ldw[0], batch, w0, dX, w0, nullptr, 0, 0, nullptr, 0, st));
  seg->last_batch = batch;
  return SLP_OK;
}

int slp_segment_step_external(slp_segment* seg, const void* X, const void* dA_out, int batch, slp_stream stream) {
  int rc = check_seg(seg, true, true);
  if (rc) return rc;
  if (!X || !dA_out) return fail(SLP_ERR_ARG, "X and dA_out must not be NULL");
  if (batch <= 0 || batch > seg->max_batch) return fail(SLP_ERR_SHAPE, "batch %d not in [1,%d]", batch, seg->max_batch);
  hipStream_t st = (hipStream_t)stream;
  rc = settle(seg, st);
  if (rc) return rc;
  const int L = seg->L, D = seg->widths[L];
  rc = ingest(seg, X, batch, true, st);
  if (rc) return rc;
  rc = forward_layers(seg, batch, true, st);
  if (rc) return rc;
  // dZ_L = dA_out * [A_L > 0] (ReLU on the last layer) or dA_out, in both layouts
  HIP_TRY(launch_copy_transpose(seg->dtype, dA_out, D, batch, D, seg->dZ[L], seg->ldw[L], seg->dZT[L], seg->ldb, 1,
                                relu_on(seg, L) ? seg->A[L] : nullptr, seg->ldw[L], st));
  rc = backward_and_update(seg, batch, st);
  if (rc) return rc;
  seg->last_batch = batch;
  return SLP_OK;
}

int slp_count_correct(const void* logits, const int32_t* targets, int batch, int classes, int dt, void* scratch,
                      size_t scratch_bytes, int accumulate, int64_t* correct_out, slp_stream stream) {
  if (!logits || !targets || !scratch || !correct_out) return fail(SLP_ERR_ARG, "slp_count_correct: null pointer");
  if (batch <= 0 || classes <= 0) return fail(SLP_ERR_ARG, "slp_count_correct: batch and classes must be positive (got %d, %d)", batch, classes);
  if (dt != SLP_F32 && dt != SLP_BF16) return fail(SLP_ERR_ARG, "slp_count_correct: unknown dtype %d", dt);
  const size_t need = (size_t)count_partials(batch) * sizeof(int32_t);
  if (scratch_bytes < need || ((uintptr_t)scratch & 3))
    return fail(SLP_ERR_ALLOC, "slp_count_correct: scratch of %zu bytes (4-byte aligned) needed, %zu given", need, scratch_bytes);
  HIP_TRY(launch_count_correct(dt, logits, targets, batch, classes, (int32_t*)scratch, accumulate, (long long*)correct_out,
                               (hipStream_t)stream));
  return SLP_OK;
}

int slp_count_correct_static(const void* logits, const int32_t* targets, int batch, int classes, int dt, int accumulate,
                             int64_t* correct_out, slp_stream stream) {
  if (!logits || !targets || !correct_out) return fail(SLP_ERR_ARG, "slp_count_correct_static: null pointer");
  if (batch <= 0 || classes <= 0)
    return fail(SLP_ERR_ARG, "slp_count_correct_static: batch and classes must be positive (got %d, %d)", batch, classes);
  if (dt != SLP_F32 && dt != SLP_BF16) return fail(SLP_ERR_ARG, "slp_count_correct_static: unknown dtype %d", dt);
  static_assert(SLP_COUNT_STATIC_MAX_BATCH == 4 * kCountStaticPartials, "header limit and array size must agree");
  if (batch > SLP_COUNT_STATIC_MAX_BATCH)
    return fail(SLP_ERR_SHAPE, "slp_count_correct_static: batch %d exceeds the static scratch's limit of %d rows", batch,
                SLP_COUNT_STATIC_MAX_BATCH);
  int32_t* partials = nullptr;
  HIP_TRY(count_static_scratch(&partials));      // looked up once per device; never the array's name itself
  HIP_TRY(launch_count_correct(dt, logits, targets, batch, classes, partials, accumulate, (long long*)correct_out,
                               (hipStream_t)stream));
  return SLP_OK;
}

int slp_mean_loss(const float* losses, int n, float* mean_out, slp_stream stream) {
  if (!losses || !mean_out) return fail(SLP_ERR_ARG, "slp_mean_loss: null pointer");
  if (n <= 0) return fail(SLP_ERR_ARG, "slp_mean_loss: n must be positive (got %d)", n);
  HIP_TRY(launch_reduce_loss(losses, n, 1.0 / (double)n, mean_out, nullptr, (hipStream_t)stream));
  return SLP_OK;
}

int slp_segment_profile_enable(slp_segment* seg, int on) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  seg->prof = on != 0;
  // on > 1: create that many event pairs now, so that none is created between timed launches
  for (int i = (int)seg->ev_pool.size(); on > 1 && i < 2 * on; ++i) {
    hipEvent_t e = nullptr;
    HIP_TRY(hipEventCreate(&e));
    seg->ev_pool.push_back(e);
  }
  return SLP_OK;
}

int slp_segment_profile_read(slp_segment* seg, double* gemm_ms, int64_t* gemm_launches, double* gemm_flops) {
  int rc = check_seg(seg, false, false);
  if (rc) return rc;
  double ms = 0.0, fl = 0.0;
  int64_t n = 0;
  for (auto& r : seg->prof_log) {
    HIP_TRY(hipEventSynchronize(r.b));
    float t = 0.0f;
    HIP_TRY(hipEventElapsedTime(&t, r.a, r.b));
    ms += t; fl += r.flops; ++n;
    seg->ev_pool.push_back(r.a);
    seg->ev_pool.push_back(r.b);
  }
  seg->prof_log.clear();
  if (gemm_ms) *gemm_ms = ms;
  if (gemm_launches) *gemm_launches = n;
  if (gemm_flops) *gemm_flops = fl;
  return SLP_OK;
}

int slp_probe_mfma_rate(int dtype, int iters, void* scratch, size_t scratch_bytes, double* tflops, double* ms, slp_stream stream) {
  if (dtype != SLP_F32 && dtype != SLP_BF16) return fail(SLP_ERR_ARG, "slp_probe_mfma_rate: unknown dtype %d", dtype);
  if (iters <= 0 || iters > (1 << 24)) return fail(SLP_ERR_ARG, "slp_probe_mfma_rate: iters %d outside [1, 2^24]", iters);
  if (!scratch || !tflops) return fail(SLP_ERR_ARG, "slp_probe_mfma_rate: null scratch or result pointer");
  int dev = 0, cus = 0;
  HIP_TRY(hipGetDevice(&dev));
  HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const size_t per_wg = 512 * sizeof(float);
  if (scratch_bytes < per_wg * (size_t)cus)
    return fail(SLP_ERR_SHAPE, "slp_probe_mfma_rate: scratch of %zu bytes, %zu needed (%d compute units x 2048)", scratch_bytes,
                per_wg * (size_t)cus, cus);
  hipStream_t s = (hipStream_t)stream;
  hipEvent_t a = nullptr, b = nullptr;
  HIP_TRY(hipEventCreate(&a));
  HIP_TRY(hipEventCreate(&b));
  double fl = 0.0;
  hipError_t e = launch_mfma_probe(dtype, iters / 8 + 1, cus, (float*)scratch, &fl, s);   // warm-up: clocks settle
  if (e == hipSuccess) e = hipEventRecord(a, s);
  if (e == hipSuccess) e = launch_mfma_probe(dtype, iters, cus, (float*)scratch, &fl, s);
  if (e == hipSuccess) e = hipEventRecord(b, s);
  if (e == hipSuccess) e = hipEventSynchronize(b);
  float t = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&t, a, b);
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  if (e != hipSuccess) return fail(SLP_ERR_DEVICE, "slp_probe_mfma_rate: %s", hipGetErrorString(e));
  *tflops = fl * cus * iters / (t * 1e-3) / 1e12;
  if (ms) *ms = t;
  return SLP_OK;
}

}  // extern "C"
