// Internal launch interface between the C ABI (api.hip) and the HIP kernels.
// Not part of the public boundary; see include/slp.h for that.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

namespace slp {

// Leading dimensions of every internal buffer are multiples of this many elements,
// so that each row starts on a 16-byte boundary for both element types and a
// 16-byte chunk never straddles two rows.  Pad elements are zero.
constexpr int kLdAlign = 8;
// What the library's own buffers use: rows that start on 128-byte boundaries (bf16), so that the 128-byte row
// segment of a k-tile is one cache line, not two halves (measured 17 % on a product with rows 16 bytes off).
constexpr int kLdRows = 64;
inline int round_up(int x, int a) { return (x + a - 1) / a * a; }
// Leading dimension of one of the library's own matrices with rows of `width` elements of `esize` bytes: a multiple
// of kLdRows, and never a multiple of 4 KB in bytes -- rows one page multiple apart keep the 256 rows of an operand
// strip on few L2 sets and memory channels (measured +1-2 % on 8192x16384x16384 with any skew of 256 bytes or more).
constexpr int kLdSkew = 192;
inline int internal_ld(int width, int esize) {
  int ld = round_up(width, kLdRows);
  if (((size_t)ld * esize) % 4096 == 0) ld += kLdSkew;
  return ld;
}

enum Epilogue { EPI_FWD = 0, EPI_DGRAD = 1, EPI_WGRAD = 2, EPI_WGRAD_UPDATE = 3 };

// C[m][n] = sum_k A[m][k] * B[n][k]  ("NT": both operands contraction-contiguous).
struct GemmArgs {
  const void* A;   // [M][lda]
  const void* B;   // [N][ldb]
  int lda, ldb;
  int M, N, K;     // logical sizes; pads up to the next chunk must be zero in A and B
  int group_m;     // tile rows per group of the workgroup -> tile walk; 0 = default, -1 = 16 x 16 regions (set by launch_gemm)
  // EPI_FWD  : v = acc + bias[n], optional ReLU; C (row-major) and/or CT (transposed) in T
  // EPI_DGRAD: v = acc * [maskT[n][m] > 0];      C and/or CT in T
  // EPI_WGRAD: Cf[m][n] = acc (float32)
  void* C;         // [M][ldc] or null
  void* CT;        // [N][ldct] or null; columns m in [M, round_up(M,8)) are written as zero
  int ldc, ldct;
  const float* bias;
  int relu;
  const void* maskT;  // [N][ldmask], element type T
  int ldmask;
  // The same mask as one bit per element, for products that run on the 256x256 bf16 tile (every other tile configuration
  // ignores both pointers): EPI_FWD writes bits_out, EPI_DGRAD reads bits instead of maskT when it is not null.
  // Row n holds ldbits dwords; dword 4 * (m / 128) + g carries, at bit 4 i + e, the element m = 128 (m / 128) + 16 i + 4 g + e
  // (g = 0..3, i = 0..7, e = 0..3: the elements one lane of the tile's accumulator layout holds), set where the stored
  // output is > 0.  ldbits >= 4 * ceil(M / 128); both products must have the same M and N.
  uint32_t* bits_out;
  const uint32_t* bits;
  int ldbits;
  float* Cf;       // [M][ldc] float32
  // EPI_WGRAD_UPDATE: the gradient never goes to memory; the epilogue applies the optimiser step to the tile it holds
  // (paper Sec. 3: SGD with momentum), v = mu v + acc; w -= lr v, on the float32 master weights uW and momentum uV
  // (both [M][ldc]), and rewrites the derived copies uW16 (bf16 [M][ldc], may be null) and uWT ([N][ldwt], element
  // type T, may be null).  Cf is not used.
  float* uW; float* uV; void* uW16; void* uWT;
  int ldwt;
  float lr, mu;
};

// dtype: 0 = float32 operands, 1 = bf16 operands (float32 accumulation in both).
hipError_t launch_gemm(int dtype, int epi, const GemmArgs& g, hipStream_t s);
// Name of the tile configuration launch_gemm would pick (for logs and profiles).
const char* gemm_config_name(int dtype, int M, int N, int K);

// in[R][ldin] -> out[R][ldo] (optional) and outT[C][ldt] (optional; with pad_t the
// columns r in [R, round_up(R,8)) of outT are zero-filled).  With mask (same shape as in,
// leading dimension ldmask) an element passes only where mask > 0.  Element type by dtype.
hipError_t launch_copy_transpose(int dtype, const void* in, int ldin, int R, int C, void* out, int ldo, void* outT,
                                 int ldt, int pad_t, const void* mask, int ldmask, hipStream_t s);

// Both loss kernels clamp a class id outside its range (memory safety) and count such rows into *bad_ids.
// Mean-squared-error loss against table[y[m]] and its gradient w.r.t. the
// pre-activation (ReLU mask applied when relu_last).  Writes dZ (row-major, optional),
// dZT (transposed, zero-filled pads) and one partial sum per block.
hipError_t launch_mse_loss_grad(int dtype, const void* AL, int ld, const int32_t* y, const float* table, int classes,
                                int B, int D, int relu_last, void* dZ, void* dZT, int ldt, float* partials, unsigned* bad_ids,
                                hipStream_t s);
int mse_partial_count(int B, int D);

// Softmax cross-entropy per row: dZ[m][c] = (softmax - onehot)/B (zeroed where the
// last layer's ReLU is inactive when relu_last), per-row loss to partials[m].
hipError_t launch_xent_loss_grad(int dtype, const void* ZL, int ld, const int32_t* y, int B, int C, int relu_last,
                                 void* dZ, float* partials, unsigned* bad_ids, hipStream_t s);

// out0[0] (and out1[0] if not null) = scale * sum(partials[0..n)), fixed summation order.
hipError_t launch_reduce_loss(const float* partials, int n, double scale, float* out0, float* out1, hipStream_t s);

// One launch per layer: SGD with momentum on the weight matrix (v = mu v + g; w -= lr v), its derived copies
// W16 (bf16 [N][ldk], bf16 mode only) and WT ([K][ldn], element type T, optional), and -- unless dZT is null --
// the bias: db[n] = sum_{m < B} dZT[n][m], then the same update on b, vb.
// refresh_only: skip the arithmetic and only rebuild the copies from W32 (dZT must be null).
// max_workgroups > 0 (weights-only launches): run on at most that many workgroups, for updates issued beside matrix products;
// pause: units of ~0.5 us each of those workgroups sleeps between two tiles (paces the update's memory traffic).
hipError_t launch_layer_update(int dtype, float* W32, float* vW, const float* dW, int N, int K, int ldk, void* W16, void* WT,
                               int ldn, const void* dZT, int ldt, int B, float* db, float* b, float* vb, float lr, float mu,
                               int refresh_only, int max_workgroups, int pause, hipStream_t s);

// Counter-based generators (Philox4x32-10).
hipError_t launch_make_labels(uint64_t seed, int classes, int dim, int dist, float kappa, void* out, int dt,
                              hipStream_t s);
hipError_t launch_make_inputs(uint64_t seed, const float* table, int classes, const int32_t* y, int64_t first_sample,
                              int batch, int dim, float sigma, void* out, int dt, hipStream_t s);
hipError_t launch_init_weights(uint64_t seed, int layer, float* W32, int N, int K, int ldk, float* b, hipStream_t s);

// Rows whose arg-max logit (lowest index among equal values) equals the row's class: logits[batch][classes] dense,
// partials = count_partials(batch) int32 of scratch (one per block of four rows, each written before it is read),
// *out = (accumulate ? *out : 0) + count.
int count_partials(int batch);
hipError_t launch_count_correct(int dtype, const void* logits, const int32_t* y, int batch, int classes, int32_t* partials,
                                int accumulate, long long* out, hipStream_t s);

// Partial counts held in a static device array instead of caller memory: enough for batches up to
// 4 * kCountStaticPartials rows.  count_static_scratch returns the array's device address on the current device.
constexpr int kCountStaticPartials = 16384;
hipError_t count_static_scratch(int32_t** ptr);

// Sets the one-time attributes of every matrix-product kernel instantiation (needs a current device).
hipError_t gemm_configure_all();

// Register-only MFMA loop (no memory traffic) on `grid` workgroups of 512 threads; sink holds grid*512 floats.
hipError_t launch_mfma_probe(int dtype, int iters, int grid, float* sink, double* flops_per_workgroup_iter, hipStream_t s);

}  // namespace slp
