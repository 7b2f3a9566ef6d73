// Inference-side reductions of the joined network (paper Sec. 2: the partitions are
// joined after training; Sec. 4 reports the joined network's test accuracy): the number
// of rows whose arg-max logit is the row's class, and the mean of a run of per-step
// losses (the per-epoch figure of the training curves).  Integer counts are summed in a
// fixed order without atomics, so they are exact and reproducible.
#include <limits.h>

#include "slp_kernels.h"

namespace slp {
namespace {

typedef __bf16 bf16;

// Per-block partial counts of the allocation-free entry point.  Device memory that lives in
// the code object: every GPU the library runs on holds its own copy until the process ends.
// Host code must never pass this name to a kernel (on the host it is only a stand-in for the
// symbol); it asks the runtime for the device address once per device and uses that.
__device__ __align__(256) int32_t scratch[kCountStaticPartials];

// One wavefront per row: arg-max with the lowest index winning among equal values (the
// convention of the usual library arg-max), compared with the row's class; the block's four
// rows are added and written as one partial count.
template <typename T>
__global__ __launch_bounds__(256) void count_correct_kernel(const T* __restrict__ logits, const int32_t* __restrict__ y,
                                                            int B, int C, int32_t* __restrict__ partials) {
  __shared__ int hits[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int m = blockIdx.x * 4 + wave;
  float best = -INFINITY;
  int bi = INT_MAX;
  if (m < B) {
    const T* z = logits + (size_t)m * C;
    for (int c = lane; c < C; c += 64) {          // ascending c: a strict comparison keeps the lowest index
      const float v = (float)z[c];
      if (v > best || bi == INT_MAX) { best = v; bi = c; }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const float ov = __shfl_xor(best, off, 64);
    const int oi = __shfl_xor(bi, off, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  if (lane == 0) hits[wave] = (m < B && bi == y[m]) ? 1 : 0;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.x] = (hits[0] + hits[1]) + (hits[2] + hits[3]);
}

// out = (accumulate ? out : 0) + sum(partials[0..n)), one block, fixed order
__global__ __launch_bounds__(256) void sum_counts_kernel(const int32_t* __restrict__ partials, int n, int accumulate,
                                                         long long* __restrict__ out) {
  __shared__ long long red[256];
  long long acc = 0;
  for (int i = threadIdx.x; i < n; i += 256) acc += partials[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = (accumulate ? out[0] : 0) + red[0];
}

constexpr int kMaxDevices = 64;
int32_t* g_static_ptr[kMaxDevices];      // device address of `scratch` on each device, filled on first use
std::mutex g_static_mu;

}  // namespace

int count_partials(int batch) { return (batch + 3) / 4; }

hipError_t launch_count_correct(int dtype, const void* logits, const int32_t* y, int batch, int classes, int32_t* partials,
                                int accumulate, long long* out, hipStream_t s) {
  const int blocks = count_partials(batch);
  if (dtype == 1) count_correct_kernel<bf16><<<blocks, 256, 0, s>>>((const bf16*)logits, y, batch, classes, partials);
  else count_correct_kernel<float><<<blocks, 256, 0, s>>>((const float*)logits, y, batch, classes, partials);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  sum_counts_kernel<<<1, 256, 0, s>>>(partials, blocks, accumulate, out);
  return hipGetLastError();
}

// Device address of the static partial-count array on the current device.  The symbol is looked up once per
// device (each GPU holds its own copy at its own address); no memory is allocated.
hipError_t count_static_scratch(int32_t** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    int32_t* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *ptr = g_static_ptr[dev];
  return hipSuccess;
}

}  // namespace slp
