// Seeded synthetic intermediate labels (paper Sec. 2, Eq. 1), the noisy label
// inputs of interior segments in the simultaneous variant (Sec. 2) and initial
// weights, all from one counter-based generator: Philox4x32-10 (Salmon et al.,
// SC'11) with key = seed and one counter per element, so that every value is a
// pure function of its coordinates and any launch shape gives the same bits.
//
// Counter convention:   labels   (i, class, 0, 0)
//                       weights  (in, out, 1, layer), bias at in = fan_in
//                       noise    (i, n_lo, 2, n_hi),  n = global sample index
//
// The float transforms are written as individually rounded IEEE float32
// operations (this file is compiled with floating-point contraction off, and the
// explicitly rounded intrinsics are used where a product feeds a sum) so that a
// CPU evaluating the same sequence gets the same bits.
#include "slp_kernels.h"

namespace slp {
namespace {

struct Words { uint32_t r0, r1, r2, r3; };

__device__ __forceinline__ Words philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
  for (int round = 0; round < 10; ++round) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
    k0 += 0x9E3779B9u;   // Weyl sequence; the bump after the last round is unused
    k1 += 0xBB67AE85u;
  }
  return Words{c0, c1, c2, c3};
}

// IEEE square root: the plain builtin is lowered to the correctly rounded sequence
// (this file is built with -fhip-fp32-correctly-rounded-divide-sqrt); the
// "__fsqrt_rn" spelling maps to the 1-ulp native instruction and must not be used.
__device__ __forceinline__ float correctly_rounded_sqrt(float x) { return __builtin_sqrtf(x); }

__device__ __forceinline__ float unit_uniform(uint32_t r) {   // (r >> 8) * 2^-24, exact
  return __fmul_rn((float)(r >> 8), 0x1p-24f);
}

// ln(u) for u = j * 2^-24, j in [1, 2^24]: mantissa/exponent split on the bit
// pattern, atanh series in s = (m-1)/(m+1) to s^9, Horner with separately rounded
// multiplies and adds; exponent contribution split into a high and a low part.
__device__ __forceinline__ float ln_unit(float u) {
  const uint32_t bits = __float_as_uint(u);
  int e = (int)(bits >> 23) - 127;
  float m = __uint_as_float((bits & 0x007FFFFFu) | 0x3F800000u);
  if (m > __uint_as_float(0x3FB504F3u)) { m = __fmul_rn(m, 0.5f); e += 1; }
  const float s = __fdiv_rn(__fsub_rn(m, 1.0f), __fadd_rn(m, 1.0f));
  const float s2 = __fmul_rn(s, s);
  float p = __fadd_rn(__fmul_rn(s2, __uint_as_float(0x3E638E39u)), __uint_as_float(0x3E924925u));   // 2/9, 2/7
  p = __fadd_rn(__fmul_rn(p, s2), __uint_as_float(0x3ECCCCCDu));                                     // 2/5
  p = __fadd_rn(__fmul_rn(p, s2), __uint_as_float(0x3F2AAAABu));                                     // 2/3
  const float lnm = __fadd_rn(__fmul_rn(s, 2.0f), __fmul_rn(__fmul_rn(s, s2), p));
  const float ef = (float)e;
  return __fadd_rn(__fmul_rn(ef, __uint_as_float(0x3F317200u)),
                   __fadd_rn(__fmul_rn(ef, __uint_as_float(0x35BFBE8Eu)), lnm));
}

// cos(2 pi k / 2^24) for a 24-bit k: exact quadrant and reflection in integers,
// then Taylor polynomials of sin and cos on [0, pi/4].
__device__ __forceinline__ float cos_turn(uint32_t k) {
  const uint32_t q = k >> 22, fi = k & 0x3FFFFFu;
  const bool swap = fi > (1u << 21);
  const uint32_t ti = swap ? (1u << 22) - fi : fi;
  const float x = __fmul_rn(__fmul_rn((float)ti, 0x1p-22f), __uint_as_float(0x3FC90FDBu));
  const float x2 = __fmul_rn(x, x);
  float sp = __fadd_rn(__fmul_rn(x2, __uint_as_float(0x3638EF1Du)), __uint_as_float(0xB9500D01u));
  sp = __fadd_rn(__fmul_rn(sp, x2), __uint_as_float(0x3C088889u));
  sp = __fadd_rn(__fmul_rn(sp, x2), __uint_as_float(0xBE2AAAABu));
  const float sinx = __fadd_rn(x, __fmul_rn(__fmul_rn(x, x2), sp));
  float cp = __fadd_rn(__fmul_rn(x2, __uint_as_float(0xB493F27Eu)), __uint_as_float(0x37D00D01u));
  cp = __fadd_rn(__fmul_rn(cp, x2), __uint_as_float(0xBAB60B61u));
  cp = __fadd_rn(__fmul_rn(cp, x2), __uint_as_float(0x3D2AAAABu));
  cp = __fadd_rn(__fmul_rn(cp, x2), -0.5f);
  const float cosx = __fadd_rn(1.0f, __fmul_rn(x2, cp));
  const float cf = swap ? sinx : cosx, sf = swap ? cosx : sinx;
  return q == 0 ? cf : (q == 1 ? -sf : (q == 2 ? -cf : sf));
}

__device__ __forceinline__ float standard_normal(uint32_t r0, uint32_t r1) {
  const float u1 = __fmul_rn((float)((r0 >> 8) + 1u), 0x1p-24f);
  const float radius = correctly_rounded_sqrt(__fmul_rn(-2.0f, ln_unit(u1)));
  return __fmul_rn(radius, cos_turn(r1 >> 8));
}

__device__ __forceinline__ float draw(int dist, float kappa, const Words& w) {
  switch (dist) {
    case 0: return __fmul_rn(kappa, unit_uniform(w.r0));
    case 1: return __fsub_rn(__fmul_rn(2.0f, unit_uniform(w.r0)), 1.0f);
    case 2: return standard_normal(w.r0, w.r1);
    default: return (w.r0 >> 31) ? 1.0f : -1.0f;
  }
}

__device__ __forceinline__ uint16_t bf16_bits_rne(float x) {
  const uint32_t b = __float_as_uint(x);
  if ((b & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((b >> 16) | 0x40u);   // quiet NaN
  return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ void store_value(void* out, size_t idx, float v, int dt) {
  if (dt == 1) ((uint16_t*)out)[idx] = bf16_bits_rne(v);
  else ((float*)out)[idx] = v;
}

__global__ void labels_kernel(uint32_t k0, uint32_t k1, int classes, int dim, int dist, float kappa, void* out, int dt) {
  const size_t total = (size_t)classes * dim;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const uint32_t j = (uint32_t)(e / dim), i = (uint32_t)(e % dim);
    store_value(out, e, draw(dist, kappa, philox4x32_10(i, j, 0u, 0u, k0, k1)), dt);
  }
}

__global__ void inputs_kernel(uint32_t k0, uint32_t k1, const float* __restrict__ table, int classes,
                              const int32_t* __restrict__ y, uint64_t first, int batch, int dim, float sigma, void* out, int dt) {
  const size_t total = (size_t)batch * dim;
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const uint32_t row = (uint32_t)(e / dim), i = (uint32_t)(e % dim);
    const uint64_t n = first + row;
    const Words w = philox4x32_10(i, (uint32_t)n, 2u, (uint32_t)(n >> 32), k0, k1);
    const float z = standard_normal(w.r0, w.r1);
    const int cls = min(max(y[row], 0), classes - 1);
    const float v = __fadd_rn(table[(size_t)cls * dim + i], __fmul_rn(sigma, z));
    store_value(out, e, v, dt);
  }
}

__global__ void init_kernel(uint32_t k0, uint32_t k1, uint32_t layer, float* W, int N, int K, int ldk, float* b) {
  const float bound = __fdiv_rn(1.0f, correctly_rounded_sqrt((float)K));
  const size_t total = (size_t)N * (K + 1);
  for (size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (size_t)gridDim.x * blockDim.x) {
    const uint32_t o = (uint32_t)(e / (K + 1)), k = (uint32_t)(e % (K + 1));
    const Words w = philox4x32_10(k, o, 1u, layer, k0, k1);
    const float v = __fmul_rn(__fsub_rn(__fmul_rn(2.0f, unit_uniform(w.r0)), 1.0f), bound);
    if ((int)k < K) W[(size_t)o * ldk + k] = v;
    else b[o] = v;
  }
}

inline int grid_for(size_t total) {
  size_t blocks = (total + 255) / 256;
  return (int)(blocks < 1 ? 1 : (blocks > 65536 ? 65536 : blocks));
}

}  // namespace

hipError_t launch_make_labels(uint64_t seed, int classes, int dim, int dist, float kappa, void* out, int dt,
                              hipStream_t s) {
  labels_kernel<<<grid_for((size_t)classes * dim), 256, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), classes, dim,
                                                                 dist, kappa, out, dt);
  return hipGetLastError();
}

hipError_t launch_make_inputs(uint64_t seed, const float* table, int classes, const int32_t* y, int64_t first_sample,
                              int batch, int dim, float sigma, void* out, int dt, hipStream_t s) {
  inputs_kernel<<<grid_for((size_t)batch * dim), 256, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), table, classes, y,
                                                              (uint64_t)first_sample, batch, dim, sigma, out, dt);
  return hipGetLastError();
}

hipError_t launch_init_weights(uint64_t seed, int layer, float* W32, int N, int K, int ldk, float* b, hipStream_t s) {
  init_kernel<<<grid_for((size_t)N * (K + 1)), 256, 0, s>>>((uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)layer,
                                                            W32, N, K, ldk, b);
  return hipGetLastError();
}

}  // namespace slp
