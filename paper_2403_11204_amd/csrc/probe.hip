// Matrix-pipe issue probe: the same MFMA instructions, accumulator count and occupancy as the
// 256x256 product kernels (8 wavefronts per workgroup, one workgroup per compute unit, 128
// accumulator registers per lane in independent blocks), but with operands that never leave
// registers -- no LDS, no global loads, no barriers.  Its rate is what the chip sustains on
// this instruction mix under its power limit, which is the ceiling the product kernel can be
// compared with next to the published peak (the clock drops under sustained MFMA load, and
// by how much depends on how the operand bits toggle, so the operands are pseudo-random
// values of mixed sign and a few exponents, not constants).
#include "../../include/slp.h"
#include "slp_kernels.h"

namespace slp {
namespace {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// two bf16 values per word: random sign, exponent in [2^-3, 2^0], random mantissa
__device__ __forceinline__ uint32_t two_bf16(uint32_t h) {
  const uint32_t lo = ((h & 1u) << 15) | ((124u + ((h >> 1) & 3u)) << 7) | ((h >> 3) & 127u);
  const uint32_t hi = (((h >> 10) & 1u) << 15) | ((124u + ((h >> 11) & 3u)) << 7) | ((h >> 13) & 127u);
  return lo | (hi << 16);
}
__device__ __forceinline__ float one_f32(uint32_t h) {
  return __builtin_bit_cast(float, ((h & 1u) << 31) | ((124u + ((h >> 1) & 3u)) << 23) | ((h >> 3) & 0x7fffffu));
}

typedef __attribute__((ext_vector_type(4))) float f32x4;

// bf16: 8 x 4 blocks of v_mfma_f32_16x16x32_bf16 per wavefront (the 128 x 64 sub-tile of the big product kernel),
// float32: 4 x 2 blocks of v_mfma_f32_32x32x2_f32 (the generic kernel's); 128 accumulator registers either way.
template <int DT>
__global__ __launch_bounds__(512) void mfma_issue_kernel(int iters, float* sink) {
  const uint32_t id = blockIdx.x * 512u + threadIdx.x;
  constexpr int NA = DT == SLP_BF16 ? 8 : 4, NB = DT == SLP_BF16 ? 4 : 2;
  // two operand sets (NA "A" and NB "B" fragments each), alternated so that operand lines toggle
  u32x4 a[2][NA], b[2][NB];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t h = mix(id * 128u + s * 64u + i * 4u + q + 1u);
        a[s][i][q] = DT == SLP_BF16 ? two_bf16(h) : __builtin_bit_cast(uint32_t, one_f32(h));
      }
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint32_t h = mix(id * 128u + s * 64u + 32u + j * 4u + q + 1u);
        b[s][j][q] = DT == SLP_BF16 ? two_bf16(h) : __builtin_bit_cast(uint32_t, one_f32(h));
      }
  }
  float t = 0.0f;
  if constexpr (DT == SLP_BF16) {
    f32x4 acc[NA * NB];
#pragma unroll
    for (int i = 0; i < NA * NB; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
            acc[i * NB + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[s][i]),
                                                                      __builtin_bit_cast(bf16x8, b[s][j]), acc[i * NB + j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NA * NB; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) t += acc[i][r];
  } else {
    f32x16 acc[NA * NB];
#pragma unroll
    for (int i = 0; i < NA * NB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int i = 0; i < NA; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q)
              acc[i * NB + j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__builtin_bit_cast(float, a[s][i][q]),
                                                                     __builtin_bit_cast(float, b[s][j][q]), acc[i * NB + j], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < NA * NB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[i][r];
  }
  sink[id] = t;
}

}  // namespace

// Launches the probe on `grid` workgroups of 512 threads; sink must hold grid*512 floats.
// flops_per_workgroup_iter: algorithmic FLOPs one workgroup issues per loop iteration.
hipError_t launch_mfma_probe(int dtype, int iters, int grid, float* sink, double* flops_per_workgroup_iter, hipStream_t s) {
  // 8 wavefronts x (bf16: 64 MFMAs of 2*16*16*32 FLOPs; float32: 16 groups of four 32x32x2) per iteration
  *flops_per_workgroup_iter = 8.0 * (dtype == SLP_BF16 ? 64 * 2.0 * 16 * 16 * 32 : 16 * 4 * 2.0 * 32 * 32 * 2);
  if (dtype == SLP_BF16) hipLaunchKernelGGL(mfma_issue_kernel<SLP_BF16>, dim3(grid), dim3(512), 0, s, iters, sink);
  else hipLaunchKernelGGL(mfma_issue_kernel<SLP_F32>, dim3(grid), dim3(512), 0, s, iters, sink);
  return hipGetLastError();
}

}  // namespace slp
