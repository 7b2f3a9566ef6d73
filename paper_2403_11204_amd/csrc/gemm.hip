// The three dense contractions of a segment step -- forward Z = A W^T (+bias, ReLU),
// data gradient dA = dZ W (masked by the ReLU of the layer below) and weight
// gradient dW = dZ^T A (paper Sec. 2-3: fully connected layers trained by
// backpropagation inside one segment) -- all run through ONE kernel family:
//
//     C[m][n] = sum_k A[m][k] * B[n][k]          ("NT": both operands k-contiguous)
//
// The producers lay their outputs out so that every product is NT: the forward and
// data-gradient epilogues store their result both row-major and transposed, and the
// update kernel keeps a transposed copy of the weights.  That way the inner loop is
// the same, best-case one for all three: 16-byte global loads, 16-byte LDS reads,
// no transposition on the operand path.
//
// gfx950 mapping
//   * 256 threads = 4 wavefronts in a 2x2 grid; a wavefront owns a (BM/2)x(BN/2)
//     sub-tile as MIxNI MFMA 32x32 blocks, accumulators in registers (AGPRs).
//   * bf16: v_mfma_f32_32x32x16_bf16, one per 16-byte chunk pair; float32:
//     v_mfma_f32_32x32x2_f32, four per 16-byte chunk pair.  A k-tile is 128 bytes
//     per row for both types (64 bf16 / 32 float), so loads, LDS layout and
//     addressing are byte-identical for the two types.
//   * global -> registers with buffer loads (out-of-range rows and k-tail chunks read
//     as zero through the resource's range check), registers -> LDS, double buffered:
//     tile k+1 is in flight while tile k is multiplied; one barrier per k-tile.
//   * LDS rows are 128 bytes; the 16-byte chunk index is XOR-ed with (row & 7) so the
//     8 lanes served together by a ds_read_b128 / ds_write_b128 hit 8 different bank
//     groups.
//   * workgroup -> tile: consecutive workgroup ids go round-robin over the 8 XCDs, so
//     ids are first regrouped per XCD (each XCD gets a contiguous range of tiles and
//     its own L2 sees a compact set of operand rows), then walked in column-major
//     groups of 8 tile-rows.
#include "slp_kernels.h"

namespace slp {
namespace {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr uint32_t kOutOfRange = 0x80000000u;   // byte offset beyond any operand (sizes are checked < 2 GiB)
constexpr int kXcds = 8;
constexpr int kGroupM = 8;

template <typename T> struct Chunk;
template <> struct Chunk<bf16> { static constexpr int elems = 8; };
template <> struct Chunk<float> { static constexpr int elems = 4; };

__device__ __forceinline__ void mma_chunk(f32x16& acc, const u32x4& a, const u32x4& b, bf16*) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_chunk(f32x16& acc, const u32x4& a, const u32x4& b, float*) {
  const f32x4 af = __builtin_bit_cast(f32x4, a), bfv = __builtin_bit_cast(f32x4, b);
#pragma unroll
  for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[q], bfv[q], acc, 0, 0, 0);
}

template <typename T> struct Vec4;
template <> struct Vec4<bf16> { typedef bf16x4 type; };
template <> struct Vec4<float> { typedef f32x4 type; };

template <typename T, int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int ES = sizeof(T);
  constexpr int CH = Chunk<T>::elems;        // elements per 16-byte chunk
  constexpr int BK = 128 / ES;               // k elements per tile
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  constexpr int LA = BM / 32, LB = BN / 32;  // 16-byte loads per thread per k-tile
  constexpr int WTM = BM / 2, WTN = BN / 2, MI = WTM / 32, NI = WTN / 32;

  // ---- workgroup -> tile ------------------------------------------------------------
  const int tilesM = (g.M + BM - 1) / BM, tilesN = (g.N + BN - 1) / BN;
  const int total = tilesM * tilesN;
  int tid;
  {
    const int pid = blockIdx.x, xcd = pid % kXcds, q = pid / kXcds;
    const int base = total / kXcds, rem = total % kXcds;
    tid = xcd * base + (xcd < rem ? xcd : rem) + q;
  }
  const int width = kGroupM * tilesN;
  const int group = tid / width, first_m = group * kGroupM;
  const int gsz = (tilesM - first_m) < kGroupM ? (tilesM - first_m) : kGroupM;
  const int tm = first_m + (tid % width) % gsz, tn = (tid % width) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wm = w & 1, wn = w >> 1;
  const int half = lane >> 5, l32 = lane & 31;

  // ---- global load addressing --------------------------------------------------------
  const int kc = t & 7, lrow = t >> 3;       // chunk column and first row handled by this thread
  const int Kr = (g.K + CH - 1) / CH * CH;   // chunk-granular contraction length
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.A), 0, (int)((size_t)g.M * g.lda * ES), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.B), 0, (int)((size_t)g.N * g.ldb * ES), 0x00020000);
  uint32_t voffA[LA], voffB[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) voffA[i] = (uint32_t)(((size_t)(m0 + lrow + 32 * i) * g.lda + kc * CH) * ES);
#pragma unroll
  for (int i = 0; i < LB; ++i) voffB[i] = (uint32_t)(((size_t)(n0 + lrow + 32 * i) * g.ldb + kc * CH) * ES);
  // rows past the end give offsets >= the resource size and read as zero
  const uint32_t lds_wr = (uint32_t)(lrow * 128 + ((kc ^ (lrow & 7)) << 4));

  u32x4 ga[LA], gb[LB];
  auto load_global = [&](int kt) {
    const bool in_k = kt * BK + kc * CH < Kr;
    const uint32_t koff = (uint32_t)kt * 128u;
#pragma unroll
    for (int i = 0; i < LA; ++i)
      ga[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcA, in_k ? voffA[i] + koff : kOutOfRange, 0, 0);
#pragma unroll
    for (int i = 0; i < LB; ++i)
      gb[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrcB, in_k ? voffB[i] + koff : kOutOfRange, 0, 0);
  };
  auto store_lds = [&](int stage) {
    unsigned char* base = smem + stage * STAGE + lds_wr;
#pragma unroll
    for (int i = 0; i < LA; ++i) *(u32x4*)(base + i * 32 * 128) = ga[i];
#pragma unroll
    for (int i = 0; i < LB; ++i) *(u32x4*)(base + A_BYTES + i * 32 * 128) = gb[i];
  };

  // ---- fragment addressing -------------------------------------------------------------
  const uint32_t fragA = (uint32_t)((wm * WTM + l32) * 128);
  const uint32_t fragB = (uint32_t)(A_BYTES + (wn * WTN + l32) * 128);
  uint32_t xo[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) xo[kk] = (uint32_t)(((kk * 2 + half) ^ (lane & 7)) << 4);

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  auto compute = [&](int stage) {
    const unsigned char* sb = smem + stage * STAGE;
    u32x4 af[2][MI], bfr[2][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = *(const u32x4*)(sb + fragA + i * 32 * 128 + xo[0]);
#pragma unroll
    for (int j = 0; j < NI; ++j) bfr[0][j] = *(const u32x4*)(sb + fragB + j * 32 * 128 + xo[0]);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk < 3) {
#pragma unroll
        for (int i = 0; i < MI; ++i) af[nxt][i] = *(const u32x4*)(sb + fragA + i * 32 * 128 + xo[kk + 1]);
#pragma unroll
        for (int j = 0; j < NI; ++j) bfr[nxt][j] = *(const u32x4*)(sb + fragB + j * 32 * 128 + xo[kk + 1]);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) mma_chunk(acc[i][j], af[cur][i], bfr[cur][j], (T*)nullptr);
    }
  };

  // ---- main loop: double-buffered LDS, next tile's global loads in flight ------------
  const int nk = (Kr + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_global(kt + 1);
    compute(cur);
    if (kt + 1 < nk) store_lds(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue ----------------------------------------------------------------------------
  // Accumulator layout of the 32x32 MFMA: lane holds column n = lane & 31 and, in
  // register r, row 8*(r/4) + 4*(lane/32) + (r%4): four consecutive rows per register
  // quad, which is what makes the transposed store a vector store.
  const int M8 = (g.M + 7) & ~7;
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int n = n0 + wn * WTN + j * 32 + l32;
    if (n >= g.N) continue;
    float bias = 0.0f;
    if (EPI == EPI_FWD) bias = g.bias[n];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int mb = m0 + wm * WTM + i * 32 + 8 * q + 4 * half;   // rows mb .. mb+3
        if (EPI == EPI_WGRAD) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (mb + e < g.M) g.Cf[(size_t)(mb + e) * g.ldc + n] = acc[i][j][4 * q + e];
        } else {
          if (mb >= M8) continue;
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
          if (EPI == EPI_FWD) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              v[e] += bias;
              if (g.relu) v[e] = fmaxf(v[e], 0.0f);
            }
          } else {
            typedef typename Vec4<T>::type mvec_t;
            const mvec_t mk = *(const mvec_t*)((const T*)g.maskT + (size_t)n * g.ldmask + mb);
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (!((float)mk[e] > 0.0f)) v[e] = 0.0f;
          }
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (mb + e >= g.M) v[e] = 0.0f;
          if (g.C) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (mb + e < g.M) ((T*)g.C)[(size_t)(mb + e) * g.ldc + n] = (T)v[e];
          }
          if (g.CT) {
            typename Vec4<T>::type o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (T)v[e];
            *(typename Vec4<T>::type*)((T*)g.CT + (size_t)n * g.ldct + mb) = o;
          }
        }
        // keep the scheduler from hoisting every block's address arithmetic and mask
        // loads to the top of the epilogue (that spills registers)
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
}

// ---- host side -------------------------------------------------------------------------------
struct TileCfg { int bm, bn; const char* name; };
const TileCfg kCfgs[3] = {{256, 256, "256x256"}, {128, 128, "128x128"}, {64, 64, "64x64"}};

int pick_cfg(int M, int N) {
  // largest tile that still gives every compute unit (256 of them) work
  for (int c = 0; c < 3; ++c) {
    const long tiles = (long)((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
    if (tiles >= 224) return c;
  }
  return 2;
}

template <typename T, int BM, int BN, int EPI>
hipError_t launch_one(const GemmArgs& g, hipStream_t s) {
  constexpr int smem = 2 * (BM + BN) * 128;
  static bool configured = false;   // one attribute call per instantiation
  auto kern = gemm_nt_kernel<T, BM, BN, EPI>;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(256), smem, s, g);
  return hipGetLastError();
}

template <typename T, int EPI>
hipError_t launch_cfg(int cfg, const GemmArgs& g, hipStream_t s) {
  switch (cfg) {
    case 0: return launch_one<T, 256, 256, EPI>(g, s);
    case 1: return launch_one<T, 128, 128, EPI>(g, s);
    default: return launch_one<T, 64, 64, EPI>(g, s);
  }
}

template <typename T>
hipError_t launch_epi(int epi, int cfg, const GemmArgs& g, hipStream_t s) {
  switch (epi) {
    case EPI_FWD: return launch_cfg<T, EPI_FWD>(cfg, g, s);
    case EPI_DGRAD: return launch_cfg<T, EPI_DGRAD>(cfg, g, s);
    default: return launch_cfg<T, EPI_WGRAD>(cfg, g, s);
  }
}

}  // namespace

const char* gemm_config_name(int dtype, int M, int N, int K) {
  (void)dtype; (void)K;
  return kCfgs[pick_cfg(M, N)].name;
}

hipError_t launch_gemm(int dtype, int epi, const GemmArgs& g, hipStream_t s) {
  const int es = dtype == 1 ? 2 : 4;
  // the kernel addresses operands with 32-bit byte offsets and a 2 GiB sentinel
  if ((size_t)g.M * g.lda * es >= 0x80000000ull || (size_t)g.N * g.ldb * es >= 0x80000000ull) return hipErrorInvalidValue;
  if (g.lda % kLdAlign || g.ldb % kLdAlign || g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (((uintptr_t)g.A | (uintptr_t)g.B) & 15) return hipErrorInvalidValue;
  const int cfg = pick_cfg(g.M, g.N);
  return dtype == 1 ? launch_epi<bf16>(epi, cfg, g, s) : launch_epi<float>(epi, cfg, g, s);
}

}  // namespace slp
