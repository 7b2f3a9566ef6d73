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
//   * bf16: v_mfma_f32_16x16x32_bf16 (16x16 blocks; a register-only loop of it sustains 2000-2100 TFLOP/s under the
//     chip's power limit, the 32x32x16 form 1800-1850); float32: v_mfma_f32_32x32x2_f32, four per 16-byte chunk pair.
//     A k-tile is 128 bytes per row for both types (64 bf16 / 32 float), so loads, LDS layout and addressing
//     are byte-identical for the two types.
//   * global -> LDS directly (buffer_load_dwordx4 ... lds): no staging registers and no ds_write instructions.
//     Out-of-range rows and k-tail chunks read as zero through the buffer resource's range check, so ragged
//     M, N and K need no branches.
//   * LDS rows are 128 bytes and the LDS has 64 banks x 4 bytes: a ds_read_b128 is served 16 lanes at a time,
//     i.e. 16 consecutive rows of one k-chunk.  Physical chunk = chunk ^ ((row >> 1) & 7) spreads those 16 rows
//     over all 64 banks (no conflicts counted).  The hardware writes lane l of an LDS-direct load at
//     base + 16 l, so the swizzle is applied on the global side: each lane fetches the chunk that belongs at its
//     physical position.
//   * big products (256x256 tile, bf16): gemm_nt_big_kernel, 8 wavefronts of 128x64, two LDS stages of 64 KB,
//     the loads of a k-tile issued evenly over the whole k-tile (two barriers per k-tile free the stage piecewise);
//     see the comment on that kernel.
//   * everything else (float32, smaller tiles): gemm_nt_kernel, NW wavefronts in a 2 x NW/2 grid, a wavefront
//     owns a (BM/2) x (BN/(NW/2)) sub-tile; NS LDS stages of (BM+BN) x 128 bytes (two for the 256x256 tile, four
//     for the small ones); one barrier per k-tile, after which the loads of tile k+NS are issued; a k-tile is 4
//     pipeline units, the fragments of unit u+1 are read from LDS while unit u multiplies.
//   * in both kernels the source order "a few LDS reads / loads, a few MFMAs" is pinned with scheduling fences,
//     because the compiler's own schedule serialises LDS latency with the matrix pipe.
//   * epilogue: a lane holds 4 consecutive rows of one output column per accumulator register quad, which
//     is one vector store into the transposed output; for the row-major output the quad of lanes holding
//     4 adjacent columns transposes its 4x4 block with DPP moves, after which a lane holds 4 consecutive
//     columns of one row: one vector store as well (2 stores per quad instead of 5).
//     The big kernel's bf16 outputs go through LDS instead and leave as whole 128- and 256-byte row segments
//     (see its epilogue).
//   * workgroup -> tile: consecutive workgroup ids go round-robin over the 8 XCDs, so
//     ids are first regrouped per XCD (each XCD gets a contiguous range of tiles and
//     its own 4 MB L2 sees a compact set of operand rows), then walked in column-major groups of 8 tile-rows.
//     Big products whose tile grid divides into 16 x 16 regions are walked region by region instead, all 8 XCDs
//     inside one region at a time (see the kernel).
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
constexpr int kRegionWalk = -1;   // GemmArgs::group_m value: walk 16 x 16 regions of tiles (big kernel only)

template <typename T> struct Chunk;
template <> struct Chunk<bf16> { static constexpr int elems = 8; };
template <> struct Chunk<float> { static constexpr int elems = 4; };

// 32x32 block forms (one 16-byte chunk pair per call), used by the contraction-split kernel for small products
__device__ __forceinline__ void mma_chunk(f32x16& acc, const u32x4& a, const u32x4& b, bf16*) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_chunk(f32x16& acc, const u32x4& a, const u32x4& b, float*) {
  const f32x4 af = __builtin_bit_cast(f32x4, a), bfv = __builtin_bit_cast(f32x4, b);
#pragma unroll
  for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[q], bfv[q], acc, 0, 0, 0);
}

// MFMA geometry per element type.  bf16: v_mfma_f32_16x16x32_bf16 (a 16x16 block over 32 k = 4 chunks per row; the
// block's 4 accumulator registers hold rows 4*(lane/16)..+3 of column lane%16); float32: v_mfma_f32_32x32x2_f32, four
// per chunk pair.  MB = block edge, AH = parts the A fragments of one k-sub-step are read in (pipeline units).
template <typename T> struct Mma;
template <> struct Mma<bf16> {
  static constexpr int MB = 16, AH = 2, ACC = 4;
  typedef f32x4 acc_t;
  static __device__ __forceinline__ void mma(acc_t& acc, const u32x4& a, const u32x4& b) {
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
  }
};
template <> struct Mma<float> {
  static constexpr int MB = 32, AH = 1, ACC = 16;
  typedef f32x16 acc_t;
  static __device__ __forceinline__ void mma(acc_t& acc, const u32x4& a, const u32x4& b) {
    const f32x4 af = __builtin_bit_cast(f32x4, a), bfv = __builtin_bit_cast(f32x4, b);
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(af[q], bfv[q], acc, 0, 0, 0);
  }
};

template <typename T> struct Vec4;
template <> struct Vec4<bf16> { typedef bf16x4 type; };
template <> struct Vec4<float> { typedef f32x4 type; };

// 4x4 transpose across the 4 lanes of a quad (lanes 4g..4g+3): on return, lane i holds in v[j] what lane j held
// in v[i].  Two butterfly stages of quad-permute DPP moves; every lane of the quad must be active.
__device__ __forceinline__ float quad_xor(float x, bool by_two) {
  const int xi = __builtin_bit_cast(int, x);
  const int r = by_two ? __builtin_amdgcn_update_dpp(0, xi, 0x4E, 0xF, 0xF, true)      // lanes [2,3,0,1]
                       : __builtin_amdgcn_update_dpp(0, xi, 0xB1, 0xF, 0xF, true);     // lanes [1,0,3,2]
  return __builtin_bit_cast(float, r);
}
__device__ __forceinline__ void quad_transpose(float (&v)[4], int lane) {
  const bool b0 = lane & 1, b1 = lane & 2;
  float r;
  r = quad_xor(b0 ? v[0] : v[1], false); if (b0) v[0] = r; else v[1] = r;
  r = quad_xor(b0 ? v[2] : v[3], false); if (b0) v[2] = r; else v[3] = r;
  r = quad_xor(b1 ? v[0] : v[2], true);  if (b1) v[0] = r; else v[2] = r;
  r = quad_xor(b1 ? v[1] : v[3], true);  if (b1) v[1] = r; else v[3] = r;
}

// Epilogue of one accumulator register quad: rows mb..mb+3 of output column n, v[e] = row mb+e.  The 4 lanes of
// a quad hold 4 consecutive columns (n - lane%4 is a multiple of 4), and a lane whose column is past N takes part
// with zeros: nothing here may diverge inside a quad before the transpose.
//   EPI_FWD  : + bias (the caller passes 0 for a column past N), optional ReLU;
//   EPI_DGRAD: zero where the mask (stored transposed) is not positive;
//   both store transposed CT in T as one vector per lane (4 rows of its column; rows past M up to the next
//   multiple of 8 are written as zero) and row-major C after a 4x4 transpose inside the quad, so that a lane
//   stores 4 consecutive columns of one row as one vector (pad columns up to the leading dimension receive
//   zeros);  EPI_WGRAD: float32 row-major, same transposed vector store.
template <typename T, int EPI>
__device__ __forceinline__ void store_quad(const GemmArgs& g, int n, int mb, float bias, float (&v)[4], int lane) {
  typedef __attribute__((ext_vector_type(4))) float f32x4_t;
  const bool col_ok = n < g.N;
  const int row = mb + (lane & 3), nb = n - (lane & 3);      // after the transpose: this lane's row, first of its 4 columns
  if (EPI == EPI_WGRAD) {
    quad_transpose(v, lane);
    if (row < g.M && nb < g.N) *(f32x4_t*)(g.Cf + (size_t)row * g.ldc + nb) = f32x4_t{v[0], v[1], v[2], v[3]};
    return;
  }
  if (EPI == EPI_WGRAD_UPDATE) {
    // The optimiser step on the 4 consecutive weights of one output row this lane holds after the transpose
    // (pad columns hold zeros in every stream and stay zero); then back through the transpose, so that the lane
    // holds 4 consecutive output rows of one input column: one vector store into the transposed copy.
    quad_transpose(v, lane);
    const bool in = row < g.M && nb < g.N;
    float w[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (in) {
      const size_t idx = (size_t)row * g.ldc + nb;
      const f32x4_t w4 = *(const f32x4_t*)(g.uW + idx);
      f32x4_t vel = f32x4_t{v[0], v[1], v[2], v[3]};
      if (g.mu != 0.0f) {
        vel = g.mu * *(const f32x4_t*)(g.uV + idx) + vel;
        *(f32x4_t*)(g.uV + idx) = vel;
      }
      const f32x4_t wn = w4 - g.lr * vel;
      *(f32x4_t*)(g.uW + idx) = wn;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = wn[e];
      if (g.uW16) {
        bf16x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (bf16)w[e];
        *(bf16x4*)((bf16*)g.uW16 + idx) = h;
      }
    }
    if (g.uWT) {      // (uniform over the launch)
      quad_transpose(w, lane);
      if (col_ok && mb < g.M) {     // rows past M inside the vector carry zeros: the pads of the copy stay zero
        typename Vec4<T>::type o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (T)w[e];
        *(typename Vec4<T>::type*)((T*)g.uWT + (size_t)n * g.ldwt + mb) = o;
      }
    }
    return;
  }
  if (mb >= ((g.M + 7) & ~7)) return;       // the same for the whole quad
  if (EPI == EPI_FWD) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[e] += bias;
      if (g.relu) v[e] = fmaxf(v[e], 0.0f);
    }
  } else if (g.maskT && col_ok) {   // no mask: the gradient w.r.t. the segment input
    typedef typename Vec4<T>::type mvec_t;
    const mvec_t mk = *(const mvec_t*)((const T*)g.maskT + (size_t)n * g.ldmask + mb);
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (!((float)mk[e] > 0.0f)) v[e] = 0.0f;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e)
    if (mb + e >= g.M || !col_ok) v[e] = 0.0f;
  if (g.CT && col_ok) {
    typename Vec4<T>::type o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (T)v[e];
    *(typename Vec4<T>::type*)((T*)g.CT + (size_t)n * g.ldct + mb) = o;
  }
  if (g.C) {
    quad_transpose(v, lane);
    if (row < g.M && nb < g.N) {
      typename Vec4<T>::type o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (T)v[e];
      *(typename Vec4<T>::type*)((T*)g.C + (size_t)row * g.ldc + nb) = o;
    }
  }
}

template <typename T, int BM, int BN, int EPI, int NW, int NS>
__global__ __launch_bounds__(NW * 64) void gemm_nt_kernel(const GemmArgs g) {
#if defined(__HIP_DEVICE_COMPILE__)   // LDS-direct builtins exist in the device pass only; the host pass needs just the launch stub
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int ES = sizeof(T);
  constexpr int CH = Chunk<T>::elems;        // elements per 16-byte chunk
  constexpr int BK = 128 / ES;               // k elements per tile
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  constexpr int RPL = 8 * NW;                  // tile rows covered by one load instruction of the whole workgroup
  constexpr int LA = BM / RPL, LB = BN / RPL;  // 16-byte loads per thread per k-tile
  typedef Mma<T> MM;
  constexpr int MB = MM::MB, AH = MM::AH;
  constexpr int CPS = 64 / MB;                 // 16-byte chunks per row that one k-sub-step consumes
  constexpr int KSUB = 8 / CPS;                // k-sub-steps per k-tile
  constexpr int UNITS = KSUB * AH;             // pipeline units per k-tile
  constexpr int WTM = BM / 2, WTN = BN / (NW / 2), MI = WTM / MB, NI = WTN / MB, MIH = MI / AH;
  static_assert(MI % AH == 0 && UNITS % 2 == 0 && KSUB % 2 == 0, "buffer parity must repeat from tile to tile");

  // ---- workgroup -> tile ------------------------------------------------------------
  const int tilesM = (g.M + BM - 1) / BM, tilesN = (g.N + BN - 1) / BN;
  const int total = tilesM * tilesN;
  int tid;
  {
    const int pid = blockIdx.x, xcd = pid % kXcds, q = pid / kXcds;
    const int base = total / kXcds, rem = total % kXcds;
    tid = xcd * base + (xcd < rem ? xcd : rem) + q;
  }
  const int group_m = g.group_m > 0 ? g.group_m : kGroupM;
  const int width = group_m * tilesN;
  const int group = tid / width, first_m = group * group_m;
  const int gsz = (tilesM - first_m) < group_m ? (tilesM - first_m) : group_m;
  const int tm = first_m + (tid % width) % gsz, tn = (tid % width) / gsz;
  const int m0 = tm * BM, n0 = tn * BN;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wm = w & 1, wn = w >> 1;
  const int lgrp = lane / MB, lrow = lane % MB;

  // ---- global load addressing --------------------------------------------------------
  const int Kr = (g.K + CH - 1) / CH * CH;   // chunk-granular contraction length
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.A), 0, (int)((size_t)g.M * g.lda * ES), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.B), 0, (int)((size_t)g.N * g.ldb * ES), 0x00020000);
  // Direct-to-LDS loads: load i of wavefront w fills LDS rows [8w + RPL i, 8w + RPL i + 8) of the tile
  // (RPL = 8 x wavefronts), lane l writing 16 bytes at (row 8w + RPL i + l/8, physical chunk l%8) --
  // the hardware places lane l at base + 16*l.  The XOR swizzle is therefore applied on the global
  // side: the lane fetches the logical chunk that belongs at its physical position.
  const int prow = w * 8 + (lane >> 3);                   // + RPL i
  const int pchunk = (lane & 7) ^ ((prow >> 1) & 7);      // logical k-chunk fetched by this lane
  uint32_t voffA[LA], voffB[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) voffA[i] = (uint32_t)(((size_t)(m0 + prow + RPL * i) * g.lda + pchunk * CH) * ES);
#pragma unroll
  for (int i = 0; i < LB; ++i) voffB[i] = (uint32_t)(((size_t)(n0 + prow + RPL * i) * g.ldb + pchunk * CH) * ES);
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  const uint32_t lds_wave = (uint32_t)__builtin_amdgcn_readfirstlane(w * 8 * 128);
  const int kc = pchunk;

  // ---- fragment addressing -------------------------------------------------------------
  const uint32_t fragA = (uint32_t)((wm * WTM + lrow) * 128);
  const uint32_t fragB = (uint32_t)(A_BYTES + (wn * WTN + lrow) * 128);
  uint32_t xo[KSUB];
#pragma unroll
  for (int kk = 0; kk < KSUB; ++kk) xo[kk] = (uint32_t)(((kk * CPS + lgrp) ^ ((lane >> 1) & 7)) << 4);

  typename MM::acc_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < MM::ACC; ++r) acc[i][j][r] = 0.0f;

  // Pipeline unit u of a k-tile = k-sub-step u / AH, part u % AH of the wavefront's rows: MIH A fragments (buffer u & 1)
  // against the sub-step's NI B fragments (buffer (u / AH) & 1, read together with part 0).
  u32x4 af[2][MIH], bfr[2][NI];
  // Every k-sub-step is written out as small groups "a few loads/stores + a few MFMAs",
  // fenced so that the compiler keeps the interleaving: the matrix pipe always has work
  // queued while LDS and global traffic for later sub-steps is in flight.
  constexpr int NRD = MIH + NI;                              // most fragment reads any unit needs (those with part 0)
  constexpr int NLD = LA + LB;                               // global loads / LDS writes per k-tile
  constexpr int NMM = MIH * NI;                              // MFMA groups per unit
  auto reads_of = [](int u) { return MIH + (u % AH == 0 ? NI : 0); };
  auto read_one = [&](int stage, int u, int r) {             // read r of the fragments unit u multiplies
    const unsigned char* sb = smem + stage * STAGE;
    const int kk = u / AH, h = u % AH;
    if (r < MIH) af[u & 1][r] = *(const u32x4*)(sb + fragA + (h * MIH + r) * MB * 128 + xo[kk]);
    else bfr[kk & 1][r - MIH] = *(const u32x4*)(sb + fragB + (r - MIH) * MB * 128 + xo[kk]);
  };
  auto mma_one = [&](int u, int m) {
    MM::mma(acc[(u % AH) * MIH + m / NI][m % NI], af[u & 1][m / NI], bfr[(u / AH) & 1][m % NI]);
  };
  auto gload_one = [&](int kt, int stage, int i) {
    const bool in_k = kt * BK + kc * CH < Kr;      // past the end of K every load becomes a zero fill
    const uint32_t koff = (uint32_t)kt * 128u;
    if (i < LA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)(smem + stage * STAGE + lds_wave + i * RPL * 128), 16,
                                               in_k ? voffA[i] + koff : kOutOfRange, 0, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)(smem + stage * STAGE + A_BYTES + lds_wave + (i - LA) * RPL * 128), 16,
                                               in_k ? voffB[i - LA] + koff : kOutOfRange, 0, 0, 0);
  };
// s_waitcnt immediate: wait until at most n vector-memory operations are outstanding (other counters untouched)
#define VMCNT(n) ((((n) & 15) | 0x0F70 | (((n) >> 4) << 14)))
#define SLP_FENCE() __builtin_amdgcn_sched_barrier(0)

  const int nk = (Kr + BK - 1) / BK;
#pragma unroll
  for (int st = 0; st < NS; ++st)
#pragma unroll
    for (int i = 0; i < NLD; ++i) gload_one(st, st, i);
  __builtin_amdgcn_s_waitcnt(VMCNT((NS - 1) * NLD));
  __syncthreads();
#pragma unroll
  for (int r = 0; r < NRD; ++r) read_one(0, 0, r);
  auto rd_lo = [](int g, int n) { return 2 * g < n ? 2 * g : n; };
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt % NS, nxt = (kt + 1) % NS;
#pragma unroll
    for (int u = 0; u < UNITS - 1; ++u) {
#pragma unroll
      for (int g = 0; g < NRD; ++g) {
#pragma unroll
        for (int r = rd_lo(g, reads_of(u + 1)); r < rd_lo(g + 1, reads_of(u + 1)); ++r) read_one(cur, u + 1, r);
#pragma unroll
        for (int m = g * NMM / NRD; m < (g + 1) * NMM / NRD; ++m) mma_one(u, m);
        SLP_FENCE();
      }
    }
    // tile kt+1 must have landed in stage nxt (this wave's part), and every wave must be done reading stage cur
    if (NS == 2) {
      __builtin_amdgcn_s_waitcnt(VMCNT(0));
      __syncthreads();
    } else {
      // tiles kt+2 .. kt+NS-1 stay in flight.  A bare barrier between compiler fences: the workgroup release fence
      // of __syncthreads() waits for EVERY outstanding LDS-direct load.  What the barrier has to order is waited for
      // by hand: this wavefront's loads of tile kt+1 (vmcnt) and its LDS reads of stage cur (lgkmcnt 0).
      __builtin_amdgcn_s_waitcnt(VMCNT((NS - 2) * NLD) & 0xF0FF);
      asm volatile("" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
    }
#pragma unroll
    for (int g = 0; g < NRD; ++g) {
#pragma unroll
      for (int r = rd_lo(g, NRD); r < rd_lo(g + 1, NRD); ++r) read_one(nxt, 0, r);
#pragma unroll
      for (int i = g * NLD / NRD; i < (g + 1) * NLD / NRD; ++i) gload_one(kt + NS, cur, i);
#pragma unroll
      for (int m = g * NMM / NRD; m < (g + 1) * NMM / NRD; ++m) mma_one(UNITS - 1, m);
      SLP_FENCE();
    }
  }
  __builtin_amdgcn_s_waitcnt(VMCNT(0));
#undef SLP_FENCE

  // ---- epilogue ----------------------------------------------------------------------------
  // Accumulator layout of an MB x MB block: lane holds column n = lane % MB and, in register r, row
  // (64 / MB * 4) * (r / 4) + 4 * (lane / MB) + (r % 4): four consecutive rows per register quad, which is what
  // makes the transposed store a vector store.
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int n = n0 + wn * WTN + j * MB + lrow;
    float bias = 0.0f;
    if (EPI == EPI_FWD && n < g.N) bias = g.bias[n];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int q = 0; q < MM::ACC / 4; ++q) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
        store_quad<T, EPI>(g, n, m0 + wm * WTM + i * MB + (256 / MB) * q + 4 * lgrp, bias, v, lane);
        // keep the scheduler from hoisting every block's address arithmetic and mask
        // loads to the top of the epilogue (that spills registers)
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
#endif
}

// Big bf16 products: 256x256 tile, NW = 8 wavefronts in a 2 x 4 grid (128 x 64 each; NW = 4, 128 x 128 each with the
// accumulators in AGPRs, is kept compilable: measured equal, but its data-gradient epilogue spills),
// v_mfma_f32_16x16x32_bf16, two LDS stages of 64 KB.
// A k-tile (64 k) is 4 units: (row half h, k-sub-step kk) in the order (0,0) (0,1) (1,0) (1,1), each 4 A fragments
// against the NB B fragments of the sub-step.  The B fragments of a k-tile stay in registers for the whole tile, the A
// fragments are read one unit ahead.  That order frees LDS early: after unit 0 nothing of this stage's B rows and h=0
// A rows is needed any more, after unit 2 the h=1 A rows are free too.  Two barriers per k-tile (X after unit 0, Y
// after unit 2) let the LDS-direct loads of tile kt+2 be issued evenly over the whole k-tile, a quarter of them per
// unit.  Issued in one burst after a single barrier (as gemm_nt_kernel does) they cost the unit that issues them 3x its
// MFMA time: measured per unit with the cycle counter, 570 / 581 / 498 / 1578 cycles against 512 of MFMAs each.
// Sustained on 8192x16384x16384: 1295-1315 -> 1365-1415 TFLOP/s.
// Register budget: 216-222 per lane (allocated as 224), two wavefronts per SIMD; the 64 that remain of the SIMD's 512
// are what the weight-update kernel running beside the products is held to -- above 224 here it no longer fits.
template <int EPI, int NW>
__global__ __launch_bounds__(NW * 64) void gemm_nt_big_kernel(const GemmArgs g) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef bf16 T;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  // highest wave priority: on a compute unit shared with an update workgroup the product's loads are issued first
  // (+0.4 % per step on the comparison configuration; no effect when the kernel runs alone)
  __builtin_amdgcn_s_setprio(3);
  constexpr int BM = 256, BN = 256, ES = 2, CH = 8, BK = 64;
  constexpr int A_BYTES = BM * 128, STAGE = (BM + BN) * 128;
  constexpr int WN = NW / 2;             // wavefront columns
  constexpr int WTN = BN / WN;           // columns per wavefront (128 or 64)
  constexpr int NB = WTN / 16;           // B fragments per sub-step (8 or 4)
  constexpr int RPL = 8 * NW;            // rows one load instruction of the workgroup covers (32 or 64)
  constexpr int NBLK = 256 / RPL;        // row blocks (= loads per lane) per operand per k-tile (8 or 4)
  constexpr int NL = 2 * NBLK;           // loads per lane per k-tile (16 or 8)
  constexpr int LPU = NL / 4;            // loads per unit (4 or 2)
  constexpr int NSLOT = 2 * NB;          // slots of 2 MFMAs per unit (16 or 8)

  const int tilesM = (g.M + BM - 1) / BM, tilesN = (g.N + BN - 1) / BN;
  const int total = tilesM * tilesN;
  int tid;
  {
    const int pid = blockIdx.x, xcd = pid % kXcds, q = pid / kXcds;
    const int base = total / kXcds, rem = total % kXcds;
    tid = xcd * base + (xcd < rem ? xcd : rem) + q;
  }
  const int group_m = g.group_m > 0 ? g.group_m : kGroupM;
  const int width = group_m * tilesN;
  const int group = tid / width, first_m = group * group_m;
  const int gsz = (tilesM - first_m) < group_m ? (tilesM - first_m) : group_m;
  int tm = first_m + (tid % width) % gsz, tn = (tid % width) / gsz;
  if (g.group_m == kRegionWalk) {
    // All 8 XCDs work on one 16 x 16 region of tiles at a time, as 2 x 4 blocks of 8 x 4 tiles (one block per XCD,
    // one tile per compute unit): 32 operand strips feed 256 concurrent tiles, and what one XCD fetched is in the
    // memory-side cache for the XCDs that share its strips.  Regions are walked down the rows first.
    const int pid = blockIdx.x, xcd = pid % kXcds, q = pid / kXcds;
    const int r = q / 32, sl = q % 32, regM = tilesM / 16;
    tm = (r % regM) * 16 + (xcd % 2) * 8 + sl % 8;
    tn = (r / regM) * 16 + (xcd / 2) * 4 + sl / 8;
  }
  const int m0 = tm * BM, n0 = tn * BN;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wm = w & 1, wn = w >> 1;
  const int lgrp = lane >> 4, lrow = lane & 15;

  const int Kr = (g.K + CH - 1) / CH * CH;
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.A), 0, (int)((size_t)g.M * g.lda * ES), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.B), 0, (int)((size_t)g.N * g.ldb * ES), 0x00020000);
  // load i of the workgroup fills rows [RPL i, RPL i + RPL) of an operand's 256; wavefront w rows 8w..8w+7 of those
  const int prow = w * 8 + (lane >> 3);
  const int pchunk = (lane & 7) ^ ((prow >> 1) & 7);
  uint32_t voffA[NBLK], voffB[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i) voffA[i] = (uint32_t)(((size_t)(m0 + prow + RPL * i) * g.lda + pchunk * CH) * ES);
#pragma unroll
  for (int i = 0; i < NBLK; ++i) voffB[i] = (uint32_t)(((size_t)(n0 + prow + RPL * i) * g.ldb + pchunk * CH) * ES);
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  const uint32_t lds_wave = (uint32_t)__builtin_amdgcn_readfirstlane(w * 8 * 128);
  const int kc = pchunk;

  const uint32_t fragA = (uint32_t)((wm * 128 + lrow) * 128);
  const uint32_t fragB = (uint32_t)(A_BYTES + (wn * WTN + lrow) * 128);
  uint32_t xo[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) xo[kk] = (uint32_t)(((kk * 4 + lgrp) ^ ((lane >> 1) & 7)) << 4);

  f32x4 acc[8][NB];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.0f;

  u32x4 af[2][4], bfr[2][NB];
  // The NL loads of a k-tile in issue order: first the 3/4 that fill the rows free after unit 0 (A rows of half h = 0 of
  // both wavefront rows, all B rows), then the A rows of half h = 1.  Entry < NBLK: A row block, else B row block.
  auto gload = [&](int kt, int stage, int idx) {
    const bool in_k = kt * BK + kc * CH < Kr;
    const uint32_t koff = (uint32_t)kt * 128u;
    constexpr int order4[16] = {0, 8, 1, 9, 4, 10, 5, 11, 12, 13, 14, 15, 2, 3, 6, 7};
    constexpr int order8[8] = {0, 4, 2, 5, 6, 7, 1, 3};
    const int o = NW == 4 ? order4[idx] : order8[idx % 8];
    if (o < NBLK)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)(smem + stage * STAGE + lds_wave + o * RPL * 128), 16,
                                               in_k ? voffA[o] + koff : kOutOfRange, 0, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)(smem + stage * STAGE + A_BYTES + lds_wave + (o - NBLK) * RPL * 128), 16,
                                               in_k ? voffB[o - NBLK] + koff : kOutOfRange, 0, 0, 0);
  };
  auto read_a = [&](int stage, int h, int kk, int buf, int r) {
    af[buf][r] = *(const u32x4*)(smem + stage * STAGE + fragA + (h * 4 + r) * 16 * 128 + xo[kk]);
  };
  auto read_b = [&](int stage, int kk, int c) {
    bfr[kk][c] = *(const u32x4*)(smem + stage * STAGE + fragB + c * 16 * 128 + xo[kk]);
  };
  // m = 0..4 NB - 1: A fragment ia = m / NB against the B fragments in turn, forwards for even ia and backwards for
  // odd ia, so that from one MFMA to the next only one of the two operands changes.  The chip is power-limited under
  // this load and operand lines that do not toggle cost less: measured +0.8 % on 8192x16384x16384 and 16384x16384x8192
  // against walking the B fragments forwards every time (three alternating runs each, spread 0.1 %).
  auto mma = [&](int h, int kk, int buf, int m) {
    const int ia = m / NB, ib = (ia & 1) ? NB - 1 - m % NB : m % NB;
    acc[h * 4 + ia][ib] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
        __builtin_bit_cast(bf16x8, af[buf][ia]), __builtin_bit_cast(bf16x8, bfr[kk][ib]), acc[h * 4 + ia][ib], 0, 0, 0);
  };
#define VMCNT(n) ((((n) & 15) | 0x0F70 | (((n) >> 4) << 14)))
#define SLP_FENCE() __builtin_amdgcn_sched_barrier(0)
#define SLP_BARRIER(n)                                              \
  do {                                                              \
    __builtin_amdgcn_s_waitcnt(VMCNT(n) & 0xF0FF);                  \
    asm volatile("" ::: "memory");                                  \
    __builtin_amdgcn_s_barrier();                                   \
    asm volatile("" ::: "memory");                                  \
  } while (0)

  const int nk = (Kr + BK - 1) / BK;
  // A slot = up to two memory operations followed by 2 MFMAs.  Operation codes: 0 none, 1 + r: read A fragment r,
  // 5 + c: read B fragment c, 13 + i: the unit's load i.  Reads are ordered by first use in the next unit (A0, B0.., A1..).
  struct Slot { int a, b; };
  constexpr Slot kWide4[16] = {{1, 0}, {5, 0}, {6, 0}, {13, 0}, {7, 0}, {8, 0}, {9, 0}, {14, 0},
                               {10, 0}, {11, 0}, {12, 0}, {15, 0}, {2, 0}, {3, 0}, {4, 0}, {16, 0}};
  constexpr Slot kNarrow4[16] = {{1, 0}, {0, 0}, {13, 0}, {0, 0}, {2, 0}, {0, 0}, {14, 0}, {0, 0},
                                 {3, 0}, {0, 0}, {15, 0}, {0, 0}, {4, 0}, {0, 0}, {16, 0}, {0, 0}};
  // 8 wavefronts: the reads go first (they have then returned when the unit ends in a barrier: +1 % over reads
  // spread through the unit), the loads after them
  constexpr Slot kWide8[8] = {{1, 5}, {6, 7}, {8, 2}, {3, 4}, {13, 0}, {0, 0}, {14, 0}, {0, 0}};
  constexpr Slot kNarrow8[8] = {{1, 2}, {3, 4}, {13, 0}, {0, 0}, {0, 0}, {14, 0}, {0, 0}, {0, 0}};
  // one unit: fragments of (h, kk) from af[buf], bfr[kk]; reads for the next unit (A fragments of (rh, rk) into
  // af[buf ^ 1], and, in a wide unit, the B fragments of sub-step rk) from stage rs; loads lbase.. of tile lkt into stage ls
  auto unit = [&](bool wide, int h, int kk, int buf, int rs, int rh, int rk, int lkt, int ls, int lbase) {
#pragma unroll
    for (int sl = 0; sl < NSLOT; ++sl) {
      const Slot so = NW == 4 ? (wide ? kWide4[sl % 16] : kNarrow4[sl % 16]) : (wide ? kWide8[sl % 8] : kNarrow8[sl % 8]);
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int op = q == 0 ? so.a : so.b;
        if (op >= 1 && op <= 4) read_a(rs, rh, rk, buf ^ 1, op - 1);
        else if (op >= 5 && op <= 12) read_b(rs, rk, op - 5);
        else if (op >= 13) gload(lkt, ls, lbase + op - 13);
      }
      mma(h, kk, buf, 2 * sl); mma(h, kk, buf, 2 * sl + 1);
      SLP_FENCE();
    }
  };
  // prologue: tile 0 completely and the first 3/4 of the loads of tile 1
#pragma unroll
  for (int i = 0; i < NL; ++i) gload(0, 0, i);
#pragma unroll
  for (int i = 0; i < 3 * LPU; ++i) gload(1, 1, i);
  SLP_BARRIER(3 * LPU);
#pragma unroll
  for (int r = 0; r < 4; ++r) read_a(0, 0, 0, 0, r);
#pragma unroll
  for (int c = 0; c < NB; ++c) read_b(0, 0, c);

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1, nxt = cur ^ 1;
    unit(true, 0, 0, 0, cur, 0, 1, kt + 1, nxt, 3 * LPU);     // reads A(0,1), B(1); last quarter of tile kt+1's loads
    SLP_BARRIER(4 * LPU);   // X: this tile's h=1 A rows have landed; nobody reads B / h=0 A rows of stage cur any more
    unit(false, 0, 1, 1, cur, 1, 0, kt + 2, cur, 0);          // reads A(1,0); first quarter of tile kt+2's loads
    unit(false, 1, 0, 0, cur, 1, 1, kt + 2, cur, LPU);        // reads A(1,1); second quarter
    SLP_BARRIER(3 * LPU);   // Y: B and h=0 A rows of tile kt+1 have landed in stage nxt; h=1 A rows of stage cur are free
    unit(true, 1, 1, 1, nxt, 0, 0, kt + 2, cur, 2 * LPU);     // reads next tile's A(0,0), B(0); third quarter
  }
  __builtin_amdgcn_s_waitcnt(VMCNT(0));
#undef SLP_FENCE
#undef SLP_BARRIER
#undef VMCNT

  if constexpr (EPI == EPI_WGRAD || EPI == EPI_WGRAD_UPDATE) {
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int n = n0 + wn * WTN + j * 16 + lrow;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][e];
        store_quad<T, EPI>(g, n, m0 + wm * 128 + i * 16 + 4 * lgrp, 0.0f, v, lane);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  } else {
    // Forward / data gradient: both outputs are bf16, and an accumulator block holds only 32 contiguous bytes of an
    // output row (or column).  Each wavefront therefore stages its own 128 x 64 sub-tile through a private 16 KB
    // region of the (now free) LDS stages, once transposed (64 rows of 256 bytes) and once row-major (128 rows of 128
    // bytes), and stores it as whole row segments in 16-byte pieces per lane: full cache lines on both sides, and no
    // workgroup barrier after the first one (LDS operations of one wavefront execute in order).  16-byte chunk c of
    // a staged row r sits at chunk c ^ (r & 15) (transposed) / c ^ ((r >> 1) & 7) (row-major), which keeps the
    // 8-byte writes and the 16-byte reads of a wavefront free of bank conflicts.
    // The data gradient's ReLU mask comes as bits when the forward product of the layer below ran on this tile too
    // (GemmArgs::bits: one dword per lane and 16-column block, 4 loads instead of 32 gathered 8-byte pieces of the
    // transposed activation; the gather was 10 of the epilogue's 17 us per tile), else it is gathered from maskT
    // before the staging.  (Applying the bf16 mask on the way out instead, from coalesced 16-byte loads of both layouts
    // of the activation, measured 2-3 % slower on short contractions.)  Against one shared 256 x 512-byte staging area
    // with a workgroup barrier around each pass: 8192 x 16384 products -4 % at K = 1024, -0.5 % at K = 16384.
    static_assert(NW == 8, "the staged epilogue is laid out for 8 wavefronts of 128 x 64");
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    const int rowW = m0 + wm * 128, colW = n0 + wn * WTN;     // origin of this wavefront's sub-tile
    // data gradient with the mask as bits: the 32 bits a lane needs per accumulator column are one dword
    uint32_t mbits[NB];
    if (EPI == EPI_DGRAD && g.bits) {
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int n = colW + j * 16 + lrow;
        mbits[j] = (n < g.N && rowW < g.M) ? g.bits[(size_t)n * g.ldbits + (rowW >> 5) + lgrp] : 0u;   // rowW >= M: no such block in the row
      }
    }
    __syncthreads();   // every wavefront's (zero-fill) loads have landed and its fragment reads are over
    unsigned char* reg = smem + w * 16384;
    const int Mr = (g.M + 7) & ~7;
    // finish the values in place: bias + ReLU, zeros outside the matrix
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int n = colW + j * 16 + lrow;
      const bool col_ok = n < g.N;
      float bias = 0.0f;
      if (EPI == EPI_FWD && col_ok) bias = g.bias[n];
      uint32_t word = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int mb = rowW + i * 16 + 4 * lgrp;
        if (EPI == EPI_FWD) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            acc[i][j][e] += bias;
            if (g.relu) acc[i][j][e] = fmaxf(acc[i][j][e], 0.0f);
          }
        } else if (g.bits) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (!((mbits[j] >> (4 * i + e)) & 1u)) acc[i][j][e] = 0.0f;
        } else if (g.maskT && col_ok && mb < Mr) {
          const bf16x4 mk = *(const bf16x4*)((const bf16*)g.maskT + (size_t)n * g.ldmask + mb);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (!((float)mk[e] > 0.0f)) acc[i][j][e] = 0.0f;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (mb + e >= g.M || !col_ok) acc[i][j][e] = 0.0f;
        if (EPI == EPI_FWD) {
#pragma unroll
          for (int e = 0; e < 4; ++e) word |= (uint32_t)((float)(bf16)acc[i][j][e] > 0.0f) << (4 * i + e);
          __builtin_amdgcn_sched_barrier(0);     // one block's conversions at a time: hoisted together they cost registers
        }
      }
      // the mask the data gradient of the layer above will need: one bit per stored (bf16-rounded) output > 0
      if (EPI == EPI_FWD && g.bits_out && col_ok && rowW < g.M) g.bits_out[(size_t)n * g.ldbits + (rowW >> 5) + lgrp] = word;
      __builtin_amdgcn_sched_barrier(0);
    }
    auto pack4 = [](float a, float b, float c, float d) {
      const bf16x4 o = {(bf16)a, (bf16)b, (bf16)c, (bf16)d};
      return __builtin_bit_cast(u32x2, o);
    };
    if (g.CT) {   // transposed: staged row = output column n; a piece = 8 consecutive rows m of it
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int r = j * 16 + lrow;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int mloc = i * 16 + 4 * lgrp;     // 8 bytes at element mloc of the staged row
          *(u32x2*)(reg + r * 256 + (((mloc >> 3) ^ (r & 15)) << 4) + (mloc & 4) * 2) =
              pack4(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]);
        }
      }
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int r = it * 4 + (lane >> 4), c = lane & 15;
        const int n = colW + r, m = rowW + c * 8;
        const u32x4 val = *(const u32x4*)(reg + r * 256 + ((c ^ (r & 15)) << 4));
        if (n < g.N && m < Mr) *(u32x4*)((bf16*)g.CT + (size_t)n * g.ldct + m) = val;
      }
    }
    if (g.C) {    // row-major: after the 4x4 transpose inside lane quads a lane holds 4 consecutive columns of one row
#pragma unroll
      for (int j = 0; j < NB; ++j) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][e];
          quad_transpose(v, lane);
          const int r = i * 16 + 4 * lgrp + (lane & 3);
          const int nloc = j * 16 + (lrow & ~3);
          *(u32x2*)(reg + r * 128 + (((nloc >> 3) ^ ((r >> 1) & 7)) << 4) + (nloc & 4) * 2) = pack4(v[0], v[1], v[2], v[3]);
        }
      }
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int r = it * 8 + (lane >> 3), c = lane & 7;
        const int m = rowW + r, n = colW + c * 8;
        const u32x4 val = *(const u32x4*)(reg + r * 128 + ((c ^ ((r >> 1) & 7)) << 4));
        if (m < g.M && n < g.N) *(u32x4*)((bf16*)g.C + (size_t)m * g.ldc + n) = val;
      }
    }
  }
#endif
}

// Small products: a grid of 64x64 tiles that covers less than half of the compute units leaves
// most matrix pipes idle, and one wavefront cannot drive more than its own SIMD's pipe.  This
// variant cuts the output into 32x32 tiles (4x as many workgroups) and splits the CONTRACTION over
// the 4 wavefronts of a workgroup instead: every k-tile of 128 bytes per row is 4 chunk pairs,
// wavefront w multiplies pair w of every k-tile into its own 32x32 accumulator, and the four
// partial accumulators are added through LDS in a fixed order (0,1,2,3: deterministic) before the
// shared epilogue.  Same LDS-direct loads, row layout and swizzle as the kernel above; four
// stages of 8 KB, loads three k-tiles ahead, one barrier per k-tile.
template <typename T, int EPI>
__global__ __launch_bounds__(256) void gemm_nt_ksplit_kernel(const GemmArgs g) {
#if defined(__HIP_DEVICE_COMPILE__)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // 4 stages of 64 rows x 128 bytes
  constexpr int ES = sizeof(T);
  constexpr int CH = Chunk<T>::elems;
  constexpr int BK = 128 / ES;
  constexpr int STAGE = 64 * 128, NS = 4;

  const int tilesM = (g.M + 31) / 32;
  const int tm = blockIdx.x % tilesM, tn = blockIdx.x / tilesM;   // neighbours share the B rows
  const int m0 = tm * 32, n0 = tn * 32;
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int half = lane >> 5, l32 = lane & 31;

  const int Kr = (g.K + CH - 1) / CH * CH;
  const __amdgpu_buffer_rsrc_t rsrcA =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.A), 0, (int)((size_t)g.M * g.lda * ES), 0x00020000);
  const __amdgpu_buffer_rsrc_t rsrcB =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(g.B), 0, (int)((size_t)g.N * g.ldb * ES), 0x00020000);
  // one load instruction of the workgroup covers 32 rows: wavefront w rows [8w, 8w+8), lane l -> (row 8w + l/8, chunk l%8)
  const int prow = w * 8 + (lane >> 3);
  const int pchunk = (lane & 7) ^ ((prow >> 1) & 7);
  const uint32_t voffA = (uint32_t)(((size_t)(m0 + prow) * g.lda + pchunk * CH) * ES);
  const uint32_t voffB = (uint32_t)(((size_t)(n0 + prow) * g.ldb + pchunk * CH) * ES);
  typedef __attribute__((address_space(3))) void* lds_ptr_t;
  const uint32_t lds_wave = (uint32_t)__builtin_amdgcn_readfirstlane(w * 8 * 128);
  auto gload = [&](int kt) {
    const bool in_k = kt * BK + pchunk * CH < Kr;      // past the end of K every load becomes a zero fill
    const uint32_t koff = (uint32_t)kt * 128u;
    unsigned char* sb = smem + (kt & (NS - 1)) * STAGE + lds_wave;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcA, (lds_ptr_t)sb, 16, in_k ? voffA + koff : kOutOfRange, 0, 0, 0);
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrcB, (lds_ptr_t)(sb + 32 * 128), 16, in_k ? voffB + koff : kOutOfRange, 0, 0, 0);
  };
  // this wavefront's chunk pair of every k-tile: chunks 2w (lanes 0-31) and 2w+1 (lanes 32-63)
  const uint32_t frag = (uint32_t)(l32 * 128 + (((w * 2 + half) ^ ((lane >> 1) & 7)) << 4));

  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#define VMCNT(n) ((((n) & 15) | 0x0F70 | (((n) >> 4) << 14)))
  const int nk = (Kr + BK - 1) / BK;
  gload(0); gload(1); gload(2);
  for (int kt = 0; kt < nk; ++kt) {
    // tile kt has landed once at most the loads of tiles kt+1 and kt+2 (two each) are outstanding
    // A bare barrier between compiler-level memory fences: the workgroup release fence of __syncthreads() makes
    // the wavefront wait for ALL outstanding LDS-direct loads, which would undo the prefetch.  What the barrier
    // has to order is covered by hand: this wavefront's loads of tile kt by the vmcnt wait, its LDS reads of tile
    // kt-1 by the lgkmcnt wait that precedes their MFMA.
    __builtin_amdgcn_s_waitcnt(VMCNT(4));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();  // every wavefront's part of tile kt is in LDS; all are done with tile kt-1
    asm volatile("" ::: "memory");
    // fragment reads as instructions, so that their completion is waited for exactly where written
    const uint32_t sb = lds_base + (uint32_t)((kt & (NS - 1)) * STAGE) + frag;
    u32x4 a, b;
    asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:4096" : "=&v"(a), "=&v"(b) : "v"(sb) : "memory");
    gload(kt + 3);                 // into the stage tile kt-1 occupied
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(a), "+v"(b) : : "memory");
    mma_chunk(acc, a, b, (T*)nullptr);
  }
  __builtin_amdgcn_s_waitcnt(VMCNT(0));
#undef VMCNT
  __syncthreads();                 // all stage reads and all (zero-fill) loads are over: the stages become the reduction buffer
  float* red = (float*)smem;       // [4 wavefronts][16 registers][64 lanes]
#pragma unroll
  for (int r = 0; r < 16; ++r) red[(w * 16 + r) * 64 + lane] = acc[r];
  __syncthreads();
  // wavefront w finishes register quad w: rows 8w + 4*half .. +3 of column l32
  float v[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    float sum = red[(0 * 16 + 4 * w + e) * 64 + lane];
#pragma unroll
    for (int p = 1; p < 4; ++p) sum += red[(p * 16 + 4 * w + e) * 64 + lane];
    v[e] = sum;
  }
  const int n = n0 + l32;
  float bias = 0.0f;
  if (EPI == EPI_FWD && n < g.N) bias = g.bias[n];
  store_quad<T, EPI>(g, n, m0 + 8 * w + 4 * half, bias, v, lane);
#endif
}

// ---- host side -------------------------------------------------------------------------------
struct TileCfg { int bm, bn; const char* name; };
const TileCfg kCfgs[3] = {{256, 256, "256x256"}, {128, 128, "128x128"}, {64, 64, "64x64"}};
constexpr int kCfg128TwoStage = 3;

long tiles_of(int M, int N, int c) {
  return (long)((M + kCfgs[c].bm - 1) / kCfgs[c].bm) * ((N + kCfgs[c].bn - 1) / kCfgs[c].bn);
}

int pick_cfg(int M, int N) {
  // largest tile that still gives every compute unit (256 of them) work
  for (int c = 0; c < 3; ++c)
    if (tiles_of(M, N, c) >= 224) {
      // 128x128 with two 32 KB stages lets two workgroups share a compute unit; with 512 or more tiles that hides
      // more latency than four stages of one workgroup do (measured 880 against 730 TFLOP/s on 8192x1000x16384),
      // with fewer tiles the four stages win (681 -> 812 TFLOP/s on 1024x4096x4096)
      if (c == 1 && tiles_of(M, N, 1) >= 512) return kCfg128TwoStage;
      return c;
    }
  return 2;
}

template <typename T, int BM, int BN, int EPI, int NW, int NS>
hipError_t configure_one() {
  constexpr int smem = NS * (BM + BN) * 128;
  static std::once_flag once;       // one attribute call per instantiation, also when two host threads launch first together
  static hipError_t result = hipSuccess;
  std::call_once(once, [] {
    result = hipFuncSetAttribute((const void*)gemm_nt_kernel<T, BM, BN, EPI, NW, NS>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  });
  return result;
}

template <typename T, int BM, int BN, int EPI, int NW, int NS>
hipError_t launch_one(const GemmArgs& g, hipStream_t s) {
  constexpr int smem = NS * (BM + BN) * 128;
  auto kern = gemm_nt_kernel<T, BM, BN, EPI, NW, NS>;
  hipError_t e = configure_one<T, BM, BN, EPI, NW, NS>();
  if (e != hipSuccess) return e;
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(NW * 64), smem, s, g);
  return hipGetLastError();
}

constexpr int kBigWaves = 8;
constexpr int kBigSmem = 2 * 512 * 128;

template <int EPI>
hipError_t configure_big() {
  static std::once_flag once;
  static hipError_t result = hipSuccess;
  std::call_once(once, [] {
    result = hipFuncSetAttribute((const void*)gemm_nt_big_kernel<EPI, kBigWaves>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigSmem);
  });
  return result;
}

template <int EPI>
hipError_t launch_big(const GemmArgs& g, hipStream_t s) {
  constexpr int smem = kBigSmem;
  hipError_t e = configure_big<EPI>();
  if (e != hipSuccess) return e;
  const int tiles = ((g.M + 255) / 256) * ((g.N + 255) / 256);
  hipLaunchKernelGGL((gemm_nt_big_kernel<EPI, kBigWaves>), dim3(tiles), dim3(kBigWaves * 64), smem, s, g);
  return hipGetLastError();
}

// LDS stages of gemm_nt_kernel (loads run stages-1 k-tiles ahead of the multiplies): a 256x256 tile fills LDS with two;
// the k-tiles of the small tiles are 4-16x shorter, too short to cover the loads of the next one, so they keep four.
template <typename T, int EPI>
hipError_t launch_cfg(int cfg, const GemmArgs& g, hipStream_t s) {
  switch (cfg) {
    case 0:
      if constexpr (sizeof(T) == 2) return launch_big<EPI>(g, s);
      else return launch_one<T, 256, 256, EPI, 8, 2>(g, s);
    case 1: return launch_one<T, 128, 128, EPI, 8, 4>(g, s);     // 8 wavefronts of 64x32: +5-10 % over 4 of 64x64 here
    case kCfg128TwoStage: return launch_one<T, 128, 128, EPI, 4, 2>(g, s);
    default: return launch_one<T, 64, 64, EPI, 4, 4>(g, s);
  }
}

template <typename T, int EPI>
hipError_t launch_ksplit(const GemmArgs& g, hipStream_t s) {
  const int tiles = ((g.M + 31) / 32) * ((g.N + 31) / 32);
  hipLaunchKernelGGL((gemm_nt_ksplit_kernel<T, EPI>), dim3(tiles), dim3(256), 4 * 64 * 128, s, g);
  return hipGetLastError();
}

// 64x64 tiles on fewer than this many workgroups: the contraction-split 32x32 variant fills the chip better
constexpr long kKsplitBelowTiles = 128;
bool use_ksplit(int M, int N) {
  return (long)((M + 63) / 64) * ((N + 63) / 64) < kKsplitBelowTiles;
}

template <typename T>
hipError_t launch_epi(int epi, int cfg, const GemmArgs& g, hipStream_t s) {
  if (cfg == 2 && use_ksplit(g.M, g.N)) {   // (pick_cfg returns 2 for everything small)
    switch (epi) {
      case EPI_FWD: return launch_ksplit<T, EPI_FWD>(g, s);
      case EPI_DGRAD: return launch_ksplit<T, EPI_DGRAD>(g, s);
      case EPI_WGRAD_UPDATE: return launch_ksplit<T, EPI_WGRAD_UPDATE>(g, s);
      default: return launch_ksplit<T, EPI_WGRAD>(g, s);
    }
  }
  switch (epi) {
    case EPI_FWD: return launch_cfg<T, EPI_FWD>(cfg, g, s);
    case EPI_DGRAD: return launch_cfg<T, EPI_DGRAD>(cfg, g, s);
    case EPI_WGRAD_UPDATE: return launch_cfg<T, EPI_WGRAD_UPDATE>(cfg, g, s);
    default: return launch_cfg<T, EPI_WGRAD>(cfg, g, s);
  }
}

template <typename T, int EPI>
hipError_t configure_epi() {
  hipError_t e;
  if constexpr (sizeof(T) == 2) e = configure_big<EPI>();
  else e = configure_one<T, 256, 256, EPI, 8, 2>();
  if (e == hipSuccess) e = configure_one<T, 128, 128, EPI, 8, 4>();
  if (e == hipSuccess) e = configure_one<T, 128, 128, EPI, 4, 2>();
  if (e == hipSuccess) e = configure_one<T, 64, 64, EPI, 4, 4>();
  return e;
}

}  // namespace

// One-time kernel attributes of every instantiation, so that no launch has to set one later
// (a launch sequence that is being captured into a graph should consist of launches only).
hipError_t gemm_configure_all() {
  hipError_t e = configure_epi<bf16, EPI_FWD>();
  if (e == hipSuccess) e = configure_epi<bf16, EPI_DGRAD>();
  if (e == hipSuccess) e = configure_epi<bf16, EPI_WGRAD>();
  if (e == hipSuccess) e = configure_epi<bf16, EPI_WGRAD_UPDATE>();
  if (e == hipSuccess) e = configure_epi<float, EPI_FWD>();
  if (e == hipSuccess) e = configure_epi<float, EPI_DGRAD>();
  if (e == hipSuccess) e = configure_epi<float, EPI_WGRAD>();
  if (e == hipSuccess) e = configure_epi<float, EPI_WGRAD_UPDATE>();
  return e;
}

const char* gemm_config_name(int dtype, int M, int N, int K) {
  (void)dtype; (void)K;
  const int c = pick_cfg(M, N);
  if (c == 2 && use_ksplit(M, N)) return "32x32 k-split";
  return c == kCfg128TwoStage ? "128x128 (2 stages)" : kCfgs[c].name;
}

hipError_t launch_gemm(int dtype, int epi, const GemmArgs& g, hipStream_t s) {
  const int es = dtype == 1 ? 2 : 4;
  // the kernel addresses operands with 32-bit byte offsets and a 2 GiB sentinel
  if ((size_t)g.M * g.lda * es >= 0x80000000ull || (size_t)g.N * g.ldb * es >= 0x80000000ull) return hipErrorInvalidValue;
  if (g.lda % kLdAlign || g.ldb % kLdAlign || g.M <= 0 || g.N <= 0 || g.K <= 0) return hipErrorInvalidValue;
  if (!g.A || !g.B) return hipErrorInvalidValue;                      // a missing operand must never reach the device
  if (((uintptr_t)g.A | (uintptr_t)g.B) & 15) return hipErrorInvalidValue;
  if (epi == EPI_FWD && !g.bias) return hipErrorInvalidValue;
  if (epi == EPI_WGRAD && !g.Cf) return hipErrorInvalidValue;
  if (epi == EPI_WGRAD_UPDATE) {
    if (!g.uW || !g.uV || g.ldc % 4 || (((uintptr_t)g.uW | (uintptr_t)g.uV | (uintptr_t)g.uW16 | (uintptr_t)g.uWT) & 15)) return hipErrorInvalidValue;
    if (g.uWT && g.ldwt % kLdAlign) return hipErrorInvalidValue;
  }
  if (epi != EPI_WGRAD && epi != EPI_WGRAD_UPDATE && !g.C && !g.CT) return hipErrorInvalidValue;
  // outputs are written as 16-byte vectors
  if (epi != EPI_WGRAD && epi != EPI_WGRAD_UPDATE && ((g.C && (g.ldc % kLdAlign || ((uintptr_t)g.C & 15))) || (g.CT && (g.ldct % kLdAlign || ((uintptr_t)g.CT & 15)))))
    return hipErrorInvalidValue;
  if (epi == EPI_WGRAD && (g.ldc % 4 || ((uintptr_t)g.Cf & 15))) return hipErrorInvalidValue;
  const int cfg = pick_cfg(g.M, g.N);
  GemmArgs h = g;
  // Height of the tile groups each XCD walks (the 32 tiles an XCD runs together are group_m tile rows x 32/group_m
  // tile columns).  8 is best everywhere except the weight gradient of a tall output (64 or more tile rows), whose
  // float32 rows are written faster when the concurrent tiles are wider than tall: measured 3.61 -> 3.47 ms on
  // 16384x16384x8192 and 1.90 -> 1.82 ms on 16384x8192x8192, no gain or a loss on every other shape tried.
  h.group_m = ((epi == EPI_WGRAD || epi == EPI_WGRAD_UPDATE) && cfg == 0 && (g.M + 255) / 256 >= 64) ? 4 : kGroupM;
  // Big bf16 products whose tile grid divides into 16 x 16 regions take the region walk instead: equal or better than
  // either group height on every shape tried (+1-4 %; +14 % on the short contraction of a first layer, K = 784).
  if (cfg == 0 && dtype == 1 && ((g.M + 255) / 256) % 16 == 0 && ((g.N + 255) / 256) % 16 == 0) h.group_m = kRegionWalk;
  return dtype == 1 ? launch_epi<bf16>(epi, cfg, h, s) : launch_epi<float>(epi, cfg, h, s);
}

}  // namespace slp
