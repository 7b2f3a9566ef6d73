// Memory-bound kernels of the segment step: input ingest / transposes, the two
// loss kernels (paper Sec. 2: regression on the synthetic label of the sample's
// class for a non-final segment, classification for the final one), bias
// gradients and the SGD-with-momentum update (Sec. 3).  All are written for
// coalesced traffic (a wavefront touches consecutive addresses on both the read
// and the write side; transposes go through LDS) and reduce with wavefront
// shuffles in a fixed order, so results are bit-reproducible from run to run.
#include "slp_kernels.h"

namespace slp {
namespace {

typedef __bf16 bf16;

template <typename T> __device__ __forceinline__ float to_f32(T v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f32(float v) { return (T)v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
  return v;
}

// ---------------------------------------------------------------------------------
// 64x64 element tiles moved as 16-byte vectors
// ---------------------------------------------------------------------------------
// A tile row is CPR = 64/V chunks of V elements (V = 8 bf16 / 4 float).  Row-major traffic: lane -> (row,
// chunk) with the chunk index fastest, so a wavefront touches whole 128-byte row segments.  Transposed
// traffic: lane -> (column, chunk of V consecutive rows) with the row chunk fastest, the V values gathered
// from LDS.  In LDS, chunk ch of row r sits at chunk position ch ^ ((r / V) mod CPR): the row-major writes
// stay permutations within a row, and the gather of one wavefront instruction -- V-row groups 0..CPR-1 of a
// few adjacent columns -- lands in distinct banks.
template <typename T> struct Vec16;
template <> struct Vec16<bf16> { typedef __attribute__((ext_vector_type(8))) __bf16 type; static constexpr int n = 8; };
template <> struct Vec16<float> { typedef __attribute__((ext_vector_type(4))) float type; static constexpr int n = 4; };

template <typename T, int TILE = 64>
__device__ __forceinline__ int tile_slot(int row, int chunk) {     // position of a chunk in the LDS tile, in chunks
  constexpr int V = Vec16<T>::n, CPR = TILE / V;
  return row * CPR + (chunk ^ ((row / V) & (CPR - 1)));
}

// Writes the transposed tile: outT[c0 + c][r0 + r] for r below rows_t, from the LDS tile.
template <typename T, int TILE = 64>
__device__ __forceinline__ void store_tile_transposed(const typename Vec16<T>::type* tile, T* __restrict__ outT, int ldt,
                                                      int r0, int c0, int rows_t, int C) {
  typedef typename Vec16<T>::type vec_t;
  constexpr int V = Vec16<T>::n, CPR = TILE / V, ITEMS = TILE * CPR / 256;
  const T* flat = (const T*)tile;
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int idx = threadIdx.x + it * 256;
    const int cl = idx / CPR, rc = idx % CPR;
    const int c = c0 + cl, rs = r0 + rc * V;
    if (c < C && rs < rows_t) {
      vec_t o;
#pragma unroll
      for (int e = 0; e < V; ++e) o[e] = flat[tile_slot<T, TILE>(rc * V + e, cl / V) * V + (cl % V)];
      *(vec_t*)(outT + (size_t)c * ldt + rs) = o;
    }
  }
}

// Needs: in/out/mask 16-byte aligned with leading dimensions that are multiples of V (a chunk never straddles
// two rows; a chunk that straddles C reads pad elements of the same row, which callers keep allocated);
// rows_t (rows written to the transposed output) a multiple of V or beyond the data (pad rows are zeros).
// TILE x TILE elements per workgroup: 64 for small matrices (more workgroups), 128 for large bf16 ones (8 instead of 2
// vectors in flight per lane and 256-byte row segments on both sides: 8192 x 16384 in 0.20 -> see the launcher).
template <typename T, int TILE>
__global__ __launch_bounds__(256) void copy_transpose_vec_kernel(const T* __restrict__ in, int ldin, int R, int C,
                                                                 T* __restrict__ out, int ldo, T* __restrict__ outT,
                                                                 int ldt, int rows_t, const T* __restrict__ mask,
                                                                 int ldmask) {
  typedef typename Vec16<T>::type vec_t;
  constexpr int V = Vec16<T>::n, CPR = TILE / V, ITEMS = TILE * CPR / 256;
  __shared__ vec_t tile[TILE * CPR];
  const int r0 = blockIdx.y * TILE, c0 = blockIdx.x * TILE;
  vec_t v[ITEMS];
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {       // every load of the lane is issued before the first store
    const int idx = threadIdx.x + it * 256;
    const int row = idx / CPR, ch = idx % CPR;
    const int r = r0 + row, c = c0 + ch * V;
#pragma unroll
    for (int e = 0; e < V; ++e) v[it][e] = from_f32<T>(0.0f);
    if (r < R && c < C) {
      v[it] = *(const vec_t*)(in + (size_t)r * ldin + c);
      if (mask) {     // optional ReLU mask: the element passes only where mask[r][c] > 0
        const vec_t mk = *(const vec_t*)(mask + (size_t)r * ldmask + c);
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (!(to_f32<T>(mk[e]) > 0.0f)) v[it][e] = from_f32<T>(0.0f);
      }
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (c + e >= C) v[it][e] = from_f32<T>(0.0f);     // pads stay zero
    }
  }
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int idx = threadIdx.x + it * 256;
    const int row = idx / CPR, ch = idx % CPR;
    const int r = r0 + row, c = c0 + ch * V;
    if (out && r < R && c < C) *(vec_t*)(out + (size_t)r * ldo + c) = v[it];
    tile[tile_slot<T, TILE>(row, ch)] = v[it];
  }
  if (!outT) return;
  __syncthreads();
  store_tile_transposed<T, TILE>(tile, outT, ldt, r0, c0, rows_t, C);
}

// ---------------------------------------------------------------------------------
// copy + transpose through a 64x64 LDS tile, element by element (any alignment)
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void copy_transpose_kernel(const T* __restrict__ in, int ldin, int R, int C,
                                                             T* __restrict__ out, int ldo, T* __restrict__ outT,
                                                             int ldt, int pad_t, const T* __restrict__ mask,
                                                             int ldmask) {
  __shared__ T tile[64][65];
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int rr = ty; rr < 64; rr += 4) {
    const int r = r0 + rr, c = c0 + tx;
    T v = from_f32<T>(0.0f);
    if (r < R && c < C) {
      v = in[(size_t)r * ldin + c];
      // optional ReLU mask: the element passes only where mask[r][c] > 0
      if (mask && !(to_f32(mask[(size_t)r * ldmask + c]) > 0.0f)) v = from_f32<T>(0.0f);
      if (out) out[(size_t)r * ldo + c] = v;
    }
    tile[rr][tx] = v;
  }
  if (!outT) return;
  __syncthreads();
  const int R8 = pad_t ? ((R + 7) & ~7) : R;
  for (int cc = ty; cc < 64; cc += 4) {
    const int c = c0 + cc, r = r0 + tx;
    if (c < C && r < R8) outT[(size_t)c * ldt + r] = tile[tx][cc];
  }
}

// ---------------------------------------------------------------------------------
// mean squared error against the synthetic label of each row's class
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void mse_loss_grad_kernel(const T* __restrict__ AL, int ld, const int32_t* __restrict__ y,
                                                            const float* __restrict__ table, int classes, int B, int D,
                                                            int relu_last,
                                                            float scale, T* __restrict__ dZ, T* __restrict__ dZT, int ldt,
                                                            float* __restrict__ partials, unsigned* __restrict__ bad_ids) {
  typedef typename Vec16<T>::type vec_t;
  typedef __attribute__((ext_vector_type(4))) float f32x4;
  constexpr int V = Vec16<T>::n, CPR = 64 / V, ITEMS = 64 * CPR / 256;
  __shared__ vec_t tile[64 * CPR];
  __shared__ float red[4];
  const int b0 = blockIdx.y * 64, d0 = blockIdx.x * 64;
  const bool table_vec = (D & 3) == 0;        // label rows start 16-byte aligned
  float lsum = 0.0f;
#pragma unroll
  for (int it = 0; it < ITEMS; ++it) {
    const int idx = threadIdx.x + it * 256;
    const int row = idx / CPR, ch = idx % CPR;
    const int m = b0 + row, i = d0 + ch * V;
    vec_t gv;
#pragma unroll
    for (int e = 0; e < V; ++e) gv[e] = from_f32<T>(0.0f);
    if (m < B && i < D) {
      const vec_t av = *(const vec_t*)(AL + (size_t)m * ld + i);     // a chunk that straddles D reads pad zeros
      const int cls = min(max(y[m], 0), classes - 1);                 // ids are the caller's; never index outside the table
      if (cls != y[m] && blockIdx.x == 0 && ch == 0) atomicAdd(bad_ids, 1u);   // once per row; rare, and the count is an integer
      const float* trow = table + (size_t)cls * D + i;
      float tv[V];
      if (table_vec && i + V <= D) {
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
          const f32x4 t4 = *(const f32x4*)(trow + 4 * q);
#pragma unroll
          for (int e = 0; e < 4; ++e) tv[4 * q + e] = t4[e];
        }
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e) tv[e] = i + e < D ? trow[e] : 0.0f;
      }
#pragma unroll
      for (int e = 0; e < V; ++e) {
        if (i + e < D) {
          const float a = to_f32<T>(av[e]);
          const float d = a - tv[e];
          lsum += d * d;
          gv[e] = from_f32<T>((relu_last && !(a > 0.0f)) ? 0.0f : scale * d);
        }
      }
      if (dZ) *(vec_t*)(dZ + (size_t)m * ld + i) = gv;
    }
    tile[tile_slot<T>(row, ch)] = gv;
  }
  lsum = wave_sum(lsum);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = lsum;
  __syncthreads();
  if (threadIdx.x == 0) partials[blockIdx.y * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
  store_tile_transposed<T>(tile, dZT, ldt, b0, d0, (B + 7) & ~7, D);
}

// ---------------------------------------------------------------------------------
// softmax cross-entropy, one wavefront per row
// ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void xent_loss_grad_kernel(const T* __restrict__ ZL, int ld, const int32_t* __restrict__ y,
                                                             int B, int C, int relu_last, float inv_b,
                                                             T* __restrict__ dZ, float* __restrict__ row_loss,
                                                             unsigned* __restrict__ bad_ids) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m < B) {
    const T* z = ZL + (size_t)m * ld;
    float mx = -INFINITY;
    for (int c = lane; c < C; c += 64) mx = fmaxf(mx, to_f32(z[c]));
    mx = wave_max(mx);
    float sum = 0.0f;
    for (int c = lane; c < C; c += 64) sum += expf(to_f32(z[c]) - mx);
    sum = wave_sum(sum);
    const float lse = mx + logf(sum);
    const int cls = min(max(y[m], 0), C - 1);
    if (lane == 0 && cls != y[m]) atomicAdd(bad_ids, 1u);
    if (lane == 0) row_loss[m] = lse - to_f32(z[cls]);
    T* g = dZ + (size_t)m * ld;
    for (int c = lane; c < C; c += 64) {
      const float zc = to_f32(z[c]);
      const float p = expf(zc - lse);
      const float d = (p - (c == cls ? 1.0f : 0.0f)) * inv_b;
      g[c] = from_f32<T>((relu_last && !(zc > 0.0f)) ? 0.0f : d);
    }
  }
}

// out = scale * sum(partials), summed in double in a fixed order by one block.  (A separate launch on purpose:
// finishing the sum inside the loss kernels -- last block counted in by an atomic -- needs a device-scope fence per
// block, which on this chip writes back the whole L2 of the block's XCD: measured 25x slower than this launch.)
__global__ __launch_bounds__(256) void reduce_loss_kernel(const float* __restrict__ partials, int n, double scale,
                                                          float* out0, float* out1) {
  __shared__ double red[256];
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) acc += (double)partials[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float v = (float)(red[0] * scale);
    out0[0] = v;
    if (out1) out1[0] = v;
  }
}

// ---------------------------------------------------------------------------------
// bias gradient: row sums of dZ^T, one wavefront per output feature
// ---------------------------------------------------------------------------------
// then the bias's own momentum update: v = mu v + db; b -= lr v (the gradient is kept for inspection)
template <typename T>
__device__ __forceinline__ void bias_grad_update_block(int block, const T* __restrict__ dZT, int ldt, int N, int B,
                                                       float* __restrict__ db, float* __restrict__ b,
                                                       float* __restrict__ vb, float lr, float mu) {
  constexpr int V = 16 / sizeof(T);
  typedef T vec_t __attribute__((ext_vector_type(V)));
  const int lane = threadIdx.x & 63;
  const int n = block * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const T* row = dZT + (size_t)n * ldt;
  const int Bv = (B + V - 1) / V;      // pads up to the chunk boundary are zero
  // four independent 16-byte loads per lane and trip, so that the row streams instead of crawling load by load;
  // the partial sums are added in a fixed order
  float a4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int c0 = lane; c0 < Bv; c0 += 256) {
    vec_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + 64 * u;
      if (c < Bv) v[u] = *(const vec_t*)(row + (size_t)c * V);
      else
#pragma unroll
        for (int e = 0; e < V; ++e) v[u][e] = from_f32<T>(0.0f);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int e = 0; e < V; ++e) a4[u] += to_f32((T)v[u][e]);
  }
  float acc = wave_sum((a4[0] + a4[1]) + (a4[2] + a4[3]));
  if (lane == 0) {
    db[n] = acc;
    float v = acc;
    if (mu != 0.0f) {
      v = mu * vb[n] + v;
      vb[n] = v;
    }
    b[n] -= lr * v;
  }
}

// ---------------------------------------------------------------------------------
// SGD with momentum on one weight matrix + derived copies
// ---------------------------------------------------------------------------------
// A block owns a 64 (out) x 64 (in) tile.  Every thread moves 16-byte vectors: four
// consecutive inputs of one output row for the float32 streams (gradient, momentum,
// master weight), and four consecutive outputs of one input row for the transposed copy,
// which goes through an LDS tile.  Pad columns (in >= K, up to the leading dimension) hold
// zeros in all three streams and stay zero under the update, so the row direction needs
// no tail handling.
template <typename T>
__device__ __forceinline__ void sgd_update_block(int bx, int by, float* __restrict__ W32, float* __restrict__ vW,
                                                 const float* __restrict__ dW, int N, int K, int ldk,
                                                 bf16* __restrict__ W16, T* __restrict__ WT, int ldn, float lr,
                                                 float mu, int refresh_only) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef T tx4 __attribute__((ext_vector_type(4)));
  typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
  __shared__ T tile[64][68];
  const int n0 = by * 64, k0 = bx * 64;
  const int q = threadIdx.x & 15, r = threadIdx.x >> 4;
  const int k = k0 + q * 4;
  // all loads of the thread's four rows are issued before the first store, so that 9 to 12
  // 16-byte requests per thread are in flight
  f32x4 w[4], gr[4], vo[4];
  const bool with_v = !refresh_only && mu != 0.0f;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int n = n0 + r + 16 * p;
    const bool in = n < N && k < K;
    const size_t idx = (size_t)n * ldk + k;
    w[p] = in ? __builtin_nontemporal_load((const f32x4*)(W32 + idx)) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    gr[p] = (in && !refresh_only) ? __builtin_nontemporal_load((const f32x4*)(dW + idx)) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    vo[p] = (in && with_v) ? __builtin_nontemporal_load((const f32x4*)(vW + idx)) : f32x4{0.0f, 0.0f, 0.0f, 0.0f};
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int rr = r + 16 * p, n = n0 + rr;
    if (n < N && k < K) {
      const size_t idx = (size_t)n * ldk + k;
      if (!refresh_only) {
        f32x4 v = gr[p];
        if (with_v) {
          v = mu * vo[p] + v;
          __builtin_nontemporal_store(v, (f32x4*)(vW + idx));
        }
        w[p] = w[p] - lr * v;
        __builtin_nontemporal_store(w[p], (f32x4*)(W32 + idx));
      }
      if (W16) {
        bf16x4 h;
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = (bf16)w[p][e];
        *(bf16x4*)(W16 + idx) = h;
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) tile[rr][q * 4 + e] = from_f32<T>(w[p][e]);
  }
  if (!WT) return;      // (uniform over the launch)
  __syncthreads();
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int kk = r + 16 * p, kg = k0 + kk, n = n0 + q * 4;
    if (kg < K && n < N) {
      tx4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = tile[q * 4 + e][kk];
      *(tx4*)(WT + (size_t)kg * ldn + n) = o;
    }
  }
}

// One launch updates a whole layer: blocks [0, kb*nb) each own a 64x64 tile of the weight matrix, the blocks after
// them 4 output features of the bias each (gradient = row sum of dZ^T, then the same momentum update).
struct LayerUpdate {
  float *W32, *vW; const float* dW; int N, K, ldk; void* W16; void* WT; int ldn;     // weights [N][ldk]
  const void* dZT; int ldt, B; float *db, *b, *vb;                                     // bias: dZT [N][ldt]; null = weights only
  float lr, mu; int refresh_only;
};

// the weight matrix alone, one block per 64x64 tile on a 2-D grid (large layers)
template <typename T>
__global__ __launch_bounds__(256) void sgd_update_kernel(float* __restrict__ W32, float* __restrict__ vW,
                                                         const float* __restrict__ dW, int N, int K, int ldk,
                                                         bf16* __restrict__ W16, T* __restrict__ WT, int ldn, float lr,
                                                         float mu, int refresh_only) {
  sgd_update_block<T>(blockIdx.x, blockIdx.y, W32, vW, dW, N, K, ldk, W16, WT, ldn, lr, mu, refresh_only);
}

// The same on a fixed number of workgroups that walk the tiles with the grid's stride: for updates that run beside
// matrix products.  At full width the update saturates HBM and the product next to it, which waits on every load,
// all but stops (measured: a 1.3 ms update stretched the product beside it from 3.15 to 4.29 ms); one workgroup per
// compute unit takes longer over the same bytes and costs the product less.
// Held to 64 registers per lane (8 wavefronts per SIMD): the 256x256 product kernel's two wavefronts per SIMD take 448 of
// the 512 registers, and a wavefront that needs more than the 64 left cannot share the SIMD with them.  At 68 the
// update's workgroups could only start on a compute unit between two product workgroups and then kept the next one
// out for as long as they ran (comparison configuration: 38.9 -> 36.9 ms per step with the limit).
// pause: units of ~0.5 us that a workgroup sleeps after each 64x64 tile.  A compute unit's vector memory path delivers
// ~56 GB/s (measured with one copy workgroup per compute unit) and the product beside the update already takes ~48 of
// them, so the update's loads queue in front of the product's; spread over twice the time they fit into the headroom
// (comparison configuration 37.1 -> 36.7 ms per step, deep configuration run serially 13.2 -> 12.9 at 8-14 units; the
// update's tail must still find products to hide behind, which is why the caller sizes the pause by the batch).
template <typename T>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(8, 8))) void sgd_update_strided_kernel(float* __restrict__ W32, float* __restrict__ vW,
                                                                 const float* __restrict__ dW, int N, int K, int ldk,
                                                                 bf16* __restrict__ W16, T* __restrict__ WT, int ldn, float lr,
                                                                 float mu, int refresh_only, int pause) {
  const int kb = (K + 63) / 64, tiles = kb * ((N + 63) / 64);
  for (int id = blockIdx.x; id < tiles; id += gridDim.x) {
    sgd_update_block<T>(id % kb, id / kb, W32, vW, dW, N, K, ldk, W16, WT, ldn, lr, mu, refresh_only);
    for (int i = 0; i < pause; ++i) __builtin_amdgcn_s_sleep(16);
    __syncthreads();   // the LDS tile is reused
  }
}

template <typename T>
__global__ __launch_bounds__(256) void layer_update_kernel(const LayerUpdate u) {
  const int kb = (u.K + 63) / 64, nb = (u.N + 63) / 64;
  const int id = blockIdx.x;
  if (id < kb * nb)
    sgd_update_block<T>(id % kb, id / kb, u.W32, u.vW, u.dW, u.N, u.K, u.ldk, (bf16*)u.W16, (T*)u.WT, u.ldn, u.lr, u.mu, u.refresh_only);
  else
    bias_grad_update_block<T>(id - kb * nb, (const T*)u.dZT, u.ldt, u.N, u.B, u.db, u.b, u.vb, u.lr, u.mu);
}

}  // namespace

hipError_t launch_copy_transpose(int dtype, const void* in, int ldin, int R, int C, void* out, int ldo, void* outT,
                                 int ldt, int pad_t, const void* mask, int ldmask, hipStream_t s) {
  dim3 grid((C + 63) / 64, (R + 63) / 64);
  // 16-byte vectors when every row of every operand starts on a 16-byte boundary and the transposed output takes
  // whole row chunks; the element-wise kernel otherwise (a dense caller matrix whose width is not a multiple of V)
  const int V = dtype == 1 ? 8 : 4;
  const int rows_t = pad_t ? ((R + 7) & ~7) : R;
  const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)outT | (uintptr_t)mask) & 15) == 0) && ldin % V == 0 &&
                       (!out || ldo % V == 0) && (!outT || (ldt % V == 0 && rows_t % V == 0)) && (!mask || ldmask % V == 0);
  if (aligned) {
    // large bf16 matrices: 128 x 128 tiles once they still give every compute unit several workgroups
    if (dtype == 1 && (long)((C + 127) / 128) * ((R + 127) / 128) >= 1024) {
      dim3 grid128((C + 127) / 128, (R + 127) / 128);
      copy_transpose_vec_kernel<bf16, 128><<<grid128, 256, 0, s>>>((const bf16*)in, ldin, R, C, (bf16*)out, ldo, (bf16*)outT, ldt,
                                                                   rows_t, (const bf16*)mask, ldmask);
    } else if (dtype == 1)
      copy_transpose_vec_kernel<bf16, 64><<<grid, 256, 0, s>>>((const bf16*)in, ldin, R, C, (bf16*)out, ldo, (bf16*)outT, ldt, rows_t,
                                                               (const bf16*)mask, ldmask);
    else
      copy_transpose_vec_kernel<float, 64><<<grid, 256, 0, s>>>((const float*)in, ldin, R, C, (float*)out, ldo, (float*)outT, ldt,
                                                                rows_t, (const float*)mask, ldmask);
    return hipGetLastError();
  }
  if (dtype == 1)
    copy_transpose_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)in, ldin, R, C, (bf16*)out, ldo, (bf16*)outT, ldt, pad_t,
                                                     (const bf16*)mask, ldmask);
  else
    copy_transpose_kernel<float><<<grid, 256, 0, s>>>((const float*)in, ldin, R, C, (float*)out, ldo, (float*)outT, ldt, pad_t,
                                                      (const float*)mask, ldmask);
  return hipGetLastError();
}

int mse_partial_count(int B, int D) { return ((D + 63) / 64) * ((B + 63) / 64); }

hipError_t launch_mse_loss_grad(int dtype, const void* AL, int ld, const int32_t* y, const float* table, int classes,
                                int B, int D, int relu_last, void* dZ, void* dZT, int ldt, float* partials, unsigned* bad_ids,
                                hipStream_t s) {
  dim3 grid((D + 63) / 64, (B + 63) / 64);
  const float scale = (float)(2.0 / ((double)B * (double)D));
  if (dtype == 1)
    mse_loss_grad_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)AL, ld, y, table, classes, B, D, relu_last, scale, (bf16*)dZ,
                                                    (bf16*)dZT, ldt, partials, bad_ids);
  else
    mse_loss_grad_kernel<float><<<grid, 256, 0, s>>>((const float*)AL, ld, y, table, classes, B, D, relu_last, scale, (float*)dZ,
                                                     (float*)dZT, ldt, partials, bad_ids);
  return hipGetLastError();
}

hipError_t launch_xent_loss_grad(int dtype, const void* ZL, int ld, const int32_t* y, int B, int C, int relu_last,
                                 void* dZ, float* partials, unsigned* bad_ids, hipStream_t s) {
  const int grid = (B + 3) / 4;
  const float inv_b = (float)(1.0 / (double)B);
  if (dtype == 1)
    xent_loss_grad_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)ZL, ld, y, B, C, relu_last, inv_b, (bf16*)dZ, partials, bad_ids);
  else
    xent_loss_grad_kernel<float><<<grid, 256, 0, s>>>((const float*)ZL, ld, y, B, C, relu_last, inv_b, (float*)dZ, partials, bad_ids);
  return hipGetLastError();
}

hipError_t launch_reduce_loss(const float* partials, int n, double scale, float* out0, float* out1, hipStream_t s) {
  reduce_loss_kernel<<<1, 256, 0, s>>>(partials, n, scale, out0, out1);
  return hipGetLastError();
}

hipError_t launch_layer_update(int dtype, float* W32, float* vW, const float* dW, int N, int K, int ldk, void* W16, void* WT,
                               int ldn, const void* dZT, int ldt, int B, float* db, float* b, float* vb, float lr, float mu,
                               int refresh_only, int max_workgroups, int pause, hipStream_t s) {
  if (!dZT) {       // weights only
    const int wgs = max_workgroups;
    if (wgs > 0 && (long)((K + 63) / 64) * ((N + 63) / 64) > wgs) {
      if (dtype == 1)
        sgd_update_strided_kernel<bf16><<<wgs, 256, 0, s>>>(W32, vW, dW, N, K, ldk, (bf16*)W16, (bf16*)WT, ldn, lr, mu, refresh_only, pause);
      else
        sgd_update_strided_kernel<float><<<wgs, 256, 0, s>>>(W32, vW, dW, N, K, ldk, nullptr, (float*)WT, ldn, lr, mu, refresh_only, pause);
      return hipGetLastError();
    }
    dim3 grid2((K + 63) / 64, (N + 63) / 64);
    if (dtype == 1)
      sgd_update_kernel<bf16><<<grid2, 256, 0, s>>>(W32, vW, dW, N, K, ldk, (bf16*)W16, (bf16*)WT, ldn, lr, mu, refresh_only);
    else
      sgd_update_kernel<float><<<grid2, 256, 0, s>>>(W32, vW, dW, N, K, ldk, nullptr, (float*)WT, ldn, lr, mu, refresh_only);
    return hipGetLastError();
  }
  const LayerUpdate u{W32, vW, dW, N, K, ldk, dtype == 1 ? W16 : nullptr, WT, ldn, dZT, ldt, B, db, b, vb, lr, mu, refresh_only};
  const int grid = ((K + 63) / 64) * ((N + 63) / 64) + (dZT ? (N + 3) / 4 : 0);
  if (dtype == 1) layer_update_kernel<bf16><<<grid, 256, 0, s>>>(u);
  else layer_update_kernel<float><<<grid, 256, 0, s>>>(u);
  return hipGetLastError();
}

}  // namespace slp
