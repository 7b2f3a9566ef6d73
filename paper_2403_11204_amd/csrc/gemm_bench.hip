// Stand-alone timing of one matrix product of the segment step (the three products of paper Sec. 2-3 all run through
// launch_gemm): random bf16 operands, `iters` launches after 0.3 s of warm-up launches, 64 sampled outputs checked against
// float64 dot products on the host, and -- with both output layouts -- the transposed output checked against the
// row-major one element by element.  A development tool: nothing in the library or the tests uses it.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops -I include \
//         -I paper_2403_11204_amd/csrc paper_2403_11204_amd/csrc/gemm_bench.hip -o _build/gemm_bench
//   _build/gemm_bench M N K epilogue iters pad data outputs
//     epilogue: 0 forward (+bias), 1 data gradient (masked), 2 weight gradient (float32 output)
//     pad     : elements added to every leading dimension (192 = what the library's own buffers use at these widths)
//     data    : 0 uniform(-1,1), 1 zeros, 2 half zeros (ReLU-like), 3 quarter steps
//     outputs : 0 row-major and transposed, 1 row-major only, 2 transposed only (epilogues 0 and 1)
#include "gemm.hip"
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cmath>
#include <cstring>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %s:%d\n", hipGetErrorString(e), __FILE__, __LINE__); return 1; } } while (0)
static uint16_t f2bf(float f) { uint32_t b; memcpy(&b, &f, 4); b += 0x7FFF + ((b >> 16) & 1); return b >> 16; }
static float bf2f(uint16_t h) { uint32_t b = (uint32_t)h << 16; float f; memcpy(&f, &b, 4); return f; }
int main(int argc, char** argv) {
  int M = argc > 1 ? atoi(argv[1]) : 8192, N = argc > 2 ? atoi(argv[2]) : 16384, K = argc > 3 ? atoi(argv[3]) : 16384;
  int epi = argc > 4 ? atoi(argv[4]) : 2, iters = argc > 5 ? atoi(argv[5]) : 10;
  int pad = argc > 6 ? atoi(argv[6]) : 0; int dmode = argc > 7 ? atoi(argv[7]) : 0; int outs = argc > 8 ? atoi(argv[8]) : 0; int lda = (K + 7) / 8 * 8 + pad, ldb = lda, ldc = (N + 7) / 8 * 8 + pad, ldct = (M + 7) / 8 * 8 + pad;
  std::vector<uint16_t> hA((size_t)M * lda), hB((size_t)N * ldb);
  uint32_t s = 12345;
  auto rnd = [&]() { s = s * 1664525u + 1013904223u; float r = ((s >> 8) & 0xFFFF) / 32768.0f - 1.0f; if (dmode == 1) return 0.0f; if (dmode == 2) return r > 0 ? r : 0.0f; if (dmode == 3) return (float)((int)(r * 4)) * 0.25f; return r; };
  for (int m = 0; m < M; m++) for (int k = 0; k < lda; k++) hA[(size_t)m * lda + k] = k < K ? f2bf(rnd()) : 0;
  for (int n = 0; n < N; n++) for (int k = 0; k < ldb; k++) hB[(size_t)n * ldb + k] = k < K ? f2bf(rnd()) : 0;
  void *dA, *dB, *dC, *dCT, *dMask; float *dCf, *dBias;
  CK(hipMalloc(&dA, hA.size() * 2)); CK(hipMalloc(&dB, hB.size() * 2));
  CK(hipMalloc(&dC, (size_t)M * ldc * 2)); CK(hipMalloc(&dCT, (size_t)N * ldct * 2)); CK(hipMalloc(&dMask, (size_t)N * ldct * 2 + (size_t)M * ldc * 2));
  CK(hipMalloc(&dCf, (size_t)M * ldc * 4)); CK(hipMalloc(&dBias, (size_t)N * 4));
  CK(hipMemcpy(dA, hA.data(), hA.size() * 2, hipMemcpyHostToDevice)); CK(hipMemcpy(dB, hB.data(), hB.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemset(dBias, 0, (size_t)N * 4));
  std::vector<uint16_t> hMask((size_t)N * ldct + (size_t)M * ldc);
  for (size_t i = 0; i < hMask.size(); i++) { s = s * 1664525u + 1013904223u; hMask[i] = f2bf((s >> 20) % 3 ? 1.0f : ((s >> 8) & 1 ? 0.0f : -0.5f)); }   // 1/3 masked out
  CK(hipMemcpy(dMask, hMask.data(), hMask.size() * 2, hipMemcpyHostToDevice));
  slp::GemmArgs g{}; g.A = dA; g.B = dB; g.lda = lda; g.ldb = ldb; g.M = M; g.N = N; g.K = K;
  g.C = dC; g.CT = dCT; g.ldc = ldc; g.ldct = ldct; g.bias = dBias; g.relu = 0; g.maskT = dMask; g.ldmask = ldct; g.Cf = dCf;
  if (outs == 1) g.CT = nullptr; if (outs == 2) g.C = nullptr;
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  // warm-up: at least two launches and at least 0.3 s of them -- the chip's clock settles over the first ~0.1 s of a
  // burst of work, and a short product timed before that reads 10-25 % low
  {
    const auto t0 = std::chrono::steady_clock::now();
    int n = 0;
    do {
      for (int i = 0; i < 2; i++) CK(slp::launch_gemm(1, epi, g, 0));
      CK(hipDeviceSynchronize());
      n += 2;
    } while (std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count() < 0.3 && n < 100000);
  }
  CK(hipEventRecord(e0, 0));
  for (int i = 0; i < iters; i++) CK(slp::launch_gemm(1, epi, g, 0));
  CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= iters;
  double tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12;
  // check 64 sampled outputs
  double maxerr = 0;
  std::vector<uint16_t> hC; std::vector<float> hCf;
  if (epi == 2) { hCf.resize((size_t)M * ldc); CK(hipMemcpy(hCf.data(), dCf, hCf.size() * 4, hipMemcpyDeviceToHost)); }
  else { hC.resize((size_t)M * ldc); CK(hipMemcpy(hC.data(), dC, hC.size() * 2, hipMemcpyDeviceToHost)); }
  std::vector<uint16_t> hCT;
  if (epi != 2) { hCT.resize((size_t)N * ldct); CK(hipMemcpy(hCT.data(), dCT, hCT.size() * 2, hipMemcpyDeviceToHost)); }
  double maxerrT = 0;
  for (int t = 0; t < 64; t++) {
    s = s * 1664525u + 1013904223u; int m = (s >> 4) % M; s = s * 1664525u + 1013904223u; int n = (s >> 4) % N;
    if (t == 0) { m = M - 1; n = N - 1; }
    double ref = 0; for (int k = 0; k < K; k++) ref += (double)bf2f(hA[(size_t)m * lda + k]) * bf2f(hB[(size_t)n * ldb + k]);
    if (epi == 1 && !(bf2f(hMask[(size_t)n * ldct + m]) > 0.0f)) ref = 0;
    double got = epi == 2 ? hCf[(size_t)m * ldc + n] : (outs == 2 ? bf2f(hCT[(size_t)n * ldct + m]) : bf2f(hC[(size_t)m * ldc + n]));
    double err = fabs(got - ref) / (fabs(ref) + 1.0); if (err > maxerr) maxerr = err;
    if (epi != 2 && outs != 1) { double gt = bf2f(hCT[(size_t)n * ldct + m]); double e2 = fabs(gt - ref) / (fabs(ref) + 1.0); if (e2 > maxerrT) maxerrT = e2; }
  }
  if (epi != 2 && outs == 0) {   // whole-matrix consistency: CT must be the exact transpose of C, pads zero
    size_t bad = 0;
    for (int m = 0; m < M; m++) for (int n = 0; n < N; n++) if (hC[(size_t)m * ldc + n] != hCT[(size_t)n * ldct + m]) bad++;
    for (int n = 0; n < N; n++) for (int m = M; m < (M + 7) / 8 * 8; m++) if (hCT[(size_t)n * ldct + m] != 0) bad++;
    for (int m = 0; m < M; m++) for (int n = N; n < (N + 7) / 8 * 8; n++) if (hC[(size_t)m * ldc + n] != 0) bad++;
    printf("transpose/pad mismatches: %zu, maxerrT=%.2e\n", bad, maxerrT);
  }
  printf("M=%d N=%d K=%d epi=%d  %.3f ms  %.1f TFLOP/s  (%.1f%% of 2516.6)  maxerr=%.2e %s\n", M, N, K, epi, ms, tf, 100 * tf / 2516.6,
         maxerr, maxerr < (epi == 2 ? 1e-4 : 1e-2) ? "OK" : "MISMATCH");
  return 0;
}
