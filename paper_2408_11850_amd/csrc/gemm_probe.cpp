// Stand-alone driver for profiling the projection kernel without Python: runs spec_gemm_partials on the
// five projection shapes of a model (default: the 70B-shape target) at a given token count, plus the
// streaming-read probe and the weight-packing copy kernel as calibration launches of known size.
// Weights are a constant byte pattern (traffic and timing do not depend on the values).
//
//   gemm_probe [M=7] [iters=5] [d_model=8192] [n_heads=64] [n_kv_heads=8] [d_ffn=28672] [vocab=32000]
//   gemm_probe dense [M=4095] [iters=5] [d_model=8192] [n_heads=64] [n_kv_heads=8] [d_ffn=28672]
//
// The second form runs the prompt-sized matrix-core projection (spec_dense_gemm) on the four layer shapes with
// the epilogue the prefill path uses for each, and prints TFLOP/s.
//
// Used under `rocprofv3 --kernel-trace --stats` and `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE`.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/spec.h"

#define CK(x)                                                                  \
  do {                                                                         \
    hipError_t e_ = (x);                                                       \
    if (e_ != hipSuccess) {                                                    \
      fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                  \
      return 1;                                                                \
    }                                                                          \
  } while (0)
#define SK(x)                                                                  \
  do {                                                                         \
    int r_ = (x);                                                              \
    if (r_ != SPEC_OK) {                                                       \
      fprintf(stderr, "%s: %d %s\n", #x, r_, spec_last_error());               \
      return 1;                                                                \
    }                                                                          \
  } while (0)

static int dense_main(int argc, char** argv) {
  const int M = argc > 2 ? atoi(argv[2]) : 4095;
  const int iters = argc > 3 ? atoi(argv[3]) : 5;
  const int d = argc > 4 ? atoi(argv[4]) : 8192;
  const int hq = argc > 5 ? atoi(argv[5]) : 64;
  const int hkv = argc > 6 ? atoi(argv[6]) : 8;
  const int F = argc > 7 ? atoi(argv[7]) : 28672;
  const int dh = d / hq;
  struct Shape { const char* name; int N, K, epi; };
  const Shape shapes[] = {{"qkv", (hq + 2 * hkv) * dh, d, 0}, {"o", d, hq * dh, 1}, {"gate_up", 2 * F, d, 2},
                          {"down", d, F, 1}};
  hipStream_t st;
  CK(hipStreamCreate(&st));
  size_t max_w = 0, max_x = 0, max_y = 0;
  for (const Shape& s : shapes) {
    if (spec_packed_bytes(s.N, s.K) > max_w) max_w = spec_packed_bytes(s.N, s.K);
    if ((size_t)M * s.K * 2 > max_x) max_x = (size_t)M * s.K * 2;
    if ((size_t)M * s.N * 4 > max_y) max_y = (size_t)M * s.N * 4;
  }
  void *w, *x, *y;
  CK(hipMalloc(&w, max_w));
  CK(hipMalloc(&x, max_x));
  CK(hipMalloc(&y, max_y));
  // operands: pseudo-random bf16 in (-1, 1) (the matrix pipe's power draw, and with it the clock, depends on how
  // the operand bits toggle: a constant pattern runs ~15 % faster than real data), a 32 MiB block tiled over both
  CK(hipMemset(y, 0, max_y));
  {
    const size_t blk = 32u << 20;
    std::vector<unsigned short> h(blk / 2);
    unsigned long long s = 0x9E3779B97F4A7C15ull;
    for (size_t i = 0; i < h.size(); ++i) {
      s = s * 6364136223846793005ull + 1442695040888963407ull;
      const float f = (float)((double)(s >> 40) / 8388608.0 - 1.0);   // 24 random bits -> [-1, 1)
      unsigned u;
      memcpy(&u, &f, 4);
      h[i] = (unsigned short)(u >> 16);
    }
    void* bufs[2] = {w, x};
    const size_t sizes[2] = {max_w, max_x};
    for (int b = 0; b < 2; ++b)
      for (size_t off = 0; off < sizes[b]; off += blk)
        CK(hipMemcpy((char*)bufs[b] + off, h.data(), sizes[b] - off < blk ? sizes[b] - off : blk, hipMemcpyHostToDevice));
  }
  CK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  printf("dense projection probe: M=%d, %d launches per shape, pseudo-random operands\n", M, iters);
  for (const Shape& s : shapes) {
    SK(spec_dense_gemm((float*)y, y, x, w, M, s.N, s.K, s.epi, st));   // warm-up
    CK(hipEventRecord(e0, st));
    for (int i = 0; i < iters; ++i) SK(spec_dense_gemm((float*)y, y, x, w, M, s.N, s.K, s.epi, st));
    CK(hipEventRecord(e1, st));
    CK(hipStreamSynchronize(st));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    const double fl = 2.0 * M * s.N * s.K;
    printf("  %-8s N=%6d K=%6d epilogue %d  %9.2f us  %7.1f TFLOP/s\n", s.name, s.N, s.K, s.epi, ms / iters * 1e3,
           fl / (ms / iters * 1e-3) / 1e12);
  }
  return 0;
}

int main(int argc, char** argv) {
  if (argc > 1 && argv[1][0] == 'd') return dense_main(argc, argv);
  const int M = argc > 1 ? atoi(argv[1]) : 7;
  const int iters = argc > 2 ? atoi(argv[2]) : 5;
  const int d = argc > 3 ? atoi(argv[3]) : 8192;
  const int hq = argc > 4 ? atoi(argv[4]) : 64;
  const int hkv = argc > 5 ? atoi(argv[5]) : 8;
  const int F = argc > 6 ? atoi(argv[6]) : 28672;
  const int V = argc > 7 ? atoi(argv[7]) : 32000;
  const int dh = d / hq;
  struct Shape { const char* name; int N, K; };
  const Shape shapes[] = {{"qkv", (hq + 2 * hkv) * dh, d}, {"o", d, hq * dh}, {"gate_up", 2 * F, d},
                          {"down", d, F}, {"lm_head", V, d}};
  hipStream_t st;
  CK(hipStreamCreate(&st));
  size_t max_w = 0, max_work = 0, max_x = 0;
  for (const Shape& s : shapes) {
    size_t b = spec_packed_bytes(s.N, s.K);
    if (b > max_w) max_w = b;
    size_t w = spec_gemm_workspace_bytes(M, s.N, s.K);
    if (w > max_work) max_work = w;
    if ((size_t)M * s.K * 2 > max_x) max_x = (size_t)M * s.K * 2;
  }
  // two weight buffers used alternately, so that a launch never finds its matrix in a cache
  void *w[2], *x, *work, *out, *rowmajor;
  CK(hipMalloc(&w[0], max_w));
  CK(hipMalloc(&w[1], max_w));
  CK(hipMalloc(&rowmajor, max_w));
  CK(hipMalloc(&x, max_x));
  CK(hipMalloc(&work, max_work));
  CK(hipMalloc(&out, 256));
  CK(hipMemset(w[0], 0x3c, max_w));
  CK(hipMemset(w[1], 0x3c, max_w));
  CK(hipMemset(rowmajor, 0x3c, max_w));
  CK(hipMemset(x, 0x3c, max_x));
  CK(hipMemset(out, 0, 256));
  CK(hipDeviceSynchronize());
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  printf("projection probe: M=%d, %d launches per shape\n", M, iters);
  for (const Shape& s : shapes) {
    const size_t bytes = spec_packed_bytes(s.N, s.K);
    SK(spec_gemm_partials(x, w[0], M, s.N, s.K, work, st));   // warm-up
    CK(hipEventRecord(e0, st));
    for (int i = 0; i < iters; ++i) SK(spec_gemm_partials(x, w[(i + 1) & 1], M, s.N, s.K, work, st));
    CK(hipEventRecord(e1, st));
    CK(hipStreamSynchronize(st));
    float ms = 0.f;
    CK(hipEventElapsedTime(&ms, e0, e1));
    printf("  %-8s N=%6d K=%6d  weight %9.3f MB  %8.2f us  %7.1f GB/s\n", s.name, s.N, s.K, bytes / 1e6,
           ms / iters * 1e3, bytes / (ms / iters * 1e-3) / 1e9);
  }
  // calibration launches of known size: a pure read of max_w bytes, and a copy (read + write) of the gate/up matrix
  for (int i = 0; i < 3; ++i) SK(spec_read_probe(w[i & 1], max_w, out, st));
  for (int i = 0; i < 3; ++i) SK(spec_pack_weight(w[i & 1], rowmajor, 2 * F, d, 0, 1, st));
  CK(hipStreamSynchronize(st));
  printf("calibration: read_probe_kernel reads %zu bytes; pack_weight_kernel reads and writes %zu bytes\n", max_w,
         spec_packed_bytes(2 * F, d));
  return 0;
}
