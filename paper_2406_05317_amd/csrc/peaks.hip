// What this GPU sustains on the two rooflines the library's kernels are measured against: a bare
// bf16 MFMA loop (no memory traffic, four independent accumulator chains per wave, one wave per
// SIMD and two, whichever is faster) and a plain copy.  A measurement aid for benchmarks: it
// implements no step of the method.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kChains = 4;        // independent accumulators per wave: the matrix pipe never waits on a result
constexpr int kMfmaFlops = 2 * 32 * 32 * 16;

__global__ __launch_bounds__(256) void mfma_loop_k(int iters, float* sink) {
  // Operands with random signs, mantissas and low exponent bits (values in +-[0.5, 2)), different
  // in every lane and for each of the four unrolled steps: the power the matrix pipe draws, and
  // with it the clock the chip holds, depends on how many operand bits toggle.
  typedef __attribute__((__vector_size__(8 * sizeof(uint16_t)))) uint16_t u16x8;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    u16x8 ra, rb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      uint32_t h = (threadIdx.x * 64u + u * 16u + i) * 2654435761u + blockIdx.x * 40503u;
      h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
      ra[i] = (uint16_t)((h & 0x80ffu) | 0x3f00u);
      rb[i] = (uint16_t)(((h >> 16) & 0x80ffu) | 0x3f00u);
    }
    a[u] = __builtin_bit_cast(bf16x8, ra);
    b[u] = __builtin_bit_cast(bf16x8, rb);
  }
  f32x16 acc[kChains];
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], b[u], acc[c], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kChains; ++c)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[c][i];
  if (s == 12345.678f) *sink = s;     // keeps the loop alive; never true in practice, and harmless if it is
}

__global__ __launch_bounds__(256) void copy_k(const u32x4* src, u32x4* dst, int64_t n16) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n16; i += (int64_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

__global__ void fill_k(uint32_t* p, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    p[i] = (uint32_t)i * 2654435761u;
}

template <class Launch>
hipError_t timed(hipStream_t s, int reps, float* ms_out, const Launch& launch) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  hipError_t e = hipEventCreate(&e0);
  if (e == hipSuccess) e = hipEventCreate(&e1);
  if (e == hipSuccess) {
    launch();                                   // warm-up: code object load, clocks
    e = hipEventRecord(e0, s);
    for (int r = 0; r < reps; ++r) launch();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms_out, e0, e1);
    if (e == hipSuccess) e = hipGetLastError();
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  if (e == hipSuccess) *ms_out /= (float)reps;
  return e;
}

}  // namespace

hipError_t measure_peaks(void* scratch, size_t bytes, int n_cu, hipStream_t s, double* mfma_tflops,
                         double* copy_gbs) {
  // ---- matrix pipe: 1 and 2 waves per SIMD (4 and 8 waves per compute unit).  Launches of >= 14 ms,
  // four in a row: long enough for the clock to settle where the power limit puts it under matrix
  // load (a burst of a millisecond still runs at the full 2.4 GHz and reads 10 - 15 % higher).
  const int iters = 65536;
  double best = 0.0;
  for (int wgs_per_cu = 1; wgs_per_cu <= 2; ++wgs_per_cu) {
    const int grid = n_cu * wgs_per_cu;
    float ms = 0.f;
    hipError_t e = timed(s, 3, &ms, [&] {
      hipLaunchKernelGGL(mfma_loop_k, dim3(grid), dim3(256), 0, s, iters, (float*)scratch);
    });
    if (e != hipSuccess) return e;
    const double flops = (double)grid * 4 /*waves*/ * iters * 4 /*unroll*/ * kChains * kMfmaFlops;
    const double tf = flops / (ms * 1e-3) / 1e12;
    if (tf > best) best = tf;
  }
  *mfma_tflops = best;

  // ---- memory: first half of the scratch buffer to the second half (reads + writes counted)
  const int64_t half16 = (int64_t)(bytes / 2 / 16);
  u32x4* src = (u32x4*)scratch;
  u32x4* dst = src + half16;
  hipLaunchKernelGGL(fill_k, dim3(n_cu * 8), dim3(256), 0, s, (uint32_t*)scratch, half16 * 4);
  float ms = 0.f;
  hipError_t e = timed(s, 5, &ms, [&] {
    hipLaunchKernelGGL(copy_k, dim3(n_cu * 16), dim3(256), 0, s, src, dst, half16);
  });
  if (e != hipSuccess) return e;
  *copy_gbs = 2.0 * (double)half16 * 16.0 / (ms * 1e-3) / 1e9;
  return hipSuccess;
}

}  // namespace lococo
