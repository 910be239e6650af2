// Shape-agnostic kernels for the LoCoCo segment step: any head_dim, cache
// size, block length and filter width, fp32 or bf16 storage, fp32 arithmetic.
// They are the fp32 path of the library and the fallback for shapes the MFMA
// kernels do not take.  One thread (or one workgroup) per output element,
// straight from the definitions (Eq. 1, Eq. 4a/4b, Eq. 5, Eq. 6).
#include <algorithm>

#include "lococo_internal.h"

namespace lococo {
namespace {

struct bf16_t { uint16_t x; };

__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return __uint_as_float((uint32_t)v.x << 16); }

__device__ __forceinline__ void from_f(float f, float* out) { *out = f; }
__device__ __forceinline__ void from_f(float f, bf16_t* out) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) { out->x = (uint16_t)((u >> 16) | 0x40); return; }  // NaN
  u += 0x7fffu + ((u >> 16) & 1u);   // round to nearest, ties to even
  out->x = (uint16_t)(u >> 16);
}

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// Block-wide reductions over kThreads threads; red is kWaves floats of LDS.
__device__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r = fmaxf(r, red[w]);
  return r;
}
__device__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
#pragma unroll
  for (int w = 1; w < kWaves; ++w) r += red[w];
  return r;
}

// Row j of [cache ; block] for chain (b, hkv): cache rows first (Eq. 3 order).
template <typename T>
__device__ __forceinline__ const T* cat_row(const void* cache, const View& blk, int M, int d,
                                            int m, int b, int hkv, int Hkv, int j) {
  if (j < m) return (const T*)cache + ((int64_t)(b * Hkv + hkv) * M + j) * d;
  return (const T*)blk.p + b * blk.sb + hkv * blk.sh + (int64_t)(j - m) * blk.st;
}

// Alg. 2 step 3 / Eq. 1: one workgroup per (query row, query head, batch).
template <typename T>
__global__ __launch_bounds__(kThreads) void attn_generic_k(StepArgs a) {
  extern __shared__ float sm[];
  float* qs = sm;                 // d
  float* sc = sm + a.d;           // m + Bn
  __shared__ float red[kWaves];
  const int r = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int hkv = hq / a.group;
  const int n_vis = a.m + r + 1;  // all cache slots + block keys up to the diagonal
  const T* q = (const T*)a.q.p + b * a.q.sb + hq * a.q.sh + (int64_t)r * a.q.st;
  for (int c = threadIdx.x; c < a.d; c += kThreads) qs[c] = to_f(q[c]);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < n_vis; j += kThreads) {
    const T* kr = cat_row<T>(a.cache_k, a.k, a.M, a.d, a.m, b, hkv, a.Hkv, j);
    float acc = 0.f;
    for (int c = 0; c < a.d; ++c) acc += qs[c] * to_f(kr[c]);
    acc *= a.scale;
    sc[j] = acc;
    mx = fmaxf(mx, acc);
  }
  mx = block_max(mx, red);
  float z = 0.f;
  for (int j = threadIdx.x; j < n_vis; j += kThreads) {
    float e = expf(sc[j] - mx);
    sc[j] = e;
    z += e;
  }
  z = block_sum(z, red);
  __syncthreads();
  if (a.colsum) {                 // accumulated attention per live cache slot
    float* cs = a.colsum + (int64_t)(b * a.Hkv + hkv) * a.M;
    for (int j = threadIdx.x; j < a.m; j += kThreads) atomicAdd(cs + j, sc[j] / z);
  }
  T* o = (T*)a.o.p + b * a.o.sb + hq * a.o.sh + (int64_t)r * a.o.st;
  for (int c = threadIdx.x; c < a.d; c += kThreads) {
    float acc = 0.f;
    for (int j = 0; j < n_vis; ++j) {
      const T* vr = cat_row<T>(a.cache_v, a.v, a.M, a.d, a.m, b, hkv, a.Hkv, j);
      acc += sc[j] * to_f(vr[c]);
    }
    from_f(acc / z, o + c);
  }
}

// Alg. 2 IF branch: append the block's K and V at slots [m, m + Bn).
template <typename T>
__global__ __launch_bounds__(kThreads) void fill_generic_k(StepArgs a) {
  const int ch = blockIdx.y, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int n = a.Bn * a.d;
  for (int e = blockIdx.x * kThreads + threadIdx.x; e < n; e += gridDim.x * kThreads) {
    int t = e / a.d, c = e % a.d;
    int64_t dst = ((int64_t)ch * a.M + a.m + t) * a.d + c;
    ((T*)a.new_k)[dst] = ((const T*)a.k.p)[b * a.k.sb + hkv * a.k.sh + (int64_t)t * a.k.st + c];
    ((T*)a.new_v)[dst] = ((const T*)a.v.p)[b * a.v.sb + hkv * a.v.sh + (int64_t)t * a.v.st + c];
  }
}

// Eq. 5: W[i, j] = bias[i] + sum_c sum_tau Wc[i, c, tau] X[j + tau - (k-1)/2, c],
// zero outside [0, T).  An implicit GEMM with inner dimension C*k, tiled through LDS: a workgroup
// owns 64 slots x 64 positions, a thread 4 x 4 of them; the inner dimension is walked in chunks of
// 8 channels x 16 taps.  For a fixed channel a thread keeps the 4 + 15 positions its taps touch
// in registers, so each LDS value feeds several multiply-adds.
constexpr int kTI = 64, kTJ = 64, kCC = 8, kTK = 16;
template <typename T>
__global__ __launch_bounds__(kThreads) void conv_logits_generic_k(StepArgs a, float* logits) {
  __shared__ float Ws[kCC][kTK][kTI + 4];            // [channel][tap][slot]
  __shared__ float Xs[kCC][kTJ + kTK + 4];           // [channel][row], rows j0 + t0 - pad ..
  const int Tn = a.m + a.Bn;
  const int j0 = blockIdx.x * kTJ, i0 = blockIdx.y * kTI, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int C = a.conv_in ? 2 * a.d : a.d, k = a.k_width, pad = (k - 1) / 2;
  const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
  const T* wbase = (const T*)a.conv_w + hkv * a.w_head_stride;
  float acc[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) acc[ii][jj] = 0.f;
  for (int c0 = 0; c0 < C; c0 += kCC)
    for (int t0 = 0; t0 < k; t0 += kTK) {
      __syncthreads();
      for (int e = threadIdx.x; e < kCC * kTK * kTI; e += kThreads) {
        const int t = e % kTK, c = (e / kTK) % kCC, i = e / (kTK * kCC);
        float v = 0.f;
        if (i0 + i < a.M && c0 + c < C && t0 + t < k)
          v = to_f(wbase[((int64_t)(i0 + i) * C + c0 + c) * k + t0 + t]);
        Ws[c][t][i] = v;
      }
      for (int e = threadIdx.x; e < kCC * (kTJ + kTK - 1); e += kThreads) {
        const int c = e % kCC, r = e / kCC, jj = j0 + t0 - pad + r;
        float v = 0.f;
        if (jj >= 0 && jj < Tn && c0 + c < C) {
          const int cc = c0 + c;
          v = cc < a.d ? to_f(cat_row<T>(a.cache_k, a.k, a.M, a.d, a.m, b, hkv, a.Hkv, jj)[cc])
                       : to_f(cat_row<T>(a.cache_v, a.v, a.M, a.d, a.m, b, hkv, a.Hkv, jj)[cc - a.d]);
          if (a.norm == 2) v = fmaxf(v, 0.f);          // the rectifier in front of the convolution layer
        }
        Xs[c][r] = v;
      }
      __syncthreads();
#pragma unroll
      for (int c = 0; c < kCC; ++c) {
        float x[4 + kTK - 1];
#pragma unroll
        for (int r = 0; r < 4 + kTK - 1; ++r) x[r] = Xs[c][tj * 4 + r];
#pragma unroll
        for (int t = 0; t < kTK; ++t) {
          const float4 wv = *(const float4*)&Ws[c][t][ti * 4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            acc[0][jj] = fmaf(wv.x, x[jj + t], acc[0][jj]);
            acc[1][jj] = fmaf(wv.y, x[jj + t], acc[1][jj]);
            acc[2][jj] = fmaf(wv.z, x[jj + t], acc[2][jj]);
            acc[3][jj] = fmaf(wv.w, x[jj + t], acc[3][jj]);
          }
        }
      }
    }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii) {
    const int i = i0 + ti * 4 + ii;
    if (i >= a.M) continue;
    const float bias = a.conv_b ? to_f(((const T*)a.conv_b)[hkv * a.b_head_stride + i]) : 0.f;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = j0 + tj * 4 + jj;
      if (j < Tn) logits[((int64_t)ch * a.M + i) * (a.ldw ? a.ldw : Tn) + j] = acc[ii][jj] + bias;
    }
  }
}

__global__ __launch_bounds__(kThreads) void normalise_generic_k(StepArgs a, float* logits) {
  __shared__ float red[kWaves];
  const int Tn = a.m + a.Bn;
  float* row = logits + ((int64_t)blockIdx.y * a.M + blockIdx.x) * (a.ldw ? a.ldw : Tn);
  if (a.norm == 0) {
    float mx = -INFINITY;
    for (int j = threadIdx.x; j < Tn; j += kThreads) mx = fmaxf(mx, row[j]);
    mx = block_max(mx, red);
    float z = 0.f;
    for (int j = threadIdx.x; j < Tn; j += kThreads) {
      float e = expf(row[j] - mx);
      row[j] = e;
      z += e;
    }
    z = block_sum(z, red);
    for (int j = threadIdx.x; j < Tn; j += kThreads) row[j] /= z;
  } else if (a.norm == 1) {
    float z = 0.f;
    for (int j = threadIdx.x; j < Tn; j += kThreads) {
      float e = fmaxf(row[j], 0.f);
      row[j] = e;
      z += e;
    }
    z = block_sum(z, red) + a.eps;
    for (int j = threadIdx.x; j < Tn; j += kThreads) row[j] /= z;
  } else {
    // Eq. 6 as printed: W / sum(W); excluded positions (-inf) carry no weight; a vanishing signed
    // sum is replaced by +-eps
    float z = 0.f;
    for (int j = threadIdx.x; j < Tn; j += kThreads) {
      const float e = isfinite(row[j]) ? row[j] : 0.f;
      row[j] = e;
      z += e;
    }
    z = block_sum(z, red);
    if (fabsf(z) < a.eps) z = z < 0.f ? -a.eps : a.eps;
    for (int j = threadIdx.x; j < Tn; j += kThreads) row[j] /= z;
  }
}

// Eq. 4a / 4b: new_k[i] = sum_j w[i, j] [Kc ; K_n]_j and the same weights for V.
// With raw != 0 the rows of w are unnormalised logits and Eq. 6 is applied on
// the fly (used where the caller supplies the logits and they must stay intact).
template <typename T>
__global__ __launch_bounds__(kThreads) void mix_generic_k(StepArgs a, const float* w, int raw) {
  __shared__ float red[kWaves];
  const int Tn = a.m + a.Bn;
  const int i = blockIdx.x, ch = blockIdx.y, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const float* wr = w + ((int64_t)ch * a.M + i) * (a.ldw ? a.ldw : Tn);
  float mx = 0.f, z = 1.f;
  if (raw) {
    if (a.norm == 0) {
      mx = -INFINITY;
      for (int j = threadIdx.x; j < Tn; j += kThreads) mx = fmaxf(mx, wr[j]);
      mx = block_max(mx, red);
      z = 0.f;
      for (int j = threadIdx.x; j < Tn; j += kThreads) z += expf(wr[j] - mx);
      z = block_sum(z, red);
    } else if (a.norm == 1) {
      z = 0.f;
      for (int j = threadIdx.x; j < Tn; j += kThreads) z += fmaxf(wr[j], 0.f);
      z = block_sum(z, red) + a.eps;
    } else {
      z = 0.f;
      for (int j = threadIdx.x; j < Tn; j += kThreads) z += isfinite(wr[j]) ? wr[j] : 0.f;
      z = block_sum(z, red);
      if (fabsf(z) < a.eps) z = z < 0.f ? -a.eps : a.eps;
    }
  }
  for (int e = threadIdx.x; e < 2 * a.d; e += kThreads) {
    const bool isv = e >= a.d;
    const int c = isv ? e - a.d : e;
    float acc = 0.f;
    for (int j = 0; j < Tn; ++j) {
      const T* y = cat_row<T>(isv ? a.cache_v : a.cache_k, isv ? a.v : a.k, a.M, a.d, a.m, b, hkv,
                              a.Hkv, j);
      float wj = wr[j];
      if (raw) wj = (a.norm == 0 ? expf(wj - mx) : a.norm == 1 ? fmaxf(wj, 0.f) : isfinite(wj) ? wj : 0.f) / z;
      acc += wj * to_f(y[c]);
    }
    T* dst = (T*)(isv ? a.new_v : a.new_k) + ((int64_t)ch * a.M + i) * a.d + c;
    from_f(acc, dst);
  }
}

// Protected slots (see lococo_cache.protect): positions of live protected slots get no weight ...
__device__ __forceinline__ bool slot_protected(const StepArgs& a, int ch, int i) {
  return i < a.m && ((a.protect[(int64_t)ch * a.protect_stride + (i >> 5)] >> (i & 31)) & 1u);
}
__global__ __launch_bounds__(kThreads) void protect_logits_generic_k(StepArgs a, float* logits) {
  const int Tn = a.m + a.Bn, ch = blockIdx.y;
  const int ld = a.ldw ? a.ldw : Tn;
  float* rows = logits + (int64_t)ch * a.M * ld;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < (int64_t)a.M * a.m;
       e += (int64_t)gridDim.x * kThreads) {
    const int i = (int)(e / a.m), j = (int)(e % a.m);
    if (slot_protected(a, ch, j)) rows[(int64_t)i * ld + j] = -INFINITY;
  }
}
// ... and the rows of live protected slots are carried over from the old cache.
template <typename T>
__global__ __launch_bounds__(kThreads) void protect_rows_generic_k(StepArgs a) {
  const int ch = blockIdx.y;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < (int64_t)a.m * a.d;
       e += (int64_t)gridDim.x * kThreads) {
    const int i = (int)(e / a.d);
    if (!slot_protected(a, ch, i)) continue;
    const int64_t at = (int64_t)ch * a.M * a.d + e;
    ((T*)a.new_k)[at] = ((const T*)a.cache_k)[at];
    ((T*)a.new_v)[at] = ((const T*)a.cache_v)[at];
  }
}

}  // namespace

// scores (T floats) + query row (d <= 1024 floats) stay within 60 KB of LDS
int generic_attn_max_T() { return 14336; }

hipError_t launch_attn_generic(int dtype, const StepArgs& a, hipStream_t s) {
  dim3 grid(a.Bn, a.Hq, a.batch);
  size_t lds = sizeof(float) * (size_t)(a.d + a.m + a.Bn);
  if (dtype == LOCOCO_F32)
    hipLaunchKernelGGL(attn_generic_k<float>, grid, dim3(kThreads), lds, s, a);
  else
    hipLaunchKernelGGL(attn_generic_k<bf16_t>, grid, dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_fill_generic(int dtype, const StepArgs& a, hipStream_t s) {
  int n = a.Bn * a.d;
  dim3 grid((n + kThreads - 1) / kThreads, a.batch * a.Hkv);
  if (grid.x > 64) grid.x = 64;
  if (dtype == LOCOCO_F32)
    hipLaunchKernelGGL(fill_generic_k<float>, grid, dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(fill_generic_k<bf16_t>, grid, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

// ---- two device-to-device copies of the same length in one launch (the final cache state, keys and values,
// from the scan's history to the caller's buffer: one kernel node instead of two copy nodes)
__global__ __launch_bounds__(kThreads) void copy_pair_k(uint4* d0, const uint4* s0, uint4* d1, const uint4* s1, size_t n16) {
  const size_t step = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += step) {
    d0[i] = s0[i];
    d1[i] = s1[i];
  }
}

// ---- zero-fill as a kernel (a memset node in a captured graph is not relied on)
__global__ __launch_bounds__(kThreads) void zero_fill_k(uint4* p, size_t n16) {
  const size_t step = (size_t)gridDim.x * kThreads;
  const uint4 z = {0u, 0u, 0u, 0u};
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n16; i += step) p[i] = z;
}

hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (((uintptr_t)p | (uintptr_t)bytes) & 15) return hipMemsetAsync(p, 0, bytes, s);   // (no caller here passes such a range)
  const size_t n16 = bytes / 16, blocks = (n16 + kThreads - 1) / kThreads;
  hipLaunchKernelGGL(zero_fill_k, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(kThreads), 0, s, (uint4*)p, n16);
  return hipGetLastError();
}

hipError_t launch_copy_pair(void* d0, const void* s0, void* d1, const void* s1, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  const uintptr_t bits = (uintptr_t)d0 | (uintptr_t)s0 | (uintptr_t)d1 | (uintptr_t)s1 | (uintptr_t)bytes;
  if (bits & 15) {                       // not all 16-byte aligned: the runtime's copies
    hipError_t e = hipMemcpyAsync(d0, s0, bytes, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(d1, s1, bytes, hipMemcpyDeviceToDevice, s);
  }
  const size_t n16 = bytes / 16;
  const size_t blocks = (n16 + kThreads - 1) / kThreads;
  hipLaunchKernelGGL(copy_pair_k, dim3((unsigned)(blocks < 2048 ? blocks : 2048)), dim3(kThreads), 0, s, (uint4*)d0,
                     (const uint4*)s0, (uint4*)d1, (const uint4*)s1, n16);
  return hipGetLastError();
}

hipError_t launch_conv_logits_generic(int dtype, const StepArgs& a, float* logits, hipStream_t s) {
  const int Tn = a.m + a.Bn;
  dim3 grid((Tn + kTJ - 1) / kTJ, (a.M + kTI - 1) / kTI, a.batch * a.Hkv);
  if (dtype == LOCOCO_F32)
    hipLaunchKernelGGL(conv_logits_generic_k<float>, grid, dim3(kThreads), 0, s, a, logits);
  else
    hipLaunchKernelGGL(conv_logits_generic_k<bf16_t>, grid, dim3(kThreads), 0, s, a, logits);
  return hipGetLastError();
}

hipError_t launch_normalise_generic(const StepArgs& a, float* logits, hipStream_t s) {
  dim3 grid(a.M, a.batch * a.Hkv);
  hipLaunchKernelGGL(normalise_generic_k, grid, dim3(kThreads), 0, s, a, logits);
  return hipGetLastError();
}

hipError_t launch_protect_logits_generic(const StepArgs& a, float* logits, hipStream_t s) {
  if (a.m == 0) return hipSuccess;
  const int64_t n = (int64_t)a.M * a.m;
  dim3 grid((unsigned)std::min<int64_t>((n + kThreads - 1) / kThreads, 1024), a.batch * a.Hkv);
  hipLaunchKernelGGL(protect_logits_generic_k, grid, dim3(kThreads), 0, s, a, logits);
  return hipGetLastError();
}

hipError_t launch_protect_rows_generic(int dtype, const StepArgs& a, hipStream_t s) {
  if (a.m == 0) return hipSuccess;
  const int64_t n = (int64_t)a.m * a.d;
  dim3 grid((unsigned)std::min<int64_t>((n + kThreads - 1) / kThreads, 1024), a.batch * a.Hkv);
  if (dtype == LOCOCO_F32)
    hipLaunchKernelGGL(protect_rows_generic_k<float>, grid, dim3(kThreads), 0, s, a);
  else
    hipLaunchKernelGGL(protect_rows_generic_k<bf16_t>, grid, dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_mix_generic(int dtype, const StepArgs& a, const float* w, int raw,
                              hipStream_t s) {
  dim3 grid(a.M, a.batch * a.Hkv);
  if (dtype == LOCOCO_F32)
    hipLaunchKernelGGL(mix_generic_k<float>, grid, dim3(kThreads), 0, s, a, w, raw);
  else
    hipLaunchKernelGGL(mix_generic_k<bf16_t>, grid, dim3(kThreads), 0, s, a, w, raw);
  return hipGetLastError();
}

}  // namespace lococo
