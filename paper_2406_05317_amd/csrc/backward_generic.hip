// Backward pass of one block step (training the convolution heads through
// the scan): chain rule on Alg. 2 step 3 (Eq. 1), the fill branch, and
// Eq. 5 / Eq. 6 / Eq. 4a-4b.  Shape-agnostic, fp32 arithmetic, fp32 gradients;
// inputs in the storage dtype (fp32 or bf16), storage rounding treated as the
// identity.  The contractions are tiled through LDS (64 x 64 outputs per
// workgroup); the row reductions between them are one workgroup per row.
//
// Notation (one chain): Y = [cache(0:m) ; block] (T = m + Bn rows) for K and V,
// P the attention rows, w the mixing rows (Eq. 6), g_k / g_v the gradients of
// the new cache.
//   attention:  dS[r,j] = P[r,j] (dO[r].Yv[j] - sum_j' P[r,j'] dO[r].Yv[j']) * scale
//               dq[r] = sum_j dS[r,j] Yk[j],  dYk[j] += sum_r dS[r,j] q[r],  dYv[j] += sum_r P[r,j] dO[r]
//   fusion:     dw[i,j] = g_k[i].Yk[j] + g_v[i].Yv[j],  dYk[j] += sum_i w[i,j] g_k[i]  (same for V)
//   Eq. 6:      softmax: dW[i,j] = w[i,j] (dw[i,j] - sum_j' w dw);
//               relu-sum: dW[i,j] = [W[i,j] > 0] (dw[i,j] - sum_j' w dw) / (z_i + eps)
//   Eq. 5:      db[i] += sum_j dW[i,j],  dWc[i,c,t] += sum_j dW[i,j] X[j+t-p, c],
//               dX[j',c] += sum_i sum_t dW[i, j'-t+p] Wc[i,c,t]   (X = Yk, or [Yk | Yv])
#include <algorithm>

#include "lococo_internal.h"

namespace lococo {
namespace {

struct bf16_t { uint16_t x; };
__device__ __forceinline__ float to_f(float v) { return v; }
__device__ __forceinline__ float to_f(bf16_t v) { return __uint_as_float((uint32_t)v.x << 16); }

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
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

template <typename T>
__device__ __forceinline__ const T* cat_row(const void* cache, const View& blk, int M, int d, int m, int b,
                                            int hkv, int Hkv, int j) {
  if (j < m) return (const T*)cache + ((int64_t)(b * Hkv + hkv) * M + j) * d;
  return (const T*)blk.p + b * blk.sb + hkv * blk.sh + (int64_t)(j - m) * blk.st;
}
// where the gradient of row j of [cache ; block] lives
__device__ __forceinline__ float* grad_row(float* d_cache, float* d_blk, int M, int d, int m, int Bn, int ch,
                                           int j) {
  if (j < m) return d_cache + ((int64_t)ch * M + j) * d;
  return d_blk + ((int64_t)ch * Bn + (j - m)) * d;
}
__device__ __forceinline__ bool slot_protected(const StepArgs& a, int ch, int i) {
  return a.protect && i < a.m && ((a.protect[(int64_t)ch * a.protect_stride + (i >> 5)] >> (i & 31)) & 1u);
}

// ---- attention.  Its five contractions are GEMMs, tiled through LDS in fp32: 64 x 64 outputs per
// workgroup, 4 x 4 per thread, operands in chunks of 16 along the contraction; the softmax and its
// backward are row reductions between them, one workgroup per query row.
constexpr int kAT = 64, kAK = 16;

// scores S[r, j] = scale q[r] . Yk[j] and dP[r, j] = dO[r] . Yv[j]  (query rows x positions, over d);
// entries a query does not see are left to the row kernel
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_attn_scores_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Qs[kAK][kAT + 4], Os[kAK][kAT + 4];     // [column][query row]
  __shared__ float Ks[kAK][kAT + 4], Vs[kAK][kAT + 4];     // [column][position]
  const int Tn = a.m + a.Bn, d = a.d;
  const int j0 = blockIdx.x * kAT, r0 = blockIdx.y * kAT;
  const int hq = blockIdx.z % a.Hq, b = blockIdx.z / a.Hq, hkv = hq / a.group;
  if (j0 > a.m + r0 + kAT - 1) return;             // the whole tile lies after its queries
  const int tr = threadIdx.x / 16, tj = threadIdx.x % 16;
  const int64_t row0 = ((int64_t)b * a.Hq + hq) * a.Bn;
  float accs[4][4], accp[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) accs[ii][jj] = accp[ii][jj] = 0.f;
  for (int c0 = 0; c0 < d; c0 += kAK) {
    __syncthreads();
    for (int e = threadIdx.x; e < kAK * kAT; e += kThreads) {
      const int c = e % kAK, x = e / kAK, cc = c0 + c;
      float qv = 0.f, ov = 0.f, kv = 0.f, vv = 0.f;
      if (cc < d) {
        if (r0 + x < a.Bn) {
          qv = to_f(((const T*)a.q.p + b * a.q.sb + hq * a.q.sh + (int64_t)(r0 + x) * a.q.st)[cc]);
          ov = g.d_o[(row0 + r0 + x) * d + cc];
        }
        if (j0 + x < Tn) {
          kv = to_f(cat_row<T>(a.cache_k, a.k, a.M, d, a.m, b, hkv, a.Hkv, j0 + x)[cc]);
          vv = to_f(cat_row<T>(a.cache_v, a.v, a.M, d, a.m, b, hkv, a.Hkv, j0 + x)[cc]);
        }
      }
      Qs[c][x] = qv; Os[c][x] = ov; Ks[c][x] = kv; Vs[c][x] = vv;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kAK; ++c) {
      const float4 q4 = *(const float4*)&Qs[c][tr * 4], o4 = *(const float4*)&Os[c][tr * 4];
      const float4 k4 = *(const float4*)&Ks[c][tj * 4], v4 = *(const float4*)&Vs[c][tj * 4];
      const float qr[4] = {q4.x, q4.y, q4.z, q4.w}, orr[4] = {o4.x, o4.y, o4.z, o4.w};
      const float kr[4] = {k4.x, k4.y, k4.z, k4.w}, vr[4] = {v4.x, v4.y, v4.z, v4.w};
#pragma unroll
      for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          accs[ii][jj] = fmaf(qr[ii], kr[jj], accs[ii][jj]);
          accp[ii][jj] = fmaf(orr[ii], vr[jj], accp[ii][jj]);
        }
    }
  }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii) {
    const int r = r0 + tr * 4 + ii;
    if (r >= a.Bn) continue;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = j0 + tj * 4 + jj;
      if (j < Tn) {
        g.ws_p[(row0 + r) * Tn + j] = accs[ii][jj] * a.scale;
        g.ws_ds[(row0 + r) * Tn + j] = accp[ii][jj];
      }
    }
  }
}

// one workgroup per (query row r, query head, batch): P[r, :] from the scores, dS[r, :] from dP
__global__ __launch_bounds__(kThreads) void bwd_attn_rows_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float red[kWaves];
  const int r = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
  const int Tn = a.m + a.Bn, n_vis = a.m + r + 1;
  float* P = g.ws_p + (((int64_t)b * a.Hq + hq) * a.Bn + r) * Tn;
  float* dS = g.ws_ds + (((int64_t)b * a.Hq + hq) * a.Bn + r) * Tn;
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < n_vis; j += kThreads) mx = fmaxf(mx, P[j]);
  mx = block_max(mx, red);
  float z = 0.f;
  for (int j = threadIdx.x; j < n_vis; j += kThreads) z += expf(P[j] - mx);
  z = block_sum(z, red);
  float dot = 0.f;
  for (int j = threadIdx.x; j < n_vis; j += kThreads) {
    const float p = expf(P[j] - mx) / z;
    P[j] = p;
    dot += p * dS[j];
  }
  dot = block_sum(dot, red);
  for (int j = threadIdx.x; j < Tn; j += kThreads) {
    if (j < n_vis) {
      dS[j] = P[j] * (dS[j] - dot) * a.scale;
    } else {
      P[j] = 0.f;
      dS[j] = 0.f;
    }
  }
}

// dq[r, c] = sum_j dS[r, j] Yk[j, c]  (query rows x columns, over the positions)
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_attn_dq_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Ss[kAK][kAT + 4];               // [position][query row]
  __shared__ float Ys[kAK][kAT + 4];               // [position][column]
  const int Tn = a.m + a.Bn, d = a.d;
  const int c0 = blockIdx.x * kAT, r0 = blockIdx.y * kAT;
  const int hq = blockIdx.z % a.Hq, b = blockIdx.z / a.Hq, hkv = hq / a.group;
  const int tr = threadIdx.x / 16, tc = threadIdx.x % 16;
  const int64_t row0 = ((int64_t)b * a.Hq + hq) * a.Bn;
  const int jend = min(Tn, a.m + r0 + kAT);        // nothing to add after the tile's last query
  float acc[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[ii][q] = 0.f;
  for (int jc = 0; jc < jend; jc += kAK) {
    __syncthreads();
    for (int e = threadIdx.x; e < kAK * kAT; e += kThreads) {
      const int jj = e % kAK, x = e / kAK;         // dS rows are contiguous along the positions
      Ss[jj][x] = (r0 + x < a.Bn && jc + jj < Tn) ? g.ws_ds[(row0 + r0 + x) * Tn + jc + jj] : 0.f;
    }
    for (int e = threadIdx.x; e < kAK * kAT; e += kThreads) {
      const int x = e % kAT, jj = e / kAT;
      Ys[jj][x] = (jc + jj < Tn && c0 + x < d)
                      ? to_f(cat_row<T>(a.cache_k, a.k, a.M, d, a.m, b, hkv, a.Hkv, jc + jj)[c0 + x]) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int jj = 0; jj < kAK; ++jj) {
      const float4 s4 = *(const float4*)&Ss[jj][tr * 4], y4 = *(const float4*)&Ys[jj][tc * 4];
      const float sr[4] = {s4.x, s4.y, s4.z, s4.w}, yr[4] = {y4.x, y4.y, y4.z, y4.w};
#pragma unroll
      for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[ii][q] = fmaf(sr[ii], yr[q], acc[ii][q]);
    }
  }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii) {
    const int r = r0 + tr * 4 + ii;
    if (r >= a.Bn) continue;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + tc * 4 + q;
      if (c < d) g.d_q[(row0 + r) * d + c] = acc[ii][q];
    }
  }
}

// dYk[j, c] = sum over the group's heads and rows of dS[r, j] q[r, c], dYv[j, c] = sum of P[r, j] dO[r, c]
// (positions x columns, over the query rows; assigned, not added: the first contribution to those rows)
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_attn_cols_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Ss[kAK][kAT + 4], Ps[kAK][kAT + 4];     // [query row][position]
  __shared__ float Qs[kAK][kAT + 4], Os[kAK][kAT + 4];     // [query row][column]
  const int Tn = a.m + a.Bn, d = a.d;
  const int c0 = blockIdx.x * kAT, j0 = blockIdx.y * kAT, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int tj = threadIdx.x / 16, tc = threadIdx.x % 16;
  const int rbeg = j0 < a.m ? 0 : (j0 - a.m) / kAK * kAK;   // block key j' is visible to rows r >= j'
  float acck[4][4], accv[4][4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int q = 0; q < 4; ++q) acck[jj][q] = accv[jj][q] = 0.f;
  for (int hh = 0; hh < a.group; ++hh) {
    const int hq = hkv * a.group + hh;
    const int64_t row0 = ((int64_t)b * a.Hq + hq) * a.Bn;
    for (int rc = rbeg; rc < a.Bn; rc += kAK) {
      __syncthreads();
      for (int e = threadIdx.x; e < kAK * kAT; e += kThreads) {
        const int x = e % kAT, rr = e / kAT, r = rc + rr;
        const bool in = r < a.Bn && j0 + x < Tn;
        Ss[rr][x] = in ? g.ws_ds[(row0 + r) * Tn + j0 + x] : 0.f;
        Ps[rr][x] = in ? g.ws_p[(row0 + r) * Tn + j0 + x] : 0.f;
        const bool inc = r < a.Bn && c0 + x < d;
        Qs[rr][x] = inc ? to_f(((const T*)a.q.p + b * a.q.sb + hq * a.q.sh + (int64_t)r * a.q.st)[c0 + x]) : 0.f;
        Os[rr][x] = inc ? g.d_o[(row0 + r) * d + c0 + x] : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int rr = 0; rr < kAK; ++rr) {
        const float4 s4 = *(const float4*)&Ss[rr][tj * 4], p4 = *(const float4*)&Ps[rr][tj * 4];
        const float4 q4 = *(const float4*)&Qs[rr][tc * 4], o4 = *(const float4*)&Os[rr][tc * 4];
        const float sr[4] = {s4.x, s4.y, s4.z, s4.w}, pr[4] = {p4.x, p4.y, p4.z, p4.w};
        const float qr[4] = {q4.x, q4.y, q4.z, q4.w}, orr[4] = {o4.x, o4.y, o4.z, o4.w};
#pragma unroll
        for (int jj = 0; jj < 4; ++jj)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acck[jj][q] = fmaf(sr[jj], qr[q], acck[jj][q]);
            accv[jj][q] = fmaf(pr[jj], orr[q], accv[jj][q]);
          }
      }
    }
  }
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const int j = j0 + tj * 4 + jj;
    if (j >= Tn) continue;
    float* dk = grad_row(g.d_cache_k, g.d_k, a.M, d, a.m, a.Bn, ch, j);
    float* dv = grad_row(g.d_cache_v, g.d_v, a.M, d, a.m, a.Bn, ch, j);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + tc * 4 + q;
      if (c < d) {
        dk[c] = acck[jj][q];
        dv[c] = accv[jj][q];
      }
    }
  }
}

// rows of d_cache that are not live before the step carry no gradient
__global__ __launch_bounds__(kThreads) void bwd_zero_dead_rows_k(BwdArgs g) {
  const StepArgs& a = g.st;
  const int64_t per = (int64_t)(a.M - a.m) * a.d;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < per; e += (int64_t)gridDim.x * kThreads) {
    const int64_t at = ((int64_t)blockIdx.y * a.M + a.m) * a.d + e;
    g.d_cache_k[at] = 0.f;
    g.d_cache_v[at] = 0.f;
  }
}

// ---- fill branch: new cache = [cache ; block], so its gradient goes straight through
__global__ __launch_bounds__(kThreads) void bwd_fill_k(BwdArgs g) {
  const StepArgs& a = g.st;
  const int ch = blockIdx.y, Tn = a.m + a.Bn;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < (int64_t)Tn * a.d;
       e += (int64_t)gridDim.x * kThreads) {
    const int j = (int)(e / a.d), c = (int)(e % a.d);
    const int64_t at = ((int64_t)ch * a.M + j) * a.d + c;
    grad_row(g.d_cache_k, g.d_k, a.M, a.d, a.m, a.Bn, ch, j)[c] += g.d_new_k[at];
    grad_row(g.d_cache_v, g.d_v, a.M, a.d, a.m, a.Bn, ch, j)[c] += g.d_new_v[at];
  }
}

// ---- Eq. 4a/4b and Eq. 6.  The two contractions of the fusion are plain GEMMs and are tiled like
// the Eq. 5 ones below (64 x 64 outputs per workgroup, 4 x 4 per thread, operands through LDS in
// chunks of 16 along the contraction); the row reductions of Eq. 6 stay one workgroup per slot.
constexpr int kMT = 64, kMK = 16;

// dw[i, j] = g_k[i] . Yk[j] + g_v[i] . Yv[j]   (slots x positions, contraction over the 2 d columns)
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_mix_dw_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Gs[kMK][kMT + 4];               // [column][slot]
  __shared__ float Ys[kMK][kMT + 4];               // [column][position]
  const int Tn = a.m + a.Bn, d = a.d;
  const int j0 = blockIdx.x * kMT, i0 = blockIdx.y * kMT, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int ti = threadIdx.x / 16, tj = threadIdx.x % 16;
  float acc[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) acc[ii][jj] = 0.f;
  for (int c0 = 0; c0 < 2 * d; c0 += kMK) {        // columns of [K | V]; d is a multiple of 16 or the tail is zero-filled
    __syncthreads();
    for (int e = threadIdx.x; e < kMK * kMT; e += kThreads) {
      const int c = e % kMK, r = e / kMK, cc = c0 + c;
      float gv = 0.f, yv = 0.f;
      if (cc < 2 * d) {
        const bool val = cc >= d;
        const int col = val ? cc - d : cc;
        if (i0 + r < a.M) gv = (val ? g.d_new_v : g.d_new_k)[((int64_t)ch * a.M + i0 + r) * d + col];
        if (j0 + r < Tn)
          yv = val ? to_f(cat_row<T>(a.cache_v, a.v, a.M, d, a.m, b, hkv, a.Hkv, j0 + r)[col])
                   : to_f(cat_row<T>(a.cache_k, a.k, a.M, d, a.m, b, hkv, a.Hkv, j0 + r)[col]);
      }
      Gs[c][r] = gv;
      Ys[c][r] = yv;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMK; ++c) {
      const float4 gq = *(const float4*)&Gs[c][ti * 4];
      const float4 yq = *(const float4*)&Ys[c][tj * 4];
      const float gr[4] = {gq.x, gq.y, gq.z, gq.w}, yr[4] = {yq.x, yq.y, yq.z, yq.w};
#pragma unroll
      for (int ii = 0; ii < 4; ++ii)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) acc[ii][jj] = fmaf(gr[ii], yr[jj], acc[ii][jj]);
    }
  }
#pragma unroll
  for (int ii = 0; ii < 4; ++ii) {
    const int i = i0 + ti * 4 + ii;
    if (i >= a.M) continue;
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      const int j = j0 + tj * 4 + jj;
      if (j < Tn) g.ws_dw[((int64_t)ch * a.M + i) * Tn + j] = acc[ii][jj];
    }
  }
}

// Eq. 6 w.r.t. the logits, one workgroup per (slot i, chain): dW[i,:] from dw[i,:] and the
// normalised row, and the bias gradient; a protected slot passes its gradient to the old row instead
__global__ __launch_bounds__(kThreads) void bwd_mix_rows_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float red[kWaves];
  const int i = blockIdx.x, ch = blockIdx.y, hkv = ch % a.Hkv;
  const int Tn = a.m + a.Bn, d = a.d;
  float* Wraw = g.ws_w + ((int64_t)ch * a.M + i) * Tn;       // raw logits in, dW out
  const float* w = g.ws_n + ((int64_t)ch * a.M + i) * Tn;    // normalised rows
  const float* dw = g.ws_dw + ((int64_t)ch * a.M + i) * Tn;
  if (slot_protected(a, ch, i)) {
    const float* gk = g.d_new_k + ((int64_t)ch * a.M + i) * d;
    const float* gv = g.d_new_v + ((int64_t)ch * a.M + i) * d;
    float* dk = g.d_cache_k + ((int64_t)ch * a.M + i) * d;
    float* dv = g.d_cache_v + ((int64_t)ch * a.M + i) * d;
    for (int c = threadIdx.x; c < d; c += kThreads) {
      dk[c] += gk[c];
      dv[c] += gv[c];
    }
    for (int j = threadIdx.x; j < Tn; j += kThreads) Wraw[j] = 0.f;
    return;
  }
  float dot = 0.f, z = 0.f;
  for (int j = threadIdx.x; j < Tn; j += kThreads) {
    dot += w[j] * dw[j];
    z += fmaxf(Wraw[j], 0.f);
  }
  dot = block_sum(dot, red);
  z = block_sum(z, red) + a.eps;
  float bsum = 0.f;
  for (int j = threadIdx.x; j < Tn; j += kThreads) {
    const float dW = a.norm == 0 ? w[j] * (dw[j] - dot) : (Wraw[j] > 0.f ? (dw[j] - dot) / z : 0.f);
    Wraw[j] = dW;
    bsum += dW;
  }
  bsum = block_sum(bsum, red);
  if (threadIdx.x == 0 && g.d_conv_b) atomicAdd(g.d_conv_b + hkv * a.b_head_stride + i, bsum);
}

// ---- Eq. 4a/4b w.r.t. the inputs: dYk[j] += sum_i w[i,j] g_k[i], same for V
// (positions x columns of [K | V], contraction over the unprotected slots)
__global__ __launch_bounds__(kThreads) void bwd_mix_cols_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Ws[kMK][kMT + 4];               // [slot][position]
  __shared__ float Gs[kMK][kMT + 4];               // [slot][column]
  const int Tn = a.m + a.Bn, d = a.d;
  const int c0 = blockIdx.x * kMT, j0 = blockIdx.y * kMT, ch = blockIdx.z;
  const int tj = threadIdx.x / 16, tc = threadIdx.x % 16;
  float acc[4][4];
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[jj][q] = 0.f;
  for (int s0 = 0; s0 < a.M; s0 += kMK) {
    __syncthreads();
    for (int e = threadIdx.x; e < kMK * kMT; e += kThreads) {
      const int x = e % kMT, r = e / kMT, i = s0 + r;
      const bool live = i < a.M && !slot_protected(a, ch, i);
      Ws[r][x] = live && j0 + x < Tn ? g.ws_n[((int64_t)ch * a.M + i) * Tn + j0 + x] : 0.f;
      const int cc = c0 + x;
      float gv = 0.f;
      if (live && cc < 2 * d)
        gv = cc < d ? g.d_new_k[((int64_t)ch * a.M + i) * d + cc] : g.d_new_v[((int64_t)ch * a.M + i) * d + cc - d];
      Gs[r][x] = gv;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kMK; ++r) {
      const float4 wq = *(const float4*)&Ws[r][tj * 4];
      const float4 gq = *(const float4*)&Gs[r][tc * 4];
      const float wr[4] = {wq.x, wq.y, wq.z, wq.w}, gr[4] = {gq.x, gq.y, gq.z, gq.w};
#pragma unroll
      for (int jj = 0; jj < 4; ++jj)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[jj][q] = fmaf(wr[jj], gr[q], acc[jj][q]);
    }
  }
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const int j = j0 + tj * 4 + jj;
    if (j >= Tn) continue;
    float* dk = grad_row(g.d_cache_k, g.d_k, a.M, d, a.m, a.Bn, ch, j);
    float* dv = grad_row(g.d_cache_v, g.d_v, a.M, d, a.m, a.Bn, ch, j);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + tc * 4 + q;
      if (c < d) dk[c] += acc[jj][q];
      else if (c < 2 * d) dv[c - d] += acc[jj][q];
    }
  }
}

// The two Eq. 5 gradients are implicit GEMMs like the forward logits and are tiled the same way:
// 64 x 64 outputs per workgroup, 4 x 4 per thread, operands through LDS, and along the Toeplitz
// direction a thread slides a 4-value register window so that one new LDS value serves 16
// multiply-adds.
constexpr int kTI = 64, kTK = 16;

// ---- Eq. 5 w.r.t. the filters: dWc[i, c, t] += sum_j dW[i, j] X[j + t - p, c].  Rows: 64 slots;
// columns: 4 channels x 16 taps; contraction over the positions in chunks of 32.
constexpr int kWC = 4, kJC = 32;
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_conv_w_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float dWs[kJC][kTI + 4];                 // [position][slot]
  __shared__ float Xs[kWC][kJC + kTK + 4];            // [channel][row], rows jc + t0 - pad ..
  const int Tn = a.m + a.Bn, d = a.d, C = a.conv_in ? 2 * d : d, k = a.k_width, pad = (k - 1) / 2;
  const int ntk = (k + kTK - 1) / kTK;
  const int c0 = (blockIdx.x / ntk) * kWC, t0 = (blockIdx.x % ntk) * kTK, i0 = blockIdx.y * kTI;
  const int ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int ti = threadIdx.x / 16, tc = (threadIdx.x % 16) / 4, tt = (threadIdx.x % 4) * 4;
  float acc[4][4];
#pragma unroll
  for (int ii = 0; ii < 4; ++ii)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[ii][q] = 0.f;
  for (int jc = 0; jc < Tn; jc += kJC) {
    __syncthreads();
    for (int e = threadIdx.x; e < kJC * kTI; e += kThreads) {
      const int j = e % kJC, i = e / kJC;
      dWs[j][i] = (i0 + i < a.M && jc + j < Tn) ? g.ws_w[((int64_t)ch * a.M + i0 + i) * Tn + jc + j] : 0.f;
    }
    for (int e = threadIdx.x; e < kWC * (kJC + kTK - 1); e += kThreads) {
      const int c = e % kWC, r = e / kWC, jj = jc + t0 - pad + r, cc = c0 + c;
      float v = 0.f;
      if (jj >= 0 && jj < Tn && cc < C)
        v = cc < d ? to_f(cat_row<T>(a.cache_k, a.k, a.M, d, a.m, b, hkv, a.Hkv, jj)[cc])
                   : to_f(cat_row<T>(a.cache_v, a.v, a.M, d, a.m, b, hkv, a.Hkv, jj)[cc - d]);
      Xs[c][r] = v;
    }
    __syncthreads();
    // x[q] = X row (j + tt + q): slides by one row per position
    float x0 = Xs[tc][tt], x1 = Xs[tc][tt + 1], x2 = Xs[tc][tt + 2], x3;
#pragma unroll 8
    for (int j = 0; j < kJC; ++j) {
      x3 = Xs[tc][j + tt + 3];
      const float4 wv = *(const float4*)&dWs[j][ti * 4];
      const float wr[4] = {wv.x, wv.y, wv.z, wv.w};
#pragma unroll
      for (int ii = 0; ii < 4; ++ii) {
        acc[ii][0] = fmaf(wr[ii], x0, acc[ii][0]);
        acc[ii][1] = fmaf(wr[ii], x1, acc[ii][1]);
        acc[ii][2] = fmaf(wr[ii], x2, acc[ii][2]);
        acc[ii][3] = fmaf(wr[ii], x3, acc[ii][3]);
      }
      x0 = x1; x1 = x2; x2 = x3;
    }
  }
  const int c = c0 + tc;
  if (c < C) {
#pragma unroll
    for (int ii = 0; ii < 4; ++ii) {
      const int i = i0 + ti * 4 + ii;
      if (i >= a.M) continue;
      float* out = g.d_conv_w + hkv * a.w_head_stride + ((int64_t)i * C + c) * k;
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (t0 + tt + q < k) atomicAdd(out + t0 + tt + q, acc[ii][q]);
    }
  }
}

// ---- Eq. 5 w.r.t. its input: dX[j, c] += sum_i sum_t dW[i, j - t + p] Wc[i, c, t].  Rows: 64
// positions; columns: 64 channels; contraction over (slot, tap) in chunks of 8 slots x 16 taps.
constexpr int kIC = 8;
template <typename T>
__global__ __launch_bounds__(kThreads) void bwd_conv_x_k(BwdArgs g) {
  const StepArgs& a = g.st;
  __shared__ float Ds[kIC][kTI + kTK + 4];            // [slot][position], positions j0 - t0 - (kTK-1) + pad ..
  __shared__ float Ws[kIC][kTK][kTI + 4];             // [slot][tap][channel]
  const int Tn = a.m + a.Bn, d = a.d, C = a.conv_in ? 2 * d : d, k = a.k_width, pad = (k - 1) / 2;
  const int j0 = blockIdx.x * kTI, c0 = blockIdx.y * kTI, ch = blockIdx.z, hkv = ch % a.Hkv;
  const int tj = threadIdx.x / 16, tc = threadIdx.x % 16;
  const T* wbase = (const T*)a.conv_w + hkv * a.w_head_stride;
  float acc[4][4];                                     // [position][channel]
#pragma unroll
  for (int jj = 0; jj < 4; ++jj)
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[jj][q] = 0.f;
  for (int i0 = 0; i0 < a.M; i0 += kIC)
    for (int t0 = 0; t0 < k; t0 += kTK) {
      __syncthreads();
      // Ds[i][r] = dW[i0 + i, base + r], base = j0 + pad - t0 - (kTK - 1): tap t0 + t of position
      // j0 + p reads r = p + (kTK - 1) - t
      const int base = j0 + pad - t0 - (kTK - 1);
      for (int e = threadIdx.x; e < kIC * (kTI + kTK - 1); e += kThreads) {
        const int r = e % (kTI + kTK - 1), i = e / (kTI + kTK - 1), jj = base + r;
        Ds[i][r] = (i0 + i < a.M && jj >= 0 && jj < Tn) ? g.ws_w[((int64_t)ch * a.M + i0 + i) * Tn + jj] : 0.f;
      }
      for (int e = threadIdx.x; e < kIC * kTK * kTI; e += kThreads) {
        const int t = e % kTK, c = (e / kTK) % kTI, i = e / (kTK * kTI);
        float v = 0.f;
        if (i0 + i < a.M && c0 + c < C && t0 + t < k) v = to_f(wbase[((int64_t)(i0 + i) * C + c0 + c) * k + t0 + t]);
        Ws[i][t][c] = v;
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < kIC; ++i) {
        // window over r for positions tj*4 .. tj*4+3 at tap t: r = p + (kTK-1) - t; walk t downwards
        // so that the window slides up by one per tap
        float w0, w1 = Ds[i][tj * 4 + 0], w2 = Ds[i][tj * 4 + 1], w3 = Ds[i][tj * 4 + 2];
#pragma unroll
        for (int t = kTK - 1; t >= 0; --t) {
          w0 = w1; w1 = w2; w2 = w3;
          w3 = Ds[i][tj * 4 + 3 + (kTK - 1) - t];
          const float4 fv = *(const float4*)&Ws[i][t][tc * 4];
          const float fr[4] = {fv.x, fv.y, fv.z, fv.w};
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            acc[0][q] = fmaf(w0, fr[q], acc[0][q]);
            acc[1][q] = fmaf(w1, fr[q], acc[1][q]);
            acc[2][q] = fmaf(w2, fr[q], acc[2][q]);
            acc[3][q] = fmaf(w3, fr[q], acc[3][q]);
          }
        }
      }
    }
#pragma unroll
  for (int jj = 0; jj < 4; ++jj) {
    const int j = j0 + tj * 4 + jj;
    if (j >= Tn) continue;
    float* dk = grad_row(g.d_cache_k, g.d_k, a.M, d, a.m, a.Bn, ch, j);
    float* dv = grad_row(g.d_cache_v, g.d_v, a.M, d, a.m, a.Bn, ch, j);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = c0 + tc * 4 + q;
      if (c < d) dk[c] += acc[jj][q];
      else if (c < C) dv[c - d] += acc[jj][q];
    }
  }
}

template <typename T>
hipError_t run(const BwdArgs& g, bool compress, hipStream_t s) {
  const StepArgs& a = g.st;
  const int Tn = a.m + a.Bn, chains = a.batch * a.Hkv;
  // with g.ws_mfma set every contraction below has a matrix-core form (tiled_mfma.hip)
  const bool conv_mfma = g.ws_mfma != nullptr;
  const bool mfma = g.gemms_mfma && bwd_gemms_mfma_fit(g);
  hipError_t e = hipSuccess;
  if (mfma) e = launch_bwd_attn_scores_mfma(g, s);
  else
    hipLaunchKernelGGL(bwd_attn_scores_k<T>, dim3((Tn + kAT - 1) / kAT, (a.Bn + kAT - 1) / kAT, a.batch * a.Hq),
                       dim3(kThreads), 0, s, g);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_attn_rows_k, dim3(a.Bn, a.Hq, a.batch), dim3(kThreads), 0, s, g);
  if (mfma) {
    if ((e = launch_bwd_attn_grads_mfma(g, s)) != hipSuccess) return e;
  } else {
    hipLaunchKernelGGL(bwd_attn_dq_k<T>, dim3((a.d + kAT - 1) / kAT, (a.Bn + kAT - 1) / kAT, a.batch * a.Hq),
                       dim3(kThreads), 0, s, g);
    hipLaunchKernelGGL(bwd_attn_cols_k<T>, dim3((a.d + kAT - 1) / kAT, (Tn + kAT - 1) / kAT, chains),
                       dim3(kThreads), 0, s, g);
  }
  if (a.m < a.M) hipLaunchKernelGGL(bwd_zero_dead_rows_k, dim3(64, chains), dim3(kThreads), 0, s, g);
  if (!compress) {
    hipLaunchKernelGGL(bwd_fill_k, dim3(64, chains), dim3(kThreads), 0, s, g);
    return hipGetLastError();
  }
  if (mfma) e = launch_bwd_mix_dw_mfma(g, s);
  else
    hipLaunchKernelGGL(bwd_mix_dw_k<T>, dim3((Tn + kMT - 1) / kMT, (a.M + kMT - 1) / kMT, chains), dim3(kThreads), 0,
                       s, g);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_mix_rows_k, dim3(a.M, chains), dim3(kThreads), 0, s, g);
  if (mfma) e = launch_bwd_mix_cols_mfma(g, s);
  else
    hipLaunchKernelGGL(bwd_mix_cols_k, dim3((2 * a.d + kMT - 1) / kMT, (Tn + kMT - 1) / kMT, chains), dim3(kThreads), 0,
                       s, g);
  if (e != hipSuccess) return e;
  if (conv_mfma) return launch_bwd_conv_mfma(g, g.banks, g.ws_mfma, s);   // the two Eq. 5 gradients
  const int C = a.conv_in ? 2 * a.d : a.d;
  hipLaunchKernelGGL(bwd_conv_x_k<T>, dim3((Tn + kTI - 1) / kTI, (C + kTI - 1) / kTI, chains), dim3(kThreads), 0, s, g);
  hipLaunchKernelGGL(bwd_conv_w_k<T>,
                     dim3(((C + kWC - 1) / kWC) * ((a.k_width + kTK - 1) / kTK), (a.M + kTI - 1) / kTI, chains),
                     dim3(kThreads), 0, s, g);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_step_backward_generic(int dtype, const BwdArgs& g, bool compress, hipStream_t s) {
  return dtype == LOCOCO_F32 ? run<float>(g, compress, s) : run<bf16_t>(g, compress, s);
}

}  // namespace lococo
