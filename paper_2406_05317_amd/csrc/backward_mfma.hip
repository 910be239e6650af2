// Eq. 5 in the backward pass of a compress step on the matrix cores (bf16 storage, head_dim =
// channels = 128, keys-only filters): the recomputed logits, their gradient w.r.t. the keys and
// w.r.t. the filters are the three large contractions of that pass (2 M T C k flops each).
//
//   logits[i, j]  = b[i] + sum_t sum_c Wc[i, c, t] X[j + t - p, c]
//   dX[j, c]     += sum_t sum_i dW[i, j - t + p] Wc[i, c, t]
//   dWc[i, c, t] += sum_j dW[i, j] X[j + t - p, c]
//
// Keys and filters are bf16 already, so the first contraction is exact up to the order of the
// fp32 sums.  The gradient of the logits dW is fp32: it enters the other two as the sum of two
// bf16 numbers (dW = hi + lo, lo = the rounding error of hi), two MFMAs per operand pair, which
// keeps about 16 bits of it: the results agree with the fp32 kernels to the usual 1e-4.
//
// All three kernels: 256 threads, 128 x 128 outputs per workgroup (64 x 64 per wave, 2 x 2 MFMA
// tiles of 32 x 32 x 16), operands staged through LDS in rows padded by 16 bytes; a tap is a
// row-shifted view of a staged tile.  Where the contraction runs down the rows of a row-major
// tile the fragments come from transposing LDS reads.  The next tile is fetched into registers
// while the current one is multiplied.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

constexpr int kThreads = 256;
constexpr int kD = 128;          // channels
constexpr int kRow = 272;        // bytes of a 128-element row in LDS (256 + 16: conflict-free 16-byte column reads)
constexpr int kRow64 = 144;      // bytes of a 64-element row in LDS
constexpr int kTile = 128;       // outputs per workgroup, both ways
constexpr int kChunk = 64;       // contraction chunk of the two gradient kernels

__device__ __forceinline__ bf16x8 frag(const unsigned char* p) { return *(const bf16x8*)p; }
// Fragment (lane: column c0 + l % 32; 8 contraction rows r0 + 8 (l / 32) ..) out of a row-major
// tile: ds_read_b64_tr_b16 hands lane i of a 16-lane group element i % 4 of the 8-byte chunks
// addressed by lanes i / 4 + {0, 4, 8, 12}, so with lane s pointing at (row s / 4, column 4 (s % 4))
// of a 4 x 16 patch every lane receives one column of the patch, 4 rows deep.  `p` already holds
// this lane's address inside the first patch (see tr_lane_offset).
__device__ __forceinline__ bf16x8 frag_tr(const unsigned char* p, int stride) {
  const s16x4 a0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
  const s16x4 a1 =
      __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(p + 4 * stride));
  const s16x8 v = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ int tr_lane_offset(int l, int stride) {
  const int s16 = l & 15, g2 = (l >> 4) & 1, lh = l >> 5;
  return (lh * 8 + (s16 >> 2)) * stride + (16 * g2 + 4 * (s16 & 3)) * 2;
}

__device__ __forceinline__ uint32_t bf16_rne(float v) {      // finite v
  uint32_t u = __float_as_uint(v);
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_val(uint32_t h) { return __uint_as_float(h << 16); }

// row j of X = [cache(0:m) ; block], 128 bf16
__device__ __forceinline__ const uint16_t* x_row(const StepArgs& a, int b, int hkv, int j) {
  if (j < a.m) return (const uint16_t*)a.cache_k + ((int64_t)(b * a.Hkv + hkv) * a.M + j) * kD;
  return (const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + (int64_t)(j - a.m) * a.k.st;
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[2][2]) {
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int y = 0; y < 2; ++y)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.f;
}

// ---- filters [bank][slot][channel][tap] -> [bank][tap][slot][channel]: every tap a row-major
// (slot x channel) matrix, which the logits read along the channels and dX down the slots
__global__ void bwd_pack_filters_k(const uint16_t* w, uint16_t* wt, int M, int KW, int banks,
                                   int64_t w_head_stride) {
  const int64_t n = (int64_t)banks * KW * M * kD;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(e % kD);
    const int s = (int)((e / kD) % M);
    const int t = (int)((e / ((int64_t)kD * M)) % KW);
    const int bank = (int)(e / ((int64_t)kD * M * KW));
    wt[e] = w[bank * w_head_stride + ((int64_t)s * kD + c) * KW + t];
  }
}

// ---- dW fp32 [chain][slot][position] -> two bf16 halves, dW = hi + lo (lo = the rounding error of
// hi), in both orientations: [chain][position][Mp] for dX, which contracts over the slots, and
// [chain][slot][Tp] for dWc, which contracts over the positions (Mp, Tp = M, T rounded up to 64,
// the tails zero, so that 16-byte loads of whole chunks stay inside)
__global__ __launch_bounds__(kThreads) void bwd_split_dl_k(const float* dl, uint16_t* hi, uint16_t* lo,
                                                           uint16_t* hi_s, uint16_t* lo_s, int M, int Mp, int Tn,
                                                           int Tp) {
  __shared__ float tile[64][65];
  const int p0 = blockIdx.x * 64, s0 = blockIdx.y * 64, ch = blockIdx.z;
  for (int e = threadIdx.x; e < 64 * 64; e += kThreads) {
    const int s = e >> 6, p = e & 63;
    const float v = (s0 + s < M && p0 + p < Tn) ? dl[((int64_t)ch * M + s0 + s) * Tn + p0 + p] : 0.f;
    tile[s][p] = v;
    if (s0 + s < M) {
      const uint32_t h = bf16_rne(v), l = bf16_rne(v - bf16_val(h));
      const int64_t o = ((int64_t)ch * M + s0 + s) * Tp + p0 + p;
      hi_s[o] = (uint16_t)h;
      lo_s[o] = (uint16_t)l;
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < 64 * 64; e += kThreads) {
    const int p = e >> 6, s = e & 63;
    if (p0 + p >= Tn) continue;
    const float v = tile[s][p];
    const uint32_t h = bf16_rne(v), l = bf16_rne(v - bf16_val(h));
    const int64_t o = ((int64_t)ch * Tn + p0 + p) * Mp + s0 + s;
    hi[o] = (uint16_t)h;
    lo[o] = (uint16_t)l;
  }
}

// ---- logits[i, j] (slots x positions, contraction over channels and taps)
// LDS: X rows p0 - pad .. p0 + 127 + (KW - 1 - pad) once; per tap the (slot x channel) matrix of
// 128 slots.  A = filters (rows: slots), B = keys (lane: position): a lane stores 32 consecutive
// positions of one slot per instruction.
__global__ __launch_bounds__(kThreads, 2) void bwd_logits_mfma_k(StepArgs a, const uint16_t* wt, float* out) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int KW = a.k_width, pad = (KW - 1) / 2, Tn = a.m + a.Bn;
  const int xrows = kTile + KW - 1;
  unsigned char* Xs = smem;
  unsigned char* Ws = smem + xrows * kRow;
  const int p0 = blockIdx.x * kTile, s0 = blockIdx.y * kTile, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w >> 1, wx = w & 1;
  const uint16_t* wtb = wt + (a.w_head_stride ? (int64_t)hkv * KW * a.M * kD : 0);

  for (int item = tid; item < xrows * 16; item += kThreads) {
    const int row = item >> 4, c16 = item & 15, p = p0 - pad + row;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (p >= 0 && p < Tn) v = *(const u32x4*)(x_row(a, b, hkv, p) + c16 * 8);
    *(u32x4*)(Xs + row * kRow + c16 * 16) = v;
  }
  u32x4 wreg[8];
  auto load_w = [&](int t) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15, s = s0 + row;
      const u32x4 z = {0u, 0u, 0u, 0u};
      wreg[i] = s < a.M ? *(const u32x4*)(wtb + ((int64_t)t * a.M + s) * kD + c16 * 8) : z;
    }
  };
  auto store_w = [&]() {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15;
      *(u32x4*)(Ws + row * kRow + c16 * 16) = wreg[i];
    }
  };
  f32x16 acc[2][2];                       // [slot block][position block]
  zero_acc(acc);
  load_w(0);
  for (int t = 0; t < KW; ++t) {
    __syncthreads();                      // the previous tap's reads are done (first time: X is staged)
    store_w();
    if (t + 1 < KW) load_w(t + 1);
    __syncthreads();
    const unsigned char* wl = Ws + (wy * 64 + l31) * kRow + lh * 16;
    const unsigned char* xl = Xs + (wx * 64 + l31 + t) * kRow + lh * 16;
#pragma unroll
    for (int kc = 0; kc < kD / 16; ++kc) {
      const bf16x8 a0 = frag(wl + kc * 32), a1 = frag(wl + 32 * kRow + kc * 32);
      const bf16x8 b0 = frag(xl + kc * 32), b1 = frag(xl + 32 * kRow + kc * 32);
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
    }
  }
  const uint16_t* bias = a.conv_b ? (const uint16_t*)a.conv_b + hkv * a.b_head_stride : nullptr;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int pb = 0; pb < 2; ++pb) {
      const int p = p0 + wx * 64 + pb * 32 + l31;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int s = s0 + wy * 64 + sb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
        if (s < a.M && p < Tn)
          out[((int64_t)ch * a.M + s) * Tn + p] = acc[sb][pb][i] + (bias ? bf16_val(bias[s]) : 0.f);
      }
    }
}

// ---- dX[j, c] (positions x channels, contraction over slots and taps)
// LDS: per chunk of 64 slots the rows j0 + pad - (KW - 1) .. of dW^T (hi and lo), read row-shifted
// per tap; per (chunk, tap) the 64 x 128 (slot x channel) filter matrix, read down its rows.
// A = dW^T (rows: positions), B = filters (lane: channel).
__global__ __launch_bounds__(kThreads, 2) void bwd_dx_mfma_k(BwdArgs g, const uint16_t* wt, const uint16_t* dhi,
                                                             const uint16_t* dlo, int Mp) {
  extern __shared__ __align__(16) unsigned char smem[];
  const StepArgs& a = g.st;
  const int KW = a.k_width, pad = (KW - 1) / 2, Tn = a.m + a.Bn;
  const int drows = kTile + KW - 1;
  unsigned char* Dh = smem;
  unsigned char* Dl = Dh + drows * kRow64;
  unsigned char* Ws = Dl + drows * kRow64;
  const int p0 = blockIdx.x * kTile, ch = blockIdx.y, hkv = ch % a.Hkv;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w >> 1, wx = w & 1;
  const uint16_t* wtb = wt + (a.w_head_stride ? (int64_t)hkv * KW * a.M * kD : 0);
  const int nsc = Mp / kChunk, nsteps = nsc * KW;

  u32x4 wreg[4];
  auto load_w = [&](int n) {
    const int sc = n / KW, t = n % KW;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15, s = sc * kChunk + row;
      const u32x4 z = {0u, 0u, 0u, 0u};
      wreg[i] = s < a.M ? *(const u32x4*)(wtb + ((int64_t)t * a.M + s) * kD + c16 * 8) : z;
    }
  };
  auto store_w = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15;
      *(u32x4*)(Ws + row * kRow + c16 * 16) = wreg[i];
    }
  };
  auto stage_d = [&](int sc) {
    for (int item = tid; item < drows * 8; item += kThreads) {
      const int row = item >> 3, c16 = item & 7, q = p0 + row - (KW - 1) + pad;
      u32x4 vh = {0u, 0u, 0u, 0u}, vl = {0u, 0u, 0u, 0u};
      if (q >= 0 && q < Tn) {
        const int64_t o = ((int64_t)ch * Tn + q) * Mp + sc * kChunk + c16 * 8;
        vh = *(const u32x4*)(dhi + o);
        vl = *(const u32x4*)(dlo + o);
      }
      *(u32x4*)(Dh + row * kRow64 + c16 * 16) = vh;
      *(u32x4*)(Dl + row * kRow64 + c16 * 16) = vl;
    }
  };
  f32x16 acc[2][2];                       // [position block][channel block]
  zero_acc(acc);
  load_w(0);
  const int tro = tr_lane_offset(l, kRow);
  for (int n = 0; n < nsteps; ++n) {
    const int sc = n / KW, t = n % KW;
    __syncthreads();
    if (t == 0) stage_d(sc);
    store_w();
    if (n + 1 < nsteps) load_w(n + 1);
    __syncthreads();
    const int arow = wy * 64 + l31 - t + (KW - 1);
    const unsigned char* dh = Dh + arow * kRow64 + lh * 16;
    const unsigned char* dl = Dl + arow * kRow64 + lh * 16;
    const unsigned char* wl = Ws + tro + (wx * 64) * 2;
#pragma unroll
    for (int kc = 0; kc < kChunk / 16; ++kc) {
      const bf16x8 b0 = frag_tr(wl + kc * 16 * kRow, kRow), b1 = frag_tr(wl + kc * 16 * kRow + 64, kRow);
#pragma unroll
      for (int pb = 0; pb < 2; ++pb) {
        const bf16x8 ah = frag(dh + pb * 32 * kRow64 + kc * 32), al = frag(dl + pb * 32 * kRow64 + kc * 32);
        acc[pb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b0, acc[pb][0], 0, 0, 0);
        acc[pb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b1, acc[pb][1], 0, 0, 0);
        acc[pb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b0, acc[pb][0], 0, 0, 0);
        acc[pb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b1, acc[pb][1], 0, 0, 0);
      }
    }
  }
  // every (position, channel) belongs to one lane: plain read-modify-write
#pragma unroll
  for (int pb = 0; pb < 2; ++pb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int p = p0 + wy * 64 + pb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
      if (p >= Tn) continue;
      float* row = p < a.m ? g.d_cache_k + ((int64_t)ch * a.M + p) * kD
                           : g.d_k + ((int64_t)ch * a.Bn + (p - a.m)) * kD;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) row[wx * 64 + cb * 32 + l31] += acc[pb][cb][i];
    }
}

// ---- dWc[i, c, t] for one tap (slots x channels, contraction over the positions of the
// workgroup's chains).  LDS per chunk of 64 positions: the key rows shifted by the tap (read down
// the rows) and the 128 x 64 tiles of the two halves of dW.
// A = dW (rows: slots), B = keys (lane: channel).  Sums go to dwt [bank][tap][slot][channel] with
// atomics (several workgroups, one per group of chains, share an output tile).
__global__ __launch_bounds__(kThreads, 2) void bwd_dw_mfma_k(BwdArgs g, const uint16_t* dhi, const uint16_t* dlo,
                                                             int Tp, float* dwt, int per_group) {
  __shared__ __align__(16) unsigned char Xs[kChunk * kRow];
  __shared__ __align__(16) unsigned char Dh[kTile * kRow64];
  __shared__ __align__(16) unsigned char Dl[kTile * kRow64];
  const StepArgs& a = g.st;
  const int KW = a.k_width, pad = (KW - 1) / 2, Tn = a.m + a.Bn;
  const int t = blockIdx.x, s0 = blockIdx.y * kTile;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w >> 1, wx = w & 1;
  const bool per_head = a.w_head_stride != 0;
  // the chains of this workgroup share a filter bank: consecutive chains when the bank is shared,
  // consecutive batch entries of one kv head otherwise
  const int hkv_fixed = per_head ? blockIdx.z % a.Hkv : 0;
  const int first = (per_head ? blockIdx.z / a.Hkv : blockIdx.z) * per_group;
  const int limit = per_head ? a.batch : a.batch * a.Hkv;
  const int count = first + per_group <= limit ? per_group : limit - first;
  const int nchunk = (Tn + kChunk - 1) / kChunk, nsteps = count * nchunk;

  u32x4 xreg[4], hreg[4], lreg[4];
  auto chain_of = [&](int n) {
    const int e = first + n / nchunk;
    return per_head ? e * a.Hkv + hkv_fixed : e;
  };
  auto load = [&](int n) {
    const int ch = chain_of(n), b = ch / a.Hkv, hkv = ch % a.Hkv, pc = (n % nchunk) * kChunk;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15, q = pc + row + t - pad;
      const u32x4 z = {0u, 0u, 0u, 0u};
      xreg[i] = (q >= 0 && q < Tn) ? *(const u32x4*)(x_row(a, b, hkv, q) + c16 * 8) : z;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, s = s0 + (item >> 3), c16 = item & 7;
      const u32x4 z = {0u, 0u, 0u, 0u};
      const int64_t o = ((int64_t)ch * a.M + s) * Tp + pc + c16 * 8;
      hreg[i] = s < a.M ? *(const u32x4*)(dhi + o) : z;
      lreg[i] = s < a.M ? *(const u32x4*)(dlo + o) : z;
    }
  };
  auto store = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15;
      *(u32x4*)(Xs + row * kRow + c16 * 16) = xreg[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 3, c16 = item & 7;
      *(u32x4*)(Dh + row * kRow64 + c16 * 16) = hreg[i];
      *(u32x4*)(Dl + row * kRow64 + c16 * 16) = lreg[i];
    }
  };
  f32x16 acc[2][2];                       // [slot block][channel block]
  zero_acc(acc);
  if (nsteps > 0) load(0);
  const int tro = tr_lane_offset(l, kRow);
  for (int n = 0; n < nsteps; ++n) {
    __syncthreads();
    store();
    if (n + 1 < nsteps) load(n + 1);
    __syncthreads();
    const unsigned char* xl = Xs + tro + (wx * 64) * 2;
    const unsigned char* dh = Dh + (wy * 64 + l31) * kRow64 + lh * 16;
    const unsigned char* dl = Dl + (wy * 64 + l31) * kRow64 + lh * 16;
#pragma unroll
    for (int kc = 0; kc < kChunk / 16; ++kc) {
      const bf16x8 b0 = frag_tr(xl + kc * 16 * kRow, kRow), b1 = frag_tr(xl + kc * 16 * kRow + 64, kRow);
#pragma unroll
      for (int sb = 0; sb < 2; ++sb) {
        const bf16x8 ah = frag(dh + sb * 32 * kRow64 + kc * 32), al = frag(dl + sb * 32 * kRow64 + kc * 32);
        acc[sb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b0, acc[sb][0], 0, 0, 0);
        acc[sb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b1, acc[sb][1], 0, 0, 0);
        acc[sb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b0, acc[sb][0], 0, 0, 0);
        acc[sb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b1, acc[sb][1], 0, 0, 0);
      }
    }
  }
  float* o = dwt + ((int64_t)(per_head ? hkv_fixed : 0) * KW + t) * a.M * kD;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int s = s0 + wy * 64 + sb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
      if (s >= a.M) continue;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) atomicAdd(o + (int64_t)s * kD + wx * 64 + cb * 32 + l31, acc[sb][cb][i]);
    }
}

__global__ void bwd_zero_k(float* p, int64_t n) {
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    p[e] = 0.f;
}
// d_conv_w[bank][slot][channel][tap] += dwt[bank][tap][slot][channel]
__global__ void bwd_add_dw_k(const float* dwt, float* d_conv_w, int M, int KW, int banks, int64_t w_head_stride) {
  const int64_t n = (int64_t)banks * M * kD * KW;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(e % KW);
    const int c = (int)((e / KW) % kD);
    const int s = (int)((e / ((int64_t)KW * kD)) % M);
    const int bank = (int)(e / ((int64_t)KW * kD * M));
    d_conv_w[bank * w_head_stride + ((int64_t)s * kD + c) * KW + t] +=
        dwt[(((int64_t)bank * KW + t) * M + s) * kD + c];
  }
}

int grid_for(int64_t n) { return (int)std::min<int64_t>((n + 255) / 256, 4096); }

}  // namespace

bool bwd_mfma_supports(int dtype, int d, int conv_in, int conv_width) {
  return dtype == LOCOCO_BF16 && d == kD && conv_in == 0 && conv_width % 2 == 1 && conv_width <= 31;
}

static int padded_slots(int n) { return (n + kChunk - 1) / kChunk * kChunk; }   // also for positions

BwdMfmaLayout bwd_mfma_layout(int batch, int Hkv, int M, int Tn, int conv_width, int banks) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  BwdMfmaLayout l;
  l.wt = 0;
  l.dhi = up((size_t)banks * conv_width * M * kD * 2);
  const size_t half = up((size_t)batch * Hkv * Tn * padded_slots(M) * 2);
  l.dlo = l.dhi + half;
  const size_t half_s = up((size_t)batch * Hkv * M * padded_slots(Tn) * 2);
  l.dhi_s = l.dlo + half;
  l.dlo_s = l.dhi_s + half_s;
  l.dwt = l.dlo_s + half_s;
  l.total = l.dwt + up((size_t)banks * conv_width * M * kD * 4);
  return l;
}

hipError_t launch_bwd_pack_filters(const StepArgs& a, int banks, void* wt, hipStream_t s) {
  const int64_t n = (int64_t)banks * a.k_width * a.M * kD;
  hipLaunchKernelGGL(bwd_pack_filters_k, dim3(grid_for(n)), dim3(256), 0, s, (const uint16_t*)a.conv_w,
                     (uint16_t*)wt, a.M, a.k_width, banks, a.w_head_stride);
  return hipGetLastError();
}

hipError_t launch_bwd_logits_mfma(const StepArgs& a, const void* wt, float* logits, hipStream_t s) {
  const int Tn = a.m + a.Bn;
  const int lds = (kTile + a.k_width - 1) * kRow + kTile * kRow;
  static bool attr_set = false;   // benign race: setting it twice is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_logits_mfma_k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (kTile + 30) * kRow + kTile * kRow);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(bwd_logits_mfma_k, dim3((Tn + kTile - 1) / kTile, (a.M + kTile - 1) / kTile, a.batch * a.Hkv),
                     dim3(kThreads), lds, s, a, (const uint16_t*)wt, logits);
  return hipGetLastError();
}

hipError_t launch_bwd_conv_mfma(const BwdArgs& g, int banks, void* ws, hipStream_t s) {
  const StepArgs& a = g.st;
  const int Tn = a.m + a.Bn, chains = a.batch * a.Hkv, Mp = padded_slots(a.M);
  const BwdMfmaLayout l = bwd_mfma_layout(a.batch, a.Hkv, a.M, Tn, a.k_width, banks);
  const uint16_t* wt = (const uint16_t*)((char*)ws + l.wt);
  uint16_t* dhi = (uint16_t*)((char*)ws + l.dhi);
  uint16_t* dlo = (uint16_t*)((char*)ws + l.dlo);
  uint16_t* dhi_s = (uint16_t*)((char*)ws + l.dhi_s);
  uint16_t* dlo_s = (uint16_t*)((char*)ws + l.dlo_s);
  const int Tp = padded_slots(Tn);
  float* dwt = (float*)((char*)ws + l.dwt);
  // (the split also writes the zero tail, slots M .. Mp, which the 16-byte loads of the dX kernel read)
  hipLaunchKernelGGL(bwd_split_dl_k, dim3((Tn + 63) / 64, Mp / 64, chains), dim3(kThreads), 0, s, g.ws_w, dhi, dlo,
                     dhi_s, dlo_s, a.M, Mp, Tn, Tp);
  {
    const int lds = 2 * (kTile + a.k_width - 1) * kRow64 + kChunk * kRow;
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute((const void*)bwd_dx_mfma_k, hipFuncAttributeMaxDynamicSharedMemorySize,
                                         2 * (kTile + 30) * kRow64 + kChunk * kRow);
      if (e != hipSuccess) return e;
      attr_set = true;
    }
    hipLaunchKernelGGL(bwd_dx_mfma_k, dim3((Tn + kTile - 1) / kTile, chains), dim3(kThreads), lds, s, g, wt, dhi, dlo,
                       Mp);
  }
  const int64_t nw = (int64_t)banks * a.k_width * a.M * kD;
  hipLaunchKernelGGL(bwd_zero_k, dim3(grid_for(nw)), dim3(256), 0, s, dwt, nw);
  {
    // chains per workgroup: enough workgroups to fill the chip several times over, as few atomics as that allows
    const int entries = banks > 1 ? a.batch : chains;
    const int tiles = a.k_width * ((a.M + kTile - 1) / kTile) * (banks > 1 ? a.Hkv : 1);
    int per_group = (int)std::min<int64_t>(8, std::max<int64_t>(1, (int64_t)tiles * entries / 1024));
    const int groups = (entries + per_group - 1) / per_group;
    hipLaunchKernelGGL(bwd_dw_mfma_k, dim3(a.k_width, (a.M + kTile - 1) / kTile, groups * (banks > 1 ? a.Hkv : 1)),
                       dim3(kThreads), 0, s, g, dhi_s, dlo_s, Tp, dwt, per_group);
  }
  hipLaunchKernelGGL(bwd_add_dw_k, dim3(grid_for(nw)), dim3(256), 0, s, dwt, g.d_conv_w, a.M, a.k_width, banks,
                     a.w_head_stride);
  return hipGetLastError();
}

}  // namespace lococo
