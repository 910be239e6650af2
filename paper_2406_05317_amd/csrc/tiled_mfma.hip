// LDS-tiled bf16 MFMA kernels for the contractions outside the two fused forward kernels:
//  * Eq. 5 as a kernel of its own (keys-only or [K | V] filters, any odd width up to 31), used by the
//    forward path for compressors the fused kernel is not built for and by the backward pass to
//    recompute the logits;
//  * the two gradients of Eq. 5 in the backward pass (head_dim = channels = 128, keys-only filters);
//  * one batched GEMM kernel (bwd_gemm_k) whose instances are the seven plain contractions of the
//    backward pass (attention and Eq. 4) and Eq. 4 of the unfused forward path.
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
// The Eq. 5 kernels: 256 threads, 128 x 128 outputs per workgroup (64 x 64 per wave, 2 x 2 MFMA
// tiles of 32 x 32 x 16), operands staged through LDS in rows padded by 16 bytes; a tap is a
// row-shifted view of a staged tile.  Where the contraction runs down the rows of a row-major
// tile the fragments come from transposing LDS reads.  The next tile is fetched into registers
// while the current one is multiplied.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>

#include "lococo_internal.h"
#include <cstdlib>

namespace lococo {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(short)))) short s16x4;
typedef __attribute__((__vector_size__(8 * sizeof(short)))) short s16x8;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

constexpr int kThreads = 256;
constexpr int kD = 128;          // channels
constexpr int kRow = 320;        // bytes of a 128-element row in LDS read by transposing reads: 64 past a multiple of 256, so
                                 // that the four rows x 64 bytes half a wave touches fall on different banks
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

__device__ __forceinline__ const uint16_t* v_row(const StepArgs& a, int b, int hkv, int j) {   // same for the values
  if (j < a.m) return (const uint16_t*)a.cache_v + ((int64_t)(b * a.Hkv + hkv) * a.M + j) * kD;
  return (const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + (int64_t)(j - a.m) * a.v.st;
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
__global__ void pack_filters_per_tap_k(const uint16_t* w, uint16_t* wt, int M, int C, int KW, int banks,
                                   int64_t w_head_stride) {
  const int64_t n = (int64_t)banks * KW * M * C;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
    const int c = (int)(e % C);
    const int s = (int)((e / C) % M);
    const int t = (int)((e / ((int64_t)C * M)) % KW);
    const int bank = (int)(e / ((int64_t)C * M * KW));
    wt[e] = w[bank * w_head_stride + ((int64_t)s * C + c) * KW + t];
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
// positions of one slot per instruction.  KV = 1: the convolution reads [K | V], 256 channels.
// ST: 128 slots per workgroup, or 64 (a wave then has one block of 32 slots instead of two) where
// 128 would leave compute units without a workgroup.
template <int KV, int ST>
__global__ __launch_bounds__(KV ? 512 : 256, KV ? 1 : 2) void conv_logits_mfma_k(StepArgs a, const uint16_t* wt,
                                                                                 float* out) {
  extern __shared__ __align__(16) unsigned char smem[];
  // 8 waves per compute unit either way: two workgroups of 4 (each wave 64 slots x 64 positions), or,
  // where the tiles of 256 channels leave LDS for one workgroup only, one of 8 (64 slots x 32 positions
  // per wave), so that every SIMD has a second wave to run while one waits for its fragments
  constexpr int NT = KV ? 512 : 256, PB = KV ? 1 : 2, SBW = ST / 64;
  constexpr int C = KV ? 2 * kD : kD, ROW = C * 2 + 16, CH16 = C / 8;   // channels, LDS row bytes, 16-byte chunks per row
  const int KW = a.k_width, pad = (KW - 1) / 2, Tn = a.m + a.Bn;
  const int xrows = kTile + KW - 1;
  unsigned char* Xs = smem;
  unsigned char* Ws = smem + xrows * ROW;
  const int p0 = blockIdx.x * kTile, s0 = blockIdx.y * ST, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int wy = w / (NT / 128), wx = w % (NT / 128);     // wave: slots 32 SBW wy .., positions 32 PB wx ..
  const uint16_t* wtb = wt + (a.w_head_stride ? (int64_t)hkv * KW * a.M * C : 0);

  {
    // every load is issued before the first store: one memory latency for the whole tile, not one per chunk
    constexpr int XPER = ((kTile + 30) * CH16 + NT - 1) / NT;
    u32x4 xr[XPER];
#pragma unroll
    for (int i = 0; i < XPER; ++i) {
      const int item = tid + i * NT, row = item / CH16, c16 = item % CH16, p = p0 - pad + row;
      const u32x4 z = {0u, 0u, 0u, 0u};
      xr[i] = (item < xrows * CH16 && p >= 0 && p < Tn)
                  ? *(const u32x4*)((c16 < 16 ? x_row(a, b, hkv, p) : v_row(a, b, hkv, p)) + (c16 & 15) * 8)
                  : z;
    }
#pragma unroll
    for (int i = 0; i < XPER; ++i) {
      const int item = tid + i * NT, row = item / CH16, c16 = item % CH16;
      if (item < xrows * CH16) *(u32x4*)(Xs + row * ROW + c16 * 16) = xr[i];
    }
  }
  constexpr int WPER = ST * CH16 / NT;
  u32x4 wreg[WPER];
  // element offsets of this thread's chunks inside a tap's matrix, computed once; a tap adds a uniform
  // base.  A slot past M reads the last slot instead: its outputs are never stored, and nothing
  // touches the loaded values before they go to LDS, so the loads stay in flight under the MFMAs.
  uint32_t woff[WPER];
#pragma unroll
  for (int i = 0; i < WPER; ++i) {
    const int item = tid + i * NT, row = item / CH16, c16 = item % CH16, s = s0 + row;
    woff[i] = (uint32_t)((s < a.M ? s : a.M - 1) * C + c16 * 8);
  }
  auto load_w = [&](int t) {
    const uint16_t* wtap = wtb + (int64_t)t * a.M * C;
#pragma unroll
    for (int i = 0; i < WPER; ++i) wreg[i] = *(const u32x4*)(wtap + woff[i]);
  };
  auto store_w = [&]() {
#pragma unroll
    for (int i = 0; i < WPER; ++i) {
      const int item = tid + i * NT, row = item / CH16, c16 = item % CH16;
      *(u32x4*)(Ws + row * ROW + c16 * 16) = wreg[i];
    }
  };
  f32x16 acc[SBW][PB];                    // [slot block][position block]
#pragma unroll
  for (int sb = 0; sb < SBW; ++sb)
#pragma unroll
    for (int pb = 0; pb < PB; ++pb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[sb][pb][i] = 0.f;
  load_w(0);
  for (int t = 0; t < KW; ++t) {
    __syncthreads();                      // the previous tap's reads are done (first time: X is staged)
    store_w();
    __syncthreads();
    if (t + 1 < KW) load_w(t + 1);        // in flight under this tap's MFMAs
    const unsigned char* wl = Ws + (wy * 32 * SBW + l31) * ROW + lh * 16;
    const unsigned char* xl = Xs + (wx * 32 * PB + l31 + t) * ROW + lh * 16;
#pragma unroll
    for (int kc = 0; kc < C / 16; ++kc) {
      bf16x8 fa[SBW], fb[PB];
#pragma unroll
      for (int sb = 0; sb < SBW; ++sb) fa[sb] = frag(wl + sb * 32 * ROW + kc * 32);
#pragma unroll
      for (int pb = 0; pb < PB; ++pb) fb[pb] = frag(xl + pb * 32 * ROW + kc * 32);
#pragma unroll
      for (int sb = 0; sb < SBW; ++sb)
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
          acc[sb][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[sb], fb[pb], acc[sb][pb], 0, 0, 0);
    }
  }
  const uint16_t* bias = a.conv_b ? (const uint16_t*)a.conv_b + hkv * a.b_head_stride : nullptr;
#pragma unroll
  for (int sb = 0; sb < SBW; ++sb)
#pragma unroll
    for (int pb = 0; pb < PB; ++pb) {
      const int p = p0 + wx * 32 * PB + pb * 32 + l31;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int s = s0 + wy * 32 * SBW + sb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
        if (s < a.M && p < Tn)
          out[((int64_t)ch * a.M + s) * (a.ldw ? a.ldw : Tn) + p] = acc[sb][pb][i] + (bias ? bf16_val(bias[s]) : 0.f);
      }
    }
}

// ---- the same logits for more than 128 slots (NQ = 2: filters over the keys, 128 channels; NQ = 4:
// over [K | V], 256 channels): 256 slots x 256 positions per workgroup, 8 waves of 64 x 128 (three fragment reads per four MFMAs instead of six).  The
// contraction walks the channels in NQ quarters of 64 and, inside a quarter, the taps: the
// keys or values of a quarter (all positions of the tile, 64 channels) are staged once, and the
// filter tile of a stage (256 slots x 64 channels of one tap) arrives by loads that write LDS
// directly, two stages ahead in a ring of three buffers: no staging registers, no LDS store
// instructions, one barrier per stage.  Such a load fills 64 consecutive 16-byte cells (8 rows of
// 128 bytes), so the filter tiles are unpadded and XOR-swizzled: chunk c of row r sits in cell
// c ^ ((r / 2) % 8), which spreads 16 consecutive rows over the 16 cells of 256 bytes; each lane
// requests whatever chunk belongs in its cell.
__device__ __forceinline__ void load_to_lds_at(const u32x4& rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  // M0 (the LDS address) is an operand the compiler sets itself; the wait state the hardware wants
  // between a write of M0 and such a load is the s_nop
  asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "{m0}"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
// A 16-byte load the compiler does not wait for; the caller counts the loads in flight (they
// complete in order, those into LDS included) and waits by hand before the first use.
__device__ __forceinline__ void load16_unwaited(u32x4& dst, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(dst) : "v"(p) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads_but() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int NQ>
__global__ __launch_bounds__(512, 1) void conv_logits_wide_k(StepArgs a, const uint16_t* wt, float* out) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NT = 512, C = NQ * 64, SL = 256, PT = 256, WBUF = SL * 128;
  const int KW = a.k_width, pad = (KW - 1) / 2, Tn = a.m + a.Bn, xrows = PT + KW - 1;
  unsigned char* Xs = smem + 3 * WBUF;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)smem);
  const int p0 = blockIdx.x * PT, s0 = blockIdx.y * SL, ch = blockIdx.z, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int wy = w >> 1, wx = w & 1;                       // wave: slots 64 wy .., positions 128 wx ..
  const int w_uniform = __builtin_amdgcn_readfirstlane(w);
  const uint16_t* wtb = wt + (a.w_head_stride ? (int64_t)hkv * KW * a.M * C : 0);

  // ---- filter tiles.  Instruction i of wave w fills rows 8 (4 w + i) .. + 7 of the tile; lane l:
  // row r = 8 (4 w + i) + l / 8, cell l % 8, so (r / 2) % 8 = 4 (i % 2) + l / 16.  A slot past M reads the last slot instead: its outputs are never stored.
  u32x4 rs;
  {
    const uint64_t base = (uint64_t)wtb;
    rs[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
    rs[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
    rs[2] = __builtin_amdgcn_readfirstlane((uint32_t)((int64_t)KW * a.M * C * 2));
    rs[3] = 0x00020000u;
  }
  uint32_t wvoff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int sl = s0 + (w * 4 + i) * 8 + (l >> 3);
    wvoff[i] = (uint32_t)((sl < a.M ? sl : a.M - 1) * (C * 2) + (((l & 7) ^ (4 * (i & 1) + (l >> 4))) << 4));
  }
  auto request_w = [&](int t, int q, int buf) {            // tap t, channels 64 q .., into ring buffer buf
    const uint32_t soff = __builtin_amdgcn_readfirstlane((uint32_t)(((int64_t)t * a.M * C + q * 64) * 2));
    const uint32_t dst = lds0 + (uint32_t)(buf * WBUF + w_uniform * 4096);
#pragma unroll
    for (int i = 0; i < 4; ++i) load_to_lds_at(rs, dst + i * 1024, wvoff[i], soff);
  };
  // ---- keys (quarters 0, 1) or values (2, 3): rows p0 - pad .. of 64 channels, padded rows in LDS.
  // Rows outside the sequence are fetched from its nearest row and zeroed when they are stored.
  constexpr int XPER = ((PT + 30) * 8 + NT - 1) / NT;
  u32x4 xr[XPER];
  auto request_x = [&](int q) {
#pragma unroll
    for (int i = 0; i < XPER; ++i) {
      const int item = tid + i * NT, p = p0 - pad + (item >> 3);
      const int pc = p < 0 ? 0 : (p < Tn ? p : Tn - 1);
      load16_unwaited(xr[i], (q < 2 ? x_row(a, b, hkv, pc) : v_row(a, b, hkv, pc)) + (q & 1) * 64 + (item & 7) * 8);
    }
  };
  auto store_x = [&]() {
#pragma unroll
    for (int i = 0; i < XPER; ++i) asm volatile("" : "+v"(xr[i]));
#pragma unroll
    for (int i = 0; i < XPER; ++i) {
      const int item = tid + i * NT, row = item >> 3, p = p0 - pad + row;
      const u32x4 z = {0u, 0u, 0u, 0u};
      if (row < xrows) *(u32x4*)(Xs + row * kRow64 + (item & 7) * 16) = (p >= 0 && p < Tn) ? xr[i] : z;
    }
  };
  int wcell[4];
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) wcell[kc] = ((2 * kc + lh) ^ ((l31 >> 1) & 7)) << 4;

  f32x16 acc[2][4];                       // [slot block][position block]
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int pb = 0; pb < 4; ++pb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[sb][pb][i] = 0.f;

  const int N = NQ * KW;                  // stage n = (quarter n / KW, tap n % KW)
  request_x(0);
  request_w(0, 0, 0);
  request_w(1 % KW, 1 / KW, 1);
  wait_loads_but<0>();
  store_x();
  __syncthreads();
  int buf = 0;
  for (int q = 0; q < NQ; ++q)
    for (int t = 0; t < KW; ++t) {
      const int n = q * KW + t;
      const bool next_quarter = t == KW - 1 && q < NQ - 1;
      if (next_quarter) request_x(q + 1);
      const bool more = n + 2 < N;
      if (more) {
        int t2 = t + 2, q2 = q;
        while (t2 >= KW) t2 -= KW, ++q2;
        request_w(t2, q2, buf == 0 ? 2 : buf - 1);         // (n + 2) % 3: the buffer stage n - 1 has finished with
      }
      const unsigned char* wl = smem + buf * WBUF + (wy * 64 + l31) * 128;
      const unsigned char* xl = Xs + (wx * 128 + l31 + t) * kRow64 + lh * 16;
#pragma unroll
      for (int kc = 0; kc < 4; ++kc) {
        bf16x8 fa[2], fb[4];
#pragma unroll
        for (int sb = 0; sb < 2; ++sb) fa[sb] = frag(wl + sb * 32 * 128 + wcell[kc]);
#pragma unroll
        for (int pb = 0; pb < 4; ++pb) fb[pb] = frag(xl + pb * 32 * kRow64 + kc * 32);
#pragma unroll
        for (int sb = 0; sb < 2; ++sb)
#pragma unroll
          for (int pb = 0; pb < 4; ++pb)
            acc[sb][pb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[sb], fb[pb], acc[sb][pb], 0, 0, 0);
      }
      // the next stage's filter tile (and the next quarter's rows, requested before it) have landed;
      // only this stage's own four requests may still be on their way
      if (more) wait_loads_but<4>(); else wait_loads_but<0>();
      __syncthreads();
      if (next_quarter) {                 // every wave has finished with the old rows
        store_x();
        __syncthreads();
      }
      buf = buf == 2 ? 0 : buf + 1;
    }
  const uint16_t* bias = a.conv_b ? (const uint16_t*)a.conv_b + hkv * a.b_head_stride : nullptr;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int pb = 0; pb < 4; ++pb) {
      const int p = p0 + wx * 128 + pb * 32 + l31;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int sl = s0 + wy * 64 + sb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
        if (sl < a.M && p < Tn)
          out[((int64_t)ch * a.M + sl) * (a.ldw ? a.ldw : Tn) + p] = acc[sb][pb][i] + (bias ? bf16_val(bias[sl]) : 0.f);
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
  // channel tile: 0 = the key channels; 1 = the value channels of [K | V] filters, whose gradient
  // belongs to the value rows
  const int c0 = blockIdx.z * kTile, C = a.conv_in ? 2 * kD : kD;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w >> 1, wx = w & 1;
  const uint16_t* wtb = wt + (a.w_head_stride ? (int64_t)hkv * KW * a.M * C : 0) + c0;
  const int nsc = Mp / kChunk, nsteps = nsc * KW;

  u32x4 wreg[4];
  auto load_w = [&](int n) {
    const int sc = n / KW, t = n % KW;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15, s = sc * kChunk + row;
      const u32x4 z = {0u, 0u, 0u, 0u};
      wreg[i] = s < a.M ? *(const u32x4*)(wtb + ((int64_t)t * a.M + s) * C + c16 * 8) : z;
    }
  };
  auto store_w = [&]() {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int item = tid + i * kThreads, row = item >> 4, c16 = item & 15;
      *(u32x4*)(Ws + row * kRow + c16 * 16) = wreg[i];
    }
  };
  auto stage_d = [&](int sc) {            // all loads before the first store: one memory latency per tile
    constexpr int DPER = ((kTile + 30) * 8 + kThreads - 1) / kThreads;
    u32x4 vh[DPER], vl[DPER];
#pragma unroll
    for (int i = 0; i < DPER; ++i) {
      const int item = tid + i * kThreads, row = item >> 3, c16 = item & 7, q = p0 + row - (KW - 1) + pad;
      const u32x4 z = {0u, 0u, 0u, 0u};
      const bool in = item < drows * 8 && q >= 0 && q < Tn;
      const int64_t o = ((int64_t)ch * Tn + (in ? q : 0)) * Mp + sc * kChunk + c16 * 8;
      vh[i] = in ? *(const u32x4*)(dhi + o) : z;
      vl[i] = in ? *(const u32x4*)(dlo + o) : z;
    }
#pragma unroll
    for (int i = 0; i < DPER; ++i) {
      const int item = tid + i * kThreads, row = item >> 3, c16 = item & 7;
      if (item < drows * 8) {
        *(u32x4*)(Dh + row * kRow64 + c16 * 16) = vh[i];
        *(u32x4*)(Dl + row * kRow64 + c16 * 16) = vl[i];
      }
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
      float* row = p < a.m ? (c0 ? g.d_cache_v : g.d_cache_k) + ((int64_t)ch * a.M + p) * kD
                           : (c0 ? g.d_v : g.d_k) + ((int64_t)ch * a.Bn + (p - a.m)) * kD;
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
  const int C = a.conv_in ? 2 * kD : kD, ctiles = C / kTile;
  const int t = blockIdx.x, s0 = (blockIdx.y / ctiles) * kTile, c0 = (blockIdx.y % ctiles) * kTile;   // c0 = 128: value channels
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
      xreg[i] = (q >= 0 && q < Tn) ? *(const u32x4*)((c0 ? v_row(a, b, hkv, q) : x_row(a, b, hkv, q)) + c16 * 8) : z;
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
  float* o = dwt + ((int64_t)(per_head ? hkv_fixed : 0) * KW + t) * a.M * C + c0;
#pragma unroll
  for (int sb = 0; sb < 2; ++sb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int s = s0 + wy * 64 + sb * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
      if (s >= a.M) continue;
#pragma unroll
      for (int cb = 0; cb < 2; ++cb) atomicAdd(o + (int64_t)s * C + wx * 64 + cb * 32 + l31, acc[sb][cb][i]);
    }
}


// ---- Eq. 6 and Eq. 4a / 4b of the unfused forward path in one kernel: from raw logits fp32
// [chain, M, ld] to the bf16 rows of the next cache, [new_K | new_V][i] = sum_j w[i, j] [Yk | Yv][j]
// with w the normalised row i.  One workgroup owns 128 slots x all 256 columns of a chain and walks
// the positions in chunks of 64: a thread holds four positions of eight rows, sixteen threads share
// a row and keep its running reference and sum (softmax: the reference moves only when the row
// maximum outgrows it by 8, so the accumulators are rescaled almost never; relu-sum: a plain sum),
// the weights go to LDS as bf16 (what the fused kernel does with its probabilities), [K | V] rows are
// read down their rows through transposing reads.  The division by the row sum comes last.
// NORM: 0 softmax, 1 relu / (sum + eps).
constexpr float kLog2e = 1.4426950408889634f;
// Reductions over the 16 lanes that share a row, on the VALU (DPP), no LDS round trip: inside quads,
// then lane i <-> 7 - i of each 8, then lane i <-> 15 - i of each 16; every lane ends with the result.
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float max16(float v) {
  v = fmaxf(v, dpp<0xB1>(v));           // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp<0x4E>(v));           // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp<0x141>(v));          // row_half_mirror
  return fmaxf(v, dpp<0x140>(v));       // row_mirror
}
__device__ __forceinline__ float sum16(float v) {
  v += dpp<0xB1>(v);
  v += dpp<0x4E>(v);
  v += dpp<0x141>(v);
  return v + dpp<0x140>(v);
}
constexpr int kYRow = 2 * kD * 2 + 64;             // bytes of a staged [K | V] row (64 past a multiple of 256: conflict-free transposing reads)
// SLOTS: 128 slots per workgroup, or 64 or 32 where that is what it takes to give the compute units one each.
// NT: 256 threads (waves 2 x 2: half the slots x the K or the V columns each), or 512 (waves 2 x 4:
// half the slots x 64 columns) so that every SIMD has a second wave to run while one waits.
template <int NORM, int SLOTS, int NT>
__global__ __launch_bounds__(NT) void mixnorm_mfma_k(StepArgs a, const float* logits, int ld) {
  constexpr int RPT = SLOTS * 16 / NT, SB = SLOTS >= 64 ? SLOTS / 64 : 1;   // rows of logits per thread; 32-slot blocks per wave
  constexpr int WY = SLOTS / (32 * SB), WX = NT / 64 / WY;   // waves down the slots and across the columns
  constexpr int YB = 8 / WX, YPER = kChunk * 32 / NT;        // 32-column blocks per wave; staged chunks per thread
  __shared__ __align__(16) unsigned char Ps[SLOTS * kRow64];      // weights of the chunk [slot][position], bf16
  __shared__ __align__(16) unsigned char Ys[kChunk * kYRow];      // [position][K | V columns]
  __shared__ __align__(16) float alpha_s[SLOTS];                  // rescale factor per slot for this chunk
  __shared__ __align__(16) float sum_s[SLOTS];                    // final row sums
  __shared__ int any_rescale[2];                                  // by chunk parity: reset two barriers after its last read
  const int Tn = a.m + a.Bn;
  // the slot tiles of a chain read the same [K | V] rows: workgroup ids are dealt round-robin to the
  // 8 XCDs, so consecutive work items go to one XCD and a chain's rows come in through one L2
  int item = blockIdx.x;
  {
    const int per = gridDim.x / 8;
    if (item < per * 8) item = (item % 8) * per + item / 8;
  }
  const int tiles = (a.M + SLOTS - 1) / SLOTS;
  const int s0 = (item % tiles) * SLOTS, ch = item / tiles, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w / WX, wx = w % WX;
  const int c4 = tid & 15;                           // this thread's four positions inside a chunk: 4 c4 ..
  const float* lrow[RPT];
#pragma unroll
  for (int n = 0; n < RPT; ++n) {
    const int srow = s0 + (tid >> 4) + (NT / 16) * n;       // a slot past M reads the last one; it is never stored
    lrow[n] = logits + ((int64_t)ch * a.M + (srow < a.M ? srow : a.M - 1)) * ld;
  }
  float m_run[RPT], l_part[RPT];
#pragma unroll
  for (int n = 0; n < RPT; ++n) { m_run[n] = -1e30f; l_part[n] = 0.f; }

  f32x16 acc[SB][YB];                                // [slot block][column block]
#pragma unroll
  for (int x = 0; x < SB; ++x)
#pragma unroll
    for (int y = 0; y < YB; ++y)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[x][y][i] = 0.f;

  u32x4 lreg[RPT], yreg[YPER];
  auto load = [&](int j0) {
#pragma unroll
    for (int n = 0; n < RPT; ++n)           // a group past T reads the row's first group (ld >= 4) and counts for nothing
      lreg[n] = *(const u32x4*)(lrow[n] + (j0 + c4 * 4 < Tn ? j0 + c4 * 4 : 0));
#pragma unroll
    for (int n = 0; n < YPER; ++n) {
      const int item = tid + n * NT, row = item >> 5, c16 = item & 31, j = j0 + row;
      const int jc = j < Tn ? j : 0;
      yreg[n] = *(const u32x4*)((c16 < 16 ? x_row(a, b, hkv, jc) : v_row(a, b, hkv, jc)) + (c16 & 15) * 8);
    }
  };
  const int tro = tr_lane_offset(l, kYRow);
  load(0);
  for (int j0 = 0; j0 < Tn; j0 += kChunk) {
    const int par = (j0 / kChunk) & 1;
    if (tid == 0) any_rescale[par] = 0;
    __syncthreads();                                 // the previous chunk's fragments have been read
    // ---- this chunk's weights
#pragma unroll
    for (int n = 0; n < RPT; ++n) {
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float x = __uint_as_float(lreg[n][e]);
        v[e] = j0 + c4 * 4 + e < Tn ? x : -INFINITY;
      }
      float al = 1.f;
      if (NORM == 0) {
        const float mx = max16(fmaxf(fmaxf(v[0], v[1]), fmaxf(v[2], v[3])));
        if (mx > m_run[n] + 8.f) {                   // same for the sixteen threads of the row
          al = __builtin_amdgcn_exp2f((m_run[n] - mx) * kLog2e);
          m_run[n] = mx;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = __builtin_amdgcn_exp2f((v[e] - m_run[n]) * kLog2e);
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = fmaxf(v[e], 0.f);
      }
      l_part[n] = l_part[n] * al + (v[0] + v[1]) + (v[2] + v[3]);
      const f32x2 x0 = {v[0], v[1]}, x1 = {v[2], v[3]};
      const bf16x2 h0 = __builtin_convertvector(x0, bf16x2), h1 = __builtin_convertvector(x1, bf16x2);
      const u32x2 pk = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1)};
      const int row = (tid >> 4) + (NT / 16) * n;
      *(u32x2*)(Ps + row * kRow64 + c4 * 8) = pk;
      if (NORM == 0 && c4 == 0) {
        alpha_s[row] = al;
        if (al != 1.f) any_rescale[par] = 1;
      }
    }
#pragma unroll
    for (int n = 0; n < YPER; ++n) {
      const int item = tid + n * NT, row = item >> 5, c16 = item & 31;
      const u32x4 z = {0u, 0u, 0u, 0u};
      *(u32x4*)(Ys + row * kYRow + c16 * 16) = j0 + row < Tn ? yreg[n] : z;
    }
    __syncthreads();
    if (j0 + kChunk < Tn) load(j0 + kChunk);         // in flight under the MFMAs
    if (NORM == 0 && any_rescale[par]) {             // rare: a reference moved
#pragma unroll
      for (int x = 0; x < SB; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float al = alpha_s[wy * 32 * SB + x * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)];
#pragma unroll
          for (int y = 0; y < YB; ++y) acc[x][y][i] *= al;
        }
    }
#pragma unroll
    for (int kc = 0; kc < kChunk / 16; ++kc) {
      bf16x8 fp[SB], fy[YB];
#pragma unroll
      for (int x = 0; x < SB; ++x) fp[x] = frag(Ps + (wy * 32 * SB + x * 32 + l31) * kRow64 + (kc * 16 + lh * 8) * 2);
#pragma unroll
      for (int y = 0; y < YB; ++y) fy[y] = frag_tr(Ys + tro + kc * 16 * kYRow + (wx * YB + y) * 32 * 2, kYRow);
#pragma unroll
      for (int x = 0; x < SB; ++x)
#pragma unroll
        for (int y = 0; y < YB; ++y)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fp[x], fy[y], acc[x][y], 0, 0, 0);
    }
  }
  // ---- row sums: over the sixteen threads of a row, then to everybody
#pragma unroll
  for (int n = 0; n < RPT; ++n) {
    const float t = sum16(l_part[n]);
    if (c4 == 0) sum_s[(tid >> 4) + (NT / 16) * n] = t;
  }
  __syncthreads();
#pragma unroll
  for (int x = 0; x < SB; ++x)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = wy * 32 * SB + x * 32 + (i >> 2) * 8 + lh * 4 + (i & 3), slot = s0 + row;
      if (slot >= a.M) continue;
      const float inv = 1.0f / (NORM == 0 ? sum_s[row] : sum_s[row] + a.eps);
      const int col0 = wx * YB * 32;                   // of [new_K | new_V]
      uint16_t* dst = (uint16_t*)(col0 >= kD ? a.new_v : a.new_k) + ((int64_t)ch * a.M + slot) * kD + (col0 & (kD - 1));
#pragma unroll
      for (int y = 0; y < YB; ++y) dst[y * 32 + l31] = (uint16_t)bf16_rne(acc[x][y][i] * inv);
    }
}

// ---- the seven plain contractions of the pass (attention: scores, dP, dq, dYk, dYv; Eq. 4: dw and
// the gradient of [K | V]) as one batched GEMM kernel, C[i, j] = sum_k A(i, k) B(j, k).
//
// An operand is a functor over a tensor in memory:
//   load4(v, z, r, c): four consecutive elements (memory row r, offsets c .. c + 3) of batch entry
//                      z as floats, zero outside the tensor;
//   kMajor:  false = memory rows are operand rows and the contraction runs along them (staged as
//            128 rows x 64 k, fragments by 16-byte reads); true = memory rows are contraction
//            steps (staged as 64 k x 128 rows, fragments by transposing reads);
//   kParts:  1 = the values are bf16 numbers; 2 = fp32 values, staged as hi + lo (the product of
//            two such operands takes three MFMAs: hi hi, hi lo, lo hi).
// The output functor decides where C[i, j] goes (store) and may skip whole tiles.
constexpr int kPartBytes = kChunk * kRow;        // 20 480 >= kTile * kRow64
static_assert(kTile * kRow64 <= kPartBytes, "a staged operand part fits its LDS area either way round");

template <class OpA, class OpB, class Out>
__global__ __launch_bounds__(kThreads, 2) void bwd_gemm_k(OpA A, OpB B, Out out, int I, int J, int K) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* As = smem;
  unsigned char* Bs = smem + OpA::kParts * kPartBytes;
  const int j0 = blockIdx.x * kTile, i0 = blockIdx.y * kTile, z = blockIdx.z;
  if (out.skip(z, i0, j0)) return;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5, wy = w >> 1, wx = w & 1;

  // A chunk is fetched as raw bits (bf16 sources: 8 bytes per group of four, fp32 sources: 16) with the
  // number of valid elements beside them; nothing reads the registers before the chunk is staged, so
  // the loads stay in flight under the MFMAs of the chunk before.
  u32x4 ra[8], rb[8];
  int na[8], nb[8];
  auto load = [&](int k0) {
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      const int gidx = tid + n * kThreads;
      na[n] = OpA::kMajor ? A.load4(ra[n], z, k0 + (gidx >> 5), i0 + (gidx & 31) * 4)
                          : A.load4(ra[n], z, i0 + (gidx >> 4), k0 + (gidx & 15) * 4);
      nb[n] = OpB::kMajor ? B.load4(rb[n], z, k0 + (gidx >> 5), j0 + (gidx & 31) * 4)
                          : B.load4(rb[n], z, j0 + (gidx >> 4), k0 + (gidx & 15) * 4);
    }
  };
  // four values -> 8 bytes of bf16 (round to nearest even), and the rounding errors likewise
  auto put = [&](unsigned char* base, int parts, bool kmajor, bool bf16_source, int gidx, const u32x4& raw, int nv) {
    unsigned char* at = kmajor ? base + (gidx >> 5) * kRow + (gidx & 31) * 8 : base + (gidx >> 4) * kRow64 + (gidx & 15) * 8;
    if (bf16_source) {                    // already bf16: as it is, or nothing
      const u32x2 v = {nv ? raw[0] : 0u, nv ? raw[1] : 0u};
      *(u32x2*)at = v;
      return;
    }
    const f32x2 x0 = {nv > 0 ? __uint_as_float(raw[0]) : 0.f, nv > 1 ? __uint_as_float(raw[1]) : 0.f};
    const f32x2 x1 = {nv > 2 ? __uint_as_float(raw[2]) : 0.f, nv > 3 ? __uint_as_float(raw[3]) : 0.f};
    const bf16x2 h0 = __builtin_convertvector(x0, bf16x2), h1 = __builtin_convertvector(x1, bf16x2);
    const u32x2 vh = {__builtin_bit_cast(uint32_t, h0), __builtin_bit_cast(uint32_t, h1)};
    *(u32x2*)at = vh;
    if (parts == 2) {
      const f32x2 e0 = x0 - __builtin_convertvector(h0, f32x2), e1 = x1 - __builtin_convertvector(h1, f32x2);
      const bf16x2 l0 = __builtin_convertvector(e0, bf16x2), l1 = __builtin_convertvector(e1, bf16x2);
      const u32x2 vl = {__builtin_bit_cast(uint32_t, l0), __builtin_bit_cast(uint32_t, l1)};
      *(u32x2*)(at + kPartBytes) = vl;
    }
  };
  auto stage = [&]() {
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      put(As, OpA::kParts, OpA::kMajor, OpA::kBf16, tid + n * kThreads, ra[n], na[n]);
      put(Bs, OpB::kParts, OpB::kMajor, OpB::kBf16, tid + n * kThreads, rb[n], nb[n]);
    }
  };
  f32x16 acc[2][2];
  zero_acc(acc);
  const int tro = tr_lane_offset(l, kRow);
  load(0);
  for (int k0 = 0; k0 < K; k0 += kChunk) {
    __syncthreads();
    stage();
    __syncthreads();
    if (k0 + kChunk < K) load(k0 + kChunk);
#pragma unroll
    for (int kc = 0; kc < kChunk / 16; ++kc) {
      bf16x8 fa[OpA::kParts][2], fb[OpB::kParts][2];
#pragma unroll
      for (int p = 0; p < OpA::kParts; ++p)
#pragma unroll
        for (int x = 0; x < 2; ++x)
          fa[p][x] = OpA::kMajor
                         ? frag_tr(As + p * kPartBytes + tro + kc * 16 * kRow + (wy * 64 + x * 32) * 2, kRow)
                         : frag(As + p * kPartBytes + (wy * 64 + x * 32 + l31) * kRow64 + (kc * 16 + lh * 8) * 2);
#pragma unroll
      for (int p = 0; p < OpB::kParts; ++p)
#pragma unroll
        for (int x = 0; x < 2; ++x)
          fb[p][x] = OpB::kMajor
                         ? frag_tr(Bs + p * kPartBytes + tro + kc * 16 * kRow + (wx * 64 + x * 32) * 2, kRow)
                         : frag(Bs + p * kPartBytes + (wx * 64 + x * 32 + l31) * kRow64 + (kc * 16 + lh * 8) * 2);
#pragma unroll
      for (int pa = 0; pa < OpA::kParts; ++pa)
#pragma unroll
        for (int pb = 0; pb < OpB::kParts; ++pb) {
          if (pa + pb == 2) continue;     // lo x lo: below the 16 bits kept
#pragma unroll
          for (int x = 0; x < 2; ++x)
#pragma unroll
            for (int y = 0; y < 2; ++y)
              acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[pa][x], fb[pb][y], acc[x][y], 0, 0, 0);
        }
    }
  }
#pragma unroll
  for (int x = 0; x < 2; ++x)
#pragma unroll
    for (int i16 = 0; i16 < 16; ++i16) {
      const int i = i0 + wy * 64 + x * 32 + (i16 >> 2) * 8 + lh * 4 + (i16 & 3);
      if (i >= I) continue;
#pragma unroll
      for (int y = 0; y < 2; ++y) {
        const int j = j0 + wx * 64 + y * 32 + l31;
        if (j < J) out.store(z, i, j, acc[x][y][i16]);
      }
    }
}

// -- operands.  load4(raw, z, r, c) fetches the raw bits of the four elements (memory row r, offsets
// c .. c + 3) of batch entry z -- 8 bytes in raw[0], raw[1] from a bf16 tensor (kBf16), 16 bytes from
// an fp32 one -- and returns how many of them count (0: the group lies outside the tensor; it is
// then read at element 0 of a valid row, never out of bounds).  It does not touch what it loaded.
// `grouped`: z is a chain and the memory row runs over the rows of all query heads of its group,
// head-major; otherwise z is (batch entry, query head).  Every width is a multiple of 4 and every base
// 16-byte aligned (the launcher checks), so a group of four is inside or outside as a whole.
struct Dims { int Bn, Tn, d, M, m, Hq, Hkv, group; };
__device__ __forceinline__ void head_row(const Dims& s, bool grouped, int z, int r, int& b, int& hq, int& rr) {
  if (grouped) {
    b = z / s.Hkv;
    hq = (z % s.Hkv) * s.group + r / s.Bn;
    rr = r % s.Bn;
  } else {
    b = z / s.Hq;
    hq = z % s.Hq;
    rr = r;
  }
}
__device__ __forceinline__ void raw_bf16x4(u32x4& raw, const uint16_t* p) {
  const u32x2 u = *(const u32x2*)p;
  raw[0] = u[0];
  raw[1] = u[1];
}
__device__ __forceinline__ void raw_f32x4(u32x4& raw, const float* p) { raw = *(const u32x4*)p; }
__device__ __forceinline__ bool is_protected(const uint32_t* protect, int64_t stride, int z, int r, int m) {
  if (!protect) return false;           // uniform
  const int rc = r < m ? r : 0;
  return r < m && ((protect[(int64_t)z * stride + (rc >> 5)] >> (rc & 31)) & 1u);
}

template <bool KMAJOR>
struct OpQ {               // query rows, bf16
  static constexpr bool kMajor = KMAJOR, kBf16 = true;
  static constexpr int kParts = 1;
  Dims s; View q; bool grouped;
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool ok = r < (grouped ? s.group * s.Bn : s.Bn) && c < s.d;
    int b, hq, rr;
    head_row(s, grouped, z, ok ? r : 0, b, hq, rr);
    raw_bf16x4(raw, (const uint16_t*)q.p + b * q.sb + hq * q.sh + (int64_t)rr * q.st + (ok ? c : 0));
    return ok ? 4 : 0;
  }
};
template <bool KMAJOR>
struct OpRowsF32 {         // fp32 [batch, Hq, Bn, width] rows: d_o (width d), ws_p / ws_ds (width Tn)
  static constexpr bool kMajor = KMAJOR, kBf16 = false;
  static constexpr int kParts = 2;
  Dims s; const float* p; int width; bool grouped;
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool ok = r < (grouped ? s.group * s.Bn : s.Bn) && c < width;
    int b, hq, rr;
    head_row(s, grouped, z, ok ? r : 0, b, hq, rr);
    raw_f32x4(raw, p + (((int64_t)b * s.Hq + hq) * s.Bn + rr) * width + (ok ? c : 0));
    return ok ? 4 : 0;
  }
};
template <bool KMAJOR, int WHICH>     // WHICH: 0 keys, 1 values, 2 [keys | values] (width 2 d)
struct OpY {               // rows of [cache(0:m) ; block], bf16
  static constexpr bool kMajor = KMAJOR, kBf16 = true;
  static constexpr int kParts = 1;
  Dims s; const void* cache_k; const void* cache_v; View k, v; bool per_qhead;
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool ok = r < s.Tn && c < (WHICH == 2 ? 2 * s.d : s.d);
    const int r2 = ok ? r : 0, c2 = ok ? c : 0;
    int b, hkv;
    if (per_qhead) { b = z / s.Hq; hkv = (z % s.Hq) / s.group; }
    else { b = z / s.Hkv; hkv = z % s.Hkv; }
    const bool val = WHICH == 1 || (WHICH == 2 && c2 >= s.d);
    const int col = WHICH == 2 && c2 >= s.d ? c2 - s.d : c2;
    const View& blk = val ? v : k;
    const bool in_cache = r2 < s.m;
    const uint16_t* crow =
        (const uint16_t*)(val ? cache_v : cache_k) + ((int64_t)(b * s.Hkv + hkv) * s.M + (in_cache ? r2 : 0)) * s.d;
    const uint16_t* brow =
        (const uint16_t*)blk.p + b * blk.sb + hkv * blk.sh + (int64_t)(in_cache ? 0 : r2 - s.m) * blk.st;
    raw_bf16x4(raw, (in_cache ? crow : brow) + col);
    return ok ? 4 : 0;
  }
};
template <bool KMAJOR>
struct OpG {               // gradient of the new cache, fp32 rows [g_k | g_v] of width 2 d
  static constexpr bool kMajor = KMAJOR, kBf16 = false;
  static constexpr int kParts = 2;
  Dims s; const float* gk; const float* gv; const uint32_t* protect; int64_t protect_stride; bool mask;
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool in = r < s.M && c < 2 * s.d;
    const int r2 = in ? r : 0, c2 = in ? c : 0;
    const bool ok = in && !(mask && is_protected(protect, protect_stride, z, r2, s.m));
    raw_f32x4(raw, (c2 < s.d ? gk : gv) + ((int64_t)z * s.M + r2) * s.d + (c2 < s.d ? c2 : c2 - s.d));
    return ok ? 4 : 0;
  }
};
struct OpWn {              // normalised mixing rows, fp32 [chain, M, Tn]; protected slots mix nothing
  static constexpr bool kMajor = true, kBf16 = false;
  static constexpr int kParts = 2;
  Dims s; const float* w; const uint32_t* protect; int64_t protect_stride;
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool in = r < s.M && c < s.Tn;
    const int r2 = in ? r : 0, c2 = in ? c : 0;
    const bool ok = in && !is_protected(protect, protect_stride, z, r2, s.m);
    raw_f32x4(raw, w + ((int64_t)z * s.M + r2) * s.Tn + c2);
    return ok ? 4 : 0;
  }
};
struct OpWrows {           // normalised mixing rows fp32 [chain, M, Tn], as rows (contraction along them);
  static constexpr bool kMajor = false, kBf16 = false;   // rounded to bf16 like the probabilities of the fused kernel
  static constexpr int kParts = 1;
  Dims s; const float* w; int ld;            // ld: row stride, a multiple of 4 (the columns T .. ld hold nothing)
  __device__ int load4(u32x4& raw, int z, int r, int c) const {
    const bool ok = r < s.M && c < s.Tn;
    raw_f32x4(raw, w + ((int64_t)z * s.M + (ok ? r : 0)) * ld + (ok ? c : 0));
    return ok ? (s.Tn - c < 4 ? s.Tn - c : 4) : 0;
  }
};

// -- outputs
struct OutNewCache {       // bf16 rows of the next cache [chain, M, d]: j < d keys, else values
  Dims s; uint16_t* nk; uint16_t* nv;
  __device__ bool skip(int, int, int) const { return false; }
  __device__ void store(int z, int i, int j, float v) const {
    uint16_t* row = (j < s.d ? nk : nv) + ((int64_t)z * s.M + i) * s.d;
    row[j < s.d ? j : j - s.d] = (uint16_t)bf16_rne(v);
  }
};
struct OutRows {           // fp32 [batch, Hq, Bn, Tn] rows, scaled; tiles wholly after their queries are skipped
  Dims s; float* p; float scale;
  __device__ bool skip(int, int i0, int j0) const { return j0 > s.m + i0 + kTile - 1; }
  __device__ void store(int z, int i, int j, float v) const { p[((int64_t)z * s.Bn + i) * s.Tn + j] = v * scale; }
};
struct OutPlain {          // fp32 [z, rows, width]
  float* p; int rows, width;
  __device__ bool skip(int, int, int) const { return false; }
  __device__ void store(int z, int i, int j, float v) const { p[((int64_t)z * rows + i) * width + j] = v; }
};
template <bool ADD>
struct OutGrad {           // gradient rows of [cache ; block]: i = position, j = column of K (or of [K | V])
  Dims s; float* d_cache_k; float* d_blk_k; float* d_cache_v; float* d_blk_v; int which;   // 0 K, 1 V, 2 [K | V]
  __device__ bool skip(int, int, int) const { return false; }
  __device__ void store(int z, int i, int j, float v) const {
    const bool val = which == 1 || (which == 2 && j >= s.d);
    const int col = which == 2 && j >= s.d ? j - s.d : j;
    float* dc = val ? d_cache_v : d_cache_k;
    float* db = val ? d_blk_v : d_blk_k;
    float* at = (i < s.m ? dc + ((int64_t)z * s.M + i) * s.d : db + ((int64_t)z * s.Bn + (i - s.m)) * s.d) + col;
    if (ADD) *at += v;
    else *at = v;
  }
};

template <class OpA, class OpB, class Out>
hipError_t launch_gemm(const OpA& A, const OpB& B, const Out& out, int I, int J, int K, int Z, hipStream_t s) {
  const int lds = (OpA::kParts + OpB::kParts) * kPartBytes;
  static bool attr_set = false;   // per instantiation; benign race
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)bwd_gemm_k<OpA, OpB, Out>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (I <= 0 || J <= 0 || Z <= 0) return hipSuccess;
  hipLaunchKernelGGL((bwd_gemm_k<OpA, OpB, Out>), dim3((J + kTile - 1) / kTile, (I + kTile - 1) / kTile, Z),
                     dim3(kThreads), lds, s, A, B, out, I, J, K);
  return hipGetLastError();
}

Dims dims_of(const StepArgs& a) { return Dims{a.Bn, a.m + a.Bn, a.d, a.M, a.m, a.Hq, a.Hkv, a.group}; }

__global__ void bwd_zero_k(float* p, int64_t n) {
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x)
    p[e] = 0.f;
}
// d_conv_w[bank][slot][channel][tap] += dwt[bank][tap][slot][channel]
__global__ void bwd_add_dw_k(const float* dwt, float* d_conv_w, int M, int C, int KW, int banks,
                             int64_t w_head_stride) {
  const int64_t n = (int64_t)banks * M * C * KW;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n; e += (int64_t)gridDim.x * blockDim.x) {
    const int t = (int)(e % KW);
    const int c = (int)((e / KW) % C);
    const int s = (int)((e / ((int64_t)KW * C)) % M);
    const int bank = (int)(e / ((int64_t)KW * C * M));
    d_conv_w[bank * w_head_stride + ((int64_t)s * C + c) * KW + t] +=
        dwt[(((int64_t)bank * KW + t) * M + s) * C + c];
  }
}

int grid_for(int64_t n) { return (int)std::min<int64_t>((n + 255) / 256, 4096); }

}  // namespace

bool bwd_mfma_supports(int dtype, int d, int conv_in, int conv_width) {
  (void)conv_in;                          // keys-only and [K | V] filters alike
  return dtype == LOCOCO_BF16 && d == kD && conv_width % 2 == 1 && conv_width <= 31;
}
bool conv_logits_mfma_supports(int dtype, int d, int conv_width) {    // keys-only or [K | V] filters
  return dtype == LOCOCO_BF16 && d == kD && conv_width % 2 == 1 && conv_width <= 31;
}
size_t packed_filter_bytes(int M, int conv_width, int conv_in, int banks) {
  return (size_t)banks * conv_width * M * (conv_in ? 2 * kD : kD) * 2;
}

static int padded_slots(int n) { return (n + kChunk - 1) / kChunk * kChunk; }   // also for positions

BwdMfmaLayout bwd_mfma_layout(int batch, int Hkv, int M, int Tn, int conv_width, int conv_in, int banks) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  const int C = conv_in ? 2 * kD : kD;
  BwdMfmaLayout l;
  l.wt = 0;
  l.dhi = up((size_t)banks * conv_width * M * C * 2);
  const size_t half = up((size_t)batch * Hkv * Tn * padded_slots(M) * 2);
  l.dlo = l.dhi + half;
  const size_t half_s = up((size_t)batch * Hkv * M * padded_slots(Tn) * 2);
  l.dhi_s = l.dlo + half;
  l.dlo_s = l.dhi_s + half_s;
  l.dwt = l.dlo_s + half_s;
  l.total = l.dwt + up((size_t)banks * conv_width * M * C * 4);
  return l;
}

hipError_t launch_pack_filters_per_tap(const StepArgs& a, int banks, void* wt, hipStream_t s) {
  const int C = a.conv_in ? 2 * kD : kD;
  const int64_t n = (int64_t)banks * a.k_width * a.M * C;
  hipLaunchKernelGGL(pack_filters_per_tap_k, dim3(grid_for(n)), dim3(256), 0, s, (const uint16_t*)a.conv_w,
                     (uint16_t*)wt, a.M, C, a.k_width, banks, a.w_head_stride);
  return hipGetLastError();
}

template <int KV, int ST>
static hipError_t launch_logits(const StepArgs& a, const void* wt, float* logits, hipStream_t s) {
  constexpr int ROW = (KV ? 2 * kD : kD) * 2 + 16;
  const int Tn = a.m + a.Bn;
  const int lds = (kTile + a.k_width - 1) * ROW + ST * ROW;
  static bool attr_set = false;   // benign race: setting it twice is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_logits_mfma_k<KV, ST>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (kTile + 30) * ROW + ST * ROW);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((conv_logits_mfma_k<KV, ST>), dim3((Tn + kTile - 1) / kTile, (a.M + ST - 1) / ST, a.batch * a.Hkv),
                     dim3(KV ? 512 : 256), lds, s, a, (const uint16_t*)wt, logits);
  return hipGetLastError();
}
template <int NQ>
static hipError_t launch_logits_wide(const StepArgs& a, const void* wt, float* logits, hipStream_t s) {
  constexpr int WBUFS = 3 * 256 * 128;    // the ring of filter tiles; behind it the rows of one channel quarter
  const int Tn = a.m + a.Bn;
  static bool attr_set = false;   // benign race: setting it twice is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_logits_wide_k<NQ>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       WBUFS + (256 + 30) * kRow64);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(conv_logits_wide_k<NQ>, dim3((Tn + 255) / 256, (a.M + 255) / 256, a.batch * a.Hkv), dim3(512),
                     WBUFS + (256 + a.k_width - 1) * kRow64, s, a, (const uint16_t*)wt, logits);
  return hipGetLastError();
}
// Three tile shapes.  64 and 128 slots give the same bits (every output element is the same sum in
// the same order: taps outermost); the 256 x 256 kernel walks the channel quarters outermost, so its
// fp32 sums differ from theirs in rounding.  The debug option LOCOCO_OPT_LOGITS_TILES (64 | 128 | 256)
// overrides the choice by grid size, for tests and measurements; 256 is ignored where there are at most
// 128 slots.
hipError_t launch_conv_logits_mfma(const StepArgs& a, const void* wt, float* logits, hipStream_t s) {
  const int Tn = a.m + a.Bn, chains = a.batch * a.Hkv;
  const int64_t tiles256 = (int64_t)((Tn + 255) / 256) * ((a.M + 255) / 256) * chains;
  const int64_t tiles128 = (int64_t)((Tn + kTile - 1) / kTile) * ((a.M + kTile - 1) / kTile) * chains;
  // 256 x 256 where there are enough of those tiles for three quarters of the compute units;
  // 64-slot tiles where 128-slot ones would be fewer than the compute units
  const int n_cu = cu_count();
  int shape = a.M > kTile && tiles256 >= n_cu * 3 / 4 ? 256 : tiles128 < n_cu ? 64 : 128;
  {
    const int v = (int)debug_options().logits_tiles;
    if (v == 64 || v == 128 || (v == 256 && a.M > kTile)) shape = v;
  }
  if (shape == 256) return a.conv_in ? launch_logits_wide<4>(a, wt, logits, s) : launch_logits_wide<2>(a, wt, logits, s);
  if (shape == 64) return a.conv_in ? launch_logits<1, 64>(a, wt, logits, s) : launch_logits<0, 64>(a, wt, logits, s);
  return a.conv_in ? launch_logits<1, 128>(a, wt, logits, s) : launch_logits<0, 128>(a, wt, logits, s);
}

// The plain contractions take whole groups of four: every row width (d, 2 d, T) a multiple of 4
// and every fp32 array 16-byte aligned.  Otherwise the caller keeps the fp32 vector kernels.
bool bwd_gemms_mfma_fit(const BwdArgs& g) {
  const StepArgs& a = g.st;
  if ((a.m + a.Bn) % 4 || a.d % 4) return false;
  for (const void* p : {(const void*)g.d_o, (const void*)g.d_new_k, (const void*)g.d_new_v, (const void*)g.ws_p,
                        (const void*)g.ws_ds, (const void*)g.ws_n})
    if ((uintptr_t)p & 15) return false;
  return true;
}

// S = scale q Yk^T into ws_p and dP = dO Yv^T into ws_ds (the row kernel turns them into P and dS)
hipError_t launch_bwd_attn_scores_mfma(const BwdArgs& g, hipStream_t s) {
  const StepArgs& a = g.st;
  const Dims dm = dims_of(a);
  const int Z = a.batch * a.Hq;
  hipError_t e = launch_gemm(OpQ<false>{dm, a.q, false}, OpY<false, 0>{dm, a.cache_k, a.cache_v, a.k, a.v, true},
                             OutRows{dm, g.ws_p, a.scale}, a.Bn, dm.Tn, a.d, Z, s);
  if (e != hipSuccess) return e;
  return launch_gemm(OpRowsF32<false>{dm, g.d_o, a.d, false}, OpY<false, 1>{dm, a.cache_k, a.cache_v, a.k, a.v, true},
                     OutRows{dm, g.ws_ds, 1.0f}, a.Bn, dm.Tn, a.d, Z, s);
}

// dq = dS Yk; dYk = dS^T q and dYv = P^T dO over the heads of a group (assigned: first contributions)
hipError_t launch_bwd_attn_grads_mfma(const BwdArgs& g, hipStream_t s) {
  const StepArgs& a = g.st;
  const Dims dm = dims_of(a);
  const int chains = a.batch * a.Hkv;
  hipError_t e = launch_gemm(OpRowsF32<false>{dm, g.ws_ds, dm.Tn, false},
                             OpY<true, 0>{dm, a.cache_k, a.cache_v, a.k, a.v, true},
                             OutPlain{g.d_q, a.Bn, a.d}, a.Bn, a.d, dm.Tn, a.batch * a.Hq, s);
  if (e != hipSuccess) return e;
  e = launch_gemm(OpRowsF32<true>{dm, g.ws_ds, dm.Tn, true}, OpQ<true>{dm, a.q, true},
                  OutGrad<false>{dm, g.d_cache_k, g.d_k, g.d_cache_v, g.d_v, 0}, dm.Tn, a.d, a.group * a.Bn, chains, s);
  if (e != hipSuccess) return e;
  return launch_gemm(OpRowsF32<true>{dm, g.ws_p, dm.Tn, true}, OpRowsF32<true>{dm, g.d_o, a.d, true},
                     OutGrad<false>{dm, g.d_cache_k, g.d_k, g.d_cache_v, g.d_v, 1}, dm.Tn, a.d, a.group * a.Bn, chains, s);
}

// dw[i, j] = g_k[i] . Yk[j] + g_v[i] . Yv[j] into ws_dw
hipError_t launch_bwd_mix_dw_mfma(const BwdArgs& g, hipStream_t s) {
  const StepArgs& a = g.st;
  const Dims dm = dims_of(a);
  return launch_gemm(OpG<false>{dm, g.d_new_k, g.d_new_v, a.protect, a.protect_stride, false},
                     OpY<false, 2>{dm, a.cache_k, a.cache_v, a.k, a.v, false}, OutPlain{g.ws_dw, a.M, dm.Tn}, a.M,
                     dm.Tn, 2 * a.d, a.batch * a.Hkv, s);
}

// Eq. 4a / 4b of the forward step from normalised rows: [new_K | new_V][i] = sum_j w[i, j] [Yk | Yv][j]
bool mix_mfma_fits(const StepArgs& a, const float* w) {
  return a.d == kD && (a.ldw ? a.ldw : a.m + a.Bn) % 4 == 0 && ((uintptr_t)w & 15) == 0;
}
hipError_t launch_mix_mfma(const StepArgs& a, const float* w, hipStream_t s) {
  const Dims dm = dims_of(a);
  return launch_gemm(OpWrows{dm, w, a.ldw ? a.ldw : dm.Tn}, OpY<true, 2>{dm, a.cache_k, a.cache_v, a.k, a.v, false},
                     OutNewCache{dm, (uint16_t*)a.new_k, (uint16_t*)a.new_v}, a.M, 2 * a.d, dm.Tn,
                     a.batch * a.Hkv, s);
}


// Eq. 6 + Eq. 4a / 4b of the forward step from raw logits (rows ld floats apart); needs mixnorm_mfma_fits
bool mixnorm_mfma_fits(const StepArgs& a, const float* logits) {
  const int ld = a.ldw ? a.ldw : a.m + a.Bn;
  return a.d == kD && ld % 4 == 0 && ((uintptr_t)logits & 15) == 0 && (a.norm == 0 || a.norm == 1);
}
hipError_t launch_mixnorm_mfma(const StepArgs& a, const float* logits, hipStream_t s) {
  const int ld = a.ldw ? a.ldw : a.m + a.Bn;
  const int chains = a.batch * a.Hkv;
  const int n_cu = cu_count();
  if ((int64_t)((a.M + 127) / 128) * chains >= n_cu) {      // enough 128-slot tiles for every compute unit
    const dim3 grid((a.M + 127) / 128 * chains);
    if (a.norm == 0) hipLaunchKernelGGL((mixnorm_mfma_k<0, 128, 512>), grid, dim3(512), 0, s, a, logits, ld);
    else hipLaunchKernelGGL((mixnorm_mfma_k<1, 128, 512>), grid, dim3(512), 0, s, a, logits, ld);
  } else if ((int64_t)((a.M + 63) / 64) * chains >= n_cu / 2) {  // (with one per compute unit of these, twice as many of 32 slots are slower)
    const dim3 grid((a.M + 63) / 64 * chains);
    if (a.norm == 0) hipLaunchKernelGGL((mixnorm_mfma_k<0, 64, 512>), grid, dim3(512), 0, s, a, logits, ld);
    else hipLaunchKernelGGL((mixnorm_mfma_k<1, 64, 512>), grid, dim3(512), 0, s, a, logits, ld);
  } else {                                                  // few chains: 32 slots per workgroup, eight waves of 32 columns
    const dim3 grid((a.M + 31) / 32 * chains);
    if (a.norm == 0) hipLaunchKernelGGL((mixnorm_mfma_k<0, 32, 512>), grid, dim3(512), 0, s, a, logits, ld);
    else hipLaunchKernelGGL((mixnorm_mfma_k<1, 32, 512>), grid, dim3(512), 0, s, a, logits, ld);
  }
  return hipGetLastError();
}

// d[Yk | Yv][j] += sum over the unprotected slots of w[i, j] [g_k | g_v][i]
hipError_t launch_bwd_mix_cols_mfma(const BwdArgs& g, hipStream_t s) {
  const StepArgs& a = g.st;
  const Dims dm = dims_of(a);
  return launch_gemm(OpWn{dm, g.ws_n, a.protect, a.protect_stride},
                     OpG<true>{dm, g.d_new_k, g.d_new_v, a.protect, a.protect_stride, true},
                     OutGrad<true>{dm, g.d_cache_k, g.d_k, g.d_cache_v, g.d_v, 2}, dm.Tn, 2 * a.d, a.M,
                     a.batch * a.Hkv, s);
}

hipError_t launch_bwd_conv_mfma(const BwdArgs& g, int banks, void* ws, hipStream_t s) {
  const StepArgs& a = g.st;
  const int Tn = a.m + a.Bn, chains = a.batch * a.Hkv, Mp = padded_slots(a.M);
  const BwdMfmaLayout l = bwd_mfma_layout(a.batch, a.Hkv, a.M, Tn, a.k_width, a.conv_in, banks);
  const int C = a.conv_in ? 2 * kD : kD, ctiles = C / kTile;
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
    hipLaunchKernelGGL(bwd_dx_mfma_k, dim3((Tn + kTile - 1) / kTile, chains, ctiles), dim3(kThreads), lds, s, g, wt,
                       dhi, dlo, Mp);
  }
  const int64_t nw = (int64_t)banks * a.k_width * a.M * C;
  hipLaunchKernelGGL(bwd_zero_k, dim3(grid_for(nw)), dim3(256), 0, s, dwt, nw);
  {
    // chains per workgroup: enough workgroups to fill the chip several times over, as few atomics as that allows
    const int entries = banks > 1 ? a.batch : chains;
    const int tiles = a.k_width * ((a.M + kTile - 1) / kTile) * ctiles * (banks > 1 ? a.Hkv : 1);
    int per_group = (int)std::min<int64_t>(8, std::max<int64_t>(1, (int64_t)tiles * entries / 1024));
    const int groups = (entries + per_group - 1) / per_group;
    hipLaunchKernelGGL(bwd_dw_mfma_k,
                       dim3(a.k_width, ((a.M + kTile - 1) / kTile) * ctiles, groups * (banks > 1 ? a.Hkv : 1)),
                       dim3(kThreads), 0, s, g, dhi_s, dlo_s, Tp, dwt, per_group);
  }
  hipLaunchKernelGGL(bwd_add_dw_k, dim3(grid_for(nw)), dim3(256), 0, s, dwt, g.d_conv_w, a.M, C, a.k_width, banks,
                     a.w_head_stride);
  return hipGetLastError();
}

}  // namespace lococo
