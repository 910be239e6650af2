// Fused compression kernel for gfx950: Eq. 5 (convolution logits), Eq. 6
// (softmax over positions) and Eq. 4a/4b (fusion of K and V with shared
// weights) in one pass, bf16 MFMA with fp32 accumulation.  The logits and the
// normalised weights never leave the compute unit.
//
// Structure.  The step is "attention with a convolution for scores": for a
// tile of BM cache slots (rows) the kernel walks the T = m + B positions of
// [cache ; block] in tiles of BN, computes the BM x BN logits as an implicit
// GEMM with inner dimension C*k (each filter tap is a row-shifted view of the
// key tile held in LDS), keeps a running row max / row sum (online softmax),
// and accumulates P . [K | V] into a BM x 2d fp32 accumulator.
//
// Register-stationary filters.  The filter bank is the same for every
// position, chain and step, and a compute unit's register file (512 KB) is
// larger than its slice of the bank, so each workgroup loads its BM x (C*k)
// filter slice into VGPRs once and streams only keys/values through LDS.
// The four waves split the inner dimension by channel quarter (wave w owns
// channels [32w, 32w+32) of every tap); their partial logits are summed
// through LDS before the softmax.  For the mixing GEMM wave w owns output
// columns [64w, 64w+64) of [K | V].
//
// Shapes taken: head_dim = C = 128, bf16, conv_in = 0, norm = 0 (softmax),
// M a multiple of BM; any T (tail positions are masked), any m.
#include <cstdlib>

#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kD = 128;            // head_dim = conv channels
constexpr int kThreads = 256;
constexpr float kLazy = 8.0f;      // softmax reference lags the row maximum by at most this much

template <int BM, int BN, int KW>
struct Geo {
  static constexpr int RT = BM / 32;                 // 32-row MFMA tiles per workgroup
  static constexpr int PT = BN / 32;                 // 32-position MFMA tiles per iteration
  static constexpr int PAD = (KW - 1) / 2;
  static constexpr int XROWS = BN + KW - 1;          // key tile rows incl. halo
  static constexpr int XSTRIDE = kD * 2 + 16;        // bytes per key-tile row (padded: conflict-free b128 reads)
  static constexpr int VSTRIDE = kD * 2 + 64;        // bytes per value-tile row (conflict-free transposing reads)
  static constexpr int SSTRIDE = BN + 8;             // floats per row of a partial-logit buffer
  static constexpr int PSTRIDE = BN * 2 + 16;        // bytes per row of the bf16 probability tile
  static constexpr int XITEMS = XROWS * 16;          // 16-byte chunks of the key tile
  static constexpr int XPER = (XITEMS + kThreads - 1) / kThreads;
  static constexpr int XALLOC = XPER * kThreads / 16;  // rows allocated: every thread stores XPER chunks, no tail test
  static constexpr int XBYTES = XALLOC * XSTRIDE;
  static constexpr int VBYTES = BN * VSTRIDE;
  static constexpr int SBYTES = 4 * BM * SSTRIDE * 4;
  static constexpr int PBYTES = BM * PSTRIDE;
  static constexpr int LDS = 2 * (XBYTES + VBYTES) + SBYTES + PBYTES + 2 * BM * 4 + 16;
  static constexpr int RPW = BM / 4;                 // rows a wave owns in the softmax phase
  static constexpr int LPR = 64 / RPW;               // lanes per row there
  static constexpr int EPL = BN / LPR;               // positions per lane there
  static constexpr int VITEMS = BN * 16;             // 16-byte chunks of the value tile
  static constexpr int VPER = VITEMS / kThreads;
  static_assert(BM == 32 || BM == 64, "BM");
  static_assert(BN % 32 == 0 && VITEMS % kThreads == 0, "BN");
  static_assert(EPL % 4 == 0, "softmax lanes read whole float4s");
};

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);   // RNE; inputs here are finite
  return (uint16_t)(u >> 16);
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s supplies the
// address of 4 consecutive 16-bit elements; lane i of the group receives element (i % 4) of the
// chunks addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lane s pointing at
// (row r0 + s/4, column c0 + 4*(s%4)) of a row-major tile, lane i ends up with column c0 + i of
// rows r0 .. r0+3: a K x N operand fragment read straight from a row-major tile.
__device__ __forceinline__ s16x4 lds_read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// 16 bytes of row p of [cache ; block] (keys or values).  Branch-free: the address is clamped
// into [0, T) so the loads of a tile can all be in flight together; rows outside [0, T) are
// zeroed later, when the data is written to LDS (mask16).
__device__ __forceinline__ u32x4 load_cat16(const void* cache, const View& blk, int M, int m, int T,
                                            int b, int hkv, int Hkv, int p, int chunk) {
  const int pc = min(max(p, 0), T - 1);
  const bool in_cache = pc < m;
  const int64_t cache_off = ((int64_t)(b * Hkv + hkv) * M + pc) * kD;
  const int64_t blk_off = b * blk.sb + hkv * blk.sh + (int64_t)(pc - m) * blk.st;
  const uint16_t* base = in_cache ? (const uint16_t*)cache : (const uint16_t*)blk.p;
  const uint16_t* row = base + (in_cache ? cache_off : blk_off);
  return *(const u32x4*)(row + chunk * 8);
}

__device__ __forceinline__ u32x4 mask16(u32x4 v, bool keep_it) {
  const uint32_t keep = keep_it ? 0xffffffffu : 0u;
  v[0] &= keep; v[1] &= keep; v[2] &= keep; v[3] &= keep;
  return v;
}

// wp: filters repacked as [bank][M][KW][C] bf16.
template <int BM, int BN, int KW>
__global__ __launch_bounds__(kThreads, 1) void compress_mfma_k(StepArgs a, const uint16_t* wp,
                                                               int64_t wp_head_stride) {
  using G = Geo<BM, BN, KW>;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Xs0 = smem;
  unsigned char* Vs0 = smem + 2 * G::XBYTES;
  float* Sred = (float*)(smem + 2 * (G::XBYTES + G::VBYTES));
  unsigned char* Ps = (unsigned char*)Sred + G::SBYTES;
  float* alphas = (float*)(Ps + G::PBYTES);
  float* lsum = alphas + BM;
  int* rescale_flag = (int*)(lsum + BM);             // one word per wave

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int ch = blockIdx.y, b = ch / a.Hkv, hkv = ch % a.Hkv;
  const int i0 = blockIdx.x * BM;
  const int T = a.m + a.Bn;
  const int NT = (T + BN - 1) / BN;

  // ---- this wave's slice of the filter bank, resident in registers for the whole kernel
  bf16x8 wreg[G::RT][KW][2];
  {
    const uint16_t* wb = wp + hkv * wp_head_stride;
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int t = 0; t < KW; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int row = i0 + rt * 32 + l31;
          const int c = 32 * w + 16 * h + lh * 8;
          wreg[rt][t][h] = *(const bf16x8*)(wb + ((int64_t)row * KW + t) * kD + c);
        }
  }

  f32x16 oacc[G::RT][2];
#pragma unroll
  for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[rt][ct][i] = 0.f;

  // softmax state of the row this lane helps with (replicated over the LPR lanes of the row)
  const int srow = w * G::RPW + l / G::LPR;
  const int sp0 = (l % G::LPR) * G::EPL;
  float m_run = -INFINITY, l_run = 0.f;
  const float bias = a.conv_b ? __uint_as_float((uint32_t)((const uint16_t*)a.conv_b)[hkv * a.b_head_stride + i0 + srow] << 16)
                              : 0.f;

  // ---- staging: global -> registers -> LDS (key tile row-major with halo; [K|V] tile transposed)
  u32x4 xreg[G::XPER];
  u32x4 vreg[G::VPER];
  auto stage_load = [&](int j0) {
#pragma unroll
    for (int it = 0; it < G::XPER; ++it) {
      const int item = tid + it * kThreads;
      const int r = item >> 4, chunk = item & 15;
      xreg[it] = load_cat16(a.cache_k, a.k, a.M, a.m, T, b, hkv, a.Hkv, j0 - G::PAD + r, chunk);
    }
#pragma unroll
    for (int it = 0; it < G::VPER; ++it) {
      const int item = tid + it * kThreads;
      vreg[it] = load_cat16(a.cache_v, a.v, a.M, a.m, T, b, hkv, a.Hkv, j0 + (item >> 4), item & 15);
    }
  };
  auto stage_store = [&](int buf, int j0) {
    unsigned char* Xs = Xs0 + buf * G::XBYTES;
    unsigned char* Vs = Vs0 + buf * G::VBYTES;
#pragma unroll
    for (int it = 0; it < G::XPER; ++it) {
      const int item = tid + it * kThreads;
      const int r = item >> 4, chunk = item & 15;
      const int p = j0 - G::PAD + r;
      *(u32x4*)(Xs + r * G::XSTRIDE + chunk * 16) = mask16(xreg[it], p >= 0 && p < T);
    }
#pragma unroll
    for (int it = 0; it < G::VPER; ++it) {
      const int item = tid + it * kThreads;
      *(u32x4*)(Vs + (item >> 4) * G::VSTRIDE + (item & 15) * 16) =
          mask16(vreg[it], j0 + (item >> 4) < T);
    }
  };

  stage_load(0);
  stage_store(0, 0);
  __syncthreads();

  for (int jt = 0; jt < NT; ++jt) {
    const int buf = jt & 1;
    const int j0 = jt * BN;
    const unsigned char* Xs = Xs0 + buf * G::XBYTES;
    const unsigned char* Vs = Vs0 + buf * G::VBYTES;
    stage_load(j0 + BN);     // past the last tile the clamped addresses still point into the chain

    // ---- Eq. 5: partial logits over this wave's channel quarter
    f32x16 sacc[G::RT][G::PT];
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int pt = 0; pt < G::PT; ++pt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[rt][pt][i] = 0.f;
    {
      // key operands are fetched from LDS kRing contraction steps ahead of their MFMAs
      constexpr int NS = KW * 2;                 // contraction steps: (tap, channel half)
      constexpr int kRing = 4;
      bf16x8 xv[kRing][G::PT];
      const unsigned char* xbase = Xs + l31 * G::XSTRIDE + (32 * w + lh * 8) * 2;
      auto fetch = [&](int st) {
        const int t = st >> 1, h = st & 1;
#pragma unroll
        for (int pt = 0; pt < G::PT; ++pt)
          xv[st % kRing][pt] = *(const bf16x8*)(xbase + (pt * 32 + t) * G::XSTRIDE + h * 32);
      };
#pragma unroll
      for (int st = 0; st < kRing - 1; ++st) fetch(st);
#pragma unroll
      for (int st = 0; st < NS; ++st) {
        if (st + kRing - 1 < NS) fetch(st + kRing - 1);
        const int t = st >> 1, h = st & 1;
#pragma unroll
        for (int pt = 0; pt < G::PT; ++pt)
#pragma unroll
          for (int rt = 0; rt < G::RT; ++rt)
            sacc[rt][pt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wreg[rt][t][h], xv[st % kRing][pt],
                                                                   sacc[rt][pt], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);       // keep the fetch-ahead order (the scheduler would sink the reads)
      }
    }
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int pt = 0; pt < G::PT; ++pt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = rt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
          Sred[(w * BM + row) * G::SSTRIDE + pt * 32 + l31] = sacc[rt][pt][i];
        }
    __syncthreads();

    // ---- sum the four partials, Eq. 6 as an online softmax over positions
    {
      float s[G::EPL];
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) s[e] = bias;
#pragma unroll
      for (int ww = 0; ww < 4; ++ww)
#pragma unroll
        for (int e4 = 0; e4 < G::EPL / 4; ++e4) {
          const float4 v = *(const float4*)(Sred + (ww * BM + srow) * G::SSTRIDE + sp0 + e4 * 4);
          s[e4 * 4 + 0] += v.x; s[e4 * 4 + 1] += v.y; s[e4 * 4 + 2] += v.z; s[e4 * 4 + 3] += v.w;
        }
      if (j0 + BN > T) {                                   // tail tile: positions past T carry no weight
#pragma unroll
        for (int e = 0; e < G::EPL; ++e)
          if (j0 + sp0 + e >= T) s[e] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) mx = fmaxf(mx, s[e]);
#pragma unroll
      for (int o = 1; o < G::LPR; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
      // Lazy reference point: the running reference only moves when the row maximum outgrows
      // it by kLazy, so exp(s - ref) stays below e^kLazy and rescaling the accumulators is rare.
      const bool bump = mx > m_run + kLazy;                // every tile has a position < T, so mx is finite
      const float m_new = bump ? mx : m_run;
      const float alpha = bump ? __expf(m_run - m_new) : 1.0f;
      const bool any_bump = __any(bump);
      float psum = 0.f;
      uint16_t pb[G::EPL];
#pragma unroll
      for (int e = 0; e < G::EPL; ++e) {
        const float p = __expf(s[e] - m_new);
        psum += p;
        pb[e] = f2bf(p);
      }
#pragma unroll
      for (int o = 1; o < G::LPR; o <<= 1) psum += __shfl_xor(psum, o, 64);
      l_run = l_run * alpha + psum;
      m_run = m_new;
#pragma unroll
      for (int e2 = 0; e2 < G::EPL / 2; ++e2)
        *(uint32_t*)(Ps + srow * G::PSTRIDE + (sp0 + 2 * e2) * 2) =
            (uint32_t)pb[2 * e2] | ((uint32_t)pb[2 * e2 + 1] << 16);
      if ((l % G::LPR) == 0) alphas[srow] = alpha;
      if (l == 0) rescale_flag[w] = any_bump;
    }
    stage_store(buf ^ 1, j0 + BN);
    __syncthreads();

    // ---- Eq. 4a/4b: (rarely) rescale, then accumulate P . [K | V] for this wave's 64 columns
    if (rescale_flag[0] | rescale_flag[1] | rescale_flag[2] | rescale_flag[3]) {
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float al = alphas[rt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)];
          oacc[rt][0][i] *= al;
          oacc[rt][1][i] *= al;
        }
    }
    {
      // wave 0/1: key columns 64w.. from the key tile (skipping its leading halo rows);
      // wave 2/3: value columns 64(w-2).. from the value tile.  Transposing reads, see lds_read_tr.
      const int s16 = l & 15, g2 = (l >> 4) & 1;
      const unsigned char* ybase =
          (w < 2 ? Xs + (G::PAD + lh * 8 + (s16 >> 2)) * G::XSTRIDE + (64 * w) * 2
                 : Vs + (lh * 8 + (s16 >> 2)) * G::VSTRIDE + (64 * (w - 2)) * 2) +
          (16 * g2 + 4 * (s16 & 3)) * 2;
      const int ystride = w < 2 ? G::XSTRIDE : G::VSTRIDE;
#pragma unroll
      for (int ks = 0; ks < BN / 16; ++ks) {
        bf16x8 pv[G::RT];
#pragma unroll
        for (int rt = 0; rt < G::RT; ++rt)
          pv[rt] = *(const bf16x8*)(Ps + (rt * 32 + l31) * G::PSTRIDE + (ks * 16 + lh * 8) * 2);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          const unsigned char* yp = ybase + (ks * 16) * ystride + (ct * 32) * 2;
          const s16x4 y0 = lds_read_tr(yp);
          const s16x4 y1 = lds_read_tr(yp + 4 * ystride);
          const s16x8 yy = {y0[0], y0[1], y0[2], y0[3], y1[0], y1[1], y1[2], y1[3]};
          const bf16x8 yv = __builtin_bit_cast(bf16x8, yy);
#pragma unroll
          for (int rt = 0; rt < G::RT; ++rt)
            oacc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pv[rt], yv, oacc[rt][ct], 0, 0, 0);
        }
      }
    }
  }

  // ---- normalise by the row sums and store the new cache rows
  if ((l % G::LPR) == 0) lsum[srow] = l_run;
  __syncthreads();
  uint16_t* nk = (uint16_t*)a.new_k + ((int64_t)ch * a.M + i0) * kD;
  uint16_t* nv = (uint16_t*)a.new_v + ((int64_t)ch * a.M + i0) * kD;
#pragma unroll
  for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = rt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
      const float inv = 1.0f / lsum[row];
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) {
        const int col = 64 * w + ct * 32 + l31;          // 0..127: K, 128..255: V
        uint16_t* dst = (col < kD ? nk : nv) + (int64_t)row * kD + (col & (kD - 1));
        *dst = f2bf(oacc[rt][ct][i] * inv);
      }
    }
}

// [M][C][k] -> [M][k][C] per bank, so that 8 consecutive channels of one tap are 16 contiguous bytes.
__global__ void repack_filters_k(const uint16_t* w, uint16_t* wp, int M, int C, int KW, int banks,
                                 int64_t w_head_stride) {
  const int64_t per = (int64_t)M * C * KW;
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < per * banks;
       e += (int64_t)gridDim.x * blockDim.x) {
    const int bank = (int)(e / per);
    const int64_t r = e % per;
    const int c = (int)(r % C), t = (int)((r / C) % KW), i = (int)(r / ((int64_t)C * KW));
    wp[e] = w[bank * w_head_stride + ((int64_t)i * C + c) * KW + t];
  }
}

template <int BM, int BN, int KW>
hipError_t launch_one(const StepArgs& a, const uint16_t* wp, int64_t wp_head_stride, hipStream_t s) {
  using G = Geo<BM, BN, KW>;
  static bool attr_set = false;   // benign race: setting it twice is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)compress_mfma_k<BM, BN, KW>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, G::LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  dim3 grid(a.M / BM, a.batch * a.Hkv);
  hipLaunchKernelGGL((compress_mfma_k<BM, BN, KW>), grid, dim3(kThreads), G::LDS, s, a, wp,
                     wp_head_stride);
  return hipGetLastError();
}

}  // namespace

bool compress_mfma_supports(int dtype, int d, int M, int conv_width, int conv_in, int norm,
                            const char** why) {
  if (dtype != LOCOCO_BF16) { *why = "the MFMA kernels take bf16 storage only"; return false; }
  if (d != kD) { *why = "the MFMA kernels take head_dim = 128 only"; return false; }
  if (conv_in != 0) { *why = "the MFMA compression kernel takes keys-only filters (conv_in = 0)"; return false; }
  if (norm != 0) { *why = "the MFMA compression kernel implements the softmax normalisation only"; return false; }
  if (conv_width != 15) { *why = "the MFMA compression kernel is built for conv_width = 15"; return false; }
  if (M % 32) { *why = "the MFMA compression kernel needs M to be a multiple of 32"; return false; }
  return true;
}

size_t compress_mfma_filter_bytes(int M, int conv_width, int banks) {
  return (size_t)banks * M * conv_width * kD * 2;
}

hipError_t launch_repack_filters(const StepArgs& a, void* wp, int banks, hipStream_t s) {
  const int64_t n = (int64_t)banks * a.M * kD * a.k_width;
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(repack_filters_k, dim3(blocks), dim3(256), 0, s, (const uint16_t*)a.conv_w,
                     (uint16_t*)wp, a.M, kD, a.k_width, banks, a.w_head_stride);
  return hipGetLastError();
}

hipError_t launch_compress_mfma(const StepArgs& a, const void* wp, int banks, int n_cu,
                                hipStream_t s) {
  const int64_t wp_head_stride = banks > 1 ? (int64_t)a.M * a.k_width * kD : 0;
  const int chains = a.batch * a.Hkv;
  // 64-row tiles when they still give every compute unit a workgroup, else 32-row tiles
  const bool big = (a.M % 64 == 0) && (int64_t)chains * (a.M / 64) >= n_cu;
  static int bn = 0;
  if (!bn) { const char* e = getenv("LOCOCO_DEV_BN"); bn = e ? atoi(e) : 32; }
  if (big && bn == 64) return launch_one<64, 64, 15>(a, (const uint16_t*)wp, wp_head_stride, s);
  if (big) return launch_one<64, 32, 15>(a, (const uint16_t*)wp, wp_head_stride, s);
  return launch_one<32, 32, 15>(a, (const uint16_t*)wp, wp_head_stride, s);
}

}  // namespace lococo
