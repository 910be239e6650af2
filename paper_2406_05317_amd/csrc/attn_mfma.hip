// Block-vs-(cache+block) causal attention for gfx950 (Alg. 2 step 3, Eq. 1):
// bf16 MFMA, fp32 accumulation and softmax, K/V tiles staged through LDS,
// online softmax.  One launch covers one block or, for a whole sequence whose
// intermediate caches were kept, every block at once.
//
// Each workgroup takes 128 query rows of one (batch, query head, block); each
// of its four waves owns 32 of them.  The kernel works on the TRANSPOSED
// score tile S^T = K Q^T (keys are MFMA rows, queries are MFMA columns), so
// that one lane holds scores of a single query: row maxima and sums need one
// cross-lane exchange, the rescale factor is a per-lane scalar, and the
// probabilities feed the second MFMA (O^T = V^T P^T) straight from registers.
// The key order inside the second contraction is permuted the same way on
// both operands so no shuffle is needed; the value operand is read with the
// transposing LDS load straight from the row-major value tile.
//
// Keys are indexed over [cache ; block]: all m cache slots are visible, block
// key j' is visible to block query j iff j' <= j; key tiles past a wave's
// diagonal are skipped.  Shapes taken: head_dim = 128, bf16.
#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kD = 128;
constexpr int kThreads = 256;
constexpr int BQ = 128;                       // query rows per workgroup
constexpr int BK = 64;                        // keys per tile
constexpr int KSTRIDE = kD * 2 + 16;          // bytes per key-tile row (conflict-free 16-byte reads)
constexpr int VSTRIDE = kD * 2 + 64;          // bytes per value-tile row (conflict-free transposing reads)
constexpr int KBYTES = BK * KSTRIDE;
constexpr int VBYTES = BK * VSTRIDE;
constexpr int LDS_BYTES = 2 * (KBYTES + VBYTES);
constexpr int PER = BK * 16 / kThreads;       // 16-byte chunks of a key (or value) tile per thread
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;                 // the softmax reference lags the row maximum by at most this much

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // v_cvt_pk_bf16_f32, RNE
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s supplies the
// address of 4 consecutive 16-bit elements; lane i of the group receives element (i % 4) of the
// chunks addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lane s pointing at
// (row r0 + s/4, column c0 + 4*(s%4)) of a row-major tile, lane i ends up with column c0 + i of
// rows r0 .. r0+3: an operand fragment (column, 4 contraction rows) straight from a row-major tile.
__device__ __forceinline__ s16x4 lds_read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// [cache ; block] rows through two raw buffer resources: an index outside a resource's range reads
// as zero without touching memory, so OR-ing the two loads gives row j of the concatenation for
// 0 <= j < T and zeros elsewhere (only tiles that straddle the seam need both).
struct CatRows {
  __amdgpu_buffer_rsrc_t cache, blk;
  int m, blk_stride;
};
__device__ __forceinline__ CatRows make_cat(const uint16_t* cache_rows, int m, const uint16_t* blk_rows,
                                            int64_t blk_st, int Bn) {
  CatRows c;
  c.cache = __builtin_amdgcn_make_buffer_rsrc((void*)cache_rows, 0, m * kD * 2, 0x00020000);
  c.blk = __builtin_amdgcn_make_buffer_rsrc((void*)blk_rows, 0, (int)((Bn - 1) * blk_st + kD) * 2,
                                            0x00020000);
  c.m = m;
  c.blk_stride = (int)blk_st * 2;
  return c;
}
struct Cat16 { u32x4 from_cache, from_blk; };

__global__ __launch_bounds__(kThreads, 2) void attn_mfma_k(AttnArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Ks0 = smem;
  unsigned char* Vs0 = smem + 2 * KBYTES;

  // ---- work item: consecutive items share K/V; spread so that they land on one XCD
  int item = blockIdx.x;
  {
    const int total = gridDim.x, per = total / 8;
    if (item < per * 8) item = (item % 8) * per + item / 8;
  }
  const int qt = item % a.qtiles;
  const int hq = (item / a.qtiles) % a.Hq;
  const int b = (item / a.qtiles / a.Hq) % a.batch;
  const int n = a.seg_first + item / a.qtiles / a.Hq / a.batch;

  const int64_t start = (int64_t)n * a.B;
  const int Bn = (int)(a.L - start < a.B ? a.L - start : a.B);
  const int m = n <= a.n_fill ? a.len0 + n * a.B : a.M;
  const int q0 = qt * BQ;
  if (q0 >= Bn) return;
  const int hkv = hq / a.group;
  const int chain = b * a.Hkv + hkv;
  const int T = m + Bn;

  const uint16_t* cache_k;
  const uint16_t* cache_v;
  if (n <= a.n_fill) {
    cache_k = (const uint16_t*)a.cache_k + (int64_t)chain * a.M * kD;
    cache_v = (const uint16_t*)a.cache_v + (int64_t)chain * a.M * kD;
  } else {
    const int64_t slot = (int64_t)(n - a.n_fill - 1) * a.hist_stride + (int64_t)chain * a.M * kD;
    cache_k = (const uint16_t*)a.hist_k + slot;
    cache_v = (const uint16_t*)a.hist_v + slot;
  }
  const CatRows cat_k =
      make_cat(cache_k, m, (const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + start * a.k.st, a.k.st, Bn);
  const CatRows cat_v =
      make_cat(cache_v, m, (const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + start * a.v.st, a.v.st, Bn);
  const uint16_t* qb = (const uint16_t*)a.q.p + b * a.q.sb + hq * a.q.sh + start * a.q.st;
  uint16_t* ob = (uint16_t*)a.o.p + b * a.o.sb + hq * a.o.sh + start * a.o.st;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int wq0 = q0 + 32 * w;          // first query row of this wave
  const int qrow = wq0 + l31;           // this lane's query (block-relative)

  // ---- this lane's query row as the B operand of S^T = K Q^T
  bf16x8 qreg[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    u32x4 v = {0u, 0u, 0u, 0u};
    if (qrow < Bn) v = *(const u32x4*)(qb + (int64_t)qrow * a.q.st + ks * 16 + lh * 8);
    qreg[ks] = __builtin_bit_cast(bf16x8, v);
  }

  f32x16 oacc[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[ct][i] = 0.f;
  // running softmax reference (in raw score units) and row sum; exp(x * scale) = exp2(x * c)
  const float c = a.scale * kLog2e;
  const float lazy_raw = kLazy / a.scale;
  float m_run = -INFINITY, l_run = 0.f;

  // keys this workgroup needs: the cache and the block up to its last query row
  const int kend = min(T, m + q0 + BQ);
  const int NT = (kend + BK - 1) / BK;

  // A tile that lies wholly in the cache or wholly in the block needs one load per chunk; only a
  // tile straddling the seam issues both and ORs them.  (src: 1 = cache, 2 = block, 3 = both.)
  Cat16 kreg[PER], vreg[PER];
  auto tile_src = [&](int key0) { return (key0 < m ? 1 : 0) | (key0 + BK > m ? 2 : 0); };
  auto stage_load = [&](int key0, int src) {
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int idx = tid + it * kThreads;
      const int j = key0 + (idx >> 4), chunk = idx & 15;
      if (src & 1) {
        kreg[it].from_cache = __builtin_amdgcn_raw_buffer_load_b128(cat_k.cache, j * (kD * 2) + chunk * 16, 0, 0);
        vreg[it].from_cache = __builtin_amdgcn_raw_buffer_load_b128(cat_v.cache, j * (kD * 2) + chunk * 16, 0, 0);
      }
      if (src & 2) {
        kreg[it].from_blk = __builtin_amdgcn_raw_buffer_load_b128(cat_k.blk, (j - m) * cat_k.blk_stride + chunk * 16, 0, 0);
        vreg[it].from_blk = __builtin_amdgcn_raw_buffer_load_b128(cat_v.blk, (j - m) * cat_v.blk_stride + chunk * 16, 0, 0);
      }
    }
  };
  auto stage_store = [&](int buf, int src) {
    unsigned char* Ks = Ks0 + buf * KBYTES;
    unsigned char* Vs = Vs0 + buf * VBYTES;
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int idx = tid + it * kThreads;
      u32x4* kd = (u32x4*)(Ks + (idx >> 4) * KSTRIDE + (idx & 15) * 16);
      u32x4* vd = (u32x4*)(Vs + (idx >> 4) * VSTRIDE + (idx & 15) * 16);
      if (src == 1) { *kd = kreg[it].from_cache; *vd = vreg[it].from_cache; }
      else if (src == 2) { *kd = kreg[it].from_blk; *vd = vreg[it].from_blk; }
      else { *kd = kreg[it].from_cache | kreg[it].from_blk; *vd = vreg[it].from_cache | vreg[it].from_blk; }
    }
  };

  stage_load(0, tile_src(0));
  stage_store(0, tile_src(0));
  __syncthreads();

  // value fragments: lane (head-dim column ct*32 + l31) x 8 keys.  The key order inside a
  // contraction step follows the layout the probabilities already have in the score accumulator:
  // slot j of step u is key u*16 + (j/4)*8 + lh*4 + j%4 (see below), so nothing is shuffled.
  const int s16 = l & 15, g2 = (l >> 4) & 1;
  const int v_lane_off = (lh * 4 + (s16 >> 2)) * VSTRIDE + (16 * g2 + 4 * (s16 & 3)) * 2;

  for (int t = 0; t < NT; ++t) {
    const int buf = t & 1;
    const int key0 = t * BK;
    const unsigned char* Ks = Ks0 + buf * KBYTES;
    const unsigned char* Vs = Vs0 + buf * VBYTES;
    // past the last tile the loads are out of range of their resource: zeros, no memory traffic
    const int src_next = tile_src(key0 + BK);
    stage_load(key0 + BK, src_next);

    if (key0 < m + wq0 + 32) {           // some key of the tile is visible to some query of this wave
      // ---- S^T tile: keys x queries
      f32x16 sacc[BK / 32];
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kv = *(const bf16x8*)(Ks + (kt * 32 + l31) * KSTRIDE + (ks * 16 + lh * 8) * 2);
          sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qreg[ks], ks == 0 ? zero : sacc[kt], 0, 0, 0);
        }
      }
      // ---- mask, online softmax with a lazy reference (everything of one query sits in one lane pair)
      if (key0 + BK > m + wq0 || key0 + BK > T) {
#pragma unroll
        for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = key0 + kt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
            if (key >= T || key - m > qrow) sacc[kt][i] = -INFINITY;
          }
      }
      float mx = sacc[0][0];
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kt][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // The reference only moves when the row maximum outgrows it by kLazy (in exponent units),
      // so exp(..) stays below e^kLazy and the accumulator is rescaled rarely.
      const bool bump = mx > m_run + lazy_raw;
      const float m_new = bump ? mx : m_run;
      if (__any(bump)) {
        const float alpha = bump ? __builtin_amdgcn_exp2f((m_run - m_new) * c) : 1.0f;
        l_run *= alpha;
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
      }
      m_run = m_new;
      const float mc = m_new * c;
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kt][i] = __builtin_amdgcn_exp2f(fmaf(sacc[kt][i], c, -mc));
      float psum = 0.f;
      // ---- O^T += V^T P^T; contraction slot j of step u holds key (u*16 + (j/4)*8 + lh*4 + j%4)
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          u32x4 pp;
#pragma unroll
          for (int j2 = 0; j2 < 4; ++j2) {
            pp[j2] = pack_bf16(sacc[kt][u * 8 + 2 * j2], sacc[kt][u * 8 + 2 * j2 + 1]);
            psum += sacc[kt][u * 8 + 2 * j2] + sacc[kt][u * 8 + 2 * j2 + 1];
          }
          const bf16x8 pv = __builtin_bit_cast(bf16x8, pp);
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            const unsigned char* vp = Vs + (kt * 32 + u * 16) * VSTRIDE + (ct * 32) * 2 + v_lane_off;
            const s16x4 y0 = lds_read_tr(vp);
            const s16x4 y1 = lds_read_tr(vp + 8 * VSTRIDE);
            const s16x8 yy = {y0[0], y0[1], y0[2], y0[3], y1[0], y1[1], y1[2], y1[3]};
            oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, yy), pv,
                                                               oacc[ct], 0, 0, 0);
          }
        }
      psum += __shfl_xor(psum, 32, 64);
      l_run += psum;
    }
    stage_store(buf ^ 1, src_next);
    __syncthreads();
  }

  // ---- O = O^T / l: lane holds query qrow, head-dim columns ct*32 + (i/4)*8 + lh*4 + i%4
  if (qrow < Bn) {
    const float inv = 1.0f / l_run;
    uint16_t* orow = ob + (int64_t)qrow * a.o.st;
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[ct][g * 4 + 0] * inv, oacc[ct][g * 4 + 1] * inv);
        pk[1] = pack_bf16(oacc[ct][g * 4 + 2] * inv, oacc[ct][g * 4 + 3] * inv);
        *(u32x2*)(orow + ct * 32 + g * 8 + lh * 4) = pk;
      }
  }
}

}  // namespace

bool attn_mfma_supports(int dtype, int d, const char** why) {
  if (dtype != LOCOCO_BF16) { *why = "the MFMA kernels take bf16 storage only"; return false; }
  if (d != kD) { *why = "the MFMA kernels take head_dim = 128 only"; return false; }
  return true;
}

hipError_t launch_attn_mfma(const AttnArgs& a_in, hipStream_t s) {
  AttnArgs a = a_in;
  a.qtiles = (a.B + BQ - 1) / BQ;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_k,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t total = (int64_t)a.qtiles * a.Hq * a.batch * a.n_seg;
  if (total <= 0) return hipSuccess;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attn_mfma_k, dim3((unsigned)total), dim3(kThreads), LDS_BYTES, s, a);
  return hipGetLastError();
}

}  // namespace lococo
