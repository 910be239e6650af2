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
// both operands so no shuffle is needed.
//
// Keys are indexed over [cache ; block]: all m cache slots are visible, block
// key j' is visible to block query j iff j' <= j; key tiles past a wave's
// diagonal are skipped.  Shapes taken: head_dim = 128, bf16.
#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kD = 128;
constexpr int kThreads = 256;
constexpr int BQ = 128;                       // query rows per workgroup
constexpr int BK = 64;                        // keys per tile
constexpr int KSTRIDE = kD * 2 + 16;          // bytes per key-tile row
constexpr int VSTRIDE = BK * 2 + 8;           // bytes per row of the transposed value tile
constexpr int KBYTES = BK * KSTRIDE;
constexpr int VBYTES = kD * VSTRIDE;
constexpr int LDS_BYTES = 2 * (KBYTES + VBYTES);
constexpr int KPER = BK * 16 / kThreads;      // 16-byte chunks of the key tile per thread
constexpr int VPER = (BK / 2) * 16 / kThreads;  // (key pair, chunk) items of the value tile per thread

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  uint32_t a = __float_as_uint(lo), b = __float_as_uint(hi);
  a += 0x7fffu + ((a >> 16) & 1u);
  b += 0x7fffu + ((b >> 16) & 1u);
  return (a >> 16) | (b & 0xffff0000u);
}

// 16 bytes of row j of [cache ; block].  Branch-free (address clamped below T) so that all loads
// of a tile are in flight together; rows j >= T are zeroed when written to LDS (mask16).
__device__ __forceinline__ u32x4 load_cat16(const uint16_t* cache_rows, const uint16_t* blk_rows,
                                            int64_t blk_st, int m, int T, int j, int chunk) {
  const int jc = min(j, T - 1);
  const bool in_cache = jc < m;
  const uint16_t* row = in_cache ? cache_rows + (int64_t)jc * kD : blk_rows + (int64_t)(jc - m) * blk_st;
  return *(const u32x4*)(row + chunk * 8);
}

__device__ __forceinline__ u32x4 mask16(u32x4 v, bool keep_it) {
  const uint32_t keep = keep_it ? 0xffffffffu : 0u;
  v[0] &= keep; v[1] &= keep; v[2] &= keep; v[3] &= keep;
  return v;
}

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
  const uint16_t* kb = (const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + start * a.k.st;
  const uint16_t* vb = (const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + start * a.v.st;
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
  float m_run = -INFINITY, l_run = 0.f;

  // keys this workgroup needs: the cache and the block up to its last query row
  const int kend = min(T, m + q0 + BQ);
  const int NT = (kend + BK - 1) / BK;

  u32x4 kreg[KPER];
  u32x4 vreg[VPER][2];
  auto stage_load = [&](int key0) {
#pragma unroll
    for (int it = 0; it < KPER; ++it) {
      const int idx = tid + it * kThreads;
      kreg[it] = load_cat16(cache_k, kb, a.k.st, m, T, key0 + (idx >> 4), idx & 15);
    }
#pragma unroll
    for (int it = 0; it < VPER; ++it) {
      const int idx = tid + it * kThreads;
      const int pair = idx % (BK / 2), chunk = idx / (BK / 2);
      vreg[it][0] = load_cat16(cache_v, vb, a.v.st, m, T, key0 + 2 * pair, chunk);
      vreg[it][1] = load_cat16(cache_v, vb, a.v.st, m, T, key0 + 2 * pair + 1, chunk);
    }
  };
  auto stage_store = [&](int buf, int key0) {
    unsigned char* Ks = Ks0 + buf * KBYTES;
    unsigned char* Vs = Vs0 + buf * VBYTES;
#pragma unroll
    for (int it = 0; it < KPER; ++it) {
      const int idx = tid + it * kThreads;
      *(u32x4*)(Ks + (idx >> 4) * KSTRIDE + (idx & 15) * 16) = mask16(kreg[it], key0 + (idx >> 4) < T);
    }
#pragma unroll
    for (int it = 0; it < VPER; ++it) {
      const int idx = tid + it * kThreads;
      const int pair = idx % (BK / 2), chunk = idx / (BK / 2);
      const u32x4 v0 = mask16(vreg[it][0], key0 + 2 * pair < T);
      const u32x4 v1 = mask16(vreg[it][1], key0 + 2 * pair + 1 < T);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const uint32_t lo = (v0[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
        const uint32_t hi = (v1[e >> 1] >> ((e & 1) * 16)) & 0xffffu;
        *(uint32_t*)(Vs + (chunk * 8 + e) * VSTRIDE + pair * 4) = lo | (hi << 16);
      }
    }
  };

  stage_load(0);
  stage_store(0, 0);
  __syncthreads();

  for (int t = 0; t < NT; ++t) {
    const int buf = t & 1;
    const int key0 = t * BK;
    const unsigned char* Ks = Ks0 + buf * KBYTES;
    const unsigned char* Vs = Vs0 + buf * VBYTES;
    const bool more = t + 1 < NT;
    if (more) stage_load(key0 + BK);

    if (key0 < m + wq0 + 32) {           // some key of the tile is visible to some query of this wave
      // ---- S^T tile: keys x queries
      f32x16 sacc[BK / 32];
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kv = *(const bf16x8*)(Ks + (kt * 32 + l31) * KSTRIDE + (ks * 16 + lh * 8) * 2);
          sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qreg[ks], sacc[kt], 0, 0, 0);
        }
      }
      // ---- scale, mask, online softmax (everything of one query sits in one lane pair)
      const bool need_mask = key0 + BK > m + wq0 || key0 + BK > T;
      float mx = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float s = sacc[kt][i] * a.scale;
          if (need_mask) {
            const int key = key0 + kt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
            if (key >= T || key - m > qrow) s = -INFINITY;
          }
          sacc[kt][i] = s;
          mx = fmaxf(mx, s);
        }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      const float alpha = __expf(m_run - m_new);
      float psum = 0.f;
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float p = __expf(sacc[kt][i] - m_new);
          sacc[kt][i] = p;
          psum += p;
        }
      psum += __shfl_xor(psum, 32, 64);
      l_run = l_run * alpha + psum;
      m_run = m_new;
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][i] *= alpha;
      // ---- O^T += V^T P^T; contraction slot j of step u holds key (u*16 + (j/4)*8 + lh*4 + j%4)
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          u32x4 pp;
#pragma unroll
          for (int j2 = 0; j2 < 4; ++j2)
            pp[j2] = pack_bf16(sacc[kt][u * 8 + 2 * j2], sacc[kt][u * 8 + 2 * j2 + 1]);
          const bf16x8 pv = __builtin_bit_cast(bf16x8, pp);
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            const unsigned char* vrow = Vs + (ct * 32 + l31) * VSTRIDE + (kt * 32 + u * 16 + lh * 4) * 2;
            const u32x2 lo = *(const u32x2*)vrow;
            const u32x2 hi = *(const u32x2*)(vrow + 16);
            const u32x4 vv = {lo[0], lo[1], hi[0], hi[1]};
            oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pv,
                                                               oacc[ct], 0, 0, 0);
          }
        }
    }
    if (more) stage_store(buf ^ 1, key0 + BK);
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
