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

#include <type_traits>

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
constexpr int BK = 64;                        // keys per tile
constexpr int KSTRIDE = kD * 2 + 16;          // bytes per key-tile row (conflict-free 16-byte reads)
constexpr int VSTRIDE = kD * 2 + 64;          // bytes per value-tile row (conflict-free transposing reads)
constexpr int KBYTES = BK * KSTRIDE;
constexpr int VBYTES = BK * VSTRIDE;
constexpr int LDS_BYTES = 2 * (KBYTES + VBYTES);
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

// The keys of a block's attention are [cache ; block].  The walk over them is split at the seam:
// tiles of 64 cache slots first (the last one ragged when m is no multiple of 64), then tiles of
// 64 block keys, so that every tile comes from one array.  Rows are fetched through raw buffer
// resources sized to the array: a row past its end reads as zero without touching memory.
struct Rows {
  u32x4 rsrc;                                 // raw buffer resource: base, 0 stride, bytes, 32-bit format
  int stride;                                 // bytes between rows
};
__device__ __forceinline__ Rows make_rows(const uint16_t* p, int n, int64_t st) {
  Rows r;
  const uint64_t base = (uint64_t)p;
  r.rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
  r.rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
  r.rsrc[2] = __builtin_amdgcn_readfirstlane(n > 0 ? (uint32_t)((n - 1) * st + kD) * 2u : 0u);
  r.rsrc[3] = 0x00020000u;
  r.stride = (int)st * 2;
  return r;
}
// A 16-byte load the compiler does not wait for: the caller counts the loads in flight and puts
// `wait_loads<N>()` (at most N of the newest still pending; they complete in order) before the
// first use of the register.  An offset beyond the resource reads zero and moves no data.
__device__ __forceinline__ void load16_async(u32x4& dst, const u32x4& rsrc, int voff) {
  asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(rsrc) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// QB = 32-query column blocks per wave, NW = waves per workgroup.  Launched with QB = 1, NW = 4:
// 128 queries per workgroup, two workgroups per compute unit.  (QB = 2 halves the LDS reads per
// flop but needs the whole register file for one wave per SIMD, which then has to issue every
// vector, LDS and matrix instruction itself; NW = 8 halves the staging per query but loses the
// second, independent workgroup.  Both measured slower on the 32 K-token workload.)
template <int QB, int NW>
__global__ __launch_bounds__(64 * NW, 8 / NW) void attn_mfma_k(AttnArgs a) {
  constexpr int kThreads = 64 * NW;           // NW waves, 32 * QB query rows each
  constexpr int BQ = 32 * QB * NW;            // query rows per workgroup
  constexpr int PER = BK * 16 / kThreads;     // 16-byte chunks of a key (or value) tile per thread
  constexpr int WQ = 32 * QB;                 // query rows per wave
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
  const Rows ck = make_rows(cache_k, m, kD), cv = make_rows(cache_v, m, kD);
  const Rows bk = make_rows((const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + start * a.k.st, Bn, a.k.st);
  const Rows bv = make_rows((const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + start * a.v.st, Bn, a.v.st);
  const uint16_t* qb_ptr = (const uint16_t*)a.q.p + b * a.q.sb + hq * a.q.sh + start * a.q.st;
  uint16_t* ob = (uint16_t*)a.o.p + b * a.o.sb + hq * a.o.sh + start * a.o.st;

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int wq0 = q0 + WQ * w;          // first query row of this wave
  // this lane's queries (block-relative): wq0 + 32*qb + l31

  // ---- this lane's query rows as the B operand of S^T = K Q^T.  The rows are fetched whole
  // (16 lanes x 16 bytes = one row per quarter wave, 1 KB contiguous per instruction), parked in a
  // wave-private piece of the key-tile area and read back as operand fragments; rows past the
  // block read as zero.
  bf16x8 qreg[QB][8];
  {
    const Rows qr = make_rows(qb_ptr, Bn, a.q.st);
    unsigned char* Qs = smem + w * (WQ * KSTRIDE);
    u32x4 qrow_regs[WQ / 4];
#pragma unroll
    for (int i = 0; i < WQ / 4; ++i)
      load16_async(qrow_regs[i], qr.rsrc, (wq0 + i * 4 + (l >> 4)) * qr.stride + (l & 15) * 16);
    wait_loads<0>();
#pragma unroll
    for (int i = 0; i < WQ / 4; ++i) asm volatile("" : "+v"(qrow_regs[i]));
#pragma unroll
    for (int i = 0; i < WQ / 4; ++i) *(u32x4*)(Qs + (i * 4 + (l >> 4)) * KSTRIDE + (l & 15) * 16) = qrow_regs[i];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        qreg[qb][ks] = *(const bf16x8*)(Qs + (32 * qb + l31) * KSTRIDE + ks * 32 + lh * 16);
  }

  f32x16 oacc[QB][4];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[qb][ct][i] = 0.f;
  // running softmax reference (in raw score units) and row sum; exp(x * scale) = exp2(x * c)
  const float c = a.scale * kLog2e;
  const float lazy_raw = kLazy / a.scale;
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

  // tiles: NTc over the cache, then over the block up to this workgroup's last query row
  const int NTc = (m + BK - 1) / BK;
  const int NT = NTc + (min(Bn, q0 + BQ) + BK - 1) / BK;

  // Two sets of staging registers: the loads of tile t + 2 are issued at the top of iteration t
  // and land in LDS at the end of iteration t + 1, so a load has two iterations to arrive (the
  // loaded latency of this access pattern is about one iteration).  Every call issues exactly
  // 2 * PER loads per lane, also past the last tile (offsets out of range: zeros, no traffic), so
  // that "at most 2 * PER pending" always means "the older set has arrived".
  u32x4 kreg0[PER], vreg0[PER], kreg1[PER], vreg1[PER];
  auto stage_load = [&](int t, u32x4* kreg, u32x4* vreg) {
    const bool blk = t >= NTc;
    const int row0 = (blk ? t - NTc : t) * BK;
    const u32x4 rk = blk ? bk.rsrc : ck.rsrc, rv = blk ? bv.rsrc : cv.rsrc;
    const int sk = blk ? bk.stride : ck.stride, sv = blk ? bv.stride : cv.stride;
    const int beyond = t >= NT ? 0x7fff0000 : 0;
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int idx = tid + it * kThreads;
      const int j = row0 + (idx >> 4), chunk = idx & 15;
      load16_async(kreg[it], rk, (j * sk + chunk * 16) | beyond);
      load16_async(vreg[it], rv, (j * sv + chunk * 16) | beyond);
    }
  };
  // `pending`: loads issued after the set being stored (0 or 2 * PER)
  auto stage_store = [&](int buf, u32x4* kreg, u32x4* vreg, auto pending) {
    unsigned char* Ks = Ks0 + buf * KBYTES;
    unsigned char* Vs = Vs0 + buf * VBYTES;
    wait_loads<decltype(pending)::value>();
#pragma unroll
    for (int it = 0; it < PER; ++it) asm volatile("" : "+v"(kreg[it]), "+v"(vreg[it]));
#pragma unroll
    for (int it = 0; it < PER; ++it) {
      const int idx = tid + it * kThreads;
      *(u32x4*)(Ks + (idx >> 4) * KSTRIDE + (idx & 15) * 16) = kreg[it];
      *(u32x4*)(Vs + (idx >> 4) * VSTRIDE + (idx & 15) * 16) = vreg[it];
    }
  };

  stage_load(0, kreg0, vreg0);
  __syncthreads();                     // every wave has its query fragments: the area is free for tile 0
  stage_store(0, kreg0, vreg0, std::integral_constant<int, 0>());
  stage_load(1, kreg1, vreg1);
  __syncthreads();

  // value fragments: lane (head-dim column ct*32 + l31) x 8 keys.  The key order inside a
  // contraction step follows the layout the probabilities already have in the score accumulator:
  // slot j of step u is key u*16 + (j/4)*8 + lh*4 + j%4 (see below), so nothing is shuffled.
  const int s16 = l & 15, g2 = (l >> 4) & 1;
  const int v_lane_off = (lh * 4 + (s16 >> 2)) * VSTRIDE + (16 * g2 + 4 * (s16 & 3)) * 2;

  auto iteration = [&](int t, u32x4* kld, u32x4* vld, u32x4* kst, u32x4* vst) {
    const int buf = t & 1;
    const bool blk = t >= NTc;
    const int row0 = (blk ? t - NTc : t) * BK;     // first key of the tile, within its array
    const unsigned char* Ks = Ks0 + buf * KBYTES;
    const unsigned char* Vs = Vs0 + buf * VBYTES;
    stage_load(t + 2, kld, vld);

    if (!blk || row0 < wq0 + WQ) {       // some key of the tile is visible to some query of this wave
      // ---- S^T tile: keys x queries
      f32x16 sacc[QB][BK / 32];
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt) {
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kv = *(const bf16x8*)(Ks + (kt * 32 + l31) * KSTRIDE + (ks * 16 + lh * 8) * 2);
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            sacc[qb][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qreg[qb][ks], ks == 0 ? zero : sacc[qb][kt], 0, 0, 0);
        }
      }
      // ---- mask: cache rows at and beyond m; block keys after the query
      if (blk ? row0 + BK - 1 > wq0 : row0 + BK > m) {
        const int lim0 = blk ? wq0 + l31 : m - 1;    // last visible row for qb = 0 (block: the query itself)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          const int lim = blk ? lim0 + 32 * qb : lim0;
#pragma unroll
          for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = row0 + kt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
              if (key > lim) sacc[qb][kt][i] = -INFINITY;
            }
        }
      }
      // ---- online softmax with a lazy reference (everything of one query sits in one lane pair)
      float psum[QB];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        float mx = sacc[qb][0][0];
#pragma unroll
        for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[qb][kt][i]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // The reference only moves when the row maximum outgrows it by kLazy (in exponent units),
        // so exp(..) stays below e^kLazy and the accumulator is rescaled rarely.
        const bool bump = mx > m_run[qb] + lazy_raw;
        const float m_new = bump ? mx : m_run[qb];
        if (__any(bump)) {
          const float alpha = bump ? __builtin_amdgcn_exp2f((m_run[qb] - m_new) * c) : 1.0f;
          l_run[qb] *= alpha;
#pragma unroll
          for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[qb][ct][i] *= alpha;
        }
        m_run[qb] = m_new;
        const float mc = m_new * c;
#pragma unroll
        for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[qb][kt][i] = __builtin_amdgcn_exp2f(fmaf(sacc[qb][kt][i], c, -mc));
        psum[qb] = 0.f;
      }
      // ---- O^T += V^T P^T; contraction slot j of step u holds key (u*16 + (j/4)*8 + lh*4 + j%4)
#pragma unroll
      for (int kt = 0; kt < BK / 32; ++kt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          bf16x8 pv[QB];
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            u32x4 pp;
#pragma unroll
            for (int j2 = 0; j2 < 4; ++j2) {
              pp[j2] = pack_bf16(sacc[qb][kt][u * 8 + 2 * j2], sacc[qb][kt][u * 8 + 2 * j2 + 1]);
              psum[qb] += sacc[qb][kt][u * 8 + 2 * j2] + sacc[qb][kt][u * 8 + 2 * j2 + 1];
            }
            pv[qb] = __builtin_bit_cast(bf16x8, pp);
          }
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) {
            const unsigned char* vp = Vs + (kt * 32 + u * 16) * VSTRIDE + (ct * 32) * 2 + v_lane_off;
            const s16x4 y0 = lds_read_tr(vp);
            const s16x4 y1 = lds_read_tr(vp + 8 * VSTRIDE);
            const s16x8 yy = {y0[0], y0[1], y0[2], y0[3], y1[0], y1[1], y1[2], y1[3]};
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              oacc[qb][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, yy), pv[qb],
                                                                     oacc[qb][ct], 0, 0, 0);
          }
        }
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) l_run[qb] += psum[qb] + __shfl_xor(psum[qb], 32, 64);
    }
    stage_store(buf ^ 1, kst, vst, std::integral_constant<int, 2 * PER>());
    __syncthreads();
  };
  for (int t = 0; t < NT; t += 2) {
    iteration(t, kreg0, vreg0, kreg1, vreg1);
    if (t + 1 < NT) iteration(t + 1, kreg1, vreg1, kreg0, vreg0);
  }

  // ---- O = O^T / l: lane holds its queries, head-dim columns ct*32 + (i/4)*8 + lh*4 + i%4.
  // The rows are put together in a wave-private piece of LDS (the loop's last barrier has been
  // passed, nobody reads tiles any more) and leave as whole rows, 1 KB contiguous per instruction.
  unsigned char* Os = smem + w * (WQ * KSTRIDE);
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float inv = 1.0f / l_run[qb];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[qb][ct][g * 4 + 0] * inv, oacc[qb][ct][g * 4 + 1] * inv);
        pk[1] = pack_bf16(oacc[qb][ct][g * 4 + 2] * inv, oacc[qb][ct][g * 4 + 3] * inv);
        *(u32x2*)(Os + (32 * qb + l31) * KSTRIDE + (ct * 32 + g * 8 + lh * 4) * 2) = pk;
      }
  }
#pragma unroll
  for (int i = 0; i < WQ / 4; ++i) {
    const int row = i * 4 + (l >> 4);
    const u32x4 v = *(const u32x4*)(Os + row * KSTRIDE + (l & 15) * 16);
    if (wq0 + row < Bn) *(u32x4*)(ob + (int64_t)(wq0 + row) * a.o.st + (l & 15) * 8) = v;
  }
}

template <int QB, int NW>
hipError_t launch_qb(const AttnArgs& a_in, hipStream_t s) {
  constexpr int kThreads = 64 * NW;
  AttnArgs a = a_in;
  constexpr int BQ = 32 * QB * NW;
  a.qtiles = (a.B + BQ - 1) / BQ;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)attn_mfma_k<QB, NW>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int64_t total = (int64_t)a.qtiles * a.Hq * a.batch * a.n_seg;
  if (total <= 0) return hipSuccess;
  if (total > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL((attn_mfma_k<QB, NW>), dim3((unsigned)total), dim3(kThreads), LDS_BYTES, s, a);
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supports(int dtype, int d, const char** why) {
  if (dtype != LOCOCO_BF16) { *why = "the MFMA kernels take bf16 storage only"; return false; }
  if (d != kD) { *why = "the MFMA kernels take head_dim = 128 only"; return false; }
  return true;
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
  // rows are addressed with 32-bit byte offsets inside resources of less than 2 GiB
  const int64_t lim = 0x7fff0000;
  for (const View* v : {&a.q, &a.k, &a.v})
    if (((int64_t)a.B * v->st + kD) * 2 >= lim) return hipErrorInvalidValue;
  if ((int64_t)a.M * kD * 2 >= lim) return hipErrorInvalidValue;
  return launch_qb<1, 4>(a, s);
}

}  // namespace lococo
