// Attention of Alg. 2 step 3 for the generation stage (one new token per
// sequence, B = 1): softmax(q [K_cache ; k_new]^T / sqrt(d)) [V_cache ; v_new]
// for one query row per head.  bf16 storage, fp32 arithmetic, head_dim 128.
//
// One query row against m + 1 keys is a matrix-vector product, not a matrix
// product: 4(m+1)d flops per head against 4(m+1)d bytes of keys and values, so
// the roofline that bounds it is HBM (or, with 32 heads, the launch itself).
// The MFMA attention kernel would spend a 128-query tile on this one row.
//
// One workgroup of 16 waves per (batch, query head).  A key row is 256 bytes =
// 16 lanes x 16 bytes, so one wave-wide load brings 4 consecutive keys; the
// waves take groups of 4 keys round-robin.  Each 16-lane group keeps its own
// online softmax state (reference, row sum, 8 output columns per lane); the 64
// states of a workgroup are merged through LDS at the end.
//
// With accumulated attention scores asked for (StepArgs::colsum), the raw
// scores of the cache slots are also kept in LDS, and once the row's reference
// and sum are known every slot's probability is added to its accumulator.
#include "lococo_internal.h"

namespace lococo {
namespace {

constexpr int kD = 128;
constexpr int kThreads = 1024;           // 16 waves: enough loads in flight to hide HBM latency on few workgroups
constexpr int kWaves = kThreads / 64, kParts = kWaves * 4;
constexpr float kLog2e = 1.4426950408889634f;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
// sum over the 16 lanes of a row, result in every lane: quad xor 1, quad xor 2, mirror inside
// 8 lanes, mirror inside 16 lanes
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp<0xB1>(v);
  v += dpp<0x4E>(v);
  v += dpp<0x141>(v);
  v += dpp<0x140>(v);
  return v;
}
__device__ __forceinline__ void unpack8(const u32x4& r, float* f) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(r[i] << 16);
    f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
  }
}

template <bool COLSUM>
__global__ __launch_bounds__(kThreads) void attn_decode_k(StepArgs a) {
  extern __shared__ float sc[];            // COLSUM: a.m raw scores (log2 units)
  __shared__ float part_o[kParts][kD + 4];
  __shared__ float part_m[kParts], part_l[kParts];
  __shared__ float fin[2];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, grp = l >> 4, c16 = l & 15;
  const int hq = blockIdx.x % a.Hq, b = blockIdx.x / a.Hq, hkv = hq / a.group;
  const int ch = b * a.Hkv + hkv;
  const int T = a.m + 1;

  float q[8];
  unpack8(*(const u32x4*)((const uint16_t*)a.q.p + b * a.q.sb + hq * a.q.sh + c16 * 8), q);
  const float c = a.scale * kLog2e;               // exp(x * scale) = exp2(x * c)
#pragma unroll
  for (int i = 0; i < 8; ++i) q[i] *= c;

  const uint16_t* ck = (const uint16_t*)a.cache_k + (int64_t)ch * a.M * kD + c16 * 8;
  const uint16_t* cv = (const uint16_t*)a.cache_v + (int64_t)ch * a.M * kD + c16 * 8;
  const uint16_t* nk = (const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + c16 * 8;
  const uint16_t* nv = (const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + c16 * 8;

  float m_run = -INFINITY, l_run = 0.f, o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // keys j = 8*kWaves*it + 4*w + grp (+ 4*kWaves); two groups of loads in flight per iteration
  for (int j0 = 4 * w + grp; j0 < T; j0 += 8 * kWaves) {
    const int j1 = j0 + 4 * kWaves;
    const bool has1 = j1 < T;
    const u32x4 k0 = *(const u32x4*)(j0 < a.m ? ck + (int64_t)j0 * kD : nk);
    const u32x4 v0 = *(const u32x4*)(j0 < a.m ? cv + (int64_t)j0 * kD : nv);
    u32x4 k1 = {0, 0, 0, 0}, v1 = {0, 0, 0, 0};
    if (has1) {
      k1 = *(const u32x4*)(j1 < a.m ? ck + (int64_t)j1 * kD : nk);
      v1 = *(const u32x4*)(j1 < a.m ? cv + (int64_t)j1 * kD : nv);
    }
    float kf[8], s0 = 0.f, s1 = 0.f;
    unpack8(k0, kf);
#pragma unroll
    for (int i = 0; i < 8; ++i) s0 = fmaf(q[i], kf[i], s0);
    unpack8(k1, kf);
#pragma unroll
    for (int i = 0; i < 8; ++i) s1 = fmaf(q[i], kf[i], s1);
    s0 = row16_sum(s0);                            // scores in log2 units
    s1 = has1 ? row16_sum(s1) : -INFINITY;
    if (COLSUM && c16 == 0) {
      if (j0 < a.m) sc[j0] = s0;
      if (j1 < a.m) sc[j1] = s1;
    }
    const float m_new = fmaxf(m_run, fmaxf(s0, s1));
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    const float p0 = __builtin_amdgcn_exp2f(s0 - m_new), p1 = __builtin_amdgcn_exp2f(s1 - m_new);
    l_run = l_run * alpha + p0 + p1;
    m_run = m_new;
    float vf[8];
    unpack8(v0, vf);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = fmaf(p0, vf[i], o[i] * alpha);
    unpack8(v1, vf);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = fmaf(p1, vf[i], o[i]);
  }

  // merge the partial states (one per wave and lane group); a group that saw no key has
  // m = -inf, l = 0 and weighs nothing
  const int pi = w * 4 + grp;
#pragma unroll
  for (int i = 0; i < 8; ++i) part_o[pi][c16 * 8 + i] = o[i];
  if (c16 == 0) {
    part_m[pi] = m_run;
    part_l[pi] = l_run;
  }
  __syncthreads();
  if (tid < kD) {
    float mx = part_m[0];
#pragma unroll
    for (int p = 1; p < kParts; ++p) mx = fmaxf(mx, part_m[p]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int p = 0; p < kParts; ++p) {
      const float wgt = __builtin_amdgcn_exp2f(part_m[p] - mx);   // exp2(-inf) = 0 for empty groups
      num = fmaf(wgt, part_o[p][tid], num);
      den = fmaf(wgt, part_l[p], den);
    }
    if (COLSUM && tid == 0) {
      fin[0] = mx;
      fin[1] = den;
    }
    const float r = num / den;
    // round to nearest even bf16
    uint32_t u = __float_as_uint(r);
    u += 0x7fffu + ((u >> 16) & 1u);
    ((uint16_t*)a.o.p)[b * a.o.sb + hq * a.o.sh + tid] = (uint16_t)(u >> 16);
  }
  if (COLSUM) {
    __syncthreads();
    const float mx = fin[0], inv = 1.f / fin[1];
    float* cs = a.colsum + (int64_t)ch * a.M;
    for (int j = tid; j < a.m; j += kThreads) atomicAdd(cs + j, __builtin_amdgcn_exp2f(sc[j] - mx) * inv);
  }
}

// LDS the kernel holds besides the scores: the partial states.
constexpr size_t kStaticLds = sizeof(float) * (kParts * (kD + 4) + 2 * kParts + 2);

}  // namespace

bool attn_decode_supports(int dtype, int d, int Bn, int M, bool colsum) {
  if (colsum && kStaticLds + sizeof(float) * (size_t)M > 64 * 1024) return false;   // scores must fit LDS
  return dtype == LOCOCO_BF16 && d == kD && Bn == 1;
}

hipError_t launch_attn_decode(const StepArgs& a, hipStream_t s) {
  if (a.colsum)
    hipLaunchKernelGGL(attn_decode_k<true>, dim3(a.batch * a.Hq), dim3(kThreads), sizeof(float) * (size_t)a.M, s, a);
  else
    hipLaunchKernelGGL(attn_decode_k<false>, dim3(a.batch * a.Hq), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace lococo
