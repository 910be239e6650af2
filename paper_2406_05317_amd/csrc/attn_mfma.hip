// Block-vs-(cache+block) causal attention for gfx950 (Alg. 2 step 3, Eq. 1):
// bf16 MFMA, fp32 accumulation and softmax, K/V tiles in LDS, online softmax.
// One launch covers one block or, for a whole sequence whose intermediate
// caches were kept, every block at once.
//
// Each workgroup takes 128 query rows of one (batch, query head, block); each
// of its four waves owns 32 of them; two workgroups share a compute unit.  The
// kernel works on the TRANSPOSED score tile S^T = K Q^T (keys are MFMA rows,
// queries are MFMA columns), so that one lane holds scores of a single query:
// row maxima and sums need one cross-lane exchange, the rescale factor is a
// per-lane scalar, and the probabilities feed the second MFMA (O^T = V^T P^T)
// straight from registers.  The key order inside the second contraction is
// permuted the same way on both operands so no shuffle is needed; the value
// operand is read with the transposing LDS load straight from the row-major
// value tile.
//
// Keys are indexed over [cache ; block]: all m cache slots are visible, block
// key j' is visible to block query j iff j' <= j; a wave past its diagonal
// only helps to bring tiles in.  Shapes taken: head_dim = 128, bf16.
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
constexpr int KSTRIDE = kD * 2 + 16;          // bytes per row of the padded output staging rows
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;                 // the softmax reference lags the row maximum by at most this much

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // v_cvt_pk_bf16_f32, RNE
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// A value combined with the one the lane 32 away holds (the two halves of a wave share a query): v_permlane32_swap
// exchanges the upper half of one register with the lower half of another, so of the two results one is the lane's
// own value and the other its partner's, in either half; a vector instruction, no trip through the LDS crossbar
// and no wait on the LDS counter in the middle of the operand reads.  (a + b and b + a are the same bits.)
__device__ __forceinline__ float max_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
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

// The parts of a tile are interleaved inside each wave by hand, and the tiles are brought in by
// loads that write LDS directly:
//   phase A of iteration t:  S(t+1) = K(t+1) Q^T on the matrix pipe  ||  exponentials of S(t) on the VALU
//   phase B of iteration t:  O += V(t) P(t)     on the matrix pipe
// so the matrix pipe has work from this wave while it does its softmax, whatever phase the other
// wave of the SIMD is in.  The slices are pinned with sched_barrier.  Key tiles run one tile ahead
// of value tiles.  K(t+2) and V(t+1) are requested at the top of iteration t into the buffers the
// previous iteration has finished with, and must have landed at the barrier that ends it: a whole
// iteration of cover, no staging registers, no LDS store instructions.
//
// Tiles are unpadded (256 bytes per row) and XOR-swizzled in units of 16 bytes so that both kinds
// of operand read stay free of bank conflicts: chunk c of key row r sits in cell c ^ (r % 16), chunk
// c of value row r in cell c ^ (4 * (r % 4)).  A load instruction fills 64 consecutive cells (four
// rows); each lane fetches whatever chunk belongs in its cell.
#define LOCOCO_SB() __builtin_amdgcn_sched_barrier(0)
constexpr int TBYTES = BK * kD * 2;            // one unpadded tile
constexpr int LDS_BYTES = 4 * TBYTES;           // K(2) + V(2)

// 64 lanes x 16 bytes from a buffer resource straight into the 1 KB of LDS at lds_addr (lane l
// writes cell l).  Counted by vmcnt; the compiler does not know that LDS is written, so the wait
// and the barrier that publish the tile are written by hand.
__device__ __forceinline__ void load_to_lds(const u32x4& rsrc, uint32_t lds_addr, int voff) {
  // M0 (the LDS address) is an operand the compiler sets itself; the wait state the hardware wants
  // between a write of M0 and such a load is the s_nop
  asm volatile("s_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "{m0}"(lds_addr), "v"(voff), "s"(rsrc) : "memory");
}

__global__ __launch_bounds__(256, 2) void attn_mfma_k(AttnArgs a) {
  constexpr int BQ = 128;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Ks0 = smem;                   // key tiles t % 2
  unsigned char* Vs0 = smem + 2 * TBYTES;      // value tiles t % 2
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)smem);

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
    const int64_t slot = (int64_t)((a.hist_first + n - a.n_fill - 1) % a.hist_ring) * a.hist_stride +
                         (int64_t)chain * a.M * kD;
    cache_k = (const uint16_t*)a.hist_k + slot;
    cache_v = (const uint16_t*)a.hist_v + slot;
  }
  const Rows ck = make_rows(cache_k, m, kD), cv = make_rows(cache_v, m, kD);
  const Rows bk = make_rows((const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + start * a.k.st, Bn, a.k.st);
  const Rows bv = make_rows((const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + start * a.v.st, Bn, a.v.st);
  const uint16_t* qb_ptr = (const uint16_t*)a.q.p + b * a.q.sb + hq * a.q.sh + start * a.q.st;
  uint16_t* ob = (uint16_t*)a.o.p + b * a.o.sb + hq * a.o.sh + start * a.o.st;

  // (the wave index as a scalar: the tests on a wave's first query row are uniform branches)
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, l31 = l & 31, lh = l >> 5;
  const int wq0 = q0 + 32 * w;          // first query row of this wave
  const int qrow = wq0 + l31;           // this lane's query (block-relative)

  f32x16 oacc[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int i = 0; i < 16; ++i) oacc[ct][i] = 0.f;
  const float c = a.scale * kLog2e;
  const float lazy_raw = kLazy / a.scale;
  float m_run = -INFINITY, l_run = 0.f;

  const int NTc = (m + BK - 1) / BK;
  const int NT = NTc + (min(Bn, q0 + BQ) + BK - 1) / BK;

  // ---- tile requests.  Instruction `it` of wave w fills the cells of tile rows 16w + 4it .. + 3;
  // lane l: row 16w + 4it + l/16, cell l%16.  Past the last tile the offset is out of range: zeros.
  const int w_uniform = w;
  const uint32_t req_row = (uint32_t)(16 * w + (l >> 4));
  const uint32_t req_cell_k = (uint32_t)(((l & 15) ^ (l >> 4)) << 4);          // it = 0; instruction it flips bits 6, 7
  const uint32_t req_cell_v = (uint32_t)(((l & 15) ^ (((l >> 4) & 3) << 2)) << 4);
  auto request_one = [&](int t, int it, const Rows& fc, const Rows& fb, uint32_t lds_tile, bool keys) {
    const bool blk = t >= NTc;
    const int row0 = (blk ? t - NTc : t) * BK;
    u32x4 r = blk ? fb.rsrc : fc.rsrc;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_readfirstlane(r[i]);   // the instruction takes scalars only
    const int st = blk ? fb.stride : fc.stride;
    // byte offset = (row0 + 16 w + 4 it + l/16) * st + 16 * chunk, split into a part per lane (a 24-bit
    // multiply-add on two values computed once) and a scalar part; rows of the tile: 16 w + 4 it + l/16
    const uint32_t chunk16 = keys ? req_cell_k ^ (uint32_t)(it << 6) : req_cell_v;   // cell ^ (row % 16), cell ^ 4 (row % 4)
    const uint32_t lane_part = __umul24(req_row, (uint32_t)st) + chunk16;
    const uint32_t tile_part = t >= NT ? 0x7fff0000u : (uint32_t)((row0 + 4 * it) * st);
    load_to_lds(r, lds_tile + (uint32_t)((16 * w_uniform + 4 * it) * (kD * 2)), (int)(lane_part + tile_part));
  };
  auto request = [&](int t, const Rows& fc, const Rows& fb, uint32_t lds_tile, bool keys) {
#pragma unroll
    for (int it = 0; it < 4; ++it) request_one(t, it, fc, fb, lds_tile, keys);
  };
  auto tiles_landed = [&]() {            // this wave's requests are in LDS; then everybody's
    wait_loads<0>();
    __syncthreads();
  };

  // ---- operand addresses inside a swizzled tile
  // keys: lane (row l31 of a 32-row half, chunks 2 ks + lh): cell (2 ks + lh) ^ (l31 % 16)
  int kaddr[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) kaddr[ks] = l31 * (kD * 2) + (((2 * ks + lh) ^ (l31 & 15)) << 4);
  // values (transposing read): lane s16 of a 16-lane group covers row (lh*4 + s16/4) of an 8-row
  // group and 8 bytes at column 32 ct + 16 g2 + 4 (s16 % 4): chunk 4 ct + 2 g2 + (s16 % 4) / 2
  const int s16 = l & 15, g2 = (l >> 4) & 1;
  int vaddr[4];
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    const int vrow = lh * 4 + (s16 >> 2), chunk = 4 * ct + 2 * g2 + ((s16 & 3) >> 1);
    vaddr[ct] = vrow * (kD * 2) + ((chunk ^ ((vrow & 3) << 2)) << 4) + (s16 & 1) * 8;
  }
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // ---- prologue.  K(0) and V(0) are requested first; the query rows come in behind them as whole
  // rows, are parked (swizzled like a key tile) in the two tile buffers nothing has been requested
  // into yet -- waves 0, 1 in key buffer 1, waves 2, 3 in value buffer 1 -- and read back as
  // operand fragments; then K(1) is requested and S(0) computed while it is on its way.
  request(0, ck, bk, lds0, true);
  request(0, cv, bv, lds0 + 2 * TBYTES, false);
  bf16x8 qreg[8];
  {
    const Rows qr = make_rows(qb_ptr, Bn, a.q.st);
    unsigned char* Qs = smem + (w < 2 ? TBYTES : 3 * TBYTES) + (w & 1) * (32 * kD * 2);
    u32x4 qrow_regs[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      load16_async(qrow_regs[i], qr.rsrc, (wq0 + i * 4 + (l >> 4)) * qr.stride + (l & 15) * 16);
    wait_loads<0>();                   // loads complete in order: K(0) and V(0) of this wave are in LDS too
#pragma unroll
    for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(qrow_regs[i]));
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = i * 4 + (l >> 4);
      *(u32x4*)(Qs + row * (kD * 2) + (((l & 15) ^ (row & 15)) << 4)) = qrow_regs[i];
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qreg[ks] = *(const bf16x8*)(Qs + kaddr[ks]);
  }
  __syncthreads();                     // every wave has its query fragments, and K(0), V(0) are complete
  request(1, ck, bk, lds0 + TBYTES, true);
  f32x16 s_a[2], s_b[2];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 kv = *(const bf16x8*)(Ks0 + kt * 32 * (kD * 2) + kaddr[ks]);
      s_a[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qreg[ks], ks == 0 ? zero : s_a[kt], 0, 0, 0);
    }
  // Mask a score tile (cache rows at and beyond m; block keys after the query) and take this
  // lane pair's maximum.  Done for tile t + 1 under the P V MFMAs of iteration t.
  auto mask_tile = [&](int t, f32x16* sx) {
    const bool blk = t >= NTc;
    const int row0 = (blk ? t - NTc : t) * BK;
    if (blk ? row0 + BK - 1 > wq0 : row0 + BK > m) {
      const int lim = blk ? qrow : m - 1;
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int key = row0 + kt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3);
          if (key > lim) sx[kt][i] = -INFINITY;
        }
    }
  };
  float mx_tile;                         // row maximum of the tile the next iteration consumes
  {
    mask_tile(0, s_a);
    float mx = s_a[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s_a[kt][i]);
    mx_tile = max_with_other_half(mx);
  }
  tiles_landed();                      // K(1) is in; key buffer 0 is refilled in the first iteration

  // sc: scores of tile t (input), sn: scores of tile t + 1 (output); PAR = t % 2
  auto iteration = [&](int t, auto par, f32x16* sc, f32x16* sn) {
    constexpr int PAR = decltype(par)::value;
    const bool blk = t >= NTc;
    const int row0 = (blk ? t - NTc : t) * BK;
    const unsigned char* Kn = Ks0 + (PAR ^ 1) * TBYTES;     // K(t+1)
    const unsigned char* Vs = Vs0 + PAR * TBYTES;           // V(t)
    const uint32_t k_dst = lds0 + PAR * TBYTES;                       // K(t+2) goes where K(t) was
    const uint32_t v_dst = lds0 + 2 * TBYTES + (PAR ^ 1) * TBYTES;    // V(t+1) goes where V(t-1) was

    if (!blk || row0 < wq0 + 32) {       // some key of the tile is visible to some query of this wave
      // ---- the lazy reference (the tile was masked and its maximum taken an iteration ago)
      const float mx = mx_tile;
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

      // ---- phase A: 16 MFMAs of S(t+1), two exponentials of S(t) behind each
      LOCOCO_SB();
      bf16x8 kf[4];
#pragma unroll
      for (int pf = 0; pf < 3; ++pf) kf[pf] = *(const bf16x8*)(Kn + (pf >> 3) * 32 * (kD * 2) + kaddr[pf & 7]);
      float psum = 0.f;
#pragma unroll
      for (int sl = 0; sl < 16; ++sl) {
        const int kt = sl >> 3, ks = sl & 7;
        if (sl + 3 < 16)
          kf[(sl + 3) & 3] = *(const bf16x8*)(Kn + ((sl + 3) >> 3) * 32 * (kD * 2) + kaddr[(sl + 3) & 7]);
        sn[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[sl & 3], qreg[ks], ks == 0 ? zero : sn[kt], 0, 0, 0);
        if (sl < 4) request_one(t + 2, sl, ck, bk, k_dst, true);          // the tile requests ride in the first slices
        else if (sl < 8) request_one(t + 1, sl - 4, cv, bv, v_dst, false);
#pragma unroll
        for (int e = sl * 2; e < sl * 2 + 2; ++e) {
          float pval = __builtin_amdgcn_exp2f(fmaf(sc[e >> 4][e & 15], c, -mc));
          asm volatile("" : "+v"(pval));   // a use here: otherwise the exponentials sink to where P is consumed
          sc[e >> 4][e & 15] = pval;
          psum += pval;
        }
        LOCOCO_SB();
      }

      // ---- phase B: 16 MFMAs of O^T += V(t)^T P^T; tile t + 1 is masked and its maximum taken behind them
      mask_tile(t + 1, sn);
      float mxn = sn[0][0];
      s16x4 vf[4][2];
#pragma unroll
      for (int pf = 0; pf < 3; ++pf) {
        const unsigned char* vp = Vs + ((pf >> 2) * 16) * (kD * 2) + vaddr[pf & 3];
        vf[pf][0] = lds_read_tr(vp);
        vf[pf][1] = lds_read_tr(vp + 8 * (kD * 2));
      }
      bf16x8 pv;
#pragma unroll
      for (int g = 0; g < 16; ++g) {
        const int ku = g >> 2, ct = g & 3;      // ku = kt*2 + u: 16 keys per contraction step
        if (g + 3 < 16) {
          const unsigned char* vp = Vs + (((g + 3) >> 2) * 16) * (kD * 2) + vaddr[(g + 3) & 3];
          vf[(g + 3) & 3][0] = lds_read_tr(vp);
          vf[(g + 3) & 3][1] = lds_read_tr(vp + 8 * (kD * 2));
        }
        if (ct == 0) {
          const int kt = ku >> 1, u = ku & 1;
          u32x4 pp;
#pragma unroll
          for (int j2 = 0; j2 < 4; ++j2) pp[j2] = pack_bf16(sc[kt][u * 8 + 2 * j2], sc[kt][u * 8 + 2 * j2 + 1]);
          pv = __builtin_bit_cast(bf16x8, pp);
        }
        const s16x4 y0 = vf[g & 3][0], y1 = vf[g & 3][1];
        const s16x8 yy = {y0[0], y0[1], y0[2], y0[3], y1[0], y1[1], y1[2], y1[3]};
        oacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, yy), pv, oacc[ct], 0, 0, 0);
        if (g >= 4 && g < 12) {
#pragma unroll
          for (int e = (g - 4) * 4; e < (g - 4) * 4 + 4; ++e) mxn = fmaxf(mxn, sn[e >> 4][e & 15]);
        }
        if (g == 13) mx_tile = max_with_other_half(mxn);
        LOCOCO_SB();
      }
      l_run += sum_with_other_half(psum);
    } else {
      request(t + 2, ck, bk, k_dst, true);
      request(t + 1, cv, bv, v_dst, false);
    }
    tiles_landed();
  };
  for (int t = 0; t < NT; t += 2) {
    iteration(t, std::integral_constant<int, 0>(), s_a, s_b);
    if (t + 1 < NT) iteration(t + 1, std::integral_constant<int, 1>(), s_b, s_a);
  }

  // ---- O = O^T / l: lane holds its query, head-dim columns ct*32 + (i/4)*8 + lh*4 + i%4.  The rows
  // are put together in a wave-private piece of LDS (the loop's last barrier has been passed, every
  // request has landed) and leave as whole rows, 1 KB contiguous per wave instruction.
  static_assert(4 * 32 * KSTRIDE <= LDS_BYTES, "the output staging rows fit the tile area");
  unsigned char* Os = smem + w * (32 * KSTRIDE);
  {
    const float inv = 1.0f / l_run;
    if (a.stats && lh == 0 && qrow < Bn) {     // for the column sums (see attn_colsum_k)
      float* st = a.stats + (((int64_t)b * a.Hq + hq) * a.L + start + qrow) * 2;
      st[0] = m_run * c;
      st[1] = inv;
    }
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[ct][g * 4 + 0] * inv, oacc[ct][g * 4 + 1] * inv);
        pk[1] = pack_bf16(oacc[ct][g * 4 + 2] * inv, oacc[ct][g * 4 + 3] * inv);
        *(u32x2*)(Os + l31 * KSTRIDE + (ct * 32 + g * 8 + lh * 4) * 2) = pk;
      }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int row = i * 4 + (l >> 4);
    const u32x4 v = *(const u32x4*)(Os + row * KSTRIDE + (l & 15) * 16);
    if (wq0 + row < Bn) *(u32x4*)(ob + (int64_t)(wq0 + row) * a.o.st + (l & 15) * 8) = v;
  }
}

// ---- accumulated attention per cache slot.  One workgroup per (block, chain, 64 cache slots): the
// slots' keys stay in registers as MFMA operands, the waves share out the block's query rows (all
// heads of the group) in chunks of 32, recompute S^T = K Q^T, turn it into probabilities with the
// row statistics the attention kernel left, and sum over the queries.  Cache slots precede every
// token of the block, so there is no mask.
__global__ __launch_bounds__(256) void attn_colsum_k(AttnArgs a, float* colsum) {
  __shared__ float sums[64];
  const int j0 = blockIdx.x * 64;
  const int chain = blockIdx.y, b = chain / a.Hkv, hkv = chain % a.Hkv;
  const int n = a.seg_first + blockIdx.z;
  const int64_t start = (int64_t)n * a.B;
  const int Bn = (int)(a.L - start < a.B ? a.L - start : a.B);
  const int m = n <= a.n_fill ? a.len0 + n * a.B : a.M;
  if (j0 >= m) return;
  const uint16_t* cache_k =
      n <= a.n_fill ? (const uint16_t*)a.cache_k + (int64_t)chain * a.M * kD
                    : (const uint16_t*)a.hist_k + (int64_t)((a.hist_first + n - a.n_fill - 1) % a.hist_ring) * a.hist_stride +
                          (int64_t)chain * a.M * kD;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, l31 = l & 31, lh = l >> 5;
  if (tid < 64) sums[tid] = 0.f;
  __syncthreads();

  // keys j0 + 32 kt + l31, channels 16 ks + 8 lh ..: rows of S^T
  bf16x8 kf[2][8];
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const int j = j0 + kt * 32 + l31;
      const u32x4 z = {0u, 0u, 0u, 0u};
      const u32x4 v = j < m ? *(const u32x4*)(cache_k + (int64_t)j * kD + ks * 16 + lh * 8) : z;
      kf[kt][ks] = __builtin_bit_cast(bf16x8, v);
    }
  const float c = a.scale * kLog2e;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 part[2] = {zero, zero};          // per lane: sums over its queries, keys as in the accumulator rows
  const int R = a.group * Bn;             // query rows of the group, head-major
  // The query fragments go from memory straight into MFMA operands; the next chunk's are fetched
  // while the current chunk is multiplied and exponentiated.
  u32x4 qv[8], qn[8];
  float mc = 0.f, inv = 0.f, mcn = 0.f, invn = 0.f;
  auto fetch = [&](int r0, u32x4 (&dst)[8], float& m_out, float& i_out) {
    const int rr = r0 + l31;
    const bool live = rr < R;
    const int gi = live ? rr / Bn : 0, r = live ? rr % Bn : 0, hq = hkv * a.group + gi;
    const uint16_t* qrow = (const uint16_t*)a.q.p + b * a.q.sb + hq * a.q.sh + (start + r) * a.q.st;
    const float* st = a.stats + (((int64_t)b * a.Hq + hq) * a.L + start + r) * 2;
    const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) dst[ks] = live ? *(const u32x4*)(qrow + ks * 16 + lh * 8) : z;
    m_out = live ? st[0] : 0.f;
    i_out = live ? st[1] : 0.f;             // a row past the end adds nothing
  };
  if (w * 32 < R) fetch(w * 32, qv, mc, inv);
  for (int r0 = w * 32; r0 < R; r0 += 4 * 32) {
    if (r0 + 4 * 32 < R) fetch(r0 + 4 * 32, qn, mcn, invn);
    f32x16 sacc[2];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      const bf16x8 qf = __builtin_bit_cast(bf16x8, qv[ks]);
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
        sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[kt][ks], qf, ks == 0 ? zero : sacc[kt], 0, 0, 0);
    }
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int i = 0; i < 16; ++i) part[kt][i] += __builtin_amdgcn_exp2f(fmaf(sacc[kt][i], c, -mc)) * inv;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qv[ks] = qn[ks];
    mc = mcn;
    inv = invn;
  }
  // sum over the 32 queries held by the lanes of a half wave, then over the waves
#pragma unroll
  for (int kt = 0; kt < 2; ++kt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float v = part[kt][i];
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
      if (l31 == 0) atomicAdd(&sums[kt * 32 + (i >> 2) * 8 + lh * 4 + (i & 3)], v);
    }
  __syncthreads();
  if (tid < 64 && j0 + tid < m) atomicAdd(colsum + (int64_t)chain * a.M + j0 + tid, sums[tid]);
}

hipError_t launch_tiles(const AttnArgs& a_in, hipStream_t s) {
  AttnArgs a = a_in;
  a.qtiles = (a.B + 127) / 128;
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
  hipLaunchKernelGGL(attn_mfma_k, dim3((unsigned)total), dim3(256), LDS_BYTES, s, a);
  return hipGetLastError();
}

}  // namespace

bool attn_mfma_supports(int dtype, int d, const char** why) {
  if (dtype != LOCOCO_BF16) { *why = "the MFMA kernels take bf16 storage only"; return false; }
  if (d != kD) { *why = "the MFMA kernels take head_dim = 128 only"; return false; }
  return true;
}

hipError_t launch_attn_colsum_mfma(const AttnArgs& a, float* colsum, hipStream_t s) {
  if (!a.stats || !colsum) return hipErrorInvalidValue;
  if (a.n_seg <= 0) return hipSuccess;
  hipLaunchKernelGGL(attn_colsum_k, dim3((a.M + 63) / 64, a.batch * a.Hkv, a.n_seg), dim3(256), 0, s, a, colsum);
  return hipGetLastError();
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
  // rows are addressed with 32-bit byte offsets inside resources of less than 2 GiB
  const int64_t lim = 0x7fff0000;
  for (const View* v : {&a.q, &a.k, &a.v})
    if (((int64_t)a.B * v->st + kD) * 2 >= lim) return hipErrorInvalidValue;
  if ((int64_t)a.M * kD * 2 >= lim) return hipErrorInvalidValue;
  return launch_tiles(a, s);
}

}  // namespace lococo
