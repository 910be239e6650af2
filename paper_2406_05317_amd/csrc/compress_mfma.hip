// Fused compression kernel for gfx950: Eq. 5 (convolution logits), Eq. 6
// (softmax over positions) and Eq. 4a/4b (fusion of K and V with shared
// weights) in one pass, bf16 MFMA with fp32 accumulation.  The logits and the
// normalised weights never leave the compute unit.
//
// Structure.  The step is "attention with a convolution for scores": for a
// tile of BM cache slots the kernel walks the T = m + B positions of
// [cache ; block] in tiles of 32, computes the logits as an implicit GEMM
// with inner dimension C*k (each filter tap is a row-shifted view of the key
// tile held in LDS), keeps a running reference / row sum per slot (online
// softmax), and accumulates [K | V]^T P^T into a 2d x BM fp32 accumulator.
//
// Register-stationary filters.  The filter bank is the same for every
// position, chain and step, and a compute unit's register file (512 KB) is
// larger than its slice of the bank, so each workgroup loads its BM x (C*k)
// filter slice into registers once and streams only keys/values through LDS.
// The four waves split the inner dimension by channel quarter (wave w owns
// channels [32w, 32w+32) of every tap); their partial logits are summed
// through LDS before the softmax.  For the mixing GEMM wave w owns output
// columns [64w, 64w+64) of [K | V].
//
// Transposed tiles.  Both GEMMs are computed transposed (positions x slots,
// then columns x slots) so that an MFMA lane always belongs to one slot: the
// partial logits leave the registers as 16-byte stores, the rescale factor is
// a per-lane scalar and the new cache rows are stored 8 bytes at a time.
//
// Software pipeline.  One wave per SIMD leaves nothing to switch to while a
// wave waits, so the loop is pipelined by hand, three tiles deep: while the
// MFMAs of tile i+1's logits issue, the wave works through tile i's reduction
// and softmax, tile i-1's mixing MFMAs and the staging of later tiles, all cut
// into small slices pinned between the logit MFMAs (loads are issued a few
// steps before they are consumed).  The two workgroup barriers of a tile sit
// inside that MFMA stream as well, so no barrier is waited for with the matrix
// pipe idle.
//
// Filters over [K | V] (C = 2d, the compressor as Eq. 5 prints it).  A slot tile's slice of such a
// bank is twice what the registers hold, and the logit is a sum of a convolution over the keys
// and one over the values, so the walk is done twice: with the key half of the filters resident
// the kernel leaves the summed key-side logits of every position tile in the workspace (4 KB per
// tile, each lane writing the four values it will read back itself); then the value half takes the
// registers' place and the ordinary pipeline runs with the value rows as the convolution's input,
// the stored key-side logits added where the four waves' partial sums meet.  In that second walk
// the two row tiles swap roles (values with halo, keys without), so the accumulator's first d
// columns are the new value rows and the pointers are swapped where the rows are written.
//
// Shapes taken: head_dim = 128, bf16, width 15 (64- or 32-slot tiles) or 21 (32-slot tiles) over the
// keys, or either width over [K | V] (32-slot tiles), either normalisation, M a multiple of BM;
// any T (tail positions are masked), any m.
#include <type_traits>

#include "lococo_internal.h"

namespace lococo {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

constexpr int kD = 128;            // head_dim = conv channels
constexpr int kThreads = 256;
constexpr int BN = 32;             // positions per tile
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazy = 8.0f;      // the softmax reference lags the row maximum by at most this much

template <int BM, int KW>
struct Geo {
  static constexpr int RT = BM / 32;                 // 32-slot MFMA tiles per workgroup
  static constexpr int NS = KW * 2;                  // contraction steps of a logit tile: (tap, channel half)
  static constexpr int PAD = (KW - 1) / 2;
  static constexpr int XROWS = BN + KW - 1;          // key tile rows incl. halo
  static constexpr int XSTRIDE = kD * 2 + 16;        // bytes per key-tile row (conflict-free 16-byte reads)
  static constexpr int VSTRIDE = kD * 2 + 64;        // bytes per value-tile row (conflict-free transposing reads)
  static constexpr int SSTRIDE = BN + 4;             // floats per slot row of a partial-logit buffer
  static constexpr int PSTRIDE = BN * 2 + 16;        // bytes per slot row of the bf16 probability tile
  static constexpr int XITEMS = XROWS * 16;          // 16-byte chunks of the key tile
  static constexpr int XPER = (XITEMS + kThreads - 1) / kThreads;
  static constexpr int XALLOC = XPER * kThreads / 16;  // rows allocated: every thread stores XPER chunks
  static constexpr int XBYTES = XALLOC * XSTRIDE;
  static constexpr int VPER = BN * 16 / kThreads;    // 16-byte chunks of the value tile per thread
  static constexpr int VBYTES = BN * VSTRIDE;
  static constexpr int SBYTES = 4 * BM * SSTRIDE * 4;
  static constexpr int PBYTES = BM * PSTRIDE;
  static constexpr int NXBUF = 5, NVBUF = 2;           // key tiles i-1 .. i+3, value tiles i-1, i
  static constexpr int LDS = NXBUF * XBYTES + NVBUF * VBYTES + SBYTES + 2 * PBYTES + 3 * BM * 4;
  static constexpr int RPW = BM / 4;                 // slots a wave owns in the softmax phase
  static constexpr int LPR = 64 / RPW;               // lanes per slot there
  static constexpr int EPL = BN / LPR;               // positions per lane there
  static_assert(BM == 32 || BM == 64, "BM");
  static constexpr int PART_FLOATS = BM * 2 * kD + 2 * BM;   // a part's accumulators [slot][2 d], references, row sums
  static_assert(EPL % 4 == 0, "softmax lanes read whole float4s");
  static_assert(NS >= 26, "the slices of the pipelined loop are laid out over 26 contraction steps");
  static_assert(LDS <= 160 * 1024, "LDS budget");
};

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // v_cvt_pk_bf16_f32, RNE
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Cross-lane exchange inside groups of 4 / 8 lanes on the VALU (DPP), no LDS round trip.
template <int CTRL>
__device__ __forceinline__ float dpp(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7 - i within 8 lanes
template <int LPR>
__device__ __forceinline__ float group_max(float v) {
  v = fmaxf(v, dpp<kDppXor1>(v));
  v = fmaxf(v, dpp<kDppXor2>(v));
  if (LPR == 8) v = fmaxf(v, dpp<kDppHalfMirror>(v));
  return v;
}
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp<kDppXor1>(v);
  v += dpp<kDppXor2>(v);
  if (LPR == 8) v += dpp<kDppHalfMirror>(v);
  return v;
}

// Transposing LDS read (ds_read_b64_tr_b16).  Within each group of 16 lanes, lane s supplies the
// address of 4 consecutive 16-bit elements; lane i of the group receives element (i % 4) of the
// chunks addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12.  With lane s pointing at
// (row r0 + s/4, column c0 + 4*(s%4)) of a row-major tile, lane i ends up with column c0 + i of
// rows r0 .. r0+3: an operand fragment (column, 4 contraction rows) straight from a row-major tile.
__device__ __forceinline__ s16x4 lds_read_tr(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p);
}

// [cache ; block] rows are read through two raw buffer resources, one over the live cache rows and
// one over the block rows.  A row index outside a resource's range (negative offsets wrap to huge
// unsigned ones) reads as zero without touching memory, so OR-ing the two loads yields row p of the
// concatenation for 0 <= p < T and zeros elsewhere: no clamps, no selects, no masks.
struct CatRows {
  __amdgpu_buffer_rsrc_t cache, blk;
  int m;            // rows in the cache part
  int blk_stride;   // bytes between block rows
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
// The two halves are OR-ed only when the data is stored to LDS, many steps after the loads were issued.
struct Cat16 { u32x4 from_cache, from_blk; };
// Cache rows are read at device scope (sc1: served by the L2, never by this CU's L1): in the
// one-launch scan they were written by other workgroups a step ago, and every row is read once per
// workgroup anyway.
constexpr int kDeviceScope = 1 << 4;
__device__ __forceinline__ Cat16 load_cat16(const CatRows& c, int p, int chunk) {
  Cat16 r;
  r.from_cache = __builtin_amdgcn_raw_buffer_load_b128(c.cache, p * (kD * 2) + chunk * 16, 0, kDeviceScope);
  r.from_blk = __builtin_amdgcn_raw_buffer_load_b128(c.blk, (p - c.m) * c.blk_stride + chunk * 16, 0, 0);
  return r;
}

// wp: filters repacked in register order, [bank][M/32][wave][tap][half][lane] x 8 channels: lane l of
// wave w holds slot (32-slot tile)*32 + l%32, channels 32w + 16*half + 8*(l/32) .. +7, so that every
// load instruction of the prologue reads 1 KB of contiguous memory.
// NORM = 0: softmax over the positions; NORM = 1: relu(W) / (sum of relu(W) + eps) (Eq. 6 as printed,
// with the rectifier of the convolution head in front of it).
// PROT = 1: the cache carries protected slots (lococo_cache.protect); a build of its own so that the
// common case pays neither the registers nor the instructions.
// MULTI = 1: a workgroup may own several chains (see below); also a build of its own, because the
// register allocation of the one-chain build is tight and the 32 K-token workload runs on it.
// SPLIT = 1: the positions of a step are shared out between sa.psplit workgroups per (chain, slot
// tile) -- for shapes whose (chain, tile) pairs would leave compute units idle.  Each part walks its
// range of position tiles with the same pipeline and leaves its running reference, row sum and
// unnormalised accumulators in the workspace; the part that arrives last merges them in a fixed
// order (so the result does not depend on who is last) and writes the rows.
// SPLIT = 2: two workgroups per (chain, slot tile) take the steps of a scan in turn.  A step of such a
// build is walked in two legs that share the running softmax and the accumulators (the order of the
// positions does not matter to either): first the tiles that lie wholly in the block, halo included --
// they do not depend on the step before, so the workgroup whose turn is next works through them while
// its partner finishes that step -- then, after the chain has been met, the tiles that touch the cache.
// Only the second leg is on the chain's critical path.  (Single-step launches use the same build, one
// workgroup of each pair idle, so that results do not depend on the kind of launch.)
// CIN = 1: filters over [K | V] (two walks, see the head of the file); wp then holds the key half of
// every bank's slices followed by the value half, each in the order above.
template <int BM, int KW, int NORM, int PROT, int MULTI, int SPLIT, int CIN>
__global__ __launch_bounds__(kThreads, 1) void compress_mfma_k(ScanArgs sa, const uint16_t* wp,
                                                               int64_t wp_head_stride) {
  using G = Geo<BM, KW>;
  static_assert(!SPLIT || (BM == 32 && !MULTI), "the splits are built for 32-slot tiles, one chain per workgroup");
  constexpr bool PSPLIT = SPLIT == 1, PIPE = SPLIT == 2;
  static_assert(!CIN || BM == 32, "[K | V] filters are built for 32-slot tiles");
  const StepArgs& a = sa.st;
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* Xs0 = smem;                                    // NXBUF key tiles (with halo)
  unsigned char* Vs0 = Xs0 + G::NXBUF * G::XBYTES;              // NVBUF value tiles
  float* Sred = (float*)(Vs0 + G::NVBUF * G::VBYTES);           // 4 partial-logit tiles [wave][slot][pos]
  unsigned char* Ps0 = (unsigned char*)Sred + G::SBYTES;        // 2 probability tiles [slot][pos], bf16
  float* alphas0 = (float*)(Ps0 + 2 * G::PBYTES);               // 2 x rescale factor per slot
  float* lsum = alphas0 + 2 * BM;                               // final row sums

  // (the wave index as a scalar: everything derived from it stays on the scalar unit, and the
  // choices between the key and the value side of the mixing are uniform branches)
  const int tid = threadIdx.x, w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, l31 = l & 31, lh = l >> 5;
  // Workgroups are dealt to the 8 XCDs round-robin by their linear id.  The slot tiles of one chain
  // all read the same keys and values, so they are given ids that land on one XCD (one L2).
  int item = blockIdx.x;
  {
    const int per = gridDim.x / 8;
    if (item < per * 8) item = (item % 8) * per + item / 8;
  }
  const int tiles = a.M / BM;
  // position split: consecutive work items are the parts of one (chain, slot tile), so they land on one XCD
  const int P = SPLIT ? sa.psplit : 1;
  const int part = SPLIT ? item % P : 0;
  if (SPLIT) item /= P;
  // A workgroup owns one slot tile of the chains grp, grp + groups, grp + 2 groups, ...  (one chain
  // when the launch has a workgroup per chain and tile).  Where filters or biases differ between
  // kv heads the host picks `groups` as a multiple of Hkv, so all of them belong to head hkv0.
  const int grp = item / tiles, groups = gridDim.x / (tiles * P), n_chains = a.batch * a.Hkv;
  const int hkv0 = grp % a.Hkv;
  const int i0 = (item % tiles) * BM;
  // per-step and per-chain quantities, set at the top of the loops
  int T = 0, m = 0, NT = 0;
  int jbase = 0;            // first position of this workgroup's range (0 unless the positions are split)
  CatRows cat_k, cat_v;
  // protected-slot bits of the chain at hand (see lococo_cache.protect), or null
  const uint32_t* pwords = nullptr;

  // ---- this wave's slice of the filter bank, resident in registers for the whole kernel:
  // lane (slot l31 of tile rt, channels 32w + 16h + 8*lh ..) for every tap
  bf16x8 wreg[G::RT][KW][2];
  // (Requesting a [K | V] bank's next half as soon as the last logit MFMA of a pass has issued, so that it
  // arrives while the pass drains, was tried: the allocator has nowhere to keep 168 registers in flight and
  // spills them.)
  auto load_filters = [&](int half_of_bank) {          // 0: the bank (or its key half), 1: its value half
    const uint16_t* wb = wp + hkv0 * wp_head_stride + (CIN ? (int64_t)half_of_bank * a.M * (KW * kD) : 0);
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int t = 0; t < KW; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          wreg[rt][t][h] =
              *(const bf16x8*)(wb + ((((int64_t)(i0 / 32 + rt) * 4 + w) * KW + t) * 2 + h) * 512 + l * 8);
    // Pin the filters to the accumulation-register half of the register file: the MFMA reads
    // them from there directly, which leaves the other 256 registers to everything else.
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int t = 0; t < KW; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) asm volatile("" : "+a"(wreg[rt][t][h]));
  };
  if (!CIN) load_filters(0);
  // key-side logits of one tile as this lane left them in the first walk (CIN only)
  f32x4 pre = {0.f, 0.f, 0.f, 0.f};
  __amdgpu_buffer_rsrc_t pre_rows = __builtin_amdgcn_make_buffer_rsrc((void*)sa.prelogits, 0, 0, 0x00020000);

  // mixing accumulator, transposed: lane = slot rt*32 + l31, rows = columns 64w + ct*32 + (i/4)*8 + lh*4 + i%4
  f32x16 oacc[2][G::RT];

  // softmax state of the slot this lane helps with (replicated over the LPR lanes of the slot)
  const int srow = w * G::RPW + l / G::LPR;
  const int sp0 = (l % G::LPR) * G::EPL;
  float m_run = 0.f, l_run = 0.f;
  // (a softmax over the positions does not see a per-slot constant: the bias only enters the relu-sum form)
  const float bias =
      a.conv_b ? __uint_as_float((uint32_t)((const uint16_t*)a.conv_b)[hkv0 * a.b_head_stride + i0 + srow] << 16)
               : 0.f;

  // ---- staging: global -> registers -> LDS (key tile with halo, value tile; both row-major)
  Cat16 xreg[G::XPER];
  Cat16 vreg[G::VPER];
  auto load_x = [&](int it, int j0) {
    const int item = tid + it * kThreads;
    xreg[it] = load_cat16(cat_k, j0 - G::PAD + (item >> 4), item & 15);
  };
  auto load_v = [&](int it, int j0) {
    const int item = tid + it * kThreads;
    vreg[it] = load_cat16(cat_v, j0 + (item >> 4), item & 15);
  };
  // the two halves of a chunk's fetch on their own, for stages that give each a slot of its own
  auto load_half = [&](Cat16& r, const CatRows& c, int p, int chunk, bool blk) {
    if (blk) r.from_blk = __builtin_amdgcn_raw_buffer_load_b128(c.blk, (p - c.m) * c.blk_stride + chunk * 16, 0, 0);
    else r.from_cache = __builtin_amdgcn_raw_buffer_load_b128(c.cache, p * (kD * 2) + chunk * 16, 0, kDeviceScope);
  };
  auto store_x = [&](int it, int j0, unsigned char* Xs) {
    const int item = tid + it * kThreads;
    (void)j0;
    *(u32x4*)(Xs + (item >> 4) * G::XSTRIDE + (item & 15) * 16) = xreg[it].from_cache | xreg[it].from_blk;
  };
  auto store_v = [&](int it, int j0, unsigned char* Vs) {
    const int item = tid + it * kThreads;
    (void)j0;
    *(u32x4*)(Vs + (item >> 4) * G::VSTRIDE + (item & 15) * 16) = vreg[it].from_cache | vreg[it].from_blk;
  };

  // Ring of key operands of the logit MFMAs, fetched kRing-1 contraction steps ahead.  kRing
  // divides the number of steps, so the last steps of a stage fetch the first operands of the
  // next stage into the slots that stage expects and the matrix pipe never waits at a stage start.
  constexpr int kRing = G::NS % 5 == 0 ? 5 : (G::NS % 6 == 0 ? 6 : 7);
  static_assert(G::NS % kRing == 0, "operand ring must wrap exactly at a stage boundary");
  bf16x8 xv[kRing];

  // Partial logits of one tile, summed over this wave's channel quarter:
  // sacc[rt] lane = slot rt*32 + l31, rows = positions (i/4)*8 + lh*4 + i%4.
  f32x16 sacc[G::RT];
  // Publish them: 16-byte stores, 4 consecutive positions of one slot each.
  auto write_partials = [&]() {
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = {sacc[rt][g * 4 + 0], sacc[rt][g * 4 + 1], sacc[rt][g * 4 + 2], sacc[rt][g * 4 + 3]};
        *(f32x4*)(Sred + (w * BM + rt * 32 + l31) * G::SSTRIDE + g * 8 + lh * 4) = v;
      }
  };

  // One pipeline stage.  With tile index i it runs, interleaved:
  //   DoConv:    logits of tile i+1 (key tile buffer (i+1)%5) into sacc, published at the end;
  //   DoSoftmax: reduction + softmax of tile i (partials in Sred) into Ps[i&1], alphas[i&1];
  //              staging of key tile i+3 and value tile i (loaded during the previous stage);
  //   DoMix:     mixing of tile i-1 (Ps[(i-1)&1], key tile buffer (i-1)%5, value buffer (i-1)&1).
  //
  // Issue model.  A wave issues in order and the matrix pipe takes one MFMA every 32 cycles, so
  // after each MFMA there is room for about seven other instructions before the next MFMA can
  // issue anyway.  Everything that is not a logit MFMA is therefore cut into micro-slices of a few
  // instructions, one per MFMA ("slot" 2*st + rt), with every load issued several slots before
  // the slice that consumes it.
  //
  // Barriers.  B1 (slot 5) publishes what the previous stage wrote to LDS -- partial logits,
  // probabilities, rescale factors, staged tiles -- so everything read before it (the key tile of
  // this stage's logits) was staged two stages ago.  B2 (slot 19) comes after every wave has
  // consumed this tile's partial logits; the buffer is rewritten at the end of the stage.
  // Neither needs outstanding global loads to finish, so they are plain barriers preceded by a
  // wait on the LDS counter only.
  // PH: 0 = the one walk of a bank over the keys; 1 = first walk of a [K | V] bank (logits of the key
  // half only: DoSoftmax then means "sum the waves' partial logits and store them"); 2 = its second walk.
  // RI: the tile index modulo the period of the buffer rings (key tiles: NXBUF; values, probabilities,
  // rescale factors: 2) where the caller knows it at compile time, so that every buffer address of the
  // stage is a constant; -1: computed from i.
  auto stage = [&](int i, auto do_conv, auto do_softmax, auto do_mix_t, auto ph_t, auto ring_t) {
    constexpr bool DoConv = decltype(do_conv)::value, DoSoftmax = decltype(do_softmax)::value;
    constexpr bool DoMix = decltype(do_mix_t)::value;
    constexpr int PH = decltype(ph_t)::value;
    constexpr int RI = decltype(ring_t)::value;
    const int ib = RI >= 0 ? RI + 2 * G::NXBUF : i;      // (kept positive: ib - 1 enters a remainder)
    const int j0 = (SPLIT ? jbase : 0) + i * BN;
    const unsigned char* Xnext = Xs0 + ((ib + 1) % G::NXBUF) * G::XBYTES;
    const unsigned char* Xnext2 = Xs0 + ((ib + 2) % G::NXBUF) * G::XBYTES;
    const unsigned char* Xprev = Xs0 + ((ib + G::NXBUF - 1) % G::NXBUF) * G::XBYTES;
    unsigned char* Xstage = Xs0 + ((ib + 3) % G::NXBUF) * G::XBYTES;
    const unsigned char* Vprev = Vs0 + ((ib - 1) & 1) * G::VBYTES;
    unsigned char* Vstage = Vs0 + (ib & 1) * G::VBYTES;
    unsigned char* Pcur = Ps0 + (ib & 1) * G::PBYTES;
    const unsigned char* Pprev = Ps0 + ((ib - 1) & 1) * G::PBYTES;
    float* alpha_cur = alphas0 + (ib & 1) * BM;
    const float* alpha_prev = alphas0 + ((ib - 1) & 1) * BM;

    // logits: operands of step st come from this stage's key tile, those of steps >= NS are the
    // first operands of the next stage's tile
    const int xlane = l31 * G::XSTRIDE + (32 * w + lh * 8) * 2;
    auto fetch = [&](int st) {
      const unsigned char* xb = (st < G::NS ? Xnext : Xnext2) + xlane;
      const int s2 = st < G::NS ? st : st - G::NS;
      xv[st % kRing] = *(const bf16x8*)(xb + (s2 >> 1) * G::XSTRIDE + (s2 & 1) * 32);
    };
    // protected positions of tile i (bits of live protected slots; BN = 32 = one mask word)
    uint32_t pmask = 0;
    if (PROT && DoSoftmax && PH != 1 && j0 < m) {
      pmask = pwords[j0 >> 5];
      if (j0 + BN > m) pmask &= (1u << (m - j0)) - 1u;
    }
    // softmax of tile i
    constexpr int E4 = G::EPL / 4;
    f32x4 part[4][E4];
    float sv[G::EPL];
    float mx = 0.f, m_new = 0.f, mc = 0.f, alpha = 1.f, psum = 0.f;
    bool bump = false;
    uint32_t packed[G::EPL / 2];
    auto sm_issue = [&](int ww) {
#pragma unroll
      for (int e4 = 0; e4 < E4; ++e4)
        part[ww][e4] = *(const f32x4*)(Sred + (ww * BM + srow) * G::SSTRIDE + sp0 + e4 * 4);
    };
    auto sm_add = [&](int ww0, int e4) {      // 4 positions: + partials ww0 and ww0+1
#pragma unroll
      for (int e = 0; e < 4; ++e)
        sv[e4 * 4 + e] = ww0 == 0 ? (PH == 2 ? pre[e] : 0.f) + (NORM == 0 || PH == 1 ? part[0][e4][e] + part[1][e4][e]
                                                                                        : bias + part[0][e4][e] + part[1][e4][e])
                                  : sv[e4 * 4 + e] + part[ww0][e4][e] + part[ww0 + 1][e4][e];
    };
    auto sm_exp = [&](int e) {
      sv[e] = NORM == 0 ? __builtin_amdgcn_exp2f(fmaf(sv[e], kLog2e, -mc)) : fmaxf(sv[e], 0.f);
    };
    // mixing of tile i-1: operand fragments, fetched ahead of the MFMAs that follow the loop
    const int s16 = l & 15, g2 = (l >> 4) & 1;
    const unsigned char* ybase =
        (w < 2 ? Xprev + (G::PAD + lh * 8 + (s16 >> 2)) * G::XSTRIDE + (64 * w) * 2
               : Vprev + (lh * 8 + (s16 >> 2)) * G::VSTRIDE + (64 * (w - 2)) * 2) +
        (16 * g2 + 4 * (s16 & 3)) * 2;
    const int ystride = w < 2 ? G::XSTRIDE : G::VSTRIDE;
    bf16x8 pv[2][G::RT];
    s16x4 y0[2][2], y1[2][2];
    float al[G::RT];
    auto mix_fetch_p = [&](int ks) {
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt)
        pv[ks][rt] = *(const bf16x8*)(Pprev + (rt * 32 + l31) * G::PSTRIDE + (ks * 16 + lh * 8) * 2);
    };
    auto mix_fetch_y = [&](int ks, int ct) {
      const unsigned char* yp = ybase + (ks * 16) * ystride + (ct * 32) * 2;
      y0[ks][ct] = lds_read_tr(yp);
      y1[ks][ct] = lds_read_tr(yp + 4 * ystride);
    };
    auto mix_mfma = [&](int ks, int ct) {
      const s16x4 a0 = y0[ks][ct], a1 = y1[ks][ct];
      const s16x8 yy = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
      const bf16x8 yv = __builtin_bit_cast(bf16x8, yy);
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt)
        oacc[ct][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yv, pv[ks][rt], oacc[ct][rt], 0, 0, 0);
    };

    // The micro-slices.  `slot` counts logit MFMAs of the stage: 0 .. RT*NS-1.
    constexpr int kSlots = G::RT * G::NS;
    constexpr int S = G::RT;                   // slots per contraction step
    auto micro = [&](int slot) {
      if (slot == 2 * S + S - 1) {             // B1
        __builtin_amdgcn_s_waitcnt(0xc07f);    // lgkmcnt(0): this wave's LDS stores of the last stage landed
        __builtin_amdgcn_s_barrier();
      }
      if (DoSoftmax) {
        // partial logits of tile i: four 16/32-byte reads, then the sums, a few steps later
        if (slot >= 3 * S && slot < 3 * S + 4) sm_issue(slot - 3 * S);
        // staging: the chunks loaded during the previous stage (key tile i+3, value tile i) go to
        // LDS, then the same registers receive key tile i+4 and value tile i+1: a whole stage
        // of latency cover, enough for a first touch that has to come from HBM
        // With 60 slots in a stage the 15 pieces (LDS store, cache-side fetch, block-side fetch of each
        // chunk) get a slot each, in the slots the softmax leaves free at the end of the stage: one LDS
        // store or one load fits the shadow of an MFMA, a store and two loads together do not.
        constexpr int kPieces = 3 * (G::XPER + G::VPER);
        constexpr bool kSpread = kSlots - kPieces - 1 >= kSlots * 3 / 5 + 8;   // behind the softmax and the mixing fetches
        static_assert(!CIN || !kSpread, "[K | V] banks run on the 32-slot tiles' staging order");
        if (kSpread) {
          constexpr int Z0 = kSlots - kPieces - 1;
          if (slot >= Z0 && slot < Z0 + kPieces) {
            const int piece = slot - Z0, it = piece / 3, what = piece % 3;
            if (it < G::XPER) {
              const int item = tid + it * kThreads, jn = j0 + 4 * BN;
              if (what == 0) store_x(it, j0 + 3 * BN, Xstage);
              else load_half(xreg[it], cat_k, jn - G::PAD + (item >> 4), item & 15, what == 2);
            } else {
              const int iv = it - G::XPER, item = tid + iv * kThreads;
              if (what == 0) store_v(iv, j0, Vstage);
              else load_half(vreg[iv], cat_v, j0 + BN + (item >> 4), item & 15, what == 2);
            }
          }
        } else {
          if ((PH != 1 || DoConv) && slot >= 5 * S && slot < 5 * S + G::XPER) {
            store_x(slot - 5 * S, j0 + 3 * BN, Xstage);
            load_x(slot - 5 * S, j0 + 4 * BN);
          }
          if (PH != 1 && slot >= 5 * S + G::XPER && slot < 5 * S + G::XPER + G::VPER) {
            store_v(slot - 5 * S - G::XPER, j0, Vstage);
            load_v(slot - 5 * S - G::XPER, j0 + BN);
          }
        }
        if (slot >= 8 * S && slot < 8 * S + E4) sm_add(0, slot - 8 * S);
        if (slot >= 8 * S + E4 && slot < 8 * S + 2 * E4) sm_add(2, slot - 8 * S - E4);
        if (slot == 8 * S + 2 * E4) __builtin_amdgcn_s_barrier();   // B2: the partial logits have been consumed
        if (PH == 1 && slot == 8 * S + 2 * E4 + 1) {
          // first walk: this lane's four sums go to the workspace; the second walk reads them back (same lane,
          // at device scope: from the L2 the store went through to, whatever this CU's L1 holds from a step ago)
          static_assert(!CIN || E4 == 1, "one 16-byte chunk of key-side logits per lane and tile");
          const f32x4 v = {sv[0], sv[1], sv[2], sv[3]};
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), pre_rows, ((j0 / BN) * (BM * BN) + tid * 4) * 4, 0, 0);
        }
        if (PH == 2 && slot == 8 * S + 2 * E4 + 1)     // the next tile's, a whole stage before they are added
          pre = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(pre_rows, ((j0 / BN + 1) * (BM * BN) + tid * 4) * 4, 0, kDeviceScope));
        if (PH != 1 && slot == 8 * S + 2 * E4 + 1) {
          if (j0 + BN > T) {                   // tail tile: positions past T carry no weight
#pragma unroll
            for (int e = 0; e < G::EPL; ++e)
              if (j0 + sp0 + e >= T) sv[e] = NORM == 0 ? -INFINITY : 0.f;
          }
          if (PROT && pmask) {                 // neither do the positions of protected slots
#pragma unroll
            for (int e = 0; e < G::EPL; ++e)
              if ((pmask >> (sp0 + e)) & 1u) sv[e] = NORM == 0 ? -INFINITY : 0.f;
          }
          if (NORM == 0) {
            mx = sv[0];
#pragma unroll
            for (int e = 1; e < G::EPL; ++e) mx = fmaxf(mx, sv[e]);
          }
        }
        if (PH != 1 && NORM == 0 && slot == 8 * S + 2 * E4 + 2) mx = group_max<G::LPR>(mx);
        if (PH != 1 && NORM == 0 && slot == 8 * S + 2 * E4 + 3) {
          // The reference only moves when the row maximum outgrows it by kLazy, so exp(s - ref)
          // stays below e^kLazy and the accumulators are rescaled rarely.  Every tile has a
          // position < T, so mx is finite -- unless all 32 positions of the tile are protected
          // slots: such a tile adds nothing and leaves the reference alone.
          const bool dead = PROT && mx == -INFINITY;
          bump = !dead && mx > m_run + kLazy;
          m_new = bump ? mx : m_run;
          alpha = bump ? __expf(m_run - m_new) : 1.0f;
          mc = dead ? 0.f : m_new * kLog2e;
        }
        constexpr int X0 = 8 * S + 2 * E4 + 4;   // one exponential per slot
        if (PH != 1 && slot >= X0 && slot < X0 + G::EPL) sm_exp(slot - X0);
        if (PH != 1 && slot == X0 + G::EPL) {
#pragma unroll
          for (int e = 0; e < G::EPL; ++e) psum += sv[e];
        }
        if (PH != 1 && slot == X0 + G::EPL + 1) {
          psum = group_sum<G::LPR>(psum);
          l_run = l_run * alpha + psum;
          m_run = m_new;
        }
        if (PH != 1 && slot == X0 + G::EPL + 2) {
#pragma unroll
          for (int e2 = 0; e2 < G::EPL / 2; ++e2) packed[e2] = pack_bf16(sv[2 * e2], sv[2 * e2 + 1]);
        }
        if (PH != 1 && slot == X0 + G::EPL + 3) {
#pragma unroll
          for (int e4 = 0; e4 < E4; ++e4) {
            const u32x2 pk = {packed[2 * e4], packed[2 * e4 + 1]};
            *(u32x2*)(Pcur + srow * G::PSTRIDE + (sp0 + e4 * 4) * 2) = pk;
          }
          if ((l % G::LPR) == 0) alpha_cur[srow] = alpha;
        }
      }
      if (DoMix) {
        constexpr int M0 = kSlots * 3 / 5;       // operand fragments of tile i-1's mixing, one fetch per slot
        if (slot == M0) {
#pragma unroll
          for (int rt = 0; rt < G::RT; ++rt) al[rt] = alpha_prev[rt * 32 + l31];
        }
        if (slot == M0 + 1) mix_fetch_p(0);
        if (slot == M0 + 2) mix_fetch_p(1);
        if (slot == M0 + 3) mix_fetch_y(0, 0);
        if (slot == M0 + 4) mix_fetch_y(0, 1);
        if (slot == M0 + 5) mix_fetch_y(1, 0);
        if (slot == M0 + 6) mix_fetch_y(1, 1);
        // (rarely) rescale the accumulators before tile i-1 is mixed in
        if (slot == M0 + 7) {
          bool any = false;
#pragma unroll
          for (int rt = 0; rt < G::RT; ++rt) any |= al[rt] != 1.0f;
          if (__any(any)) {
#pragma unroll
            for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
              for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                for (int q = 0; q < 16; ++q) oacc[ct][rt][q] *= al[rt];
          }
        }
      }
    };

    if (DoConv && i < 0) {                     // only the very first stage has nobody to fetch for it
#pragma unroll
      for (int st = 0; st < kRing - 1; ++st) fetch(st);
    }
    __builtin_amdgcn_sched_barrier(0);

#pragma unroll
    for (int st = 0; st < G::NS; ++st) {
      const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt) {
        if (DoConv) {
          sacc[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xv[st % kRing], wreg[rt][st >> 1][st & 1],
                                                             st == 0 ? zero : sacc[rt], 0, 0, 0);
          if (rt == G::RT - 1) fetch(st + kRing - 1);   // the ring slot of step st-1 is free now
        }
        micro(st * S + rt);
        __builtin_amdgcn_sched_barrier(0);     // pin the order: MFMA, then this slot's slice
      }
    }
    // Mixing MFMAs of tile i-1 run while the last logit MFMAs drain; the partial logits are
    // published in between.  The next stage's B1 makes them visible.
    if (DoMix && DoConv) {
      // one partial-logit store behind each mixing MFMA: the stores issue in the shadow of the matrix
      // pipe instead of as one burst
      int nw = 0;
      auto one_write = [&]() {
        const int rt = nw / 4, g = nw % 4;
        if (rt < G::RT) {
          const f32x4 v = {sacc[rt][g * 4 + 0], sacc[rt][g * 4 + 1], sacc[rt][g * 4 + 2], sacc[rt][g * 4 + 3]};
          *(f32x4*)(Sred + (w * BM + rt * 32 + l31) * G::SSTRIDE + g * 8 + lh * 4) = v;
        }
        ++nw;
      };
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          const s16x4 a0 = y0[ks][ct], a1 = y1[ks][ct];
          const s16x8 yy = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
          const bf16x8 yv = __builtin_bit_cast(bf16x8, yy);
#pragma unroll
          for (int rt = 0; rt < G::RT; ++rt) {
            oacc[ct][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(yv, pv[ks][rt], oacc[ct][rt], 0, 0, 0);
            one_write();
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      while (nw < 4 * G::RT) one_write();
    } else {
      if (DoMix) { mix_mfma(0, 0); mix_mfma(0, 1); }
      if (DoConv) write_partials();
      if (DoMix) { mix_mfma(1, 0); mix_mfma(1, 1); }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- meeting point of the slot tiles of a chain between two steps of the one-launch scan:
  // a counter per chain.  A tile signals when its rows of the new cache are written and waits,
  // before it reads the chain's cache for the next step, until the counter says that every tile
  // has signalled: round r is complete at tiles * (r + 1).  A workgroup with several chains goes
  // through them in the same order as the other tiles of its group, so by the time it comes back to a
  // chain the others have long signalled and the wait costs one load; with one chain per
  // workgroup the wait follows the signal directly.
  //
  // General form: workgroup barrier, thread 0 does a device-scope release increment (which writes
  // the L2 back: every dirty line of the XCD, about 3 us per step on the 32 K-token workload);
  // the wait polls, then a device-scope acquire, then a workgroup barrier.  One wave pays for the
  // cache maintenance.
  //
  // When all tiles of the chain run on one XCD they share one L2, and nothing has to be written
  // back or invalidated there: stores go through the CU's L1 to the L2 and have arrived when the
  // wave's store counter reaches zero, and the cache rows are read at device scope (see
  // load_cat16).  So each wave waits for its stores, the workgroup meets, thread 0 increments with
  // a relaxed device-scope atomic and polls with relaxed loads.  Whether the tiles share an XCD is
  // not assumed from the workgroup numbering: round 0, before the first step, is a general-form
  // meeting in which every tile reports the XCD it runs on.
  __shared__ int bail;                       // a chain wait timed out: leave
  __shared__ int same_l2;
  if (tid == 0) { bail = 0; same_l2 = 0; }
  __syncthreads();
  auto chain_signal = [&](int c) {
    const bool fast = same_l2 != 0;          // LDS word written before the previous workgroup barrier
    if (fast) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0) {
      if (fast) __hip_atomic_fetch_add(sa.sync + c, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else __hip_atomic_fetch_add(sa.sync + c, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
  };
  auto chain_wait = [&](int c, int round) -> bool {
    if (tid == 0) {
      // round 0 (the census) is signalled by every workgroup of the chain, later rounds by the one
      // workgroup per slot tile that writes the rows
      const uint32_t target = (uint32_t)(tiles * P) + (uint32_t)tiles * (uint32_t)round;
      int polls = 0;
      while (__hip_atomic_load(sa.sync + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        __builtin_amdgcn_s_sleep(2);
        if (++polls > sa.spin_limit) {         // bounded: never spin forever on a workgroup that is not there
          __hip_atomic_store(sa.status, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          bail = 1;
          break;
        }
      }
      if (same_l2 == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
    return bail == 0;
  };
  if (PSPLIT && tid == 0) {
    // every part registers the XCD it runs on in the census word of its (chain, tile); read at the hand-off
    const uint32_t xcd = __builtin_amdgcn_s_getreg(20 | ((4 - 1) << 11)) & 7u;
    __hip_atomic_fetch_add(sa.psync + 2 * (grp * tiles + i0 / BM) + 1, 1u << (3u * xcd), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
  }
  if (sa.n_steps > 1) {
    uint32_t* xcd_mask = sa.sync + n_chains + 1;
    if (tid == 0) {
      const uint32_t xcd = __builtin_amdgcn_s_getreg(20 | ((4 - 1) << 11));   // XCC_ID, bits [3:0]
      for (int c = grp; c < n_chains; c += groups)
        __hip_atomic_fetch_or(xcd_mask + c, 1u << xcd, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    for (int c = grp; c < n_chains; c += groups) chain_signal(c);
    bool one_xcd = true;
    for (int c = grp; c < n_chains; c += groups) {
      if (!chain_wait(c, 0)) return;
      if (tid == 0) {
        const uint32_t mask = __hip_atomic_load(xcd_mask + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        one_xcd = one_xcd && (mask & (mask - 1)) == 0;
      }
    }
    if (tid == 0) same_l2 = one_xcd && sa.same_l2_allowed;
    __syncthreads();
  }

  const int n_mine = MULTI ? (n_chains - grp + groups - 1) / groups : 1;
  // A bank over [K | V] makes two passes over the workgroup's chains per step -- every chain's first walk
  // with the key half of the filters in the registers, then every chain's second walk with the value
  // half -- so that a step costs two loads of a filter slice however many chains share it.
  for (int step = 0; step < sa.n_steps; ++step)
  for (int pass = 0; pass < (CIN ? 2 : 1); ++pass) {
  if (PIPE && (step & 1) != part) continue;            // the partner's step
  if (CIN) load_filters(pass);
  for (int ci = 0; ci < n_mine; ++ci) {
  const int ch = grp + ci * groups;
  // ---- the step reads what every slot tile of this chain wrote in the step before
  if (!PIPE && pass == 0 && step > 0 && !chain_wait(ch, step)) return;
  // PIPE: the chain is met between the two legs of the walk
  const bool meet_between = PIPE && pass == 0 && step > 0;
  int first_blk = 0, NT_all = 0;
  // ---- this step's inputs: source state, occupancy, block
  {
    const int b = ch / a.Hkv, hkv = ch % a.Hkv;
    if (PROT) pwords = a.protect + (int64_t)ch * a.protect_stride;
    const int64_t tok = (int64_t)step * sa.B;
    const int Bn = step == 0 ? a.Bn : (int)(sa.tokens_left - tok < sa.B ? sa.tokens_left - tok : sa.B);
    m = step == 0 ? a.m : a.M;
    T = m + Bn;
    NT = (T + BN - 1) / BN;
    if (PIPE) {                        // tiles from first_blk on read block rows only, halo included
      NT_all = NT;
      first_blk = (m + G::PAD + BN - 1) / BN;
      if (first_blk > NT_all) first_blk = NT_all;
    }
    if (PSPLIT) {                      // this part's range of position tiles (possibly empty)
      const int per = (NT + P - 1) / P, lo = part * per;
      const int hi = lo + per < NT ? lo + per : NT;
      jbase = lo * BN;
      NT = hi > lo ? hi - lo : 0;
    }
    const int64_t prev = (int64_t)((sa.slot0 + step - 1) % sa.ring) * sa.out_stride;   // (unused for step 0)
    const uint16_t* src_k = step == 0 ? (const uint16_t*)a.cache_k : (const uint16_t*)sa.out_k + prev;
    const uint16_t* src_v = step == 0 ? (const uint16_t*)a.cache_v : (const uint16_t*)sa.out_v + prev;
    cat_k = make_cat(src_k + (int64_t)ch * a.M * kD, m,
                     (const uint16_t*)a.k.p + b * a.k.sb + hkv * a.k.sh + tok * a.k.st, a.k.st, Bn);
    cat_v = make_cat(src_v + (int64_t)ch * a.M * kD, m,
                     (const uint16_t*)a.v.p + b * a.v.sb + hkv * a.v.sh + tok * a.v.st, a.v.st, Bn);
  }
  // ---- prologue of a walk: key tiles 0, 1 and 2 staged; key tile 3 and value tile 0 on their way.  All
  // loads are issued before the first store (the accumulators' registers are free here), so the
  // walk starts after one memory latency, not three.
  auto prologue = [&](bool with_v) {
    const int jb = SPLIT ? jbase : 0;
    Cat16 xpro[3][G::XPER];
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int it = 0; it < G::XPER; ++it) {
        const int item = tid + it * kThreads;
        xpro[t][it] = load_cat16(cat_k, jb + t * BN - G::PAD + (item >> 4), item & 15);
      }
#pragma unroll
    for (int it = 0; it < G::XPER; ++it) load_x(it, jb + 3 * BN);
    if (with_v) {
#pragma unroll
      for (int it = 0; it < G::VPER; ++it) load_v(it, jb);
    }
#pragma unroll
    for (int t = 0; t < 3; ++t)
#pragma unroll
      for (int it = 0; it < G::XPER; ++it) {
        const int item = tid + it * kThreads;
        *(u32x4*)(Xs0 + t * G::XBYTES + (item >> 4) * G::XSTRIDE + (item & 15) * 16) =
            xpro[t][it].from_cache | xpro[t][it].from_blk;
      }
    __syncthreads();
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  constexpr std::integral_constant<int, -1> dyn{};
  // The steady stages with the phase of the buffer rings known at compile time: one copy of the stage per
  // residue of the tile index modulo 2 * NXBUF, chained, so that the ring addresses are constants (about 30
  // scalar and 14 vector instructions per stage otherwise).  Ten copies of a stage still fit the instruction
  // cache.  Built where the register allocation takes it without spilling (32-slot tiles, width 15, filters over
  // the keys; measured: 3 % on the smaller and 9 % on the larger of the shapes that run on pairs of workgroups);
  // the 64-slot builds answered with spills inside the copies and ran 1.6 times as long (two copies, with only the
  // parity of the index a constant, did not spill and gained 0.7 %, but the launch then fetched 18 % more from
  // HBM), so they and every other build keep the one copy.
  constexpr bool RINGU = BM == 32 && KW == 15 && !CIN && SPLIT != 1 && !(PROT && SPLIT == 2);
  auto steady_unrolled = [&](auto ph_t) {
    int i = 1;
    auto one = [&](auto r_t) {
      if (!(i + 1 < NT)) return false;
      stage(i, yes, yes, yes, ph_t, r_t);
      ++i;
      return true;
    };
    for (;;) {
      if (!one(std::integral_constant<int, 1>{})) break;
      if (!one(std::integral_constant<int, 2>{})) break;
      if (!one(std::integral_constant<int, 3>{})) break;
      if (!one(std::integral_constant<int, 4>{})) break;
      if (!one(std::integral_constant<int, 5>{})) break;
      if (!one(std::integral_constant<int, 6>{})) break;
      if (!one(std::integral_constant<int, 7>{})) break;
      if (!one(std::integral_constant<int, 8>{})) break;
      if (!one(std::integral_constant<int, 9>{})) break;
      if (!one(std::integral_constant<int, 0>{})) break;
    }
  };
  static_assert(G::NXBUF == 5 && G::NVBUF == 2, "the unrolled steady stages assume a ring period of ten");
  if constexpr (PIPE) {
  // ---- a step in two legs: the same sequence of stages as the one-walk form below, as functions of the
  // leg's range.  The two forms are kept apart on purpose: the one-walk builds' register allocation is
  // tight (all 512 registers in use) and has answered to small changes of this code with spills inside the
  // stage loop, so they keep their code as it was.
  constexpr std::integral_constant<int, 1> first{};
  constexpr std::integral_constant<int, CIN ? 2 : 0> ph{};
  // first walk over a [K | V] bank: the key half of the filters, the key rows; summed logits to the workspace
  auto walk_first = [&]() {
    prologue(false);
    stage(-1, yes, no, no, first, dyn);
    for (int i = 0; i + 1 < NT; ++i) stage(i, yes, yes, no, first, dyn);
    stage(NT - 1, no, yes, no, first, dyn);
  };
  // the walk that mixes: pipeline fill, steady state, drain
  auto walk_main = [&]() {
    if (CIN)
      pre = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(pre_rows, (((SPLIT ? jbase : 0) / BN) * (BM * BN) + tid * 4) * 4, 0, kDeviceScope));
    prologue(true);
    if constexpr (RINGU) {
      stage(-1, yes, no, no, ph, std::integral_constant<int, 9>{});
      if (NT > 1) {
        stage(0, yes, yes, no, ph, std::integral_constant<int, 0>{});
        steady_unrolled(ph);
        stage(NT - 1, no, yes, yes, ph, dyn);
      } else {
        stage(0, no, yes, no, ph, std::integral_constant<int, 0>{});
      }
      stage(NT, no, no, yes, ph, dyn);
      return;
    }
    stage(-1, yes, no, no, ph, dyn);                          // logits of tile 0 only
    if (NT > 1) {
      stage(0, yes, yes, no, ph, dyn);
      for (int i = 1; i + 1 < NT; ++i) stage(i, yes, yes, yes, ph, dyn);
      stage(NT - 1, no, yes, yes, ph, dyn);
    } else {
      stage(0, no, yes, no, ph, dyn);
    }
    stage(NT, no, no, yes, ph, dyn);
  };
  auto zero_state = [&]() {
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][rt][i] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
  };
  // PIPE: the range of a leg of the walk; the chain is met before the leg that touches the cache
  auto set_leg = [&](int leg) -> bool {
    if (leg == 0) {
      jbase = first_blk * BN;
      NT = NT_all - first_blk;
    } else {
      if (meet_between && !chain_wait(ch, step)) return false;
      jbase = 0;
      NT = first_blk;
    }
    return true;
  };
  if constexpr (CIN) {
    // (the two workgroups of a pair work on different steps at the same time: an area each)
    pre_rows = __builtin_amdgcn_make_buffer_rsrc((void*)(sa.prelogits + (int64_t)((ch * tiles + i0 / BM) * (PIPE ? 2 : 1) + (PIPE ? part : 0)) * sa.pre_stride), 0,
                                                 (int)sa.pre_stride * 4, 0x00020000);
    if (pass == 0) {
      for (int leg = 0; leg < 2; ++leg) {
        if (!set_leg(leg)) return;
        if (NT > 0) walk_first();
        __syncthreads();                 // the next leg's prologue writes the tiles this one read last
      }
      continue;
    }
    // ---- second walk: the value half, the value rows where the key rows were and the other way round
    { const CatRows t = cat_k; cat_k = cat_v; cat_v = t; }
  }
  zero_state();
  for (int leg = 0; leg < 2; ++leg) {
    if (!set_leg(leg)) return;
    if (NT > 0) walk_main();
    if (leg == 0) __syncthreads();
  }

  } else {
  if constexpr (CIN) {
    pre_rows = __builtin_amdgcn_make_buffer_rsrc((void*)(sa.prelogits + (int64_t)(ch * tiles + i0 / BM) * sa.pre_stride), 0,
                                                 (int)sa.pre_stride * 4, 0x00020000);
    if (pass == 0) {
      // ---- first walk: the key half of the filters, the key rows; summed logits to the workspace
      constexpr std::integral_constant<int, 1> first{};
      if (!SPLIT || NT > 0) {
        prologue(false);
        stage(-1, yes, no, no, first, dyn);
        for (int i = 0; i + 1 < NT; ++i) stage(i, yes, yes, no, first, dyn);
        stage(NT - 1, no, yes, no, first, dyn);
      }
      continue;
    }
    // ---- second walk: the value half, the value rows where the key rows were and the other way round
    { const CatRows t = cat_k; cat_k = cat_v; cat_v = t; }
    pre = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(pre_rows, (((SPLIT ? jbase : 0) / BN) * (BM * BN) + tid * 4) * 4, 0, kDeviceScope));
  }
  if (!SPLIT || NT > 0) {
#pragma unroll
  for (int ct = 0; ct < 2; ++ct)
#pragma unroll
    for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[ct][rt][i] = 0.f;
  m_run = -INFINITY;
  l_run = 0.f;
  constexpr std::integral_constant<int, CIN ? 2 : 0> ph{};
  prologue(true);
  if constexpr (RINGU) {
  stage(-1, yes, no, no, ph, std::integral_constant<int, 9>{});
  if (NT > 1) {
    stage(0, yes, yes, no, ph, std::integral_constant<int, 0>{});
    steady_unrolled(ph);
    stage(NT - 1, no, yes, yes, ph, dyn);
  } else {
    stage(0, no, yes, no, ph, std::integral_constant<int, 0>{});
  }
  stage(NT, no, no, yes, ph, dyn);
  } else {
  stage(-1, yes, no, no, ph, dyn);                          // logits of tile 0 only

  // ---- pipeline fill, steady state, drain
  if (NT > 1) {
    stage(0, yes, yes, no, ph, dyn);
    for (int i = 1; i + 1 < NT; ++i) stage(i, yes, yes, yes, ph, dyn);
    stage(NT - 1, no, yes, yes, ph, dyn);
  } else {
    stage(0, no, yes, no, ph, dyn);
  }
  stage(NT, no, no, yes, ph, dyn);
  }
  } else {                                 // a part without positions hands in an empty result
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int rt = 0; rt < G::RT; ++rt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[ct][rt][i] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
  }

  }   // one walk per step

  uint16_t* nk;
  uint16_t* nv;
  {
    const int64_t out_at = (int64_t)((sa.slot0 + step) % sa.ring) * sa.out_stride + ((int64_t)ch * a.M + i0) * kD;
    // (after the second walk of a [K | V] bank the accumulator's first d columns are the value rows)
    nk = (uint16_t*)(CIN ? sa.out_v : sa.out_k) + out_at;
    nv = (uint16_t*)(CIN ? sa.out_k : sa.out_v) + out_at;
  }
  if constexpr (PSPLIT) {
    // ---- this part's result goes to the workspace: accumulators [slot][2 d] as they are
    // (unnormalised, relative to this part's reference), then the references, then the row sums
    float* mine = sa.partials + ((int64_t)(ch * tiles + i0 / BM) * P + part) * G::PART_FLOATS;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const f32x4 v = {oacc[ct][0][g * 4 + 0], oacc[ct][0][g * 4 + 1], oacc[ct][0][g * 4 + 2], oacc[ct][0][g * 4 + 3]};
        *(f32x4*)(mine + l31 * (2 * kD) + 64 * w + ct * 32 + g * 8 + lh * 4) = v;
      }
    if ((l % G::LPR) == 0) {
      mine[BM * 2 * kD + srow] = m_run;
      mine[BM * 2 * kD + BM + srow] = l_run;
    }
    // ---- hand-off.  The parts of a (chain, tile) count themselves in; the one that completes the
    // count merges.  Two forms, as for the meeting of a chain: when all parts run on one XCD they
    // share its L2, so a part's stores have arrived once its store counter is at zero and the merging
    // part reads them at device scope (from the L2); otherwise device-scope release / acquire.  Which
    // form applies is read from the census word of the (chain, tile), where every part registered
    // its XCD when the kernel started: P registrations, all in this workgroup's field.  (A part that
    // looks before everybody has registered takes the general form, which is always safe.)
    __shared__ int i_merge;
    __shared__ int split_fast;
    uint32_t* cnt = sa.psync + 2 * (ch * tiles + i0 / BM);
    if (tid == 0) {
      const uint32_t xcd = __builtin_amdgcn_s_getreg(20 | ((4 - 1) << 11)) & 7u;   // XCC_ID
      split_fast = sa.same_l2_allowed &&
                   __hip_atomic_load(cnt + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ((uint32_t)P << (3u * xcd));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    const bool fast = split_fast != 0;
    if (tid == 0) {
      const uint32_t old = fast ? __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                                : __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
      i_merge = (old + 1u) % (uint32_t)P == 0u;
    }
    __syncthreads();
    if (!i_merge) continue;              // the merging part signals the chain; this one goes on to the next step
    // ---- merge: reference = the largest of the parts' references; every part's sums and
    // accumulators are scaled to it and added in the order of the parts.  All loads are issued
    // before the first is used: one trip to the L2 for the lot.
    float* scale_s = Sred;               // [part][slot]
    float* inv_s = Sred + 4 * BM;        // 1 / row sum
    const __amdgpu_buffer_rsrc_t parts = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(sa.partials + (int64_t)(ch * tiles + i0 / BM) * P * G::PART_FLOATS), 0, P * G::PART_FLOATS * 4, 0x00020000);
    constexpr int kIters = BM * (2 * kD / 4) / kThreads;      // (slot, four columns of [K | V]) chunks per thread
    u32x4 raw[kIters][4];
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int e = tid + it * kThreads, slot = e / (2 * kD / 4), c4 = e % (2 * kD / 4);
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < P)
          raw[it][p] = __builtin_amdgcn_raw_buffer_load_b128(parts, (p * G::PART_FLOATS + slot * (2 * kD) + c4 * 4) * 4, 0, kDeviceScope);
    }
    if (tid < BM) {
      float mp[4], lp[4], mstar = -INFINITY;
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < P) {
          mp[p] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(parts, (p * G::PART_FLOATS + BM * 2 * kD + tid) * 4, 0, kDeviceScope));
          lp[p] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(parts, (p * G::PART_FLOATS + BM * 2 * kD + BM + tid) * 4, 0, kDeviceScope));
        }
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < P) mstar = fmaxf(mstar, mp[p]);
      float lsum_all = 0.f;
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < P) {
          const float sc = (NORM == 0) ? (mp[p] == -INFINITY ? 0.f : __expf(mp[p] - mstar)) : 1.0f;
          scale_s[p * BM + tid] = sc;
          lsum_all += sc * lp[p];
        }
      inv_s[tid] = 1.0f / (NORM == 0 ? lsum_all : lsum_all + a.eps);
    }
    __syncthreads();
    uint32_t keep = 0;                     // live protected slots keep their old rows (BM = 32: one mask word)
    if (PROT && i0 < m) {
      keep = pwords[i0 >> 5];
      if (i0 + 32 > m) keep &= (1u << (m - i0)) - 1u;
    }
#pragma unroll
    for (int it = 0; it < kIters; ++it) {
      const int e = tid + it * kThreads, slot = e / (2 * kD / 4), c4 = e % (2 * kD / 4);
      if (PROT && ((keep >> slot) & 1u)) continue;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int p = 0; p < 4; ++p)
        if (p < P) {
          const float sc = scale_s[p * BM + slot];
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[q] = fmaf(sc, __uint_as_float(raw[it][p][q]), acc[q]);
        }
      const float inv = inv_s[slot];
      u32x2 pk;
      pk[0] = pack_bf16(acc[0] * inv, acc[1] * inv);
      pk[1] = pack_bf16(acc[2] * inv, acc[3] * inv);
      uint16_t* dst = (c4 < kD / 4 ? nk : nv) + (int64_t)slot * kD + (c4 % (kD / 4)) * 4;
      *(u32x2*)dst = pk;
    }
    if (PROT && keep) {
#pragma unroll
      for (int it = 0; it < 2 * BM * 16 / kThreads; ++it) {
        const int e = tid + it * kThreads;
        const int kv = e / (BM * 16), r = (e >> 4) % BM, c16 = e & 15;
        if ((keep >> r) & 1u) {
          const int off = (i0 + r) * (kD * 2) + c16 * 16;
          *(u32x4*)((kv ? nv : nk) + (int64_t)r * kD + c16 * 8) =
              __builtin_amdgcn_raw_buffer_load_b128(kv ? cat_v.cache : cat_k.cache, off, 0, kDeviceScope);
        }
      }
    }
  } else {
  // ---- normalise by the row sums and store the new cache rows.  A lane holds 4 columns of a
  // slot at a time; the rows are put together in the key-tile area of LDS (free after the last
  // stage) and leave as whole rows, 1 KB of contiguous memory per wave instruction.
  if ((l % G::LPR) == 0) lsum[srow] = l_run;
  __syncthreads();
  unsigned char* Orows = Xs0;                // [K rows of the tile ; V rows of the tile][XSTRIDE]
  static_assert(2 * BM * G::XSTRIDE <= G::NXBUF * G::XBYTES, "the output rows fit the key-tile area");
  uint32_t keep[G::RT];
#pragma unroll
  for (int rt = 0; rt < G::RT; ++rt) {
    // a live protected slot keeps its old row (copied below) instead of Eq. 4a / 4b
    keep[rt] = 0;
    if (PROT && i0 + rt * 32 < m) {
      keep[rt] = pwords[(i0 >> 5) + rt];
      if (i0 + rt * 32 + 32 > m) keep[rt] &= (1u << (m - i0 - rt * 32)) - 1u;
    }
    const int slot = rt * 32 + l31;
    const float inv = 1.0f / (NORM == 0 ? lsum[slot] : lsum[slot] + a.eps);
    unsigned char* orow = Orows + ((w >> 1) * BM + slot) * G::XSTRIDE + (64 * (w & 1)) * 2;
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        u32x2 pk;
        pk[0] = pack_bf16(oacc[ct][rt][g * 4 + 0] * inv, oacc[ct][rt][g * 4 + 1] * inv);
        pk[1] = pack_bf16(oacc[ct][rt][g * 4 + 2] * inv, oacc[ct][rt][g * 4 + 3] * inv);
        *(u32x2*)(orow + (ct * 32 + g * 8 + lh * 4) * 2) = pk;
      }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2 * BM * 16 / kThreads; ++it) {      // (K or V, slot, 16-byte chunk)
    const int e = tid + it * kThreads;
    const int kv = e / (BM * 16), r = (e >> 4) % BM, c16 = e & 15;
    uint16_t* dst = (kv ? nv : nk) + (int64_t)r * kD + c16 * 8;
    if (PROT && ((keep[r >> 5] >> (r & 31)) & 1u)) {         // live protected slot: inside the cache resources
      const int off = (i0 + r) * (kD * 2) + c16 * 16;
      *(u32x4*)dst = __builtin_amdgcn_raw_buffer_load_b128(kv ? cat_v.cache : cat_k.cache, off, 0, kDeviceScope);
    } else {
      *(u32x4*)dst = *(const u32x4*)(Orows + (kv * BM + r) * G::XSTRIDE + c16 * 16);
    }
  }
  }  // not split

  // ---- the rows are on their way: tell the other tiles of the chain.  (The barrier also keeps
  // the next prologue's LDS stores behind the copy-out above.)
  if (step + 1 < sa.n_steps) chain_signal(ch);
  else __syncthreads();
  }  // chains
  }  // steps and passes
}

// [M][C][k] per bank -> register order (see compress_mfma_k); one thread per 16-byte chunk.  C = 128,
// or 256 ([K | V] filters): then a bank is its key half (channels 0..127 of every slot) in that
// order followed by its value half.
__global__ void repack_filters_k(const uint16_t* w, uint16_t* wp, int M, int C, int KW, int banks,
                                 int64_t w_head_stride) {
  const int64_t chunks_per_bank = (int64_t)M * KW * (C / 8);
  for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < chunks_per_bank * banks;
       e += (int64_t)gridDim.x * blockDim.x) {
    const int bank = (int)(e / chunks_per_bank);
    int64_t r = e % chunks_per_bank;
    const int lane = (int)(r % 64); r /= 64;
    const int h = (int)(r % 2); r /= 2;
    const int t = (int)(r % KW); r /= KW;
    const int wv = (int)(r % 4); r /= 4;
    const int tile = (int)(r % (M / 32)); r /= M / 32;      // r: which half of a [K | V] bank
    const int slot = tile * 32 + (lane & 31);
    const int c0 = (int)r * kD + 32 * wv + 16 * h + (lane >> 5) * 8;
    const uint16_t* src = w + bank * w_head_stride + ((int64_t)slot * C + c0) * KW + t;
#pragma unroll
    for (int q = 0; q < 8; ++q) wp[e * 8 + q] = src[(int64_t)q * KW];
  }
}

__global__ void zero_words_k(uint32_t* p, int n, uint32_t* p2, int n2) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = 0u;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n2; i += gridDim.x * blockDim.x) p2[i] = 0u;
}

// The instantiation a shape runs on, handed to `f` as compile-time constants (BM, KW, NORM, PROT, MULTI).
// 64-slot tiles when they still give every compute unit a workgroup, else 32-slot tiles; the filter
// slice of a 64-slot tile fits the registers for width 15 only.
bool use_big_tiles(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  return k_width == 15 && !conv_in && (M % 64 == 0) && (int64_t)batch * Hkv * (M / 64) >= n_cu;
}
template <int V> using ic = std::integral_constant<int, V>;
// Parts the positions of a step are shared out between (1: no split).  Only with 32-slot tiles and
// one chain per workgroup, as long as the grid still fits the compute units and the cache part of
// a step alone gives every part four position tiles (with fewer, handing the partial results over
// costs more than the shorter walk saves: measured on the 3.5 K-token shape, M = 128).  A function of the shape and the device only:
// every schedule and every block of a scan use the same number, so results do not depend on them.
// Two workgroups per (chain, 32-slot tile) that take the steps of a scan in turn (SPLIT = 2 builds): whenever
// that still fits the compute units.  A function of the shape and the device only, like the position split
// (which it replaces where both would apply: a scan gains more from it).
bool step_pipeline(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  if (debug_options().no_step_pipeline) return false;
  if (use_big_tiles(batch, Hkv, M, k_width, conv_in, n_cu)) return false;
  return (int64_t)batch * Hkv * (M / 32) * 2 <= n_cu;
}
int position_split(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  if (use_big_tiles(batch, Hkv, M, k_width, conv_in, n_cu)) return 1;
  if (step_pipeline(batch, Hkv, M, k_width, conv_in, n_cu)) return 1;
  const int64_t grid = (int64_t)batch * Hkv * (M / 32);
  int p = 1;
  while (p < 4 && grid * (2 * p) <= n_cu && M / 32 >= 4 * (2 * p)) p *= 2;
  return p;
}
template <class F>
hipError_t with_instantiation(const StepArgs& t, bool multi, int split, int n_cu, F&& f) {   // split: 0, 1 positions, 2 steps
  const bool big = use_big_tiles(t.batch, t.Hkv, t.M, t.k_width, t.conv_in, n_cu);
  auto pick_cin = [&](auto bm, auto kw, auto norm, auto prot, auto mu, auto spl) {
    if constexpr (decltype(bm)::value == 32) {
      if (t.conv_in) return f(bm, kw, norm, prot, mu, spl, ic<1>{});
    }
    return f(bm, kw, norm, prot, mu, spl, ic<0>{});
  };
  auto pick_multi = [&](auto bm, auto kw, auto norm, auto prot) {
    if constexpr (decltype(bm)::value == 32) {
      if (split == 1 && !multi) return pick_cin(bm, kw, norm, prot, ic<0>{}, ic<1>{});
      if (split == 2 && !multi) return pick_cin(bm, kw, norm, prot, ic<0>{}, ic<2>{});
    }
    return multi ? pick_cin(bm, kw, norm, prot, ic<1>{}, ic<0>{}) : pick_cin(bm, kw, norm, prot, ic<0>{}, ic<0>{});
  };
  auto pick_prot = [&](auto bm, auto kw, auto norm) {
    return t.protect ? pick_multi(bm, kw, norm, ic<1>{}) : pick_multi(bm, kw, norm, ic<0>{});
  };
  auto pick_norm = [&](auto bm, auto kw) {
    return t.norm == 1 ? pick_prot(bm, kw, ic<1>{}) : pick_prot(bm, kw, ic<0>{});
  };
  if (t.k_width == 15) return big ? pick_norm(ic<64>{}, ic<15>{}) : pick_norm(ic<32>{}, ic<15>{});
  if (t.k_width == 21) return pick_norm(ic<32>{}, ic<21>{});
  return hipErrorInvalidValue;   // compress_mfma_supports() keeps other shapes away
}

template <int BM, int KW, int NORM, int PROT, int MULTI, int SPLIT, int CIN>
hipError_t prepare_kernel() {
  static bool attr_set = false;   // benign race: setting it twice is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)compress_mfma_k<BM, KW, NORM, PROT, MULTI, SPLIT, CIN>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Geo<BM, KW>::LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  return hipSuccess;
}

hipError_t dispatch(const ScanArgs& a, const uint16_t* wp, int64_t wp_head_stride, int n_cu, hipStream_t s) {
  const bool multi = a.groups < a.st.batch * a.st.Hkv;
  return with_instantiation(a.st, multi, a.pipe ? 2 : (a.psplit > 1 ? 1 : 0), n_cu, [&](auto bm, auto kw, auto norm, auto prot, auto mu, auto sp, auto ci) {
    constexpr int BM = decltype(bm)::value, KW = decltype(kw)::value, NORM = decltype(norm)::value;
    constexpr int PROT = decltype(prot)::value, MULTI = decltype(mu)::value, SPLIT = decltype(sp)::value;
    constexpr int CIN = decltype(ci)::value;
    hipError_t e = prepare_kernel<BM, KW, NORM, PROT, MULTI, SPLIT, CIN>();
    if (e != hipSuccess) return e;
    dim3 grid((a.st.M / BM) * a.groups * (SPLIT ? a.psplit : 1));
    constexpr int kLds = Geo<BM, KW>::LDS;
    hipLaunchKernelGGL((compress_mfma_k<BM, KW, NORM, PROT, MULTI, SPLIT, CIN>), grid, dim3(kThreads), kLds, s, a, wp,
                       wp_head_stride);
    return hipGetLastError();
  });
}

}  // namespace

bool compress_mfma_supports(int dtype, int d, int M, int conv_width, int conv_in, int norm,
                            const char** why) {
  if (dtype != LOCOCO_BF16) { *why = "the MFMA kernels take bf16 storage only"; return false; }
  if (d != kD) { *why = "the MFMA kernels take head_dim = 128 only"; return false; }
  (void)conv_in;                     // filters over the keys or over [K | V]
  if (norm != 0 && norm != 1) { *why = "unknown normalisation"; return false; }
  if (conv_width != 15 && conv_width != 21) {
    *why = "the MFMA compression kernel is built for conv_width = 15 and 21";
    return false;
  }
  if (M % 32) { *why = "the MFMA compression kernel needs M to be a multiple of 32"; return false; }
  return true;
}

size_t compress_mfma_filter_bytes(int M, int conv_width, int conv_in, int banks) {
  return (size_t)banks * M * conv_width * kD * (conv_in ? 2 : 1) * 2;
}

// key-side logits of the first walk of a [K | V] bank: per (chain, 32-slot tile), one 32 x 32 fp32 tile per
// position tile of the longest step
static int64_t prelogits_stride(int M, int B) { return (int64_t)((M + B + BN - 1) / BN) * 32 * BN; }
size_t compress_prelogits_bytes(int batch, int Hkv, int M, int B, int conv_in, int n_cu) {
  const int64_t pairs = (int64_t)batch * Hkv * (M / 32);
  const int areas = pairs * 2 <= n_cu ? 2 : 1;     // one per workgroup of a pair that takes the steps in turn
  return conv_in ? (size_t)pairs * areas * prelogits_stride(M, B) * sizeof(float) : 0;
}

hipError_t launch_repack_filters(const StepArgs& a, void* wp, int banks, hipStream_t s) {
  const int C = a.conv_in ? 2 * kD : kD;
  const int64_t n = (int64_t)banks * a.M * (C / 8) * a.k_width;   // 16-byte chunks
  int blocks = (int)((n + 255) / 256);
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(repack_filters_k, dim3(blocks), dim3(256), 0, s, (const uint16_t*)a.conv_w,
                     (uint16_t*)wp, a.M, C, a.k_width, banks, a.w_head_stride);
  return hipGetLastError();
}

// [chain counters][status word][per chain: bit mask of the XCDs its workgroups run on][per (chain,
// 32-slot tile): count of the parts of a split step that have handed in their result, census of the
// XCDs the parts run on (3 bits per XCD)]
size_t compress_scan_sync_bytes(int batch, int Hkv, int M) {
  return ((size_t)batch * Hkv * (2 + 2 * (M / 32)) + 1) * sizeof(uint32_t);
}
static uint32_t* psync_of(void* sync_ws, int batch, int Hkv) { return (uint32_t*)sync_ws + 2 * batch * Hkv + 1; }

int compress_position_split(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  return position_split(batch, Hkv, M, k_width, conv_in, n_cu);
}
int compress_step_pipeline(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  return step_pipeline(batch, Hkv, M, k_width, conv_in, n_cu) ? 2 : 1;
}
// room for every part's result of one step: [chain][tile][part] x (32 x 2 d accumulators + 32 references + 32 sums)
size_t compress_partials_bytes(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  const int p = position_split(batch, Hkv, M, k_width, conv_in, n_cu);
  return p > 1 ? (size_t)batch * Hkv * (M / 32) * p * Geo<32, 15>::PART_FLOATS * sizeof(float) : 0;
}

hipError_t launch_scan_sync_clear(void* sync_ws, int batch, int Hkv, int M, bool keep_status, hipStream_t s) {
  const int chains = batch * Hkv;
  // everything, or the chain counters and the part counters only
  hipLaunchKernelGGL(zero_words_k, dim3(1), dim3(256), 0, s, (uint32_t*)sync_ws, keep_status ? chains : 2 * chains + 1,
                     psync_of(sync_ws, batch, Hkv), 2 * chains * (M / 32));
  return hipGetLastError();
}

hipError_t launch_compress_mfma(const StepArgs& a, const void* wp, int banks, int n_cu, void* sync_ws,
                                void* partials, void* prelogits, int B, hipStream_t s) {
  ScanArgs sa;
  sa.st = a;
  sa.n_steps = 1;
  sa.B = a.Bn;
  sa.tokens_left = a.Bn;
  sa.out_k = a.new_k;
  sa.out_v = a.new_v;
  sa.out_stride = 0;
  sa.slot0 = 0;
  sa.ring = 1;
  sa.sync = nullptr;
  sa.status = nullptr;
  sa.spin_limit = 0;
  sa.same_l2_allowed = debug_options().chain_sync_device ? 0 : 1;   // (only the hand-off of a split step looks at it here)
  // more (chain, tile) pairs than compute units: one resident workgroup per compute unit, each
  // taking several chains on one load of its filter slice (nothing to wait for within one step)
  sa.groups = compress_scan_groups(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, a.w_head_stride != 0 || a.b_head_stride != 0, n_cu);
  if (sa.groups <= 0) sa.groups = a.batch * a.Hkv;
  sa.prelogits = (float*)prelogits;
  sa.pre_stride = prelogits_stride(a.M, B > a.Bn ? B : a.Bn);
  // fewer than half as many: the positions of the step are shared out between several workgroups,
  // whose count per (chain, tile) starts at zero
  sa.psplit = sa.groups < a.batch * a.Hkv ? 1 : position_split(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, n_cu);
  sa.pipe = sa.groups == a.batch * a.Hkv && step_pipeline(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, n_cu) ? 1 : 0;
  sa.partials = (float*)partials;
  sa.psync = psync_of(sync_ws, a.batch, a.Hkv);
  if (sa.pipe) sa.psplit = 2;            // (workgroups per pair; nothing is handed over)
  if (sa.psplit > 1 && !sa.pipe) {
    hipLaunchKernelGGL(zero_words_k, dim3(1), dim3(256), 0, s, sa.psync, 2 * a.batch * a.Hkv * (a.M / 32), sa.psync, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int64_t wp_head_stride = banks > 1 ? (int64_t)a.M * a.k_width * kD * (a.conv_in ? 2 : 1) : 0;
  return dispatch(sa, (const uint16_t*)wp, wp_head_stride, n_cu, s);
}

int compress_tile_slots(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu) {
  return use_big_tiles(batch, Hkv, M, k_width, conv_in, n_cu) ? 64 : 32;
}

int compress_scan_max_resident(const StepArgs& a, int n_cu) {
  if (debug_options().max_resident > 0) return (int)debug_options().max_resident;
  const int groups = compress_scan_groups(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, a.w_head_stride != 0 || a.b_head_stride != 0, n_cu);
  const bool multi = groups < a.batch * a.Hkv;
  const int split = multi ? 0 : step_pipeline(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, n_cu) ? 2
                    : position_split(a.batch, a.Hkv, a.M, a.k_width, a.conv_in, n_cu) > 1 ? 1 : 0;
  int per_cu = 0;
  hipError_t e = with_instantiation(a, multi, split, n_cu, [&](auto bm, auto kw, auto norm, auto prot, auto mu, auto sp, auto ci) {
    constexpr int BM = decltype(bm)::value, KW = decltype(kw)::value, NORM = decltype(norm)::value;
    constexpr int PROT = decltype(prot)::value, MULTI = decltype(mu)::value, SPLIT = decltype(sp)::value;
    constexpr int CIN = decltype(ci)::value;
    hipError_t e2 = prepare_kernel<BM, KW, NORM, PROT, MULTI, SPLIT, CIN>();
    if (e2 != hipSuccess) return e2;
    constexpr int kLds = Geo<BM, KW>::LDS;
    return hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (const void*)compress_mfma_k<BM, KW, NORM, PROT, MULTI, SPLIT, CIN>,
                                                        kThreads, kLds);
  });
  if (e != hipSuccess) { (void)hipGetLastError(); return 0; }
  return per_cu * n_cu;
}

int compress_scan_groups(int batch, int Hkv, int M, int k_width, int conv_in, bool per_head, int n_cu) {
  const int bm = use_big_tiles(batch, Hkv, M, k_width, conv_in, n_cu) ? 64 : 32;
  const int tiles = M / bm, chains = batch * Hkv;
  // one workgroup per compute unit (LDS): every workgroup of the launch must be resident at once
  int g = n_cu / tiles;
  if (g >= chains) return chains;
  // Fewer workgroups than (chain, tile) pairs: each takes several chains.  They must share its
  // resident filter slice, and the tiles of a group should share an XCD (ids are dealt round-robin
  // over 8 XCDs: a multiple of 8 groups does that).
  const int unit = per_head ? (Hkv % 8 == 0 ? Hkv : (8 % Hkv == 0 ? 8 : 8 * Hkv)) : 8;
  if (g >= unit) g -= g % unit;
  else if (per_head) g -= g % Hkv;
  return g;
}

hipError_t launch_compress_scan(const ScanArgs& a_in, const void* wp, int banks, int n_cu,
                                void* sync_ws, void* partials, void* prelogits, hipStream_t s) {
  ScanArgs a = a_in;
  const int chains = a.st.batch * a.st.Hkv;
  a.sync = (uint32_t*)sync_ws;
  a.status = (int32_t*)sync_ws + chains;
  a.groups = compress_scan_groups(a.st.batch, a.st.Hkv, a.st.M, a.st.k_width, a.st.conv_in,
                                  a.st.w_head_stride != 0 || a.st.b_head_stride != 0, n_cu);
  a.prelogits = (float*)prelogits;
  a.pre_stride = prelogits_stride(a.st.M, a.B > a.st.Bn ? a.B : a.st.Bn);
  if (a.groups <= 0) return hipErrorInvalidValue;   // the caller keeps such shapes away
  a.psplit = a.groups < chains ? 1 : position_split(a.st.batch, a.st.Hkv, a.st.M, a.st.k_width, a.st.conv_in, n_cu);
  a.pipe = a.groups == chains && step_pipeline(a.st.batch, a.st.Hkv, a.st.M, a.st.k_width, a.st.conv_in, n_cu) ? 1 : 0;
  if (a.pipe) a.psplit = 2;
  a.partials = (float*)partials;
  a.psync = psync_of(sync_ws, a.st.batch, a.st.Hkv);
  const int64_t wp_head_stride = banks > 1 ? (int64_t)a.st.M * a.st.k_width * kD * (a.st.conv_in ? 2 : 1) : 0;
  return dispatch(a, (const uint16_t*)wp, wp_head_stride, n_cu, s);
}

}  // namespace lococo
