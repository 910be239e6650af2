/*
 * lococo.h -- C ABI of the MI355X (gfx950) LoCoCo segment-step library.
 *
 * The library computes, for already projected and position-encoded Q/K/V,
 * the forward pass of the paper's Algorithm 2 ("LoCoCo attention"):
 *
 *   step 3   O_n = Attn([Kc, K_n], Q_n, [Vc, V_n])            (Eq. 1, Alg. 2 step 3)
 *   IF       #cache + B <= M : append K_n, V_n to the cache     (Alg. 2, IF branch)
 *   step 4   W = g (*) [Kc ; K_n]   (1-D convolution, Eq. 5),
 *            w = W normalised per slot over the positions       (Eq. 6)
 *   step 5   Kc' = w [Kc ; K_n],  Vc' = w [Vc ; V_n]            (Eq. 3, Eq. 4a/4b)
 *
 * and the scan of that step over a sequence cut into blocks of B tokens.
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library
 *    allocates and frees no device memory; scratch comes from the caller's
 *    `workspace` argument (see lococo_workspace_bytes).
 *  - Struct pointers (config, cache, qkvo, plan rows) are HOST pointers.
 *  - Layouts are row-major with head_dim contiguous.  Strides are in ELEMENTS.
 *  - Arguments are validated synchronously; on a validation status (LOCOCO_EINVAL,
 *    LOCOCO_EUNSUPPORTED, LOCOCO_ESTATE, LOCOCO_EWORKSPACE) nothing was enqueued and
 *    nothing the caller owns has changed.  LOCOCO_EHIP means that a HIP call failed
 *    after some kernels of the call may already have been enqueued: the `cache`
 *    struct (cur / len) is still unchanged, but the cache buffers, the outputs and
 *    the workspace hold undefined contents.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and the call returns without synchronising.
 *    `cache->cur` / `cache->len` are updated on the host at enqueue time.
 *  - No C++ exception crosses the boundary.  lococo_last_error() returns a
 *    thread-local message for the last non-OK status on this thread.
 *  - Calls that use the same cache or workspace must be ordered by the caller
 *    (same stream, or events).
 *
 * Readings of the paper fixed by this interface
 * ---------------------------------------------
 *  - Blocks are 0-based: block n covers tokens [n*B, min((n+1)*B, L)); the
 *    last one may be short.
 *  - Concatenation is cache first, then block (Alg. 2 step 3, Eq. 3), for
 *    attention, for the convolution input and for the fusion.
 *  - Mask: every cache slot is visible to every block query; block key j' is
 *    visible to block query j iff j' <= j.
 *  - Convolution: cross-correlation, zero padding (k-1)/2 on both sides,
 *    stride 1, odd width only.
 *  - Eq. 6 as a softmax over the positions (norm = 0) or, literally,
 *    relu(W) / (sum relu(W) + eps) (norm = 1), or W / sum(W) behind a rectifier
 *    on the convolution's input (norm = 2).
 *  - A compress step with a partly filled cache (m < M, m + B > M) mixes the
 *    m + B entries present.
 */
#ifndef LOCOCO_H
#define LOCOCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; only the functions below are exported. */
#define LOCOCO_API __attribute__((visibility("default")))

typedef enum lococo_status {
  LOCOCO_OK = 0,
  LOCOCO_EINVAL = 1,       /* null pointer, non-positive size, bad stride, aliasing, ...    */
  LOCOCO_EUNSUPPORTED = 2, /* well-formed but not implemented (even conv width, huge T ...) */
  LOCOCO_ESTATE = 3,       /* cache occupancy / buffer index out of range                   */
  LOCOCO_EHIP = 4,         /* a HIP runtime call failed; message holds hipGetErrorString    */
  LOCOCO_EWORKSPACE = 5    /* workspace missing, misaligned or smaller than required        */
} lococo_status;

enum { LOCOCO_F32 = 0, LOCOCO_BF16 = 1 };
enum { LOCOCO_IMPL_AUTO = 0, LOCOCO_IMPL_GENERIC = 1, LOCOCO_IMPL_MFMA = 2 };

/* Problem description.  Plain data, filled by the caller. */
/* lococo_config.flags */
#define LOCOCO_FLAG_FILTERS_PREPARED 1  /* the workspace already holds what lococo_prepare_filters made of
                                           conv_w: steps do not repeat that work (generation stage: the
                                           filters do not change from token to token)                    */

typedef struct lococo_config {
  uint32_t struct_size;   /* sizeof(lococo_config); guards against ABI skew                       */
  int32_t dtype;          /* LOCOCO_F32 / LOCOCO_BF16: storage type of q,k,v,o, cache and filters */
  int32_t batch;
  int32_t n_q_heads;      /* multiple of n_kv_heads; query head h reads kv head h / group         */
  int32_t n_kv_heads;     /* one cache and one compression per (batch, kv head) chain             */
  int32_t head_dim;       /* d                                                                    */
  int32_t M;              /* cache slots (Eq. 3: the compressed length)                           */
  int32_t conv_width;     /* k, odd, >= 1 (Eq. 5; the paper's default is 21)                      */
  int32_t conv_in;        /* 0: filters read keys only, C = d; 1: keys stacked on values along
                             channels, C = 2d (Eq. 5 as printed), K channels first               */
  int32_t norm;           /* 0: softmax over the positions; 1: relu(W)/(sum relu(W)+norm_eps);
                             2: the other reading of the rectifier the paper puts in the head: on the
                             convolution's INPUT (Eq. 4 still fuses the stored entries), and Eq. 6 as
                             printed, W / sum(W), a row sum below norm_eps in magnitude replaced by
                             +-norm_eps (shape-agnostic kernels and forward only)                    */
  int32_t impl;           /* LOCOCO_IMPL_*: AUTO picks the fused MFMA kernels when the shape allows
                             (bf16, head_dim 128, filters of width 15 or 21 over the keys or over
                             [K|V], M a multiple of 32), separate MFMA kernels for Eq. 5 and Eq. 4 for
                             other bf16 / head_dim 128 compressors (odd width <= 31, any M), else
                             the shape-agnostic kernels; GENERIC forces the shape-agnostic kernels;
                             MFMA asks for the fused kernels and fails with LOCOCO_EUNSUPPORTED
                             when the shape does not allow them                                   */
  int32_t flags;          /* LOCOCO_FLAG_* bits, 0 by default                                     */
  int64_t w_head_stride;  /* elements between per-kv-head filter banks; 0 = one shared bank       */
  int64_t b_head_stride;  /* same for the bias                                                    */
  float attn_scale;       /* 0 => 1/sqrt(head_dim)                                                */
  float norm_eps;         /* only for norm = 1; 0 => 1e-6                                         */
} lococo_config;

/* Recurrent state of the scan: the fixed-size KV cache, double buffered. */
typedef struct lococo_cache {
  void* k[2];   /* each [batch, n_kv_heads, M, head_dim], contiguous, 16-byte aligned */
  void* v[2];
  int32_t cur;  /* which of the two buffers is live (0/1)                             */
  int32_t len;  /* live slots 0..M, the same for every chain                          */
  /* Protected slots, for combining the method with an eviction policy that keeps some tokens as
   * they are (the ablation on attention sinks / heavy hitters; the paper does not spell the
   * mechanism out, this is this library's reading).  Device pointer or NULL.  Bit (i % 32) of
   * word [chain * protect_chain_stride + i / 32] set = slot i is protected: once live it is
   * copied unchanged by every compression step (Eq. 4a/4b are not applied to it) and its
   * position gets no weight in the other slots' rows of Eq. 6.  Attention (step 3) is not
   * affected.  ceil(M / 32) words per mask; protect_chain_stride = 0 shares one mask between
   * all (batch, kv head) chains.  The words are read when the kernels run. */
  const uint32_t* protect;
  int64_t protect_chain_stride;
  /* Accumulated attention scores, for policies that pick the slots to protect by them (heavy
   * hitters).  Device pointer or NULL; fp32 [batch, n_kv_heads, M], ADDED to: every attention
   * (step 3) adds, for each live cache slot, the probabilities that the block's queries (all
   * query heads of the group) put on it.  The library never clears or remaps it: after a
   * compression step an unprotected slot holds a different mixture, what its old score means is
   * the caller's business.  On the MFMA path the attention kernel then also writes its row
   * statistics into the workspace and a second pass over the cache keys sums the normalised
   * probabilities per slot (lococo_sequence_forward does it for all blocks at once: the sums
   * commute); a call without workspace (lococo_attn_only, or a fill step given none) attends
   * such a block with the shape-agnostic kernel instead.  One-token blocks (the generation stage)
   * have the sums inside their kernel. */
  float* attn_colsum;
} lococo_cache;

/* A [batch, heads, tokens, head_dim] tensor view; head_dim contiguous. */
typedef struct lococo_tensor {
  void* p;
  int64_t stride_b, stride_h, stride_t;  /* elements; stride_t >= head_dim, multiples of 8 for bf16 */
} lococo_tensor;

/* One block (or one whole sequence) of inputs and the attention output.
 * q, o: n_q_heads heads; k, v: n_kv_heads heads.  o must not alias an input. */
typedef struct lococo_qkvo {
  lococo_tensor q, k, v, o;
} lococo_qkvo;

/* One row of the integer plan of a scan (Alg. 2 loop and its IF). */
typedef struct lococo_seg {
  int64_t start;       /* first token of the block                         */
  int32_t len;         /* tokens in the block (B, or fewer for the last)   */
  int32_t branch;      /* 0: fill (append), 1: compress (steps 4-5)        */
  int32_t len_before;  /* cache occupancy seen by the attention            */
  int32_t len_after;   /* occupancy after the step                         */
  int32_t buf_after;   /* live buffer index after the step                 */
  int32_t reserved;
} lococo_seg;

/* Alg. 2 loop bounds and IF, as integers.  *n_inout holds the capacity of
 * `out` on entry (out may be NULL with capacity 0) and the number of blocks
 * on return; at most the capacity is written.  Host pointers. */
LOCOCO_API lococo_status lococo_plan(int64_t L, int32_t B, int32_t M, int32_t len0, int32_t cur0,
                          lococo_seg* out, int64_t* n_inout);

/* Bytes of device workspace lococo_segment_step (L = B) or
 * lococo_sequence_forward (L = sequence length) need for this shape.
 *   history = 0: the step-by-step schedule (one block's scratch);
 *   history = 1: room for the cache state after every block, with which
 *                lococo_sequence_forward runs the whole compression scan first and then
 *                all blocks' attention as one batched launch;
 *   history = G >= 2: room for a window of G blocks (G + 1 cache states): the same
 *                schedule window by window, memory independent of L.
 * The three schedules return the same bits: which kernel a block's attention runs on depends
 * on the block alone (a block of one token takes the generation-stage kernel in all of them).
 * May return 0. */
LOCOCO_API lococo_status lococo_workspace_bytes(const lococo_config* cfg, int64_t L, int32_t B,
                                     int32_t history, size_t* out);

/* The filter bank in the form the kernels read (for the MFMA path: Eq. 5's [M, C, k] weights
 * repacked into register order at the start of `workspace`; otherwise nothing).  Every call of
 * lococo_segment_step / lococo_sequence_forward does this itself unless the configuration
 * carries LOCOCO_FLAG_FILTERS_PREPARED, in which case the caller must have called this function
 * on the same workspace with the same conv_w since either last changed.  Enqueued on `stream`. */
LOCOCO_API lococo_status lococo_prepare_filters(const lococo_config* cfg, const void* conv_w, void* workspace,
                                     size_t ws_bytes, void* stream);

/* Alg. 2 step 3 alone: o = Attn([Kc, K_blk], Q_blk, [Vc, V_blk]) for one block
 * of B tokens against the live cache (cache->len slots).  Does not modify the
 * cache.  With an empty cache this is plain causal attention (Eq. 1). */
LOCOCO_API lococo_status lococo_attn_only(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                               const lococo_cache* cache, void* stream);

/* One pass of the Alg. 2 loop body: step 3, then either the fill branch or
 * steps 4-5 (Eq. 5, Eq. 6, Eq. 4a/4b) into the other cache buffer.
 * conv_w: [M, C, k] (device, storage dtype); conv_b: [M] or NULL.
 * workspace: device, 256-byte aligned, ws_bytes >= lococo_workspace_bytes(cfg, B, B, 0). */
LOCOCO_API lococo_status lococo_segment_step(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                  const void* conv_w, const void* conv_b, lococo_cache* cache,
                                  void* workspace, size_t ws_bytes, void* stream);

/* lococo_segment_step for callers that cannot allocate device memory or keep a workspace of their
 * own: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, same kernels and the same results as lococo_segment_step, but the scratch the step
 * needs (the repacked filter bank, the row statistics of the attention, on the other paths the
 * logits) lives in an array of LOCOCO_NOALLOC_SCRATCH_BYTES that is part of the library's device
 * code: each GPU the library runs on holds one copy from the moment the library is loaded until the
 * process ends, and the call itself allocates and frees nothing (no hipMalloc, no hipFree, no stream
 * or event creation; the optional kernel timing of lococo_timing_begin, which creates events, must
 * be off).
 *   - A step whose lococo_workspace_bytes(cfg, B, B, 0) exceeds the array is refused with
 *     LOCOCO_EWORKSPACE (enough for the fused path with filters over the keys: 32 heads, M = 512,
 *     width 15 needs 2.1 MB; not for the logits of large shapes on the other paths, nor for the
 *     key-side logits of large shapes with filters over [K | V]).
 *   - LOCOCO_FLAG_FILTERS_PREPARED is refused (LOCOCO_EINVAL): the array is shared by every caller on
 *     the device and keeps whatever the last call left in it, so each call repacks the filters itself.
 *   - Calls that overlap on one GPU (two streams, two threads) race on the array: the caller must
 *     order them, as for any shared workspace.  Nothing in it has to start at zero. */
#define LOCOCO_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
LOCOCO_API lococo_status lococo_segment_step_noalloc(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                                     const void* conv_w, const void* conv_b, lococo_cache* cache,
                                                     void* stream);

/* The whole Alg. 2 loop over a sequence of L tokens in blocks of B, starting
 * from `cache` (len = 0 for a fresh sequence) and leaving the final cache in
 * it.  seq.q/o: [batch, n_q_heads, L, d]; seq.k/v: [batch, n_kv_heads, L, d].
 * The schedule follows from ws_bytes: with lococo_workspace_bytes(cfg, L, B, 1) or more the
 * batched-attention schedule over the whole sequence; with less, the same schedule over
 * windows of as many blocks as the workspace holds states for (at least two); below that
 * the step-by-step schedule.  Results are the same bit for bit. */
LOCOCO_API lococo_status lococo_sequence_forward(const lococo_config* cfg, const lococo_qkvo* seq, int64_t L,
                                      int32_t B, const void* conv_w, const void* conv_b,
                                      lococo_cache* cache, void* workspace, size_t ws_bytes,
                                      void* stream);

/* When lococo_sequence_forward runs a whole scan's compression steps in one launch, the
 * workgroups that share a chain wait for each other between steps with a bounded number of
 * polls (a few seconds).  That form is chosen only when the whole grid can be resident at once
 * (the runtime's occupancy figure for the kernel) and no other such launch of this process is
 * still running on another stream of the device; otherwise every step gets a launch of its own.
 * Work from elsewhere that keeps compute units busy for longer than the bound (another process, a
 * long kernel on another stream) can still make a wait run out: the kernel then leaves early, a
 * status word in the workspace is set, and THE OUTPUTS AND THE CACHE OF THAT CALL ARE INVALID
 * although it returned LOCOCO_OK at enqueue time.  A caller that shares the GPU must therefore
 * check lococo_scan_status() == 0 before it uses the results of a lococo_sequence_forward call
 * made with the larger (history) workspace; a caller that has the GPU to itself need not.
 *
 * This call SYNCHRONISES with the device and returns that word in *out: 0 = fine, 1 = a wait
 * gave up.  `workspace` is the one passed to lococo_sequence_forward (at least
 * lococo_workspace_bytes(history = 0) bytes); the word is cleared at the start of every such call
 * and means nothing before the first one.  Configurations the MFMA kernels do not serve never
 * wait: *out is 0.  Under stream capture the in-flight check is skipped: replays of graphs that
 * hold such a scan must not overlap each other on one device. */
LOCOCO_API lococo_status lococo_scan_status(const lococo_config* cfg, const void* workspace, int32_t* out);

/* Test and measurement hooks, process-wide, not thread safe against running calls; none changes
 * what is computed, and only those that say so below change the order of an fp32 sum (so the last
 * bits).  (Nothing in the library reads environment variables.) */
enum {
  LOCOCO_OPT_RESET = 0,             /* every option back to its default; value ignored                         */
  LOCOCO_OPT_SPIN_LIMIT = 1,        /* polls a waiting workgroup of the one-launch scan makes before it gives
                                       up (0 = default, 2^21); negative: give up at once                       */
  LOCOCO_OPT_SCAN_PER_STEP = 2,     /* 1: one launch per compression step even where one per scan fits         */
  LOCOCO_OPT_CHAIN_SYNC_DEVICE = 3, /* 1: workgroups of a chain always meet with device-scope release and
                                       acquire (default: without the L2 write-back when they find themselves
                                       on one XCD)                                                             */
  LOCOCO_OPT_LOGITS_TILES = 4,      /* 64 | 128 | 256: slots per workgroup of the Eq. 5 kernel of the unfused
                                       MFMA path (0 = chosen from the grid size; 256 needs more than 128 slots
                                       and adds up Eq. 5's fp32 sum in another order)                          */
  LOCOCO_OPT_MAX_RESIDENT = 5,      /* > 0: pretend the device holds only this many workgroups of the scan
                                       kernel at once (exercises the fall-back to one launch per step)         */
  LOCOCO_OPT_UNFUSED_KV = 6,        /* 1: filters over [K | V] go to the unfused MFMA path (Eq. 5 as a kernel
                                       of its own, logits through the workspace) even where the fused kernel
                                       takes them: same definition, another order of the fp32 sums            */
  LOCOCO_OPT_NO_STEP_PIPELINE = 7   /* 1: shapes with at most half as many (chain, slot tile) pairs as compute
                                       units run without the pairs of workgroups that take the steps of a scan
                                       in turn (then the position split applies where it did before): same
                                       definition, another order of the fp32 sums                             */
};
LOCOCO_API lococo_status lococo_debug_option(int32_t option, int64_t value);

/* Which kernels a configuration runs on, on the current device (for tests and benchmark reports). */
typedef struct lococo_path_info {
  int32_t path;                 /* 0: shape-agnostic kernels; 1: fused MFMA compression kernel + MFMA attention;
                                   2: MFMA attention with separate MFMA kernels for Eq. 5 and Eq. 6 / Eq. 4    */
  int32_t compute_units;        /* of the current device                                                       */
  int32_t tile_slots;           /* path 1: cache slots per workgroup of the compression kernel (64 or 32)      */
  int32_t scan_groups;          /* path 1: workgroups per slot tile when lococo_sequence_forward runs all
                                   compression steps in one launch (each takes every scan_groups-th chain);
                                   0 when it would launch every step separately                                */
  int32_t scan_resident_limit;  /* path 1: workgroups of that kernel the device holds at once                  */
  int32_t position_split;       /* path 1: workgroups that share out the positions of a step of one (chain,
                                   slot tile) where one each would leave compute units idle; 1 = no split
                                   (several chains per workgroup never split)                                  */
  int32_t step_pipeline;        /* path 1: 2 where two workgroups per (chain, slot tile) take the steps of a
                                   scan in turn (shapes with at most half as many pairs as compute units:
                                   the one whose turn is next works through the part of its step that does
                                   not depend on the step before while its partner finishes that step); else 1 */
  int32_t reserved;
} lococo_path_info;
LOCOCO_API lococo_status lococo_describe_path(const lococo_config* cfg, int32_t B, lococo_path_info* out);

/* Steps 4-5 with Eq. 5's output supplied by the caller: the cache becomes
 * normalise(logits) . [cache ; block] (Eq. 6, Eq. 4a/4b).  logits: device fp32
 * [batch, n_kv_heads, M, T] contiguous with T = cache->len + B.  Only blk->k
 * and blk->v are read.  Exists so that tests can drive the fusion with chosen
 * weights (e.g. one-hot rows: token selection, the paper's "token dropping"
 * special case).  Always compresses, whatever the occupancy.  With bf16 storage, head_dim 128,
 * impl != LOCOCO_IMPL_GENERIC and T a multiple of 4 the kernel is the MFMA one of the unfused path
 * (Eq. 6 and Eq. 4 together), otherwise the shape-agnostic one; a one-hot row selects its entry bit
 * for bit on either.  Returns LOCOCO_EUNSUPPORTED when cache->protect is set. */
LOCOCO_API lococo_status lococo_mix_from_logits(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                     const float* logits, lococo_cache* cache, void* stream);

/* Backward pass of one block step (lococo_segment_step), for training the convolution heads
 * through the scan: chain rule on Alg. 2 step 3, the fill branch and Eq. 5 / Eq. 6 / Eq. 4a-4b,
 * storage rounding treated as the identity.  The caller walks the blocks in reverse with the
 * cache states it kept from the forward pass.
 *   blk: q, k, v of the block as in the forward (o is not read); cache_before: the state the
 *   forward step started from (cur / len / protect as they were then).
 *   Gradients are fp32 device arrays, contiguous:
 *     in   d_o [batch, n_q_heads, B, d]; d_new_k, d_new_v [batch, n_kv_heads, M, d]: gradient
 *          w.r.t. the cache AFTER the step (rows at and beyond its occupancy are ignored by a
 *          fill step and must be zero for a compress step's unused slots: there are none);
 *     out  d_q [batch, n_q_heads, B, d]; d_k, d_v [batch, n_kv_heads, B, d]; d_cache_k,
 *          d_cache_v [batch, n_kv_heads, M, d]: gradient w.r.t. the cache BEFORE the step
 *          (rows that were not live are zero); all five are overwritten;
 *     acc  d_conv_w (laid out like conv_w, with w_head_stride) and d_conv_b (like conv_b, may be
 *          NULL) are ADDED to, so one buffer collects the whole scan; untouched by a fill step.
 *   workspace: lococo_backward_workspace_bytes(cfg, B, cache_before->len) bytes, 256-byte aligned.
 * Any shape; fp32 vector arithmetic, except that with bf16 storage and cfg->impl !=
 * LOCOCO_IMPL_GENERIC the contractions run on the matrix cores, every fp32 operand entering as
 * the sum of two bf16 numbers (about 16 bits kept): the plain ones when block length + live
 * slots is a multiple of 4, the three convolution ones (Eq. 5 and its two gradients) with
 * head_dim 128 and a filter width up to 31 (the workspace is larger then).  Filter gradients are summed
 * with floating-point atomics, so their last bits depend on the order. */
LOCOCO_API lococo_status lococo_backward_workspace_bytes(const lococo_config* cfg, int32_t B, int32_t len, size_t* out);
LOCOCO_API lococo_status lococo_segment_step_backward(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                           const void* conv_w, const void* conv_b,
                                           const lococo_cache* cache_before, const float* d_o,
                                           const float* d_new_k, const float* d_new_v, float* d_q,
                                           float* d_k, float* d_v, float* d_cache_k, float* d_cache_v,
                                           float* d_conv_w, float* d_conv_b, void* workspace,
                                           size_t ws_bytes, void* stream);

/* Backward pass of a whole scan (lococo_sequence_forward's recurrence), for training the
 * convolution heads through Alg. 2's loop: the chain rule through every block step in reverse, the
 * gradient w.r.t. a block's starting state being handed to the block before it as the gradient
 * w.r.t. that block's resulting state.  The call runs the cache recurrence once more block by
 * block (the fill branch or steps 4-5), keeping the state every block starts from in the workspace, then walks the
 * blocks backwards through lococo_segment_step_backward; gradients therefore match that entry
 * point's composed by hand, launch for launch.
 *   seq: q, k, v of the L tokens as in the forward (o is not read); cache0: the state the scan
 *   starts from (not modified; its attn_colsum is neither read nor written).
 *   Gradients are fp32 device arrays, contiguous:
 *     in   d_o [batch, n_q_heads, L, d]; d_final_k, d_final_v [batch, n_kv_heads, M, d]: gradient
 *          w.r.t. the state after the last block, or NULL for zero;
 *     out  d_q [batch, n_q_heads, L, d]; d_k, d_v [batch, n_kv_heads, L, d]; d_cache0_k, d_cache0_v
 *          [batch, n_kv_heads, M, d] (rows that were not live in cache0 are zero); all overwritten;
 *     acc  d_conv_w, d_conv_b: ADDED to, as in the step (d_conv_b may be NULL).
 *   workspace: lococo_sequence_backward_workspace_bytes(cfg, L, B) bytes, 256-byte aligned: two
 *   states per block (storage type) plus one step's worth of everything else.
 * LOCOCO_FLAG_FILTERS_PREPARED is refused (the call owns its workspaces); norm = 2 is forward only. */
LOCOCO_API lococo_status lococo_sequence_backward_workspace_bytes(const lococo_config* cfg, int64_t L, int32_t B,
                                                                  size_t* out);
LOCOCO_API lococo_status lococo_sequence_backward(const lococo_config* cfg, const lococo_qkvo* seq, int64_t L,
                                                  int32_t B, const void* conv_w, const void* conv_b,
                                                  const lococo_cache* cache0, const float* d_o,
                                                  const float* d_final_k, const float* d_final_v, float* d_q,
                                                  float* d_k, float* d_v, float* d_cache0_k, float* d_cache0_v,
                                                  float* d_conv_w, float* d_conv_b, void* workspace,
                                                  size_t ws_bytes, void* stream);

/* Optional per-kernel timing.  Between lococo_timing_begin() and
 * lococo_timing_end() every kernel the library launches (from any thread) is
 * bracketed by a pair of HIP events recorded on the stream it is launched on.
 * lococo_timing_end() waits for those events and returns one row per kernel
 * that ran: its name (static storage), the number of launches and the summed
 * device time in milliseconds.  *n_inout: capacity of `out` on entry, rows
 * available on return.  Host pointers.  Meant for benchmarks; not thread safe
 * against concurrent begin/end. */
typedef struct lococo_kernel_time {
  const char* name;
  int64_t launches;
  double total_ms;
} lococo_kernel_time;
LOCOCO_API lococo_status lococo_timing_begin(void);
LOCOCO_API lococo_status lococo_timing_end(lococo_kernel_time* out, int32_t* n_inout);

/* Measurement aid for benchmarks (no step of the method): what the current
 * GPU sustains on a bare bf16 MFMA loop (32x32x16, no memory traffic; the
 * better of one and two waves per SIMD) and on a plain copy inside `scratch`
 * (bytes read + bytes written per second), so that a kernel's rate can be
 * quoted against the measured ceilings next to the published ones.
 *   scratch: device, 16-byte aligned, bytes >= 32 MiB (use >= 1 GiB for a
 *            figure that is not a cache's); contents overwritten.
 *   mfma_tflops, copy_gbs: host, written on success.
 * Runs for about 0.2 s (long enough for the clock to settle under matrix load)
 * and waits for the stream.
 * LOCOCO_EINVAL for null / misaligned / too small arguments. */
LOCOCO_API lococo_status lococo_measure_peaks(void* scratch, size_t bytes, void* stream, double* mfma_tflops,
                                   double* copy_gbs);

/* Message for the last non-OK status returned on the calling thread
 * (static thread-local storage; never NULL). */
LOCOCO_API const char* lococo_last_error(void);

/* Library version, "major.minor.patch". */
LOCOCO_API const char* lococo_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOCOCO_H */
