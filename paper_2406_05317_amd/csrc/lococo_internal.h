// Internal declarations shared by the host API and the kernel translation
// units of the library.  Nothing here is part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lococo.h"

namespace lococo {

// Process-wide test and measurement hooks (lococo_debug_option); every field 0 by default.
struct DebugOptions {
  int64_t spin_limit;         // polls a waiting workgroup makes before it gives up (0: the default)
  int64_t scan_per_step;      // 1: one launch per compression step even where one launch per scan fits
  int64_t chain_sync_device;  // 1: the slot tiles of a chain always meet with device-scope release / acquire
  int64_t logits_tiles;       // 64 | 128 | 256: slots per workgroup of the Eq. 5 kernel of the unfused MFMA path
  int64_t max_resident;       // > 0: pretend that only this many workgroups of the scan kernel fit the GPU at once
  int64_t unfused_kv;         // 1: [K | V] filters on the unfused MFMA path
  int64_t no_step_pipeline;   // 1: no pairs of workgroups that take the steps of a scan in turn
};
const DebugOptions& debug_options();
// compute units of the current device
int cu_count();

// View of a [batch, heads, tokens, d] tensor, strides in elements.
struct View {
  const void* p;
  int64_t sb, sh, st;
};

// Everything a kernel needs to know about one block step.  Pointers of the
// q/k/v/o views already point at the first token of the block.
struct StepArgs {
  View q, k, v;
  View o;                  // written
  const void* cache_k;     // live cache  [chains, M, d]
  const void* cache_v;
  void* new_k;             // other buffer [chains, M, d] (compress) / live buffer (fill)
  void* new_v;
  const void* conv_w;      // [M, C, k] (+ w_head_stride per kv head)
  const void* conv_b;      // [M] or null
  int64_t w_head_stride, b_head_stride;
  int32_t batch, Hq, Hkv, group, d, M;
  int32_t m;               // live slots before the step
  int32_t Bn;              // tokens in the block
  int32_t k_width;         // conv width
  int32_t conv_in, norm;
  float scale, eps;
  const uint32_t* protect;     // protected-slot bits (see lococo_cache), or null
  int64_t protect_stride;      // words between chains' masks, 0 = shared
  float* colsum;               // accumulated attention per slot [chains, M] (see lococo_cache), or null
  int32_t ldw;                 // elements between the rows of a logits / weights array [chains, M, .]; 0 = m + Bn
};

// Arguments of the fused compression kernel: `n_steps` consecutive compress steps of the scan in
// one launch.  Step 0 is described by `st` (source cache, occupancy st.m, block at the k/v views,
// st.Bn tokens).  Step s > 0 reads the state step s-1 wrote, has a full cache (M slots) and takes
// the block s*B tokens further on (B tokens, fewer if tokens_left runs out).  Step s writes its
// new cache to slot (slot0 + s) % ring of out_k/out_v, slots out_stride elements apart (a ring of
// states: the whole history of a sequence, or a window of it).  Between steps the slot tiles of a chain wait
// for each other on sync[chain] (zeroed by the caller); a wait that exceeds spin_limit polls sets
// *status to 1 and makes the workgroup leave the kernel.
struct ScanArgs {
  StepArgs st;
  int32_t n_steps;
  int32_t B;
  int64_t tokens_left;
  void* out_k;
  void* out_v;
  int64_t out_stride;
  int32_t slot0, ring;       // ring >= 1
  uint32_t* sync;
  int32_t* status;
  int32_t spin_limit;
  int32_t same_l2_allowed;   // 0: always meet with device-scope release / acquire (see compress_mfma.hip)
  int32_t groups;            // workgroups per slot tile; group g runs chains g, g + groups, ... (filled in by the launcher)
  int32_t psplit;            // workgroups that share out the positions of a step of one (chain, slot tile); 1 = no split (launcher)
  int32_t pipe;              // 1: two workgroups per (chain, slot tile) take the steps in turn (psplit = 2 then; launcher)
  float* partials;           // where the parts of a split step leave their results (launcher)
  uint32_t* psync;           // per (chain, 32-slot tile): parts that have handed in (launcher)
  float* prelogits;          // [K | V] filters: key-side logits between the two walks of a step (launcher)
  int64_t pre_stride;        // floats per (chain, 32-slot tile) there (launcher)
};

// Arguments of the MFMA attention kernel: one block, or every block of a scan
// whose intermediate caches were kept.  Block n = seg_first + (launch index)
// covers tokens [n*B, min((n+1)*B, L)) of the q/k/v/o views.  Blocks n <= n_fill
// see the base cache with len0 + n*B live slots (the fill phase appends in
// place; with n_fill = 0 the base is simply the state before block 0); block
// n > n_fill sees history slot (hist_first + n - n_fill - 1) % hist_ring with M live slots.
struct AttnArgs {
  View q, k, v;
  View o;
  const void* cache_k;     // base cache [chains, M, d]
  const void* cache_v;
  const void* hist_k;      // history slots, hist_stride elements apart (may be null if unused)
  const void* hist_v;
  int64_t hist_stride;
  int32_t hist_first, hist_ring;   // hist_ring >= 1 whenever hist_k is used
  int64_t L;
  int32_t B, M, len0, n_fill, seg_first, n_seg;
  int32_t batch, Hq, Hkv, group;
  int32_t qtiles;          // filled in by the launcher
  float scale;
  // Row statistics of the softmax, written when not null: pairs (m, 1 / l) per query row,
  // [batch, Hq, L] with the row index counted like the token index of the q view, such that the
  // probability of a key with raw score s is exp2(s * scale * log2(e) - m) / l.
  float* stats;
};

// Arguments of the backward pass of one block step (backward_generic.hip).  `st` describes the
// step as for the forward (cache = state before the step).  Gradients are fp32, contiguous:
// d_o, d_q [batch, Hq, Bn, d]; d_k, d_v [batch, Hkv, Bn, d]; d_new_k/v, d_cache_k/v [chains, M, d];
// d_conv_w / d_conv_b laid out like conv_w / conv_b (added to).  Workspace: ws_p, ws_ds
// [batch, Hq, Bn, T] (attention rows and their gradient), ws_w [chains, M, T] (raw logits on entry,
// their gradient on exit), ws_n [chains, M, T] (normalised rows), ws_dw [chains, M, T] (gradient of the
// normalised rows).
struct BwdArgs {
  StepArgs st;
  const float* d_o;
  const float* d_new_k;
  const float* d_new_v;
  float* d_q;
  float* d_k;
  float* d_v;
  float* d_cache_k;
  float* d_cache_v;
  float* d_conv_w;
  float* d_conv_b;
  float* ws_p;
  float* ws_ds;
  float* ws_w;
  float* ws_n;
  float* ws_dw;
  void* ws_mfma;           // workspace of the MFMA form of the Eq. 5 contractions (see BwdMfmaLayout), or null
  int32_t banks;           // filter banks (1 = shared by the kv heads)
  int32_t gemms_mfma;      // the plain contractions may take their MFMA form (bf16 storage; see bwd_gemms_mfma_fit)
};
hipError_t launch_step_backward_generic(int dtype, const BwdArgs& g, bool compress, hipStream_t s);

// ---- shape-agnostic kernels (generic_kernels.hip); dtype: LOCOCO_F32 / LOCOCO_BF16
hipError_t launch_attn_generic(int dtype, const StepArgs& a, hipStream_t s);
hipError_t launch_fill_generic(int dtype, const StepArgs& a, hipStream_t s);
hipError_t launch_copy_pair(void* d0, const void* s0, void* d1, const void* s1, size_t bytes, hipStream_t s);
hipError_t launch_zero_fill(void* p, size_t bytes, hipStream_t s);
// logits: fp32 [chains, M, T], T = m + Bn
hipError_t launch_conv_logits_generic(int dtype, const StepArgs& a, float* logits, hipStream_t s);
hipError_t launch_normalise_generic(const StepArgs& a, float* logits, hipStream_t s);
// raw != 0: w holds unnormalised logits, Eq. 6 is applied inside the kernel
hipError_t launch_mix_generic(int dtype, const StepArgs& a, const float* w, int raw,
                              hipStream_t s);
// protected slots on the generic path: logits of protected positions -> -inf (before the
// normalisation); protected rows of the new cache <- the old rows (after the mix)
hipError_t launch_protect_logits_generic(const StepArgs& a, float* logits, hipStream_t s);
hipError_t launch_protect_rows_generic(int dtype, const StepArgs& a, hipStream_t s);
// largest T = m + Bn the generic attention kernel can hold in LDS
int generic_attn_max_T();


// ---- fused compression on MFMA (compress_mfma.hip)
// true if the kernel takes this configuration; otherwise *why names the limit
bool compress_mfma_supports(int dtype, int d, int M, int conv_width, int conv_in, int norm,
                            const char** why);
// bytes of the repacked filter bank ([bank][M][k][C] bf16) the kernel reads
size_t compress_mfma_filter_bytes(int M, int conv_width, int conv_in, int banks);
// bytes the kernel needs between the two walks of a step over a [K | V] bank (0 for filters over the keys);
// B: the longest block of the call
size_t compress_prelogits_bytes(int batch, int Hkv, int M, int B, int conv_in, int n_cu);
// conv_w [M][C][k] (+ w_head_stride per bank) -> wp [bank][M][k][C]
hipError_t launch_repack_filters(const StepArgs& a, void* wp, int banks, hipStream_t s);
// Eq. 5 + Eq. 6 + Eq. 4a/4b in one kernel; writes a.new_k / a.new_v
// sync_ws / partials: compress_scan_sync_bytes() / compress_partials_bytes() of device memory
// prelogits: compress_prelogits_bytes(.., B, ..) of device memory, B >= a.Bn
hipError_t launch_compress_mfma(const StepArgs& a, const void* wp, int banks, int n_cu, void* sync_ws,
                                void* partials, void* prelogits, int B, hipStream_t s);
// workgroups per (chain, slot tile) that share out the positions of a step (1: no split)
int compress_position_split(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu);
// workgroups per (chain, slot tile) that take the steps of a scan in turn: 2, or 1 where the shape does not
int compress_step_pipeline(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu);
size_t compress_partials_bytes(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu);
// Workgroups per slot tile with which all steps of a scan run in one launch, every workgroup
// resident at once (each takes every groups-th chain); 0 if there is no such number.  per_head:
// filters or biases differ between kv heads.
int compress_scan_groups(int batch, int Hkv, int M, int k_width, int conv_in, bool per_head, int n_cu);
// Workgroups of the scan kernel (the instantiation this shape runs on) the current device can hold at
// once, from the runtime's occupancy query; <= 0 if the query failed.  The one-launch scan needs its
// whole grid resident.
int compress_scan_max_resident(const StepArgs& a, int n_cu);
// cache slots per workgroup of the fused kernel for this shape on a device with n_cu compute units
int compress_tile_slots(int batch, int Hkv, int M, int k_width, int conv_in, int n_cu);
// bytes of the sync counters + status word the scan launch needs
size_t compress_scan_sync_bytes(int batch, int Hkv, int M);
// zero them (a fill kernel, so the call may sit inside a captured graph); keep_status: only the chain
// counters, not the status word (between the launches of one call)
hipError_t launch_scan_sync_clear(void* sync_ws, int batch, int Hkv, int M, bool keep_status, hipStream_t s);
// the same kernel over n_steps consecutive compress steps (see ScanArgs); `sync_ws` is
// compress_scan_sync_bytes() of device memory, cleared beforehand
hipError_t launch_compress_scan(const ScanArgs& a, const void* wp, int banks, int n_cu, void* sync_ws,
                                void* partials, void* prelogits, hipStream_t s);


// ---- attention on MFMA (attn_mfma.hip)
bool attn_mfma_supports(int dtype, int d, const char** why);
hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s);
// Adds to colsum [chains, M], for every block of `a` and every live cache slot, the probabilities
// the block's queries (all heads of the group) put on it; reads the statistics the attention
// launch with the same arguments left in a.stats.
hipError_t launch_attn_colsum_mfma(const AttnArgs& a, float* colsum, hipStream_t s);

// ---- attention of one new token per sequence (attn_decode.hip): bf16, head_dim 128, Bn = 1
bool attn_decode_supports(int dtype, int d, int Bn, int M, bool colsum);
hipError_t launch_attn_decode(const StepArgs& a, hipStream_t s);

// ---- Eq. 5 of the backward pass on MFMA (tiled_mfma.hip): bf16, head_dim 128, keys-only or [K | V] filters
bool bwd_mfma_supports(int dtype, int d, int conv_in, int conv_width);
// byte offsets inside its workspace: filters per tap, dW split into two bf16 halves (transposed, then as it is),
// filter gradient per tap
struct BwdMfmaLayout { size_t wt, dhi, dlo, dhi_s, dlo_s, dwt, total; };
BwdMfmaLayout bwd_mfma_layout(int batch, int Hkv, int M, int Tn, int conv_width, int conv_in, int banks);
// conv_w -> [bank][tap][slot][channel] at the layout's wt
hipError_t launch_pack_filters_per_tap(const StepArgs& a, int banks, void* wt, hipStream_t s);
// raw logits fp32 [chains, M, T] (bias added), from the packed filters; keys-only or [K | V] input (a.conv_in)
hipError_t launch_conv_logits_mfma(const StepArgs& a, const void* wt, float* logits, hipStream_t s);
bool conv_logits_mfma_supports(int dtype, int d, int conv_width);
// bytes of the filters packed per tap [bank][tap][slot][channel]
size_t packed_filter_bytes(int M, int conv_width, int conv_in, int banks);
// Eq. 4a / 4b from normalised rows w [chains, M, T] into a.new_k / a.new_v (bf16); needs mix_mfma_fits
bool mix_mfma_fits(const StepArgs& a, const float* w);
hipError_t launch_mix_mfma(const StepArgs& a, const float* w, hipStream_t s);
// Eq. 6 and Eq. 4a / 4b in one kernel, from raw logits [chains, M, ldw] into a.new_k / a.new_v (bf16)
bool mixnorm_mfma_fits(const StepArgs& a, const float* logits);
hipError_t launch_mixnorm_mfma(const StepArgs& a, const float* logits, hipStream_t s);
// dX into d_k / d_cache_k (added) and dWc into d_conv_w (added), from the logit gradient in g.ws_w
hipError_t launch_bwd_conv_mfma(const BwdArgs& g, int banks, void* ws, hipStream_t s);
// the plain contractions of the pass (fp32 operands enter as two bf16 halves): same inputs,
// outputs and workspace arrays as the fp32 kernels of backward_generic.hip they stand in for
bool bwd_gemms_mfma_fit(const BwdArgs& g);                                 // widths multiples of 4, arrays 16-byte aligned
hipError_t launch_bwd_attn_scores_mfma(const BwdArgs& g, hipStream_t s);   // ws_p = scale q Yk^T, ws_ds = dO Yv^T
hipError_t launch_bwd_attn_grads_mfma(const BwdArgs& g, hipStream_t s);    // d_q; first contributions to dYk, dYv
hipError_t launch_bwd_mix_dw_mfma(const BwdArgs& g, hipStream_t s);        // ws_dw
hipError_t launch_bwd_mix_cols_mfma(const BwdArgs& g, hipStream_t s);      // Eq. 4 w.r.t. [K | V], added

// ---- measurement aid (peaks.hip): sustained bf16 MFMA rate of a bare loop and bandwidth of a plain
// copy inside `scratch` (device, overwritten); synchronises the stream
hipError_t measure_peaks(void* scratch, size_t bytes, int n_cu, hipStream_t s, double* mfma_tflops,
                         double* copy_gbs);

}  // namespace lococo
