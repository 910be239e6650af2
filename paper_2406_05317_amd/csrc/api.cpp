// Host side of the C ABI declared in lococo.h: argument validation, the
// integer plan of the scan (Alg. 2 loop and IF), path selection and kernel
// sequencing.  No arithmetic of the method happens here.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <vector>

#include "lococo_internal.h"

using namespace lococo;

// The library's own scratch array (see lococo_segment_step_noalloc): device memory that exists from
// the moment the code object is loaded.  On the host this name is only a handle for
// hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[LOCOCO_NOALLOC_SCRATCH_BYTES];

namespace {
DebugOptions g_debug = {0, 0, 0, 0, 0, 0, 0};
}
namespace lococo {
const DebugOptions& debug_options() { return g_debug; }
int cu_count() {
  static int n = 0;
  if (!n) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      n = prop.multiProcessorCount;
    if (n <= 0) n = 256;
  }
  return n;
}
}  // namespace lococo

namespace {

thread_local char g_err[512] = "";

lococo_status fail(lococo_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

lococo_status hip_fail(hipError_t e, const char* what) {
  return fail(LOCOCO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(expr, what)                         \
  do {                                              \
    hipError_t e_ = (expr);                         \
    if (e_ != hipSuccess) return hip_fail(e_, what); \
  } while (0)

// ---- optional per-kernel timing with HIP events (lococo_timing_begin / _end)
enum KernelId { K_ATTN_GENERIC, K_FILL, K_CONV_GENERIC, K_NORM_GENERIC, K_MIX_GENERIC,
                K_REPACK, K_COMPRESS_MFMA, K_ATTN_MFMA, K_ATTN_DECODE, K_ATTN_COLSUM, K_CONV_MFMA, K_MIX_MFMA,
                K_COUNT };
const char* const kKernelNames[K_COUNT] = {"attn_generic", "fill", "conv_logits_generic",
                                           "normalise_generic", "mix_generic", "repack_filters",
                                           "compress_mfma", "attn_mfma", "attn_decode", "attn_colsum",
                                           "conv_logits_mfma", "mix_mfma"};
struct TimedLaunch { int id; hipEvent_t start, stop; };
std::mutex g_timing_mu;
bool g_timing_on = false;
std::vector<TimedLaunch> g_timed;

// Records an event pair around the launches made while it is alive.
struct KTimer {
  int id;
  hipStream_t s;
  hipEvent_t start = nullptr, stop = nullptr;
  KTimer(int id_, hipStream_t s_) : id(id_), s(s_) {
    if (!g_timing_on) return;
    if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) {
      start = stop = nullptr;
      return;
    }
    (void)hipEventRecord(start, s);
  }
  ~KTimer() {
    if (!start) return;
    (void)hipEventRecord(stop, s);
    std::lock_guard<std::mutex> lk(g_timing_mu);
    g_timed.push_back(TimedLaunch{id, start, stop});
  }
};

size_t esize(int dtype) { return dtype == LOCOCO_F32 ? 4 : 2; }
size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

lococo_status check_config(const lococo_config* c) {
  if (!c) return fail(LOCOCO_EINVAL, "config is NULL");
  if (c->struct_size != sizeof(lococo_config))
    return fail(LOCOCO_EINVAL, "config.struct_size is %u, this library expects %zu", c->struct_size,
                sizeof(lococo_config));
  if (c->dtype != LOCOCO_F32 && c->dtype != LOCOCO_BF16)
    return fail(LOCOCO_EINVAL, "config.dtype %d is neither LOCOCO_F32 nor LOCOCO_BF16", c->dtype);
  if (c->batch <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 || c->M <= 0)
    return fail(LOCOCO_EINVAL, "batch, head counts, head_dim and M must be positive");
  if (c->n_q_heads % c->n_kv_heads)
    return fail(LOCOCO_EINVAL, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", c->n_q_heads,
                c->n_kv_heads);
  if (c->conv_width < 1) return fail(LOCOCO_EINVAL, "conv_width must be >= 1");
  if (c->conv_width % 2 == 0)
    return fail(LOCOCO_EUNSUPPORTED, "conv_width %d is even; only odd widths have a centred "
                "same-length convolution", c->conv_width);
  if (c->conv_in != 0 && c->conv_in != 1) return fail(LOCOCO_EINVAL, "conv_in must be 0 or 1");
  if (c->norm < 0 || c->norm > 2) return fail(LOCOCO_EINVAL, "norm must be 0, 1 or 2");
  if (c->impl < LOCOCO_IMPL_AUTO || c->impl > LOCOCO_IMPL_MFMA)
    return fail(LOCOCO_EINVAL, "impl must be one of LOCOCO_IMPL_*");
  if (c->flags & ~LOCOCO_FLAG_FILTERS_PREPARED) return fail(LOCOCO_EINVAL, "config.flags has unknown bits set");
  if (c->w_head_stride < 0 || c->b_head_stride < 0)
    return fail(LOCOCO_EINVAL, "filter head strides must be >= 0");
  if (!(c->attn_scale >= 0.f) || !(c->norm_eps >= 0.f) || std::isinf(c->attn_scale))
    return fail(LOCOCO_EINVAL, "attn_scale and norm_eps must be finite and >= 0");
  if (c->head_dim > 1024) return fail(LOCOCO_EUNSUPPORTED, "head_dim > 1024");
  if (c->n_q_heads > 65535 || c->batch > 65535 || c->M > 65535 ||
      (int64_t)c->batch * c->n_kv_heads > 65535)
    return fail(LOCOCO_EUNSUPPORTED, "batch, heads, M or batch*n_kv_heads above 65535");
  return LOCOCO_OK;
}

lococo_status check_tensor(const lococo_config* c, const lococo_tensor& t, const char* name,
                           int64_t tokens) {
  if (!t.p) return fail(LOCOCO_EINVAL, "%s pointer is NULL", name);
  if (t.stride_t < c->head_dim)
    return fail(LOCOCO_EINVAL, "%s.stride_t (%lld) is below head_dim", name, (long long)t.stride_t);
  if (t.stride_h < 0 || t.stride_b < 0)
    return fail(LOCOCO_EINVAL, "%s strides must be non-negative", name);
  if (c->dtype == LOCOCO_BF16 &&
      ((t.stride_t | t.stride_h | t.stride_b) % 8 || ((uintptr_t)t.p & 15)))
    return fail(LOCOCO_EINVAL, "%s: bf16 tensors need 16-byte aligned pointers and strides that "
                "are multiples of 8 elements", name);
  if (c->dtype == LOCOCO_F32 && ((uintptr_t)t.p & 3))
    return fail(LOCOCO_EINVAL, "%s pointer is not 4-byte aligned", name);
  (void)tokens;
  return LOCOCO_OK;
}

lococo_status check_cache(const lococo_config* c, const lococo_cache* ca) {
  if (!ca) return fail(LOCOCO_EINVAL, "cache is NULL");
  for (int i = 0; i < 2; ++i) {
    if (!ca->k[i] || !ca->v[i]) return fail(LOCOCO_EINVAL, "cache buffer pointer is NULL");
    if (((uintptr_t)ca->k[i] | (uintptr_t)ca->v[i]) & 15)
      return fail(LOCOCO_EINVAL, "cache buffers must be 16-byte aligned");
  }
  const void* p[4] = {ca->k[0], ca->k[1], ca->v[0], ca->v[1]};
  for (int i = 0; i < 4; ++i)
    for (int j = i + 1; j < 4; ++j)
      if (p[i] == p[j]) return fail(LOCOCO_EINVAL, "cache buffers alias each other");
  if (ca->cur != 0 && ca->cur != 1) return fail(LOCOCO_ESTATE, "cache.cur is %d", ca->cur);
  if (ca->len < 0 || ca->len > c->M)
    return fail(LOCOCO_ESTATE, "cache.len %d is outside [0, M=%d]", ca->len, c->M);
  if (ca->protect) {
    if ((uintptr_t)ca->protect & 3) return fail(LOCOCO_EINVAL, "cache.protect is not 4-byte aligned");
    if (ca->protect_chain_stride != 0 && ca->protect_chain_stride < (c->M + 31) / 32)
      return fail(LOCOCO_EINVAL, "cache.protect_chain_stride must be 0 or at least ceil(M / 32) words");
  }
  if ((uintptr_t)ca->attn_colsum & 3) return fail(LOCOCO_EINVAL, "cache.attn_colsum is not 4-byte aligned");
  return LOCOCO_OK;
}

lococo_status check_qkvo(const lococo_config* c, const lococo_qkvo* x, int64_t tokens,
                         bool need_q_o) {
  if (!x) return fail(LOCOCO_EINVAL, "qkvo is NULL");
  lococo_status st;
  if (need_q_o) {
    if ((st = check_tensor(c, x->q, "q", tokens))) return st;
    if ((st = check_tensor(c, x->o, "o", tokens))) return st;
    if (x->o.p == x->q.p || x->o.p == x->k.p || x->o.p == x->v.p)
      return fail(LOCOCO_EINVAL, "o aliases an input");
  }
  if ((st = check_tensor(c, x->k, "k", tokens))) return st;
  if ((st = check_tensor(c, x->v, "v", tokens))) return st;
  return LOCOCO_OK;
}

// PATH_MFMA: the fused compression kernel.  PATH_MFMA_UNFUSED: shapes it does not take (other filter
// widths, [K | V] filters, M not a multiple of 32) with bf16 storage and head_dim 128: attention on
// MFMA, Eq. 5 and Eq. 4 as two MFMA kernels around the shape-agnostic normalisation, the logits
// passing through the workspace in fp32.
enum Path { PATH_GENERIC = 0, PATH_MFMA = 1, PATH_MFMA_UNFUSED = 2 };

// Which kernels take this shape.  *why is set when the fused kernel is refused.
Path choose_path(const lococo_config* c, int32_t B, const char** why) {
  (void)B;
  const char* ignore = "";
  if (!attn_mfma_supports(c->dtype, c->head_dim, why)) return PATH_GENERIC;
  if (compress_mfma_supports(c->dtype, c->head_dim, c->M, c->conv_width, c->conv_in, c->norm, why) &&
      !(c->conv_in && g_debug.unfused_kv))
    return PATH_MFMA;
  if (c->norm != 2 &&                 // the input-side rectifier exists in the shape-agnostic kernels only
      conv_logits_mfma_supports(c->dtype, c->head_dim, c->conv_width) && attn_mfma_supports(c->dtype, c->head_dim, &ignore))
    return PATH_MFMA_UNFUSED;
  return PATH_GENERIC;
}

int filter_banks(const lococo_config* c) { return c->w_head_stride ? c->n_kv_heads : 1; }

lococo_status resolve_path(const lococo_config* c, int32_t B, Path* out) {
  const char* why = "";
  Path p = c->impl == LOCOCO_IMPL_GENERIC ? PATH_GENERIC : choose_path(c, B, &why);
  if (c->impl == LOCOCO_IMPL_MFMA && p != PATH_MFMA)     // MFMA means the fused kernel, nothing less
    return fail(LOCOCO_EUNSUPPORTED, "impl = MFMA requested but %s", why);
  *out = p;
  return LOCOCO_OK;
}

// Workspace of one step.  Generic: fp32 logits [chains, M, T], T <= M + B.
// MFMA: the repacked filter bank.
size_t filter_ws_bytes(const lococo_config* c) {
  return align_up(compress_mfma_filter_bytes(c->M, c->conv_width, c->conv_in, filter_banks(c)), 256);
}
// chain sync counters + status word of the one-launch scan
size_t scan_sync_bytes(const lococo_config* c) {
  return align_up(compress_scan_sync_bytes(c->batch, c->n_kv_heads, c->M), 256);
}
// softmax statistics of `rows` query rows per head (what the column sums of the MFMA attention need)
size_t stats_bytes(const lococo_config* c, int64_t rows) {
  return align_up((size_t)c->batch * c->n_q_heads * (size_t)rows * 2 * sizeof(float), 256);
}
// filters packed per tap for the unfused MFMA path
size_t packed_ws_bytes(const lococo_config* c) {
  return align_up(packed_filter_bytes(c->M, c->conv_width, c->conv_in, filter_banks(c)), 256);
}
size_t logits_bytes(const lococo_config* c, int32_t B) {     // rows of up to M + B logits, padded to a multiple of 4
  return align_up((size_t)c->batch * c->n_kv_heads * c->M * (((size_t)c->M + B + 3) / 4 * 4) * sizeof(float), 256);
}
// results of the parts of a split step (see compress_mfma.hip), 0 where the shape is not split
size_t partials_ws_bytes(const lococo_config* c) {
  return align_up(compress_partials_bytes(c->batch, c->n_kv_heads, c->M, c->conv_width, c->conv_in, cu_count()), 256);
}
// key-side logits between the two walks of a step over [K | V] filters (see compress_mfma.hip), 0 for filters over the keys
size_t prelogits_ws_bytes(const lococo_config* c, int32_t B) {
  return align_up(compress_prelogits_bytes(c->batch, c->n_kv_heads, c->M, B, c->conv_in, cu_count()), 256);
}
// MFMA path: [repacked filters][chain sync counters + status word][row statistics of one block][results of
// the parts of a split step][key-side logits of a step over [K | V] filters]; unfused MFMA path: [filters packed per tap][row statistics of one block][logits];
// generic path: the logits.
size_t step_ws_bytes(const lococo_config* c, Path path, int32_t B) {
  if (path == PATH_MFMA)
    return filter_ws_bytes(c) + scan_sync_bytes(c) + stats_bytes(c, B) + partials_ws_bytes(c) + prelogits_ws_bytes(c, B);
  if (path == PATH_MFMA_UNFUSED) return packed_ws_bytes(c) + stats_bytes(c, B) + logits_bytes(c, B);
  return logits_bytes(c, B);
}
void* partials_of(const lococo_config* c, void* ws, int32_t B) {
  return (char*)ws + filter_ws_bytes(c) + scan_sync_bytes(c) + stats_bytes(c, B);
}
void* prelogits_of(const lococo_config* c, void* ws, int32_t B) { return (char*)partials_of(c, ws, B) + partials_ws_bytes(c); }

// Bytes of one history slot pair member: one cache state [chains, M, d].
size_t state_bytes(const lococo_config* c) {
  return (size_t)c->batch * c->n_kv_heads * c->M * c->head_dim * esize(c->dtype);
}

// Workspace of the batched-attention schedule: the step workspace followed by
// K and V history slots for n_compress cache states.
// Layout: [step workspace][row statistics of the sequence][K history][V history].
size_t history_ws_bytes(const lococo_config* c, Path path, int32_t B, int64_t n_compress, int64_t L) {
  return step_ws_bytes(c, path, B) + stats_bytes(c, L) + 2 * (size_t)n_compress * align_up(state_bytes(c), 256);
}

// Polls a waiting workgroup makes before it gives up on its chain (each poll sleeps ~128 cycles and
// reads the counter from the L2: roughly a microsecond, so the default bounds a wait to a few
// seconds).  The tests force the give-up path from the host with a limit of -1.
int spin_limit() {
  return g_debug.spin_limit ? (int)g_debug.spin_limit : (1 << 21);
}
// By default the slot tiles of a chain skip the L2 write-back between the steps of the one-launch
// scan when they find themselves on one XCD (see compress_mfma.hip).
bool chain_sync_through_l2() { return g_debug.chain_sync_device == 0; }

// One launch for all compression steps of a scan needs every workgroup of it resident at once: the
// grid must fit the occupancy the runtime reports for the kernel, and no other such launch of this
// process may still be running on another stream of the device (two of them could each hold part of
// the compute units and wait for workgroups that never become resident).
constexpr int kMaxDevices = 64;
struct ScanInFlight { hipEvent_t done = nullptr; hipStream_t stream = nullptr; bool valid = false; };
ScanInFlight g_scan[kMaxDevices];
std::mutex g_scan_mu;

bool stream_is_capturing(hipStream_t s) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(s, &st) != hipSuccess) { (void)hipGetLastError(); return false; }
  return st != hipStreamCaptureStatusNone;
}

// call with g_scan_mu held
bool another_scan_in_flight(hipStream_t s) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return true;
  ScanInFlight& g = g_scan[dev];
  if (!g.valid || g.stream == s) return false;        // same stream: ordered behind it
  const hipError_t e = hipEventQuery(g.done);
  if (e == hipSuccess) { g.valid = false; return false; }
  (void)hipGetLastError();
  return true;                                        // not ready (or unknown): assume it still runs
}
void note_scan_launched(hipStream_t s) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
  ScanInFlight& g = g_scan[dev];
  if (!g.done && hipEventCreateWithFlags(&g.done, hipEventDisableTiming) != hipSuccess) {
    (void)hipGetLastError();
    g.done = nullptr;
    return;
  }
  if (hipEventRecord(g.done, s) == hipSuccess) { g.stream = s; g.valid = true; }
  else (void)hipGetLastError();
}

// Whether the shape allows the one-launch form at all (grid rule and occupancy); the in-flight check
// is made under the lock right before the launch.
bool scan_fits_one_launch(const lococo_config* c, const StepArgs& a) {
  if (g_debug.scan_per_step) return false;
  const int groups = compress_scan_groups(c->batch, c->n_kv_heads, c->M, c->conv_width, c->conv_in,
                                          c->w_head_stride != 0 || c->b_head_stride != 0, cu_count());
  if (groups <= 0) return false;
  const int split = groups < c->batch * c->n_kv_heads
                        ? 1 : compress_position_split(c->batch, c->n_kv_heads, c->M, c->conv_width, c->conv_in, cu_count());
  const int pipe = groups < c->batch * c->n_kv_heads
                       ? 1 : compress_step_pipeline(c->batch, c->n_kv_heads, c->M, c->conv_width, c->conv_in, cu_count());
  const int64_t grid = (int64_t)groups * split * pipe *
                       (c->M / compress_tile_slots(c->batch, c->n_kv_heads, c->M, c->conv_width, c->conv_in, cu_count()));
  return grid <= compress_scan_max_resident(a, cu_count());
}

View view_at(const lococo_tensor& t, int64_t tok, size_t es) {
  return View{(const char*)t.p + (size_t)(tok * t.stride_t) * es, t.stride_b, t.stride_h, t.stride_t};
}

StepArgs make_args(const lococo_config* c, const lococo_qkvo* x, int64_t tok, int32_t Bn,
                   const lococo_cache* ca, const void* conv_w, const void* conv_b, bool with_q) {
  StepArgs a;
  std::memset(&a, 0, sizeof(a));
  const size_t es = esize(c->dtype);
  if (with_q) {
    a.q = view_at(x->q, tok, es);
    a.o = view_at(x->o, tok, es);
  }
  a.k = view_at(x->k, tok, es);
  a.v = view_at(x->v, tok, es);
  a.cache_k = ca->k[ca->cur];
  a.cache_v = ca->v[ca->cur];
  a.conv_w = conv_w;
  a.conv_b = conv_b;
  a.w_head_stride = c->w_head_stride;
  a.b_head_stride = c->b_head_stride;
  a.batch = c->batch;
  a.Hq = c->n_q_heads;
  a.Hkv = c->n_kv_heads;
  a.group = c->n_q_heads / c->n_kv_heads;
  a.d = c->head_dim;
  a.M = c->M;
  a.m = ca->len;
  a.Bn = Bn;
  a.k_width = c->conv_width;
  a.conv_in = c->conv_in;
  a.norm = c->norm;
  a.scale = c->attn_scale > 0.f ? c->attn_scale : 1.0f / std::sqrt((float)c->head_dim);
  a.eps = c->norm_eps > 0.f ? c->norm_eps : 1e-6f;
  a.protect = ca->protect;
  a.protect_stride = ca->protect_chain_stride;
  a.colsum = ca->attn_colsum;
  return a;
}

lococo_status check_step_shape(const lococo_config* c, int32_t B, int32_t len) {
  if (B <= 0) return fail(LOCOCO_EINVAL, "block length B must be positive");
  if (B > 65535) return fail(LOCOCO_EUNSUPPORTED, "block length above 65535");
  if ((int64_t)len + B > generic_attn_max_T())
    return fail(LOCOCO_EUNSUPPORTED, "cache.len + B = %lld exceeds the supported %d",
                (long long)len + B, generic_attn_max_T());
  return LOCOCO_OK;
}

// The MFMA kernels address the rows of a block with 32-bit byte offsets inside buffer resources of
// less than 2 GiB (out-of-range rows must read as zero): a block's rows have to span less than that.
lococo_status check_mfma_strides(const lococo_config* c, Path path, const lococo_qkvo* x, int32_t B, bool with_q) {
  if (path == PATH_GENERIC) return LOCOCO_OK;
  const int64_t lim = 0x7fff0000;
  const lococo_tensor* t[4] = {&x->k, &x->v, &x->q, &x->o};
  const char* names[4] = {"k", "v", "q", "o"};
  for (int i = 0; i < (with_q ? 4 : 2); ++i)
    if (((int64_t)B * t[i]->stride_t + c->head_dim) * (int64_t)esize(c->dtype) >= lim)
      return fail(LOCOCO_EUNSUPPORTED, "%s: a block of %d tokens with stride_t %lld spans 2 GiB or more; the MFMA "
                  "kernels address a block's rows with 32-bit offsets (use impl = GENERIC)", names[i], B,
                  (long long)t[i]->stride_t);
  if ((int64_t)c->M * c->head_dim * (int64_t)esize(c->dtype) >= lim)
    return fail(LOCOCO_EUNSUPPORTED, "a chain's cache spans 2 GiB or more");
  return LOCOCO_OK;
}

AttnArgs attn_args_one_block(const StepArgs& a) {
  AttnArgs t;
  std::memset(&t, 0, sizeof(t));
  t.q = a.q; t.k = a.k; t.v = a.v; t.o = a.o;
  t.cache_k = a.cache_k;
  t.cache_v = a.cache_v;
  t.L = a.Bn;
  t.B = a.Bn;
  t.M = a.M;
  t.len0 = a.m;
  t.n_fill = 0;            // block 0 sees the base cache with len0 slots
  t.hist_ring = 1;
  t.seg_first = 0;
  t.n_seg = 1;
  t.batch = a.batch; t.Hq = a.Hq; t.Hkv = a.Hkv; t.group = a.group;
  t.scale = a.scale;
  return t;
}

// Enqueue the attention of one block.  `stats`: room for the block's row statistics (see
// stats_bytes), or null; without it a block whose attention is to be accumulated per slot goes
// to the shape-agnostic kernel.
lococo_status enqueue_attn(const lococo_config* c, Path path, const StepArgs& a, float* stats, hipStream_t s) {
  if (path != PATH_GENERIC && attn_decode_supports(c->dtype, c->head_dim, a.Bn, c->M, a.colsum != nullptr)) {
    KTimer t(K_ATTN_DECODE, s);          // one query row per head: a matrix-vector product
    HIP_TRY(launch_attn_decode(a, s), "attention launch");
    return LOCOCO_OK;
  }
  if (path != PATH_GENERIC && (!a.colsum || stats)) {
    AttnArgs t = attn_args_one_block(a);
    t.stats = a.colsum ? stats : nullptr;
    {
      KTimer kt(K_ATTN_MFMA, s);
      HIP_TRY(launch_attn_mfma(t, s), "attention launch");
    }
    if (a.colsum && a.m > 0) {
      KTimer kt(K_ATTN_COLSUM, s);
      HIP_TRY(launch_attn_colsum_mfma(t, a.colsum, s), "attention column-sum launch");
    }
    return LOCOCO_OK;
  }
  KTimer t(K_ATTN_GENERIC, s);
  HIP_TRY(launch_attn_generic(c->dtype, a, s), "attention launch");
  return LOCOCO_OK;
}

// The statistics area of a step workspace, if the caller passed one that holds it.
float* step_stats(const lococo_config* c, Path path, int32_t B, void* workspace, size_t ws_bytes) {
  if (path == PATH_GENERIC || !workspace || ((uintptr_t)workspace & 255) || ws_bytes < step_ws_bytes(c, path, B))
    return nullptr;
  return (float*)((char*)workspace + (path == PATH_MFMA ? filter_ws_bytes(c) + scan_sync_bytes(c) : packed_ws_bytes(c)));
}

// Repack the filter bank into the workspace (MFMA path; once per call unless the caller says
// the workspace already holds it).
lococo_status enqueue_repack(const lococo_config* c, Path path, const StepArgs& a, void* ws, hipStream_t s) {
  if (c->flags & LOCOCO_FLAG_FILTERS_PREPARED) return LOCOCO_OK;
  KTimer t(K_REPACK, s);
  if (path == PATH_MFMA) HIP_TRY(launch_repack_filters(a, ws, filter_banks(c), s), "filter repack launch");
  else HIP_TRY(launch_pack_filters_per_tap(a, filter_banks(c), ws, s), "filter packing launch");
  return LOCOCO_OK;
}

// Enqueue Eq. 5, Eq. 6 and Eq. 4 of one block: from a.cache_k / a.cache_v (a.m live slots) and the block
// into a.new_k / a.new_v.  `B`: the block length the workspace was laid out for (a.Bn may be a shorter
// last block).
lococo_status enqueue_compress(const lococo_config* c, Path path, StepArgs a, void* ws, int32_t B, hipStream_t s) {
  if (path == PATH_MFMA) {
    KTimer t(K_COMPRESS_MFMA, s);
    HIP_TRY(launch_compress_mfma(a, ws, filter_banks(c), cu_count(), (char*)ws + filter_ws_bytes(c), partials_of(c, ws, B),
                                 prelogits_of(c, ws, B), B, s),
            "compress launch");
    return LOCOCO_OK;
  }
  const bool unfused = path == PATH_MFMA_UNFUSED;
  float* logits = unfused ? (float*)((char*)ws + packed_ws_bytes(c) + stats_bytes(c, B)) : (float*)ws;
  if (unfused) a.ldw = (a.m + a.Bn + 3) / 4 * 4;      // whole groups of four for the MFMA form of Eq. 4
  if (unfused) {
    KTimer t(K_CONV_MFMA, s);
    HIP_TRY(launch_conv_logits_mfma(a, ws, logits, s), "conv launch");
  } else {
    KTimer t(K_CONV_GENERIC, s);
    HIP_TRY(launch_conv_logits_generic(c->dtype, a, logits, s), "conv launch");
  }
  if (a.protect) HIP_TRY(launch_protect_logits_generic(a, logits, s), "protect launch");
  if (unfused && mixnorm_mfma_fits(a, logits)) {       // Eq. 6 inside the mixing kernel: the logits are read once
    {
      KTimer t(K_MIX_MFMA, s);
      HIP_TRY(launch_mixnorm_mfma(a, logits, s), "mix launch");
    }
    if (a.protect) HIP_TRY(launch_protect_rows_generic(c->dtype, a, s), "protect launch");
    return LOCOCO_OK;
  }
  {
    KTimer t(K_NORM_GENERIC, s);
    HIP_TRY(launch_normalise_generic(a, logits, s), "normalise launch");
  }
  if (unfused && mix_mfma_fits(a, logits)) {
    KTimer t(K_MIX_MFMA, s);
    HIP_TRY(launch_mix_mfma(a, logits, s), "mix launch");
  } else {
    KTimer t(K_MIX_GENERIC, s);
    HIP_TRY(launch_mix_generic(c->dtype, a, logits, 0, s), "mix launch");
  }
  if (a.protect) HIP_TRY(launch_protect_rows_generic(c->dtype, a, s), "protect launch");
  return LOCOCO_OK;
}

// Enqueue fill or compress of one block and update the host-side state.
lococo_status enqueue_update(const lococo_config* c, Path path, StepArgs a, lococo_cache* ca,
                             void* ws, int32_t B, hipStream_t s) {
  if (a.m + a.Bn <= a.M) {
    a.new_k = ca->k[ca->cur];
    a.new_v = ca->v[ca->cur];
    KTimer t(K_FILL, s);
    HIP_TRY(launch_fill_generic(c->dtype, a, s), "fill launch");
    ca->len = a.m + a.Bn;
    return LOCOCO_OK;
  }
  a.new_k = ca->k[ca->cur ^ 1];
  a.new_v = ca->v[ca->cur ^ 1];
  lococo_status st = enqueue_compress(c, path, a, ws, B, s);
  if (st) return st;
  ca->cur ^= 1;
  ca->len = a.M;
  return LOCOCO_OK;
}

lococo_status segment_step_impl(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                const void* conv_w, const void* conv_b, lococo_cache* cache,
                                void* workspace, size_t ws_bytes, void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache))) return st;
  if ((st = check_step_shape(cfg, B, cache->len))) return st;
  if ((st = check_qkvo(cfg, blk, B, true))) return st;
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  if ((st = check_mfma_strides(cfg, path, blk, B, true))) return st;
  const bool compress = cache->len + B > cfg->M;
  if (compress) {
    if (!conv_w) return fail(LOCOCO_EINVAL, "conv_w is NULL but this step compresses");
    const size_t need = step_ws_bytes(cfg, path, B);
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)))
      return fail(LOCOCO_EWORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
                  workspace ? ws_bytes : (size_t)0);
  }
  StepArgs a = make_args(cfg, blk, 0, B, cache, conv_w, conv_b, true);
  lococo_cache tmp = *cache;
  if (compress && path != PATH_GENERIC &&
      (st = enqueue_repack(cfg, path, a, workspace, (hipStream_t)stream)))
    return st;
  if ((st = enqueue_attn(cfg, path, a, step_stats(cfg, path, B, workspace, ws_bytes), (hipStream_t)stream)))
    return st;
  if ((st = enqueue_update(cfg, path, a, &tmp, workspace, B, (hipStream_t)stream))) return st;
  *cache = tmp;
  return LOCOCO_OK;
}

// ---- device address of the library's own scratch array on the current device, looked up once per
// device (every device the library runs on holds its own copy at its own address) and used from then
// on wherever host code needs the array's memory
constexpr size_t kScratchBytes = LOCOCO_NOALLOC_SCRATCH_BYTES;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
std::mutex g_scratch_mu;

lococo_status scratch_on_this_device(void** out) {
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(LOCOCO_EUNSUPPORTED, "device index %d above %d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "address of the library's scratch array");
    if (!p || ((uintptr_t)p & 255)) return fail(LOCOCO_EHIP, "the library's scratch array has no usable device address");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return LOCOCO_OK;
}

}  // namespace

extern "C" {

const char* lococo_last_error(void) { return g_err; }
const char* lococo_version(void) { return "0.3.0"; }

lococo_status lococo_debug_option(int32_t option, int64_t value) {
  switch (option) {
    case LOCOCO_OPT_RESET: g_debug = DebugOptions{0, 0, 0, 0, 0, 0, 0}; return LOCOCO_OK;
    case LOCOCO_OPT_SPIN_LIMIT: g_debug.spin_limit = value; return LOCOCO_OK;
    case LOCOCO_OPT_SCAN_PER_STEP: g_debug.scan_per_step = value != 0; return LOCOCO_OK;
    case LOCOCO_OPT_CHAIN_SYNC_DEVICE: g_debug.chain_sync_device = value != 0; return LOCOCO_OK;
    case LOCOCO_OPT_LOGITS_TILES:
      if (value != 0 && value != 64 && value != 128 && value != 256)
        return fail(LOCOCO_EINVAL, "LOCOCO_OPT_LOGITS_TILES takes 0, 64, 128 or 256");
      g_debug.logits_tiles = value;
      return LOCOCO_OK;
    case LOCOCO_OPT_MAX_RESIDENT:
      if (value < 0) return fail(LOCOCO_EINVAL, "LOCOCO_OPT_MAX_RESIDENT takes a count >= 0");
      g_debug.max_resident = value;
      return LOCOCO_OK;
    case LOCOCO_OPT_UNFUSED_KV:
      if (value != 0 && value != 1) return fail(LOCOCO_EINVAL, "LOCOCO_OPT_UNFUSED_KV takes 0 or 1");
      g_debug.unfused_kv = value;
      return LOCOCO_OK;
    case LOCOCO_OPT_NO_STEP_PIPELINE:
      if (value != 0 && value != 1) return fail(LOCOCO_EINVAL, "LOCOCO_OPT_NO_STEP_PIPELINE takes 0 or 1");
      g_debug.no_step_pipeline = value;
      return LOCOCO_OK;
    default: return fail(LOCOCO_EINVAL, "unknown debug option %d", option);
  }
}

lococo_status lococo_describe_path(const lococo_config* cfg, int32_t B, lococo_path_info* out) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!out) return fail(LOCOCO_EINVAL, "out is NULL");
  if (B <= 0) return fail(LOCOCO_EINVAL, "block length B must be positive");
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  std::memset(out, 0, sizeof(*out));
  out->path = (int32_t)path;
  out->compute_units = cu_count();
  if (path == PATH_MFMA) {
    out->tile_slots = compress_tile_slots(cfg->batch, cfg->n_kv_heads, cfg->M, cfg->conv_width, cfg->conv_in, cu_count());
    out->position_split = compress_position_split(cfg->batch, cfg->n_kv_heads, cfg->M, cfg->conv_width, cfg->conv_in, cu_count());
    out->step_pipeline = compress_step_pipeline(cfg->batch, cfg->n_kv_heads, cfg->M, cfg->conv_width, cfg->conv_in, cu_count());
    StepArgs a;
    std::memset(&a, 0, sizeof(a));
    a.batch = cfg->batch; a.Hkv = cfg->n_kv_heads; a.M = cfg->M; a.k_width = cfg->conv_width; a.norm = cfg->norm;
    a.conv_in = cfg->conv_in;
    a.w_head_stride = cfg->w_head_stride; a.b_head_stride = cfg->b_head_stride;
    out->scan_resident_limit = compress_scan_max_resident(a, cu_count());
    if (scan_fits_one_launch(cfg, a))
      out->scan_groups = compress_scan_groups(cfg->batch, cfg->n_kv_heads, cfg->M, cfg->conv_width, cfg->conv_in,
                                              cfg->w_head_stride != 0 || cfg->b_head_stride != 0, cu_count());
  }
  return LOCOCO_OK;
}

lococo_status lococo_scan_status(const lococo_config* cfg, const void* workspace, int32_t* out) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!workspace || !out) return fail(LOCOCO_EINVAL, "workspace or out is NULL");
  Path path;
  if ((st = resolve_path(cfg, 1, &path))) return st;
  if (path != PATH_MFMA) {
    *out = 0;
    return LOCOCO_OK;
  }
  const char* word = (const char*)workspace + filter_ws_bytes(cfg) +
                     (size_t)cfg->batch * cfg->n_kv_heads * sizeof(uint32_t);
  HIP_TRY(hipMemcpy(out, word, sizeof(int32_t), hipMemcpyDeviceToHost), "reading the scan status");
  return LOCOCO_OK;
}

lococo_status lococo_measure_peaks(void* scratch, size_t bytes, void* stream, double* mfma_tflops,
                                   double* copy_gbs) {
  if (!scratch || !mfma_tflops || !copy_gbs) return fail(LOCOCO_EINVAL, "null argument");
  if ((uintptr_t)scratch & 15) return fail(LOCOCO_EINVAL, "scratch must be 16-byte aligned");
  if (bytes < ((size_t)32 << 20)) return fail(LOCOCO_EINVAL, "scratch must hold at least 32 MiB (got %zu bytes)", bytes);
  HIP_TRY(measure_peaks(scratch, bytes, cu_count(), (hipStream_t)stream, mfma_tflops, copy_gbs),
          "peak measurement");
  return LOCOCO_OK;
}

lococo_status lococo_timing_begin(void) {
  std::lock_guard<std::mutex> lk(g_timing_mu);
  for (auto& t : g_timed) {
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  g_timed.clear();
  g_timing_on = true;
  return LOCOCO_OK;
}

lococo_status lococo_timing_end(lococo_kernel_time* out, int32_t* n_inout) {
  if (!n_inout) return fail(LOCOCO_EINVAL, "n_inout is NULL");
  std::lock_guard<std::mutex> lk(g_timing_mu);
  g_timing_on = false;
  int64_t launches[K_COUNT] = {0};
  double ms[K_COUNT] = {0.0};
  lococo_status st = LOCOCO_OK;
  for (auto& t : g_timed) {
    float dt = 0.f;
    hipError_t e = hipEventSynchronize(t.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&dt, t.start, t.stop);
    if (e != hipSuccess && st == LOCOCO_OK) st = hip_fail(e, "timing events");
    launches[t.id] += 1;
    ms[t.id] += dt;
    (void)hipEventDestroy(t.start);
    (void)hipEventDestroy(t.stop);
  }
  g_timed.clear();
  const int32_t cap = out ? *n_inout : 0;
  int32_t n = 0;
  for (int id = 0; id < K_COUNT; ++id) {
    if (!launches[id]) continue;
    if (n < cap) out[n] = lococo_kernel_time{kKernelNames[id], launches[id], ms[id]};
    ++n;
  }
  *n_inout = n;
  return st;
}

lococo_status lococo_plan(int64_t L, int32_t B, int32_t M, int32_t len0, int32_t cur0,
                          lococo_seg* out, int64_t* n_inout) {
  if (!n_inout) return fail(LOCOCO_EINVAL, "n_inout is NULL");
  if (L < 0 || B <= 0 || M <= 0) return fail(LOCOCO_EINVAL, "need L >= 0, B > 0, M > 0");
  if (len0 < 0 || len0 > M) return fail(LOCOCO_ESTATE, "len0 %d is outside [0, M=%d]", len0, M);
  if (cur0 != 0 && cur0 != 1) return fail(LOCOCO_ESTATE, "cur0 must be 0 or 1");
  const int64_t cap = out ? *n_inout : 0;
  if (cap < 0) return fail(LOCOCO_EINVAL, "negative capacity");
  const int64_t n = (L + B - 1) / B;
  int32_t occ = len0, buf = cur0;
  for (int64_t i = 0; i < n; ++i) {
    const int64_t start = i * B;
    const int32_t len = (int32_t)std::min<int64_t>(B, L - start);
    const bool fits = (int64_t)occ + len <= M;
    const int32_t occ_after = fits ? occ + len : M;
    if (!fits) buf = 1 - buf;
    if (i < cap) out[i] = lococo_seg{start, len, fits ? 0 : 1, occ, occ_after, buf, 0};
    occ = occ_after;
  }
  *n_inout = n;
  return LOCOCO_OK;
}

lococo_status lococo_workspace_bytes(const lococo_config* cfg, int64_t L, int32_t B,
                                     int32_t history, size_t* out) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!out) return fail(LOCOCO_EINVAL, "out is NULL");
  if (L < 0 || B <= 0) return fail(LOCOCO_EINVAL, "need L >= 0 and B > 0");
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  const int64_t n_blocks = (L + B - 1) / B;
  if (history < 0) return fail(LOCOCO_EINVAL, "history must be >= 0");
  if (history == 0 || path == PATH_GENERIC || n_blocks == 0)
    *out = step_ws_bytes(cfg, path, B);
  else if (history == 1 || history >= n_blocks)
    *out = history_ws_bytes(cfg, path, B, n_blocks, L);             // every block may compress
  else {
    const int64_t g = std::max<int64_t>(history, 2);
    *out = history_ws_bytes(cfg, path, B, g + 1, g * (int64_t)B);   // a window of g blocks: g + 1 states
  }
  return LOCOCO_OK;
}

lococo_status lococo_attn_only(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                               const lococo_cache* cache, void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache))) return st;
  if ((st = check_step_shape(cfg, B, cache->len))) return st;
  if ((st = check_qkvo(cfg, blk, B, true))) return st;
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  if ((st = check_mfma_strides(cfg, path, blk, B, true))) return st;
  StepArgs a = make_args(cfg, blk, 0, B, cache, nullptr, nullptr, true);
  return enqueue_attn(cfg, path, a, nullptr, (hipStream_t)stream);
}

lococo_status lococo_prepare_filters(const lococo_config* cfg, const void* conv_w, void* workspace,
                                     size_t ws_bytes, void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!conv_w) return fail(LOCOCO_EINVAL, "conv_w is NULL");
  Path path;
  if ((st = resolve_path(cfg, 1, &path))) return st;
  if (path == PATH_GENERIC) return LOCOCO_OK;    // the shape-agnostic kernels read [M, C, k] as given
  const size_t need = path == PATH_MFMA ? filter_ws_bytes(cfg) : packed_ws_bytes(cfg);
  if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))
    return fail(LOCOCO_EWORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
                workspace ? ws_bytes : (size_t)0);
  StepArgs a{};
  a.conv_w = conv_w;
  a.w_head_stride = cfg->w_head_stride;
  a.M = cfg->M;
  a.k_width = cfg->conv_width;
  a.conv_in = cfg->conv_in;
  lococo_config once = *cfg;
  once.flags &= ~LOCOCO_FLAG_FILTERS_PREPARED;
  return enqueue_repack(&once, path, a, workspace, (hipStream_t)stream);
}

lococo_status lococo_segment_step(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                  const void* conv_w, const void* conv_b, lococo_cache* cache,
                                  void* workspace, size_t ws_bytes, void* stream) {
  return segment_step_impl(cfg, blk, B, conv_w, conv_b, cache, workspace, ws_bytes, stream);
}

lococo_status lococo_segment_step_noalloc(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                          const void* conv_w, const void* conv_b, lococo_cache* cache,
                                          void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (cfg->flags & LOCOCO_FLAG_FILTERS_PREPARED)
    return fail(LOCOCO_EINVAL, "LOCOCO_FLAG_FILTERS_PREPARED cannot be used with the library's own scratch "
                "array: every caller on the device shares it, so nothing prepared can be assumed to be there");
  if (B <= 0) return fail(LOCOCO_EINVAL, "block length B must be positive");
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  const size_t need = step_ws_bytes(cfg, path, B);
  if (need > kScratchBytes)
    return fail(LOCOCO_EWORKSPACE, "this step needs %zu bytes of scratch, the library's own array holds %zu: "
                "use lococo_segment_step with a workspace of the caller's", need, kScratchBytes);
  void* ws = nullptr;
  if ((st = scratch_on_this_device(&ws))) return st;
  return segment_step_impl(cfg, blk, B, conv_w, conv_b, cache, ws, kScratchBytes, stream);
}

lococo_status lococo_sequence_forward(const lococo_config* cfg, const lococo_qkvo* seq, int64_t L,
                                      int32_t B, const void* conv_w, const void* conv_b,
                                      lococo_cache* cache, void* workspace, size_t ws_bytes,
                                      void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache))) return st;
  if (L < 0) return fail(LOCOCO_EINVAL, "L must be >= 0");
  if (B <= 0) return fail(LOCOCO_EINVAL, "block length B must be positive");
  if (L == 0) return LOCOCO_OK;  // nothing to do; tensors may be empty
  if ((st = check_step_shape(cfg, B, std::min<int64_t>(cfg->M, (int64_t)cache->len + L))))
    return st;
  if ((st = check_qkvo(cfg, seq, L, true))) return st;
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  int64_t n = 0;
  if ((st = lococo_plan(L, B, cfg->M, cache->len, cache->cur, nullptr, &n))) return st;
  std::vector<lococo_seg> plan((size_t)n);
  if (n && (st = lococo_plan(L, B, cfg->M, cache->len, cache->cur, plan.data(), &n))) return st;
  bool any_compress = false;
  for (const auto& sg : plan) any_compress |= sg.branch == 1;
  if (any_compress) {
    if (!conv_w) return fail(LOCOCO_EINVAL, "conv_w is NULL but the scan compresses");
    const size_t need = step_ws_bytes(cfg, path, B);
    if (need && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)))
      return fail(LOCOCO_EWORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", need,
                  workspace ? ws_bytes : (size_t)0);
  }
  lococo_cache tmp = *cache;
  if (any_compress && path != PATH_GENERIC) {
    StepArgs a0 = make_args(cfg, seq, 0, B, &tmp, conv_w, conv_b, true);
    if ((st = enqueue_repack(cfg, path, a0, workspace, (hipStream_t)stream))) return st;
  }
  if (path == PATH_MFMA && workspace && ws_bytes >= step_ws_bytes(cfg, path, B)) {
    // the scan status of this call starts at "no wait gave up", whichever schedule runs
    HIP_TRY(launch_scan_sync_clear((char*)workspace + filter_ws_bytes(cfg), cfg->batch, cfg->n_kv_heads, cfg->M, false,
                                   (hipStream_t)stream), "clearing the scan counters");
  }
  int64_t n_compress = 0;
  for (const auto& sg : plan) n_compress += sg.branch;
  // Batched-attention schedules: run the fill / compress recurrence of a window of blocks first,
  // keeping the cache state after each of them in a ring of history slots, then one attention
  // launch over the window's blocks.  The window is the whole sequence when the workspace holds
  // every state, otherwise as many blocks as it holds (at least two: a ring of G + 1 slots serves a
  // window of G blocks, the extra one being the state the window starts from); memory then stays
  // independent of the sequence length, as in the step-by-step schedule.
  int64_t window = 0, ring = 0;
  if (path != PATH_GENERIC && any_compress && workspace) {
    if (ws_bytes >= history_ws_bytes(cfg, path, B, n_compress, L)) {
      window = n;
      ring = n_compress;
    } else {
      for (int64_t g = std::min<int64_t>(n, 4096); g >= 2; --g)
        if (ws_bytes >= history_ws_bytes(cfg, path, B, g + 1, g * (int64_t)B)) { window = g; ring = g + 1; break; }
    }
  }
  if (window > 0) {
    hipStream_t s = (hipStream_t)stream;
    const size_t slot = align_up(state_bytes(cfg), 256);
    const int64_t window_rows = std::min<int64_t>(L, window * (int64_t)B);
    char* sync_ws = (char*)workspace + filter_ws_bytes(cfg);      // fused path only
    float* win_stats = (float*)((char*)workspace + step_ws_bytes(cfg, path, B));
    char* hist_k = (char*)win_stats + stats_bytes(cfg, window_rows);
    char* hist_v = hist_k + (size_t)ring * slot;
    const int64_t hist_stride = (int64_t)(slot / esize(cfg->dtype));
    auto slot_k = [&](int64_t c) { return hist_k + (size_t)(c % ring) * slot; };
    auto slot_v = [&](int64_t c) { return hist_v + (size_t)(c % ring) * slot; };
    bool one_launch = false;
    if (path == PATH_MFMA) {
      StepArgs probe = make_args(cfg, seq, 0, B, &tmp, conv_w, conv_b, true);
      one_launch = scan_fits_one_launch(cfg, probe);
    }
    int64_t c_done = 0;                       // compress steps enqueued so far: state c_done - 1 is the newest
    for (int64_t w0 = 0; w0 < n; w0 += window) {
      const int64_t w1 = std::min<int64_t>(n, w0 + window);
      // the state the window starts from: the caller's live buffer until the first compression
      const int64_t c0 = c_done;
      const void* base_k = c0 == 0 ? tmp.k[tmp.cur] : slot_k(c0 - 1);
      const void* base_v = c0 == 0 ? tmp.v[tmp.cur] : slot_v(c0 - 1);
      int64_t fills = 0;                      // fill blocks at the head of the window
      while (w0 + fills < w1 && plan[(size_t)(w0 + fills)].branch == 0) ++fills;
      for (int64_t bi = w0; bi < w1; ++bi) {
        const lococo_seg& sg = plan[(size_t)bi];
        StepArgs a = make_args(cfg, seq, sg.start, sg.len, &tmp, conv_w, conv_b, true);
        a.m = sg.len_before;
        if (sg.branch == 0) {
          a.new_k = tmp.k[tmp.cur];
          a.new_v = tmp.v[tmp.cur];
          KTimer t(K_FILL, s);
          HIP_TRY(launch_fill_generic(cfg->dtype, a, s), "fill launch");
          continue;
        }
        a.cache_k = c_done == 0 ? tmp.k[tmp.cur] : slot_k(c_done - 1);
        a.cache_v = c_done == 0 ? tmp.v[tmp.cur] : slot_v(c_done - 1);
        if (one_launch) {
          // every later block of the window compresses too (the cache stays full): one launch runs
          // them all, the slot tiles of a chain handing the new cache to each other through the ring
          const bool capturing = stream_is_capturing(s);
          std::unique_lock<std::mutex> lk(g_scan_mu);
          if (!capturing && another_scan_in_flight(s)) {
            one_launch = false;          // another persistent scan holds compute units: one launch per step
          } else {
            if (c_done > 0)              // the counters start every launch at zero; the status word is kept
              HIP_TRY(launch_scan_sync_clear(sync_ws, cfg->batch, cfg->n_kv_heads, cfg->M, true, s), "clearing the scan counters");
            ScanArgs sa;
            sa.st = a;
            sa.n_steps = (int32_t)(w1 - bi);
            sa.B = B;
            sa.tokens_left = L - sg.start;
            sa.out_k = hist_k;
            sa.out_v = hist_v;
            sa.out_stride = hist_stride;
            sa.slot0 = (int32_t)(c_done % ring);
            sa.ring = (int32_t)ring;
            sa.sync = nullptr;
            sa.status = nullptr;
            sa.spin_limit = spin_limit();
            sa.same_l2_allowed = chain_sync_through_l2() ? 1 : 0;
            {
              KTimer t(K_COMPRESS_MFMA, s);
              HIP_TRY(launch_compress_scan(sa, workspace, filter_banks(cfg), cu_count(), sync_ws,
                                           partials_of(cfg, workspace, B), prelogits_of(cfg, workspace, B), s),
                      "compress scan launch");
            }
            if (!capturing) note_scan_launched(s);
            c_done += w1 - bi;
            break;
          }
        }
        a.new_k = slot_k(c_done);
        a.new_v = slot_v(c_done);
        if ((st = enqueue_compress(cfg, path, a, workspace, B, s))) return st;
        ++c_done;
      }
      // A block of one token (every block when B = 1, else a ragged last block) goes to the kernel of the
      // generation stage here as in the step-by-step schedule: which kernel a block's attention runs on depends on
      // the block, never on the schedule, so the bits do not either.  Such blocks can only end a window, and they
      // come after the window's other blocks, as they do in time (the order matters to sums kept per slot).
      int64_t w_batched = w1;
      while (w_batched > w0 && path != PATH_GENERIC &&
             attn_decode_supports(cfg->dtype, cfg->head_dim, plan[(size_t)(w_batched - 1)].len, cfg->M,
                                  cache->attn_colsum != nullptr))
        --w_batched;
      if (w_batched > w0) {
        const lococo_seg& first = plan[(size_t)w0];
        StepArgs a0 = make_args(cfg, seq, first.start, B, &tmp, conv_w, conv_b, true);
        AttnArgs t = attn_args_one_block(a0);
        t.cache_k = base_k;
        t.cache_v = base_v;
        t.hist_k = hist_k;
        t.hist_v = hist_v;
        t.hist_stride = hist_stride;
        t.hist_first = (int32_t)(c0 % ring);
        t.hist_ring = (int32_t)ring;
        t.L = std::min<int64_t>(L - first.start, (w_batched - w0) * (int64_t)B);
        t.B = B;
        t.len0 = first.len_before;
        t.n_fill = (int32_t)std::min<int64_t>(fills, w_batched - w0);
        t.n_seg = (int32_t)(w_batched - w0);
        t.stats = cache->attn_colsum ? win_stats : nullptr;
        {
          KTimer kt(K_ATTN_MFMA, s);
          HIP_TRY(launch_attn_mfma(t, s), "attention launch");
        }
        if (cache->attn_colsum) {           // sums over blocks commute: one launch for all of the window's
          KTimer kt(K_ATTN_COLSUM, s);
          HIP_TRY(launch_attn_colsum_mfma(t, cache->attn_colsum, s), "attention column-sum launch");
        }
      }
      if (w_batched < w1) {
        int64_t c_before = c0;                  // compress steps ahead of block bi
        for (int64_t bi = w0; bi < w1; ++bi) {
          const lococo_seg& sg = plan[(size_t)bi];
          if (bi >= w_batched) {
            StepArgs a = make_args(cfg, seq, sg.start, sg.len, &tmp, conv_w, conv_b, true);
            a.m = sg.len_before;
            a.cache_k = c_before == 0 ? tmp.k[tmp.cur] : slot_k(c_before - 1);
            a.cache_v = c_before == 0 ? tmp.v[tmp.cur] : slot_v(c_before - 1);
            KTimer kt(K_ATTN_DECODE, s);
            HIP_TRY(launch_attn_decode(a, s), "attention launch");
          }
          if (sg.branch != 0) ++c_before;
        }
      }
    }
    const lococo_seg& last = plan.back();
    if (c_done > 0) {
      HIP_TRY(launch_copy_pair(tmp.k[last.buf_after], slot_k(c_done - 1), tmp.v[last.buf_after], slot_v(c_done - 1),
                               state_bytes(cfg), s),
              "publishing the final cache");
    }
    tmp.cur = last.buf_after;
    tmp.len = last.len_after;
    *cache = tmp;
    return LOCOCO_OK;
  }
  for (const auto& sg : plan) {
    StepArgs a = make_args(cfg, seq, sg.start, sg.len, &tmp, conv_w, conv_b, true);
    if ((st = enqueue_attn(cfg, path, a, step_stats(cfg, path, B, workspace, ws_bytes), (hipStream_t)stream)))
      return st;
    if ((st = enqueue_update(cfg, path, a, &tmp, workspace, B, (hipStream_t)stream))) return st;
  }
  *cache = tmp;
  return LOCOCO_OK;
}

namespace {
// the Eq. 5 contractions of the backward pass run on MFMA unless the shape-agnostic kernels are asked for
bool bwd_on_mfma(const lococo_config* c) {
  return c->impl != LOCOCO_IMPL_GENERIC && bwd_mfma_supports(c->dtype, c->head_dim, c->conv_in, c->conv_width);
}
struct BwdLayout { size_t p, ds, w, n, dw, mf, total; };
BwdLayout bwd_layout(const lococo_config* c, int32_t B, int32_t len) {
  const size_t T = (size_t)len + B;
  const size_t rows = (size_t)c->batch * c->n_q_heads * B * T * sizeof(float);
  const bool compress = len + B > c->M;
  const size_t mat = compress ? (size_t)c->batch * c->n_kv_heads * c->M * T * sizeof(float) : 0;
  BwdLayout l;
  l.p = 0;
  l.ds = align_up(rows, 256);
  l.w = l.ds + align_up(rows, 256);
  l.n = l.w + align_up(mat, 256);
  l.dw = l.n + align_up(mat, 256);
  l.mf = l.dw + align_up(mat, 256);
  l.total = l.mf;
  if (compress && bwd_on_mfma(c))
    l.total += bwd_mfma_layout(c->batch, c->n_kv_heads, c->M, (int)T, c->conv_width, c->conv_in, filter_banks(c)).total;
  return l;
}
}  // namespace

lococo_status lococo_backward_workspace_bytes(const lococo_config* cfg, int32_t B, int32_t len, size_t* out) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!out) return fail(LOCOCO_EINVAL, "out is NULL");
  if (B <= 0 || len < 0 || len > cfg->M) return fail(LOCOCO_EINVAL, "B must be positive and len in [0, M]");
  *out = bwd_layout(cfg, B, len).total;
  return LOCOCO_OK;
}

lococo_status lococo_segment_step_backward(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                           const void* conv_w, const void* conv_b,
                                           const lococo_cache* cache_before, const float* d_o,
                                           const float* d_new_k, const float* d_new_v, float* d_q,
                                           float* d_k, float* d_v, float* d_cache_k, float* d_cache_v,
                                           float* d_conv_w, float* d_conv_b, void* workspace,
                                           size_t ws_bytes, void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache_before))) return st;
  if ((st = check_step_shape(cfg, B, cache_before->len))) return st;
  if (!blk) return fail(LOCOCO_EINVAL, "qkvo is NULL");
  if ((st = check_tensor(cfg, blk->q, "q", B)) || (st = check_tensor(cfg, blk->k, "k", B)) ||
      (st = check_tensor(cfg, blk->v, "v", B)))
    return st;
  if (!d_o || !d_new_k || !d_new_v || !d_q || !d_k || !d_v || !d_cache_k || !d_cache_v)
    return fail(LOCOCO_EINVAL, "a gradient pointer is NULL");
  if (cfg->norm == 2) return fail(LOCOCO_EUNSUPPORTED, "norm = 2 (rectifier on the convolution input) is forward only");
  const bool compress = cache_before->len + B > cfg->M;
  if (compress && (!conv_w || !d_conv_w))
    return fail(LOCOCO_EINVAL, "conv_w or d_conv_w is NULL but the step compresses");
  const BwdLayout l = bwd_layout(cfg, B, cache_before->len);
  if (!workspace || ws_bytes < l.total || ((uintptr_t)workspace & 255))
    return fail(LOCOCO_EWORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", l.total,
                workspace ? ws_bytes : (size_t)0);
  hipStream_t s = (hipStream_t)stream;
  lococo_qkvo x = *blk;
  x.o = x.q;                                  // not read; keeps make_args' view arithmetic defined
  BwdArgs g;
  g.st = make_args(cfg, &x, 0, B, cache_before, conv_w, conv_b, true);
  g.d_o = d_o;
  g.d_new_k = d_new_k;
  g.d_new_v = d_new_v;
  g.d_q = d_q;
  g.d_k = d_k;
  g.d_v = d_v;
  g.d_cache_k = d_cache_k;
  g.d_cache_v = d_cache_v;
  g.d_conv_w = d_conv_w;
  g.d_conv_b = d_conv_b;
  char* ws = (char*)workspace;
  g.ws_p = (float*)(ws + l.p);
  g.ws_ds = (float*)(ws + l.ds);
  g.ws_w = (float*)(ws + l.w);
  g.ws_n = (float*)(ws + l.n);
  g.ws_dw = (float*)(ws + l.dw);
  g.ws_mfma = compress && bwd_on_mfma(cfg) ? ws + l.mf : nullptr;
  g.banks = filter_banks(cfg);
  g.gemms_mfma = cfg->impl != LOCOCO_IMPL_GENERIC && cfg->dtype == LOCOCO_BF16 ? 1 : 0;
  if (compress) {
    // recompute Eq. 5 and Eq. 6 of the forward step: raw logits and normalised rows
    if (g.ws_mfma) {
      HIP_TRY(launch_pack_filters_per_tap(g.st, g.banks, g.ws_mfma, s), "filter packing launch");
      HIP_TRY(launch_conv_logits_mfma(g.st, g.ws_mfma, g.ws_w, s), "conv launch");
    } else {
      HIP_TRY(launch_conv_logits_generic(cfg->dtype, g.st, g.ws_w, s), "conv launch");
    }
    if (g.st.protect) HIP_TRY(launch_protect_logits_generic(g.st, g.ws_w, s), "protect launch");
    const size_t mat = (size_t)cfg->batch * cfg->n_kv_heads * cfg->M * ((size_t)cache_before->len + B) *
                       sizeof(float);
    HIP_TRY(hipMemcpyAsync(g.ws_n, g.ws_w, mat, hipMemcpyDeviceToDevice, s), "copying the logits");
    HIP_TRY(launch_normalise_generic(g.st, g.ws_n, s), "normalise launch");
  }
  HIP_TRY(launch_step_backward_generic(cfg->dtype, g, compress, s), "backward launches");
  return LOCOCO_OK;
}

lococo_status lococo_mix_from_logits(const lococo_config* cfg, const lococo_qkvo* blk, int32_t B,
                                     const float* logits, lococo_cache* cache, void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache))) return st;
  if ((st = check_step_shape(cfg, B, cache->len))) return st;
  if ((st = check_qkvo(cfg, blk, B, false))) return st;
  if (!logits) return fail(LOCOCO_EINVAL, "logits is NULL");
  if (cache->protect)
    return fail(LOCOCO_EUNSUPPORTED, "lococo_mix_from_logits does not take protected slots");
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  if ((st = check_mfma_strides(cfg, path, blk, B, false))) return st;
  StepArgs a = make_args(cfg, blk, 0, B, cache, nullptr, nullptr, false);
  a.new_k = cache->k[cache->cur ^ 1];
  a.new_v = cache->v[cache->cur ^ 1];
  // bf16 / head_dim 128 unless the shape-agnostic kernels are asked for: Eq. 6 and Eq. 4 on the matrix
  // cores (the kernel of the unfused MFMA path), which needs rows of logits that start 16-byte aligned
  if (path != PATH_GENERIC && mixnorm_mfma_fits(a, logits)) {
    KTimer t(K_MIX_MFMA, (hipStream_t)stream);
    HIP_TRY(launch_mixnorm_mfma(a, logits, (hipStream_t)stream), "mix launch");
  } else {
    KTimer t(K_MIX_GENERIC, (hipStream_t)stream);
    HIP_TRY(launch_mix_generic(cfg->dtype, a, logits, 1, (hipStream_t)stream), "mix launch");
  }
  cache->cur ^= 1;
  cache->len = cfg->M;
  return LOCOCO_OK;
}

}  // extern "C"

// ---- backward of a whole scan: the forward recurrence is run once more to keep the state every block
// started from, then the blocks are walked in reverse, each through lococo_segment_step_backward
namespace {
struct SeqBwdLayout {
  size_t cache[4];        // ping-pong buffers of the recomputed forward: k0, k1, v0, v1 (storage type)
  size_t states_k, states_v, state;   // the state BEFORE every block: n_blocks slots of `state` bytes each
  size_t o_blk;           // attention output of one block of the recomputed forward (storage type; discarded)
  size_t fwd_ws, fwd_ws_bytes;        // step workspace of the recomputed forward
  size_t d_o, d_q, d_k, d_v;          // one block of gradients, contiguous fp32
  size_t g[2][2];         // gradient w.r.t. the cache state, ping-pong: [which][k, v], fp32 [chains, M, d]
  size_t step_ws;         // workspace of one backward step
  size_t total;
};
lococo_status seq_bwd_layout(const lococo_config* c, int64_t L, int32_t B, SeqBwdLayout* out) {
  SeqBwdLayout l;
  size_t at = 0;
  auto take = [&](size_t bytes) { const size_t here = at; at += align_up(bytes, 256); return here; };
  const size_t chains = (size_t)c->batch * c->n_kv_heads, es = esize(c->dtype);
  l.state = align_up(chains * c->M * c->head_dim * es, 256);
  const int64_t n = (L + B - 1) / B;
  for (int i = 0; i < 4; ++i) l.cache[i] = take(l.state);
  l.states_k = take((size_t)n * l.state);
  l.states_v = take((size_t)n * l.state);
  l.o_blk = take((size_t)c->batch * c->n_q_heads * B * c->head_dim * es);
  Path path;
  lococo_status st = resolve_path(c, B, &path);
  if (st) return st;
  l.fwd_ws_bytes = step_ws_bytes(c, path, B);
  l.fwd_ws = take(l.fwd_ws_bytes);
  l.d_o = take((size_t)c->batch * c->n_q_heads * B * c->head_dim * sizeof(float));
  l.d_q = take((size_t)c->batch * c->n_q_heads * B * c->head_dim * sizeof(float));
  l.d_k = take(chains * B * c->head_dim * sizeof(float));
  l.d_v = take(chains * B * c->head_dim * sizeof(float));
  for (int w = 0; w < 2; ++w)
    for (int kv = 0; kv < 2; ++kv) l.g[w][kv] = take(chains * c->M * c->head_dim * sizeof(float));
  size_t step = 0;                    // a step's workspace grows with the occupancy: the full cache bounds all
  if ((st = lococo_backward_workspace_bytes(c, B, c->M, &step))) return st;
  l.step_ws = take(step);
  l.total = at;
  *out = l;
  return LOCOCO_OK;
}
}  // namespace

extern "C" {

lococo_status lococo_sequence_backward_workspace_bytes(const lococo_config* cfg, int64_t L, int32_t B, size_t* out) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if (!out) return fail(LOCOCO_EINVAL, "out is NULL");
  if (L < 0 || B <= 0) return fail(LOCOCO_EINVAL, "need L >= 0 and B > 0");
  SeqBwdLayout l;
  if ((st = seq_bwd_layout(cfg, L, B, &l))) return st;
  *out = l.total;
  return LOCOCO_OK;
}

lococo_status lococo_sequence_backward(const lococo_config* cfg, const lococo_qkvo* seq, int64_t L, int32_t B,
                                       const void* conv_w, const void* conv_b, const lococo_cache* cache0,
                                       const float* d_o, const float* d_final_k, const float* d_final_v,
                                       float* d_q, float* d_k, float* d_v, float* d_cache0_k, float* d_cache0_v,
                                       float* d_conv_w, float* d_conv_b, void* workspace, size_t ws_bytes,
                                       void* stream) {
  lococo_status st;
  if ((st = check_config(cfg))) return st;
  if ((st = check_cache(cfg, cache0))) return st;
  if (L <= 0) return fail(LOCOCO_EINVAL, "L must be positive");
  if (B <= 0) return fail(LOCOCO_EINVAL, "block length B must be positive");
  if (cfg->norm == 2) return fail(LOCOCO_EUNSUPPORTED, "norm = 2 (rectifier on the convolution input) is forward only");
  if (!seq) return fail(LOCOCO_EINVAL, "qkvo is NULL");
  if ((st = check_tensor(cfg, seq->q, "q", L)) || (st = check_tensor(cfg, seq->k, "k", L)) ||
      (st = check_tensor(cfg, seq->v, "v", L)))
    return st;
  if ((st = check_step_shape(cfg, B, std::min<int64_t>(cfg->M, (int64_t)cache0->len + L)))) return st;
  if (!d_o || !d_q || !d_k || !d_v || !d_cache0_k || !d_cache0_v) return fail(LOCOCO_EINVAL, "a gradient pointer is NULL");
  if (cfg->flags & LOCOCO_FLAG_FILTERS_PREPARED)
    return fail(LOCOCO_EINVAL, "LOCOCO_FLAG_FILTERS_PREPARED has no meaning here: the call uses workspaces of its own");
  int64_t n = 0;
  if ((st = lococo_plan(L, B, cfg->M, cache0->len, 0, nullptr, &n))) return st;
  std::vector<lococo_seg> plan((size_t)n);
  if ((st = lococo_plan(L, B, cfg->M, cache0->len, 0, plan.data(), &n))) return st;
  bool any_compress = false;
  for (const auto& sg : plan) any_compress |= sg.branch == 1;
  if (any_compress && (!conv_w || !d_conv_w)) return fail(LOCOCO_EINVAL, "conv_w or d_conv_w is NULL but the scan compresses");
  SeqBwdLayout l;
  if ((st = seq_bwd_layout(cfg, L, B, &l))) return st;
  if (!workspace || ws_bytes < l.total || ((uintptr_t)workspace & 255))
    return fail(LOCOCO_EWORKSPACE, "workspace needs %zu bytes, 256-byte aligned (got %zu)", l.total,
                workspace ? ws_bytes : (size_t)0);
  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const size_t es = esize(cfg->dtype), d = (size_t)cfg->head_dim;
  const size_t chains = (size_t)cfg->batch * cfg->n_kv_heads, state = chains * cfg->M * d * es;

  // ---- the recurrence once more, block by block, keeping the state every block starts from: the fill
  // branch or steps 4-5 only (the same kernels as in lococo_segment_step, so the same states); nobody reads
  // the attention outputs of step 3 here
  Path path;
  if ((st = resolve_path(cfg, B, &path))) return st;
  if ((st = check_mfma_strides(cfg, path, seq, B, false))) return st;
  bool filters_ready = false;
  lococo_cache fc = *cache0;
  fc.k[0] = ws + l.cache[0]; fc.k[1] = ws + l.cache[1];
  fc.v[0] = ws + l.cache[2]; fc.v[1] = ws + l.cache[3];
  fc.cur = 0;
  fc.attn_colsum = nullptr;
  HIP_TRY(hipMemcpyAsync(fc.k[0], cache0->k[cache0->cur], state, hipMemcpyDeviceToDevice, s), "copying the first state");
  HIP_TRY(hipMemcpyAsync(fc.v[0], cache0->v[cache0->cur], state, hipMemcpyDeviceToDevice, s), "copying the first state");
  for (int64_t i = 0; i < n; ++i) {
    const lococo_seg& sg = plan[(size_t)i];
    HIP_TRY(hipMemcpyAsync(ws + l.states_k + (size_t)i * l.state, fc.k[fc.cur], state, hipMemcpyDeviceToDevice, s), "keeping a state");
    HIP_TRY(hipMemcpyAsync(ws + l.states_v + (size_t)i * l.state, fc.v[fc.cur], state, hipMemcpyDeviceToDevice, s), "keeping a state");
    if (i + 1 == n) break;                                   // the last block's own update is not needed
    lococo_qkvo blk = *seq;
    for (lococo_tensor* t : {&blk.q, &blk.k, &blk.v}) t->p = (char*)t->p + (size_t)(sg.start * t->stride_t) * es;
    blk.o.p = ws + l.o_blk;                                  // (never written)
    blk.o.stride_t = (int64_t)d;
    blk.o.stride_h = (int64_t)sg.len * (int64_t)d;
    blk.o.stride_b = (int64_t)cfg->n_q_heads * blk.o.stride_h;
    const StepArgs a = make_args(cfg, &blk, 0, sg.len, &fc, conv_w, conv_b, true);
    if (sg.branch == 1 && path != PATH_GENERIC && !filters_ready) {
      if ((st = enqueue_repack(cfg, path, a, ws + l.fwd_ws, s))) return st;
      filters_ready = true;
    }
    lococo_cache next = fc;
    if ((st = enqueue_update(cfg, path, a, &next, ws + l.fwd_ws, B, s))) return st;
    fc = next;
  }

  // ---- reverse walk.  g[w] = gradient w.r.t. the state AFTER the block at hand.
  int w = 0;
  const size_t gbytes = chains * cfg->M * d * sizeof(float);
  for (int kv = 0; kv < 2; ++kv) {
    const float* src = kv ? d_final_v : d_final_k;
    if (src) HIP_TRY(hipMemcpyAsync(ws + l.g[w][kv], src, gbytes, hipMemcpyDeviceToDevice, s), "copying the final gradient");
    else HIP_TRY(launch_zero_fill(ws + l.g[w][kv], gbytes, s), "clearing the final gradient");
  }
  for (int64_t i = n - 1; i >= 0; --i) {
    const lococo_seg& sg = plan[(size_t)i];
    const size_t Bn = (size_t)sg.len;
    lococo_qkvo blk = *seq;
    for (lococo_tensor* t : {&blk.q, &blk.k, &blk.v}) t->p = (char*)t->p + (size_t)(sg.start * t->stride_t) * es;
    lococo_cache before = fc;
    before.k[0] = ws + l.states_k + (size_t)i * l.state;
    before.v[0] = ws + l.states_v + (size_t)i * l.state;
    before.k[1] = ws + l.cache[1];
    before.v[1] = ws + l.cache[3];
    before.cur = 0;
    before.len = sg.len_before;
    // the block's slice of d_o as a contiguous array; its slices of d_q, d_k, d_v go back the same way
    const size_t row = Bn * d * sizeof(float), pitch = (size_t)L * d * sizeof(float);
    HIP_TRY(hipMemcpy2DAsync(ws + l.d_o, row, (const char*)d_o + (size_t)sg.start * d * sizeof(float), pitch, row,
                             (size_t)cfg->batch * cfg->n_q_heads, hipMemcpyDeviceToDevice, s), "slicing d_o");
    if ((st = lococo_segment_step_backward(cfg, &blk, sg.len, conv_w, conv_b, &before, (const float*)(ws + l.d_o),
                                           (const float*)(ws + l.g[w][0]), (const float*)(ws + l.g[w][1]),
                                           (float*)(ws + l.d_q), (float*)(ws + l.d_k), (float*)(ws + l.d_v),
                                           (float*)(ws + l.g[w ^ 1][0]), (float*)(ws + l.g[w ^ 1][1]), d_conv_w, d_conv_b,
                                           ws + l.step_ws, l.total - l.step_ws, s)))
      return st;
    HIP_TRY(hipMemcpy2DAsync((char*)d_q + (size_t)sg.start * d * sizeof(float), pitch, ws + l.d_q, row, row,
                             (size_t)cfg->batch * cfg->n_q_heads, hipMemcpyDeviceToDevice, s), "placing d_q");
    HIP_TRY(hipMemcpy2DAsync((char*)d_k + (size_t)sg.start * d * sizeof(float), pitch, ws + l.d_k, row, row, chains,
                             hipMemcpyDeviceToDevice, s), "placing d_k");
    HIP_TRY(hipMemcpy2DAsync((char*)d_v + (size_t)sg.start * d * sizeof(float), pitch, ws + l.d_v, row, row, chains,
                             hipMemcpyDeviceToDevice, s), "placing d_v");
    w ^= 1;
  }
  HIP_TRY(hipMemcpyAsync(d_cache0_k, ws + l.g[w][0], gbytes, hipMemcpyDeviceToDevice, s), "returning the gradient of the first state");
  HIP_TRY(hipMemcpyAsync(d_cache0_v, ws + l.g[w][1], gbytes, hipMemcpyDeviceToDevice, s), "returning the gradient of the first state");
  return LOCOCO_OK;
}

}  // extern "C"
