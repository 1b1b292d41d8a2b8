// C ABI of the library: argument checks, workspace planning and kernel sequencing.
// Every check happens before the first HIP call of an entry point.
#include <cmath>
#include <cstring>
#include <mutex>

#include "gc_common.h"

// The workspace of gc_loss_and_rep_grad_bf16_static (see static_scratch below): a fixed array in the device image.
static __device__ __align__(256) unsigned char scratch[GC_STATIC_SCRATCH_BYTES];

namespace gc {

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
static inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Compute units of the current device (sizes grids and the stream splits of the workspace plan), asked once per
// process; without a device (the host-only checks of the test-suite) the MI355X count.
int num_cu() {
  static int cached = 0;
  if (cached > 0) return cached;
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
    cached = n;
  else
    cached = kNumCUDefault;
  (void)hipGetLastError();
  return cached;
}

LossPlan make_loss_plan(int B, int P, int d, gc_dtype dt, bool ntxent) {
  LossPlan pl{};
  const int kNumCU = num_cu();
  pl.use_mfma = (dt == GC_BF16 && d % 128 == 0 && d >= 128 && d <= 768) ? 1 : 0;
  if (pl.use_mfma) {
    const int n_ablk = ceil_div(B, 256), tiles = ceil_div(P, 256);
    // d = 128 has a statistics kernel of 256 threads, two workgroups to a CU
    int splits = ceil_div(d == 128 ? 2 * kNumCU : kNumCU, n_ablk);
    if (splits > 64) splits = 64;  // the merge kernel combines at most 64 splits per anchor
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    pl.stat_cols_per_split = ceil_div(tiles, splits) * 256;
    pl.stat_splits = ceil_div(P, pl.stat_cols_per_split);
    // gradient pass: one workgroup per CU, equal streamed length for both roles
    const int own = (d == 128) ? 256 : 64;   // owner rows per workgroup of the gradient kernel for this width
    const long long obQ = ceil_div(B, own), obP = ceil_div(P, own);
    // NT-Xent on these kernels is one walk (the score matrix is symmetric: see launch_grad_mfma)
    pl.one_walk = ntxent ? 1 : 0;
    const long long W = pl.one_walk ? obQ * P : obQ * P + obP * B;
    long long L = (W + kNumCU - 1) / kNumCU;
    if (L < 256) L = 256;
    L = (L + 31) / 32 * 32;
    auto split_of = [&](int n, int& ns, int& len) {
      ns = (int)((n + L - 1) / L);
      if (ns > 16) ns = 16;
      if (ns < 1) ns = 1;
      len = (ceil_div(n, ns) + 31) / 32 * 32;
      ns = ceil_div(n, len);
    };
    split_of(P, pl.nsq, pl.q_stream_len);
    split_of(B, pl.nsp, pl.p_stream_len);
    if (pl.one_walk) { pl.nsp = 1; pl.p_stream_len = B; }
    // fused mode (workspace is planned for it wherever it can run; fused_auto says where it is also the faster one):
    // each walk is a launch of its own and has to fill the GPU alone
    // (it pays where the statistics pass it replaces is expensive against the extra partial sums: measured faster
    // from d = 512 and 2^24 scores up, e.g. 0.251 against 0.261 ms at config 3 and 0.156 against 0.226 ms at
    // B = 1024, P = 16384, and slower below, where launches and partials dominate)
    // d = 384: a tie at config 3's size, 0.110 against 0.153 ms at B = 1024, P = 16384)
    pl.fused = (d >= 256 && !ntxent) ? 1 : 0;
    pl.fused_auto = (pl.fused && d >= 384 && (long long)B * P >= (1ll << 24)) ? 1 : 0;
    if (pl.fused) {
      auto split_alone = [&](long long own_blocks, int n, int& ns, int& len) {
        long long La = (own_blocks * n + kNumCU - 1) / kNumCU;
        if (La < 256) La = 256;
        ns = (int)((n + La - 1) / La);
        if (ns > 16) ns = 16;
        if (ns < 1) ns = 1;
        len = (ceil_div(n, ns) + 31) / 32 * 32;
        ns = ceil_div(n, len);
      };
      split_alone(obQ, P, pl.fz_nsq, pl.fz_q_stream_len);
      split_alone(obP, B, pl.fz_nsp, pl.fz_p_stream_len);
    }
  } else {
    const int blocks = ceil_div(B, 16), tiles = ceil_div(P, 16);
    int splits = ceil_div(4 * kNumCU, blocks);
    if (splits > 64) splits = 64;
    if (splits > tiles) splits = tiles;
    if (splits < 1) splits = 1;
    pl.stat_cols_per_split = ceil_div(tiles, splits) * 16;
    pl.stat_splits = ceil_div(P, pl.stat_cols_per_split);
    pl.nsq = pl.nsp = 1;
    pl.q_stream_len = P;
    pl.p_stream_len = B;
  }
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  pl.off_err = take(256);
  const int stat_parts = pl.stat_splits > pl.fz_nsq ? pl.stat_splits : pl.fz_nsq;   // fz_* are 0 outside fused mode
  pl.off_part_m = take((size_t)stat_parts * B * 4);
  pl.off_part_l = take((size_t)stat_parts * B * 4);
  pl.off_part_idx = take((size_t)stat_parts * B * 4);
  pl.off_pos = take((size_t)B * 4);
  pl.b_pad = (B + 63) / 64 * 64;
  pl.off_lse2 = take((size_t)pl.b_pad * 4);
  pl.off_pos_pad = take((size_t)pl.b_pad * 4);
  pl.off_rowloss = take((size_t)B * 4);
  // an anchor per target (see PosFix); among the statistics: everything below off_dq_part is what a call that only
  // forms statistics touches (the symmetric loss sizes its second workspace by that)
  pl.off_inv = take(pl.use_mfma ? (size_t)P * 4 : 0);
  int dq_parts = (pl.nsq > 1 || ntxent) ? pl.nsq : 0, dp_parts = ((pl.nsp > 1 || ntxent) && !pl.one_walk) ? pl.nsp : 0;
  if (pl.use_mfma && !ntxent) {  // the MFMA walks always write partials: the kernel that sums them adds the
    if (dq_parts < 1) dq_parts = 1;  // positive's term in fp32 (PosFix) and rounds a bf16 cache
    if (dp_parts < 1) dp_parts = 1;
  }
  if (pl.fused) {
    if (pl.fz_nsq > dq_parts) dq_parts = pl.fz_nsq;            // the online walk always writes partials
    if (pl.fz_nsp > 1 && pl.fz_nsp > dp_parts) dp_parts = pl.fz_nsp;
  }
  pl.off_dq_part = take((size_t)dq_parts * B * d * 4);
  pl.off_dp_part = take((size_t)dp_parts * P * d * 4);
  pl.off_on_ref = take((size_t)pl.fz_nsq * B * 4);
  pl.off_pos_idx = take(ntxent ? (size_t)B * 4 : 0);
  pl.total = off;
  return pl;
}

static bool shape_ok(int B, int P, int d) {
  if (B < 1 || P < 1 || d < 1) return false;
  if ((long long)B * d > (1ll << 40) || (long long)P * d > (1ll << 40)) return false;
  return true;
}

// per-device buffer behind the entry points that take no workspace
static std::mutex g_ws_mutex;
static void* g_ws_ptr[64];
static size_t g_ws_bytes[64];

static int own_workspace(size_t need, hipStream_t stream, void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  if (g_ws_bytes[dev] < need) {
    // growing allocates, and frees the old buffer (which waits for the device): neither is legal while the
    // caller's stream is being captured into a graph
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) { (void)hipGetLastError(); cap = hipStreamCaptureStatusNone; }
    if (cap != hipStreamCaptureStatusNone) return GC_ERR_UNSUPPORTED;
    if (g_ws_ptr[dev]) (void)hipFree(g_ws_ptr[dev]);  // waits for work that still uses it
    g_ws_ptr[dev] = nullptr;
    g_ws_bytes[dev] = 0;
    size_t sz = align_up(need + need / 4, 1 << 20);
    if (hipMalloc(&g_ws_ptr[dev], sz) != hipSuccess) return GC_ERR_HIP;
    g_ws_bytes[dev] = sz;
  }
  *out = g_ws_ptr[dev];
  return GC_OK;
}

// Calls that share the library's buffer from different streams are put in order: each call leaves an event behind
// its last kernel, and a call on another stream waits for it first.  (Not while a stream is being captured: an
// event of ordinary work cannot be waited for inside a capture; a captured call must not overlap with other calls
// on the buffer.)
static hipEvent_t g_ws_done[64];
static hipStream_t g_ws_last[64];
static bool g_ws_used[64];
static bool is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &cap) != hipSuccess) { (void)hipGetLastError(); return false; }
  return cap != hipStreamCaptureStatusNone;
}
static int own_workspace_enter(hipStream_t stream) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  if (is_capturing(stream)) return GC_OK;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  if (g_ws_used[dev] && g_ws_last[dev] != stream && hipStreamWaitEvent(stream, g_ws_done[dev], 0) != hipSuccess) return GC_ERR_HIP;
  return GC_OK;
}
static int own_workspace_leave(hipStream_t stream) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  if (is_capturing(stream)) return GC_OK;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  if (!g_ws_done[dev] && hipEventCreateWithFlags(&g_ws_done[dev], hipEventDisableTiming) != hipSuccess) return GC_ERR_HIP;
  if (hipEventRecord(g_ws_done[dev], stream) != hipSuccess) return GC_ERR_HIP;
  g_ws_last[dev] = stream;
  g_ws_used[dev] = true;
  return GC_OK;
}

// ---- the workspace of the entry point that allocates nothing: a fixed array in the device image ---------------
// One copy per GPU, at an address of its own.  Host code never uses the array's name as an address (on the host
// it is only a handle for the lookup): the address is asked for once per device, with that device current, and
// kept; kernels get it as an ordinary pointer argument, exactly as they get a caller's workspace.
static void* g_scratch_ptr[64];   // per device: what hipGetSymbolAddress answered (under g_ws_mutex)

static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return GC_ERR_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GC_OK;
}

// ---- measurement aid: HIP events around the phases of the loss path ------------------------------
struct Profile {
  bool on = false;
  int max_calls = 0, calls = 0;
  hipEvent_t* ev = nullptr;  // [max_calls][kMarks]
};
constexpr int kMarks = 5;  // start | after stats | after merge | after gradient kernel | after partial sums
static Profile g_prof;

static void prof_mark(int call, int mark, hipStream_t s) {
  if (g_prof.on && call < g_prof.max_calls) (void)hipEventRecord(g_prof.ev[call * kMarks + mark], s);
}
void prof_mark_grad_kernel_done(hipStream_t s) { prof_mark(g_prof.calls, 3, s); }
bool prof_active() { return g_prof.on; }

static int run_loss(const LossArgs& a_in, const LossPlan& pl) {
  LossArgs a = a_in;
  // does the gradient pass of this call end in a sum of split partials (launch_grad_mfma)?
  a.loss_with_partials = pl.use_mfma && !a.lse2_t && (a.dz || a.dq || a.dp);
  const int call = g_prof.calls;
  prof_mark(call, 0, a.stream);
  hipError_t e;
  const bool want_online = (a.flags & GC_PATH_ONLINE) || (pl.fused_auto && !(a.flags & GC_PATH_STATS_PASS));
  if (pl.fused && want_online && a.dq && !a.dz && !a.lse2_t) {
    // fused mode: online-statistics dQ walk | merge of its splits (lse2, row losses, dQ) | dP walk | partial sums
    e = launch_grad_online(a, pl);
    if (e != hipSuccess) return GC_ERR_HIP;
    prof_mark(call, 1, a.stream);
    e = launch_online_finish(a, pl);
    if (e != hipSuccess) return GC_ERR_HIP;
    prof_mark(call, 2, a.stream);
    bool loss_done = false;
    if (a.dp) {
      LossArgs b = a;
      LossPlan pb = pl;
      b.dq = nullptr;
      pb.nsp = pl.fz_nsp; pb.p_stream_len = pl.fz_p_stream_len;
      b.loss_with_partials = true;   // the dP walk always ends in the sum of its partials
      loss_done = true;
      e = launch_grad_mfma(b, pb);   // records mark 3 after the walk
      if (e != hipSuccess) return GC_ERR_HIP;
    } else {
      prof_mark(call, 3, a.stream);
    }
    if (!loss_done && !a.defer_loss_sum && launch_loss_sum(a, pl) != hipSuccess) return GC_ERR_HIP;
    prof_mark(call, 4, a.stream);
    if (g_prof.on) g_prof.calls++;
    return GC_OK;
  }
  if (!a.lse2_t) {
    e = pl.use_mfma ? launch_stats_mfma(a, pl) : launch_stats_generic(a, pl);
    if (e != hipSuccess) return GC_ERR_HIP;
  }
  prof_mark(call, 1, a.stream);
  if (!a.lse2_t) {
    e = launch_stats_merge(a, pl);
    if (e != hipSuccess) return GC_ERR_HIP;
  }
  prof_mark(call, 2, a.stream);
  if (a.dq || a.dp || a.dz) {
    e = pl.use_mfma ? launch_grad_mfma(a, pl) : launch_grad_generic(a, pl);  // records mark 3 after its main kernel(s)
    if (e != hipSuccess) return GC_ERR_HIP;
  } else {
    prof_mark(call, 3, a.stream);
  }
  prof_mark(call, 4, a.stream);
  if (g_prof.on) g_prof.calls++;
  return GC_OK;
}

static int check_loss_args(int dt, const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                           float scale, float temp, unsigned flags) {
  if (!q || !p || !pos_idx) return GC_ERR_NULL;
  if (!shape_ok(B, P, d)) return GC_ERR_SHAPE;
  if (!(scale > 0.f) || !(temp > 0.f) || !std::isfinite(scale) || !std::isfinite(temp)) return GC_ERR_SHAPE;
  if (!std::isfinite(scale / temp) || !(scale / temp > 0.f)) return GC_ERR_SHAPE;
  if (dt != GC_F32 && dt != GC_BF16) return GC_ERR_UNSUPPORTED;
  if (flags & ~(GC_MASK_SELF | GC_PATH_ONLINE | GC_PATH_STATS_PASS | GC_CACHE_BF16)) return GC_ERR_UNSUPPORTED;
  if ((flags & GC_CACHE_BF16) && !(dt == GC_BF16 && d % 128 == 0 && d >= 128 && d <= 768)) return GC_ERR_UNSUPPORTED;
  if ((flags & GC_PATH_ONLINE) && (flags & GC_PATH_STATS_PASS)) return GC_ERR_UNSUPPORTED;
  if ((flags & GC_MASK_SELF) && (B != P || P < 2)) return GC_ERR_SHAPE;
  return GC_OK;
}

__global__ void pair_index_kernel(int32_t* r, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) r[i] = i ^ 1;
}

// rinv[r[i]] = i; entries that no r[i] points at keep -1 (then r is no bijection, and the second direction of the
// symmetric loss reports them as positives out of range)
__global__ void fill_i32_kernel(int32_t* x, int n, int v) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) x[i] = v;
}
__global__ void invert_perm_kernel(const int32_t* r, int32_t* rinv, int n) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int j = r[i];
    if (j >= 0 && j < n) rinv[j] = i;
  }
}

}  // namespace gc

using namespace gc;

extern "C" {

const char* gc_strerror(int status) {
  switch (status) {
    case GC_OK: return "ok";
    case GC_ERR_NULL: return "a required pointer is NULL";
    case GC_ERR_SHAPE: return "invalid size, scale or temperature";
    case GC_ERR_UNSUPPORTED: return "unsupported dtype, flag or shape";
    case GC_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case GC_ERR_POS_IDX: return "pos_idx value outside [0, P)";
    case GC_ERR_HIP: return "HIP runtime call failed";
    case GC_ERR_TOO_LARGE: return "shape needs more scratch than the static buffer holds (GC_STATIC_SCRATCH_BYTES)";
    default: return "unknown gc_status";
  }
}

size_t gc_workspace_bytes(int B, int P, int d, int dt) {
  if (!shape_ok(B, P, d) || (dt != GC_F32 && dt != GC_BF16)) return 0;
  return make_loss_plan(B, P, d, (gc_dtype)dt, false).total;
}

int gc_loss_and_rep_grad_ex(int dt_int, const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                            float scale, float temp, unsigned flags, float* loss, float* dq, float* dp, float* lse,
                            int32_t* argmax, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_loss_args(dt_int, q, p, pos_idx, B, P, d, scale, temp, flags);
  if (rc != GC_OK) return rc;
  const gc_dtype dt = (gc_dtype)dt_int;
  const LossPlan pl = make_loss_plan(B, P, d, dt, false);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pl.total) return GC_ERR_WORKSPACE;
  LossArgs a{};
  a.dt = dt; a.q = q; a.p = p; a.pos_idx = pos_idx; a.B = B; a.P = P; a.d = d;
  a.alpha = scale / temp; a.flags = flags;
  a.loss = loss; a.dq = dq; a.dp = dp; a.lse = lse; a.argmax = argmax; a.dz = nullptr;
  a.ws = (char*)workspace; a.stream = (hipStream_t)stream;
  return run_loss(a, pl);
}

static int simple_loss(gc_dtype dt, const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                       float scale, float temp, float* loss, float* dq, float* dp, void* stream) {
  int rc = check_loss_args(dt, q, p, pos_idx, B, P, d, scale, temp, 0);
  if (rc != GC_OK) return rc;
  if (!loss || !dq || !dp) return GC_ERR_NULL;
  const size_t need = make_loss_plan(B, P, d, dt, false).total;
  void* ws = nullptr;
  rc = own_workspace(need, (hipStream_t)stream, &ws);
  if (rc != GC_OK) return rc;
  rc = own_workspace_enter((hipStream_t)stream);
  if (rc != GC_OK) return rc;
  rc = gc_loss_and_rep_grad_ex(dt, q, p, pos_idx, B, P, d, scale, temp, 0, loss, dq, dp, nullptr, nullptr, ws, need, stream);
  const int rc2 = own_workspace_leave((hipStream_t)stream);   // also after a failed launch: some kernels may be queued
  return rc != GC_OK ? rc : rc2;
}

int gc_loss_and_rep_grad_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d, float scale,
                              float temp, float* loss, float* dq, float* dp, void* stream) {
  return simple_loss(GC_BF16, q, p, pos_idx, B, P, d, scale, temp, loss, dq, dp, stream);
}

int gc_loss_and_rep_grad_bf16_static(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                     float scale, float temp, float* loss, float* dq, float* dp, void* stream) {
  int rc = check_loss_args(GC_BF16, q, p, pos_idx, B, P, d, scale, temp, 0);
  if (rc != GC_OK) return rc;
  if (!loss || !dq || !dp) return GC_ERR_NULL;
  const size_t need = make_loss_plan(B, P, d, GC_BF16, false).total;
  if (need > (size_t)GC_STATIC_SCRATCH_BYTES) return GC_ERR_TOO_LARGE;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != GC_OK) return rc;
  // every word of the workspace that a kernel of this path reads has been written by an earlier kernel of the same
  // call (statistics, partial sums, the error word): nothing has to start at zero
  return gc_loss_and_rep_grad_ex(GC_BF16, q, p, pos_idx, B, P, d, scale, temp, 0, loss, dq, dp, nullptr, nullptr, ws,
                                 need, stream);
}

int gc_loss_and_rep_grad_f32(const float* q, const float* p, const int32_t* pos_idx, int B, int P, int d, float scale,
                             float temp, float* loss, float* dq, float* dp, void* stream) {
  return simple_loss(GC_F32, q, p, pos_idx, B, P, d, scale, temp, loss, dq, dp, stream);
}

int gc_check_async_error(const void* workspace) {
  const void* ws[2] = {workspace, nullptr};
  if (!workspace) {   // the library's own buffers of this device, as far as they have been used
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_ws_mutex);
    ws[0] = g_ws_ptr[dev];
    ws[1] = g_scratch_ptr[dev];
  }
  for (const void* w : ws) {
    if (!w) continue;
    int word = 0;
    if (hipMemcpy(&word, w, sizeof(int), hipMemcpyDeviceToHost) != hipSuccess) return GC_ERR_HIP;
    if (word) return GC_ERR_POS_IDX;
  }
  return GC_OK;
}

int gc_profile_begin(int max_calls) {
  if (max_calls < 1 || max_calls > (1 << 16)) return GC_ERR_SHAPE;
  if (g_prof.ev) return GC_ERR_UNSUPPORTED;  // already open
  g_prof.ev = new hipEvent_t[(size_t)max_calls * kMarks];
  for (int i = 0; i < max_calls * kMarks; i++)
    if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {   // give back what was made: a later begin starts afresh
      for (int k = 0; k < i; k++) (void)hipEventDestroy(g_prof.ev[k]);
      delete[] g_prof.ev;
      g_prof.ev = nullptr;
      return GC_ERR_HIP;
    }
  g_prof.max_calls = max_calls;
  g_prof.calls = 0;
  g_prof.on = true;
  return GC_OK;
}

int gc_profile_end(float* ms_stats, float* ms_merge, float* ms_grad, float* ms_reduce, int* calls) {
  if (!g_prof.ev) return GC_ERR_UNSUPPORTED;
  g_prof.on = false;
  const int n = g_prof.calls < g_prof.max_calls ? g_prof.calls : g_prof.max_calls;
  double acc[4] = {0, 0, 0, 0};
  int rc = GC_OK;
  for (int c = 0; c < n && rc == GC_OK; c++) {
    if (hipEventSynchronize(g_prof.ev[c * kMarks + 4]) != hipSuccess) { rc = GC_ERR_HIP; break; }
    for (int k = 0; k < 4; k++) {
      float ms = 0.f;
      if (hipEventElapsedTime(&ms, g_prof.ev[c * kMarks + k], g_prof.ev[c * kMarks + k + 1]) != hipSuccess) rc = GC_ERR_HIP;
      acc[k] += ms;
    }
  }
  for (int i = 0; i < g_prof.max_calls * kMarks; i++) (void)hipEventDestroy(g_prof.ev[i]);
  delete[] g_prof.ev;
  g_prof.ev = nullptr;
  if (rc != GC_OK) return rc;
  if (ms_stats) *ms_stats = n ? (float)(acc[0] / n) : 0.f;
  if (ms_merge) *ms_merge = n ? (float)(acc[1] / n) : 0.f;
  if (ms_grad) *ms_grad = n ? (float)(acc[2] / n) : 0.f;
  if (ms_reduce) *ms_reduce = n ? (float)(acc[3] / n) : 0.f;
  if (calls) *calls = n;
  g_prof.max_calls = g_prof.calls = 0;
  return GC_OK;
}

size_t gc_ntxent_workspace_bytes(int n_views, int d) {
  if (n_views < 2 || (n_views & 1) || !shape_ok(n_views, n_views, d)) return 0;
  return make_loss_plan(n_views, n_views, d, GC_BF16, true).total;
}

int gc_ntxent_loss_and_grad_bf16(const void* z, int n_views, int d, float temp, float* loss, float* dz,
                                 void* workspace, size_t workspace_bytes, void* stream) {
  if (!z) return GC_ERR_NULL;
  if (n_views < 2 || (n_views & 1) || !shape_ok(n_views, n_views, d)) return GC_ERR_SHAPE;
  if (!(temp > 0.f) || !std::isfinite(temp) || !std::isfinite(1.f / temp)) return GC_ERR_SHAPE;
  const LossPlan pl = make_loss_plan(n_views, n_views, d, GC_BF16, true);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pl.total) return GC_ERR_WORKSPACE;
  LossArgs a{};
  a.dt = GC_BF16; a.q = z; a.p = z; a.B = n_views; a.P = n_views; a.d = d;
  a.alpha = 1.f / temp; a.flags = GC_MASK_SELF;
  a.loss = loss; a.dz = dz;
  a.ws = (char*)workspace; a.stream = (hipStream_t)stream;
  int32_t* r = (int32_t*)(a.ws + pl.off_pos_idx);
  pair_index_kernel<<<(n_views + 255) / 256, 256, 0, a.stream>>>(r, n_views);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  a.pos_idx = r;
  return run_loss(a, pl);
}

// Workspace of the symmetric loss: [loss workspace, direction 1][direction 2][r^-1][two losses][4 gradient buffers].
// With the MFMA kernels one gradient pass serves both directions: the second workspace then holds statistics only
// and there are no gradient buffers.
struct SymPlan { LossPlan pl; size_t off2, off_rinv, off_l, off_g, total; };
static SymPlan make_sym_plan(int n, int d) {
  SymPlan sp{};
  sp.pl = make_loss_plan(n, n, d, GC_BF16, false);
  size_t off = align_up(sp.pl.total, 256);
  sp.off2 = off; off = align_up(off + (sp.pl.use_mfma ? sp.pl.off_dq_part : sp.pl.total), 256);
  sp.off_rinv = off; off = align_up(off + (size_t)n * 4, 256);
  sp.off_l = off; off += 256;
  sp.off_g = off; off += sp.pl.use_mfma ? 0 : 4 * align_up((size_t)n * d * 4, 256);
  sp.total = off;
  return sp;
}

size_t gc_bidirectional_workspace_bytes(int n, int d) {
  if (n < 1 || !shape_ok(n, n, d)) return 0;
  return make_sym_plan(n, d).total;
}

int gc_bidirectional_loss_and_rep_grad_bf16(const void* q, const void* p, const int32_t* pos_idx, int n, int d, float scale,
                                            float temp, float* loss, float* dq, float* dp, void* workspace,
                                            size_t workspace_bytes, void* stream) {
  int rc = check_loss_args(GC_BF16, q, p, pos_idx, n, n, d, scale, temp, 0);
  if (rc != GC_OK) return rc;
  if (!loss || !dq || !dp) return GC_ERR_NULL;
  const SymPlan sp = make_sym_plan(n, d);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sp.total) return GC_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t s = (hipStream_t)stream;
  int32_t* rinv = (int32_t*)(ws + sp.off_rinv);
  float* l = (float*)(ws + sp.off_l);
  fill_i32_kernel<<<(n + 255) / 256, 256, 0, s>>>(rinv, n, -1);
  invert_perm_kernel<<<(n + 255) / 256, 256, 0, s>>>(pos_idx, rinv, n);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  LossArgs a{};
  a.dt = GC_BF16; a.B = n; a.P = n; a.d = d; a.alpha = scale / temp; a.stream = s;
  a.defer_loss_sum = true;   // one launch sums the row losses of both directions at the end
  LossArgs a1, a2;
  if (sp.pl.use_mfma) {
    // statistics of both directions (Eq. 1 as it stands, then with the two sides exchanged) ...
    a.q = q; a.p = p; a.pos_idx = pos_idx; a.loss = l; a.ws = ws;
    a1 = a;
    rc = run_loss(a, sp.pl);
    if (rc != GC_OK) return rc;
    a.q = p; a.p = q; a.pos_idx = rinv; a.loss = l + 1; a.ws = ws + sp.off2;
    a2 = a;
    rc = run_loss(a, sp.pl);
    if (rc != GC_OK) return rc;
    // ... and one gradient pass with the mean of the two softmaxes as coefficients
    a.q = q; a.p = p; a.pos_idx = pos_idx; a.loss = nullptr; a.ws = ws; a.dq = dq; a.dp = dp;
    a.lse2_t = (const float*)(ws + sp.off2 + sp.pl.off_lse2);
    a.pos_inv = rinv;
    a.zero_word = (const int*)(ws + sp.pl.off_err) + 1;   // zeroed by the first direction's merge, raised by nobody here
    rc = run_loss(a, sp.pl);
    if (rc != GC_OK) return rc;
  } else {
    const size_t gsz = align_up((size_t)n * d * 4, 256);
    float* g[4];
    for (int i = 0; i < 4; i++) g[i] = (float*)(ws + sp.off_g + i * gsz);
    a.grad_mul = 0.5f;
    // direction 1: anchors against targets (Eq. 1); direction 2: the same with the two sides exchanged
    a.q = q; a.p = p; a.pos_idx = pos_idx; a.loss = l; a.dq = g[0]; a.dp = g[1]; a.ws = ws;
    a1 = a;
    rc = run_loss(a, sp.pl);
    if (rc != GC_OK) return rc;
    a.q = p; a.p = q; a.pos_idx = rinv; a.loss = l + 1; a.dq = g[2]; a.dp = g[3]; a.ws = ws + sp.off2;
    a2 = a;
    rc = run_loss(a, sp.pl);
    if (rc != GC_OK) return rc;
    // dL/df = Eq. 5 of direction 1 + Eq. 6 of direction 2, dL/dg the other two; fixed order
    const size_t ne = (size_t)n * d;
    { const float* srcs[2] = {g[0], g[3]}; int counts[2] = {1, 1}; size_t strides[2] = {ne, ne};
      if (launch_partial_reduce(dq, srcs, counts, strides, 2, ne, s) != hipSuccess) return GC_ERR_HIP; }
    { const float* srcs[2] = {g[1], g[2]}; int counts[2] = {1, 1}; size_t strides[2] = {ne, ne};
      if (launch_partial_reduce(dp, srcs, counts, strides, 2, ne, s) != hipSuccess) return GC_ERR_HIP; }
  }
  return launch_sym_loss_sum(a1, a2, sp.pl, loss) == hipSuccess ? GC_OK : GC_ERR_HIP;
}

}  // extern "C"
