// Shared host/device declarations of the gfx950 Gradient Cache library
// (internal; the public C ABI is include/gradcache.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gradcache.h"

namespace gc {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kNumCUDefault = 256;  // MI355X; what num_cu() answers when no device can be asked
int num_cu();                       // compute units of the current device: sizes grids and workspace splits

// fp32 -> bf16 bits, round to nearest even (inputs here are finite).
__device__ __forceinline__ unsigned short f2bf(float f) {
  unsigned u = __builtin_bit_cast(unsigned, f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ __forceinline__ unsigned pack2bf(float lo, float hi) {
  return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16);
}
__device__ __forceinline__ float bf2f(unsigned short b) { return __builtin_bit_cast(float, (unsigned)b << 16); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---------------------------------------------------------------------------
// Workspace plan of gc_loss_and_rep_grad_ex: one host function decides the
// splits and the byte offsets, so gc_workspace_bytes and the launch agree.
// ---------------------------------------------------------------------------
struct LossPlan {
  int use_mfma;          // 1: bf16 MFMA kernels, 0: general fp32-FMA kernels
  int one_walk;          // NT-Xent on the MFMA kernels: dz from a single walk (no dP role, no dP partials)
  int stat_splits;       // column (target) ranges of the statistics pass
  int stat_cols_per_split;
  int nsq, nsp;          // stream splits of the dQ-role / dP-role workgroups of the gradient pass
  int q_stream_len, p_stream_len;  // stream rows per split (multiple of the stream tile)
  int b_pad;             // B rounded up to 64: length of the padded lse2 / pos_pad arrays
  // fused mode (MFMA kernels, d >= 256, dQ wanted): no statistics pass; an online-statistics dQ walk, a kernel that
  // merges its splits into lse2 and dQ, then the dP walk.  Each walk fills the GPU alone, so they have splits of their own
  int fused, fused_auto, fz_nsq, fz_nsp, fz_q_stream_len, fz_p_stream_len;   // can run / is chosen without a flag
  size_t off_err, off_part_m, off_part_l, off_part_idx, off_pos, off_lse2, off_pos_pad, off_rowloss, off_dq_part,
      off_dp_part, off_pos_idx, off_on_ref, off_inv, total;
};

LossPlan make_loss_plan(int B, int P, int d, gc_dtype dt, bool ntxent);

struct LossArgs {
  gc_dtype dt;
  const void* q;
  const void* p;
  const int32_t* pos_idx;
  int B, P, d;
  float alpha;       // scale / temp
  unsigned flags;
  float* loss;
  float* dq;
  float* dp;
  float* lse;
  int32_t* argmax;
  float* dz;         // NT-Xent: dq + dp summed into one buffer (dq, dp then unused)
  float grad_mul;    // extra factor on the gradients (0 = 1; the symmetric loss halves both terms)
  // symmetric loss in one gradient pass (MFMA kernels only): log2-domain log-sum-exp per target over the anchors,
  // padded like the per-anchor one; with it set the statistics of this call are taken as already in `ws`
  const float* lse2_t;
  // ... with the inverse of the pairing (pos_inv[r_i] = i, a bijection there) and a device word that holds 0, for
  // the positive's term of the dP rows (PosFix)
  const int32_t* pos_inv;
  const int* zero_word;
  // set by run_loss when the gradient pass ends in a sum of split partials: that launch then also sums the row
  // losses (one launch less); the statistics merge leaves the sum to it
  bool loss_with_partials;
  bool defer_loss_sum;   // the caller sums the row losses itself (the symmetric loss: both directions in one launch)
  char* ws;
  hipStream_t stream;
};

// The positive's own term of Eq. 5 / Eq. 6, (p_{i r_i} - 1) g(t_{r_i}) resp. (p_{i r_i} - 1) f(s_i), is not part of the bf16
// contractions of the MFMA walks (they take the coefficient 0 at the positive): rounded to bf16, this one coefficient
// of size up to 1 next to P - 1 small ones would be the whole error of its gradient row.  The kernel that sums the
// split partials adds it in fp32 from the row statistics:
//   c_i = scale * (2^(pos_t_i - lse2_i) - 1)                                       one direction
//   c_i = scale * (1/2 (2^(pos_t_i - lse2_i) + 2^(pos_t_i - lse2_t[r_i])) - 1)     symmetric loss, NT-Xent
struct PosFix {
  int mode;                     // 0: nothing to add; 1: output rows are anchors (dq, dz); 2: output rows are targets (dp)
  const int32_t* pos;           // [B] r_i
  const int32_t* inv;           // mode 2: [P], inv[j] = an anchor i with r_i = j where there is one (always checked)
  const int* shared;            // mode 2: nonzero when some target is the positive of several anchors (then: a scan)
  const float* pos_t;           // [B] base-2 logit of the positive
  const float* lse2;            // [B] base-2 log-sum-exp per anchor
  const float* lse2_t;          // [P] the same per target over the anchors (symmetric forms), else nullptr
  const unsigned short* other;  // bf16 rows that the term multiplies: targets (mode 1), anchors (mode 2)
  int B, P, d;
  float scale;
};

// kernel-launching halves (one per .hip file)
hipError_t launch_stats_generic(const LossArgs& a, const LossPlan& pl);
hipError_t launch_grad_generic(const LossArgs& a, const LossPlan& pl);
hipError_t launch_stats_mfma(const LossArgs& a, const LossPlan& pl);
hipError_t launch_grad_mfma(const LossArgs& a, const LossPlan& pl);
hipError_t launch_grad_online(const LossArgs& a, const LossPlan& pl);    // fused mode: dQ walk with online statistics
hipError_t launch_online_finish(const LossArgs& a, const LossPlan& pl);  // ... its splits -> lse2, row losses, dQ
hipError_t launch_loss_sum(const LossArgs& a, const LossPlan& pl);       // the fixed-order sum of the row losses alone
// symmetric loss: both directions' sums in one launch, loss = (l1 + l2) / 2, the first error word takes the second's
hipError_t launch_sym_loss_sum(const LossArgs& a1, const LossArgs& a2, const LossPlan& pl, float* loss);
hipError_t launch_stats_merge(const LossArgs& a, const LossPlan& pl);
void prof_mark_grad_kernel_done(hipStream_t s);  // measurement aid: event after the main gradient kernel(s)
bool prof_active();  // the measurement events of the loss path are being recorded
// loss_of / pl: also carry the sum of the row losses of that call (see LossArgs::loss_with_partials)
hipError_t launch_partial_reduce(float* out, const float* const* srcs, const int* counts, const size_t* strides,
                                 int nsrc, size_t n, hipStream_t stream, const LossArgs* loss_of = nullptr,
                                 const LossPlan* pl = nullptr, bool out_bf16 = false, const PosFix* fix = nullptr);

// Workgroups are handed to the 8 XCDs round-robin by their id, and each XCD has its own L2.  This
// turns the hardware id into a task id such that each XCD works on one contiguous range of tasks
// (tasks that stream the same rows are numbered consecutively by the launchers).
__device__ __forceinline__ int xcd_task_id() {
  const int id = blockIdx.x, n = gridDim.x;
  return (n % 8 == 0) ? (id % 8) * (n / 8) + id / 8 : id;
}

// A kernel that uses more than 64 KB of dynamic LDS has to be opted in (hipFuncSetAttribute): once per kernel and
// device, remembered in `done` (a function-local array of the launcher, one per kernel instantiation).
inline hipError_t ensure_dyn_lds(const void* fn, int bytes, bool (&done)[64]) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess) done[dev] = true;
  return e;
}

}  // namespace gc
