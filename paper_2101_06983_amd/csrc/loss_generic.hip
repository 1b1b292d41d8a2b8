// General (any d, fp32 or bf16 storage) kernels of the loss / representation-
// gradient path, fp32 FMA arithmetic.  They serve the fp32 entry point and the
// shapes the MFMA kernels do not cover, and they hold the pieces both paths
// share: the merge of split row statistics, the loss reduction and the
// fixed-order sum of split gradient partials.
//
// Scores are kept in the base-2 domain: t_ij = s_ij * log2(e), so that
// softmax_j = 2^(t_ij - lse2_i) with lse2_i = log2 sum_j 2^t_ij (Eq. 4).
#include <type_traits>

#include "gc_common.h"

namespace gc {

template <typename T>
__device__ __forceinline__ float ldf(const T* p, size_t i);
template <>
__device__ __forceinline__ float ldf<float>(const float* p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float ldf<unsigned short>(const unsigned short* p, size_t i) { return bf2f(p[i]); }

constexpr int GT = 16;  // tile edge of the general kernels (16 x 16 scores per workgroup step)
constexpr int GK = 32;  // k-chunk staged through LDS

// One 16x16 tile of base-2 scores: thread (ty, tx) gets t for anchor row0+ty, target col0+tx.
template <typename T>
__device__ __forceinline__ float score_tile(const T* __restrict__ Q, const T* __restrict__ Pm, int B, int P, int d,
                                            int row0, int col0, float alpha2, float (*Qs)[GK + 1], float (*Ps)[GK + 1]) {
  const int tx = threadIdx.x % GT, ty = threadIdx.x / GT;
  float acc = 0.f;
  for (int k0 = 0; k0 < d; k0 += GK) {
    // 256 threads stage 16 x 32 of each operand (2 elements per thread per operand)
    for (int e = threadIdx.x; e < GT * GK; e += GT * GT) {
      int r = e / GK, k = e % GK;
      int qi = min(row0 + r, B - 1), pj = min(col0 + r, P - 1);
      bool kin = (k0 + k) < d;
      Qs[r][k] = kin ? ldf<T>(Q, (size_t)qi * d + k0 + k) : 0.f;
      Ps[r][k] = kin ? ldf<T>(Pm, (size_t)pj * d + k0 + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < GK; k++) acc = fmaf(Qs[ty][k], Ps[tx][k], acc);
    __syncthreads();
  }
  return acc * alpha2;
}

// Row statistics (Eq. 4's denominator, online over target tiles), one column split per blockIdx.y.
template <typename T>
__global__ void __launch_bounds__(256) stats_generic_kernel(const T* __restrict__ Q, const T* __restrict__ Pm,
                                                           const int32_t* __restrict__ pos_idx, int B, int P, int d,
                                                           float alpha2, int mask_self, int cols_per_split,
                                                           float* __restrict__ part_m, float* __restrict__ part_l,
                                                           int* __restrict__ part_idx, float* __restrict__ pos_t) {
  __shared__ float Qs[GT][GK + 1], Ps[GT][GK + 1];
  __shared__ float red_m[GT][GT], red_l[GT][GT];
  __shared__ int red_i[GT][GT];
  const int tx = threadIdx.x % GT, ty = threadIdx.x / GT;
  const int row0 = blockIdx.x * GT;
  const int split = blockIdx.y;
  const int cbeg = split * cols_per_split, cend = min(P, cbeg + cols_per_split);
  const int i = row0 + ty;
  const int ri = (i < B) ? pos_idx[i] : -1;
  float m = -INFINITY, l = 0.f;
  int best = 0x7fffffff;
  for (int col0 = cbeg; col0 < cend; col0 += GT) {
    float t = score_tile<T>(Q, Pm, B, P, d, row0, col0, alpha2, Qs, Ps);
    int j = col0 + tx;
    bool valid = (j < cend) && !(mask_self && j == i);
    // (a positive that the self-mask removes has the logit -inf: its row loss is then +inf)
    if (j < cend && j == ri && i < B) pos_t[i] = valid ? t : -INFINITY;
    if (valid) {
      if (t > m) {  // strict: ties keep the smaller index (columns are visited in increasing order)
        l = l * exp2f(m - t) + 1.f;
        m = t;
        best = j;
      } else {
        l += exp2f(t - m);
      }
    }
  }
  red_m[ty][tx] = m; red_l[ty][tx] = l; red_i[ty][tx] = best;
  __syncthreads();
  if (tx == 0 && i < B) {
    float mm = -INFINITY; int bi = 0x7fffffff;
    for (int x = 0; x < GT; x++) {
      float v = red_m[ty][x];
      if (v > mm || (v == mm && red_i[ty][x] < bi)) { mm = v; bi = red_i[ty][x]; }
    }
    float ll = 0.f;
    if (mm > -INFINITY)
      for (int x = 0; x < GT; x++) ll += red_l[ty][x] * exp2f(red_m[ty][x] - mm);
    part_m[(size_t)split * B + i] = mm;
    part_l[(size_t)split * B + i] = ll;
    part_idx[(size_t)split * B + i] = bi;
  }
}

// Merge of the split statistics of every anchor: lse2_i, row loss (Eq. 1's summand), argmax.
// LANES (a power of two >= nsplit, <= 64) consecutive lanes share one anchor, one split each, and
// combine with a fixed butterfly, so every load of the kernel is issued at once.  lse2 and the
// copy of pos_idx are padded to b_pad rows with +inf / -1, so that the gradient pass can read
// whole tiles without bounds checks (a padded row gives g = 0).
template <int LANES>
__global__ void __launch_bounds__(256) stats_merge_kernel(const float* __restrict__ part_m, const float* __restrict__ part_l,
                                                         const int* __restrict__ part_idx, const float* __restrict__ pos_t,
                                                         const int32_t* __restrict__ pos_idx, int B, int P, int nsplit,
                                                         int b_pad, float* __restrict__ lse2, int32_t* __restrict__ pos_pad,
                                                         float* __restrict__ rowloss, float* __restrict__ lse_out,
                                                         int32_t* __restrict__ argmax_out, int32_t* __restrict__ inv,
                                                         int* __restrict__ shared) {
  constexpr int ROWS = 256 / LANES;
  if (shared && blockIdx.x == 0 && threadIdx.x == 0) *shared = 0;   // raised later by the gradient kernel's check
  const int s = threadIdx.x % LANES;
  const int i = blockIdx.x * ROWS + threadIdx.x / LANES;
  const bool live = (i < B) && (s < nsplit);
  float m = live ? part_m[(size_t)s * B + i] : -INFINITY;
  float l = live ? part_l[(size_t)s * B + i] : 0.f;
  int bi = live ? part_idx[(size_t)s * B + i] : 0x7fffffff;
#pragma unroll
  for (int w = 1; w < LANES; w <<= 1) {
    const float m2 = __shfl_xor(m, w), l2 = __shfl_xor(l, w);
    const int b2 = __shfl_xor(bi, w);
    const float mn = fmaxf(m, m2);
    const float ms = (mn == -INFINITY) ? 0.f : mn;
    // both partners evaluate the same expression with the operands in the same (lower lane first) order
    const bool lower = (s & w) == 0;
    const float la = lower ? l : l2, ma = lower ? m : m2, lb = lower ? l2 : l, mb = lower ? m2 : m;
    l = la * exp2f(ma - ms) + lb * exp2f(mb - ms);
    bi = (m2 > m || (m2 == m && b2 < bi)) ? b2 : bi;
    m = mn;
  }
  if (s != 0 || i >= b_pad) return;
  if (i >= B) { lse2[i] = INFINITY; pos_pad[i] = -1; return; }
  const float l2 = m + log2f(l);
  lse2[i] = l2;
  const int r = pos_idx[i];
  pos_pad[i] = r;
  const bool ok = (r >= 0 && r < P);
  rowloss[i] = ok ? (l2 - pos_t[i]) * kLn2 : NAN;
  if (inv && ok) inv[r] = i;   // an anchor per target; which one, when several share it, is not relied upon
  if (lse_out) lse_out[i] = l2 * kLn2;
  if (argmax_out) argmax_out[i] = bi;
}

// loss = (1/B) sum_i rowloss_i by one workgroup; raises the error word when a row was flagged because its
// pos_idx was out of range.  The order is fixed and does not depend on the size of the workgroup: 1024 strided
// partial sums, then a binary tree over them (so the value has the same bits whichever kernel carries the sum).
struct LossSum {
  const float* rowloss;      // nullptr: nothing to do
  const int32_t* pos_idx;
  int B, P;
  float* loss;               // may be nullptr
  int* err;
};
template <int NT>  // threads of the workgroup
__device__ __forceinline__ void loss_sum_block(const LossSum& ls, float* red /* [1024] in LDS */) {
  constexpr int SL = 1024 / NT;   // partial sums per thread: slots threadIdx.x + NT * j
  float s[SL];
  int b = 0;
#pragma unroll
  for (int j = 0; j < SL; j++) s[j] = 0.f;
  // rows i0 + slot, i0 = 0, 1024, ...: the loads of four such steps are issued together, then summed in order
  for (int i0 = 0; i0 < ls.B; i0 += 4096) {
    float v[4][SL];
    int r[4][SL];
#pragma unroll
    for (int k = 0; k < 4; k++)
#pragma unroll
      for (int j = 0; j < SL; j++) {
        const int i = i0 + 1024 * k + (int)threadIdx.x + NT * j;
        const int ic = min(i, ls.B - 1);
        v[k][j] = ls.rowloss[ic];
        r[k][j] = ls.pos_idx[ic];
      }
#pragma unroll
    for (int k = 0; k < 4; k++)
#pragma unroll
      for (int j = 0; j < SL; j++) {
        const int i = i0 + 1024 * k + (int)threadIdx.x + NT * j;
        if (i < ls.B) {
          s[j] += v[k][j];
          b |= (r[k][j] < 0 || r[k][j] >= ls.P);
        }
      }
  }
#pragma unroll
  for (int j = 0; j < SL; j++) red[threadIdx.x + NT * j] = s[j];
  const int bad = __syncthreads_or(b);
  for (int w = 512; w > 0; w >>= 1) {
    for (int x = threadIdx.x; x < w; x += NT) red[x] += red[x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    if (ls.loss) *ls.loss = bad ? NAN : red[0] / (float)ls.B;
    *ls.err = bad ? 1 : 0;
  }
}
__global__ void __launch_bounds__(1024) loss_reduce_kernel(LossSum ls) {
  __shared__ float red[1024];
  loss_sum_block<1024>(ls, red);
}

// Gradient pass, general form.  owner = the matrix whose gradient rows this workgroup owns
// (Q for Eq. 5, P for Eq. 6); the other matrix is streamed 16 rows at a time.  The owned
// 16 x d block of the output is updated in place tile by tile (one owner per row: no atomics).
template <typename T, bool OWNER_IS_Q>
__global__ void __launch_bounds__(256) grad_generic_kernel(const T* __restrict__ Q, const T* __restrict__ Pm,
                                                          const int32_t* __restrict__ pos_idx, const float* __restrict__ lse2,
                                                          int B, int P, int d, float alpha2, float out_scale, int mask_self,
                                                          float* __restrict__ out) {
  __shared__ float Qs[GT][GK + 1], Ps[GT][GK + 1];
  __shared__ float g[GT][GT + 1];  // g[owner row][stream row]
  const int tx = threadIdx.x % GT, ty = threadIdx.x / GT;
  const int own0 = blockIdx.x * GT;
  const int n_own = OWNER_IS_Q ? B : P, n_str = OWNER_IS_Q ? P : B;
  const T* S = OWNER_IS_Q ? Pm : Q;
  bool first = true;
  for (int str0 = 0; str0 < n_str; str0 += GT) {
    const int row0 = OWNER_IS_Q ? own0 : str0;  // anchors on ty
    const int col0 = OWNER_IS_Q ? str0 : own0;  // targets on tx
    float t = score_tile<T>(Q, Pm, B, P, d, row0, col0, alpha2, Qs, Ps);
    int i = row0 + ty, j = col0 + tx;
    float gv = 0.f;
    if (i < B && j < P && !(mask_self && i == j)) {
      gv = exp2f(t - lse2[i]) - ((pos_idx[i] == j) ? 1.f : 0.f);
    }
    if (OWNER_IS_Q) g[ty][tx] = gv * out_scale; else g[tx][ty] = gv * out_scale;
    __syncthreads();
    for (int e = threadIdx.x; e < GT * d; e += 256) {
      int r = e / d, c = e % d;
      if (own0 + r < n_own) {
        float acc = 0.f;
        for (int b = 0; b < GT; b++) {
          int sr = min(str0 + b, n_str - 1);  // g is 0 past the end
          acc = fmaf(g[r][b], ldf<T>(S, (size_t)sr * d + c), acc);
        }
        size_t o = (size_t)(own0 + r) * d + c;
        out[o] = first ? acc : out[o] + acc;
      }
    }
    first = false;
    __syncthreads();
  }
}

// out[e] = sum over sources s, over parts k < counts[s] of srcs[s][k * strides[s] + e], fixed order.
struct ReduceSrc {
  const float* ptr[4];
  int count[4];
  size_t stride[4];
  int nsrc;
  int out_bf16;   // the sum is stored as bf16 (round to nearest even), `out` then points to bf16 elements
};
// With a loss sum attached the grid has one more workgroup, the first (so that it runs beside the others), which carries it (it has nothing to do with
// the partial sums; it only saves a launch on the path that needs both).
// coefficient of the positive of anchor i (target r), see PosFix
__device__ __forceinline__ float pos_coeff(const PosFix& f, int i, int r) {
  const float t = f.pos_t[i];
  float c = exp2f(t - f.lse2[i]);
  if (f.lse2_t) c = 0.5f * (c + exp2f(t - f.lse2_t[r]));
  return f.scale * (c - 1.f);
}
__device__ __forceinline__ void add_row4(f32x4& acc, float c, const unsigned short* row, int col) {
  const s16x4 v = *(const s16x4*)(row + col);
#pragma unroll
  for (int k = 0; k < 4; k++) acc[k] += c * bf2f((unsigned short)v[k]);
}
__global__ void __launch_bounds__(256) partial_reduce_kernel(float* __restrict__ out, ReduceSrc rs, size_t n4, LossSum ls,
                                                            PosFix fx) {
  __shared__ float red[1024];
  if (ls.rowloss && blockIdx.x == 0) {
    loss_sum_block<256>(ls, red);
    return;
  }
  size_t e = (size_t)(blockIdx.x - (ls.rowloss ? 1 : 0)) * blockDim.x + threadIdx.x;
  if (e >= n4) return;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < rs.nsrc; s++)
    for (int k = 0; k < rs.count[s]; k++) acc += ((const f32x4*)(rs.ptr[s] + (size_t)k * rs.stride[s]))[e];
  if (fx.mode) {   // the positive's term, in fp32, after the partials (d is a multiple of 4 here)
    const int row = (int)((e * 4) / (size_t)fx.d), col = (int)((e * 4) % (size_t)fx.d);
    if (fx.mode == 1) {
      const int r = fx.pos[row];
      if (r >= 0 && r < fx.P) add_row4(acc, pos_coeff(fx, row, r), fx.other + (size_t)r * fx.d, col);
    } else if (*fx.shared == 0) {
      const int i = fx.inv[row];   // whatever the workspace held if no anchor names this target: checked
      if (i >= 0 && i < fx.B && fx.pos[i] == row) add_row4(acc, pos_coeff(fx, i, row), fx.other + (size_t)i * fx.d, col);
    } else {   // some target is shared: every anchor that names this one, in index order
      for (int i = 0; i < fx.B; i++)
        if (fx.pos[i] == row) add_row4(acc, pos_coeff(fx, i, row), fx.other + (size_t)i * fx.d, col);
    }
  }
  if (rs.out_bf16) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
    ((bf16x4_t*)out)[e] = __builtin_convertvector(acc, bf16x4_t);
  } else {
    ((f32x4*)out)[e] = acc;
  }
}
__global__ void __launch_bounds__(256) partial_reduce_tail_kernel(float* __restrict__ out, ReduceSrc rs, size_t beg, size_t n) {
  size_t e = beg + (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n) return;
  float acc = 0.f;
  for (int s = 0; s < rs.nsrc; s++)
    for (int k = 0; k < rs.count[s]; k++) acc += rs.ptr[s][(size_t)k * rs.stride[s] + e];
  if (rs.out_bf16) ((__bf16*)out)[e] = (__bf16)acc;
  else out[e] = acc;
}

// Fused mode: merge of what the splits of the online dQ walk left per anchor (reference, sum 2^(t - reference), and
// when the arg-max is asked for the true maximum with its first index) into lse2_i, the row loss and the arg-max, and
//   dQ_i = sum_s 2^(ref_s,i - lse2_i) part_s,i + (alpha / B) (p_{i r_i} - 1) p_{r_i}
// where part_s,i = (alpha / B) sum_{j in split s, j != r_i} 2^(t_ij - ref_s,i) p_j (Eq. 5; the positive's own term is
// formed here in fp32, so a softmax that has converged on the positive does not cancel in bf16).  Splits are
// combined in index order.  64 threads per anchor, 4 anchors per workgroup.
struct FinishArgs {
  const float* on_ref; const float* on_l; const float* on_best; const int* on_idx; const float* on_pos;
  const int32_t* pos_idx; const unsigned short* P;
  const float* part; size_t part_stride;
  int nsq, B, Pn, d, b_pad;
  float out_scale;
  float* lse2; int32_t* pos_pad; float* rowloss; float* lse_out; int32_t* argmax_out; float* dq;
  int dq_bf16;   // dq points to bf16 elements
  int32_t* inv; int* shared;   // an anchor per target and the "several anchors share a target" word (see PosFix)
};
__global__ void __launch_bounds__(256) online_finish_kernel(FinishArgs f) {
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (blockIdx.x == 0 && threadIdx.x == 0) *f.shared = 0;   // raised later by the dP walk's check
  if (i >= f.b_pad) return;
  if (i >= f.B) {
    if (lane == 0) { f.lse2[i] = INFINITY; f.pos_pad[i] = -1; }
    return;
  }
  // every load of the row's statistics is issued before the first result is needed
  float sl[16], sr[16];
#pragma unroll
  for (int s = 0; s < 16; s++) {
    const bool live = s < f.nsq;
    const size_t o = (size_t)(live ? s : 0) * f.B + i;
    sl[s] = live ? f.on_l[o] : 0.f; sr[s] = live ? f.on_ref[o] : -INFINITY;
  }
  const int r = f.pos_idx[i];
  const bool ok = (r >= 0 && r < f.Pn);
  const int r_safe = ok ? r : 0;
  const float pos = f.on_pos[i];
  float M = -INFINITY;
#pragma unroll
  for (int s = 0; s < 16; s++) M = fmaxf(M, sr[s]);
  float L = 0.f;
  if (M > -INFINITY) {
#pragma unroll
    for (int s = 0; s < 16; s++) L += sl[s] * exp2f(sr[s] - M);   // dead splits: 0 * 2^-inf = 0
  }
  const float l2 = M + log2f(L);
  if (lane == 0) {
    f.lse2[i] = l2;
    f.pos_pad[i] = r;
    f.rowloss[i] = ok ? (l2 - pos) * kLn2 : NAN;
    if (ok) f.inv[r] = i;
    if (f.lse_out) f.lse_out[i] = l2 * kLn2;
    if (f.argmax_out) {
      float bv = -INFINITY; int bi = 0x7fffffff;
      for (int s = 0; s < f.nsq; s++) {
        const float v = f.on_best[(size_t)s * f.B + i];
        const int idx = f.on_idx[(size_t)s * f.B + i];
        if (v > bv || (v == bv && idx < bi)) { bv = v; bi = idx; }
      }
      f.argmax_out[i] = bi;
    }
  }
  if (!f.dq) return;
  float w[16];
#pragma unroll
  for (int s = 0; s < 16; s++) w[s] = exp2f(sr[s] - l2);
  // coefficient of the positive: p_{i r_i} - 1
  const float cpos = ok ? f.out_scale * (exp2f(pos - l2) - 1.f) : 0.f;
  for (int c = lane; c < f.d / 4; c += 64) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 16; s++)
      if (s < f.nsq) acc += w[s] * ((const f32x4*)(f.part + (size_t)s * f.part_stride + (size_t)i * f.d))[c];
    const s16x4 pv = ((const s16x4*)(f.P + (size_t)r_safe * f.d))[c];
#pragma unroll
    for (int e = 0; e < 4; e++) acc[e] += cpos * bf2f((unsigned short)pv[e]);
    if (f.dq_bf16) {
      typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
      ((bf16x4_t*)((__bf16*)f.dq + (size_t)i * f.d))[c] = __builtin_convertvector(acc, bf16x4_t);
    } else {
      ((f32x4*)(f.dq + (size_t)i * f.d))[c] = acc;
    }
  }
}

hipError_t launch_online_finish(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  FinishArgs f{};
  f.on_ref = (const float*)(ws + pl.off_on_ref); f.on_best = (const float*)(ws + pl.off_part_m);
  f.on_l = (const float*)(ws + pl.off_part_l); f.on_idx = (const int*)(ws + pl.off_part_idx);
  f.on_pos = (const float*)(ws + pl.off_pos); f.pos_idx = a.pos_idx; f.P = (const unsigned short*)a.p;
  f.part = (const float*)(ws + pl.off_dq_part); f.part_stride = (size_t)a.B * a.d;
  f.nsq = pl.fz_nsq; f.B = a.B; f.Pn = a.P; f.d = a.d; f.b_pad = pl.b_pad;
  f.out_scale = a.alpha / (float)a.B * (a.grad_mul != 0.f ? a.grad_mul : 1.f);
  f.lse2 = (float*)(ws + pl.off_lse2); f.pos_pad = (int32_t*)(ws + pl.off_pos_pad); f.rowloss = (float*)(ws + pl.off_rowloss);
  f.lse_out = a.lse; f.argmax_out = a.argmax; f.dq = a.dq; f.dq_bf16 = (a.flags & GC_CACHE_BF16) ? 1 : 0;
  f.inv = (int32_t*)(ws + pl.off_inv); f.shared = (int*)(ws + pl.off_err) + 1;
  online_finish_kernel<<<(pl.b_pad + 3) / 4, 256, 0, a.stream>>>(f);
  return hipGetLastError();
}

static LossSum loss_sum_of(const LossArgs& a, const LossPlan& pl) {
  LossSum ls{};
  ls.rowloss = (const float*)(a.ws + pl.off_rowloss); ls.pos_idx = a.pos_idx; ls.B = a.B; ls.P = a.P;
  ls.loss = a.loss; ls.err = (int*)(a.ws + pl.off_err);
  return ls;
}

hipError_t launch_partial_reduce(float* out, const float* const* srcs, const int* counts, const size_t* strides,
                                 int nsrc, size_t n, hipStream_t stream, const LossArgs* loss_of, const LossPlan* pl,
                                 bool out_bf16, const PosFix* fix) {
  ReduceSrc rs{};
  rs.nsrc = nsrc;
  rs.out_bf16 = out_bf16 ? 1 : 0;
  for (int s = 0; s < nsrc; s++) { rs.ptr[s] = srcs[s]; rs.count[s] = counts[s]; rs.stride[s] = strides[s]; }
  LossSum ls{};
  if (loss_of) ls = loss_sum_of(*loss_of, *pl);
  PosFix fx{};
  if (fix) fx = *fix;
  if (fx.mode && (n % 4 || fx.d % 4)) return hipErrorInvalidValue;   // the term is added by the 4-element kernel only
  size_t n4 = n / 4;
  if (n4 || loss_of)
    partial_reduce_kernel<<<dim3((unsigned)((n4 + 255) / 256 + (loss_of ? 1 : 0))), 256, 0, stream>>>(out, rs, n4, ls, fx);
  if (n4 * 4 < n) partial_reduce_tail_kernel<<<1, 256, 0, stream>>>(out, rs, n4 * 4, n);
  return hipGetLastError();
}

template <typename T>
static hipError_t stats_generic_t(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  dim3 grid((a.B + GT - 1) / GT, pl.stat_splits);
  stats_generic_kernel<T><<<grid, 256, 0, a.stream>>>((const T*)a.q, (const T*)a.p, a.pos_idx, a.B, a.P, a.d,
                                                      a.alpha * kLog2e, (a.flags & GC_MASK_SELF) ? 1 : 0,
                                                      pl.stat_cols_per_split, (float*)(ws + pl.off_part_m),
                                                      (float*)(ws + pl.off_part_l), (int*)(ws + pl.off_part_idx),
                                                      (float*)(ws + pl.off_pos));
  return hipGetLastError();
}
hipError_t launch_stats_generic(const LossArgs& a, const LossPlan& pl) {
  return a.dt == GC_F32 ? stats_generic_t<float>(a, pl) : stats_generic_t<unsigned short>(a, pl);
}

hipError_t launch_loss_sum(const LossArgs& a, const LossPlan& pl) {
  loss_reduce_kernel<<<1, 1024, 0, a.stream>>>(loss_sum_of(a, pl));
  return hipGetLastError();
}

__global__ void __launch_bounds__(1024) sym_loss_reduce_kernel(LossSum l1, LossSum l2, float* loss) {
  __shared__ float red[1024];
  loss_sum_block<1024>(l1, red);   // thread 0 writes *l1.loss and *l1.err ...
  __syncthreads();
  loss_sum_block<1024>(l2, red);
  if (threadIdx.x == 0) {          // ... and reads them back itself
    if (loss) *loss = 0.5f * (*l1.loss + *l2.loss);
    if (*l2.err) *l1.err = *l2.err;
  }
}
hipError_t launch_sym_loss_sum(const LossArgs& a1, const LossArgs& a2, const LossPlan& pl, float* loss) {
  sym_loss_reduce_kernel<<<1, 1024, 0, a1.stream>>>(loss_sum_of(a1, pl), loss_sum_of(a2, pl), loss);
  return hipGetLastError();
}

hipError_t launch_stats_merge(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  auto merge = [&](auto lanes_tag) {
    constexpr int LANES = decltype(lanes_tag)::value;
    constexpr int ROWS = 256 / LANES;
    stats_merge_kernel<LANES><<<(pl.b_pad + ROWS - 1) / ROWS, 256, 0, a.stream>>>(
        (const float*)(ws + pl.off_part_m), (const float*)(ws + pl.off_part_l), (const int*)(ws + pl.off_part_idx),
        (const float*)(ws + pl.off_pos), a.pos_idx, a.B, a.P, pl.stat_splits, pl.b_pad, (float*)(ws + pl.off_lse2),
        (int32_t*)(ws + pl.off_pos_pad), (float*)(ws + pl.off_rowloss), a.lse, a.argmax,
        pl.use_mfma ? (int32_t*)(ws + pl.off_inv) : nullptr, pl.use_mfma ? (int*)(ws + pl.off_err) + 1 : nullptr);
  };
  if (pl.stat_splits <= 1) merge(std::integral_constant<int, 1>{});
  else if (pl.stat_splits <= 4) merge(std::integral_constant<int, 4>{});
  else if (pl.stat_splits <= 16) merge(std::integral_constant<int, 16>{});
  else merge(std::integral_constant<int, 64>{});
  // the sum of the row losses: by a launch of its own, unless a sum of gradient partials follows that carries it
  if (!a.loss_with_partials && !a.defer_loss_sum) loss_reduce_kernel<<<1, 1024, 0, a.stream>>>(loss_sum_of(a, pl));
  return hipGetLastError();
}

template <typename T>
static hipError_t grad_generic_t(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  const float* lse2 = (const float*)(ws + pl.off_lse2);
  const float alpha2 = a.alpha * kLog2e, osc = a.alpha / (float)a.B * (a.grad_mul != 0.f ? a.grad_mul : 1.f);
  const int ms = (a.flags & GC_MASK_SELF) ? 1 : 0;
  float* dq = a.dz ? (float*)(ws + pl.off_dq_part) : a.dq;
  float* dp = a.dz ? (float*)(ws + pl.off_dp_part) : a.dp;
  if (dq)
    grad_generic_kernel<T, true><<<(a.B + GT - 1) / GT, 256, 0, a.stream>>>((const T*)a.q, (const T*)a.p, a.pos_idx, lse2,
                                                                           a.B, a.P, a.d, alpha2, osc, ms, dq);
  if (dp)
    grad_generic_kernel<T, false><<<(a.P + GT - 1) / GT, 256, 0, a.stream>>>((const T*)a.q, (const T*)a.p, a.pos_idx, lse2,
                                                                            a.B, a.P, a.d, alpha2, osc, ms, dp);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  prof_mark_grad_kernel_done(a.stream);
  if (a.dz) {
    const float* srcs[2] = {dq, dp};
    int counts[2] = {1, 1};
    size_t strides[2] = {0, 0};
    return launch_partial_reduce(a.dz, srcs, counts, strides, 2, (size_t)a.B * a.d, a.stream);
  }
  return hipSuccess;
}
hipError_t launch_grad_generic(const LossArgs& a, const LossPlan& pl) {
  return a.dt == GC_F32 ? grad_generic_t<float>(a, pl) : grad_generic_t<unsigned short>(a, pl);
}

}  // namespace gc
