// Stand-in encoder y = GELU(x W1 + b1) W2 + b2 around the gradient cache: the graph-less forward of
// Step 1, the per-sub-batch re-encode and surrogate backward of Step 3 (the inner sums of Eq. 8 / 9)
// and the one-GPU driver that runs Steps 1-3.
//
// Every contraction is the same skinny-GEMM tile kernel: a workgroup (4 waves) produces a
// 32 x 128 tile of C = A * B with v_mfma_f32_32x32x16_bf16, each wave one 32 x 32 block, the
// k dimension staged through LDS 64 (or 32) at a time.  An operand is stored either with k
// contiguous ("KC": fragments are plain 16-byte LDS reads) or with its m / n index contiguous
// ("MN": fragments come from transposing ds_read_b64_tr_b16 loads).  The five uses:
//   H  = X  W1          A = X [rows][din]   KC      B = W1 [din][dh]   MN    +b1, GELU
//   Y  = A  W2          A = Act (fp32) [rows][dh] KC   B = W2 [dh][dout]  MN    +b2
//   dA = U  W2^T        A = U (fp32) [rows][dout] KC   B = W2 [dh][dout] KC   * GELU'(H), column sums -> db1
//   dW2 += Act^T U      A = Act (fp32) [rows][dh] MN   B = U (fp32) [rows][dout] MN   k = rows
//   dW1 += X^T dH       A = X [rows][din]   MN      B = dH (fp32) [rows][dh] MN    k = rows
// An fp32 operand (the cached gradient rows U, dH, and the activations kept for Step 3) is fed to the bf16 MFMA as hi + lo, two
// bf16 numbers per value and two MFMAs per step, so that it keeps ~16 mantissa bits: with only
// rows <= 32 terms per sum a single bf16 rounding (2^-9) would sit right at the error budget.
#include "gc_common.h"

namespace gc {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4m;

enum Layout { KC = 0, MN = 1 };
enum Epilogue { EP_GELU = 0, EP_BIAS = 1, EP_DH = 2, EP_ACC = 3 };

struct GemmArgs {
  const void* A; int lda;   // elements
  const void* B; int ldb;
  int M, N, K;              // logical sizes; M or K may be ragged (rows), N is a multiple of 128
  const unsigned short* bias;   // EP_GELU / EP_BIAS: [N] bf16
  float* H; int ldh;            // EP_GELU: optional fp32 pre-activation out; EP_DH: fp32 pre-activation in
  float* ActF;                  // EP_GELU: optional fp32 activation out (ldh)
  unsigned short* Cb; int ldc;  // bf16 output (EP_GELU: Act, EP_BIAS: Y)
  float* Cf;                    // EP_ACC: fp32 accumulator, += ; EP_DH: dH out (fp32); ldc
  float* colsum;                // EP_DH: db1 [N] += column sums of the tile; EP_ACC: db2 [N] += column sums of B (m-tile 0 only)
};

__device__ __forceinline__ float gelu_f(float h) { return 0.5f * h * (1.f + erff(h * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_prime_f(float h) {
  return 0.5f * (1.f + erff(h * 0.70710678118654752f)) + h * 0.3989422804014327f * __expf(-0.5f * h * h);
}

// 8 consecutive elements starting at index idx as packed bf16.  fp32 source: hi = bf16(v) and
// lo = bf16(v - hi); bf16 source: lo is unused.
template <bool F32>
__device__ __forceinline__ void load8(const void* base, size_t idx, bool live, u32x4& hi, u32x4& lo) {
  hi = u32x4{0u, 0u, 0u, 0u};
  lo = hi;
  if (!live) return;
  if (F32) {
    const f32x4* p = (const f32x4*)((const float*)base + idx);
    f32x4 a = p[0], b = p[1];
    typedef __attribute__((ext_vector_type(8))) float f32x8;
    f32x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    bf16x8 h = __builtin_convertvector(v, bf16x8);
    f32x8 r = v - __builtin_convertvector(h, f32x8);
    hi = __builtin_bit_cast(u32x4, h);
    lo = __builtin_bit_cast(u32x4, __builtin_convertvector(r, bf16x8));
  } else {
    hi = *(const u32x4*)((const unsigned short*)base + idx);
  }
}

template <int KCH, Layout AL, Layout BL, bool A_F32, bool B_F32, Epilogue EP>
__global__ void __launch_bounds__(256) mlp_gemm_kernel(GemmArgs g) {
  // LDS tiles (bf16 elements).  KC layout: [rows of m/n][KCH + 8]; MN layout: [KCH rows of k][width + 8]
  constexpr int A_LD = (AL == KC) ? KCH + 8 : 32 + 8;
  constexpr int A_ROWS = (AL == KC) ? 32 : KCH;
  constexpr int B_LD = (BL == KC) ? KCH + 8 : 128 + 8;
  constexpr int B_ROWS = (BL == KC) ? 128 : KCH;
  __shared__ __attribute__((aligned(16))) unsigned short As[(A_F32 ? 2 : 1) * A_ROWS * A_LD];  // [hi | lo]
  __shared__ __attribute__((aligned(16))) unsigned short Bs[(B_F32 ? 2 : 1) * B_ROWS * B_LD];
  constexpr int A_LO = A_ROWS * A_LD, B_LO = B_ROWS * B_LD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ln = lane & 31;
  const int n0 = blockIdx.x * 128, m0 = blockIdx.y * 32;

  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f;

  for (int k0 = 0; k0 < g.K; k0 += KCH) {
    // ---- stage A ---------------------------------------------------------------------------
    if (AL == KC) {  // memory A[m][k]: 32 rows x KCH, 16-byte chunks
      constexpr int CH = KCH / 8;
      for (int c = tid; c < 32 * CH; c += 256) {
        const int r = c / CH, cc = c % CH;
        const int m = min(m0 + r, g.M - 1);
        u32x4 vh, vl;
        load8<A_F32>(g.A, (size_t)m * g.lda + k0 + cc * 8, true, vh, vl);
        *(u32x4*)(As + r * A_LD + cc * 8) = vh;
        if (A_F32) *(u32x4*)(As + A_LO + r * A_LD + cc * 8) = vl;
      }
    } else {         // memory A[k][m]: KCH rows x 32
      for (int c = tid; c < KCH * 4; c += 256) {
        const int r = c / 4, cc = c % 4;
        u32x4 vh, vl;
        load8<A_F32>(g.A, (size_t)(k0 + r) * g.lda + m0 + cc * 8, k0 + r < g.K, vh, vl);
        *(u32x4*)(As + r * A_LD + cc * 8) = vh;
        if (A_F32) *(u32x4*)(As + A_LO + r * A_LD + cc * 8) = vl;
      }
    }
    // ---- stage B ---------------------------------------------------------------------------
    if (BL == KC) {  // memory B[n][k]: 128 rows x KCH
      constexpr int CH = KCH / 8;
      for (int c = tid; c < 128 * CH; c += 256) {
        const int r = c / CH, cc = c % CH;
        u32x4 vh, vl;
        load8<B_F32>(g.B, (size_t)(n0 + r) * g.ldb + k0 + cc * 8, true, vh, vl);
        *(u32x4*)(Bs + r * B_LD + cc * 8) = vh;
        if (B_F32) *(u32x4*)(Bs + B_LO + r * B_LD + cc * 8) = vl;
      }
    } else {         // memory B[k][n]: KCH rows x 128
      for (int c = tid; c < KCH * 16; c += 256) {
        const int r = c / 16, cc = c % 16;
        u32x4 vh, vl;
        load8<B_F32>(g.B, (size_t)(k0 + r) * g.ldb + n0 + cc * 8, k0 + r < g.K, vh, vl);
        *(u32x4*)(Bs + r * B_LD + cc * 8) = vh;
        if (B_F32) *(u32x4*)(Bs + B_LO + r * B_LD + cc * 8) = vl;
      }
    }
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KCH / 16; ks++) {
      auto a_frag = [&](const unsigned short* T) -> bf16x8 {
        if (AL == KC) return *(const bf16x8*)(T + ln * A_LD + 16 * ks + 8 * h);
        const unsigned short* p = T + (16 * ks + 8 * h + ((lane & 15) >> 2)) * A_LD + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)p);
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)(p + 4 * A_LD));
        s16x8 t = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, t);
      };
      auto b_frag = [&](const unsigned short* T) -> bf16x8 {
        if (BL == KC) return *(const bf16x8*)(T + (wave * 32 + ln) * B_LD + 16 * ks + 8 * h);
        const unsigned short* p = T + (16 * ks + 8 * h + ((lane & 15) >> 2)) * B_LD + wave * 32 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)p);
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)(p + 4 * B_LD));
        s16x8 t = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, t);
      };
      const bf16x8 af = a_frag(As), bfv = b_frag(Bs);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfv, acc, 0, 0, 0);
      if (A_F32) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_frag(As + A_LO), bfv, acc, 0, 0, 0);
      if (B_F32) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, b_frag(Bs + B_LO), acc, 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds column n, rows m0 + 8 (r / 4) + 4 h + r % 4 -------------------------------------
  const int n = n0 + wave * 32 + ln;
  if (EP == EP_GELU || EP == EP_BIAS) {
    const float b = bf2f(g.bias[n]);
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (m < g.M) {
        const float v = acc[r] + b;
        if (EP == EP_GELU) {
          const float a = gelu_f(v);
          if (g.H) g.H[(size_t)m * g.ldh + n] = v;
          if (g.ActF) g.ActF[(size_t)m * g.ldh + n] = a;
          if (g.Cb) g.Cb[(size_t)m * g.ldc + n] = f2bf(a);
        } else {
          g.Cb[(size_t)m * g.ldc + n] = f2bf(v);
        }
      }
    }
  } else if (EP == EP_DH) {
    float s = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (m < g.M) {
        const float v = acc[r] * gelu_prime_f(g.H[(size_t)m * g.ldh + n]);
        g.Cf[(size_t)m * g.ldc + n] = v;
        s += v;
      }
    }
    s += __shfl_xor(s, 32);
    // one workgroup row (blockIdx.y) at a time would race on db1: the launcher runs EP_DH with a
    // single m-tile per launch row, see launch_dh
    if (h == 0) g.colsum[n] += s;
  } else {  // EP_ACC
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + 8 * (r >> 2) + 4 * h + (r & 3);
      if (m < g.M) g.Cf[(size_t)m * g.ldc + n] += acc[r];
    }
    if (g.colsum && blockIdx.y == 0 && tid < 128) {  // db2 += column sums of the fp32 B operand (k = rows)
      float s = 0.f;
      for (int k = 0; k < g.K; k++) s += ((const float*)g.B)[(size_t)k * g.ldb + n0 + tid];
      g.colsum[n0 + tid] += s;
    }
  }
}

struct MlpWs {
  float* H;             // [rows][dh] fp32 pre-activations
  float* ActF;          // [rows][dh] fp32 GELU(H)
  float* dH;            // [rows][dh] fp32
  size_t total;
};

static inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

static MlpWs carve_mlp_ws(char* base, int rows, int dh) {
  MlpWs w{};
  size_t off = 0;
  w.H = (float*)(base + off); off += up256((size_t)rows * dh * 4);
  w.ActF = (float*)(base + off); off += up256((size_t)rows * dh * 4);
  w.dH = (float*)(base + off); off += up256((size_t)rows * dh * 4);
  w.total = off;
  return w;
}

static int check_mlp_params(const gc_mlp_params* w) {
  if (!w) return GC_ERR_NULL;
  if (!w->W1 || !w->b1 || !w->W2 || !w->b2) return GC_ERR_NULL;
  if (w->din < 64 || w->dh < 128 || w->dout < 128) return GC_ERR_SHAPE;
  if (w->din % 64 || w->dh % 128 || w->dout % 128) return GC_ERR_UNSUPPORTED;
  if (w->din > (1 << 20) || w->dh > (1 << 20) || w->dout > (1 << 20)) return GC_ERR_SHAPE;
  return GC_OK;
}

// forward of one sub-batch; keepH: also write the fp32 pre-activations (Step 3)
static hipError_t mlp_forward(const void* x, int rows, const gc_mlp_params* w, const MlpWs& ws, bool keepH, void* y,
                              hipStream_t s) {
  GemmArgs g{};
  g.A = x; g.lda = w->din; g.B = w->W1; g.ldb = w->dh; g.M = rows; g.N = w->dh; g.K = w->din;
  g.bias = (const unsigned short*)w->b1; g.H = keepH ? ws.H : nullptr; g.ActF = ws.ActF; g.ldh = w->dh;
  g.Cb = nullptr; g.ldc = w->dh;
  mlp_gemm_kernel<64, KC, MN, false, false, EP_GELU><<<dim3(w->dh / 128, (rows + 31) / 32), 256, 0, s>>>(g);
  if (y) {
    GemmArgs g2{};
    g2.A = ws.ActF; g2.lda = w->dh; g2.B = w->W2; g2.ldb = w->dout; g2.M = rows; g2.N = w->dout; g2.K = w->dh;
    g2.bias = (const unsigned short*)w->b2; g2.Cb = (unsigned short*)y; g2.ldc = w->dout;
    mlp_gemm_kernel<64, KC, MN, true, false, EP_BIAS><<<dim3(w->dout / 128, (rows + 31) / 32), 256, 0, s>>>(g2);
  }
  return hipGetLastError();
}

static hipError_t mlp_backward(const void* x, int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc,
                               const MlpWs& ws, hipStream_t s) {
  hipError_t e = mlp_forward(x, rows, w, ws, true, nullptr, s);  // re-encode keeping H and Act
  if (e != hipSuccess) return e;
  // dA = U W2^T, dH = dA * GELU'(H), db1 += column sums.  One launch per 32-row block so that the
  // += on db1 has a single writer per column at any time (launches on one stream run in order).
  for (int mb = 0; mb < rows; mb += 32) {
    const int mrows = rows - mb < 32 ? rows - mb : 32;
    GemmArgs g{};
    g.A = u + (size_t)mb * w->dout; g.lda = w->dout; g.B = w->W2; g.ldb = w->dout; g.M = mrows; g.N = w->dh; g.K = w->dout;
    g.H = ws.H + (size_t)mb * w->dh; g.ldh = w->dh; g.Cf = ws.dH + (size_t)mb * w->dh; g.ldc = w->dh; g.colsum = acc->db1;
    mlp_gemm_kernel<64, KC, KC, true, false, EP_DH><<<dim3(w->dh / 128, 1), 256, 0, s>>>(g);
  }
  {  // dW2 += Act^T U, db2 += column sums of U
    GemmArgs g{};
    g.A = ws.ActF; g.lda = w->dh; g.B = u; g.ldb = w->dout; g.M = w->dh; g.N = w->dout; g.K = rows;
    g.Cf = acc->dW2; g.ldc = w->dout; g.colsum = acc->db2;
    mlp_gemm_kernel<32, MN, MN, true, true, EP_ACC><<<dim3(w->dout / 128, w->dh / 32), 256, 0, s>>>(g);
  }
  {  // dW1 += X^T dH
    GemmArgs g{};
    g.A = x; g.lda = w->din; g.B = ws.dH; g.ldb = w->dh; g.M = w->din; g.N = w->dh; g.K = rows;
    g.Cf = acc->dW1; g.ldc = w->dh; g.colsum = nullptr;
    mlp_gemm_kernel<32, MN, MN, false, true, EP_ACC><<<dim3(w->dh / 128, w->din / 32), 256, 0, s>>>(g);
  }
  return hipGetLastError();
}

struct StepWs {
  size_t off_q, off_p, off_dq, off_dp, off_loss, off_mlp, total;
  size_t loss_bytes, mlp_bytes;
};

static StepWs plan_step(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w) {
  StepWs s{};
  size_t off = 0;
  auto take = [&](size_t b) { size_t o = off; off = up256(off + b); return o; };
  s.off_q = take((size_t)B * w->dout * 2);
  s.off_p = take((size_t)P * w->dout * 2);
  s.off_dq = take((size_t)B * w->dout * 4);
  s.off_dp = take((size_t)P * w->dout * 4);
  s.loss_bytes = make_loss_plan(B, P, w->dout, GC_BF16, false).total;
  s.off_loss = take(s.loss_bytes);
  const int cmax = chunk_q > chunk_p ? chunk_q : chunk_p;
  s.mlp_bytes = carve_mlp_ws(nullptr, cmax, w->dh).total;
  s.off_mlp = take(s.mlp_bytes);
  s.total = off;
  return s;
}

}  // namespace gc

using namespace gc;

extern "C" {

size_t gc_mlp_workspace_bytes(int rows, const gc_mlp_params* w) {
  if (rows < 1 || check_mlp_params(w) != GC_OK) return 0;
  return carve_mlp_ws(nullptr, rows, w->dh).total;
}

int gc_mlp_forward_nograd_bf16(const void* x, int rows, const gc_mlp_params* w, void* y, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (!x || !y) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (rows < 1 || rows > (1 << 24)) return GC_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < carve_mlp_ws(nullptr, rows, w->dh).total)
    return GC_ERR_WORKSPACE;
  const MlpWs ws = carve_mlp_ws((char*)workspace, rows, w->dh);
  return mlp_forward(x, rows, w, ws, false, y, (hipStream_t)stream) == hipSuccess ? GC_OK : GC_ERR_HIP;
}

int gc_chunk_surrogate_backward_bf16(const void* x_chunk, int rows, const gc_mlp_params* w, const float* cached_grad_rows,
                                     const gc_mlp_grads* acc, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x_chunk || !cached_grad_rows || !acc) return GC_ERR_NULL;
  if (!acc->dW1 || !acc->db1 || !acc->dW2 || !acc->db2) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (rows < 1 || rows > (1 << 24)) return GC_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < carve_mlp_ws(nullptr, rows, w->dh).total)
    return GC_ERR_WORKSPACE;
  const MlpWs ws = carve_mlp_ws((char*)workspace, rows, w->dh);
  return mlp_backward(x_chunk, rows, w, cached_grad_rows, acc, ws, (hipStream_t)stream) == hipSuccess ? GC_OK : GC_ERR_HIP;
}

size_t gc_step_mlp_workspace_bytes(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w) {
  if (B < 1 || P < 1 || chunk_q < 1 || chunk_p < 1 || check_mlp_params(w) != GC_OK) return 0;
  return plan_step(B, P, chunk_q, chunk_p, w).total;
}

int gc_step_mlp_bf16(const void* x_q, int B, const void* x_p, int P, const int32_t* pos_idx, int chunk_q, int chunk_p,
                     const gc_mlp_params* w, float scale, float temp, float* loss, const gc_mlp_grads* grads, void* q_rep,
                     void* p_rep, float* dq, float* dp, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x_q || !x_p || !pos_idx || !loss || !grads) return GC_ERR_NULL;
  if (!grads->dW1 || !grads->db1 || !grads->dW2 || !grads->db2) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (B < 1 || P < 1 || chunk_q < 1 || chunk_p < 1 || B > (1 << 24) || P > (1 << 24)) return GC_ERR_SHAPE;
  if (!(scale > 0.f) || !(temp > 0.f) || !(scale / temp > 0.f) || !(scale / temp < 3.0e38f)) return GC_ERR_SHAPE;
  const StepWs sw = plan_step(B, P, chunk_q, chunk_p, w);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sw.total) return GC_ERR_WORKSPACE;
  char* base = (char*)workspace;
  hipStream_t s = (hipStream_t)stream;
  unsigned short* Q = q_rep ? (unsigned short*)q_rep : (unsigned short*)(base + sw.off_q);
  unsigned short* Pm = p_rep ? (unsigned short*)p_rep : (unsigned short*)(base + sw.off_p);
  float* dQ = dq ? dq : (float*)(base + sw.off_dq);
  float* dP = dp ? dp : (float*)(base + sw.off_dp);
  const int cmax = chunk_q > chunk_p ? chunk_q : chunk_p;
  const MlpWs mw = carve_mlp_ws(base + sw.off_mlp, cmax, w->dh);
  // Step 1: graph-less forward, sub-batch by sub-batch, representations kept
  for (int a = 0; a < B; a += chunk_q) {
    const int rows = B - a < chunk_q ? B - a : chunk_q;
    if (mlp_forward((const unsigned short*)x_q + (size_t)a * w->din, rows, w, mw, false, Q + (size_t)a * w->dout, s) != hipSuccess)
      return GC_ERR_HIP;
  }
  for (int a = 0; a < P; a += chunk_p) {
    const int rows = P - a < chunk_p ? P - a : chunk_p;
    if (mlp_forward((const unsigned short*)x_p + (size_t)a * w->din, rows, w, mw, false, Pm + (size_t)a * w->dout, s) != hipSuccess)
      return GC_ERR_HIP;
  }
  // Step 2: loss and the representation gradient cache
  rc = gc_loss_and_rep_grad_ex(GC_BF16, Q, Pm, pos_idx, B, P, w->dout, scale, temp, 0, loss, dQ, dP, nullptr, nullptr,
                               base + sw.off_loss, sw.loss_bytes, stream);
  if (rc != GC_OK) return rc;
  // Step 3: per sub-batch re-encode and backward of the cached rows, gradients accumulated in index order
  for (int a = 0; a < B; a += chunk_q) {
    const int rows = B - a < chunk_q ? B - a : chunk_q;
    if (mlp_backward((const unsigned short*)x_q + (size_t)a * w->din, rows, w, dQ + (size_t)a * w->dout, grads, mw, s) != hipSuccess)
      return GC_ERR_HIP;
  }
  for (int a = 0; a < P; a += chunk_p) {
    const int rows = P - a < chunk_p ? P - a : chunk_p;
    if (mlp_backward((const unsigned short*)x_p + (size_t)a * w->din, rows, w, dP + (size_t)a * w->dout, grads, mw, s) != hipSuccess)
      return GC_ERR_HIP;
  }
  return GC_OK;
}

}  // extern "C"
