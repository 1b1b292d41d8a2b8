// Stand-in encoder y = GELU(x W1 + b1) W2 + b2 around the gradient cache: the graph-less forward of
// Step 1, the per-sub-batch re-encode and surrogate backward of Step 3 (the inner sums of Eq. 8 / 9)
// and the one-GPU driver that runs Steps 1-3.
//
// A sub-batch has few rows (32 at the paper's setting), so every contraction of Step 3 is skinny and is bound by
// how fast the weights and the gradient accumulators move, not by the MFMAs.  Three kernels:
//
// mlp_skinny_kernel: C[32 x 32 per workgroup] = A[rows x K] * Bt[N x K]^T, both operands with k contiguous, so
//   every MFMA fragment is a plain 16-byte global load and nothing is staged through LDS.  The four waves of a
//   workgroup split K (64-wide chunks, round-robin), keep two to four chunks of loads in flight each, and sum their
//   partial tiles through LDS in a fixed order.  Used for
//     H  = X  W1  (+b1, GELU)              Bt = W1^T [dh][din]   (transposed copy, made once per call)
//     Y  = Act W2 (+b2)                    Bt = W2^T [dout][dh]  (transposed copy)      A = Act, fp32
//     dA = U  W2^T, dH = dA * GELU'(H)     Bt = W2 [dh][dout] as stored                 A = U, fp32
// mlp_wgrad_kernel: the weight-gradient contractions, whose k index is the row of the sub-batch (the slow index
//   of both operands in memory): 64 x 128 tiles, operands through LDS (loaded a 32-row chunk ahead) and transposing
//   ds_read_b64_tr_b16 loads, fp32 accumulators in HBM updated in place (+=)
//     dW2 += Act^T U      A = Act (fp32) [rows][dh]    B = U (fp32) [rows][dout]   db2 += column sums of U
//     dW1 += X^T dH       A = X [rows][din]            B = dH (fp32) [rows][dh]    db1 += column sums of dH
// gemm_nt_kernel: the same product as the skinny kernel for MANY rows at once (the graph-less forward of Step 1 over
//   up to 2048 rows, the batch-wide projections of the distance functions): 64 x 128 or 128 x 128 tiles, both
//   operands through LDS, optionally with the contraction cut into ranges (split-K).
// An fp32 operand (the cached gradient rows U, dH, and the activations kept for Step 3) is fed to the bf16 MFMA as
// hi + lo, two bf16 numbers per value and two MFMAs per step, so that it keeps ~16 mantissa bits: with only
// rows <= 32 terms per sum a single bf16 rounding (2^-9) would sit right at the error budget.
#include "gc_common.h"
#include <mutex>
#include <vector>
#include <string.h>

namespace gc {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4m;

enum Epilogue { EP_GELU = 0, EP_BIAS = 1, EP_DH = 2, EP_PLAIN = 3 };

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

// C[M x N] += A^T B over the rows of a sub-batch: A [K][M] (bf16 or fp32), B [K][N] fp32, C fp32 in HBM.
struct WgradArgs {
  const void* A; int lda;   // elements
  const void* B; int ldb;   // fp32, or bf16 where the kernel is instantiated with B_F32 = false
  int M, N, K;              // M a multiple of 64 (WG_M), N a multiple of 128, K = rows of the sub-batch (any)
  float* C; int ldc;        // += in place (one workgroup per tile: single writer)
  float* colsum;            // optional: [N] += column sums of B (db2; written by the m-tile 0 workgroups)
  int colsum_rows;          // the column sums are added colsum_rows rows at a time (0: all K rows in one sum): a launch
                            // that covers several sub-batches adds them one sub-batch after the other, as single launches do
};

// a workgroup's tile of C is WG_M x 128 (two 32-row MFMA tiles that share the B operand in LDS)
constexpr int WG_M = 64;
// LDS tiles (bf16): [k rows][width + 32], hi then lo part.  Rows are padded by 64 bytes (row stride = 64 mod 128): the
// transposing reads (four consecutive k rows per 16 lanes, again four rows further on) then show no bank conflicts
// (SQ_LDS_BANK_CONFLICT 0; with pads of 16, 32, 48 or 80 bytes a quarter to a half of the LDS cycles were conflicts)
constexpr int WG_KCH = 32, WG_A_LD = WG_M + 32, WG_B_LD = 128 + 32;

// raw 8 consecutive elements (one 16-byte load, two for fp32), and their conversion to packed bf16 hi (+ lo) later:
// between the two a kernel can do other work while the load is in flight
template <bool F32>
struct Raw8 { u32x4 v[F32 ? 2 : 1]; };
template <bool F32>
__device__ __forceinline__ void fetch8(const void* base, size_t idx, bool live, Raw8<F32>& r) {
#pragma unroll
  for (int i = 0; i < (F32 ? 2 : 1); i++) r.v[i] = u32x4{0u, 0u, 0u, 0u};
  if (!live) return;
#pragma unroll
  for (int i = 0; i < (F32 ? 2 : 1); i++) r.v[i] = *(const u32x4*)((const char*)base + idx * (F32 ? 4 : 2) + 16 * i);
}
template <bool F32>
__device__ __forceinline__ void split8(const Raw8<F32>& r, u32x4& hi, u32x4& lo) {
  if (F32) {
    typedef __attribute__((ext_vector_type(8))) float f32x8;
    const f32x4 a = __builtin_bit_cast(f32x4, r.v[0]), b = __builtin_bit_cast(f32x4, r.v[F32 ? 1 : 0]);
    const f32x8 v = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
    const bf16x8 h = __builtin_convertvector(v, bf16x8);
    const f32x8 rest = v - __builtin_convertvector(h, f32x8);
    hi = __builtin_bit_cast(u32x4, h);
    lo = __builtin_bit_cast(u32x4, __builtin_convertvector(rest, bf16x8));
  } else {
    hi = r.v[0];
    lo = u32x4{0u, 0u, 0u, 0u};
  }
}

// ACCUM: the tile starts from the value of C in HBM (+=); otherwise from zero (C is written, not read)
template <bool A_F32, bool B_F32 = true, bool ACCUM = true>
__device__ __forceinline__ void wgrad_tile(const WgradArgs& g, int bx, int by, unsigned short* As, unsigned short* Bs) {
  constexpr int KCH = WG_KCH, A_LD = WG_A_LD, B_LD = WG_B_LD;
  constexpr int A_LO = KCH * A_LD, B_LO = KCH * B_LD;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ln = lane & 31;
  const int n0 = bx * 128, m0 = by * WG_M;

  // the accumulator tile starts from its current value in HBM (read issued first: it is the longest wait);
  // lane holds column n, rows m0 + 32 mt + 8 (r / 4) + 4 h + r % 4
  const int n = n0 + wave * 32 + ln;
  f32x16 acc[2];
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + 32 * mt + 8 * (r >> 2) + 4 * h + (r & 3);
      acc[mt][r] = (ACCUM && m < g.M) ? g.C[(size_t)m * g.ldc + n] : 0.f;
    }

  // the 32 rows of a k-chunk: one 8-element piece of A and two of B per thread, loaded a chunk ahead of their use
  static_assert(KCH * (WG_M / 8) == 256 && KCH * 16 == 512, "staging pieces per thread");
  const int ar = tid / (WG_M / 8), ac = tid % (WG_M / 8);
  Raw8<A_F32> ra;
  Raw8<B_F32> rb[2];
  auto fetch = [&](int k0) __attribute__((always_inline)) {
    fetch8<A_F32>(g.A, (size_t)(k0 + ar) * g.lda + m0 + ac * 8, k0 + ar < g.K, ra);   // A[k][m0 .. m0 + WG_M - 1]
#pragma unroll
    for (int i = 0; i < 2; i++) {                                                     // B[k][n0 .. n0 + 127]
      const int c = tid + 256 * i, r = c / 16, cc = c % 16;
      fetch8<B_F32>(g.B, (size_t)(k0 + r) * g.ldb + n0 + cc * 8, k0 + r < g.K, rb[i]);
    }
  };
  fetch(0);
  for (int k0 = 0; k0 < g.K; k0 += KCH) {
    {
      u32x4 vh, vl;
      split8<A_F32>(ra, vh, vl);
      *(u32x4*)(As + ar * A_LD + ac * 8) = vh;
      if (A_F32) *(u32x4*)(As + A_LO + ar * A_LD + ac * 8) = vl;
#pragma unroll
      for (int i = 0; i < 2; i++) {
        const int c = tid + 256 * i, r = c / 16, cc = c % 16;
        split8<B_F32>(rb[i], vh, vl);
        *(u32x4*)(Bs + r * B_LD + cc * 8) = vh;
        if (B_F32) *(u32x4*)(Bs + B_LO + r * B_LD + cc * 8) = vl;
      }
    }
    if (k0 + KCH < g.K) fetch(k0 + KCH);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < KCH / 16; ks++) {
      // both operands have k as the slow index in LDS: transposing reads
      auto frag = [&](const unsigned short* T, int ld, int col0) -> bf16x8 {
        const unsigned short* p = T + (16 * ks + 8 * h + ((lane & 15) >> 2)) * ld + col0 + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)p);
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4m*)(p + 4 * ld));
        s16x8 t = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, t);
      };
      const bf16x8 bfv = frag(Bs, B_LD, wave * 32);
      bf16x8 bfl = bfv;
      if (B_F32) bfl = frag(Bs + B_LO, B_LD, wave * 32);
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
        const bf16x8 af = frag(As, A_LD, 32 * mt);
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfv, acc[mt], 0, 0, 0);
        if (A_F32) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(As + A_LO, A_LD, 32 * mt), bfv, acc[mt], 0, 0, 0);
        if (B_F32) acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, bfl, acc[mt], 0, 0, 0);
      }
    }
    __syncthreads();
  }
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int m = m0 + 32 * mt + 8 * (r >> 2) + 4 * h + (r & 3);
      if (m < g.M) g.C[(size_t)m * g.ldc + n] = acc[mt][r];
    }
  if (g.colsum && by == 0 && tid < 128) {
    const int step = g.colsum_rows > 0 ? g.colsum_rows : g.K;
    const float* col = (const float*)g.B + n0 + tid;   // (fp32 B only)
    float total = g.colsum[n0 + tid];
    for (int k0 = 0; k0 < g.K; k0 += step) {
      const int k1 = min(g.K, k0 + step);
      float s = 0.f;
      for (int k = k0; k < k1; k += 8) {   // eight loads in flight, added in row order
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = (k + j < k1) ? col[(size_t)(k + j) * g.ldb] : 0.f;
#pragma unroll
        for (int j = 0; j < 8; j++)
          if (k + j < k1) s += v[j];
      }
      total += s;
    }
    g.colsum[n0 + tid] = total;
  }
}

// both weight gradients of a sub-batch in one launch: workgroups [0, n2) take the tiles of dW2 (A = Act, fp32),
// the rest the tiles of dW1 (A = X, bf16)
__global__ void __launch_bounds__(256) mlp_wgrad_kernel(WgradArgs g2, WgradArgs g1, int n2) {
  __shared__ __attribute__((aligned(16))) unsigned short As[2 * WG_KCH * WG_A_LD];
  __shared__ __attribute__((aligned(16))) unsigned short Bs[2 * WG_KCH * WG_B_LD];
  const int id = blockIdx.x;
  if (id < n2) {
    const int nb = g2.N / 128;
    wgrad_tile<true>(g2, id % nb, id / nb, As, Bs);
  } else {
    const int nb = g1.N / 128;
    wgrad_tile<false>(g1, (id - n2) % nb, (id - n2) / nb, As, Bs);
  }
}

// C = A^T B with the rows (K) cut into slices: workgroup (tile, slice) adds its slice's product to partial s of C
// (g.C + s * M * ldc, written whole: one workgroup per tile and slice), which a fixed-order sum combines afterwards.  A bf16.
template <bool A_F32, bool B_F32>
__global__ void __launch_bounds__(256) wgrad_splitk_kernel(WgradArgs g, int rows_per_slice) {
  __shared__ __attribute__((aligned(16))) unsigned short As[2 * WG_KCH * WG_A_LD];
  __shared__ __attribute__((aligned(16))) unsigned short Bs[2 * WG_KCH * WG_B_LD];
  const int nb = g.N / 128, tiles = nb * (g.M / WG_M);
  const int tile = blockIdx.x % tiles, slice = blockIdx.x / tiles;
  const int k0 = slice * rows_per_slice;
  WgradArgs s = g;
  s.A = (const char*)g.A + (size_t)k0 * g.lda * (A_F32 ? 4 : 2);
  s.B = (const char*)g.B + (size_t)k0 * g.ldb * (B_F32 ? 4 : 2);
  s.K = min(rows_per_slice, g.K - k0);
  s.C = g.C + (size_t)slice * g.M * g.ldc;
  s.colsum = nullptr;
  wgrad_tile<A_F32, B_F32, false>(s, tile % nb, tile / nb, As, Bs);
}

// ---------------------------------------------------------------------------------------------------
struct SkinnyArgs {
  const void* A; int lda;            // [M][K], bf16 or fp32
  const unsigned short* Bt; int ldb; // [N][K] bf16
  int M, N, K;                       // M may be ragged; N a multiple of 32, K a multiple of 64
  const unsigned short* bias;        // EP_GELU / EP_BIAS: [N] bf16
  float* H; int ldh;                 // EP_GELU: optional fp32 pre-activation out; EP_DH: fp32 pre-activation in
  float* ActF;                       // EP_GELU: fp32 activation out (ldh)
  unsigned short* Cb; int ldc;       // EP_BIAS: bf16 output; EP_PLAIN: bf16 output if set
  float* Cf;                         // EP_DH: dH out (fp32, ldc); EP_PLAIN: fp32 output if Cb is not set
  float plain_mul;                   // EP_PLAIN: factor on the product (0 means 1)
};

typedef float SkinnyRed[32][33];   // one partial tile; a workgroup holds four

// one 32 x 32 output tile (n-tile bx, m-tile by); red: the workgroup's four partial tiles in LDS;
// PD: 64-wide chunks of loads in flight per wave (registers against latency)
template <bool A_F32, Epilogue EP, int PD>
__device__ __forceinline__ void skinny_tile(const SkinnyArgs& g, int bx, int by, SkinnyRed* red) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ln = lane & 31;
  const int n0 = bx * 32, m0 = by * 32;
  const int nch = g.K / 64;
  // lane (ln, h) holds elements 32 h .. 32 h + 31 of each 64-wide chunk of row ln of A and of Bt; MFMA j of a
  // chunk contracts elements 8 j .. 8 j + 7 of both half-chunks (any order of k works if both operands share it)
  constexpr int AE = A_F32 ? 4 : 2;
  constexpr int AV = A_F32 ? 8 : 4;   // 16-byte loads per chunk for A
  const int m = min(m0 + ln, g.M - 1);
  const char* ap = (const char*)g.A + ((size_t)m * g.lda + 32 * h) * AE;
  const char* bp = (const char*)(g.Bt + (size_t)(n0 + ln) * g.ldb + 32 * h);
  u32x4 fa[PD][AV], fb[PD][4];
  auto issue = [&](int slot, int c) __attribute__((always_inline)) {
#pragma unroll
    for (int v = 0; v < AV; v++) fa[slot][v] = *(const u32x4*)(ap + (size_t)c * 64 * AE + 16 * v);
#pragma unroll
    for (int v = 0; v < 4; v++) fb[slot][v] = *(const u32x4*)(bp + (size_t)c * 128 + 16 * v);
  };
  f32x16 acc;
#pragma unroll
  for (int r = 0; r < 16; r++) acc[r] = 0.f;
#pragma unroll
  for (int sl = 0; sl < PD; sl++)
    if (wave + 4 * sl < nch) issue(sl, wave + 4 * sl);
  for (int base = wave; base < nch; base += 4 * PD) {
#pragma unroll
    for (int sl = 0; sl < PD; sl++) {
      const int c = base + 4 * sl;
      if (c < nch) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, fb[sl][j]);
          if (A_F32) {
            typedef __attribute__((ext_vector_type(8))) float f32x8;
            const f32x4 x0 = __builtin_bit_cast(f32x4, fa[sl][(2 * j) % AV]), x1 = __builtin_bit_cast(f32x4, fa[sl][(2 * j + 1) % AV]);
            const f32x8 v = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
            const bf16x8 hi = __builtin_convertvector(v, bf16x8);
            const bf16x8 lo = __builtin_convertvector(v - __builtin_convertvector(hi, f32x8), bf16x8);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hi, bv, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo, bv, acc, 0, 0, 0);
          } else {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[sl][j % AV]), bv, acc, 0, 0, 0);
          }
        }
        if (c + 4 * PD < nch) issue(sl, c + 4 * PD);
      }
    }
  }
  // ---- partial tiles of the four waves, summed in a fixed order; lane holds column ln, rows 8 (r / 4) + 4 h + r % 4
#pragma unroll
  for (int r = 0; r < 16; r++) red[wave][8 * (r >> 2) + 4 * h + (r & 3)][ln] = acc[r];
  __syncthreads();
  const int en = tid & 31, n = n0 + en;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int em = (tid >> 5) + 8 * i, mm = m0 + em;
    const float sum = ((red[0][em][en] + red[1][em][en]) + red[2][em][en]) + red[3][em][en];
    if (EP == EP_GELU) {
      const float v = sum + bf2f(g.bias[n]);
      if (mm < g.M) {
        if (g.H) g.H[(size_t)mm * g.ldh + n] = v;
        g.ActF[(size_t)mm * g.ldh + n] = gelu_f(v);
      }
    } else if (EP == EP_BIAS) {
      if (mm < g.M) g.Cb[(size_t)mm * g.ldc + n] = f2bf(sum + bf2f(g.bias[n]));
    } else if (EP == EP_PLAIN) {  // the product itself
      if (mm < g.M) {
        if (g.Cb) g.Cb[(size_t)mm * g.ldc + n] = f2bf(sum);
        else g.Cf[(size_t)mm * g.ldc + n] = g.plain_mul != 0.f ? sum * g.plain_mul : sum;
      }
    } else {  // EP_DH (the column sums of dH, db1, are formed by the weight-gradient kernel that reads dH next)
      if (mm < g.M) g.Cf[(size_t)mm * g.ldc + n] = sum * gelu_prime_f(g.H[(size_t)mm * g.ldh + n]);
    }
  }
  __syncthreads();  // red may be reused by the caller's next tile
}

// grid (N / 32, m-tiles)
template <bool A_F32, Epilogue EP>
__global__ void __launch_bounds__(256) mlp_skinny_kernel(SkinnyArgs g) {
  __shared__ float red[4][32][33];
  skinny_tile<A_F32, EP, 4>(g, blockIdx.x, blockIdx.y, red);
}

// ---------------------------------------------------------------------------------------------------
// C[M x N] = A[M x K] * Bt[N x K]^T for many rows (the whole batch at once: the projections of the distance function,
// the graph-less forward), where the skinny kernel above would stream Bt once per 32 rows.  A workgroup owns a BM x 128
// tile of C (BM = 128 or 64), its four waves BM/2 x 64 each (MFMA tiles 32x32x16); both operands go through LDS in
// 64-wide k-steps (whole 128-byte lines of every row), two buffers, one barrier per step; the global loads run two steps
// ahead in two register sets used in turn.  An fp32 A is split into hi + lo bf16 planes as everywhere in this file.
// Rows of LDS are padded to 144 bytes, which spreads the 16-byte fragment reads of 8 consecutive rows over all banks.
struct GemmArgs {
  const void* A; int lda;             // [M][K], bf16 or fp32
  const unsigned short* Bt; int ldb;  // [N][K] bf16
  int M, N, K;                        // M may be ragged; N a multiple of 128, K a multiple of 64
  void* C; int ldc;                   // fp32 or bf16, see GemmOut
  float mul;                          // GO_F32 / GO_BF16: factor on the product (0 means 1)
  const unsigned short* bias;         // GO_GELU_F32 / GO_BIAS_BF16: [N] bf16
  int k_split;                        // GO_F32 only: > 1 cuts K into that many equal ranges (each a multiple of 64); range s
  size_t split_stride;                //   writes its partial product to C + s * split_stride (elements)
  // two row segments (anchors, then targets, in one launch): rows from M1 on are rows 0.. of A2 / C2 when those are set
  int M1; const void* A2; void* C2;
};
// what a tile writes: the product (times mul) as fp32 or bf16, GELU(product + bias) as fp32, product + bias as bf16
enum GemmOut { GO_F32 = 0, GO_BF16 = 1, GO_GELU_F32 = 2, GO_BIAS_BF16 = 3 };
constexpr int GM_T = 128, GM_BK = 64, GM_LD = GM_BK + 8;
template <bool A_F32, int BM>
constexpr int gemm_lds_bytes() { return 2 * ((A_F32 ? 2 : 1) * BM + GM_T) * GM_LD * 2; }
template <bool A_F32, GemmOut OUT, int BM>
__global__ void __launch_bounds__(256) gemm_nt_kernel(GemmArgs g) {
  constexpr int AP = A_F32 ? 2 : 1;   // planes of A
  constexpr int MT = BM / 64;         // 32-row MFMA tiles per wave
  constexpr int NA = BM / 32;         // staging pieces of A per thread (8 elements each); 4 of Bt
  constexpr int A_PLANE = BM * GM_LD, BUF = (AP * BM + GM_T) * GM_LD;   // elements
  extern __shared__ __attribute__((aligned(16))) unsigned short gemm_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ln = lane & 31;
  const int nbn = g.N / GM_T;
  const int tiles = ((g.M + BM - 1) / BM) * nbn;
  const int bid = xcd_task_id();   // consecutive tiles (they share rows of A) on one XCD, behind one L2
  const int tile = bid % tiles, split = bid / tiles;   // split > 0 only for GO_F32 with k_split > 1
  const int m0 = (tile / nbn) * BM, n0 = (tile % nbn) * GM_T;
  const int klen = g.K / (g.k_split > 1 ? g.k_split : 1), kbeg = split * klen;
  const int wm = wave >> 1, wn = wave & 1;
  // staging: piece q = tid + 256 i of a tile is 8 elements: row q / 8, k 8 (q % 8)
  constexpr int AV = A_F32 ? 2 : 1;   // 16-byte loads per piece of A
  struct Regs { u32x4 a[NA][AV]; u32x4 b[4]; };
  Regs rg[2];
  auto fetch = [&](Regs& r, int k0) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int q = tid + 256 * i, row = q >> 3, kc = q & 7;
      if (i < NA) {
        const int am = min(m0 + row, g.M - 1);   // rows past the end repeat the last one; their results are not stored
        const bool second = g.A2 && am >= g.M1;
        const size_t ia = (size_t)(second ? am - g.M1 : am) * g.lda + kbeg + k0 + 8 * kc;
#pragma unroll
        for (int v = 0; v < AV; v++) r.a[i][v] = *(const u32x4*)((const char*)(second ? g.A2 : g.A) + ia * (A_F32 ? 4 : 2) + 16 * v);
      }
      r.b[i] = *(const u32x4*)(g.Bt + (size_t)(n0 + row) * g.ldb + kbeg + k0 + 8 * kc);
    }
  };
  auto stash = [&](const Regs& r, int buf) __attribute__((always_inline)) {
    unsigned short* As = gemm_lds + buf * BUF;
    unsigned short* Bs = As + AP * A_PLANE;
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int q = tid + 256 * i, row = q >> 3, kc = q & 7;
      if (i < NA) {
        if (A_F32) {
          typedef __attribute__((ext_vector_type(8))) float f32x8;
          const f32x4 x0 = __builtin_bit_cast(f32x4, r.a[i][0]), x1 = __builtin_bit_cast(f32x4, r.a[i][AV - 1]);
          const f32x8 v = {x0[0], x0[1], x0[2], x0[3], x1[0], x1[1], x1[2], x1[3]};
          const bf16x8 hi = __builtin_convertvector(v, bf16x8);
          const bf16x8 lo = __builtin_convertvector(v - __builtin_convertvector(hi, f32x8), bf16x8);
          *(bf16x8*)&As[row * GM_LD + 8 * kc] = hi;
          *(bf16x8*)&As[(AP - 1) * A_PLANE + row * GM_LD + 8 * kc] = lo;
        } else {
          *(u32x4*)&As[row * GM_LD + 8 * kc] = r.a[i][0];
        }
      }
      *(u32x4*)&Bs[row * GM_LD + 8 * kc] = r.b[i];
    }
  };
  f32x16 acc[MT][2];
#pragma unroll
  for (int mt = 0; mt < MT; mt++)
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mt][nt][r] = 0.f;
  const int nk = klen / GM_BK;
  // one k-step: the set that held step kt (already in LDS) takes the loads of step kt + 2, the MFMAs of step kt run,
  // the set of step kt + 1 goes to the other LDS buffer.  (STEADY: steps kt + 1 and kt + 2 exist; without branches
  // around the loads the compiler counts them, and its waits for a set let the loads of the newer set stay in flight.)
  auto step = [&](int kt, Regs& mine, const Regs& next, auto steady_tag) __attribute__((always_inline)) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    const int buf = kt & 1;
    const unsigned short* As = gemm_lds + buf * BUF;
    const unsigned short* Bs = As + AP * A_PLANE;
    if (STEADY || kt + 2 < nk) fetch(mine, (kt + 2) * GM_BK);
#pragma unroll
    for (int sub = 0; sub < GM_BK / 16; sub++) {   // 16 k each; lane (ln, h): row ln of a fragment, k 16 sub + 8 h ..
      bf16x8 fa[AP][MT], fb[2];
#pragma unroll
      for (int t = 0; t < 2; t++) {
        const int ra = (wm * 32 * MT + t * 32 + ln) * GM_LD + 16 * sub + 8 * h;
        const int rb = (wn * 64 + t * 32 + ln) * GM_LD + 16 * sub + 8 * h;
#pragma unroll
        for (int pl = 0; pl < AP; pl++)
          if (t < MT) fa[pl][t] = *(const bf16x8*)&As[pl * A_PLANE + ra];
        fb[t] = *(const bf16x8*)&Bs[rb];
      }
#pragma unroll
      for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int nt = 0; nt < 2; nt++)
#pragma unroll
          for (int pl = 0; pl < AP; pl++)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[pl][mt], fb[nt], acc[mt][nt], 0, 0, 0);
    }
    if (STEADY || kt + 1 < nk) stash(next, buf ^ 1);
    __syncthreads();
  };
  fetch(rg[0], 0);
  if (nk > 1) fetch(rg[1], GM_BK);
  stash(rg[0], 0);
  __syncthreads();
  int kt = 0;
  for (; kt + 3 < nk; kt += 2) {
    step(kt, rg[0], rg[1], std::true_type{});
    step(kt + 1, rg[1], rg[0], std::true_type{});
  }
  for (; kt < nk; kt += 2) {
    step(kt, rg[0], rg[1], std::false_type{});
    if (kt + 1 < nk) step(kt + 1, rg[1], rg[0], std::false_type{});
  }
  // lane (ln, h) holds column ln of each MFMA tile, rows 8 (r / 4) + 4 h + r % 4
  const float mul = g.mul != 0.f ? g.mul : 1.f;
#pragma unroll
  for (int mt = 0; mt < MT; mt++)
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int m = m0 + wm * 32 * MT + mt * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
        const int n = n0 + wn * 64 + nt * 32 + ln;
        if (m < g.M) {
          const bool second = g.C2 && m >= g.M1;
          void* cb = second ? g.C2 : g.C;
          const size_t at = (size_t)(second ? m - g.M1 : m) * g.ldc + n;
          if (OUT == GO_F32) ((float*)cb)[(size_t)split * g.split_stride + at] = acc[mt][nt][r] * mul;
          else if (OUT == GO_BF16) ((unsigned short*)cb)[at] = f2bf(acc[mt][nt][r] * mul);
          else if (OUT == GO_GELU_F32) ((float*)cb)[at] = gelu_f(acc[mt][nt][r] + bf2f(g.bias[n]));
          else ((unsigned short*)cb)[at] = f2bf(acc[mt][nt][r] + bf2f(g.bias[n]));
        }
      }
}
template <bool A_F32, GemmOut OUT>
static hipError_t launch_gemm_nt(const GemmArgs& g, hipStream_t s) {
  const int ks = g.k_split > 1 ? g.k_split : 1;
  if (g.M < 1 || g.N % GM_T || g.K % (GM_BK * ks) || g.K < GM_BK * ks || (ks > 1 && OUT != GO_F32)) return hipErrorInvalidValue;
  // 64-row tiles while 128-row tiles would leave compute units without one: several small workgroups per unit
  // then cover each other's barriers and waits
  const int t128 = ((g.M + 127) / 128) * (g.N / GM_T);
  if (t128 * ks >= 2 * num_cu()) {
    static bool done[64];
    constexpr int lds = gemm_lds_bytes<A_F32, 128>();
    if (hipError_t e = ensure_dyn_lds((const void*)gemm_nt_kernel<A_F32, OUT, 128>, lds, done); e != hipSuccess) return e;
    gemm_nt_kernel<A_F32, OUT, 128><<<t128 * ks, 256, lds, s>>>(g);
  } else {
    static bool done[64];
    constexpr int lds = gemm_lds_bytes<A_F32, 64>();
    if (hipError_t e = ensure_dyn_lds((const void*)gemm_nt_kernel<A_F32, OUT, 64>, lds, done); e != hipSuccess) return e;
    gemm_nt_kernel<A_F32, OUT, 64><<<((g.M + 63) / 64) * (g.N / GM_T) * ks, 256, lds, s>>>(g);
  }
  return hipGetLastError();
}

// out[m][n] = bf16(sum over the k_split partial products, in index order, + bias[n]); 4 elements per thread
// (rows from M1 on go to rows 0.. of out2 when that is set)
__global__ void __launch_bounds__(256) splitk_bias_bf16_kernel(const float* __restrict__ part, int k_split, size_t stride,
                                                              const unsigned short* __restrict__ bias, int N,
                                                              unsigned short* __restrict__ out, size_t n4, int M1,
                                                              unsigned short* __restrict__ out2) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= n4) return;
  f32x4 acc = ((const f32x4*)part)[e];
  for (int s = 1; s < k_split; s++) acc += ((const f32x4*)(part + (size_t)s * stride))[e];
  const int n = (int)((e * 4) % (size_t)N);
  const s16x4 b = *(const s16x4*)(bias + n);
  s16x4 o;
#pragma unroll
  for (int k = 0; k < 4; k++) o[k] = (short)f2bf(acc[k] + bf2f((unsigned short)b[k]));
  const size_t first4 = (size_t)M1 * N / 4;
  if (out2 && e >= first4) ((s16x4*)out2)[e - first4] = o;
  else ((s16x4*)out)[e] = o;
}

// One iteration of Step 3's software pipeline in one launch: the weight gradients of sub-batch c-2, dH and db1 of
// sub-batch c-1 and the re-encode of sub-batch c are independent of each other (three sets of buffers), and none of
// them fills the GPU alone.  The first n_dh workgroups take the n-tiles of dH, the next n_enc the tiles of the
// re-encode, the remaining n_wg the weight-gradient tiles (n_wg2 of them dW2).  A count of 0 switches a part off
// (pipeline ends).
struct Step3Args {
  WgradArgs g2, g1; int n_wg2, n_wg;
  SkinnyArgs dh; int n_dh;
  SkinnyArgs enc; int n_enc;
};
__global__ void __launch_bounds__(256, 3) mlp_step3_kernel(Step3Args a) {
  constexpr size_t kA = sizeof(unsigned short) * 2 * WG_KCH * WG_A_LD, kB = sizeof(unsigned short) * 2 * WG_KCH * WG_B_LD;
  constexpr size_t kLds = kA + kB > sizeof(SkinnyRed) * 4 ? kA + kB : sizeof(SkinnyRed) * 4;
  __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];
  int id = blockIdx.x;
  // the long-running workgroups (they stream whole weight rows) come first, the many short weight-gradient tiles
  // fill in behind them (1.16 -> 1.08 ms per step at config 5 against the other order)
  SkinnyRed* red = (SkinnyRed*)lds;
  if (id < a.n_dh) {
    const int nb = a.dh.N / 32;
    skinny_tile<true, EP_DH, 2>(a.dh, id % nb, id / nb, red);
    return;
  }
  id -= a.n_dh;
  if (id < a.n_enc) {
    const int nb = a.enc.N / 32;
    skinny_tile<false, EP_GELU, 2>(a.enc, id % nb, id / nb, red);
    return;
  }
  id -= a.n_enc;
  unsigned short* As = (unsigned short*)lds;
  unsigned short* Bs = (unsigned short*)(lds + kA);
  if (id < a.n_wg2) {
    const int nb = a.g2.N / 128;
    wgrad_tile<true>(a.g2, id % nb, id / nb, As, Bs);
  } else {
    const int nb = a.g1.N / 128;
    wgrad_tile<false>(a.g1, (id - a.n_wg2) % nb, (id - a.n_wg2) / nb, As, Bs);
  }
}

// Wt[n][k] = W[k][n] (bf16), 32 x 32 tiles through LDS; K and N multiples of 32
__global__ void __launch_bounds__(256) transpose_bf16_kernel(const unsigned short* __restrict__ W, int K, int N,
                                                            unsigned short* __restrict__ Wt) {
  __shared__ unsigned short t[32][33];
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  const int n0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
#pragma unroll
  for (int i = 0; i < 4; i++) t[ty + 8 * i][tx] = W[(size_t)(k0 + ty + 8 * i) * N + n0 + tx];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; i++) Wt[(size_t)(n0 + ty + 8 * i) * K + k0 + tx] = t[tx][ty + 8 * i];
}

struct MlpWs {
  float* H;             // [rows][dh] fp32 pre-activations
  float* ActF;          // [rows][dh] fp32 GELU(H)
  float* dH;            // [rows][dh] fp32
  unsigned short* W1T;  // [dh][din] bf16: W1 transposed
  unsigned short* W2T;  // [dout][dh] bf16: W2 transposed
  size_t total;
};

static inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

static MlpWs carve_mlp_ws(char* base, int rows, const gc_mlp_params* w) {
  MlpWs m{};
  size_t off = 0;
  // integer arithmetic: the sizing calls carve from a null base
  auto at = [base](size_t o) { return (uintptr_t)base + o; };
  m.H = (float*)at(off); off += up256((size_t)rows * w->dh * 4);
  m.ActF = (float*)at(off); off += up256((size_t)rows * w->dh * 4);
  m.dH = (float*)at(off); off += up256((size_t)rows * w->dh * 4);
  m.W1T = (unsigned short*)at(off); off += up256((size_t)w->din * w->dh * 2);
  m.W2T = (unsigned short*)at(off); off += up256((size_t)w->dh * w->dout * 2);
  m.total = off;
  return m;
}

static int check_mlp_params(const gc_mlp_params* w) {
  if (!w) return GC_ERR_NULL;
  if (!w->W1 || !w->b1 || !w->W2 || !w->b2) return GC_ERR_NULL;
  if (w->din < 64 || w->dh < 128 || w->dout < 128) return GC_ERR_SHAPE;
  if (w->din % 64 || w->dh % 128 || w->dout % 128) return GC_ERR_UNSUPPORTED;
  if (w->din > (1 << 20) || w->dh > (1 << 20) || w->dout > (1 << 20)) return GC_ERR_SHAPE;
  return GC_OK;
}

// the transposed weight copies that the skinny kernel streams (once per entry-point call: the weights do
// not change inside a call)
static hipError_t mlp_prepare(const gc_mlp_params* w, const MlpWs& ws, hipStream_t s) {
  transpose_bf16_kernel<<<dim3(w->dh / 32, w->din / 32), 256, 0, s>>>((const unsigned short*)w->W1, w->din, w->dh, ws.W1T);
  transpose_bf16_kernel<<<dim3(w->dout / 32, w->dh / 32), 256, 0, s>>>((const unsigned short*)w->W2, w->dh, w->dout, ws.W2T);
  return hipGetLastError();
}

// H = x W1 + b1 (kept when keepH), Act = GELU(H)
static SkinnyArgs layer1_args(const void* x, int rows, const gc_mlp_params* w, const MlpWs& ws, bool keepH) {
  SkinnyArgs g{};
  g.A = x; g.lda = w->din; g.Bt = ws.W1T; g.ldb = w->din; g.M = rows; g.N = w->dh; g.K = w->din;
  g.bias = (const unsigned short*)w->b1; g.H = keepH ? ws.H : nullptr; g.ActF = ws.ActF; g.ldh = w->dh;
  return g;
}
// dA = U W2^T, dH = dA * GELU'(H), db1 += column sums
static SkinnyArgs dh_args(int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc, const MlpWs& ws) {
  SkinnyArgs g{};
  g.A = u; g.lda = w->dout; g.Bt = (const unsigned short*)w->W2; g.ldb = w->dout; g.M = rows; g.N = w->dh; g.K = w->dout;
  g.H = ws.H; g.ldh = w->dh; g.Cf = ws.dH; g.ldc = w->dh;
  return g;
}
// dW2 += Act^T U, db2 += column sums of U (g2);  dW1 += X^T dH (g1)
static void wgrad_args(const void* x, int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc,
                       const MlpWs& ws, WgradArgs& g2, WgradArgs& g1) {
  g2 = WgradArgs{}; g1 = WgradArgs{};
  g2.A = ws.ActF; g2.lda = w->dh; g2.B = u; g2.ldb = w->dout; g2.M = w->dh; g2.N = w->dout; g2.K = rows;
  g2.C = acc->dW2; g2.ldc = w->dout; g2.colsum = acc->db2;
  g1.A = x; g1.lda = w->din; g1.B = ws.dH; g1.ldb = w->dh; g1.M = w->din; g1.N = w->dh; g1.K = rows;
  g1.C = acc->dW1; g1.ldc = w->dh; g1.colsum = acc->db1; g1.colsum_rows = 32;   // db1: 32-row tiles of dH, in order
}

constexpr int kGemmRows = 128;   // from this many rows on the graph-less forward runs as tiled GEMMs
constexpr int kStep1Rows = 2048;  // rows per launch of Step 1 (see group_rows)
// forward of one sub-batch (after mlp_prepare); keepH: also write the fp32 pre-activations (Step 3)
// tiled: the graph-less forward of many rows; the caller decides it per input (not per launch), so that a row's bits do
// not depend on how the rows are cut into launches
// x2 / rows2 / y2 (tiled only): a second input whose rows follow those of x in the same launches (the targets behind the
// anchors: together they fill the GPU better than one after the other)
static hipError_t mlp_forward(const void* x, int rows, const gc_mlp_params* w, const MlpWs& ws, bool keepH, void* y,
                              hipStream_t s, bool tiled = false, const void* x2 = nullptr, int rows2 = 0, void* y2 = nullptr) {
  if (tiled && !keepH && y) {
    const int all = rows + rows2;
    // many rows and nothing kept for a backward (Step 1): both layers as tiled GEMMs over all the rows at once, which
    // read the weights once per 64 or 128 rows instead of once per 32
    GemmArgs g1{};
    g1.A = x; g1.lda = w->din; g1.Bt = ws.W1T; g1.ldb = w->din; g1.M = all; g1.N = w->dh; g1.K = w->din;
    g1.C = ws.ActF; g1.ldc = w->dh; g1.bias = (const unsigned short*)w->b1; g1.M1 = rows; g1.A2 = x2;
    if (hipError_t e = launch_gemm_nt<false, GO_GELU_F32>(g1, s); e != hipSuccess) return e;
    GemmArgs g2{};
    g2.A = ws.ActF; g2.lda = w->dh; g2.Bt = ws.W2T; g2.ldb = w->dh; g2.M = all; g2.N = w->dout; g2.K = w->dh;
    g2.C = y; g2.ldc = w->dout; g2.bias = (const unsigned short*)w->b2; g2.M1 = rows; g2.C2 = y2;
    // The second layer is narrow (dout columns) and long (dh): few tiles, each a long chain of k-steps.  While the tiles
    // do not fill the GPU, the contraction is cut into up to four ranges whose fp32 partial products go to the dH
    // buffer (unused by a graph-less forward; rows x dh floats hold dh / dout partial outputs) and are summed, in
    // index order, by a kernel that adds the bias.  The split depends on the shape only, not on the rows of a launch.
    int ks = 1;
    const int tiles64 = ((kStep1Rows + 63) / 64) * (w->dout / GM_T);   // tiles of a full Step-1 launch
    while (ks < 4 && tiles64 * ks < 2 * num_cu() && (ks * 2) * w->dout <= w->dh && w->dh % (GM_BK * ks * 2) == 0) ks *= 2;
    if (ks == 1) return launch_gemm_nt<true, GO_BIAS_BF16>(g2, s);
    g2.C = ws.dH; g2.C2 = nullptr; g2.bias = nullptr; g2.k_split = ks; g2.split_stride = (size_t)all * w->dout;
    if (hipError_t e = launch_gemm_nt<true, GO_F32>(g2, s); e != hipSuccess) return e;
    const size_t n4 = (size_t)all * w->dout / 4;
    splitk_bias_bf16_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, s>>>(ws.dH, ks, g2.split_stride, (const unsigned short*)w->b2,
                                                                      w->dout, (unsigned short*)y, n4, rows, (unsigned short*)y2);
    return hipGetLastError();
  }
  mlp_skinny_kernel<false, EP_GELU><<<dim3(w->dh / 32, (rows + 31) / 32), 256, 0, s>>>(layer1_args(x, rows, w, ws, keepH));
  if (y) {
    SkinnyArgs g2{};
    g2.A = ws.ActF; g2.lda = w->dh; g2.Bt = ws.W2T; g2.ldb = w->dh; g2.M = rows; g2.N = w->dout; g2.K = w->dh;
    g2.bias = (const unsigned short*)w->b2; g2.Cb = (unsigned short*)y; g2.ldc = w->dout;
    mlp_skinny_kernel<true, EP_BIAS><<<dim3(w->dout / 32, (rows + 31) / 32), 256, 0, s>>>(g2);
  }
  return hipGetLastError();
}

// the surrogate backward of one sub-batch in three parts: (1) re-encode keeping H and Act = mlp_forward with
// keepH, (2) dH and db1, (3) the weight gradients
static hipError_t mlp_backward_dh(int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc,
                                  const MlpWs& ws, hipStream_t s) {
  mlp_skinny_kernel<true, EP_DH><<<dim3(w->dh / 32, (rows + 31) / 32), 256, 0, s>>>(dh_args(rows, w, u, acc, ws));
  return hipGetLastError();
}

// second half: the weight gradients, from what the first half left in ws
static hipError_t mlp_backward_wgrad(const void* x, int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc,
                                     const MlpWs& ws, hipStream_t s) {
  WgradArgs g2, g1;
  wgrad_args(x, rows, w, u, acc, ws, g2, g1);
  const int n2 = (w->dout / 128) * (w->dh / WG_M), n1 = (w->dh / 128) * (w->din / WG_M);
  mlp_wgrad_kernel<<<n2 + n1, 256, 0, s>>>(g2, g1, n2);
  return hipGetLastError();
}

static hipError_t mlp_backward(const void* x, int rows, const gc_mlp_params* w, const float* u, const gc_mlp_grads* acc,
                               const MlpWs& ws, hipStream_t s) {
  hipError_t e = mlp_forward(x, rows, w, ws, true, nullptr, s);
  if (e != hipSuccess) return e;
  e = mlp_backward_dh(rows, w, u, acc, ws, s);
  if (e != hipSuccess) return e;
  return mlp_backward_wgrad(x, rows, w, u, acc, ws, s);
}

// ---- the one-GPU driver of Steps 1-3 -----------------------------------------------------------------------
// Sub-batches are small, so one of them cannot fill the GPU.  Step 1 keeps nothing but the representations and
// its rows do not depend on each other, so many consecutive sub-batches go through each launch (group_rows; a row's
// result does not depend on how many rows share the launch; only transient buffers grow).  In Step 3 the
// accumulation order is fixed (sub-batch order), so it runs as a software pipeline of three stages, one launch
// (mlp_step3_kernel) per iteration: re-encode of sub-batch c, dH and db1 of c-1, weight gradients of c-2, on three
// sets of activation buffers.  Everything is enqueued on the caller's stream, in an order that does not depend
// on timing.
constexpr int kLanes = 3;   // buffer sets = pipeline stages of Step 3
constexpr int kGroup = 8;   // sub-batches per launch in Step 1
static std::mutex g_step_mutex;

// rows per launch of Step 1: whole sub-batches, kGroup of them or as many as fit into kStep1Rows rows (enough for the
// tiled GEMMs of the graph-less forward to fill the GPU), at most n.  Only the transient activation buffer of Step 1
// grows with it (rows x dh fp32), not what the step keeps.  (kStep1Rows is defined with the forward above.)
static int group_rows(int chunk, int n) {
  long long g = (long long)kGroup * chunk;
  const long long fit = (long long)(kStep1Rows / chunk) * chunk;
  if (fit > g) g = fit;
  return (int)(g < n ? g : n);
}

// both inputs in the same launches of Step 1: when each side takes the tiled forward and together they fit a launch
static bool step1_joint(int B, int P) { return B >= kGemmRows && P >= kGemmRows && (long long)B + P <= kStep1Rows; }
// rows of the activation buffers that Step 1 (and lane 0 of Step 3) needs
static int step1_ws_rows(int B, int P, int chunk_q, int chunk_p) {
  const int cmax = chunk_q > chunk_p ? chunk_q : chunk_p;
  const int r = group_rows(cmax, B > P ? B : P);
  return step1_joint(B, P) && B + P > r ? B + P : r;
}

struct StepWs {
  size_t off_q, off_p, off_dq, off_dp, off_loss, off_mlp, off_act, total;
  size_t loss_bytes, mlp_bytes, act_bytes;
};

// sub-batches that one launch of Step 3 covers: the caller's accumulate_group where the sub-batch sizes allow the
// result to stay bit-identical (whole 32-row MFMA k-chunks per sub-batch), else 1
static int effective_group(int group, int chunk_q, int chunk_p) {
  if (group < 1) group = 1;
  if (group > kGroup) group = kGroup;
  return (chunk_q % 32 == 0 && chunk_p % 32 == 0) ? group : 1;
}

static StepWs plan_step(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w, int group) {
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
  s.mlp_bytes = carve_mlp_ws(nullptr, step1_ws_rows(B, P, chunk_q, chunk_p), w).total;
  s.off_mlp = take(s.mlp_bytes);
  const int g3 = effective_group(group, chunk_q, chunk_p);
  s.act_bytes = 3 * up256((size_t)cmax * g3 * w->dh * 4);  // H, Act, dH of one more lane
  s.off_act = take((kLanes - 1) * s.act_bytes);
  s.total = off;
  return s;
}

// everything a step call depends on besides the contents of its buffers
struct StepCall {
  const void* x_q; const void* x_p; const int32_t* pos_idx;
  int B, P, chunk_q, chunk_p;
  gc_mlp_params w;
  float scale, temp;
  float* loss;
  gc_mlp_grads grads;
  void* q_rep; void* p_rep; float* dq; float* dp;
  void* workspace;
  int group;   // accumulate_group
};

// enqueues Steps 1-3 on s
static int enqueue_step(const StepCall& c, hipStream_t s) {
  const void* x_q = c.x_q; const void* x_p = c.x_p; const int32_t* pos_idx = c.pos_idx;
  const int B = c.B, P = c.P, chunk_q = c.chunk_q, chunk_p = c.chunk_p;
  const gc_mlp_params* w = &c.w; const gc_mlp_grads* grads = &c.grads;
  const float scale = c.scale, temp = c.temp;
  float* loss = c.loss; void* q_rep = c.q_rep; void* p_rep = c.p_rep; float* dq = c.dq; float* dp = c.dp;
  void* workspace = c.workspace;
  const StepWs sw = plan_step(B, P, chunk_q, chunk_p, w, c.group);
  const int g3 = effective_group(c.group, chunk_q, chunk_p);
  char* base = (char*)workspace;
  unsigned short* Q = q_rep ? (unsigned short*)q_rep : (unsigned short*)(base + sw.off_q);
  unsigned short* Pm = p_rep ? (unsigned short*)p_rep : (unsigned short*)(base + sw.off_p);
  float* dQ = dq ? dq : (float*)(base + sw.off_dq);
  float* dP = dp ? dp : (float*)(base + sw.off_dp);
  const int cmax = chunk_q > chunk_p ? chunk_q : chunk_p;
  MlpWs lane[kLanes];  // buffer sets (set 0 also serves Step 1); all share the transposed weights
  lane[0] = carve_mlp_ws(base + sw.off_mlp, step1_ws_rows(B, P, chunk_q, chunk_p), w);
  for (int l = 1; l < kLanes; l++) {
    lane[l] = lane[0];
    char* ab = base + sw.off_act + (size_t)(l - 1) * sw.act_bytes;
    const size_t one = up256((size_t)cmax * g3 * w->dh * 4);
    lane[l].H = (float*)ab; lane[l].ActF = (float*)(ab + one); lane[l].dH = (float*)(ab + 2 * one);
  }
  auto ok = [](hipError_t e) { return e == hipSuccess; };
  if (!ok(mlp_prepare(w, lane[0], s))) return GC_ERR_HIP;
  // the sub-batches in index order: anchors first, then targets.  With accumulate_group = G > 1 an entry covers G
  // consecutive sub-batches of one side (their rows are contiguous): the kernels of Step 3 visit the rows in the same
  // order and 32-row k-chunks as G single launches would, and add the bias gradients one sub-batch after the other
  // (`chunk`), so the parameter gradients keep their bits while the fp32 accumulators make one trip through HBM
  // instead of G.
  struct Sub { const unsigned short* x; int rows; unsigned short* y; const float* u; int chunk; };
  std::vector<Sub> subs;
  for (int a = 0; a < B; a += chunk_q * g3)
    subs.push_back({(const unsigned short*)x_q + (size_t)a * w->din, B - a < chunk_q * g3 ? B - a : chunk_q * g3, Q + (size_t)a * w->dout, dQ + (size_t)a * w->dout, chunk_q});
  for (int a = 0; a < P; a += chunk_p * g3)
    subs.push_back({(const unsigned short*)x_p + (size_t)a * w->din, P - a < chunk_p * g3 ? P - a : chunk_p * g3, Pm + (size_t)a * w->dout, dP + (size_t)a * w->dout, chunk_p});
  const int nsub = (int)subs.size();
  // Step 1: graph-less forward, representations kept: both inputs through the same launches where they fit one
  // (step1_joint), else group_rows rows of one input per launch
  if (step1_joint(B, P)) {
    if (!ok(mlp_forward(x_q, B, w, lane[0], false, Q, s, true, x_p, P, Pm))) return GC_ERR_HIP;
  } else {
    const int gq = group_rows(chunk_q, B), gp = group_rows(chunk_p, P);
    for (int a = 0; a < B; a += gq) {
      const int rows = B - a < gq ? B - a : gq;
      if (!ok(mlp_forward((const unsigned short*)x_q + (size_t)a * w->din, rows, w, lane[0], false, Q + (size_t)a * w->dout, s,
                          B >= kGemmRows)))
        return GC_ERR_HIP;
    }
    for (int a = 0; a < P; a += gp) {
      const int rows = P - a < gp ? P - a : gp;
      if (!ok(mlp_forward((const unsigned short*)x_p + (size_t)a * w->din, rows, w, lane[0], false, Pm + (size_t)a * w->dout, s,
                          P >= kGemmRows)))
        return GC_ERR_HIP;
    }
  }
  // Step 2: loss and the representation gradient cache
  int rc = gc_loss_and_rep_grad_ex(GC_BF16, Q, Pm, pos_idx, B, P, w->dout, scale, temp, 0, loss, dQ, dP, nullptr, nullptr,
                               base + sw.off_loss, sw.loss_bytes, (void*)s);
  if (rc != GC_OK) return rc;
  // Step 3: per sub-batch re-encode and backward of the cached rows; gradients accumulated in index order
  const int n2 = (w->dout / 128) * (w->dh / WG_M), n1 = (w->dh / 128) * (w->din / WG_M);
  for (int i = 0; i < nsub + 2; i++) {
    Step3Args a3{};
    if (i >= 2) {                      // weight gradients of sub-batch i-2
      const Sub& sb = subs[i - 2];
      wgrad_args(sb.x, sb.rows, w, sb.u, grads, lane[(i - 2) % kLanes], a3.g2, a3.g1);
      a3.g2.colsum_rows = sb.chunk;
      a3.n_wg2 = n2; a3.n_wg = n2 + n1;
    }
    if (i >= 1 && i - 1 < nsub) {      // dH, db1 of sub-batch i-1
      const Sub& sb = subs[i - 1];
      a3.dh = dh_args(sb.rows, w, sb.u, grads, lane[(i - 1) % kLanes]);
      a3.n_dh = (w->dh / 32) * ((sb.rows + 31) / 32);
    }
    if (i < nsub) {                    // re-encode of sub-batch i, keeping H and Act
      const Sub& sb = subs[i];
      a3.enc = layer1_args(sb.x, sb.rows, w, lane[i % kLanes], true);
      a3.n_enc = (w->dh / 32) * ((sb.rows + 31) / 32);
    }
    mlp_step3_kernel<<<a3.n_wg + a3.n_dh + a3.n_enc, 256, 0, s>>>(a3);
  }
  if (!ok(hipGetLastError())) return GC_ERR_HIP;
  return GC_OK;
}

// A step is some seventy small launches, and a host that enqueues them one by one can fall behind the GPU.  The second time a call comes with exactly the same arguments, it is recorded into a HIP graph (on a
// stream of the library's: the caller's may be the null stream, which cannot be captured) and from then on
// replayed with one launch.  The graph holds kernel nodes only, no memset nodes.  Up to
// kMaxGraphs argument sets are remembered per device (a graph in flight is never destroyed); others, calls
// made while the measurement events of the loss path are on, and calls whose capture fails are enqueued directly.
constexpr int kMaxGraphs = 8;
struct StepGraph { StepCall call; int seen; hipGraphExec_t exec; };
struct StepGraphs { StepGraph g[kMaxGraphs]; int n = 0; hipStream_t cap = nullptr; };
static StepGraphs g_step_graphs[64];

static int run_step(const StepCall& c, hipStream_t s) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  if (prof_active()) return enqueue_step(c, s);
  std::lock_guard<std::mutex> lock(g_step_mutex);
  StepGraphs& G = g_step_graphs[dev];
  StepGraph* e = nullptr;
  for (int i = 0; i < G.n; i++)
    if (memcmp(&G.g[i].call, &c, sizeof(StepCall)) == 0) e = &G.g[i];
  if (!e) {
    if (G.n < kMaxGraphs) { G.g[G.n].call = c; G.g[G.n].seen = 1; G.g[G.n].exec = nullptr; G.n++; }
    return enqueue_step(c, s);
  }
  if (!e->exec && e->seen == 1) {
    e->seen = 2;  // one attempt
    if (!G.cap && hipStreamCreateWithFlags(&G.cap, hipStreamNonBlocking) != hipSuccess) G.cap = nullptr;
    if (G.cap && hipStreamBeginCapture(G.cap, hipStreamCaptureModeThreadLocal) == hipSuccess) {
      const int rc = enqueue_step(c, G.cap);
      hipGraph_t graph = nullptr;
      const hipError_t ee = hipStreamEndCapture(G.cap, &graph);
      hipGraphExec_t exec = nullptr;
      if (rc == GC_OK && ee == hipSuccess && graph && hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0) == hipSuccess) e->exec = exec;
      if (graph) (void)hipGraphDestroy(graph);
      (void)hipGetLastError();
    }
  }
  if (e->exec) return hipGraphLaunch(e->exec, s) == hipSuccess ? GC_OK : GC_ERR_HIP;
  return enqueue_step(c, s);
}


// ---- deep (non-bilinear) distance function (Sec. "Extend to Deep Distance Function") ---------------------------
//   Phi_Omega(f, g) = sum_k w_k tanh((A f)_k + (C g)_k),  Omega = (A [h,d], C [h,d], w [h]).
// Phi does not factor over its two arguments, so each of the B * P distances is an evaluation of its own: h tanh per
// pair, plain vector arithmetic (no contraction for the MFMAs to take).  The pair part works on a_i = A f_i and
// c_j = C g_j (two skinny products), both scaled by 2 log2(e), so that with r = 1 / (1 + 2^(a + c)):
//   tanh z = 1 - 2 r,   1 - tanh^2 z = 4 r (1 - r).
// One kernel walks the pairs in two roles, each with an owner side whose rows a workgroup keeps in registers and a
// streamed side that passes through LDS 32 rows at a time:
//   DD_DA     owner = anchors: d_ij for every pair and, in the same walk, the row's softmax statistics and the sums
//             sum_j 2^(t_ij - m) t'_ijk and sum_j 2^(t_ij - m) t_ijk relative to a reference m that is raised (the
//             sums scaled down) only when a logit exceeds it by more than a margin; a finish kernel merges the splits
//             into lse_i, the loss, dL/da_i (hence u_i and dL/dA) and the rows whose column sums are dL/dw.  The weight
//             w_ij = dL/dd_ij of a pair (the section's Distance Gradient Cache) is 2^(t_ij - lse_i) - [j = r_i]: it
//             exists as the factor 2^(t_ij - m) for one pair at a time in a register, times 2^(m - lse_i) at the
//             finish, where the positive's -1 is subtracted too (its r values are put aside by the walk)
//   DD_DC     owner = targets: the same pairs walked the other way, with the final lse_i of the streamed anchors, for
//             sum_i w_ij t'_ijk (-> dL/dc_j, hence v_j, dL/dC); a second walk instead of a cross-workgroup sum: no
//             atomics, fixed order.
// Thread (o, kq) of a workgroup owns owner row o (64 rows) and the quarter kq of the k range: the four threads of a
// row add their partial distances with two cross-lane moves, everything else stays in the thread's registers.
constexpr int DD_OWN = 64, DD_TS = 32;
enum DdRole { DD_DA = 0, DD_DC = 1 };
constexpr float kDdMargin = 16.f;   // DD_DA: the reference of a row is raised when a logit exceeds it by more than this
struct DdArgs {
  const float* own; const float* str;   // [n_own][H], [n_str][H]: 2 log2(e) (A f) resp. (C g), owner and streamed side
  const unsigned short* wv;             // [H] bf16: w
  int n_own, n_str, n_oblk, stream_len; // owner blocks; streamed rows per split
  float alpha2, out_scale;              // alpha log2(e); alpha / B
  const int32_t* pos_idx;               // [B] r_i (DD_DA: of the owner rows)
  float* part_m; float* part_l; float* pos_t;   // DD_DA out, per split and anchor: reference m, sum_j 2^(t_ij - m); the positive's logit
  const float* lse2; const int32_t* pos_pad;                   // DD_DC in: per anchor, padded (+inf, -1)
  float* out_a;   // [split][n_own][H]: DD_DA: sum_j 2^(t_ij - m) r (1 - r), unscaled; DD_DC: dL/dc partial, final scale applied
  float* out_e;   // DD_DA: [split][n_own][H]: sum_j 2^(t_ij - m) r, unscaled
  float* pos_r;   // DD_DA: [n_own][H]: r_{i r_i k} of the positive pair (its -1 term is subtracted by the finish kernel)
};

__device__ __forceinline__ float quad_sum(float x) {   // over the four lanes 4 i .. 4 i + 3
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  return x;
}

template <int H, int ROLE>
__global__ void __launch_bounds__(256, 2) deepdist_walk_kernel(DdArgs g) {
  constexpr int HQ = H / 4;            // k values per thread
  constexpr int LD4 = DD_TS * H / 4 / 256;   // float4 loads per thread and tile
  __shared__ __attribute__((aligned(16))) float tile[2][DD_TS][H];
  __shared__ float st_lse[2][DD_TS];
  __shared__ int st_pos[2][DD_TS];
  const int tid = threadIdx.x, o = tid >> 2, kq = tid & 3;
  const int oblk = blockIdx.x % g.n_oblk, split = blockIdx.x / g.n_oblk;
  const int row = oblk * DD_OWN + o, rowc = min(row, g.n_own - 1);
  const int sbeg = split * g.stream_len, send = min(g.n_str, sbeg + g.stream_len);
  const int nt = (send - sbeg + DD_TS - 1) / DD_TS;

  float ao[HQ], wq[HQ];
#pragma unroll
  for (int k = 0; k < HQ; k += 4) {
    const f32x4 v = *(const f32x4*)(g.own + (size_t)rowc * H + kq * HQ + k);
    ao[k] = v[0]; ao[k + 1] = v[1]; ao[k + 2] = v[2]; ao[k + 3] = v[3];
  }
  float w1 = 0.f;
#pragma unroll
  for (int k = 0; k < HQ; k++) { wq[k] = bf2f(g.wv[kq * HQ + k]); w1 += wq[k]; }
  w1 = quad_sum(w1);   // sum_k w_k

  int r_o = -1;
  if (ROLE == DD_DA && row < g.n_own) r_o = g.pos_idx[row];
  float acc_a[HQ], acc_e[HQ];
#pragma unroll
  for (int k = 0; k < HQ; k++) { acc_a[k] = 0.f; acc_e[k] = 0.f; }
  float m = -INFINITY, l = 0.f, pos = 0.f;
  bool got = false;

  // tile u of the streamed rows: global -> registers -> LDS, one tile ahead
  f32x4 pre[LD4]; float pre_lse = INFINITY; int pre_pos = -1;
  auto fetch = [&](int u) __attribute__((always_inline)) {
    const int t0 = sbeg + u * DD_TS;
#pragma unroll
    for (int v = 0; v < LD4; v++) {
      const int e4 = tid + 256 * v, rr = e4 / (H / 4), c4 = e4 % (H / 4);
      pre[v] = *(const f32x4*)(g.str + (size_t)min(t0 + rr, g.n_str - 1) * H + 4 * c4);
    }
    if (ROLE == DD_DC && tid < DD_TS) {   // statistics of the streamed anchors (padded: +inf / -1 past the end)
      pre_lse = g.lse2[t0 + tid]; pre_pos = g.pos_pad[t0 + tid];
    }
  };
  auto stash = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int v = 0; v < LD4; v++) {
      const int e4 = tid + 256 * v, rr = e4 / (H / 4), c4 = e4 % (H / 4);
      // 16-byte piece j of quarter kq sits at piece 4 j + kq: the four threads of a row then read 64 contiguous bytes
      *(f32x4*)&tile[buf][rr][4 * ((c4 % (HQ / 4)) * 4 + c4 / (HQ / 4))] = pre[v];
    }
    if (ROLE == DD_DC && tid < DD_TS) { st_lse[buf][tid] = pre_lse; st_pos[buf][tid] = pre_pos; }
  };
  fetch(0);
  stash(0);
  __syncthreads();
  for (int u = 0; u < nt; u++) {
    const int buf = u & 1;
    if (u + 1 < nt) fetch(u + 1);
    const int t0 = sbeg + u * DD_TS, rows = min(DD_TS, send - t0);
    for (int s_ = 0; s_ < rows; s_++) {
      const float* cs = &tile[buf][s_][4 * kq];
      float rr[HQ], part = 0.f;
#pragma unroll
      for (int k = 0; k < HQ; k += 4) {
        const f32x4 c4 = *(const f32x4*)(cs + 4 * k);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          const float r = __builtin_amdgcn_rcpf(1.f + fast_exp2(ao[k + e] + c4[e]));   // 1 / (1 + e^(2 z))
          rr[k + e] = r;
          part = __builtin_fmaf(wq[k + e], r, part);
        }
      }
      const float t = g.alpha2 * (w1 - 2.f * quad_sum(part));   // base-2 logit of the pair
      const int gs = t0 + s_;
      if (ROLE == DD_DA) {
        // statistics and gradient sums in one walk: sums relative to a reference m that is raised (and the sums scaled
        // down with it) only when a logit exceeds it by more than the margin -- at the first pair, and rarely afterwards
        if (gs == r_o) {
          pos = t; got = true;
          if (row < g.n_own) {
#pragma unroll
            for (int k = 0; k < HQ; k += 4)
              *(f32x4*)(g.pos_r + (size_t)row * H + kq * HQ + k) = f32x4{rr[k], rr[k + 1], rr[k + 2], rr[k + 3]};
          }
        }
        if (t > m + kDdMargin) {
          const float f = fast_exp2(m - t);   // 2^-inf = 0 the first time
#pragma unroll
          for (int k = 0; k < HQ; k++) { acc_a[k] *= f; acc_e[k] *= f; }
          l *= f;
          m = t;
        }
        const float e = fast_exp2(t - m);
        l += e;
#pragma unroll
        for (int k = 0; k < HQ; k++) {
          acc_a[k] = __builtin_fmaf(e, __builtin_fmaf(-rr[k], rr[k], rr[k]), acc_a[k]);
          acc_e[k] = __builtin_fmaf(e, rr[k], acc_e[k]);
        }
      } else {
        const float wij = fast_exp2(t - st_lse[buf][s_]) - (st_pos[buf][s_] == row ? 1.f : 0.f);   // dL/dd_ij in units of alpha / B
#pragma unroll
        for (int k = 0; k < HQ; k++) acc_a[k] = __builtin_fmaf(wij, __builtin_fmaf(-rr[k], rr[k], rr[k]), acc_a[k]);   // w_ij r (1 - r)
      }
    }
    if (u + 1 < nt) stash(buf ^ 1);
    __syncthreads();
  }
  if (row >= g.n_own) return;
  if (ROLE == DD_DA) {
    if (kq == 0) {
      const size_t oo = (size_t)split * g.n_own + row;
      g.part_m[oo] = m; g.part_l[oo] = l;
      if (got) g.pos_t[row] = pos;
    }
    float* oa = g.out_a + ((size_t)split * g.n_own + row) * H + kq * HQ;
    float* oe = g.out_e + ((size_t)split * g.n_own + row) * H + kq * HQ;
#pragma unroll
    for (int k = 0; k < HQ; k += 4) {
      *(f32x4*)(oa + k) = f32x4{acc_a[k], acc_a[k + 1], acc_a[k + 2], acc_a[k + 3]};
      *(f32x4*)(oe + k) = f32x4{acc_e[k], acc_e[k + 1], acc_e[k + 2], acc_e[k + 3]};
    }
  } else {
    // dL/dc_jk = w_k (alpha/B) 4 sum_i w_ij r (1 - r)
    float* oa = g.out_a + ((size_t)split * g.n_own + row) * H + kq * HQ;
#pragma unroll
    for (int k = 0; k < HQ; k += 4)
      *(f32x4*)(oa + k) = f32x4{acc_a[k] * wq[k], acc_a[k + 1] * wq[k + 1], acc_a[k + 2] * wq[k + 2], acc_a[k + 3] * wq[k + 3]} * (4.f * g.out_scale);
  }
}

// After the DD_DA walk: merge of what its splits left per anchor (reference m_s, l_s = sum_j 2^(t_ij - m_s)) into
// lse2_i and the row loss, and with the weights 2^(m_s - lse2_i) of the splits (index order)
//   dL/da_ik   = (alpha/B) 4 w_k (sum_j p_ij r (1 - r) - r_pos (1 - r_pos))
//   e_ik       = (alpha/B) sum_j w_ij tanh_ijk = -2 (alpha/B) (sum_j p_ij r - r_pos)       (sum_j w_ij = 0)
// with r = r_ijk, r_pos = r_{i r_i k}, p_ij the softmax and w_ij = p_ij - [j = r_i].  One thread per (anchor, k).
struct DdFinish {
  const float* part_m; const float* part_l; const float* pos_t; const int32_t* pos_idx;
  const float* part_a; const float* part_e; const float* pos_r; const unsigned short* wv;
  int ns, B, P, b_pad;
  float out_scale;
  float* lse2; int32_t* pos_pad; float* rowloss; float* da; float* e;
};
template <int H>
__global__ void __launch_bounds__(256) deepdist_finish_kernel(DdFinish f) {
  constexpr int ROWS = 256 / H;
  const int i = blockIdx.x * ROWS + threadIdx.x / H, k = threadIdx.x % H;
  const bool live = i < f.B;
  if (!live && i < f.b_pad && k == 0) { f.lse2[i] = INFINITY; f.pos_pad[i] = -1; }
  // the row's split statistics, loaded once by its first ns threads (ns <= 64 <= H)
  __shared__ float sm[ROWS][64], sl[ROWS][64];
  const int rr = threadIdx.x / H;
  if (live && k < f.ns) { sm[rr][k] = f.part_m[(size_t)k * f.B + i]; sl[rr][k] = f.part_l[(size_t)k * f.B + i]; }
  __syncthreads();
  if (!live) return;
  float M = -INFINITY;
  for (int s = 0; s < f.ns; s++) M = fmaxf(M, sm[rr][s]);
  float L = 0.f;
  for (int s = 0; s < f.ns; s++) L += sl[rr][s] * exp2f(sm[rr][s] - M);
  const float l2 = M + log2f(L);
  const int r = f.pos_idx[i];
  const bool ok = (r >= 0 && r < f.P);
  if (k == 0) {
    f.lse2[i] = l2;
    f.pos_pad[i] = r;
    f.rowloss[i] = ok ? (l2 - f.pos_t[i]) * kLn2 : NAN;
  }
  float sa = 0.f, se = 0.f;
#pragma unroll 4
  for (int s = 0; s < f.ns; s++) {
    const float w = exp2f(sm[rr][s] - l2);
    sa += w * f.part_a[((size_t)s * f.B + i) * H + k];
    se += w * f.part_e[((size_t)s * f.B + i) * H + k];
  }
  const float pr = ok ? f.pos_r[(size_t)i * H + k] : 0.f;
  f.da[(size_t)i * H + k] = 4.f * f.out_scale * bf2f(f.wv[k]) * (sa - (pr - pr * pr));
  f.e[(size_t)i * H + k] = -2.f * f.out_scale * (se - pr);
}

// column sums of x[rows][cols] over a slice of the rows: partial[slice][cols] (fixed order; cols a multiple of 32)
__global__ void __launch_bounds__(256) colsum_slices_kernel(const float* __restrict__ x, int rows, int cols, int rows_per_slice,
                                                           float* __restrict__ partial) {
  __shared__ float red[8][33];
  const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cx, slice = blockIdx.y;
  const int r0 = slice * rows_per_slice, r1 = min(rows, r0 + rows_per_slice);
  float s = 0.f;
  for (int r = r0 + ry; r < r1; r += 8) s += x[(size_t)r * cols + c];
  red[ry][cx] = s;
  __syncthreads();
  if (ry == 0) {
    float t = 0.f;
#pragma unroll
    for (int k = 0; k < 8; k++) t += red[k][cx];
    partial[(size_t)slice * cols + c] = t;
  }
}

struct DeepWs {
  LossPlan st;                 // the statistics part of a loss workspace (split statistics, lse2, row losses, error word)
  size_t off_stat, off_a, off_c, off_AT, off_CT, off_da_part, off_e_part, off_dc_part, off_da, off_dc, off_e, off_wpart,
      off_gpart, off_pos_r, total;
  int nsa, len_a, nsc, len_c;  // stream splits of the anchor-owner walks / of the target-owner walk
  int slices_b, rps_b, slices_p, rps_p;   // row slices of the two parameter-gradient products
};
static void dd_split(int n_oblk, int n_str, int& ns, int& len) {
  const int target = 2 * num_cu();               // two workgroups per CU
  ns = (target + n_oblk - 1) / n_oblk;
  const int max_ns = (n_str + 4 * DD_TS - 1) / (4 * DD_TS);   // at least four tiles per split
  if (ns > max_ns) ns = max_ns;
  if (ns > 64) ns = 64;
  if (ns < 1) ns = 1;
  len = ((n_str + ns - 1) / ns + DD_TS - 1) / DD_TS * DD_TS;
  ns = (n_str + len - 1) / len;
}
static DeepWs plan_deep(int B, int P, int d, int h) {
  DeepWs w{};
  const int obA = (B + DD_OWN - 1) / DD_OWN, obC = (P + DD_OWN - 1) / DD_OWN;
  dd_split(obA, P, w.nsa, w.len_a);
  dd_split(obC, B, w.nsc, w.len_c);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = up256(off + bytes); return o; };
  // statistics, laid out as the loss kernels' merge expects them
  LossPlan& st = w.st;
  st.use_mfma = 0; st.stat_splits = w.nsa; st.b_pad = (B + 63) / 64 * 64;
  w.off_stat = 0;
  st.off_err = take(256);
  st.off_part_m = take((size_t)w.nsa * B * 4); st.off_part_l = take((size_t)w.nsa * B * 4); st.off_part_idx = take((size_t)w.nsa * B * 4);
  st.off_pos = take((size_t)B * 4); st.off_lse2 = take((size_t)st.b_pad * 4); st.off_pos_pad = take((size_t)st.b_pad * 4);
  st.off_rowloss = take((size_t)B * 4);
  w.off_a = take((size_t)B * h * 4); w.off_c = take((size_t)P * h * 4);
  w.off_AT = take((size_t)d * h * 2); w.off_CT = take((size_t)d * h * 2);
  w.off_da_part = take((size_t)w.nsa * B * h * 4); w.off_e_part = take((size_t)w.nsa * B * h * 4);
  w.off_dc_part = take((size_t)w.nsc * P * h * 4);
  w.off_da = take((size_t)B * h * 4); w.off_dc = take((size_t)P * h * 4); w.off_e = take((size_t)B * h * 4);
  w.off_wpart = take((size_t)64 * h * 4);
  w.off_pos_r = take((size_t)B * h * 4);
  auto slices_of = [&](int rows, int& sl, int& rps) {
    const int tiles = (d / 128) * (h / WG_M);
    sl = (2 * num_cu() + tiles - 1) / tiles;
    const int mx = (rows + 127) / 128;
    if (sl > mx) sl = mx;
    if (sl > 64) sl = 64;
    if (sl < 1) sl = 1;
    rps = ((rows + sl - 1) / sl + 31) / 32 * 32;
    sl = (rows + rps - 1) / rps;
  };
  slices_of(B, w.slices_b, w.rps_b);
  slices_of(P, w.slices_p, w.rps_p);
  const int smax = w.slices_b > w.slices_p ? w.slices_b : w.slices_p;
  w.off_gpart = take((size_t)smax * h * d * 4);
  w.total = off;
  return w;
}
static int deep_shape_status(int B, int P, int d, int h) {
  if (B < 1 || P < 1 || d < 1 || h < 1 || (long long)B * d > (1ll << 40) || (long long)P * d > (1ll << 40)) return GC_ERR_SHAPE;
  if (d % 128 || h != 128) return GC_ERR_UNSUPPORTED;
  return GC_OK;
}

// Drops what run_step has recorded for the current device: waits for the device, then destroys the graph
// executables and the capture stream.
static int release_step_graphs() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return GC_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_step_mutex);
  StepGraphs& G = g_step_graphs[dev];
  if (G.n == 0 && !G.cap) return GC_OK;
  if (hipDeviceSynchronize() != hipSuccess) return GC_ERR_HIP;   // a graph in flight is never destroyed
  int rc = GC_OK;
  for (int i = 0; i < G.n; i++)
    if (G.g[i].exec && hipGraphExecDestroy(G.g[i].exec) != hipSuccess) rc = GC_ERR_HIP;
  G.n = 0;
  if (G.cap && hipStreamDestroy(G.cap) != hipSuccess) rc = GC_ERR_HIP;
  G.cap = nullptr;
  return rc;
}

}  // namespace gc

using namespace gc;

extern "C" {

int gc_step_mlp_release(void) { return release_step_graphs(); }

size_t gc_mlp_workspace_bytes(int rows, const gc_mlp_params* w) {
  if (rows < 1 || check_mlp_params(w) != GC_OK) return 0;
  return carve_mlp_ws(nullptr, rows, w).total;
}

int gc_mlp_forward_nograd_bf16(const void* x, int rows, const gc_mlp_params* w, void* y, void* workspace,
                               size_t workspace_bytes, void* stream) {
  if (!x || !y) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (rows < 1 || rows > (1 << 24)) return GC_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < carve_mlp_ws(nullptr, rows, w).total)
    return GC_ERR_WORKSPACE;
  const MlpWs ws = carve_mlp_ws((char*)workspace, rows, w);
  if (mlp_prepare(w, ws, (hipStream_t)stream) != hipSuccess) return GC_ERR_HIP;
  return mlp_forward(x, rows, w, ws, false, y, (hipStream_t)stream, rows >= kGemmRows) == hipSuccess ? GC_OK : GC_ERR_HIP;
}

int gc_chunk_surrogate_backward_bf16(const void* x_chunk, int rows, const gc_mlp_params* w, const float* cached_grad_rows,
                                     const gc_mlp_grads* acc, void* workspace, size_t workspace_bytes, void* stream) {
  if (!x_chunk || !cached_grad_rows || !acc) return GC_ERR_NULL;
  if (!acc->dW1 || !acc->db1 || !acc->dW2 || !acc->db2) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (rows < 1 || rows > (1 << 24)) return GC_ERR_SHAPE;
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < carve_mlp_ws(nullptr, rows, w).total)
    return GC_ERR_WORKSPACE;
  const MlpWs ws = carve_mlp_ws((char*)workspace, rows, w);
  if (mlp_prepare(w, ws, (hipStream_t)stream) != hipSuccess) return GC_ERR_HIP;
  return mlp_backward(x_chunk, rows, w, cached_grad_rows, acc, ws, (hipStream_t)stream) == hipSuccess ? GC_OK : GC_ERR_HIP;
}

size_t gc_step_mlp_grouped_workspace_bytes(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w, int accumulate_group) {
  if (B < 1 || P < 1 || chunk_q < 1 || chunk_p < 1 || accumulate_group < 1 || check_mlp_params(w) != GC_OK) return 0;
  return plan_step(B, P, chunk_q, chunk_p, w, accumulate_group).total;
}
size_t gc_step_mlp_workspace_bytes(int B, int P, int chunk_q, int chunk_p, const gc_mlp_params* w) {
  return gc_step_mlp_grouped_workspace_bytes(B, P, chunk_q, chunk_p, w, 1);
}

int gc_step_mlp_bf16(const void* x_q, int B, const void* x_p, int P, const int32_t* pos_idx, int chunk_q, int chunk_p,
                     const gc_mlp_params* w, float scale, float temp, float* loss, const gc_mlp_grads* grads, void* q_rep,
                     void* p_rep, float* dq, float* dp, void* workspace, size_t workspace_bytes, void* stream) {
  return gc_step_mlp_grouped_bf16(x_q, B, x_p, P, pos_idx, chunk_q, chunk_p, 1, w, scale, temp, loss, grads, q_rep, p_rep,
                                  dq, dp, workspace, workspace_bytes, stream);
}

int gc_step_mlp_grouped_bf16(const void* x_q, int B, const void* x_p, int P, const int32_t* pos_idx, int chunk_q,
                             int chunk_p, int accumulate_group, const gc_mlp_params* w, float scale, float temp, float* loss,
                             const gc_mlp_grads* grads, void* q_rep, void* p_rep, float* dq, float* dp, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (accumulate_group < 1 || accumulate_group > 8) return GC_ERR_SHAPE;
  if (!x_q || !x_p || !pos_idx || !loss || !grads) return GC_ERR_NULL;
  if (!grads->dW1 || !grads->db1 || !grads->dW2 || !grads->db2) return GC_ERR_NULL;
  int rc = check_mlp_params(w);
  if (rc != GC_OK) return rc;
  if (B < 1 || P < 1 || chunk_q < 1 || chunk_p < 1 || B > (1 << 24) || P > (1 << 24)) return GC_ERR_SHAPE;
  if (!(scale > 0.f) || !(temp > 0.f) || !(scale / temp > 0.f) || !(scale / temp < 3.0e38f)) return GC_ERR_SHAPE;
  const StepWs sw = plan_step(B, P, chunk_q, chunk_p, w, accumulate_group);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sw.total) return GC_ERR_WORKSPACE;
  StepCall c;
  memset(&c, 0, sizeof(c));  // the struct is compared bytewise: no stray padding
  c.x_q = x_q; c.x_p = x_p; c.pos_idx = pos_idx; c.B = B; c.P = P; c.chunk_q = chunk_q; c.chunk_p = chunk_p;
  c.w = *w; c.scale = scale; c.temp = temp; c.loss = loss; c.grads = *grads; c.q_rep = q_rep; c.p_rep = p_rep;
  c.dq = dq; c.dp = dp; c.workspace = workspace; c.group = accumulate_group;
  return run_step(c, (hipStream_t)stream);
}


// ---- parameterised distance function (Sec. "Extend to Deep Distance Function"), bilinear form ---------------
// d_ij = f_i^T Omega g_j = <h_i, g_j> with h_i = Omega^T f_i: the loss path on (H, G) gives the loss, A = dL/dH
// (rows a_i = sum_j w_ij g_j) and v = dL/dG (rows sum_i w_ij h_i); then u = A Omega^T and dOmega = F^T A.
// The weights w_ij live only inside the tiles of the loss kernels.
struct BilinearWs { size_t off_loss, loss_bytes, off_omT, off_H, off_A, off_part, total; int slices, rows_per_slice; };
static BilinearWs plan_bilinear(int B, int P, int d) {
  BilinearWs w{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = up256(off + bytes); return o; };
  w.loss_bytes = gc_workspace_bytes(B, P, d, GC_BF16);
  w.off_loss = take(w.loss_bytes);
  w.off_omT = take((size_t)d * d * 2);
  w.off_H = take((size_t)B * d * 2);
  w.off_A = take((size_t)B * d * 4);
  const int tiles = (d / 128) * (d / WG_M);
  int slices = (4 * num_cu() + tiles - 1) / tiles;           // about four workgroups per CU
  const int max_slices = (B + 127) / 128;                   // at least 128 rows per slice
  if (slices > max_slices) slices = max_slices;
  if (slices > 64) slices = 64;
  if (slices < 1) slices = 1;
  w.rows_per_slice = ((B + slices - 1) / slices + 31) / 32 * 32;
  w.slices = (B + w.rows_per_slice - 1) / w.rows_per_slice;
  w.off_part = take((size_t)w.slices * d * d * 4);
  w.total = off;
  return w;
}
static bool bilinear_shape_ok(int B, int P, int d) {
  return B >= 1 && P >= 1 && d >= 1 && (long long)B * d <= (1ll << 40) && (long long)P * d <= (1ll << 40);
}

size_t gc_bilinear_workspace_bytes(int B, int P, int d) {
  if (!bilinear_shape_ok(B, P, d) || d % 128 || d > 768) return 0;
  return plan_bilinear(B, P, d).total;
}

int gc_bilinear_workspace_layout(int B, int P, int d, size_t* off_h, size_t* off_a) {
  if (!off_h || !off_a) return GC_ERR_NULL;
  if (!bilinear_shape_ok(B, P, d)) return GC_ERR_SHAPE;
  if (d % 128 || d > 768) return GC_ERR_UNSUPPORTED;
  const BilinearWs w = plan_bilinear(B, P, d);
  *off_h = w.off_H;
  *off_a = w.off_A;
  return GC_OK;
}

int gc_bilinear_loss_and_grads_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                    const void* omega, float scale, float temp, float* loss, float* u, float* v,
                                    float* domega, void* workspace, size_t workspace_bytes, void* stream) {
  if (!q || !p || !pos_idx || !omega || !loss || !u || !v || !domega) return GC_ERR_NULL;
  if (!bilinear_shape_ok(B, P, d)) return GC_ERR_SHAPE;
  if (!(scale > 0.f) || !(temp > 0.f) || !std::isfinite(scale) || !std::isfinite(temp) || !std::isfinite(scale / temp) ||
      !(scale / temp > 0.f))
    return GC_ERR_SHAPE;
  if (d % 128 || d > 768) return GC_ERR_UNSUPPORTED;
  const BilinearWs w = plan_bilinear(B, P, d);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return GC_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t s = (hipStream_t)stream;
  unsigned short* omT = (unsigned short*)(ws + w.off_omT);
  unsigned short* H = (unsigned short*)(ws + w.off_H);
  float* A = (float*)(ws + w.off_A);
  float* part = (float*)(ws + w.off_part);
  // H = F Omega (bf16): Bt[n][k] = Omega[k][n]
  transpose_bf16_kernel<<<dim3(d / 32, d / 32), 256, 0, s>>>((const unsigned short*)omega, d, d, omT);
  {
    GemmArgs g{};
    g.A = q; g.lda = d; g.Bt = omT; g.ldb = d; g.M = B; g.N = d; g.K = d; g.C = H; g.ldc = d;
    if (launch_gemm_nt<false, GO_BF16>(g, s) != hipSuccess) return GC_ERR_HIP;
  }
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  // loss, A = dL/dH, v = dL/dG
  int rc = gc_loss_and_rep_grad_ex(GC_BF16, H, p, pos_idx, B, P, d, scale, temp, 0, loss, A, v, nullptr, nullptr,
                                   ws + w.off_loss, w.loss_bytes, stream);
  if (rc != GC_OK) return rc;
  {  // u = A Omega^T: Bt[n][k] = Omega[n][k]
    GemmArgs g{};
    g.A = A; g.lda = d; g.Bt = (const unsigned short*)omega; g.ldb = d; g.M = B; g.N = d; g.K = d; g.C = u; g.ldc = d;
    if (launch_gemm_nt<true, GO_F32>(g, s) != hipSuccess) return GC_ERR_HIP;
  }
  {  // dOmega = F^T A, the rows cut into slices, partial sums in a fixed order
    WgradArgs g{};
    g.A = q; g.lda = d; g.B = A; g.ldb = d; g.M = d; g.N = d; g.K = B; g.C = part; g.ldc = d;
    wgrad_splitk_kernel<false, true><<<(d / 128) * (d / WG_M) * w.slices, 256, 0, s>>>(g, w.rows_per_slice);
    if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
    const float* srcs[1] = {part}; int counts[1] = {w.slices}; size_t strides[1] = {(size_t)d * d};
    if (launch_partial_reduce(domega, srcs, counts, strides, 1, (size_t)d * d, s) != hipSuccess) return GC_ERR_HIP;
  }
  return GC_OK;
}

// ---- deep distance function, Phi = sum_k w_k tanh((A f)_k + (C g)_k) --------------------------------------------
size_t gc_deepdist_workspace_bytes(int B, int P, int d, int h) {
  if (deep_shape_status(B, P, d, h) != GC_OK) return 0;
  return plan_deep(B, P, d, h).total;
}

int gc_deepdist_loss_and_grads_bf16(const void* q, const void* p, const int32_t* pos_idx, int B, int P, int d,
                                    const void* A, const void* C, const void* w, int h, float scale, float temp,
                                    float* loss, float* u, float* v, float* dA, float* dC, float* dw, void* workspace,
                                    size_t workspace_bytes, void* stream) {
  if (!q || !p || !pos_idx || !A || !C || !w || !loss || !u || !v || !dA || !dC || !dw) return GC_ERR_NULL;
  int rc = deep_shape_status(B, P, d, h);
  if (rc != GC_OK) return rc;
  if (!(scale > 0.f) || !(temp > 0.f) || !std::isfinite(scale) || !std::isfinite(temp) || !std::isfinite(scale / temp) ||
      !(scale / temp > 0.f))
    return GC_ERR_SHAPE;
  const DeepWs pw = plan_deep(B, P, d, h);
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < pw.total) return GC_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  hipStream_t s = (hipStream_t)stream;
  const float alpha = scale / temp;
  float* a2 = (float*)(ws + pw.off_a);
  float* c2 = (float*)(ws + pw.off_c);
  unsigned short* AT = (unsigned short*)(ws + pw.off_AT);
  unsigned short* CT = (unsigned short*)(ws + pw.off_CT);
  // a = 2 log2(e) F A^T, c = 2 log2(e) G C^T (fp32): Bt[n][k] = A[n][k] as stored
  auto project = [&](const void* x, int rows, const void* M, float* out) {
    SkinnyArgs g{};
    g.A = x; g.lda = d; g.Bt = (const unsigned short*)M; g.ldb = d; g.M = rows; g.N = h; g.K = d; g.Cf = out; g.ldc = h;
    g.plain_mul = 2.f * kLog2e;
    mlp_skinny_kernel<false, EP_PLAIN><<<dim3(h / 32, (rows + 31) / 32), 256, 0, s>>>(g);
  };
  project(q, B, A, a2);
  project(p, P, C, c2);
  transpose_bf16_kernel<<<dim3(d / 32, h / 32), 256, 0, s>>>((const unsigned short*)A, h, d, AT);   // A^T [d][h]
  transpose_bf16_kernel<<<dim3(d / 32, h / 32), 256, 0, s>>>((const unsigned short*)C, h, d, CT);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  const int obA = (B + DD_OWN - 1) / DD_OWN, obC = (P + DD_OWN - 1) / DD_OWN;
  DdArgs g{};
  g.wv = (const unsigned short*)w; g.alpha2 = alpha * kLog2e; g.out_scale = alpha / (float)B; g.pos_idx = pos_idx;
  g.part_m = (float*)(ws + pw.st.off_part_m); g.part_l = (float*)(ws + pw.st.off_part_l);
  g.pos_t = (float*)(ws + pw.st.off_pos);
  g.lse2 = (const float*)(ws + pw.st.off_lse2); g.pos_pad = (const int32_t*)(ws + pw.st.off_pos_pad);
  // anchors own, targets streamed: statistics and the sums of dL/da and e in one walk (no statistics pass), then the
  // merge of its splits (lse2, row losses, dL/da, e) and the loss
  float* da = (float*)(ws + pw.off_da);
  float* dc = (float*)(ws + pw.off_dc);
  float* e = (float*)(ws + pw.off_e);
  g.own = a2; g.str = c2; g.n_own = B; g.n_str = P; g.n_oblk = obA; g.stream_len = pw.len_a;
  g.out_a = (float*)(ws + pw.off_da_part); g.out_e = (float*)(ws + pw.off_e_part); g.pos_r = (float*)(ws + pw.off_pos_r);
  deepdist_walk_kernel<128, DD_DA><<<obA * pw.nsa, 256, 0, s>>>(g);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  {
    DdFinish f{};
    f.part_m = g.part_m; f.part_l = g.part_l; f.pos_t = g.pos_t; f.pos_idx = pos_idx;
    f.part_a = g.out_a; f.part_e = g.out_e; f.pos_r = g.pos_r; f.wv = g.wv;
    f.ns = pw.nsa; f.B = B; f.P = P; f.b_pad = pw.st.b_pad; f.out_scale = g.out_scale;
    f.lse2 = (float*)(ws + pw.st.off_lse2); f.pos_pad = (int32_t*)(ws + pw.st.off_pos_pad);
    f.rowloss = (float*)(ws + pw.st.off_rowloss); f.da = da; f.e = e;
    deepdist_finish_kernel<128><<<(pw.st.b_pad + 1) / 2, 256, 0, s>>>(f);
    if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  }
  LossArgs la{};
  la.dt = GC_BF16; la.pos_idx = pos_idx; la.B = B; la.P = P; la.d = d; la.alpha = alpha; la.loss = loss; la.ws = ws; la.stream = s;
  if (launch_loss_sum(la, pw.st) != hipSuccess) return GC_ERR_HIP;
  // targets own, anchors streamed (with their final lse2)
  g.own = c2; g.str = a2; g.n_own = P; g.n_str = B; g.n_oblk = obC; g.stream_len = pw.len_c;
  g.out_a = (float*)(ws + pw.off_dc_part); g.out_e = nullptr;
  deepdist_walk_kernel<128, DD_DC><<<obC * pw.nsc, 256, 0, s>>>(g);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  auto sum_parts = [&](float* out, size_t off_part, int parts, size_t n) {
    const float* srcs[1] = {(const float*)(ws + off_part)}; int counts[1] = {parts}; size_t strides[1] = {n};
    return launch_partial_reduce(out, srcs, counts, strides, 1, n, s);
  };
  if (sum_parts(dc, pw.off_dc_part, pw.nsc, (size_t)P * h) != hipSuccess) return GC_ERR_HIP;
  {  // dL/dw_k = sum_i e_ik: row slices, then their fixed-order sum
    int sl = (B + 255) / 256;
    if (sl > 64) sl = 64;
    const int rps = (B + sl - 1) / sl;
    sl = (B + rps - 1) / rps;
    float* wp = (float*)(ws + pw.off_wpart);
    colsum_slices_kernel<<<dim3(h / 32, sl), 256, 0, s>>>(e, B, h, rps, wp);
    if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
    if (sum_parts(dw, pw.off_wpart, sl, (size_t)h) != hipSuccess) return GC_ERR_HIP;
  }
  // u = dL/da A, v = dL/dc C (third and fourth equation): Bt[n][k] = A^T[n][k]
  auto pull = [&](const float* grad, int rows, const unsigned short* MT, float* out) {
    SkinnyArgs k{};
    k.A = grad; k.lda = h; k.Bt = MT; k.ldb = h; k.M = rows; k.N = d; k.K = h; k.Cf = out; k.ldc = d;
    mlp_skinny_kernel<true, EP_PLAIN><<<dim3(d / 32, (rows + 31) / 32), 256, 0, s>>>(k);
  };
  pull(da, B, AT, u);
  pull(dc, P, CT, v);
  if (hipGetLastError() != hipSuccess) return GC_ERR_HIP;
  // dL/dA = (dL/da)^T F, dL/dC = (dL/dc)^T G (second equation): rows cut into slices, partial sums in a fixed order
  auto param_grad = [&](const float* grad, const void* x, int rows, int slices, int rps, float* out) {
    float* part = (float*)(ws + pw.off_gpart);
    WgradArgs k{};
    k.A = grad; k.lda = h; k.B = x; k.ldb = d; k.M = h; k.N = d; k.K = rows; k.C = part; k.ldc = d;
    wgrad_splitk_kernel<true, false><<<(d / 128) * (h / WG_M) * slices, 256, 0, s>>>(k, rps);
    if (hipGetLastError() != hipSuccess) return hipErrorUnknown;
    return sum_parts(out, pw.off_gpart, slices, (size_t)h * d);
  };
  if (param_grad(da, q, B, pw.slices_b, pw.rps_b, dA) != hipSuccess) return GC_ERR_HIP;
  if (param_grad(dc, p, P, pw.slices_p, pw.rps_p, dC) != hipSuccess) return GC_ERR_HIP;
  return GC_OK;
}

}  // extern "C"
