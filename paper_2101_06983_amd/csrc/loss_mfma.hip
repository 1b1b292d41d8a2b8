// bf16 MFMA kernels of the loss / representation-gradient path for gfx950.
//
//   stats pass   Eq. 1 / Eq. 4: per anchor, online max and sum of 2^t over target tiles, the
//                positive's score and the argmax; the score tile lives in MFMA accumulators only.
//   gradient pass  Eq. 5 / Eq. 6: a workgroup owns 64 rows of dQ (or dP), streams the other
//                matrix 32 rows at a time, recomputes the score tile, forms
//                g = softmax - Y in registers and accumulates g * rows with MFMA.
//
// MFMA operand layouts used throughout (v_mfma_f32_32x32x16_bf16, D = A * B + C, wave of 64):
//   A fragment: lane l holds A[m = l % 32][k = 8 * (l / 32) + 0..7]
//   B fragment: lane l holds B[k = 8 * (l / 32) + 0..7][n = l % 32]
//   C/D:        lane l, register r holds D[m = 8 * (r / 4) + 4 * (l / 32) + r % 4][n = l % 32]
// The reduction over targets is put on the M axis (registers) so that every lane owns one
// anchor column and the softmax statistics need no cross-lane traffic inside a tile.
#include <type_traits>

#include "gc_common.h"

namespace gc {

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ===========================================================================
// Statistics pass.  Workgroup = 512 threads = 8 waves as 2 (targets, M) x 4 (anchors, N);
// workgroup tile 256 targets x 256 anchors, wave tile 128 x 64 (4 x 2 MFMA tiles).
// k is staged through LDS in chunks of 64, two stages.
// ===========================================================================
constexpr int ST_TM = 256, ST_TN = 256, ST_KC = 64;
constexpr int ST_LD = ST_KC + 8;  // LDS row stride in bf16 elements (144 B: 16 B skew per row)
constexpr int ST_STAGE = (ST_TM + ST_TN) * ST_LD;  // elements per stage

__device__ __forceinline__ void stat_merge(float& m, float& l, int& idx, float m2, float l2, int idx2) {
  // (m, idx): larger value wins, ties to the smaller index
  bool take = (m2 > m) || (m2 == m && idx2 < idx);
  float mn = fmaxf(m, m2);
  float ms = (mn == -INFINITY) ? 0.f : mn;
  l = l * fast_exp2(m - ms) + l2 * fast_exp2(m2 - ms);
  idx = take ? idx2 : idx;
  m = mn;
}

__global__ void __launch_bounds__(512) stats_mfma_kernel(const unsigned short* __restrict__ Q,
                                                         const unsigned short* __restrict__ Pm,
                                                         const int32_t* __restrict__ pos_idx, int B, int P, int d,
                                                         float alpha2, int mask_self, int n_ablk, int cols_per_split,
                                                         float* __restrict__ part_m, float* __restrict__ part_l,
                                                         int* __restrict__ part_idx, float* __restrict__ pos_t) {
  extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int ablk = blockIdx.x % n_ablk, split = blockIdx.x / n_ablk;
  const int a0 = ablk * ST_TN;
  const int cbeg = split * cols_per_split, cend = min(P, cbeg + cols_per_split);
  const int nk = d / ST_KC;

  // global -> LDS mapping: a row of a stage is 64 bf16 = 8 x 16 B; thread covers (row = tid/8 + 64*pass, c16 = tid%8)
  const int lrow = tid >> 3, lc16 = tid & 7;

  // per-lane running statistics for its two anchor columns
  float rm[2], rl[2], rpos[2];
  int ridx[2], a_col[2], r_of[2];
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    rm[nt] = -INFINITY; rl[nt] = 0.f; rpos[nt] = 0.f; ridx[nt] = 0x7fffffff;
    a_col[nt] = a0 + wn * 64 + nt * 32 + (lane & 31);
    r_of[nt] = (a_col[nt] < B) ? pos_idx[a_col[nt]] : -1;
  }

  for (int b0 = cbeg; b0 < cend; b0 += ST_TM) {
    f32x16 acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
      for (int nt = 0; nt < 2; nt++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[mt][nt][r] = 0.f;

    u32x4 stg[8];
    auto gload = [&](int kc) {
#pragma unroll
      for (int ps = 0; ps < 4; ps++) {
        int rb = min(b0 + lrow + 64 * ps, P - 1);
        stg[ps] = *(const u32x4*)(Pm + (size_t)rb * d + kc * ST_KC + lc16 * 8);
        int ra = min(a0 + lrow + 64 * ps, B - 1);
        stg[4 + ps] = *(const u32x4*)(Q + (size_t)ra * d + kc * ST_KC + lc16 * 8);
      }
    };
    auto lstore = [&](int stage) {
      unsigned short* As = smem + stage * ST_STAGE;
      unsigned short* Bs = As + ST_TM * ST_LD;
#pragma unroll
      for (int ps = 0; ps < 4; ps++) {
        *(u32x4*)(As + (lrow + 64 * ps) * ST_LD + lc16 * 8) = stg[ps];
        *(u32x4*)(Bs + (lrow + 64 * ps) * ST_LD + lc16 * 8) = stg[4 + ps];
      }
    };
    __syncthreads();  // previous tile's readers are done with both stages
    gload(0);
    lstore(0);
    __syncthreads();
    for (int kc = 0; kc < nk; kc++) {
      if (kc + 1 < nk) gload(kc + 1);
      const unsigned short* As = smem + (kc & 1) * ST_STAGE;
      const unsigned short* Bs = As + ST_TM * ST_LD;
#pragma unroll
      for (int ks = 0; ks < ST_KC / 16; ks++) {
        bf16x8 af[4], bfg[2];
        const int kof = ks * 16 + 8 * (lane >> 5);
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
          af[mt] = *(const bf16x8*)(As + (wm * 128 + mt * 32 + (lane & 31)) * ST_LD + kof);
#pragma unroll
        for (int nt = 0; nt < 2; nt++)
          bfg[nt] = *(const bf16x8*)(Bs + (wn * 64 + nt * 32 + (lane & 31)) * ST_LD + kof);
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int nt = 0; nt < 2; nt++) acc[mt][nt] = mfma32(af[mt], bfg[nt], acc[mt][nt]);
      }
      if (kc + 1 < nk) lstore((kc + 1) & 1);
      __syncthreads();
    }

    // ---- tile epilogue: online softmax statistics, all in registers -----------------------------
    const int brow0 = b0 + wm * 128 + 4 * (lane >> 5);  // + mt*32 + 8*(r/4) + r%4
    const bool edge = (b0 + ST_TM > cend);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const int a = a_col[nt];
      // scale to base-2 logits, apply the masks that can touch this tile
      const bool diag = mask_self && (a >= b0 && a < b0 + ST_TM);
      const bool haspos = (unsigned)(r_of[nt] - b0) < (unsigned)ST_TM;
#pragma unroll
      for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[mt][nt][r] *= alpha2;
      if (edge || diag || haspos) {  // rare: the general slow walk
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            int j = brow0 + mt * 32 + 8 * (r >> 2) + (r & 3);
            float t = acc[mt][nt][r];
            if (j == r_of[nt]) rpos[nt] = t;
            if (j >= cend || (mask_self && j == a)) acc[mt][nt][r] = -INFINITY;
          }
      }
      // tile max + first index attaining it (rows are visited in increasing j within mt; across
      // register order j is increasing too, so a strict > keeps the smallest index)
      float tm = -INFINITY; int ti = 0x7fffffff;
#pragma unroll
      for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float t = acc[mt][nt][r];
          int j = brow0 + mt * 32 + 8 * (r >> 2) + (r & 3);
          bool gt = t > tm;
          tm = gt ? t : tm;
          ti = gt ? j : ti;
        }
      if (tm > -INFINITY) {
        float mn = fmaxf(rm[nt], tm);
        float s = 0.f;
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int r = 0; r < 16; r++) s += fast_exp2(acc[mt][nt][r] - mn);
        rl[nt] = rl[nt] * fast_exp2(rm[nt] - mn) + s;
        if (tm > rm[nt]) ridx[nt] = ti;  // later tiles have larger j: strict >
        rm[nt] = mn;
      }
    }
  }

  // ---- combine the two half-waves (same anchor column, different target rows) -------------------
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    float m2 = __shfl_xor(rm[nt], 32), l2 = __shfl_xor(rl[nt], 32);
    int i2 = __shfl_xor(ridx[nt], 32);
    stat_merge(rm[nt], rl[nt], ridx[nt], m2, l2, i2);
  }
  // ---- combine the two waves along M through LDS, then write the split partial ------------------
  __syncthreads();
  float* xs = (float*)smem;  // [4 wn][2 nt][32][3]
  if (wm == 1 && lane < 32) {
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      float* x = xs + ((wn * 2 + nt) * 32 + lane) * 3;
      x[0] = rm[nt]; x[1] = rl[nt]; x[2] = __builtin_bit_cast(float, ridx[nt]);
    }
  }
  __syncthreads();
  if (wm == 0 && lane < 32) {
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const float* x = xs + ((wn * 2 + nt) * 32 + lane) * 3;
      stat_merge(rm[nt], rl[nt], ridx[nt], x[0], x[1], __builtin_bit_cast(int, x[2]));
      int a = a_col[nt];
      if (a < B) {
        part_m[(size_t)split * B + a] = rm[nt];
        part_l[(size_t)split * B + a] = rl[nt];
        part_idx[(size_t)split * B + a] = ridx[nt];
      }
    }
  }
  // the positive's score is seen by exactly one lane of one workgroup
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    int a = a_col[nt], r = r_of[nt];
    if (a < B && r >= cbeg && r < cend && !(mask_self && r == a)) {
      // lane that held row r: rows of this lane are brow(mt, reg) with 4*(lane>>5) offset
      int rel = (r - cbeg) % ST_TM;  // row inside its tile
      int wmr = rel / 128, in = rel % 128;
      int half = (in % 8) / 4;
      if (wmr == wm && half == (lane >> 5)) pos_t[a] = rpos[nt];
    }
  }
}

hipError_t launch_stats_mfma(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  const int n_ablk = (a.B + ST_TN - 1) / ST_TN;
  const size_t smem = (size_t)2 * ST_STAGE * sizeof(unsigned short);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)stats_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  stats_mfma_kernel<<<n_ablk * pl.stat_splits, 512, smem, a.stream>>>(
      (const unsigned short*)a.q, (const unsigned short*)a.p, a.pos_idx, a.B, a.P, a.d, a.alpha * kLog2e,
      (a.flags & GC_MASK_SELF) ? 1 : 0, n_ablk, pl.stat_cols_per_split, (float*)(ws + pl.off_part_m),
      (float*)(ws + pl.off_part_l), (int*)(ws + pl.off_part_idx), (float*)(ws + pl.off_pos));
  return hipGetLastError();
}


// ===========================================================================
// Gradient pass.  Workgroup = 256 threads = 4 waves, one per SIMD (up to 512 registers a lane).
// It owns 64 rows of the output (dQ rows: "owner" = Q, streamed = P; dP rows: owner = P,
// streamed = Q) and walks the streamed matrix 16 rows at a time:
//   phase 1  S^T tile [16 streamed x 64 owner] = R_tile * O^T (v_mfma_f32_16x16x32_bf16).  The
//            contraction over d is split four ways over the waves (wave w takes columns
//            [w*D/4, (w+1)*D/4)), so that each wave keeps its slice of the owner rows in
//            registers for the whole kernel and only ever touches its own D/4-column slice of
//            every streamed tile (a wave-private LDS ring of four stages, filled by direct
//            global->LDS loads issued three tiles ahead).
//   exchange the four partial tiles are summed through LDS (each wave finishes 16 owner rows, in
//            a fixed order), turned into g = 2^(t - lse2) - [j = r_i] (Eq. 5 / Eq. 6 with eps_j
//            of Eq. 7 folded in), rounded to bf16 and published as ready-made MFMA A fragments.
//   phase 2  dO[64 x D/4 slice] += g[64 x 16] * R_tile[16 x D/4 slice] (v_mfma_f32_32x32x16_bf16);
//            the streamed slice is read back from the same LDS stage with transposing loads
//            (ds_read_b64_tr_b16).
// The three steps of consecutive tiles are software-pipelined so that one workgroup barrier per
// tile suffices: iteration u publishes the partials of tile u+1 and the fragments of tile u,
// then runs phase 1 of tile u+2 and phase 2 of tile u while the exchanged data is in flight.
//
// 16x16x32 layouts: A lane l holds A[m = l % 16][k = 8 * (l / 16) + 0..7], B likewise with n,
// D register r of lane l holds D[m = 4 * (l / 16) + r][n = l % 16].
// ds_read_b64_tr_b16: in each group of 16 lanes, lane j supplies the address of 4 consecutive
// 16-bit elements; lane i receives element (i % 4) of the addresses of lanes i / 4 + {0, 4, 8, 12}.
// ===========================================================================
constexpr int GR_OWN = 64, GR_T = 16, GR_STAGES = 4;

template <int D>
struct GradCfg {
  static constexpr int DS = D / 4;        // columns per wave
  static constexpr int KS = DS / 32;      // MFMA k-steps of phase 1 (k = 32 each)
  static constexpr int CT = DS / 32;      // 32-column output tiles of phase 2
  static constexpr int C16 = DS / 8;      // 16-byte chunks per slice row
  static constexpr int SLOTS = C16 + 1;   // + one 16-byte pad chunk per row (bank skew)
  static constexpr int LD = SLOTS * 8;    // LDS row stride of the streamed slice (bf16 elements)
  static constexpr int TILE_SLOTS = GR_T * SLOTS;       // 16-byte slots holding tile data
  static constexpr int NI = (TILE_SLOTS + 63) / 64;     // direct-to-LDS load instructions per tile slice
  static constexpr int STAGE = NI * 1024;               // bytes: one wave, one stage
  static constexpr int RS_BYTES = 4 * GR_STAGES * STAGE;
  static constexpr int X_BYTES = 2 * 4 * 4 * 64 * 16;   // [parity][src][dst][lane] float4
  static constexpr int G_BYTES = 2 * 2 * 64 * 16;       // [parity][m-tile][lane] bf16x8
  static constexpr int SMEM = RS_BYTES + X_BYTES + G_BYTES;
  // the slots after the tile data in the last load instruction carry the row statistics of the
  // streamed rows (dP role): 4 slots of lse2, 4 slots of pos_idx
  static_assert(NI * 64 - TILE_SLOTS >= 8, "no room for the row statistics");
  static_assert(SMEM <= 160 * 1024, "LDS budget");
};

struct GradArgs {
  const unsigned short* Q;
  const unsigned short* P;
  const int32_t* pos_pad;   // pos_idx copied and padded with -1 to a multiple of 64 rows
  const float* lse2;        // log2-domain log-sum-exp per anchor, padded with +inf
  int B, Pn;
  float alpha2, out_scale;
  int mask_self;
  int obQ, nsq, q_stream_len;  // dQ-role workgroups: obQ owner blocks x nsq stream splits
  int obP, nsp, p_stream_len;
  float* dq_out; size_t dq_split_stride;  // split s writes dq_out + s * stride
  float* dp_out; size_t dp_split_stride;
};

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

// 16 bytes per lane from global memory straight into LDS at lds_base + lane * 16 (wave-uniform
// base in M0).  The compiler does not see these loads: the reader waits with wait_vmem<N>().
__device__ __forceinline__ void dma16(const void* gbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(gbase) : "memory");
}
__device__ __forceinline__ void dma16v(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

template <int D, bool OWNER_IS_Q>
__device__ __forceinline__ void grad_body(const GradArgs& ga, int oblk, int split, unsigned char* smem) {
  using C = GradCfg<D>;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, ln = lane & 31;
  const int l16 = lane & 15, g16 = lane >> 4;
  const unsigned short* O = OWNER_IS_Q ? ga.Q : ga.P;
  const unsigned short* R = OWNER_IS_Q ? ga.P : ga.Q;
  const int No = OWNER_IS_Q ? ga.B : ga.Pn, Nr = OWNER_IS_Q ? ga.Pn : ga.B;
  const int slen = OWNER_IS_Q ? ga.q_stream_len : ga.p_stream_len;
  const int a0 = oblk * GR_OWN;
  const int sbeg = split * slen, send = min(Nr, sbeg + slen);
  const int nt = (send - sbeg + GR_T - 1) / GR_T;  // streamed tiles of this workgroup (>= 1)

  unsigned char* rs_wave = smem + w * (GR_STAGES * C::STAGE);  // this wave's ring of stages
  const unsigned rs_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)rs_wave);
  unsigned char* Xb = smem + C::RS_BYTES;
  unsigned char* Gb = smem + C::RS_BYTES + C::X_BYTES;

  // owner slice, kept in registers as MFMA B fragments of phase 1 (16 owner rows per fragment)
  bf16x8 ofrag[4][C::KS];
#pragma unroll
  for (int nq = 0; nq < 4; nq++) {
    const int row = min(a0 + 16 * nq + l16, No - 1);
#pragma unroll
    for (int ks = 0; ks < C::KS; ks++)
      ofrag[nq][ks] = *(const bf16x8*)(O + (size_t)row * D + w * C::DS + 32 * ks + 8 * g16);
  }
  // this wave finishes the scores of owner rows 16 w .. 16 w + 15; a lane holds streamed rows 4 * g16 + 0..3
  const int a_q = a0 + 16 * w + l16;
  float lse_a = 0.f; int r_a = -1;
  if (OWNER_IS_Q) {
    lse_a = ga.lse2[a_q];      // padded: +inf past the end, so g = 0 there
    r_a = ga.pos_pad[a_q];
  }

  // per-lane byte offsets of the direct-to-LDS loads inside a streamed tile (slot q = it * 64 + lane
  // -> row, chunk); a full tile needs no clamping, the ragged last tile recomputes them
  unsigned src_off[C::NI];
#pragma unroll
  for (int it = 0; it < C::NI; it++) {
    const int q = it * 64 + lane;
    const int row = min(q / C::SLOTS, GR_T - 1), c = min(q % C::SLOTS, C::C16 - 1);
    src_off[it] = (unsigned)((row * D + w * C::DS + c * 8) * 2);
  }
  const int q_last = (C::NI - 1) * 64 + lane;  // slot of this lane in the last load instruction
  auto prefetch = [&](int u, bool known_full) {  // tile u -> stage u & 3
    const int t0 = sbeg + u * GR_T;
    const unsigned short* tile = R + (size_t)t0 * D;  // wave-uniform
    const unsigned lds0 = rs_base + (u & (GR_STAGES - 1)) * C::STAGE;
    const bool full = known_full || (t0 + GR_T <= Nr);
#pragma unroll
    for (int it = 0; it < C::NI; it++) {
      unsigned off = src_off[it];
      if (!full) {
        const int q = it * 64 + lane;
        const int row = min(min(q / C::SLOTS, GR_T - 1), Nr - 1 - t0), c = min(q % C::SLOTS, C::C16 - 1);
        off = (unsigned)((row * D + w * C::DS + c * 8) * 2);
      }
      if (OWNER_IS_Q || it + 1 < C::NI) {
        dma16(tile, off, lds0 + it * 1024);
      } else {
        // last instruction of the dP role: slots TILE_SLOTS..+3 fetch lse2[t0 .. t0+15], the next four pos_pad
        const char* ptr = (const char*)tile + off;
        const int e = q_last - C::TILE_SLOTS;
        if (e >= 0 && e < 4) ptr = (const char*)(ga.lse2 + t0 + 4 * e);
        if (e >= 4 && e < 8) ptr = (const char*)(ga.pos_pad + t0 + 4 * (e - 4));
        dma16v(ptr, lds0 + it * 1024);
      }
    }
  };

  f32x16 acc[2][C::CT];
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int ct = 0; ct < C::CT; ct++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mt][ct][r] = 0.f;

  f32x4 sacc[4];  // partial S^T of the tile most recently through phase 1: [owner 16-block]
  auto phase1 = [&](int u) {
    const unsigned short* Rs = (const unsigned short*)(rs_wave + (u & (GR_STAGES - 1)) * C::STAGE);
#pragma unroll
    for (int nq = 0; nq < 4; nq++) sacc[nq] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < C::KS; ks++) {
      const bf16x8 af = *(const bf16x8*)(Rs + l16 * C::LD + 32 * ks + 8 * g16);
#pragma unroll
      for (int nq = 0; nq < 4; nq++) sacc[nq] = mfma16(af, ofrag[nq][ks], sacc[nq]);
    }
  };
  auto phase2 = [&](int u, const bf16x8 (&gf)[2]) {
    const unsigned short* Rs = (const unsigned short*)(rs_wave + (u & (GR_STAGES - 1)) * C::STAGE);
    const int col = 16 * (g16 & 1) + 4 * (lane & 3);
    const int row = 8 * h + (l16 >> 2);
#pragma unroll
    for (int ct = 0; ct < C::CT; ct++) {
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Rs + row * C::LD + 32 * ct + col));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Rs + (row + 4) * C::LD + 32 * ct + col));
      s16x8 bb = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      bf16x8 bfr = __builtin_bit_cast(bf16x8, bb);
      acc[0][ct] = mfma32(gf[0], bfr, acc[0][ct]);
      acc[1][ct] = mfma32(gf[1], bfr, acc[1][ct]);
    }
  };

  bf16x4 gq = {0, 0, 0, 0};  // g of the tile whose scores were finished last (4 streamed rows of owner row a_q)

  // One pipeline iteration (see the header comment).  STEADY: every stage is live and every tile full.
  auto body = [&](int u, auto steady_tag) {
    constexpr bool STEADY = decltype(steady_tag)::value;
    const bool xw = STEADY || (u + 1 < nt);            // tile u+1: publish partials, finish scores
    const bool gw = STEADY || (u >= 0);                // tile u: publish fragments, phase 2   (u < nt always)
    const bool p1 = STEADY || (u + 2 < nt);            // tile u+2: phase 1
    const bool pf = STEADY || (u >= 0 && u + 4 < nt);  // tile u+4: start its loads
    const int par1 = (u + 1) & 1, par0 = u & 1;
    if (xw) {
#pragma unroll
      for (int dst = 0; dst < 4; dst++)
        *(f32x4*)(Xb + (((par1 * 4 + w) * 4 + dst) * 64 + lane) * 16) = sacc[dst];
    }
    if (gw) {
      // lane (w, l16, g16) holds rows 4 g16 + 0..3 of owner row 16 w + l16: half (g16 & 1) of the A fragment
      // element vector of lane 16 (w & 1) + l16 + 32 (g16 >> 1) in m-tile w >> 1
      *(bf16x4*)(Gb + (((par0 * 2 + (w >> 1)) * 64 + 16 * (w & 1) + l16 + 32 * (g16 >> 1)) * 16) + 8 * (g16 & 1)) = gq;
    }
    __syncthreads();
    f32x4 xr[4];
    if (xw) {
#pragma unroll
      for (int src = 0; src < 4; src++) xr[src] = *(const f32x4*)(Xb + (((par1 * 4 + src) * 4 + w) * 64 + lane) * 16);
    }
    bf16x8 gf[2];
    if (gw) {
#pragma unroll
      for (int mt = 0; mt < 2; mt++) gf[mt] = *(const bf16x8*)(Gb + ((par0 * 2 + mt) * 64 + lane) * 16);
    }
    f32x4 lse_r = {0.f, 0.f, 0.f, 0.f}; i32x4 pos_r = {0, 0, 0, 0};
    if (!OWNER_IS_Q && xw) {  // row statistics of tile u+1 ride in its LDS stage
      const unsigned char* st = rs_wave + ((u + 1) & (GR_STAGES - 1)) * C::STAGE + C::TILE_SLOTS * 16;
      lse_r = *(const f32x4*)(st + 16 * g16);
      pos_r = *(const i32x4*)(st + 64 + 16 * g16);
    }
    if (p1) {
      if (STEADY) wait_vmem<C::NI>(); else wait_vmem<0>();  // tile u+2 has landed (tile u+3 may be in flight)
    }
    f32x4 sv = {0.f, 0.f, 0.f, 0.f};
    if (xw) {
#pragma unroll
      for (int src = 0; src < 4; src++) sv += xr[src];  // fixed order: bit-identical whichever wave sums
    }
    if (p1) phase1(u + 2);
    if (gw) phase2(u, gf);
    if (xw) {
      typedef __attribute__((ext_vector_type(4))) float f32x4v;
      const int t1 = sbeg + (u + 1) * GR_T;
      f32x4v gv;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        const int b = t1 + 4 * g16 + e;  // streamed row
        float lse_i; int r_i, i, j;
        if (OWNER_IS_Q) {
          lse_i = lse_a; r_i = r_a; i = a_q; j = b;
        } else {
          lse_i = lse_r[e]; r_i = pos_r[e]; i = b; j = a_q;
        }
        const float p = fast_exp2(sv[e] * ga.alpha2 - lse_i);
        const float g = p - ((j == r_i) ? 1.f : 0.f);
        const bool dead = (b >= send) | ((ga.mask_self != 0) & (i == j));
        gv[e] = dead ? 0.f : g;
      }
      gq = __builtin_convertvector(gv, bf16x4);
    }
    if (pf) prefetch(u + 4, STEADY);  // a steady iteration never starts the last (possibly ragged) tile
  };

  // ---- prologue: start the first tiles, phase 1 of tile 0 ------------------------------------------------------
#pragma unroll 1
  for (int u = 0; u < min(nt, GR_STAGES); u++) prefetch(u, false);
  wait_vmem<0>();
  phase1(0);
  body(-1, std::false_type{});
  int u = 0;
#pragma unroll 1
  for (; u + 5 < nt; u++) body(u, std::true_type{});
#pragma unroll 1
  for (; u < nt; u++) body(u, std::false_type{});

  // ---- epilogue: scale by alpha / B and store the owned rows ---------------------------------------------------------
  float* out = OWNER_IS_Q ? (ga.dq_out + (size_t)split * ga.dq_split_stride) : (ga.dp_out + (size_t)split * ga.dp_split_stride);
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int ct = 0; ct < C::CT; ct++)
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const int a = a0 + 32 * mt + 8 * (r >> 2) + 4 * h + (r & 3);
        if (a < No) out[(size_t)a * D + w * C::DS + 32 * ct + ln] = acc[mt][ct][r] * ga.out_scale;
      }
}

template <int D>
__global__ void __launch_bounds__(256) grad_mfma_kernel(GradArgs ga) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gsmem[];
  const int nQ = ga.obQ * ga.nsq;
  const int id = blockIdx.x;
  if (id < nQ) {
    grad_body<D, true>(ga, id % ga.obQ, id / ga.obQ, gsmem);
  } else {
    const int t = id - nQ;
    grad_body<D, false>(ga, t % ga.obP, t / ga.obP, gsmem);
  }
}

template <int D>
static hipError_t grad_mfma_launch(const GradArgs& ga, int nwg, hipStream_t stream) {
  const int smem = GradCfg<D>::SMEM;
  hipError_t e = hipFuncSetAttribute((const void*)grad_mfma_kernel<D>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  if (e != hipSuccess) return e;
  grad_mfma_kernel<D><<<nwg, 256, smem, stream>>>(ga);
  return hipGetLastError();
}

hipError_t launch_grad_mfma(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  GradArgs ga{};
  ga.Q = (const unsigned short*)a.q; ga.P = (const unsigned short*)a.p;
  ga.pos_pad = (const int32_t*)(ws + pl.off_pos_pad); ga.lse2 = (const float*)(ws + pl.off_lse2);
  ga.B = a.B; ga.Pn = a.P;
  ga.alpha2 = a.alpha * kLog2e; ga.out_scale = a.alpha / (float)a.B;
  ga.mask_self = (a.flags & GC_MASK_SELF) ? 1 : 0;
  const bool want_q = a.dq || a.dz, want_p = a.dp || a.dz;
  const size_t nq = (size_t)a.B * a.d, np = (size_t)a.P * a.d;
  ga.obQ = want_q ? (a.B + GR_OWN - 1) / GR_OWN : 0; ga.nsq = pl.nsq; ga.q_stream_len = pl.q_stream_len;
  ga.obP = want_p ? (a.P + GR_OWN - 1) / GR_OWN : 0; ga.nsp = pl.nsp; ga.p_stream_len = pl.p_stream_len;
  const bool q_direct = (pl.nsq == 1 && !a.dz), p_direct = (pl.nsp == 1 && !a.dz);
  ga.dq_out = q_direct ? a.dq : (float*)(ws + pl.off_dq_part); ga.dq_split_stride = nq;
  ga.dp_out = p_direct ? a.dp : (float*)(ws + pl.off_dp_part); ga.dp_split_stride = np;
  const int nwg = ga.obQ * ga.nsq + ga.obP * ga.nsp;
  if (nwg == 0) { prof_mark_grad_kernel_done(a.stream); return hipSuccess; }
  hipError_t e;
  switch (a.d) {
    case 128: e = grad_mfma_launch<128>(ga, nwg, a.stream); break;
    case 256: e = grad_mfma_launch<256>(ga, nwg, a.stream); break;
    case 384: e = grad_mfma_launch<384>(ga, nwg, a.stream); break;
    case 512: e = grad_mfma_launch<512>(ga, nwg, a.stream); break;
    case 640: e = grad_mfma_launch<640>(ga, nwg, a.stream); break;
    case 768: e = grad_mfma_launch<768>(ga, nwg, a.stream); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  prof_mark_grad_kernel_done(a.stream);
  // fixed-order sums of the split partials
  if (a.dz) {
    const float* srcs[2] = {ga.dq_out, ga.dp_out};
    int counts[2] = {pl.nsq, pl.nsp};
    size_t strides[2] = {nq, np};
    return launch_partial_reduce(a.dz, srcs, counts, strides, 2, nq, a.stream);
  }
  if (want_q && !q_direct) {
    const float* srcs[1] = {ga.dq_out}; int counts[1] = {pl.nsq}; size_t strides[1] = {nq};
    e = launch_partial_reduce(a.dq, srcs, counts, strides, 1, nq, a.stream);
    if (e != hipSuccess) return e;
  }
  if (want_p && !p_direct) {
    const float* srcs[1] = {ga.dp_out}; int counts[1] = {pl.nsp}; size_t strides[1] = {np};
    e = launch_partial_reduce(a.dp, srcs, counts, strides, 1, np, a.stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace gc
