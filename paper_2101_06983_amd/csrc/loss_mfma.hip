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
// streamed = Q) and walks the streamed matrix 32 rows at a time:
//   phase 1  S^T tile [32 streamed x 64 owner] = R_tile * O^T.  The contraction over d is split
//            four ways over the waves (wave w takes columns [w*D/4, (w+1)*D/4)), so that each
//            wave keeps its slice of the owner rows in registers for the whole kernel and only
//            ever touches its own D/4-column slice of every streamed tile.
//   exchange the four partial tiles are summed through LDS (each wave reduces one quarter in a
//            fixed order), turned into g = 2^(t - lse2) - [j = r_i] (Eq. 5 / Eq. 6 with eps_j of
//            Eq. 7 folded in), rounded to bf16 and published as ready-made MFMA A fragments.
//   phase 2  dO[64 x D/4 slice] += g[64 x 32] * R_tile[32 x D/4 slice]; the streamed slice is read
//            back from the same LDS buffer with transposing loads (ds_read_b64_tr_b16).
// ===========================================================================
constexpr int GR_OWN = 64, GR_T = 32;

template <int D>
struct GradCfg {
  static constexpr int DS = D / 4;        // columns per wave
  static constexpr int KS = DS / 16;      // MFMA k-steps of phase 1
  static constexpr int CT = DS / 32;      // 32-column output tiles of phase 2
  static constexpr int C16 = DS / 8;      // 16-byte chunks per slice row
  static constexpr int SLOTS = C16 + 1;   // + one 16-byte pad chunk per row (bank skew)
  static constexpr int LD = SLOTS * 8;    // LDS row stride of the streamed slice (bf16 elements)
  static constexpr int NI = (GR_T * SLOTS + 63) / 64;   // direct-to-LDS load instructions per tile slice
  static constexpr int RS_WAVE_BYTES = NI * 1024;       // one wave, one stage
  static constexpr int RS_BYTES = 2 * 4 * RS_WAVE_BYTES;  // two stages, four waves
  static constexpr int X_BYTES = 4 * 4 * 2 * 64 * 16;   // [src][dst][quad][lane] float4
  static constexpr int G_BYTES = 4 * 64 * 16;           // [frag][lane] bf16x8
  static constexpr int SMEM = RS_BYTES + X_BYTES + G_BYTES;
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

// 16 bytes per lane from global memory straight into LDS at lds_base + lane * 16 (wave-uniform
// base in M0).  The compiler does not see the LDS write: the reader waits with wait_vmem0().
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
__device__ __forceinline__ void wait_vmem0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

template <int D, bool OWNER_IS_Q>
__device__ __forceinline__ void grad_body(const GradArgs& ga, int oblk, int split, unsigned char* smem) {
  using C = GradCfg<D>;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, ln = lane & 31;
  const unsigned short* O = OWNER_IS_Q ? ga.Q : ga.P;
  const unsigned short* R = OWNER_IS_Q ? ga.P : ga.Q;
  const int No = OWNER_IS_Q ? ga.B : ga.Pn, Nr = OWNER_IS_Q ? ga.Pn : ga.B;
  const int slen = OWNER_IS_Q ? ga.q_stream_len : ga.p_stream_len;
  const int a0 = oblk * GR_OWN;
  const int sbeg = split * slen, send = min(Nr, sbeg + slen);

  unsigned char* rs_wave = smem + w * (2 * C::RS_WAVE_BYTES);  // this wave's two stages
  const unsigned rs_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)rs_wave);
  f32x4* X = (f32x4*)(smem + C::RS_BYTES);
  bf16x8* Gf = (bf16x8*)(smem + C::RS_BYTES + C::X_BYTES);

  // owner slice, kept in registers as MFMA B fragments of phase 1
  bf16x8 ofrag[2][C::KS];
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const int row = min(a0 + 32 * nt + ln, No - 1);
#pragma unroll
    for (int ks = 0; ks < C::KS; ks++)
      ofrag[nt][ks] = *(const bf16x8*)(O + (size_t)row * D + w * C::DS + 16 * ks + 8 * h);
  }
  // the quarter of the score tile this wave finishes: owner column block nt_q, streamed rows 16*s_q + ...
  const int nt_q = w >> 1, s_q = w & 1;
  const int a_q = a0 + 32 * nt_q + ln;  // owner row of every value this lane finishes
  float lse_a = 0.f; int r_a = -1;
  if (OWNER_IS_Q) {
    lse_a = ga.lse2[a_q];      // padded: +inf past the end, so g = 0 there
    r_a = ga.pos_pad[a_q];
  }

  // per-lane source offsets of the direct-to-LDS loads (slot q = it * 64 + lane -> row, chunk)
  int src_off[C::NI];  // element offset inside the streamed tile: row * D + chunk * 8
  int src_row[C::NI];
#pragma unroll
  for (int it = 0; it < C::NI; it++) {
    const int q = it * 64 + lane;
    const int row = min(q / C::SLOTS, GR_T - 1), c = min(q % C::SLOTS, C::C16 - 1);
    src_row[it] = row;
    src_off[it] = w * C::DS + c * 8;
  }
  auto prefetch = [&](int t0, int stage) {
#pragma unroll
    for (int it = 0; it < C::NI; it++) {
      const int grow = min(t0 + src_row[it], Nr - 1);
      dma16(R + (size_t)grow * D + src_off[it], rs_base + stage * C::RS_WAVE_BYTES + it * 1024);
    }
  };

  f32x16 acc[2][C::CT];
#pragma unroll
  for (int mt = 0; mt < 2; mt++)
#pragma unroll
    for (int ct = 0; ct < C::CT; ct++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mt][ct][r] = 0.f;

  // softmax statistics of the streamed rows this lane finishes (dP role), fetched one tile ahead
  const int brel = 16 * s_q + 4 * h;  // rows brel + {0..3} and brel + 8 + {0..3}
  f32x4 nx_lse[2]; i32x4 nx_pos[2];
  auto fetch_rowinfo = [&](int t0) {
    if (!OWNER_IS_Q) {
#pragma unroll
      for (int g = 0; g < 2; g++) {
        nx_lse[g] = *(const f32x4*)(ga.lse2 + t0 + brel + 8 * g);
        nx_pos[g] = *(const i32x4*)(ga.pos_pad + t0 + brel + 8 * g);
      }
    }
  };

  fetch_rowinfo(sbeg);
  prefetch(sbeg, 0);
  int stage = 0;
  for (int t0 = sbeg; t0 < send; t0 += GR_T, stage ^= 1) {
    wait_vmem0();  // tile t0 (issued one step ago) has landed in this wave's LDS stage
    f32x4 cur_lse[2]; i32x4 cur_pos[2];
    if (!OWNER_IS_Q) {
#pragma unroll
      for (int g = 0; g < 2; g++) { cur_lse[g] = nx_lse[g]; cur_pos[g] = nx_pos[g]; }
    }
    if (t0 + GR_T < send) {
      fetch_rowinfo(t0 + GR_T);
      prefetch(t0 + GR_T, stage ^ 1);
    }
    const unsigned short* Rs = (const unsigned short*)(rs_wave + stage * C::RS_WAVE_BYTES);
    // ---- phase 1: partial S^T over this wave's k-slice ---------------------------------------------
    f32x16 sacc[2];
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int r = 0; r < 16; r++) sacc[nt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::KS; ks++) {
      bf16x8 af = *(const bf16x8*)(Rs + ln * C::LD + 16 * ks + 8 * h);
      sacc[0] = mfma32(af, ofrag[0][ks], sacc[0]);
      sacc[1] = mfma32(af, ofrag[1][ks], sacc[1]);
    }
    // ---- exchange: hand the other waves their quarters ----------------------------------------------
#pragma unroll
    for (int dst = 0; dst < 4; dst++) {
      // (the wave's own quarter is written too: one branch-free store pattern for all waves)
#pragma unroll
      for (int qd = 0; qd < 2; qd++) {
        f32x4 v;
#pragma unroll
        for (int x = 0; x < 4; x++) v[x] = sacc[dst >> 1][8 * (dst & 1) + 4 * qd + x];
        X[((w * 4 + dst) * 2 + qd) * 64 + lane] = v;
      }
    }
    __syncthreads();
    float sv[8];
#pragma unroll
    for (int e = 0; e < 8; e++) sv[e] = 0.f;
#pragma unroll
    for (int src = 0; src < 4; src++) {  // fixed order: bit-identical whichever wave sums
#pragma unroll
      for (int qd = 0; qd < 2; qd++) {
        f32x4 v = X[((src * 4 + w) * 2 + qd) * 64 + lane];
#pragma unroll
        for (int x = 0; x < 4; x++) sv[4 * qd + x] += v[x];
      }
    }
    // ---- g = softmax - Y for the 8 finished scores of this lane ------------------------------------------
    unsigned gp[4];
    {
      float gv[8];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const int b = t0 + brel + 8 * (e >> 2) + (e & 3);  // streamed row
        float lse_i; int r_i, i, j;
        if (OWNER_IS_Q) {
          lse_i = lse_a; r_i = r_a; i = a_q; j = b;
        } else {
          lse_i = cur_lse[e >> 2][e & 3]; r_i = cur_pos[e >> 2][e & 3]; i = b; j = a_q;
        }
        float p = fast_exp2(sv[e] * ga.alpha2 - lse_i);
        float g = p - ((j == r_i) ? 1.f : 0.f);
        if (b >= send || (ga.mask_self && i == j)) g = 0.f;
        gv[e] = g;
      }
#pragma unroll
      for (int x = 0; x < 4; x++) gp[x] = pack2bf(gv[2 * x], gv[2 * x + 1]);
    }
    {
      u32x4 pk = {gp[0], gp[1], gp[2], gp[3]};
      ((u32x4*)Gf)[w * 64 + lane] = pk;  // fragment (mt = nt_q, k-step = s_q)
    }
    __syncthreads();
    // ---- phase 2: dO += g * R_tile slice ---------------------------------------------------------------------
    bf16x8 gf[2][2];
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int s = 0; s < 2; s++) gf[mt][s] = Gf[(mt * 2 + s) * 64 + lane];
#pragma unroll
    for (int ct = 0; ct < C::CT; ct++) {
#pragma unroll
      for (int s = 0; s < 2; s++) {
        const int col = 32 * ct + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
        const int row = 16 * s + 4 * h + ((lane & 15) >> 2);
        s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Rs + row * C::LD + col));
        s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(Rs + (row + 8) * C::LD + col));
        s16x8 bb = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        bf16x8 bfr = __builtin_bit_cast(bf16x8, bb);
        acc[0][ct] = mfma32(gf[0][s], bfr, acc[0][ct]);
        acc[1][ct] = mfma32(gf[1][s], bfr, acc[1][ct]);
      }
    }
  }

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
