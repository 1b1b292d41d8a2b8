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

// N (1..4) direct global->LDS loads of 16 bytes per lane that share one M0 value.  Load k lands at
// lds_base + 1024 k + lane * 16 and reads gbase + voff[k] + 1024 k: the instruction's immediate
// offset moves both addresses, so callers pass voff[k] with 1024 k already subtracted.  The
// compiler does not see these loads: the reader waits with wait_vmem<N>().
// Every statement below that sets M0 says so in its clobber list.  M0 is a register the backend reserves (it never
// keeps a value of its own there across other code and sets it right before each instruction of its own that needs
// it); the clobber states the write, so that nothing it may ever cache there is assumed to survive.
template <int N>
__device__ __forceinline__ void dma_group(const void* gbase, const unsigned* voff, unsigned lds_base) {
  if constexpr (N == 1) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff[0]), "s"(gbase) : "memory", "m0");
  } else if constexpr (N == 2) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\tglobal_load_lds_dwordx4 %2, %3 offset:1024"
                 ::"s"(lds_base), "v"(voff[0]), "v"(voff[1]), "s"(gbase) : "memory", "m0");
  } else if constexpr (N == 3) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %4\n\tglobal_load_lds_dwordx4 %2, %4 offset:1024\n\t"
                 "global_load_lds_dwordx4 %3, %4 offset:2048"
                 ::"s"(lds_base), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "s"(gbase) : "memory", "m0");
  } else {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\tglobal_load_lds_dwordx4 %2, %5 offset:1024\n\t"
                 "global_load_lds_dwordx4 %3, %5 offset:2048\n\tglobal_load_lds_dwordx4 %4, %5 offset:3072"
                 ::"s"(lds_base), "v"(voff[0]), "v"(voff[1]), "v"(voff[2]), "v"(voff[3]), "s"(gbase) : "memory", "m0");
  }
}
// One such load with immediate offset IMM (a multiple of 1024 below 4096): lands at lds_base + IMM +
// lane * 16 and reads gbase + voff + IMM.  No memory clobber: the compiler may move unrelated LDS
// traffic across it; callers order it against the readers of its target with wait_vmem / barriers.
template <int IMM>
__device__ __forceinline__ void dma_piece(const void* gbase, unsigned voff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3" ::"s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM) : "m0");
}
// The same, placed by data dependences instead of fences: the statement claims to rewrite the
// registers pin_a / pin_b (it does not touch them), so it is scheduled after the last reader of
// their old values and before the first reader of the new ones, and nothing else is held up.
// LANES8: only lanes 0-7 load (128 bytes); EXEC is narrowed inside the statement and restored.
template <int IMM, bool LANES8, bool TWO>
__device__ __forceinline__ void dma_piece_pinned(const void* gbase, unsigned voff, unsigned lds_base, u32x4& pin_a, u32x4& pin_b) {
  unsigned pa = pin_a[0], pb = TWO ? pin_b[0] : 0u;
  if constexpr (LANES8) {
    unsigned long long keep;
    if constexpr (TWO)
      asm volatile("s_mov_b64 %2, exec\n\ts_mov_b64 exec, 0xff\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %4, %5 offset:%6\n\ts_mov_b64 exec, %2"
                   : "+v"(pa), "+v"(pb), "=&s"(keep) : "s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM) : "m0");
    else
      asm volatile("s_mov_b64 %1, exec\n\ts_mov_b64 exec, 0xff\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %4 offset:%5\n\ts_mov_b64 exec, %1"
                   : "+v"(pa), "=&s"(keep) : "s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM) : "m0");
  } else {
    if constexpr (TWO)
      asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %3, %4 offset:%5"
                   : "+v"(pa), "+v"(pb) : "s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM) : "m0");
    else
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3 offset:%4"
                   : "+v"(pa) : "s"(lds_base), "v"(voff), "s"(gbase), "n"(IMM) : "m0");
  }
  pin_a[0] = pa;
  if constexpr (TWO) pin_b[0] = pb;
}
template <int N>
__device__ __forceinline__ void wait_vmem() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// ===========================================================================
// Statistics pass.  Workgroup = 512 threads = 8 waves as 2 (targets, M) x 4 (anchors, N);
// workgroup tile 256 targets x 256 anchors, wave tile 128 x 64 (4 x 2 MFMA tiles).
// k is staged through LDS in chunks of 64, two stages.
// ===========================================================================
constexpr int ST_TM = 256, ST_TN = 256, ST_KC = 64;
constexpr int ST_ROWB = ST_KC * 2;                       // bytes per LDS row (8 chunks of 16 bytes, unpadded)
constexpr int ST_STAGE_BYTES = (ST_TM + ST_TN) * ST_ROWB;  // one stage: 256 target rows, then 256 anchor rows
// LDS layout: chunk c of row r is stored at chunk position c ^ ((r >> 1) & 7): the 16 rows that a
// 16-lane group reads in one fragment load then fall into 16 different 16-byte bank groups.

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
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_b[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;
  const int task = xcd_task_id();
  const int ablk = task % n_ablk, split = task / n_ablk;
  const int a0 = ablk * ST_TN;
  const int cbeg = split * cols_per_split, cend = min(P, cbeg + cols_per_split);
  const int nk = d / ST_KC;

  // ---- direct global->LDS loads: wave w fills rows 64 w .. 64 w + 63 of a stage (waves 0-3 the target
  // rows, waves 4-7 the anchor rows), 8 instructions of 8 rows x 8 chunks each -------------------------
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);  // as a scalar: what follows from it stays uniform
  const bool loads_q = wave_u >= 4;
  const unsigned short* lmat = loads_q ? Q : Pm;
  const int lrows = loads_q ? B : P;
  const int lrow_in = (wave_u & 3) * 64 + (lane >> 3);  // + 8 j: row inside the 256-row tile
  const unsigned stage_m0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)smem_b + wave_u * 64 * ST_ROWB);
  auto src_of = [&](int j, int tile_row0, bool clamp) -> unsigned {  // byte offset from the tile's first row, chunk kc = 0
    int r = lrow_in + 8 * j;
    const int c = (lane & 7) ^ ((r >> 1) & 7);
    if (clamp) r = min(r, lrows - 1 - tile_row0);
    return (unsigned)(r * d * 2 + c * 16);
  };
  unsigned voff_full[8];  // full tile, with the instruction offset 1024 (j % 4) pre-subtracted
#pragma unroll
  for (int j = 0; j < 8; j++) voff_full[j] = src_of(j, 0, false) - 1024u * (j & 3);
  auto prefetch = [&](int tile_row0, int kc, int stage) __attribute__((always_inline)) {
    const unsigned short* base_v = lmat + (size_t)tile_row0 * d + kc * ST_KC;  // the same in every lane of a wave
    const unsigned long long bu = (unsigned long long)(uintptr_t)base_v;
    const unsigned short* base = (const unsigned short*)(uintptr_t)(
        // readfirstlane returns int: go through unsigned, or the low half sign-extends into the high one
        ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)(bu >> 32)) << 32) |
        (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((unsigned)bu));
    const unsigned m0 = stage_m0 + stage * ST_STAGE_BYTES;
    if (tile_row0 + 256 <= lrows) {
      dma_group<4>(base, &voff_full[0], m0);
      dma_group<4>(base, &voff_full[4], m0 + 4096);
    } else {  // ragged tile: rows past the end re-read the last valid row (masked later)
#pragma unroll
      for (int j = 0; j < 8; j++) {
        const unsigned off = src_of(j, tile_row0, true);
        dma_group<1>(base, &off, m0 + j * 1024);
      }
    }
  };

  // ---- fragment addresses: row (lane & 31) of an MFMA tile, chunk 2 ks + (lane >> 5), swizzled ---------
  const int swz_l = ((lane & 31) >> 1) & 7;
  unsigned koff[4];
#pragma unroll
  for (int ks = 0; ks < 4; ks++) koff[ks] = (unsigned)(((2 * ks + (lane >> 5)) ^ swz_l) * 16);
  const unsigned char* a_base = smem_b + (wm * 128 + (lane & 31)) * ST_ROWB;               // + mt * 32 rows
  const unsigned char* b_base = smem_b + (ST_TM + wn * 64 + (lane & 31)) * ST_ROWB;        // + nt * 32 rows

  // per-lane running statistics for its two anchor columns
  float rm[2], rl[2], rpos[2];
  int ridx[2], a_col[2], r_of[2];
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    rm[nt] = -INFINITY; rl[nt] = 0.f; rpos[nt] = 0.f; ridx[nt] = 0x7fffffff;
    a_col[nt] = a0 + wn * 64 + nt * 32 + (lane & 31);
    r_of[nt] = (a_col[nt] < B) ? pos_idx[a_col[nt]] : -1;
  }

  // The k-chunks of all the tiles of this workgroup form one sequence of steps; step st lives in stage st & 1 and
  // its loads are issued one step ahead inside a tile.  (Loading the first chunk of the next tile under the last
  // MFMAs of this one was measured too: no gain at 2 tiles of 12 chunks, a loss at 16 tiles of 2 chunks.)
  int st = 0;
  for (int b0 = cbeg; b0 < cend; b0 += ST_TM) {
    f32x16 acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; mt++)
#pragma unroll
      for (int nt = 0; nt < 2; nt++)
#pragma unroll
        for (int r = 0; r < 16; r++) acc[mt][nt][r] = 0.f;

    const int row0 = loads_q ? a0 : b0;
    // nothing is in flight and every reader is past the last barrier: both stages are free
    prefetch(row0, 0, st & 1);
    wait_vmem<0>();
    __syncthreads();
    bf16x8 af[2][4], bfg[2][2];
    for (int kc = 0; kc < nk; kc++, st++) {
      if (kc + 1 < nk) prefetch(row0, kc + 1, (st + 1) & 1);
      const int so = (st & 1) * ST_STAGE_BYTES;
      __builtin_amdgcn_iglp_opt(0);  // scheduler hint: interleave the fragment reads with the MFMA stream
      auto load_frags = [&](int ks, int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int mt = 0; mt < 4; mt++) af[buf][mt] = *(const bf16x8*)(a_base + so + mt * 32 * ST_ROWB + koff[ks]);
#pragma unroll
        for (int nt = 0; nt < 2; nt++) bfg[buf][nt] = *(const bf16x8*)(b_base + so + nt * 32 * ST_ROWB + koff[ks]);
      };
      load_frags(0, 0);
#pragma unroll
      for (int ks = 0; ks < ST_KC / 16; ks++) {
        if (ks + 1 < ST_KC / 16) load_frags(ks + 1, (ks + 1) & 1);
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int nt = 0; nt < 2; nt++) acc[mt][nt] = mfma32(af[ks & 1][mt], bfg[ks & 1][nt], acc[mt][nt]);
      }
      wait_vmem<0>();   // this wave's part of the next stage has landed
      __syncthreads();  // ... and everybody's; nobody still reads the stage that is overwritten next
    }

    // ---- tile epilogue: online softmax statistics, all in registers; acc holds the raw dot products, the
    // base-2 logit is t = alpha2 * acc (alpha2 > 0: the order of the raw values is the order of the logits) -------
    const int brow0 = b0 + wm * 128 + 4 * (lane >> 5);  // + mt*32 + 8*(r/4) + r%4
    const bool edge = (b0 + ST_TM > cend);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const int a = a_col[nt];
      // the masks that can touch this tile
      const bool diag = mask_self && (a >= b0 && a < b0 + ST_TM);
      const bool haspos = (unsigned)(r_of[nt] - b0) < (unsigned)ST_TM;
      if (edge || diag || haspos) {  // rare: the general slow walk
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            int j = brow0 + mt * 32 + 8 * (r >> 2) + (r & 3);
            if (j == r_of[nt]) rpos[nt] = acc[mt][nt][r] * alpha2;
            if (j >= cend || (mask_self && j == a)) acc[mt][nt][r] = -INFINITY;
          }
      }
      // tile max + first index attaining it (rows are visited in increasing j within mt; across
      // register order j is increasing too, so a strict > keeps the smallest index)
      float tmr = -INFINITY; int tc = 0;
#pragma unroll
      for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const float t = acc[mt][nt][r];
          const bool le = t <= tmr;
          tmr = le ? tmr : t;
          tc = le ? tc : (mt * 32 + 8 * (r >> 2) + (r & 3));
        }
      if (tmr > -INFINITY) {
        const float tm = tmr * alpha2;
        const float mn = fmaxf(rm[nt], tm);
        float s = 0.f;
#pragma unroll
        for (int mt = 0; mt < 4; mt++)
#pragma unroll
          for (int r = 0; r < 16; r++) s += fast_exp2(__builtin_fmaf(acc[mt][nt][r], alpha2, -mn));
        rl[nt] = rl[nt] * fast_exp2(rm[nt] - mn) + s;
        if (tm > rm[nt]) ridx[nt] = brow0 + tc;  // later tiles have larger j: strict >
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
  float* xs = (float*)smem_b;  // [4 wn][2 nt][32][3]
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
    if (a < B && r >= cbeg && r < cend) {
      // lane that held row r: rows of this lane are brow(mt, reg) with 4*(lane>>5) offset
      int rel = (r - cbeg) % ST_TM;  // row inside its tile
      int wmr = rel / 128, in = rel % 128;
      int half = (in % 8) / 4;
      // a positive that the self-mask removes has the logit -inf (its row loss is then +inf)
      if (wmr == wm && half == (lane >> 5)) pos_t[a] = (mask_self && r == a) ? -INFINITY : rpos[nt];
    }
  }
}

static hipError_t launch_stats128(const LossArgs& a, const LossPlan& pl);
hipError_t launch_stats_mfma(const LossArgs& a, const LossPlan& pl) {
  if (a.d == 128) return launch_stats128(a, pl);   // whole anchor rows in registers: a kernel of its own
  char* ws = a.ws;
  const int n_ablk = (a.B + ST_TN - 1) / ST_TN;
  const size_t smem = (size_t)2 * ST_STAGE_BYTES;
  static bool attr_done[64];
  if (hipError_t e = ensure_dyn_lds((const void*)stats_mfma_kernel, (int)smem, attr_done); e != hipSuccess) return e;
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
//            every streamed tile (a wave-private LDS ring of five stages, filled by direct
//            global->LDS loads issued four tiles ahead: the loads of iteration u go to the stage
//            that iteration u-1 has finished with, so they can sit anywhere in the iteration).
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
constexpr int GR_OWN = 64, GR_T = 16, GR_STAGES = 5;

template <int D>
struct GradCfg {
  static constexpr int DS = D / 4;        // columns per wave
  static constexpr int KS = DS / 32;      // MFMA k-steps of phase 1 (k = 32 each)
  static constexpr int CT = DS / 32;      // 32-column output tiles of phase 2
  static constexpr int C16 = DS / 8;      // 16-byte chunks per slice row
  // LDS layout of a streamed slice: 16 rows of C16 chunks.  When C16 = 8 (mod 16) the rows are
  // stored unpadded with the low three bits of the chunk index XORed by swz3(row): the 16 rows
  // of a phase-1 fragment read and the 4 rows x 4 chunks of a transposing phase-2 read then fall
  // into 16 different 16-byte bank groups.  Other widths keep one pad chunk per row instead.
  static constexpr bool SWZ = (C16 % 16) == 8;
  static constexpr int SLOTS = SWZ ? C16 : C16 + 1;
  static constexpr int LDB = SLOTS * 16;                // LDS row stride in bytes
  static constexpr int TILE_SLOTS = GR_T * SLOTS;       // 16-byte slots holding tile data
  static constexpr int NI_Q = (TILE_SLOTS + 63) / 64;   // direct-to-LDS load instructions (1 KB each) per tile slice
  // a stage starts with the row statistics of the streamed rows (dP role): 64 bytes of lse2, then
  // 64 bytes of pos_idx; the tile data follows
  static constexpr int TOFF = 128;
  static constexpr int STAGE = TOFF + NI_Q * 1024;      // bytes: one wave, one stage
  static constexpr int RS_BYTES = 4 * GR_STAGES * STAGE;
  static constexpr int X_BYTES = 2 * 4 * 4 * 64 * 16;   // [parity][src][dst][lane] float4
  static constexpr int G_BYTES = 2 * 2 * 64 * 16;       // [parity][m-tile][lane] bf16x8
  // online-statistics walk: [parity][64 rescale factors (float) | 4 flag words, one per finishing wave]
  static constexpr int F_PAR = 64 * 4 + 16;
  static constexpr int F_BYTES = 1024;
  static constexpr int SMEM = RS_BYTES + X_BYTES + G_BYTES + F_BYTES;
  static_assert(SMEM <= 160 * 1024, "LDS budget");
};

// (Measured with the bank-conflict counter on the two read patterns, all 4096 linear maps of the row bits: this one
// and 767 others are free of conflicts for both; the first choice, bits 2 and 3 of the row into bits 0 and 1, left
// the 16-byte fragment reads of phase 1 with a two-way conflict, 21 % of the walks' LDS cycles.)
__device__ __forceinline__ int swz3(int row) { return (((row >> 1) & 1) << 2) | (((row >> 2) & 1) << 1); }

struct GradArgs {
  const unsigned short* Q;
  const unsigned short* P;
  const int32_t* pos_pad;   // pos_idx copied and padded with -1 to a multiple of 64 rows
  const float* lse2;        // log2-domain log-sum-exp per anchor, padded with +inf
  const float* lse2_t;      // symmetric loss only: the same per target (over the anchors), padded alike
  int B, Pn;
  float alpha2, out_scale;
  int mask_self;
  int obQ, nsq, q_stream_len;  // dQ-role workgroups: obQ owner blocks x nsq stream splits
  int obP, nsp, p_stream_len;
  float* dq_out; size_t dq_split_stride;  // split s writes dq_out + s * stride
  float* dp_out; size_t dp_split_stride;
  // online-statistics walk (dQ role, no statistics pass before it): per split and anchor the reference the
  // accumulators are relative to and sum 2^(t - reference); per anchor the positive's logit
  float* on_ref; float* on_l; int* on_idx; float* on_pos;
  float* on_best;  // per split and anchor: the true maximum, written (with on_idx) only when on_argmax is set
  int on_argmax;   // track the true maximum and its first index
  // an anchor per target, as the statistics merge left it, and the word that check_shared_positives raises
  const int32_t* inv; int* shared;
};

// The kernel that sums the partials adds each positive's own term to its dP row through inv[j] (an anchor with
// r_i = j).  That is enough when no two anchors share a target; here every workgroup looks at a slice of the anchors
// and raises *shared when one of them is not the anchor recorded for its target (the sum kernel then scans).
__device__ __forceinline__ void check_shared_positives(const GradArgs& ga) {
  if (!ga.inv) return;
  const int per = (ga.B + (int)gridDim.x - 1) / (int)gridDim.x;
  const int i0 = (int)blockIdx.x * per, i1 = min(ga.B, i0 + per);
  for (int i = i0 + (int)threadIdx.x; i < i1; i += (int)blockDim.x) {
    const int r = ga.pos_pad[i];
    if (r >= 0 && r < ga.Pn && ga.inv[r] != i) *ga.shared = 1;
  }
}

// max / sum over the four lanes that share lane % 16 (v_permlane16_swap / v_permlane32_swap give every lane both
// partners' values, so all four lanes end with the same bits)
__device__ __forceinline__ void swap16(unsigned x, unsigned& a, unsigned& b) {
  auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false); a = r[0]; b = r[1];
}
__device__ __forceinline__ void swap32(unsigned x, unsigned& a, unsigned& b) {
  auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false); a = r[0]; b = r[1];
}
__device__ __forceinline__ float max_g16(float x) {
  unsigned a, b;
  swap16(__builtin_bit_cast(unsigned, x), a, b);
  x = fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
  swap32(__builtin_bit_cast(unsigned, x), a, b);
  return fmaxf(__builtin_bit_cast(float, a), __builtin_bit_cast(float, b));
}
__device__ __forceinline__ float sum_g16(float x) {
  unsigned a, b;
  swap16(__builtin_bit_cast(unsigned, x), a, b);
  x = __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
  swap32(__builtin_bit_cast(unsigned, x), a, b);
  return __builtin_bit_cast(float, a) + __builtin_bit_cast(float, b);
}
// (value, index): larger value wins, ties go to the smaller index
__device__ __forceinline__ void argmax_g16(float& v, int& i) {
  unsigned a, b, ia, ib;
  auto pick = [&]() {
    const float va = __builtin_bit_cast(float, a), vb = __builtin_bit_cast(float, b);
    const bool tb = (vb > va) || (vb == va && (int)ib < (int)ia);
    v = tb ? vb : va; i = tb ? (int)ib : (int)ia;
  };
  swap16(__builtin_bit_cast(unsigned, v), a, b); swap16((unsigned)i, ia, ib); pick();
  swap32(__builtin_bit_cast(unsigned, v), a, b); swap32((unsigned)i, ia, ib); pick();
}

__device__ __forceinline__ f32x4 mfma16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

template <int N, int I = 0, class F>
__device__ __forceinline__ void static_for(F&& f) {  // f(integral_constant<int, I>) for I = 0 .. N-1
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<N, I + 1>(f);
  }
}

template <int D>
constexpr bool grad_offsets_fit() {  // voff[k] - 1024 (k % 4) must stay >= 0 for a full tile
  using C = GradCfg<D>;
  for (int it = 0; it < C::NI_Q; it++)
    if ((64 * it / C::SLOTS) * 2 * D < (it & 3) * 1024) return false;
  return true;
}

// SYM: the symmetric loss 1/2 [L(F, G, r) + L(G, F, r^-1)].  Its coefficient matrix is
//   g_ij = 1/2 (2^(t_ij - lse2[i]) + 2^(t_ij - lse2_t[j])) - [j = r_i]
// (row softmax and column softmax of the same scores), and dQ = g P, dP = g^T Q as before: one walk per side,
// in which the streamed rows always bring their statistic along.
// ONLINE (dQ role only): no statistics pass has run.  The walk keeps, per owner row, a reference m (the row
// maximum of the first tile; raised, with the accumulators and the running sum rescaled by 2^(old - new), only when
// a later score exceeds it by more than kOnlineMargin), accumulates sum_j 2^(t_ij - m) p_j and sum_j 2^(t_ij - m),
// and tracks the true maximum, its first index and the positive's logit.  A later kernel turns these into lse2 and
// dQ (softmax_ij = 2^(t_ij - m) 2^(m - lse2_i); the positive's -p_{r_i} is subtracted there).
constexpr float kOnlineMargin = 16.f;
template <int D, bool OWNER_IS_Q, bool SYM, bool ONLINE = false>
__device__ __forceinline__ void grad_body(const GradArgs& ga, int oblk, int split, unsigned char* smem) {
  using C = GradCfg<D>;
  static_assert(!ONLINE || (OWNER_IS_Q && !SYM), "the online walk is the dQ role of the one-direction loss");
  constexpr bool STR_STATS = SYM || !OWNER_IS_Q;   // the streamed rows' statistics ride in the LDS stage
  const float* lse_own = (SYM && !OWNER_IS_Q) ? ga.lse2_t : ga.lse2;
  const float* lse_str = (SYM && OWNER_IS_Q) ? ga.lse2_t : ga.lse2;
  static_assert(grad_offsets_fit<D>(), "direct-to-LDS load offsets");
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, ln = lane & 31;
  const int l16 = lane & 15, g16 = lane >> 4;
  const unsigned short* O = OWNER_IS_Q ? ga.Q : ga.P;
  const unsigned short* R = OWNER_IS_Q ? ga.P : ga.Q;
  const int No = OWNER_IS_Q ? ga.B : ga.Pn, Nr = OWNER_IS_Q ? ga.Pn : ga.B;
  const int slen = OWNER_IS_Q ? ga.q_stream_len : ga.p_stream_len;
  const int a0 = oblk * GR_OWN;
  const int sbeg = split * slen, send = min(Nr, sbeg + slen);
  const int nt = (send - sbeg + GR_T - 1) / GR_T;  // streamed tiles of this workgroup (>= 1)

  // ---- LDS map (bytes): [wave rings: 4 waves x 5 stages x STAGE][X: 2 x 4 x 4 x 1024][G: 2 x 2 x 1024]
  constexpr int NT = C::NI_Q;                                 // load instructions that carry tile data
  constexpr unsigned RING = GR_STAGES * C::STAGE;
  const unsigned ring_off = w * RING;                         // this wave's ring of stages
  const unsigned ring_m0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)smem + ring_off);
  // per-lane byte offsets; every access adds the stage offset and a compile-time constant (k-step ...)
  auto lane_base = [&](int row, int j, int parity) __attribute__((always_inline)) -> unsigned {
    // chunk 4 i + j of a row is stored at 4 (i ^ s2) + (j ^ s01), (s2, s01) from swz3(row): one
    // base for even i and one for odd i, the loops add the compile-time part 64 i
    const int sw = C::SWZ ? swz3(row) : 0;
    const int s2 = sw >> 2, s01 = sw & 3;
    return ring_off + C::TOFF + (unsigned)(row * C::LDB + 16 * (j ^ s01) + (parity ? -64 * s2 : 64 * s2));
  };
  // phase 1 reads row l16, chunk 4 ks + g16
  const unsigned char* p1p[2] = {smem + lane_base(l16, g16, 0), smem + lane_base(l16, g16, 1)};
  // phase 2 (transposing read): rows 8 h + l16 / 4 (+4), chunk 4 ct + 2 (g16 & 1) + (lane & 3) / 2, 8 bytes
  const int tr_row = 8 * h + (l16 >> 2), tr_j = 2 * (g16 & 1) + ((lane & 3) >> 1), tr_in = 8 * (lane & 1);
  const unsigned char* p2lo[2] = {smem + lane_base(tr_row, tr_j, 0) + tr_in, smem + lane_base(tr_row, tr_j, 1) + tr_in};
  const unsigned char* p2hi[2] = {smem + lane_base(tr_row + 4, tr_j, 0) + tr_in, smem + lane_base(tr_row + 4, tr_j, 1) + tr_in};
  unsigned char* xwp = smem + C::RS_BYTES + (w * 4) * 1024 + lane * 16;          // + par * 16384 + dst * 1024
  const unsigned char* xrp = smem + C::RS_BYTES + w * 1024 + lane * 16;          // + par * 16384 + src * 4096
  // lane (w, l16, g16) finishes rows 4 g16 + 0..3 of owner row 16 w + l16: half (g16 & 1) of the A fragment
  // elements of lane 16 (w & 1) + l16 + 32 (g16 >> 1) in m-tile w >> 1
  unsigned char* gwp = smem + C::RS_BYTES + C::X_BYTES + ((w >> 1) * 64 + 16 * (w & 1) + l16 + 32 * (g16 >> 1)) * 16 + 8 * (g16 & 1);
  const unsigned char* grp = smem + C::RS_BYTES + C::X_BYTES + lane * 16;        // + par * 2048 + mt * 1024
  const unsigned char* rip = smem + ring_off + 16 * g16;                         // + stage offset (+ 64: pos_idx)

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
  if ((OWNER_IS_Q || SYM) && !ONLINE) lse_a = lse_own[a_q];   // padded: +inf past the end, so g = 0 there
  if (OWNER_IS_Q && !ONLINE) r_a = ga.pos_pad[a_q];
  if (ONLINE) r_a = (a_q < No) ? ga.pos_pad[a_q] : -1;   // here pos_pad is the caller's pos_idx itself (B entries)

  // ---- direct-to-LDS loads of a streamed tile: slot q = it * 64 + lane -> (row, chunk) -------------------------
  auto slot_src = [&](int q, int max_row) __attribute__((always_inline)) -> unsigned {
    const int row = min(min(q / C::SLOTS, GR_T - 1), max_row);
    int c = min(q % C::SLOTS, C::C16 - 1);
    if (C::SWZ) c ^= swz3(row);
    return (unsigned)((row * D + w * C::DS + c * 8) * 2);
  };
  unsigned src_off[NT];  // full tile, with the instruction offset 1024 (it % 4) pre-subtracted
#pragma unroll
  for (int it = 0; it < NT; it++) src_off[it] = slot_src(it * 64 + lane, GR_T - 1) - 1024u * (it & 3);
  // row statistics of the streamed rows: lanes 0-3 load lse_str[t0 + 4 l ..], lanes 4-7 pos_pad (dP role; in
  // the dQ role of the symmetric loss they load the same as lanes 0-3 and nobody reads it)
  const unsigned ri_off = ((lane & 4) && !OWNER_IS_Q) ? (unsigned)((const char*)ga.pos_pad - (const char*)ga.lse2) + 16u * (lane & 3) : 16u * (lane & 3);
  constexpr int NI = STR_STATS ? NT + 1 : NT;  // load instructions per tile
  // piece k (0 .. NI-1) of the loads of a full tile that starts at row t0, into the stage at byte offset so
  auto prefetch_piece = [&](auto k_tag, auto two_tag, int t0, unsigned so, u32x4& pin_a, u32x4& pin_b) __attribute__((always_inline)) {
    constexpr int K = decltype(k_tag)::value;
    constexpr bool TWO = decltype(two_tag)::value;
    if constexpr (STR_STATS && K == 0) {
      dma_piece_pinned<0, true, TWO>(lse_str + t0, ri_off, ring_m0 + so, pin_a, pin_b);
    } else {
      constexpr int IT = STR_STATS ? K - 1 : K;
      dma_piece_pinned<1024 * (IT & 3), false, TWO>(R + (size_t)t0 * D, src_off[IT], ring_m0 + so + C::TOFF + 4096 * (IT >> 2), pin_a, pin_b);
    }
  };
  auto prefetch = [&](int u, unsigned so) __attribute__((always_inline)) {  // whole tile u -> stage at offset so
    const int t0 = sbeg + u * GR_T;
    const unsigned short* tile = R + (size_t)t0 * D;  // wave-uniform
    const unsigned lds0 = ring_m0 + so + C::TOFF;
    if (STR_STATS) {
      if (lane < 8) dma_piece<0>(lse_str + t0, ri_off, ring_m0 + so);
    }
    if (t0 + GR_T <= Nr) {
#pragma unroll
      for (int g = 0; g < NT; g += 4) {
        if (NT - g >= 4) dma_group<4>(tile, &src_off[g], lds0 + g * 1024);
        else if (NT - g == 3) dma_group<3>(tile, &src_off[g], lds0 + g * 1024);
        else if (NT - g == 2) dma_group<2>(tile, &src_off[g], lds0 + g * 1024);
        else dma_group<1>(tile, &src_off[g], lds0 + g * 1024);
      }
    } else {  // ragged last tile: rows past the end re-read the last valid row (their g is forced to 0)
#pragma unroll
      for (int it = 0; it < NT; it++) {
        const unsigned off = slot_src(it * 64 + lane, Nr - 1 - t0);
        dma_group<1>(tile, &off, lds0 + it * 1024);
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
  u32x4 afr[C::KS];  // phase-1 A fragments of the tile being started (bf16x8 each)
  auto p1_load = [&](unsigned so, int ks0, int ks1) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = ks0; ks < ks1; ks++) afr[ks] = *(const u32x4*)(p1p[ks & 1] + so + 64 * ks);
  };
  auto p1_mfma = [&](int ks0, int ks1) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = ks0; ks < ks1; ks++)
#pragma unroll
      for (int nq = 0; nq < 4; nq++)
        sacc[nq] = mfma16(__builtin_bit_cast(bf16x8, afr[ks]), ofrag[nq][ks], ks == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : sacc[nq]);
  };
  // The load unit of a compute unit takes one 1 KB load every 16 cycles, and a wave waits at the load
  // until the unit accepts it.  The four waves run in step (one barrier per tile), so a steady iteration
  // spreads its 4 NI loads evenly over the MFMA time of the iteration and the waves take turns: the code
  // of the steady loop is specialised per wave (WAVE = 0 .. 3), piece k of wave WAVE follows the MFMA
  // that runs at 1 / (4 NI) * (4 k + WAVE) of that time.  Sections: 0 = phase 1 before the barrier,
  // 1 = phase 1 after it, 2 = phase 2.
  constexpr int KS_PRE = (C::KS + 1) / 2;            // k-steps of phase 1 issued before the barrier
  static_assert(C::KS == C::CT, "the steady loop pairs the k-steps of phase 1 with the column tiles of phase 2");
  constexpr int MA = 4 * KS_PRE, MB = 4 * (C::KS - KS_PRE), MC = 2 * C::CT;  // MFMAs per section
  constexpr int T16 = 19, T32 = 33;                  // measured issue-to-issue cycles of the two MFMA shapes
  auto slot_of = [](int wave, int k, int sec) constexpr -> int {  // MFMA index in section sec, or -1
    constexpr int TOTAL = T16 * (MA + MB) + T32 * MC;
    int t = ((4 * k + wave) * TOTAL) / (4 * NI);
    if (t < T16 * MA) return sec == 0 ? t / T16 : -1;
    t -= T16 * MA;
    if (t < T16 * MB) return sec == 1 ? t / T16 : -1;
    t -= T16 * MB;
    return sec == 2 ? (t / T32 < MC ? t / T32 : MC - 1) : -1;
  };
  // loads of tile u+4 that a steady iteration of wave `wave` has issued once the round of phase-2 MFMA `idx` is over
  auto issued_by = [slot_of](int wave, int idx) constexpr -> int {
    int n = 0;
    for (int k = 0; k < NI; k++) {
      const int s2 = slot_of(wave, k, 2);
      if (slot_of(wave, k, 0) >= 0 || slot_of(wave, k, 1) >= 0 || (s2 >= 0 && s2 <= idx)) n++;
    }
    return n;
  };
  // called after MFMA number IDX of section SEC; pin_a: a register that MFMA read, pin_b: one that the
  // next MFMA reads (TWO: they differ)
  auto spread = [&](auto wave_tag, auto sec_tag, auto idx_tag, auto two_tag, int t_pf, unsigned so_pf, u32x4& pin_a, u32x4& pin_b) __attribute__((always_inline)) {
    constexpr int WAVE = decltype(wave_tag)::value, SEC = decltype(sec_tag)::value, IDX = decltype(idx_tag)::value;
    if constexpr (WAVE >= 0) {
      static_for<NI>([&](auto k_tag) __attribute__((always_inline)) {
        if constexpr (slot_of(WAVE, decltype(k_tag)::value, SEC) == IDX) prefetch_piece(k_tag, two_tag, t_pf, so_pf, pin_a, pin_b);
      });
    }
  };
  // phase 2 of the tile in the stage at `so` (WAVE >= 0: a steady iteration, which also issues its share
  // of the loads of the tile that starts at row t_pf into the stage at so_pf)
  u32x4 bfr[C::CT];  // phase-2 B fragments (bf16x8 each)
  auto p2_load = [&](unsigned so, int c0, int c1) __attribute__((always_inline)) {
#pragma unroll
    for (int ct = c0; ct < c1; ct++) {
      s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p2lo[ct & 1] + so + 64 * ct));
      s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p2hi[ct & 1] + so + 64 * ct));
      s16x8 bb = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      bfr[ct] = __builtin_bit_cast(u32x4, bb);
    }
  };
  // The LDS pipe is shared by the four waves, which run in step: fragment reads bunched at the start of a phase
  // leave the MFMAs waiting for LDS and LDS idle during the MFMAs.  A steady iteration therefore reads every fragment
  // half an iteration ahead, into the registers of a fragment that has just been used up: the transposed fragment ct
  // of phase 2 (tile u, stage so_p2) right behind the four MFMAs of k-step ct of phase 1, and the fragment of k-step ks
  // of the NEXT iteration's phase 1 (tile u+3, stage so_p1n) right behind the two MFMAs of column tile ks of phase 2.
  auto p1_mfma_spread = [&](auto wave_tag, auto sec_tag, int t_pf, unsigned so_pf, unsigned so_p2) __attribute__((always_inline)) {
    constexpr int SEC = decltype(sec_tag)::value, WAVE = decltype(wave_tag)::value;
    constexpr int KS0 = SEC == 0 ? 0 : KS_PRE, KS1 = SEC == 0 ? KS_PRE : C::KS;
    static_for<4 * (KS1 - KS0)>([&](auto i_tag) __attribute__((always_inline)) {
      constexpr int i = decltype(i_tag)::value, ks = KS0 + i / 4, nq = i % 4;
      sacc[nq] = mfma16(__builtin_bit_cast(bf16x8, afr[ks]), ofrag[nq][ks], ks == 0 ? f32x4{0.f, 0.f, 0.f, 0.f} : sacc[nq]);
      constexpr int ksn = KS0 + (i + 1) / 4;  // k-step of the next MFMA of the section
      if constexpr (ksn != ks && ksn < KS1) spread(wave_tag, sec_tag, i_tag, std::true_type{}, t_pf, so_pf, afr[ks], afr[ksn]);
      else spread(wave_tag, sec_tag, i_tag, std::false_type{}, t_pf, so_pf, afr[ks], afr[ks]);
      if constexpr (WAVE >= 0 && nq == 3) p2_load(so_p2, ks, ks + 1);
    });
  };
  // after_round(i): arithmetic of the caller that is to run in the shadow of MFMA i
  auto phase2 = [&](const bf16x8 (&gf)[2], auto wave_tag, int t_pf, unsigned so_pf, unsigned so_p1n, auto&& after_round) __attribute__((always_inline)) {
    constexpr int WAVE = decltype(wave_tag)::value;
    static_for<MC>([&](auto i_tag) __attribute__((always_inline)) {
      constexpr int i = decltype(i_tag)::value, ct = i / 2, mt = i % 2;
      acc[mt][ct] = mfma32(gf[mt], __builtin_bit_cast(bf16x8, bfr[ct]), acc[mt][ct]);
      constexpr std::integral_constant<int, 2> sec{};
      if constexpr (mt == 1 && ct + 1 < C::CT) spread(wave_tag, sec, i_tag, std::true_type{}, t_pf, so_pf, bfr[ct], bfr[ct + 1]);
      else spread(wave_tag, sec, i_tag, std::false_type{}, t_pf, so_pf, bfr[ct], bfr[ct]);
      if constexpr (WAVE >= 0 && mt == 1) {
        // tile u+3 has landed once at most the loads this iteration has issued so far (for tile u+4) are in flight
        if constexpr (ct == 0) wait_vmem<issued_by(WAVE, i)>();
        p1_load(so_p1n, ct, ct + 1);
      }
      after_round(i_tag);
    });
  };

  bf16x4 gq = {0, 0, 0, 0};  // g of the tile whose scores were finished last (4 streamed rows of owner row a_q)
  // online walk: state of owner row a_q (m_run is the same in the four lanes that share the row, the rest is per lane)
  float m_run = -INFINITY, l_run = 0.f, best_v = -INFINITY, f_pub = 1.f;
  int best_i = 0x7fffffff, need_pub = 0;
  unsigned char* fwp = smem + C::RS_BYTES + C::X_BYTES + C::G_BYTES;            // + par * F_PAR

  // One pipeline iteration (see the header comment); so0 = ring offset of the stage of tile u.  STEADY:
  // every pipeline slot is live, the tiles involved are full and not the last ones.
  // STG >= 0: the ring stage of tile u is known at compile time (the steady loop is unrolled over the five stages), so
  // every LDS address of the iteration is a per-lane base plus an immediate and no address arithmetic is issued: a
  // single wave per SIMD issues everything itself, and what it issues besides the MFMAs is what the loop's time is made of.
  auto body = [&](int u, unsigned so0_dyn, auto stage_tag, auto wave_tag) __attribute__((always_inline)) {
    constexpr int WAVE = decltype(wave_tag)::value, STG = decltype(stage_tag)::value;
    constexpr bool STEADY = WAVE >= 0;
    const unsigned so0 = STG >= 0 ? (unsigned)(STG * C::STAGE) : so0_dyn;
    const int t_pf = sbeg + (u + 4) * GR_T;  // first row of tile u+4
    const unsigned so1 = (so0 + C::STAGE >= RING) ? so0 + C::STAGE - RING : so0 + C::STAGE;   // tile u+1
    const unsigned so2 = (so1 + C::STAGE >= RING) ? so1 + C::STAGE - RING : so1 + C::STAGE;   // tile u+2
    const unsigned so4 = (so0 == 0) ? RING - C::STAGE : so0 - C::STAGE;                        // tile u+4 (= u-1)
    const int PAR0 = u & 1, PAR1 = PAR0 ^ 1;           // X / G parity of tiles u and u+1
    const bool xw = STEADY || (u + 1 < nt);            // tile u+1: publish partials, finish scores
    const bool gw = STEADY || (u >= 0);                // tile u: publish fragments, phase 2   (u < nt always)
    const bool p1 = STEADY || (u + 2 < nt);            // tile u+2: phase 1
    const bool pf = STEADY || (u >= 0 && u + 4 < nt);  // tile u+4: start its loads
    __builtin_amdgcn_iglp_opt(0);  // scheduler hint: interleave the LDS reads with the MFMA stream
    if (p1 && !STEADY) {
      // tile u+2 has landed; its fragment reads are issued ahead of the writes below, so they come back first.  (A
      // steady iteration finds them in registers: the iteration before it has read them during its phase 2.)
      wait_vmem<0>();
      p1_load(so2, 0, C::KS);
    }
    // the partial tile of the owner rows this wave finishes itself stays in registers (steady loop: the wave
    // index is a compile-time constant there); the other three go through LDS
    f32x4 own = {0.f, 0.f, 0.f, 0.f};
    if constexpr (STEADY) own = sacc[WAVE];
    if (xw) {
#pragma unroll
      for (int dst = 0; dst < 4; dst++)
        if (!(STEADY && dst == WAVE)) *(f32x4*)(xwp + PAR1 * 16384 + dst * 1024) = sacc[dst];
    }
    if (gw) *(bf16x4*)(gwp + PAR0 * 2048) = gq;
    if (ONLINE && gw) {  // the rescale factors of tile u's rows and this wave's "some row was rescaled" word
      if (g16 == 0) *(float*)(fwp + PAR0 * C::F_PAR + (16 * w + l16) * 4) = f_pub;
      if (lane == 0) *(int*)(fwp + PAR0 * C::F_PAR + 256 + 4 * w) = need_pub;
    }
    if (p1) p1_mfma_spread(wave_tag, std::integral_constant<int, 0>{}, t_pf, so4, so0);  // while the writes drain and the barrier gathers the waves
    __syncthreads();
    f32x4 xr[4];
    if (xw) {
#pragma unroll
      for (int src = 0; src < 4; src++) {
        if (STEADY && src == WAVE) xr[src] = own;
        else xr[src] = *(const f32x4*)(xrp + PAR1 * 16384 + src * 4096);
      }
    }
    bf16x8 gf[2];
    if (gw) {
#pragma unroll
      for (int mt = 0; mt < 2; mt++) gf[mt] = *(const bf16x8*)(grp + PAR0 * 2048 + mt * 1024);
    }
    f32x4 lse_r = {0.f, 0.f, 0.f, 0.f}; i32x4 pos_r = {0, 0, 0, 0};
    if (STR_STATS && xw) {  // row statistics of tile u+1 ride in its LDS stage
      lse_r = *(const f32x4*)(rip + so1);
      if (!OWNER_IS_Q) pos_r = *(const i32x4*)(rip + so1 + 64);
    }
    i32x4 fl = {0, 0, 0, 0};
    if (ONLINE && gw) fl = *(const i32x4*)(fwp + PAR0 * C::F_PAR + 256);
    if (p1) p1_mfma_spread(wave_tag, std::integral_constant<int, 1>{}, t_pf, so4, so0);
    if constexpr (ONLINE) __builtin_amdgcn_sched_barrier(0);  // the flag test (and its wait for LDS) stays behind these MFMAs
    if (!STEADY && gw) p2_load(so0, 0, C::CT);   // (a steady iteration has read them behind the MFMAs of phase 1)
    if (ONLINE && gw) {
      // rare after the first tile: some row's reference went up, every wave rescales its columns of those rows
      if (__builtin_amdgcn_ballot_w64((fl[0] | fl[1] | fl[2] | fl[3]) != 0) != 0) {
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
#pragma unroll
          for (int j = 0; j < 4; j++) {
            const f32x4 f4 = *(const f32x4*)(fwp + PAR0 * C::F_PAR + (32 * mt + 8 * j + 4 * h) * 4);
#pragma unroll
            for (int ct = 0; ct < C::CT; ct++)
#pragma unroll
              for (int i = 0; i < 4; i++) {
                // in place on the accumulation register (written in the compiler's own way this cold path moved
                // every accumulator into ordinary registers and cost the loop 200 spilled ones); the MFMAs that
                // wrote and will read these registers are a barrier and many instructions away
                float x = acc[mt][ct][4 * j + i], tmp;
                asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\tv_accvgpr_write_b32 %0, %1"
                             : "+a"(x), "=&v"(tmp) : "v"(f4[i]));
                acc[mt][ct][4 * j + i] = x;
              }
          }
      }
    }
    // ---- from the summed scores of tile u+1 to its coefficients.  The arithmetic that every tile needs is cut into
    // pieces; in a steady iteration (not for SYM) piece k runs right behind MFMA k * MC / NP of phase 2, where a
    // wave's own arithmetic is free, instead of after the last MFMA, where it is not.  What only few tiles need
    // (the positive, masks, the arg-max) stays behind phase 2.
    constexpr bool INTER = STEADY && !SYM;
    constexpr int NP = ONLINE ? 10 : 5;
    const int b0 = sbeg + (u + 1) * GR_T + 4 * g16;      // first of this lane's 4 streamed rows
    f32x4 sv = {0.f, 0.f, 0.f, 0.f}, tt = {0.f, 0.f, 0.f, 0.f}, gv = {0.f, 0.f, 0.f, 0.f};
    float tmx = 0.f, mref = 0.f;
    bool need = false;
    auto piece = [&](auto k_tag) __attribute__((always_inline)) {
      constexpr int K = decltype(k_tag)::value;
      if constexpr (K == 0) sv = xr[0] + xr[1];            // fixed order ((x0 + x1) + x2) + x3: bit-identical
      else if constexpr (K == 1) sv = sv + xr[2];           // whichever wave sums
      else if constexpr (K == 2) sv = sv + xr[3];
      else if constexpr (!ONLINE) {
        if constexpr (K == 3) {
#pragma unroll
          for (int e = 0; e < 4; e++) tt[e] = sv[e] * ga.alpha2 - (OWNER_IS_Q ? lse_a : lse_r[e]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; e++) gv[e] = fast_exp2(tt[e]);  // softmax
        }
      } else {
        if constexpr (K == 3) {
#pragma unroll
          for (int e = 0; e < 4; e++) tt[e] = sv[e] * ga.alpha2;
          if constexpr (!STEADY) {  // rows past the end of the split, the diagonal under mask_self
            const int t1o = b0 - 4 * g16;
            if ((t1o + GR_T > send) || (ga.mask_self && (t1o < a0 + GR_OWN) && (t1o + GR_T > a0))) {
#pragma unroll
              for (int e = 0; e < 4; e++)
                if (b0 + e >= send || (ga.mask_self && b0 + e == a_q)) tt[e] = -INFINITY;
            }
          }
        } else if constexpr (K == 4) tmx = fmaxf(fmaxf(tt[0], tt[1]), fmaxf(tt[2], tt[3]));
        else if constexpr (K == 5) {
          unsigned x0, x1;
          swap16(__builtin_bit_cast(unsigned, tmx), x0, x1);
          tmx = fmaxf(__builtin_bit_cast(float, x0), __builtin_bit_cast(float, x1));
        } else if constexpr (K == 6) {
          unsigned x0, x1;
          swap32(__builtin_bit_cast(unsigned, tmx), x0, x1);
          tmx = fmaxf(__builtin_bit_cast(float, x0), __builtin_bit_cast(float, x1));   // this tile's maximum of row a_q
        } else if constexpr (K == 7) {
          // raise the reference when the tile exceeds it by more than the margin (always at the first tile with a
          // finite score: m_run = -inf); without branches: the factor is 2^0 when nothing changes, 2^-inf the first time
          need = tmx > m_run + kOnlineMargin;
          f_pub = fast_exp2(need ? m_run - tmx : 0.f);
          l_run *= f_pub;
          m_run = need ? tmx : m_run;
          mref = (m_run == -INFINITY) ? 0.f : m_run;
        } else if constexpr (K == 8) {
#pragma unroll
          for (int e = 0; e < 4; e++) gv[e] = fast_exp2(tt[e] - mref);
        } else {
          l_run += (gv[0] + gv[1]) + (gv[2] + gv[3]);
        }
      }
      if constexpr (INTER) {  // an empty statement that "uses" the results keeps the piece in its round
        if constexpr (ONLINE) asm volatile("" : "+v"(sv), "+v"(tt), "+v"(gv), "+v"(tmx), "+v"(l_run), "+v"(m_run), "+v"(f_pub));
        else asm volatile("" : "+v"(sv), "+v"(tt), "+v"(gv));
      }
    };
    auto after_round = [&](auto i_tag) __attribute__((always_inline)) {
      if constexpr (INTER) {
        constexpr int i = decltype(i_tag)::value;
        static_for<NP>([&](auto k_tag) __attribute__((always_inline)) {
          if constexpr (decltype(k_tag)::value * MC / NP == i) piece(k_tag);
        });
        __builtin_amdgcn_sched_barrier(0);  // the rounds stay in order
      }
    };
    const unsigned so3 = (so2 + C::STAGE >= RING) ? so2 + C::STAGE - RING : so2 + C::STAGE;   // tile u+3
    if (gw) phase2(gf, wave_tag, t_pf, so4, so3, after_round);
    if (xw) {
      if constexpr (!INTER) static_for<NP>(piece);
      if constexpr (ONLINE) {
        need_pub = __builtin_amdgcn_ballot_w64(need) != 0 ? 1 : 0;
        if (ga.on_argmax) {
#pragma unroll
          for (int e = 0; e < 4; e++) {   // increasing j: a strict > keeps the smallest index
            const bool gt = tt[e] > best_v;
            best_v = gt ? tt[e] : best_v;
            best_i = gt ? b0 + e : best_i;
          }
        }
        if ((unsigned)(r_a - b0) < 4u) {
          // the positive: seen by exactly one lane of one split.  Its own term (p_{i r_i} - 1) p_{r_i} is formed in
          // fp32 by the kernel that finishes dQ: left in the bf16 sum it would cancel against - p_{r_i} with the
          // rounding error of a coefficient near 1
          // (rows past the end of this split belong to the next one; a positive that the self-mask removes keeps
          // its -inf, so that row's loss is +inf)
          if (a_q < No && r_a < send) ga.on_pos[a_q] = tt[r_a - b0];
#pragma unroll
          for (int e = 0; e < 4; e++)
            if (r_a - b0 == e) gv[e] = 0.f;
        }
        gq = __builtin_convertvector(gv, bf16x4);
      } else {
        if constexpr (SYM) {  // mean of the row softmax and the column softmax
#pragma unroll
          for (int e = 0; e < 4; e++)
            gv[e] = fast_exp2(__builtin_fmaf(sv[e], ga.alpha2, -(lse_a + 1.f))) + fast_exp2(__builtin_fmaf(sv[e], ga.alpha2, -(lse_r[e] + 1.f)));
        }
        // the rest touches few tiles and is decided per wave: 0 at the positive (j == r_i; its term is added in fp32
        // by the kernel that sums the partials, see PosFix), zeros for rows past the end of the split and on the
        // diagonal (i == j)
        bool hit_any;
        if (OWNER_IS_Q) hit_any = (unsigned)(r_a - b0) < 4u;
        else hit_any = (pos_r[0] == a_q) | (pos_r[1] == a_q) | (pos_r[2] == a_q) | (pos_r[3] == a_q);
        const int t1 = b0 - 4 * g16;
        const bool tail = !STEADY && (t1 + GR_T > send);
        const bool diag = ga.mask_self && (t1 < a0 + GR_OWN) && (t1 + GR_T > a0);
        if (__builtin_amdgcn_ballot_w64(hit_any) != 0 || tail || diag) {
#pragma unroll
          for (int e = 0; e < 4; e++) {
            const bool hit = OWNER_IS_Q ? (r_a - b0 == e) : (pos_r[e] == a_q);
            if (hit || b0 + e >= send || (ga.mask_self && b0 + e == a_q)) gv[e] = 0.f;
          }
        }
        gq = __builtin_convertvector(gv, bf16x4);
      }
    }
    // the iteration after this one may be a steady one, which expects the phase-1 fragments of its tile (u+3) in
    // registers
    if (!STEADY && u + 3 < nt) {
      wait_vmem<0>();
      p1_load(so3, 0, C::KS);
    }
    if (!STEADY && pf) prefetch(u + 4, so4);  // in a steady iteration phase 2 has issued these loads
  };
  // ---- prologue: start the first tiles, phase 1 of tile 0 ------------------------------------------------------
#pragma unroll 1
  for (int u = 0; u < min(nt, 4); u++) prefetch(u, u * C::STAGE);
  wait_vmem<0>();
  p1_load(0, 0, C::KS);
  p1_mfma(0, C::KS);
  auto next_stage = [&](unsigned so) __attribute__((always_inline)) -> unsigned { return (so + C::STAGE >= RING) ? so + C::STAGE - RING : so + C::STAGE; };
  unsigned so = RING - C::STAGE;  // stage of "tile -1"
  constexpr std::integral_constant<int, -1> unsteady{};
  constexpr std::integral_constant<int, -1> any_stage{};
  body(-1, so, any_stage, unsteady);
  so = 0;
  int u = 0;
  auto steady_loop = [&](auto wave_tag) __attribute__((always_inline)) {
    if constexpr (D == 768) {
      // the widest kernel (the headline shape) is unrolled over the ring: five iterations per trip, tile u is in
      // stage u % 5 and u is a multiple of 5 here (so stays 0); measured 4 % on the dP walk.  The other widths keep
      // the rolled loop (five copies of every width would more than double the time this file takes to compile).
#pragma unroll 1
      for (; u + GR_STAGES + 4 < nt; u += GR_STAGES) {
        static_for<GR_STAGES>([&](auto stage_tag) __attribute__((always_inline)) {
          body(u + decltype(stage_tag)::value, 0u, stage_tag, wave_tag);
        });
      }
    } else {
#pragma unroll 1
      for (; u + 5 < nt; u++) { body(u, so, any_stage, wave_tag); so = next_stage(so); }
    }
  };
  // (the steady body of the one-direction kernels has no place for the diagonal mask: with mask_self every
  // iteration takes the general body)
  if (SYM || !ga.mask_self) {
    switch (__builtin_amdgcn_readfirstlane(w)) {
      case 0: steady_loop(std::integral_constant<int, 0>{}); break;
      case 1: steady_loop(std::integral_constant<int, 1>{}); break;
      case 2: steady_loop(std::integral_constant<int, 2>{}); break;
      default: steady_loop(std::integral_constant<int, 3>{}); break;
    }
  }
#pragma unroll 1
  for (; u < nt; u++) { body(u, so, any_stage, unsteady); so = next_stage(so); }

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
  if constexpr (ONLINE) {  // the row's statistics of this split
    const float l_sum = sum_g16(l_run);
    if (ga.on_argmax) argmax_g16(best_v, best_i);
    if (g16 == 0 && a_q < No) {
      // (reference, sum 2^(t - reference)) is all the log-sum-exp needs: the same bits whether or not the
      // arg-max is tracked
      const size_t o = (size_t)split * No + a_q;
      ga.on_ref[o] = m_run;
      ga.on_l[o] = l_sum;
      if (ga.on_argmax) { ga.on_best[o] = best_v; ga.on_idx[o] = best_i; }
    }
  }
}


// ===========================================================================
// Gradient pass for d = 128 (the NT-Xent workload).  At this width a wave can hold whole owner rows, so
// nothing is exchanged between waves: a workgroup (4 waves, one per SIMD) owns 256 rows, each wave 64 of
// them with all 128 columns in registers (64 VGPRs as MFMA B fragments), and all four share the streamed
// tiles (32 rows x 128 columns, 8 KB) through one LDS ring of four stages.  Per tile and wave:
//   phase 1  S^T[32 streamed x 64 owner] = R_tile * O^T, 16 MFMAs 32x32x16.  Lane (n, h) then holds, for owner
//            row n, the scores of streamed rows 8 j + 4 h + i (j, i = 0..3): registers 8 kk .. 8 kk + 7 are
//            streamed rows 16 kk + {4 h .. 4 h + 3, 8 + 4 h .. 8 + 4 h + 3}.
//   g        = 2^(t - lse2) - [j = r_i] in place, rounded to bf16: registers 8 kk .. 8 kk + 7 ARE the B
//            fragment (k = those streamed rows, n = owner) of
//   phase 2  dO^T[128 x 64 owner] += R_tile^T * g^T, 16 MFMAs 32x32x16, whose A fragments (columns of the tile,
//            the same streamed rows in the same k order) come from two transposing LDS reads each.
// The contraction order over the streamed rows is thus a permutation that both operands of phase 2 share.
// LDS per tile: every wave reads the tile twice (8 KB + 8 KB), 72 KB per workgroup against 64 MFMAs per SIMD.
// ===========================================================================
constexpr int G1_OWN = 256, G1_OWN_W = 64, G1_T = 32, G1_STAGES = 8, G1_AHEAD = 6;  // tiles u-1 .. u+1 alive, up to u+5 started
constexpr int G1_STAT = 256;                      // a stage starts with lse2[32], then pos_idx[32] of the streamed rows
constexpr int G1_STAGE = G1_STAT + G1_T * 256;    // bytes
constexpr int G1_SMEM = G1_STAGES * G1_STAGE;
// chunk c (16 bytes) of tile row r is stored at chunk position c ^ swz128(r): 8 consecutive rows of a
// fragment read, and the 4 rows x 2 chunks of a transposing read, fall into different 16-byte bank groups.
// (The bank-conflict counter still shows a conflict on every second LDS cycle of these kernels.  4-bit maps that remove
// them all -- e.g. ((row & 3) << 2) | ((row >> 2) & 3): the low row bits pick the 64-byte quarter, the next two the
// chunk inside it -- were measured on the kernels themselves: LDS cycles halved, waits for LDS a tenth, the time of the
// gradient kernel equal within 1 %.  With a 3-bit map fragment k + 4 of a row sits a fixed 128 bytes behind fragment k,
// an immediate offset; a 4-bit map needs a second set of address registers, which this kernel, at 512 of 512, does not
// have: it spills again.  The loop is paced by its barrier and the waits for the tile loads, not by LDS.)
__device__ __forceinline__ int swz128(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }

// the first `LANES` lanes of the wave load 16 bytes each to lds_base + lane * 16 (EXEC narrowed inside)
__device__ __forceinline__ void dma_lanes16(const void* gbase, unsigned voff, unsigned lds_base) {
  unsigned long long keep;
  asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xffff\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
               : "=&s"(keep) : "s"(lds_base), "v"(voff), "s"(gbase) : "memory", "m0");
}

template <bool OWNER_IS_Q, bool SYM>
__device__ __forceinline__ void grad128_body(const GradArgs& ga, int oblk, int split, unsigned char* smem) {
  constexpr int D = 128;
  constexpr bool STR_STATS = SYM || !OWNER_IS_Q;   // as in grad_body
  const float* lse_own = (SYM && !OWNER_IS_Q) ? ga.lse2_t : ga.lse2;
  const float* lse_str = (SYM && OWNER_IS_Q) ? ga.lse2_t : ga.lse2;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, ln = lane & 31;
  const int l16 = lane & 15, g16 = lane >> 4;
  const unsigned short* O = OWNER_IS_Q ? ga.Q : ga.P;
  const unsigned short* R = OWNER_IS_Q ? ga.P : ga.Q;
  const int No = OWNER_IS_Q ? ga.B : ga.Pn, Nr = OWNER_IS_Q ? ga.Pn : ga.B;
  const int slen = OWNER_IS_Q ? ga.q_stream_len : ga.p_stream_len;
  const int a0 = oblk * G1_OWN + w * G1_OWN_W;   // this wave's first owner row
  const int sbeg = split * slen, send = min(Nr, sbeg + slen);
  const int nt = (send - sbeg + G1_T - 1) / G1_T;   // >= 1
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)smem);
  const int wu = __builtin_amdgcn_readfirstlane(w);   // the wave index as a scalar

  // owner rows as phase-1 B fragments: lane (ln, h) holds owner row 32 n + ln, columns 16 ks + 8 h .. + 7
  bf16x8 ofrag[2][8];
  int own_idx[2];
  float lse_o[2]; int r_o[2];
#pragma unroll
  for (int n = 0; n < 2; n++) {
    own_idx[n] = a0 + 32 * n + ln;
    const int row = min(own_idx[n], No - 1);
#pragma unroll
    for (int ks = 0; ks < 8; ks++) ofrag[n][ks] = *(const bf16x8*)(O + (size_t)row * D + 16 * ks + 8 * h);
    lse_o[n] = INFINITY; r_o[n] = -1;            // a row past the end: g = 0
    if ((OWNER_IS_Q || SYM) && own_idx[n] < No) lse_o[n] = lse_own[own_idx[n]];
    if (OWNER_IS_Q && own_idx[n] < No) r_o[n] = ga.pos_pad[own_idx[n]];
  }
  // The compiler's own loads end here: it does not see the direct-to-LDS loads below, and a wait of its own for
  // these registers inside the loop would also wait for those.  An empty statement that "uses" every loaded register.
#pragma unroll
  for (int n = 0; n < 2; n++) {
#pragma unroll
    for (int ks = 0; ks < 8; ks++) asm volatile("" : "+v"(ofrag[n][ks]));
    asm volatile("" : "+v"(lse_o[n]), "+v"(r_o[n]));
  }

  // ---- loads of a streamed tile: 8 instructions of 4 rows, two per wave; lane -> (row, chunk position) ------
  auto src_of = [&](int it, int max_row) __attribute__((always_inline)) -> unsigned {
    const int row = 4 * it + (lane >> 4);
    const int c = (lane & 15) ^ swz128(row);
    return (unsigned)(min(row, max_row) * (D * 2) + c * 16);
  };
  const unsigned voff_full[2] = {src_of(2 * w, G1_T - 1), src_of(2 * w + 1, G1_T - 1)};
  const unsigned stat_off = ((lane & 8) && !OWNER_IS_Q) ? (unsigned)((const char*)ga.pos_pad - (const char*)ga.lse2) + 16u * (lane & 7) : 16u * (lane & 7);
  const bool stat_wave = STR_STATS && wu == 0;
  auto prefetch = [&](int u) __attribute__((always_inline)) {   // tile u -> stage u % 4
    const int t0 = sbeg + u * G1_T;
    const unsigned st = lds0 + (u & (G1_STAGES - 1)) * G1_STAGE;
    const unsigned short* tile = R + (size_t)t0 * D;
    if (stat_wave) dma_lanes16(lse_str + t0, stat_off, st);
    if (t0 + G1_T <= Nr) {
      dma_group<1>(tile, &voff_full[0], st + G1_STAT + (2 * wu) * 1024);
      dma_group<1>(tile, &voff_full[1], st + G1_STAT + (2 * wu + 1) * 1024);
    } else {  // ragged last tile: rows past the end re-read the last valid row (their g is forced to 0)
#pragma unroll
      for (int k = 0; k < 2; k++) {
        const unsigned off = src_of(2 * w + k, Nr - 1 - t0);
        dma_group<1>(tile, &off, st + G1_STAT + (2 * wu + k) * 1024);
      }
    }
  };

  // per-lane LDS addresses inside a stage
  const unsigned sw_ln = swz128(ln);
  // transposing reads: rows 16 kk + 8 e + 4 h + (l16 >> 2), chunk 4 mt + 2 (g16 & 1) + ((l16 & 3) >> 1), half l16 & 1
  const int tr_r = 4 * h + (l16 >> 2), tr_c = 2 * (g16 & 1) + ((l16 & 3) >> 1);
  unsigned troff[2][2];  // [kk][e]: the swizzle depends on the row, so one base per (kk, e); + 64 * mt
#pragma unroll
  for (int kk = 0; kk < 2; kk++)
#pragma unroll
    for (int e = 0; e < 2; e++) {
      const int row = 16 * kk + 8 * e + tr_r;
      troff[kk][e] = G1_STAT + row * 256 + 8 * (l16 & 1);   // chunk part added per mt (it is swizzled)
    }

  f32x16 acc[4][2];
#pragma unroll
  for (int mt = 0; mt < 4; mt++)
#pragma unroll
    for (int n = 0; n < 2; n++)
#pragma unroll
      for (int r = 0; r < 16; r++) acc[mt][n][r] = 0.f;

  // ---- software pipeline over the tiles: iteration u interleaves, MFMA by MFMA, phase 1 of tile u+1, the
  // exp2 arithmetic of tile u (whose scores iteration u-1 left in registers) and phase 2 of tile u-1 (whose g the
  // previous iteration left as fragments): a wave's VALU work hides behind its own MFMAs only when interleaved.
  // Tiles u-1, u, u+1 are alive in the ring, u+2 .. u+5 in flight.
  f32x16 sacc[2][2];     // [tile parity][owner half]
  bf16x8 gfr[2][2];      // g of the tile last through the softmax: [owner half][kk]
#pragma unroll
  for (int n = 0; n < 2; n++)
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int e = 0; e < 8; e++) gfr[n][kk][e] = 0;

#pragma unroll 1
  for (int u = 0; u < min(nt, G1_AHEAD - 1); u++) prefetch(u);   // iteration -1 starts tile G1_AHEAD - 1

  // PT: parity of tile u+1 (where phase 1 writes); the softmax reads parity PT ^ 1
  // STEADY: all three parts are live (1 <= u, u + 1 < nt): no branches inside the MFMA stream
  auto body = [&](int u, auto pt_tag, auto steady_tag) __attribute__((always_inline)) {
    constexpr int PT = decltype(pt_tag)::value;
    constexpr bool STEADY = decltype(steady_tag)::value;
    const bool p1 = STEADY || (u + 1 < nt), sm = STEADY || (u >= 0 && u < nt), p2 = STEADY || (u >= 1);
    // my loads of tile u+1 have landed (tiles up to u + G1_AHEAD - 1 have been started)
    if (p1) {
      const int later = min(nt - 1, u + G1_AHEAD - 1) - (u + 1);   // tiles started after u+1: 0 .. G1_AHEAD - 2
      if (stat_wave) { if (later >= 4) wait_vmem<12>(); else if (later == 3) wait_vmem<9>(); else if (later == 2) wait_vmem<6>(); else if (later == 1) wait_vmem<3>(); else wait_vmem<0>(); }
      else { if (later >= 4) wait_vmem<8>(); else if (later == 3) wait_vmem<6>(); else if (later == 2) wait_vmem<4>(); else if (later == 1) wait_vmem<2>(); else wait_vmem<0>(); }
    }
    __syncthreads();  // ... and everybody's; everybody is done with tile u-2, whose stage is loaded next
    if (u + G1_AHEAD < nt) prefetch(u + G1_AHEAD);
    const unsigned char* st_p1 = smem + ((u + 1) & (G1_STAGES - 1)) * G1_STAGE;
    const unsigned char* st_sm = smem + (u & (G1_STAGES - 1)) * G1_STAGE;
    const unsigned char* st_p2 = smem + ((u - 1) & (G1_STAGES - 1)) * G1_STAGE;
    const int t0 = sbeg + u * G1_T;   // first streamed row of tile u

    // fragments: row statistics of tile u, then tile u+1 for phase 1 and transposed tile u-1 for phase 2 in
    // the order in which the rounds below consume them (LDS returns reads in order, and the 24 reads of the
    // four waves keep the LDS busy for most of an iteration: the first MFMAs must not wait for the last read)
    f32x4 lse_r[4]; i32x4 pos_r[4];
    if (STR_STATS && sm) {
#pragma unroll
      for (int j = 0; j < 4; j++) {
        lse_r[j] = *(const f32x4*)(st_sm + (8 * j + 4 * h) * 4);
        if (!OWNER_IS_Q) pos_r[j] = *(const i32x4*)(st_sm + 128 + (8 * j + 4 * h) * 4);
      }
    }
    bf16x8 pfr[8];
    bf16x8 afr[4][2];
    // round 2 k needs pfr[k] and afr[k / 2][k % 2]: the first four pairs are read here, pair k + 4 behind round 2 k + 1,
    // into the registers that pair k has just left (all eight at once cost 32 registers that the loop does not have)
    auto load_pair = [&](auto k_tag) __attribute__((always_inline)) {
      constexpr int k = decltype(k_tag)::value;
      if (p1) pfr[k] = *(const bf16x8*)(st_p1 + G1_STAT + ln * 256 + (((2 * k + h) ^ (int)sw_ln) * 16));
      if (p2) {
        constexpr int mt = k / 2, kk = k % 2;
        s16x4 q[2];
#pragma unroll
        for (int e = 0; e < 2; e++) {
          const int row = 16 * kk + 8 * e + tr_r;
          const int c = (4 * mt + tr_c) ^ swz128(row);
          q[e] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(st_p2 + troff[kk][e] + c * 16));
        }
        s16x8 t = {q[0][0], q[0][1], q[0][2], q[0][3], q[1][0], q[1][1], q[1][2], q[1][3]};
        afr[mt][kk] = __builtin_bit_cast(bf16x8, t);
      }
    };
    static_for<4>(load_pair);
    // 16 rounds: one phase-1 MFMA pair position, one phase-2 MFMA, the exp2 of two scores
    static_for<16>([&](auto i_tag) __attribute__((always_inline)) {
      constexpr int i = decltype(i_tag)::value;
      if (p1) {
        constexpr int ks = i / 2, n = i % 2;
        if constexpr (ks == 0) {
          f32x16 z;
#pragma unroll
          for (int r = 0; r < 16; r++) z[r] = 0.f;
          sacc[PT][n] = mfma32(pfr[ks], ofrag[n][ks], z);
        } else {
          sacc[PT][n] = mfma32(pfr[ks], ofrag[n][ks], sacc[PT][n]);
        }
      }
      if (p2) {
        constexpr int mt = i / 4, kk = (i / 2) % 2, n = i % 2;
        acc[mt][n] = mfma32(afr[mt][kk], gfr[n][kk], acc[mt][n]);
      }
      if (sm) {
#pragma unroll
        for (int n = 0; n < 2; n++) {
          float e;
          if constexpr (SYM) {  // mean of the row softmax and the column softmax (folding the halves into the
            // exponents saves two operations per score and measured slower here: 8 % while the kernel spilled, 1 % since)
            const float t = sacc[PT ^ 1][n][i] * ga.alpha2;
            e = 0.5f * fast_exp2(t - lse_o[n]) + 0.5f * fast_exp2(t - lse_r[i >> 2][i & 3]);
          } else {
            const float l = OWNER_IS_Q ? lse_o[n] : lse_r[i >> 2][i & 3];
            e = fast_exp2(sacc[PT ^ 1][n][i] * ga.alpha2 - l);
          }
          // an empty statement that "uses" the value: it keeps the arithmetic inside this round (pure
          // arithmetic would otherwise be moved behind all the MFMAs and run exposed)
          if constexpr (STEADY) asm volatile("" : "+v"(e));
          sacc[PT ^ 1][n][i] = e;
        }
      }
      if constexpr (i % 2 == 1 && i / 2 + 4 < 8) load_pair(std::integral_constant<int, i / 2 + 4>{});
      if constexpr (STEADY) __builtin_amdgcn_sched_barrier(0);  // the rounds stay in order
    });
    if (sm) {
      // 0 at the positive (j == r_i: its term is added in fp32 by the kernel that sums the partials, see PosFix),
      // zeros for rows past the end of the split and on the diagonal: few tiles
      bool rare = (t0 + G1_T > send) || (ga.mask_self && (t0 < a0 + G1_OWN_W) && (t0 + G1_T > a0));
      if (OWNER_IS_Q) {
        rare = rare || (unsigned)(r_o[0] - t0) < (unsigned)G1_T || (unsigned)(r_o[1] - t0) < (unsigned)G1_T;
      } else {
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
          for (int e = 0; e < 4; e++) rare = rare || (unsigned)(pos_r[j][e] - a0) < (unsigned)G1_OWN_W;
      }
      if (__builtin_amdgcn_ballot_w64(rare) != 0) {
#pragma unroll
        for (int n = 0; n < 2; n++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            const int m = t0 + 8 * (r >> 2) + 4 * h + (r & 3);   // streamed row of this register
            const bool hit = OWNER_IS_Q ? (r_o[n] == m) : (pos_r[r >> 2][r & 3] == own_idx[n]);
            if (hit || m >= send || (ga.mask_self && m == own_idx[n])) sacc[PT ^ 1][n][r] = 0.f;
          }
      }
    }
    // the phase-2 MFMAs above have read the old fragments: now they take the g of tile u
    if (sm) {
#pragma unroll
      for (int n = 0; n < 2; n++)
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
          typedef __attribute__((ext_vector_type(8))) float f32x8;
          const f32x16& g = sacc[PT ^ 1][n];
          const f32x8 v = {g[8 * kk], g[8 * kk + 1], g[8 * kk + 2], g[8 * kk + 3], g[8 * kk + 4], g[8 * kk + 5], g[8 * kk + 6], g[8 * kk + 7]};
          gfr[n][kk] = __builtin_convertvector(v, bf16x8);
        }
    }
  };
  // iterations u = -1 .. nt (phase 1 of tile 0 first, phase 2 of tile nt-1 last), two per trip so that the
  // parity of the score registers is a compile-time constant
  constexpr std::integral_constant<int, 0> pt0{};   // u odd: tile u+1 has parity 0
  constexpr std::integral_constant<int, 1> pt1{};
  body(-1, pt0, std::false_type{});
  body(0, pt1, std::false_type{});
  int u = 1;
#pragma unroll 1
  for (; u + 2 < nt; u += 2) {
    body(u, pt0, std::true_type{});
    body(u + 1, pt1, std::true_type{});
  }
#pragma unroll 1
  for (; u <= nt; u += 2) {
    body(u, pt0, std::false_type{});
    if (u + 1 <= nt) body(u + 1, pt1, std::false_type{});
  }

  // ---- epilogue: lane (ln, h) holds owner row 32 n + ln, columns 32 mt + 8 (r / 4) + 4 h + r % 4 -----------------
  float* out = OWNER_IS_Q ? (ga.dq_out + (size_t)split * ga.dq_split_stride) : (ga.dp_out + (size_t)split * ga.dp_split_stride);
#pragma unroll
  for (int n = 0; n < 2; n++) {
    if (own_idx[n] < No) {
#pragma unroll
      for (int mt = 0; mt < 4; mt++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
          const f32x4 v = {acc[mt][n][4 * j] * ga.out_scale, acc[mt][n][4 * j + 1] * ga.out_scale,
                           acc[mt][n][4 * j + 2] * ga.out_scale, acc[mt][n][4 * j + 3] * ga.out_scale};
          *(f32x4*)(out + (size_t)own_idx[n] * D + 32 * mt + 8 * j + 4 * h) = v;
        }
    }
  }
}

template <bool SYM>
__global__ void __launch_bounds__(256) grad128_kernel(GradArgs ga) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gsmem[];
  check_shared_positives(ga);
  const int nQ = ga.obQ * ga.nsq;
  const int id = xcd_task_id();
  if (id < nQ) {
    grad128_body<true, SYM>(ga, id % ga.obQ, id / ga.obQ, gsmem);
  } else {
    const int t = id - nQ;
    grad128_body<false, SYM>(ga, t % ga.obP, t / ga.obP, gsmem);
  }
}

// ===========================================================================
// Statistics pass for d = 128 (Eq. 4's normaliser, the positive's logit and the arg-max, per anchor and split).
// The layout of the d = 128 gradient pass without its second contraction: a workgroup (4 waves) owns 256 anchors,
// each wave 64 of them with all 128 columns in registers, and all four share the streamed target tiles (32 rows)
// through the same LDS ring.  Lane (n, h) holds, for its two anchors 32 i + n, the scores of 16 of a tile's 32
// targets; the other 16 are in lane (n, h ^ 1).  The running (max, sum, arg-max) of an anchor therefore lives in
// a lane of its own and no lane talks to another before the end of the stream: 16 MFMAs against about 5 vector
// operations per score, which a second workgroup on the same CU runs behind the first one's MFMAs.
// ===========================================================================
constexpr int S1_AHEAD = 6;   // tile u is read, tiles u+1 .. u+5 are in flight, tile u+6 goes where tile u-2 was
template <bool ARGMAX>
__global__ void __launch_bounds__(256, 2) stats128_kernel(const unsigned short* __restrict__ Q,
                                                          const unsigned short* __restrict__ Pm,
                                                          const int32_t* __restrict__ pos_idx, int B, int P,
                                                          float alpha2, int mask_self, int n_ablk, int cols_per_split,
                                                          float* __restrict__ part_m, float* __restrict__ part_l,
                                                          int* __restrict__ part_idx, float* __restrict__ pos_t) {
  extern __shared__ __attribute__((aligned(16))) unsigned char s1mem[];
  constexpr int D = 128;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, h = lane >> 5, ln = lane & 31;
  const int task = xcd_task_id();
  const int ablk = task % n_ablk, split = task / n_ablk;
  const int a0 = ablk * G1_OWN + w * G1_OWN_W;   // this wave's first anchor
  const int sbeg = split * cols_per_split, send = min(P, sbeg + cols_per_split);
  const int nt = (send - sbeg + G1_T - 1) / G1_T;   // >= 1
  const unsigned lds0 = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)s1mem);
  const int wu = __builtin_amdgcn_readfirstlane(w);

  // anchors as B fragments: lane (ln, h) holds anchor 32 n + ln, columns 16 ks + 8 h .. + 7
  bf16x8 ofrag[2][8];
  int own_idx[2], r_o[2];
#pragma unroll
  for (int n = 0; n < 2; n++) {
    own_idx[n] = a0 + 32 * n + ln;
    const int row = min(own_idx[n], B - 1);
#pragma unroll
    for (int ks = 0; ks < 8; ks++) ofrag[n][ks] = *(const bf16x8*)(Q + (size_t)row * D + 16 * ks + 8 * h);
    r_o[n] = (own_idx[n] < B) ? pos_idx[own_idx[n]] : -1;
  }
  // the compiler's own loads end here (it does not see the direct-to-LDS loads counted by wait_vmem below)
#pragma unroll
  for (int n = 0; n < 2; n++) {
#pragma unroll
    for (int ks = 0; ks < 8; ks++) asm volatile("" : "+v"(ofrag[n][ks]));
    asm volatile("" : "+v"(r_o[n]));
  }

  // loads of a streamed tile: 8 instructions of 4 rows, two per wave; lane -> (row, chunk position)
  auto src_of = [&](int it, int max_row) __attribute__((always_inline)) -> unsigned {
    const int row = 4 * it + (lane >> 4);
    const int c = (lane & 15) ^ swz128(row);
    return (unsigned)(min(row, max_row) * (D * 2) + c * 16);
  };
  const unsigned voff_full[2] = {src_of(2 * w, G1_T - 1), src_of(2 * w + 1, G1_T - 1)};
  auto prefetch = [&](int u) __attribute__((always_inline)) {
    const int t0 = sbeg + u * G1_T;
    const unsigned st = lds0 + (u & (G1_STAGES - 1)) * G1_STAGE;
    const unsigned short* tile = Pm + (size_t)t0 * D;
    if (t0 + G1_T <= P) {
      dma_group<1>(tile, &voff_full[0], st + G1_STAT + (2 * wu) * 1024);
      dma_group<1>(tile, &voff_full[1], st + G1_STAT + (2 * wu + 1) * 1024);
    } else {  // ragged last tile: rows past the end re-read the last valid row (masked below)
#pragma unroll
      for (int k = 0; k < 2; k++) {
        const unsigned off = src_of(2 * w + k, P - 1 - t0);
        dma_group<1>(tile, &off, st + G1_STAT + (2 * wu + k) * 1024);
      }
    }
  };
  const unsigned sw_ln = swz128(ln);

  float rm[2], rl[2], rpos[2];
  int ridx[2];
  bool got[2];
#pragma unroll
  for (int n = 0; n < 2; n++) { rm[n] = -INFINITY; rl[n] = 0.f; rpos[n] = 0.f; ridx[n] = 0x7fffffff; got[n] = false; }

#pragma unroll 1
  for (int u = 0; u < min(nt, S1_AHEAD); u++) prefetch(u);

#pragma unroll 1
  for (int u = 0; u < nt; u++) {
    // my loads of tile u have landed: two instructions per tile, tiles up to u + S1_AHEAD - 1 have been started
    const int later = min(nt - 1, u + S1_AHEAD - 1) - u;
    if (later >= 5) wait_vmem<10>(); else if (later == 4) wait_vmem<8>(); else if (later == 3) wait_vmem<6>();
    else if (later == 2) wait_vmem<4>(); else if (later == 1) wait_vmem<2>(); else wait_vmem<0>();
    __syncthreads();  // ... and everybody's; everybody is past tile u-1, so the stage of tile u-2 is free
    if (u + S1_AHEAD < nt) prefetch(u + S1_AHEAD);
    const unsigned char* st = s1mem + (u & (G1_STAGES - 1)) * G1_STAGE;
    const int t0 = sbeg + u * G1_T;

    bf16x8 pfr[8];
#pragma unroll
    for (int k = 0; k < 8; k++) pfr[k] = *(const bf16x8*)(st + G1_STAT + ln * 256 + (((2 * k + h) ^ (int)sw_ln) * 16));
    f32x16 s[2];
#pragma unroll
    for (int n = 0; n < 2; n++)
#pragma unroll
      for (int r = 0; r < 16; r++) s[n][r] = 0.f;
#pragma unroll
    for (int k = 0; k < 8; k++)
#pragma unroll
      for (int n = 0; n < 2; n++) s[n] = mfma32(pfr[k], ofrag[n][k], s[n]);

    // online statistics; s holds raw dot products, the base-2 logit is alpha2 * s (alpha2 > 0: same order).
    // Register r of lane (ln, h) is target t0 + 8 (r / 4) + 4 h + r % 4: increasing in r.
    // the masks that can touch this tile: few tiles, and one scalar branch for the wave (as a per-lane condition the
    // compiler turns the masking into selects that every tile then pays for)
    bool rare = (t0 + G1_T > send) || (mask_self && t0 < a0 + G1_OWN_W && t0 + G1_T > a0);
    rare = rare || (unsigned)(r_o[0] - t0) < (unsigned)G1_T || (unsigned)(r_o[1] - t0) < (unsigned)G1_T;
    if (__builtin_amdgcn_ballot_w64(rare) != 0) {
#pragma unroll
      for (int n = 0; n < 2; n++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          const int j = t0 + 8 * (r >> 2) + 4 * h + (r & 3);
          const bool self = mask_self && j == own_idx[n];
          const bool masked = j >= send || self;
          // (a positive that the self-mask removes has the logit -inf: its row loss is then +inf)
          if (j == r_o[n] && j < send) { rpos[n] = self ? -INFINITY : s[n][r] * alpha2; got[n] = true; }
          if (masked) s[n][r] = -INFINITY;
        }
    }
#pragma unroll
    for (int n = 0; n < 2; n++) {
      float tmr = -INFINITY; int tc = 0;
#pragma unroll
      for (int r = 0; r < 16; r++) {
        const float t = s[n][r];
        if (ARGMAX) {
          const bool le = t <= tmr;   // strict >: the first (smallest) index attaining the maximum
          tmr = le ? tmr : t;
          tc = le ? tc : r;
        } else {
          tmr = fmaxf(tmr, t);
        }
      }
      if (tmr > -INFINITY) {
        const float tm = tmr * alpha2;
        const float mn = fmaxf(rm[n], tm);
        float sum = 0.f;
#pragma unroll
        for (int r = 0; r < 16; r++) sum += fast_exp2(__builtin_fmaf(s[n][r], alpha2, -mn));
        rl[n] = rl[n] * fast_exp2(rm[n] - mn) + sum;
        if (ARGMAX && tm > rm[n]) ridx[n] = t0 + 8 * (tc >> 2) + 4 * h + (tc & 3);  // later tiles have larger indices
        rm[n] = mn;
      }
    }
  }

  // the positive's score is seen by exactly one lane of one workgroup
#pragma unroll
  for (int n = 0; n < 2; n++)
    if (got[n] && own_idx[n] < B) pos_t[own_idx[n]] = rpos[n];
  // combine the two half-waves (same anchor, the other 16 targets of every tile), then write the split partial
#pragma unroll
  for (int n = 0; n < 2; n++) {
    const float m2 = __shfl_xor(rm[n], 32), l2 = __shfl_xor(rl[n], 32);
    const int i2 = __shfl_xor(ridx[n], 32);
    stat_merge(rm[n], rl[n], ridx[n], m2, l2, i2);
    if (h == 0 && own_idx[n] < B) {
      const size_t o = (size_t)split * B + own_idx[n];
      part_m[o] = rm[n]; part_l[o] = rl[n]; part_idx[o] = ridx[n];
    }
  }
}

template <bool ARGMAX>
static hipError_t stats128_launch(const LossArgs& a, const LossPlan& pl) {
  static bool attr_done[64];
  if (hipError_t e = ensure_dyn_lds((const void*)stats128_kernel<ARGMAX>, G1_SMEM, attr_done); e != hipSuccess) return e;
  char* ws = a.ws;
  const int n_ablk = (a.B + G1_OWN - 1) / G1_OWN;
  stats128_kernel<ARGMAX><<<n_ablk * pl.stat_splits, 256, G1_SMEM, a.stream>>>(
      (const unsigned short*)a.q, (const unsigned short*)a.p, a.pos_idx, a.B, a.P, a.alpha * kLog2e,
      (a.flags & GC_MASK_SELF) ? 1 : 0, n_ablk, pl.stat_cols_per_split, (float*)(ws + pl.off_part_m),
      (float*)(ws + pl.off_part_l), (int*)(ws + pl.off_part_idx), (float*)(ws + pl.off_pos));
  return hipGetLastError();
}
static hipError_t launch_stats128(const LossArgs& a, const LossPlan& pl) {
  return a.argmax ? stats128_launch<true>(a, pl) : stats128_launch<false>(a, pl);
}

template <int D, bool SYM>
__global__ void __launch_bounds__(256) grad_mfma_kernel(GradArgs ga) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gsmem[];
  check_shared_positives(ga);
  const int nQ = ga.obQ * ga.nsq;
  const int id = xcd_task_id();
  if (id < nQ) {
    grad_body<D, true, SYM>(ga, id % ga.obQ, id / ga.obQ, gsmem);
  } else {
    const int t = id - nQ;
    grad_body<D, false, SYM>(ga, t % ga.obP, t / ga.obP, gsmem);
  }
}

// the online-statistics walk: every workgroup has the dQ role
template <int D>
__global__ void __launch_bounds__(256) grad_online_kernel(GradArgs ga) {
  extern __shared__ __attribute__((aligned(16))) unsigned char gsmem[];
  const int id = xcd_task_id();
  grad_body<D, true, false, true>(ga, id % ga.obQ, id / ga.obQ, gsmem);
}
template <int D>
static hipError_t grad_online_launch(const GradArgs& ga, int nwg, hipStream_t stream) {
  const int smem = GradCfg<D>::SMEM;
  static bool attr_done[64];
  if (hipError_t e = ensure_dyn_lds((const void*)grad_online_kernel<D>, smem, attr_done); e != hipSuccess) return e;
  grad_online_kernel<D><<<nwg, 256, smem, stream>>>(ga);
  return hipGetLastError();
}

// dQ partials (scaled by alpha / B, relative to each split's reference) and the statistics of every split
hipError_t launch_grad_online(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  GradArgs ga{};
  ga.Q = (const unsigned short*)a.q; ga.P = (const unsigned short*)a.p;
  ga.pos_pad = a.pos_idx; ga.lse2 = nullptr; ga.lse2_t = nullptr;
  ga.B = a.B; ga.Pn = a.P;
  ga.alpha2 = a.alpha * kLog2e; ga.out_scale = a.alpha / (float)a.B * (a.grad_mul != 0.f ? a.grad_mul : 1.f);
  ga.mask_self = (a.flags & GC_MASK_SELF) ? 1 : 0;
  ga.obQ = (a.B + GR_OWN - 1) / GR_OWN; ga.nsq = pl.fz_nsq; ga.q_stream_len = pl.fz_q_stream_len;
  ga.dq_out = (float*)(ws + pl.off_dq_part); ga.dq_split_stride = (size_t)a.B * a.d;
  ga.on_ref = (float*)(ws + pl.off_on_ref); ga.on_best = (float*)(ws + pl.off_part_m); ga.on_l = (float*)(ws + pl.off_part_l);
  ga.on_idx = (int*)(ws + pl.off_part_idx); ga.on_pos = (float*)(ws + pl.off_pos);
  ga.on_argmax = a.argmax ? 1 : 0;
  const int nwg = ga.obQ * ga.nsq;
  switch (a.d) {
    case 256: return grad_online_launch<256>(ga, nwg, a.stream);
    case 384: return grad_online_launch<384>(ga, nwg, a.stream);
    case 512: return grad_online_launch<512>(ga, nwg, a.stream);
    case 640: return grad_online_launch<640>(ga, nwg, a.stream);
    case 768: return grad_online_launch<768>(ga, nwg, a.stream);
    default: return hipErrorInvalidValue;
  }
}

template <int D, bool SYM>
static hipError_t grad_mfma_launch_as(const GradArgs& ga, int nwg, hipStream_t stream) {
  const int smem = GradCfg<D>::SMEM;
  static bool attr_done[64];
  if (hipError_t e = ensure_dyn_lds((const void*)grad_mfma_kernel<D, SYM>, smem, attr_done); e != hipSuccess) return e;
  grad_mfma_kernel<D, SYM><<<nwg, 256, smem, stream>>>(ga);
  return hipGetLastError();
}
template <int D>
static hipError_t grad_mfma_launch(const GradArgs& ga, int nwg, hipStream_t stream) {
  return ga.lse2_t ? grad_mfma_launch_as<D, true>(ga, nwg, stream) : grad_mfma_launch_as<D, false>(ga, nwg, stream);
}
template <bool SYM>
static hipError_t grad128_launch(const GradArgs& ga, int nwg, hipStream_t stream) {
  static bool attr_done[64];
  if (hipError_t e = ensure_dyn_lds((const void*)grad128_kernel<SYM>, G1_SMEM, attr_done); e != hipSuccess) return e;
  grad128_kernel<SYM><<<nwg, 256, G1_SMEM, stream>>>(ga);
  return hipGetLastError();
}

hipError_t launch_grad_mfma(const LossArgs& a, const LossPlan& pl) {
  char* ws = a.ws;
  GradArgs ga{};
  ga.Q = (const unsigned short*)a.q; ga.P = (const unsigned short*)a.p;
  ga.pos_pad = (const int32_t*)(ws + pl.off_pos_pad); ga.lse2 = (const float*)(ws + pl.off_lse2);
  ga.lse2_t = a.lse2_t;
  ga.B = a.B; ga.Pn = a.P;
  ga.alpha2 = a.alpha * kLog2e; ga.out_scale = a.alpha / (float)a.B * (a.grad_mul != 0.f ? a.grad_mul : 1.f);
  ga.mask_self = (a.flags & GC_MASK_SELF) ? 1 : 0;
  // NT-Xent in one walk: q = p = z, so the score matrix is symmetric, target j's log-sum-exp is anchor j's, and
  //   dz_i = (alpha/n) sum_j (g_ij + g_ji) z_j,   g_ij + g_ji = 2^(t_ij - lse2_i) + 2^(t_ij - lse2_j) - 2 [j = pair(i)]:
  // twice the coefficient of the symmetric loss with both statistics taken from the one array.  Only the dQ role runs.
  const bool one_walk = pl.one_walk && a.dz;
  if (one_walk) { ga.lse2_t = ga.lse2; ga.out_scale *= 2.f; }
  const bool want_q = a.dq || a.dz, want_p = (a.dp || a.dz) && !one_walk;
  const size_t nq = (size_t)a.B * a.d, np = (size_t)a.P * a.d;
  const int own = (a.d == 128) ? G1_OWN : GR_OWN;   // owner rows per workgroup
  ga.obQ = want_q ? (a.B + own - 1) / own : 0; ga.nsq = pl.nsq; ga.q_stream_len = pl.q_stream_len;
  ga.obP = want_p ? (a.P + own - 1) / own : 0; ga.nsp = pl.nsp; ga.p_stream_len = pl.p_stream_len;
  // every output goes through the kernel that sums the split partials (a single split included): it adds the
  // positive's term in fp32 (PosFix) and rounds a bf16 cache
  const bool cache_bf16 = (a.flags & GC_CACHE_BF16) != 0;
  ga.dq_out = (float*)(ws + pl.off_dq_part); ga.dq_split_stride = nq;
  ga.dp_out = (float*)(ws + pl.off_dp_part); ga.dp_split_stride = np;
  // the symmetric loss inverts its pairing itself (a bijection); one direction: the merge left an anchor per target
  const bool sym_pairs = a.lse2_t != nullptr;
  if (want_p && !sym_pairs) { ga.inv = (const int32_t*)(ws + pl.off_inv); ga.shared = (int*)(ws + pl.off_err) + 1; }
  const int nwg = ga.obQ * ga.nsq + ga.obP * ga.nsp;
  if (nwg == 0) { prof_mark_grad_kernel_done(a.stream); return hipSuccess; }
  hipError_t e;
  switch (a.d) {
    case 128: e = ga.lse2_t ? grad128_launch<true>(ga, nwg, a.stream) : grad128_launch<false>(ga, nwg, a.stream); break;
    case 256: e = grad_mfma_launch<256>(ga, nwg, a.stream); break;
    case 384: e = grad_mfma_launch<384>(ga, nwg, a.stream); break;
    case 512: e = grad_mfma_launch<512>(ga, nwg, a.stream); break;
    case 640: e = grad_mfma_launch<640>(ga, nwg, a.stream); break;
    case 768: e = grad_mfma_launch<768>(ga, nwg, a.stream); break;
    default: return hipErrorInvalidValue;
  }
  if (e != hipSuccess) return e;
  prof_mark_grad_kernel_done(a.stream);
  // fixed-order sums of the split partials, each with the positive's term of its rows; the first of these
  // launches also sums the row losses if asked to
  PosFix fx{};
  fx.pos = ga.pos_pad; fx.pos_t = (const float*)(ws + pl.off_pos); fx.lse2 = ga.lse2; fx.lse2_t = ga.lse2_t;
  fx.B = a.B; fx.P = a.P; fx.d = a.d; fx.scale = ga.out_scale;
  const LossArgs* loss_of = a.loss_with_partials ? &a : nullptr;
  if (a.dz) {   // NT-Xent, one walk: rows are anchors, the positive of view i is view i ^ 1
    fx.mode = 1; fx.other = ga.P;
    const float* srcs[1] = {ga.dq_out}; int counts[1] = {pl.nsq}; size_t strides[1] = {nq};
    return launch_partial_reduce(a.dz, srcs, counts, strides, 1, nq, a.stream, loss_of, &pl, false, &fx);
  }
  if (want_q) {
    fx.mode = 1; fx.other = ga.P;
    const float* srcs[1] = {ga.dq_out}; int counts[1] = {pl.nsq}; size_t strides[1] = {nq};
    e = launch_partial_reduce(a.dq, srcs, counts, strides, 1, nq, a.stream, loss_of, &pl, cache_bf16, &fx);
    if (e != hipSuccess) return e;
    loss_of = nullptr;
  }
  if (want_p) {
    fx.mode = 2; fx.other = ga.Q;
    fx.inv = sym_pairs ? a.pos_inv : ga.inv; fx.shared = sym_pairs ? a.zero_word : ga.shared;
    const float* srcs[1] = {ga.dp_out}; int counts[1] = {pl.nsp}; size_t strides[1] = {np};
    e = launch_partial_reduce(a.dp, srcs, counts, strides, 1, np, a.stream, loss_of, &pl, cache_bf16, &fx);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace gc
