// fp16 x fp16 -> fp32 GEMM on the gfx950 matrix cores, C[M,N] = A[M,K] . W[N,K]^T, with the
// epilogues the decoder needs fused in.  (Weights are the caller's bf16 values held in fp16, which
// represents them exactly; activations are fp16, whose 11 significant bits keep the logits within
// the parity bound where bf16 activations do not.)  Both operands are K-block major (see kblk_off), so a
// block's tile is one contiguous run in memory and every MFMA operand fragment is one 16-byte LDS read.
// A block of WM x WN waves owns a BM x BN tile; each wave a (BM/WM) x (BN/WN) sub-tile built from 32x32x16
// MFMAs.  A and W tiles of depth 64 go from global memory straight into LDS (16-byte chunks, XOR-swizzled by
// row so that fragment reads spread over all banks), two or four stages deep, with one barrier per K step;
// a K that is not a multiple of 64 takes the older path through registers, which can zero-fill the tail.
#include "kernels.h"
#include <algorithm>

namespace {

constexpr int BK = 64;            // fp16 elements of K per LDS stage (128 bytes per row)
#ifndef SWZ_SHIFT
#define SWZ_SHIFT 1
#endif
// LDS rows are 8 chunks of 16 bytes; chunk c of row r is stored at chunk position c ^ swz(r).  The LDS of
// gfx950 has 64 banks of 4 bytes: 16 lanes of a 128-bit read are served per cycle, and rows r, r + 1 sit in
// opposite halves of the banks, so the swizzle steps every second row (measured: SQ_LDS_BANK_CONFLICT = 0).
__device__ __forceinline__ int swz(int r) { return (r >> SWZ_SHIFT) & 7; }

// Blocks are handed to the 8 XCDs round-robin by the hardware.  Renumber them so that each XCD
// (one L2) works on a contiguous range of logical tile ids, then walk tiles M-fastest inside groups
// of 8 M-tiles: the blocks that share a weight tile run on the same L2 at the same time.
// With split-K the `splits` blocks of one tile are neighbours in that order.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int splits, int& tm, int& tn, int& split) {
  const int nb = gridDim.x, bid = blockIdx.x;
  const int per = (nb + 7) >> 3;
  const int full = (nb & 7) == 0 ? 8 : (nb & 7);
  const int xcd = bid & 7, slot = bid >> 3;
  int logical = xcd < full ? xcd * per + slot : full * per + (xcd - full) * (per - 1) + slot;
  split = logical % splits;
  logical /= splits;
  constexpr int GROUP_M = 8;
  const int per_group = GROUP_M * tiles_n;
  const int group = logical / per_group;
  const int first_m = group * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int in_group = logical - group * per_group;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

// erf by the rational-exponential form of Abramowitz & Stegun 7.1.26 (absolute error < 1.5e-7, far below the
// fp16 rounding of the result): a third of the instructions of the library erff, which matters in an epilogue.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(1.0f + 0.3275911f * ax);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float r = 1.0f - poly * __expf(-ax * ax);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.0f + erf_as(v * 0.70710678118654752f)); }
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

// nothing may be scheduled across this point
#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

template <int N>
__device__ __forceinline__ void wait_loads_then_barrier() {
  // all but the N most recent vector-memory loads of this wave have landed; then every wave of the block is here
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

// NS = 0: tiles travel global -> registers -> LDS (two LDS stages).  NS >= 2: NS LDS stages filled by direct
// global -> LDS loads, issued NS - 1 K steps ahead (needs K % 64 == 0).
// PR: precise mode (see GemmArgs): bf16 operands, A as hi/lo pairs; every K block of W meets the hi and then the lo
// block of A in two consecutive steps of the K loop.
template <int BM, int BN, int WM, int WN, int EPI, bool KTAIL, int NS = 0, bool PR = false>
__global__ __launch_bounds__(WM * WN * 64) void gemm_f16_kernel(GemmArgs g) {
  constexpr int NT = WM * WN * 64;               // threads
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32;   // 32x32 MFMA tiles per wave in each direction
  constexpr int RPP = NT / 8;                    // rows covered by one pass of 16-byte loads
  constexpr int PA = BM / RPP, PB = BN / RPP;
  static_assert(PA >= 1 && PB >= 1 && TM >= 1 && TN >= 1, "tile too small for the thread count");
  static_assert(NS == 0 || (NS >= 2 && NS <= 4 && !KTAIL), "direct loads need whole K tiles");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];   // max(2, NS) x (BM + BN) x BK
  // GEMM waves issue ahead of whatever shares their SIMD: in a decode step that is the other half's attention, whose
  // waves mostly wait for memory (measured: the GEMMs' time in that company -10 %, the decode phase -0.8 %)
  __builtin_amdgcn_s_setprio(3);
  constexpr int STAGE = (BM + BN) * BK;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  int tile_m, tile_n, split;
  const int splits = EPI == EPI_PARTIAL ? g.splits : 1;
  tile_of_block(tiles_m, tiles_n, splits, tile_m, tile_n, split);
  const int row0 = tile_m * BM, col0 = tile_n * BN;

  // ---- global -> register staging: thread t covers chunk (t % 8) of rows (t / 8) + RPP i
  const int ld_chunk = tid & 7, ld_row = tid >> 3;
  const uint16_t* __restrict__ A = (const uint16_t*)g.A;
  const uint16_t* __restrict__ W = (const uint16_t*)g.W;
  // operands are K-block major: K tile kt of rows r0.. is the contiguous run starting at (kt * rows + r0) * 64,
  // and thread t reads bytes [16 t, 16 t + 16) of it (rows past the end repeat the last row)
  u32x4 ra[PA], rb[PB];
  const uint16_t* pa[PA];
  const uint16_t* pb[PB];
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    int r = min(row0 + ld_row + RPP * i, g.M - 1);
    pa[i] = A + (size_t)r * 64 + ld_chunk * 8;
  }
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    int r = min(col0 + ld_row + RPP * i, g.N - 1);
    pb[i] = W + (size_t)r * 64 + ld_chunk * 8;
  }
  const size_t ka = (size_t)g.M * 64, kw = (size_t)g.N * 64;    // elements between K tiles
  const int nkb = (g.K + BK - 1) / BK;                          // K blocks of W (and of each half of a hi/lo A)
  // K tile kt of the loop reads block ak(kt) of A and block wk(kt) of W.  Precise mode takes the hi and the lo block of A
  // against the same block of W in consecutive steps (A holds its nkb hi blocks, then its nkb lo blocks): the second
  // request for the W block finds it in L2, so the weights cross HBM once
  auto wk = [&](int kt) { return PR ? kt >> 1 : kt; };
  auto ak = [&](int kt) { return PR ? (kt >> 1) + (kt & 1) * nkb : kt; };
  auto load_global = [&](int kt) {
    if constexpr (KTAIL) {     // K is not a multiple of BK: chunks beyond K read as zero
      const bool ok = wk(kt) * BK + ld_chunk * 8 < g.K;
#pragma unroll
      for (int i = 0; i < PA; ++i) ra[i] = ok ? *(const u32x4*)(pa[i] + ak(kt) * ka) : u32x4{0, 0, 0, 0};
#pragma unroll
      for (int i = 0; i < PB; ++i) rb[i] = ok ? *(const u32x4*)(pb[i] + wk(kt) * kw) : u32x4{0, 0, 0, 0};
    } else {
#pragma unroll
      for (int i = 0; i < PA; ++i) ra[i] = *(const u32x4*)(pa[i] + ak(kt) * ka);
#pragma unroll
      for (int i = 0; i < PB; ++i) rb[i] = *(const u32x4*)(pb[i] + wk(kt) * kw);
    }
  };
  // one 32x32x16 matrix instruction on 16-bit fragments: fp16, or bf16 in precise mode
  auto mfma = [](f16x8 b, f16x8 a, f32x16 c) {
    if constexpr (PR) return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, b), __builtin_bit_cast(bf16x8, a), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_32x32x16_f16(b, a, c, 0, 0, 0);
  };
  auto store_lds = [&](int buf) {
    uint16_t* la = lds + buf * STAGE;
    uint16_t* lb = la + BM * BK;
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      int r = ld_row + RPP * i;
      *(u32x4*)(la + r * BK + ((ld_chunk ^ swz(r)) * 8)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      int r = ld_row + RPP * i;
      *(u32x4*)(lb + r * BK + ((ld_chunk ^ swz(r)) * 8)) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk_all = PR ? 2 * nkb : nkb;
  const int kt0 = (int)((long long)split * nk_all / splits);          // this block's share of the K tiles
  const int nk = (int)((long long)(split + 1) * nk_all / splits);
  const int frow = lane & 31, fhalf = lane >> 5;
  // one K step on the LDS stage `buf`; `mid` runs between the last two MFMA groups
  auto k_step = [&](int buf, auto&& mid) {
    const uint16_t* la = lds + buf * STAGE + (wm * (BM / WM)) * BK;
    const uint16_t* lb = lds + buf * STAGE + BM * BK + (wn * (BN / WN)) * BK;
    // fragments of step kk + 1 are fetched from LDS while the MFMAs of step kk run
    f16x8 fa[2][TM], fb[2][TN];
    auto load_frags = [&](int kk, int slot) {
      const int chunk = kk * 2 + fhalf;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int r = i * 32 + frow;
        fa[slot][i] = *(const f16x8*)(la + r * BK + ((chunk ^ swz(r)) * 8));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int r = j * 32 + frow;
        fb[slot][j] = *(const f16x8*)(lb + r * BK + ((chunk ^ swz(r)) * 8));
      }
    };
    load_frags(0, 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      if (kk + 1 < BK / 16) load_frags(kk + 1, (kk + 1) & 1);
      if (kk == BK / 16 - 2) mid();
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = mfma(fb[kk & 1][j], fa[kk & 1][i], acc[i][j]);
    }
  };

  if constexpr (NS == 0) {
    load_global(kt0);
    store_lds(kt0 & 1);
    __syncthreads();
    for (int kt = kt0; kt < nk; ++kt) {
      const int cur = kt & 1;
      if (kt + 1 < nk) load_global(kt + 1);
      // the next tile moves from registers to the other LDS buffer under the last MFMAs of this one
      k_step(cur, [&] { if (kt + 1 < nk) store_lds(cur ^ 1); });
      __syncthreads();
    }
  } else {
    // Direct loads: a wave instruction moves 64 16-byte chunks = 8 tile rows into 1 KB of LDS in lane order, so
    // the XOR swizzle is applied on the source side: the lane that fills chunk position p of row r fetches chunk
    // p ^ swz(r).  Rows advance by a multiple of 16 per pass, which leaves swz(r) unchanged.
    static_assert(RPP % 16 == 0, "the swizzle must not depend on the pass");
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int lrow = wave_u * 8 + (lane >> 3);
    const int schunk = (lane & 7) ^ swz(lrow);
    const uint16_t* qa[PA];
    const uint16_t* qb[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i) qa[i] = A + (size_t)min(row0 + lrow + RPP * i, g.M - 1) * 64 + schunk * 8;
#pragma unroll
    for (int i = 0; i < PB; ++i) qb[i] = W + (size_t)min(col0 + lrow + RPP * i, g.N - 1) * 64 + schunk * 8;
    typedef const __attribute__((address_space(1))) void* gptr_t;
    typedef __attribute__((address_space(3))) void* lptr_t;
    auto issue = [&](int kt, int buf) {
      uint16_t* la = lds + buf * STAGE + wave_u * 8 * BK;
#pragma unroll
      for (int i = 0; i < PA; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(qa[i] + ak(kt) * ka), (lptr_t)(la + i * RPP * BK), 16, 0, 0);
#pragma unroll
      for (int i = 0; i < PB; ++i)
        __builtin_amdgcn_global_load_lds((gptr_t)(qb[i] + wk(kt) * kw), (lptr_t)(la + (BM + i * RPP) * BK), 16, 0, 0);
    };
    constexpr int L = PA + PB;                      // loads per wave and stage
    if constexpr (NS == 2) {
      // Skewed by a quarter of a K step: the wait for the next stage and the barrier sit before the last of the four
      // MFMA groups of a stage, whose fragments are in registers by then.  Behind the barrier nobody reads this
      // stage's LDS any more, so its buffer is refilled at once, and the first fragments of the next stage are
      // fetched while the last MFMA group runs: the matrix pipe does not drain at the stage boundary.
      f16x8 fa[2][TM], fb[2][TN];
      auto frags = [&](int buf, int kk, int slot) {
        const uint16_t* la = lds + buf * STAGE + (wm * (BM / WM)) * BK;
        const uint16_t* lb = lds + buf * STAGE + BM * BK + (wn * (BN / WN)) * BK;
        const int chunk = kk * 2 + fhalf;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          int r = i * 32 + frow;
          fa[slot][i] = *(const f16x8*)(la + r * BK + ((chunk ^ swz(r)) * 8));
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          int r = j * 32 + frow;
          fb[slot][j] = *(const f16x8*)(lb + r * BK + ((chunk ^ swz(r)) * 8));
        }
      };
      constexpr int HEAD = TM * TN >= 8 ? 2 : 1;
      auto mma = [&](int slot, int lo, int hi) {     // MFMAs lo .. hi - 1 of the group, row-major over the wave's tiles
#pragma unroll
        for (int t = 0; t < TM * TN; ++t)
          if (t >= lo && t < hi)
            acc[t / TN][t % TN] = mfma(fb[slot][t % TN], fa[slot][t / TN], acc[t / TN][t % TN]);
      };
      issue(kt0, 0);
      wait_loads_then_barrier<0>();
      if (kt0 + 1 < nk) issue(kt0 + 1, 1);
      frags(0, 0, 0);
      for (int kt = kt0; kt < nk; ++kt) {
        const int buf = (kt - kt0) & 1;
        // Per MFMA group: the first MFMAs, then the LDS reads of the next group's fragments, then the rest, in exactly
        // this order (the fences stop the compiler from sinking the reads behind the MFMAs, where the wait for them
        // would sit directly in front of their first use).
        mma(0, 0, HEAD);
        SCHED_FENCE();
        frags(buf, 1, 1);
        SCHED_FENCE();
        mma(0, HEAD, TM * TN);
        SCHED_FENCE();
        mma(1, 0, HEAD);
        SCHED_FENCE();
        frags(buf, 2, 0);
        SCHED_FENCE();
        mma(1, HEAD, TM * TN);
        SCHED_FENCE();
        mma(0, 0, HEAD);
        SCHED_FENCE();
        frags(buf, 3, 1);
        SCHED_FENCE();
        mma(0, HEAD, TM * TN);
        SCHED_FENCE();
        mma(1, 0, HEAD);
        SCHED_FENCE();
        if (kt + 1 < nk) {
          // stage kt + 1 has landed, and every wave holds its last fragments of stage kt in registers
          asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
          if (kt + 2 < nk) issue(kt + 2, buf);
          frags(buf ^ 1, 0, 0);
          SCHED_FENCE();
        }
        mma(1, HEAD, TM * TN);
        SCHED_FENCE();
      }
    } else {
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (kt0 + s < nk) issue(kt0 + s, s);
    for (int kt = kt0; kt < nk; ++kt) {
      // stage kt must have landed; up to NS - 2 younger stages may still be in flight
      const int younger = min(nk - 1 - kt, NS - 2);
      if (younger >= 2) wait_loads_then_barrier<2 * L>();
      else if (younger == 1) wait_loads_then_barrier<L>();
      else wait_loads_then_barrier<0>();
      // every wave has left stage kt - 1: its buffer takes stage kt + NS - 1
      if (kt + NS - 1 < nk) issue(kt + NS - 1, (kt - kt0 + NS - 1) % NS);
      k_step((kt - kt0) % NS, [] {});
    }
    }
  }

  // ---- epilogue.  The products were issued as W_tile . A_tile^T, so acc[i][j][e] is C[m][n] with
  // m = lane % 32 (row of the 32x32 tile) and n = 8 (e / 4) + 4 (lane / 32) + e % 4: every lane holds runs of four
  // consecutive columns of one row, which makes outputs, bias and residual 16-byte accesses and turns the
  // row-wise softmax statistics of the LM head into in-register reductions.
  const int wrow0 = row0 + wm * (BM / WM), wcol0 = col0 + wn * (BN / WN);
  if constexpr (EPI == EPI_LMHEAD) {
    // per row and per 64-column group: max and sum of exp of the tempered logits; optional capture
    // of the target column's tempered logit.  Nothing of size [M, N] is written.
    static_assert(TN % 2 == 0, "a wave must own whole 64-column groups");
    const int ngroups = (g.N + 63) >> 6;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = wrow0 + i * 32 + frow;
      const int tgt = (g.target != nullptr && row < g.M) ? g.target[row] : -1;
#pragma unroll
      for (int gi = 0; gi < TN / 2; ++gi) {
        const int group = (wcol0 >> 6) + gi;
        float l[32];
        float mx = -INFINITY;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int col = wcol0 + (2 * gi + jj) * 32 + 8 * (e >> 2) + 4 * fhalf + (e & 3);
            const float v = col < g.N ? acc[i][2 * gi + jj][e] / g.temperature : -INFINITY;
            l[jj * 16 + e] = v;
            mx = fmaxf(mx, v);
            if (col == tgt) g.target_logit[row] = v;
          }
        mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
        float sum = 0.f;
#pragma unroll
        for (int e = 0; e < 32; ++e) sum += (l[e] == -INFINITY) ? 0.f : __expf(l[e] - mx);
        sum += __shfl_xor(sum, 32, WAVE);
        if (fhalf == 0 && row < g.M && group < ngroups) g.partial[(size_t)row * ngroups + group] = make_float2(mx, sum);
      }
    }
  } else {
    [[maybe_unused]] bool sat = false;        // an fp16 output was clamped
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int row = wrow0 + i * 32 + frow;
      if (row >= g.M) continue;
      // EPI_QKV: this row's rotary table row, its q and staging rows, and where its key / value start inside
      // kv head 0's stream of its cache sequence (the parts of KvLayout::k_elem / v_elem that depend on the
      // slot alone; kv heads are per_head elements apart)
      [[maybe_unused]] const float2* rope_row = nullptr;
      [[maybe_unused]] uint16_t *q_row = nullptr, *stage_row = nullptr, *k_row = nullptr, *v_row = nullptr;
      [[maybe_unused]] int per_head = 0;
      if constexpr (EPI == EPI_QKV) {
        const QkvEpi& e = g.qe;
        const int qpos = e.pos[row] + e.pos_add;
        rope_row = e.table + (size_t)qpos * (e.r >> 1);
        q_row = e.q + (size_t)row * (e.Hq * e.h) * (PR ? 2 : 1);         // precise: a row of floats
        if (e.kvstage) {
          stage_row = e.kvstage + (size_t)row * (2 * e.Hkv * e.h);
        } else {
          const int seq = e.dst_seq[row];
          const int slot = qpos - (e.slot_sub ? e.slot_sub[row] : 0);
          const int cap = e.kv_cap[seq];
          uint16_t* base = e.kv + e.lay.seq_base(e.kv_off[seq]);
          k_row = base + e.lay.k_elem(slot, 0);
          v_row = base + e.lay.v_elem(slot, 0);
          per_head = 2 * cap * e.h;
        }
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = wcol0 + j * 32 + 8 * q + 4 * fhalf;       // first of four consecutive columns
          if (col >= g.N) continue;
          const bool full = col + 3 < g.N;
          f32x4 v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[i][j][4 * q + r];
          if constexpr (EPI == EPI_PARTIAL) {
            float* p = g.ws + ((size_t)split * g.M + row) * g.N + col;
            if (full && (g.N & 3) == 0) *(f32x4*)p = v;
            else
              for (int r = 0; r < 4 && col + r < g.N; ++r) p[r] = v[r];
            continue;
          }
          if (g.bias) {
            if (full) v += *(const f32x4*)(g.bias + col);
            else
              for (int r = 0; r < 4 && col + r < g.N; ++r) v[r] += g.bias[col + r];
          }
          if constexpr (EPI == EPI_F32 || EPI == EPI_RESID) {
            float* p = (float*)g.out + (size_t)row * g.ldo + col;
            if (full && (g.ldo & 3) == 0) {
              if constexpr (EPI == EPI_RESID) v += *(const f32x4*)p;
              *(f32x4*)p = v;
            } else {
              for (int r = 0; r < 4 && col + r < g.N; ++r) p[r] = (EPI == EPI_RESID ? p[r] : 0.f) + v[r];
            }
          } else if constexpr (EPI == EPI_QKV) {
            // head dims of a group of four packed columns: a rotary group holds the pairs (d0, d0 + r/2) and
            // (d0 + 1, d0 + 1 + r/2) as (v0, v2) and (v1, v3); any other group holds four consecutive dims
            const QkvEpi& e = g.qe;
            const int head = (int)(((float)col + 0.5f) * e.inv_h);
            const int p0 = col - head * e.h;
            const bool is_v = head >= e.Hq + e.Hkv;
            int d0 = p0, d1 = p0 + 2;                         // dims of (v0, v1) and of (v2, v3)
            if (!is_v && p0 < e.r) {
              d0 = p0 >> 1;
              d1 = d0 + (e.r >> 1);
              const f32x4 cs = *(const f32x4*)(rope_row + d0);     // cos, sin of pairs d0 and d0 + 1
              const float lo0 = v[0] * cs[0] - v[2] * cs[1], hi0 = v[2] * cs[0] + v[0] * cs[1];
              const float lo1 = v[1] * cs[2] - v[3] * cs[3], hi1 = v[3] * cs[2] + v[1] * cs[3];
              v[0] = lo0; v[1] = lo1; v[2] = hi0; v[3] = hi1;
            }
            if constexpr (PR) {
              // precise mode: q stays fp32; keys and values are stored as bf16 hi/lo pairs (the lo halves a fixed
              // distance behind the hi halves)
              if (head < e.Hq) {
                float* qp = (float*)q_row + head * e.h;
                *(float2*)(qp + d0) = make_float2(v[0], v[1]);
                *(float2*)(qp + d1) = make_float2(v[2], v[3]);
              } else {
                uint32_t h01, l01, h23, l23;
                SPLIT_BF16X2(v[0], v[1], h01, l01);
                SPLIT_BF16X2(v[2], v[3], h23, l23);
                if (e.kvstage) {
                  uint16_t* sp = stage_row + (head - e.Hq) * e.h;
                  *(uint32_t*)(sp + d0) = h01;
                  *(uint32_t*)(sp + d1) = h23;
                  *(uint32_t*)(sp + e.stage_lo_off + d0) = l01;
                  *(uint32_t*)(sp + e.stage_lo_off + d1) = l23;
                } else if (!is_v) {
                  uint16_t* st = k_row + (size_t)(head - e.Hq) * per_head;
                  *(uint32_t*)(st + ((d0 >> 3) << 7) + (d0 & 7)) = h01;
                  *(uint32_t*)(st + ((d1 >> 3) << 7) + (d1 & 7)) = h23;
                  *(uint32_t*)(st + e.kv_lo_off + ((d0 >> 3) << 7) + (d0 & 7)) = l01;
                  *(uint32_t*)(st + e.kv_lo_off + ((d1 >> 3) << 7) + (d1 & 7)) = l23;
                } else {
                  uint16_t* st = v_row + (size_t)(head - e.Hq - e.Hkv) * per_head + ((p0 >> 4) << 9) + ((p0 & 15) << 3);
                  st[0] = (uint16_t)h01; st[8] = (uint16_t)(h01 >> 16); st[16] = (uint16_t)h23; st[24] = (uint16_t)(h23 >> 16);
                  st += e.kv_lo_off;
                  st[0] = (uint16_t)l01; st[8] = (uint16_t)(l01 >> 16); st[16] = (uint16_t)l23; st[24] = (uint16_t)(l23 >> 16);
                }
              }
            } else {
            // q is fp16; cached keys and values are bf16 but enter the attention products as fp16
#pragma unroll
            for (int r = 0; r < 4; ++r) sat |= f16_out_of_range(v[r]);
            if (head < e.Hq) {
              uint16_t* qp = q_row + head * e.h;
              *(uint32_t*)(qp + d0) = pack_f16x2(v[0], v[1]);
              *(uint32_t*)(qp + d1) = pack_f16x2(v[2], v[3]);
            } else if (e.kvstage) {
              // prompt pass: keys (rotated) and values as bf16 rows [k heads | v heads]; a second kernel moves them
              // into the cache layout, to every copy, in 16-byte units
              uint16_t* sp = stage_row + (head - e.Hq) * e.h;
              *(uint32_t*)(sp + d0) = pack_bf16x2(v[0], v[1]);
              *(uint32_t*)(sp + d1) = pack_bf16x2(v[2], v[3]);
            } else if (!is_v) {
              uint16_t* st = k_row + (size_t)(head - e.Hq) * per_head;
              *(uint32_t*)(st + ((d0 >> 3) << 7) + (d0 & 7)) = pack_bf16x2(v[0], v[1]);
              *(uint32_t*)(st + ((d1 >> 3) << 7) + (d1 & 7)) = pack_bf16x2(v[2], v[3]);
            } else {
              uint16_t* st = v_row + (size_t)(head - e.Hq - e.Hkv) * per_head + ((p0 >> 4) << 9) + ((p0 & 15) << 3);
#pragma unroll
              for (int r = 0; r < 4; ++r) st[r << 3] = f32_to_bf16_bits(v[r]);
            }
            }
          } else if constexpr (EPI == EPI_GELU_F16) {
            uint16_t* p = (uint16_t*)g.out + kblk_off(row, col, g.M);     // four columns never straddle a K block
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              v[r] = gelu_erf(v[r]);
              if constexpr (!PR) sat |= f16_out_of_range(v[r]) && col + r < g.N;
            }
            if constexpr (PR) {
              u32x2 wh, wl;
              SPLIT_BF16X2(v[0], v[1], wh[0], wl[0]);
              SPLIT_BF16X2(v[2], v[3], wh[1], wl[1]);
              if (full) {
                *(u32x2*)p = wh;
                *(u32x2*)(p + g.out_lo_off) = wl;
              } else {
                for (int r = 0; r < 4 && col + r < g.N; ++r) {
                  p[r] = (uint16_t)(wh[r >> 1] >> (16 * (r & 1)));
                  p[g.out_lo_off + r] = (uint16_t)(wl[r >> 1] >> (16 * (r & 1)));
                }
              }
            } else if (full) {
              u32x2 w;
              w[0] = pack_f16x2(v[0], v[1]);
              w[1] = pack_f16x2(v[2], v[3]);
              *(u32x2*)p = w;
            } else {
              for (int r = 0; r < 4 && col + r < g.N; ++r) p[r] = f32_to_f16_bits(v[r]);
            }
          } else if constexpr (EPI == EPI_SWIGLU_F16) {
            // weight rows come in blocks of 32: block 2b = gate rows [32b, 32b+32), block 2b+1 = the
            // matching up rows, so tile j (even) and tile j+1 hold gate and up of the same features.
            static_assert(TN % 2 == 0, "a wave must own gate and up of the same features");
            if ((j & 1) == 0) {
              const int f = ((wcol0 + j * 32) >> 1) + 8 * q + 4 * fhalf;
              u32x2 w;
              const int ju = j + 1 < TN ? j + 1 : j;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                v[r] = silu(v[r]) * acc[i][ju][4 * q + r];
                if constexpr (!PR) sat |= f16_out_of_range(v[r]);
              }
              uint16_t* p = (uint16_t*)g.out + kblk_off(row, f, g.M);
              if constexpr (PR) {
                u32x2 wl;
                SPLIT_BF16X2(v[0], v[1], w[0], wl[0]);
                SPLIT_BF16X2(v[2], v[3], w[1], wl[1]);
                *(u32x2*)(p + g.out_lo_off) = wl;
              } else {
                w[0] = pack_f16x2(v[0], v[1]);
                w[1] = pack_f16x2(v[2], v[3]);
              }
              *(u32x2*)p = w;
            }
          }
        }
      }
    }
    if constexpr (EPI == EPI_QKV || EPI == EPI_GELU_F16 || EPI == EPI_SWIGLU_F16) flag_f16_range(sat, g.status);
  }
}

// Second half of a split-K product: sums the partial results in split order (so the result does not depend
// on scheduling) and applies the epilogue.
template <int EPI>
__global__ void splitk_epilogue_kernel(GemmArgs g) {
  const size_t n = (size_t)g.M * g.N;
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int row = (int)(i / g.N), col = (int)(i % g.N);
  float v = 0.f;
  for (int sp = 0; sp < g.splits; ++sp) v += g.ws[(size_t)sp * n + i];
  if (g.bias) v += g.bias[col];
  if constexpr (EPI == EPI_F32) {
    ((float*)g.out)[(size_t)row * g.ldo + col] = v;
  } else if constexpr (EPI == EPI_RESID) {
    float* p = (float*)g.out + (size_t)row * g.ldo + col;
    *p = *p + v;
  } else if constexpr (EPI == EPI_GELU_F16) {
    v = gelu_erf(v);
    uint16_t* p = (uint16_t*)g.out + kblk_off(row, col, g.M);
    if (g.precise) {
      split_bf16(v, p[0], p[g.out_lo_off]);
    } else {
      flag_f16_range(f16_out_of_range(v), g.status);
      *p = f32_to_f16_bits(v);
    }
  }
}

template <int BM, int BN, int WM, int WN, int EPI, bool KTAIL, int NS = 0, bool PR = false>
hipError_t launch_k(const GemmArgs& g, hipStream_t s) {
  constexpr size_t lds_bytes = (NS ? NS : 2) * (size_t)(BM + BN) * BK * sizeof(uint16_t);
  static_assert(lds_bytes <= 160 * 1024, "LDS of one CU");
  // once per device and instantiation (a repeated call is harmless, so no lock)
  static bool configured_on[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  bool& configured = configured_on[dev];
  if (!configured) {
    if (lds_bytes > 65536) {
      hipError_t e = hipFuncSetAttribute((const void*)gemm_f16_kernel<BM, BN, WM, WN, EPI, KTAIL, NS, PR>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
      if (e != hipSuccess) return e;
    }
    configured = true;
  }
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * (EPI == EPI_PARTIAL ? g.splits : 1);
  hipLaunchKernelGGL((gemm_f16_kernel<BM, BN, WM, WN, EPI, KTAIL, NS, PR>), dim3(tiles), dim3(WM * WN * 64), lds_bytes, s, g);
  return hipGetLastError();
}

// Whole K tiles take the direct-load pipeline with two LDS stages (more stages measured slower: the extra LDS
// costs a resident block); a ragged K falls back to register staging, which can zero-fill the tail.
template <int BM, int BN, int WM, int WN, int EPI, int NS = 2, bool PR = false>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
  return g.K % BK == 0 ? launch_k<BM, BN, WM, WN, EPI, false, NS, PR>(g, s) : launch_k<BM, BN, WM, WN, EPI, true, 0, PR>(g, s);
}

// precise mode is compiled for four of the tile shapes (128x128, 256x256, 256x128 with 8 waves, 64x128)
template <int EPI>
hipError_t launch_variant_precise(const GemmArgs& g, int variant, hipStream_t s) {
  switch (variant) {
    case 0: return launch<128, 128, 2, 2, EPI, 2, true>(g, s);
    case 3: return launch<256, 256, 4, 2, EPI, 2, true>(g, s);
    case 5: return launch<256, 128, 4, 2, EPI, 2, true>(g, s);
    case 7:
      if constexpr (EPI != EPI_SWIGLU_F16 && EPI != EPI_LMHEAD) return launch<64, 128, 1, 4, EPI, 2, true>(g, s);
      else return hipErrorInvalidValue;
  }
  return hipErrorInvalidValue;
}

template <int EPI>
hipError_t launch_variant(const GemmArgs& g, int variant, hipStream_t s) {
  if (g.precise) return launch_variant_precise<EPI>(g, variant, s);
  switch (variant) {
    case 0: return launch<128, 128, 2, 2, EPI>(g, s);
    case 1: return launch<256, 128, 2, 2, EPI>(g, s);
    case 2: return launch<256, 256, 2, 2, EPI>(g, s);
    case 3: return launch<256, 256, 4, 2, EPI>(g, s);
    case 4: return launch<128, 256, 2, 2, EPI>(g, s);
    case 5: return launch<256, 128, 4, 2, EPI>(g, s);
    case 6:
      if constexpr (EPI != EPI_SWIGLU_F16 && EPI != EPI_LMHEAD) return launch<128, 64, 2, 2, EPI>(g, s);
      else return hipErrorInvalidValue;
    case 7:
      if constexpr (EPI != EPI_SWIGLU_F16 && EPI != EPI_LMHEAD) return launch<64, 128, 1, 4, EPI>(g, s);
      else return hipErrorInvalidValue;
    case 8:      // the smallest tile with four LDS stages: loads three K steps ahead, for launches with few blocks per CU
      if constexpr (EPI != EPI_SWIGLU_F16 && EPI != EPI_LMHEAD) return launch<64, 128, 1, 4, EPI, 4>(g, s);
      else return hipErrorInvalidValue;
    case 9:      // the same tile and ring on eight waves of 32x32: two waves per SIMD cover each other's waits for LDS
                 // fragments and for the stage barrier (12-15 % faster than four waves on long-K shapes with few tiles)
      if constexpr (EPI != EPI_SWIGLU_F16 && EPI != EPI_LMHEAD) return launch<64, 128, 2, 4, EPI, 4>(g, s);
      else return hipErrorInvalidValue;
    case 10:     // the largest tile on sixteen waves of 64x64: four waves per SIMD hide more of each other's waits than two,
                 // for a third more LDS fragment traffic (a ragged K takes the eight-wave form: its register staging does
                 // not fit 128 registers per lane)
      return g.K % BK == 0 ? launch_k<256, 256, 4, 4, EPI, false, 2, false>(g, s) : launch_k<256, 256, 4, 2, EPI, true, 0, false>(g, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace

hipError_t rl_gemm_variant(const GemmArgs& g, int epi, int variant, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K % 8 != 0) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_F32: return launch_variant<EPI_F32>(g, variant, s);
    case EPI_RESID: return launch_variant<EPI_RESID>(g, variant, s);
    case EPI_GELU_F16: return launch_variant<EPI_GELU_F16>(g, variant, s);
    case EPI_SWIGLU_F16:
      if (g.N % 64 != 0) return hipErrorInvalidValue;
      return launch_variant<EPI_SWIGLU_F16>(g, variant, s);
    case EPI_LMHEAD: return launch_variant<EPI_LMHEAD>(g, variant, s);
    case EPI_PARTIAL: return launch_variant<EPI_PARTIAL>(g, variant, s);
    case EPI_QKV: {
      const QkvEpi& e = g.qe;
      if (e.r % 4 != 0 || e.h % 16 != 0 || g.N != (e.Hq + 2 * e.Hkv) * e.h || !e.q || !e.pos || (e.r > 0 && !e.table) ||
          (!e.kvstage && (!e.kv || !e.dst_seq || !e.kv_off || !e.kv_cap)))
        return hipErrorInvalidValue;
      return launch_variant<EPI_QKV>(g, variant, s);
    }
  }
  return hipErrorInvalidValue;
}

// Split-K: `splits` blocks per tile each take a share of K and write fp32 partial tiles to g.ws
// ([splits, M, N]); a second kernel adds them in order and applies the epilogue.
hipError_t rl_gemm_splitk(const GemmArgs& g, int epi, int variant, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.splits < 2 || !g.ws || (epi != EPI_F32 && epi != EPI_RESID && epi != EPI_GELU_F16)) return hipErrorInvalidValue;
  if ((size_t)g.splits * g.M * g.N > g.ws_elems) return hipErrorInvalidValue;      // the partial sums must fit
  hipError_t e = rl_gemm_variant(g, EPI_PARTIAL, variant, s);
  if (e != hipSuccess) return e;
  const size_t n = (size_t)g.M * g.N;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (epi == EPI_F32) hipLaunchKernelGGL(splitk_epilogue_kernel<EPI_F32>, grid, block, 0, s, g);
  else if (epi == EPI_RESID) hipLaunchKernelGGL(splitk_epilogue_kernel<EPI_RESID>, grid, block, 0, s, g);
  else hipLaunchKernelGGL(splitk_epilogue_kernel<EPI_GELU_F16>, grid, block, 0, s, g);
  return hipGetLastError();
}

// Tile shape by problem size (measured on MI355X): the largest tile that still gives every CU work.  The K split is
// the caller's (g.splits >= 2 with g.ws set), never chosen here: it fixes the order of the sums.
hipError_t rl_gemm(const GemmArgs& g, int epi, hipStream_t s) {
  auto tiles = [&](int bm, int bn) { return (long long)((g.M + bm - 1) / bm) * ((g.N + bn - 1) / bn); };
  const bool wide_only = (epi == EPI_SWIGLU_F16 || epi == EPI_LMHEAD);   // a wave must own 64 columns
  int variant;
  if (tiles(256, 256) >= 160) variant = 3;
  else if (tiles(256, 128) >= 200) variant = 5;
  else if (tiles(128, 128) >= 400 || wide_only) variant = 0;
  else variant = 7;
  if (g.splits >= 2 && g.ws) return rl_gemm_splitk(g, epi, wide_only ? 0 : 7, s);
  return rl_gemm_variant(g, epi, variant, s);
}
