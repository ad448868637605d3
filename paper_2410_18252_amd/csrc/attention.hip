// Softmax attention over the per-sequence bf16 KV cache, for the decode step (one query per
// sequence and query head: the bandwidth-bound part of generation) and for causal prefill.
//
// One wave owns 16 "columns" (queries) and streams one (sequence, kv head) K/V stream in
// super-blocks of 32 keys.  The matrix cores serve as dot-product engines fed straight from global
// memory: no LDS, no cross-lane reduction over head_dim.
//   S^T[key, col] = sum_d K[key, d] q[col, d]       2 x ceil(h/32) MFMA 16x16x32 per super-block
//   O^T[d, col]  += sum_key V^T[d, key] P^T[key, col]   h/16 MFMA 16x16x32 per super-block
// K and V are stored as bf16 and widened to fp16 in registers (exact for every value in fp16's
// normal range); queries, probabilities and the MFMAs are fp16 with fp32 accumulation.
// The cache is read once and never again within a launch, so its loads are non-temporal (measured:
// +7 % bandwidth), and the next super-block is requested before the current one is consumed.
// The cache layout (see KvLayout) makes every operand fragment one 16-byte load per lane and every
// load instruction one contiguous kilobyte per wave.  The K rows of a super-block are assigned to
// MFMA rows so that the score registers of lane group g (keys 8g..8g+7) are exactly the B-operand
// fragment P^T the second product needs: probabilities never leave registers.
// Decode with one kv head serving G query heads (grouped-query attention) puts the G heads in the
// columns, so K/V are read once per group; with G = 1 the query is replicated over the columns.
// With a shared prompt cache (share_k = K samples per prompt) the K samples sit in the columns as well:
// the prompt's stream is read once for all of them, then each sample's short stream of new tokens.
// Precise mode (PR): every operand is a bf16 hi/lo pair -- the cache holds a second plane with the lo halves, the
// queries arrive as fp32 and are split in registers, the probabilities are split after the softmax -- and each product
// is three bf16 matrix instructions (hi hi + lo hi + hi lo; the lo lo term is below fp32's own rounding).
#include "kernels.h"

#ifndef ATTN_PREFETCH
#define ATTN_PREFETCH 1
#endif
#ifndef ATTN_PREFETCH2
#define ATTN_PREFETCH2 1
#endif
// The prompt pass is not bound by memory but by the latency of a wave's serial chain (load, convert, MFMA, softmax,
// MFMA): it is compiled for at least ATTN_PROMPT_BLOCKS blocks per CU (256 registers), and without the register
// prefetch of the next super-block it needs 162 registers at head size 80, so three waves share a SIMD and hide
// each other's L2 latency (measured on the 2.8B shape: 596 -> 345 us with two blocks, -> 312 us without the prefetch).
#ifndef ATTN_PROMPT_NOPF
#define ATTN_PROMPT_NOPF 1
#endif
#ifndef ATTN_PROMPT_BLOCKS
#define ATTN_PROMPT_BLOCKS 2
#endif
#ifndef ATTN_NT
#define ATTN_NT 1
#endif
#if ATTN_NT
#define ATTN_LOAD(p) __builtin_nontemporal_load(p)
#else
#define ATTN_LOAD(p) (*(p))
#endif

namespace {

// QB = query blocks of 16 columns a wave carries through one pass over the keys (prompt pass only: two blocks halve
// the key / value traffic per query; a.jobs then counts blocks of 16 QB tokens).
template <int HD, bool DECODE, int QB = 1, bool PR = false>
__global__ __launch_bounds__(256, (!DECODE && HD <= 128 && !PR) ? ATTN_PROMPT_BLOCKS : 1) void attention_kernel(AttnArgs a) {
  static_assert(!DECODE || QB == 1, "decode has one query block");
  constexpr int NCH = HD / 8;            // 16-byte chunks per key row
  constexpr int KSTEPS = (HD + 31) / 32; // MFMA steps over head_dim for the scores
  constexpr int VT = HD / 16;            // 16-row tiles of V^T / O^T
  // is the next super-block requested one iteration ahead (precise mode holds two planes per super-block in registers
  // and loads them at the top of the iteration instead)
  constexpr bool PF = (DECODE || !ATTN_PROMPT_NOPF) && !PR;
  constexpr int NP = PR ? 2 : 1;         // cache planes: hi, lo
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int c = lane & 15, g = lane >> 4;
  const int Hkv = a.lay.Hkv, G = a.Hq / Hkv;
  const int job = blockIdx.x * 4 + wave;

  // A job streams one or more segments.  Segment i is the stream of cache sequence seg_seq(i) with seg_len(i)
  // keys; column c takes part in it if seg_col(i) < 0 or seg_col(i) == c / G (its sample).
  int kvh, qrow[QB], qhead, qpos[QB], nseg;
  int seq0, len0;           // first segment
  int sfx_seq0 = 0, sfx_len = 0;   // shared-prompt decode: segments 1.. are the samples' own suffix streams
  bool store_col[QB];
  if constexpr (DECODE) {
    const int units = a.share_k ? a.S / a.share_k : a.S;       // prompts or sequences
    if (job >= units * Hkv) return;
    const int slot = job / Hkv;
    kvh = job - slot * Hkv;
    const int u = a.order ? a.order[slot] : slot;     // longest contexts first: the tail of the launch is short jobs
    if (a.share_k) {
      // the K samples of prompt u sit in the MFMA columns (next to the G query heads of the kv head): the
      // prompt's keys and values are read once for all of them, then each sample's own new tokens
      const int j = (c / G) % a.share_k;
      if (a.finished) {           // nothing to do once every sample of the prompt has ended
        bool live = false;
        for (int jj = 0; jj < a.share_k; ++jj) live |= a.finished[u * a.share_k + jj] == 0;
        if (!live) return;
      }
      qrow[0] = u * a.share_k + j;
      seq0 = u;
      len0 = a.ctx_base[u * a.share_k];
      sfx_seq0 = a.sfx_first + u * a.share_k;
      sfx_len = a.ctx_add;
      nseg = 1 + a.share_k;
      store_col[0] = c < G * a.share_k;
    } else {
      if (a.finished && a.finished[u]) return;      // an ended completion's output is never used: do not stream its cache
      qrow[0] = u;
      seq0 = a.cache_seq_of ? a.cache_seq_of[u] : u;       // rows of a compacted batch name their cache sequence
      len0 = a.ctx_base[u] + a.ctx_add;
      nseg = 1;
      store_col[0] = c < G;
    }
    qhead = kvh * G + (c % G);
    qpos[0] = 0x7fffffff;      // a decode query sees every key of its segments
  } else {
    // a.jobs lists blocks of 16 tokens, QB consecutive ones (of one sequence, the first a multiple of QB) per wave
    if (job >= a.njobs / QB * a.Hq) return;
    AttnJob jb = a.jobs[job / a.Hq * QB];
    jb.qblock /= QB;
    qhead = job % a.Hq;
    kvh = qhead / G;
    seq0 = jb.cache_seq;
#pragma unroll
    for (int b = 0; b < QB; ++b) {
      const int tok = (jb.qblock * QB + b) * 16 + c;
      store_col[b] = tok < jb.len;
      qpos[b] = min(tok, jb.len - 1);
      qrow[b] = jb.row0 + qpos[b];
    }
    len0 = min((jb.qblock + 1) * 16 * QB, jb.len);      // keys the last query of the job sees
    nseg = jb.pre_len > 0 ? 2 : 1;                      // a shared prefix is walked first
    sfx_seq0 = jb.pre_seq;
    sfx_len = jb.pre_len;
  }

  // query fragments (B operand): lane (c, g) holds q[col c][32 i + 8 g .. + 7]
  f16x8 qf[QB][KSTEPS];
  [[maybe_unused]] u32x4 qlo[QB][KSTEPS];          // precise mode: qf holds the bf16 hi halves (as bits), qlo the lo halves
#pragma unroll
  for (int b = 0; b < QB; ++b) {
    const uint16_t* qp = a.q + ((size_t)qrow[b] * a.q_ld + qhead * HD) * (PR ? 2 : 1);
#pragma unroll
    for (int i = 0; i < KSTEPS; ++i) {
      const int d0 = 32 * i + 8 * g;
      if constexpr (PR) {
        u32x4 hi = u32x4{0, 0, 0, 0}, lo = u32x4{0, 0, 0, 0};
        if (d0 < HD) {
          const f32x4 x0 = *(const f32x4*)((const float*)qp + d0), x1 = *(const f32x4*)((const float*)qp + d0 + 4);
          SPLIT_BF16X2(x0[0], x0[1], hi[0], lo[0]);
          SPLIT_BF16X2(x0[2], x0[3], hi[1], lo[1]);
          SPLIT_BF16X2(x1[0], x1[1], hi[2], lo[2]);
          SPLIT_BF16X2(x1[2], x1[3], hi[3], lo[3]);
        }
        qf[b][i] = __builtin_bit_cast(f16x8, hi);
        qlo[b][i] = lo;
      } else {
      if (d0 < HD) qf[b][i] = *(const f16x8*)(qp + d0);
      else
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[b][i][e] = (f16_t)0.f;
      }
    }
  }
  // one 16x16x32 matrix instruction on 16-bit fragments: fp16, or bf16 in precise mode
  auto mfma = [](f16x8 x, f16x8 y, f32x4 acc) {
    if constexpr (PR) return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x), __builtin_bit_cast(bf16x8, y), acc, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_f16(x, y, acc, 0, 0, 0);
  };

  f32x4 o[QB][VT];
  float m[QB], lsum[QB];
#pragma unroll
  for (int b = 0; b < QB; ++b) {
#pragma unroll
    for (int t = 0; t < VT; ++t) o[b][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    m[b] = -INFINITY;
    lsum[b] = 0.f;
  }

  for (int seg = 0; seg < nseg; ++seg) {
    if (seg > 0 && a.finished && a.finished[qrow[0] - (c / G) % a.share_k + seg - 1]) continue;     // ended sample: skip its stream
    // prompt pass with a shared prefix: segment 0 is the prefix (every key visible), segment 1 the sequence itself
    const bool prefix_seg = !DECODE && nseg == 2 && seg == 0;
    const int cache_seq = DECODE ? (seg == 0 ? seq0 : sfx_seq0 + seg - 1) : (prefix_seg ? sfx_seq0 : seq0);
    const int nkeys = DECODE ? (seg == 0 ? len0 : sfx_len) : (prefix_seg ? sfx_len : len0);
    const bool mine = !DECODE || seg == 0 || (c / G) % a.share_k == seg - 1;     // does column c attend to this segment
    const int cap = a.kv_cap[cache_seq];
    const long long off = a.kv_off[cache_seq];
    const uint16_t* __restrict__ st = a.kv + a.lay.stream(off, cap, kvh);
    int klimit[QB];                                                     // last visible key index for this column
#pragma unroll
    for (int b = 0; b < QB; ++b) klimit[b] = !mine ? -1 : prefix_seg ? nkeys - 1 : min(nkeys - 1, qpos[b]);

  const int nsb = (nkeys + 31) >> 5;
  // the whole next super-block (32 keys, 32 values) is requested before the current one is consumed
  auto load_sb = [&](int sb, u32x4 (&kraw)[2][KSTEPS], u32x4 (&vraw)[VT], int plane = 0) {
    const uint16_t* kb = st + (size_t)sb * 64 * HD + (plane ? a.kv_lo_off : 0);      // 32 keys, then the 32 values of the same positions
    const uint16_t* vb = kb + 32 * HD;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i) {
        const int chunk = 4 * i + g;
        kraw[t][i] = chunk < NCH ? ATTN_LOAD((const u32x4*)(kb + (((t * NCH + chunk) * 16 + c) << 3))) : u32x4{0, 0, 0, 0};
      }
#pragma unroll
    for (int t = 0; t < VT; ++t) vraw[t] = ATTN_LOAD((const u32x4*)(vb + ((((t * 4 + g) * 16) + c) << 3)));
  };
  u32x4 kraw[2][KSTEPS], vraw[VT];
  [[maybe_unused]] u32x4 kraw_lo[NP - 1 ? 2 : 1][KSTEPS], vraw_lo[VT];
#if ATTN_PREFETCH
  u32x4 knext[2][KSTEPS], vnext[VT];
  if (PF && nsb > 0) load_sb(0, kraw, vraw);
#endif
#if ATTN_PREFETCH2
  // decode: a second super-block in flight (the kernel is bound by bytes in flight, and registers allow it)
  u32x4 knext2[2][KSTEPS], vnext2[VT];
  // measured: head size 128 gains 4 % from it, head sizes 64 and 80 lose (fewer waves fit), 256 would spill
  constexpr bool P2 = DECODE && HD > 96 && HD <= 128 && !PR;
  if (P2 && nsb > 1) load_sb(1, knext, vnext);
#endif
  for (int sb = 0; sb < nsb; ++sb) {
#if ATTN_PREFETCH2
    if (P2) {
      if (sb + 2 < nsb) load_sb(sb + 2, knext2, vnext2);
    } else if (PF) { if (sb + 1 < nsb) load_sb(sb + 1, knext, vnext); }
    else {
      load_sb(sb, kraw, vraw);
      if constexpr (PR) load_sb(sb, kraw_lo, vraw_lo, 1);
    }
#elif ATTN_PREFETCH
    if (sb + 1 < nsb) load_sb(sb + 1, knext, vnext);
#else
    load_sb(sb, kraw, vraw);
#endif

    // the super-block's operands are widened once and serve every query block
    f16x8 kf[2][KSTEPS], vf[VT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i) kf[t][i] = PR ? __builtin_bit_cast(f16x8, kraw[t][i]) : bf16x8_to_f16x8(kraw[t][i]);
#pragma unroll
    for (int t = 0; t < VT; ++t) vf[t] = PR ? __builtin_bit_cast(f16x8, vraw[t]) : bf16x8_to_f16x8(vraw[t]);
    // straight-line code over the query blocks: their chains (MFMA -> softmax -> MFMA) are independent, and the
    // scheduler interleaves them only if no branch separates them
    f32x4 sc[QB][2];
#pragma unroll
    for (int b = 0; b < QB; ++b)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        sc[b][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < KSTEPS; ++i) {
          sc[b][t] = mfma(kf[t][i], qf[b][i], sc[b][t]);
          if constexpr (PR) {
            sc[b][t] = mfma(__builtin_bit_cast(f16x8, kraw_lo[t][i]), qf[b][i], sc[b][t]);
            sc[b][t] = mfma(kf[t][i], __builtin_bit_cast(f16x8, qlo[b][i]), sc[b][t]);
          }
        }
      }
    // lane (c, g) now holds the scores of keys 32 sb + 8 g + 4 t + j against column c
    float p[QB][8], alpha[QB];
#pragma unroll
    for (int b = 0; b < QB; ++b) {
      float bmax = -INFINITY;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int key = sb * 32 + 8 * g + 4 * t + j;
          const float v = key <= klimit[b] ? sc[b][t][j] * a.scale : -INFINITY;
          p[b][4 * t + j] = v;
          bmax = fmaxf(bmax, v);
        }
      bmax = fmaxf(bmax, __shfl_xor(bmax, 16, WAVE));
      bmax = fmaxf(bmax, __shfl_xor(bmax, 32, WAVE));
      const float mnew = fmaxf(m[b], bmax);
      // a column that has seen no key yet (m and mnew both -inf) keeps alpha = 1 and p = 0
      alpha[b] = mnew == -INFINITY ? 1.f : __expf(m[b] - mnew);
      m[b] = mnew;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        p[b][e] = mnew == -INFINITY ? 0.f : __expf(p[b][e] - mnew);
        psum += p[b][e];
      }
      lsum[b] = lsum[b] * alpha[b] + psum;
    }
#pragma unroll
    for (int b = 0; b < QB; ++b) {
      f16x8 pf;
      [[maybe_unused]] u32x4 plo;
      if constexpr (PR) {
        u32x4 phi;
#pragma unroll
        for (int e = 0; e < 4; ++e) SPLIT_BF16X2(p[b][2 * e], p[b][2 * e + 1], phi[e], plo[e]);
        pf = __builtin_bit_cast(f16x8, phi);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[e] = (f16_t)p[b][e];
      }
#pragma unroll
      for (int t = 0; t < VT; ++t) {
        o[b][t] *= alpha[b];
        o[b][t] = mfma(vf[t], pf, o[b][t]);
        if constexpr (PR) {
          o[b][t] = mfma(__builtin_bit_cast(f16x8, vraw_lo[t]), pf, o[b][t]);
          o[b][t] = mfma(vf[t], __builtin_bit_cast(f16x8, plo), o[b][t]);
        }
      }
    }
#if ATTN_PREFETCH
    if (PF) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < KSTEPS; ++i) kraw[t][i] = knext[t][i];
#pragma unroll
    for (int t = 0; t < VT; ++t) vraw[t] = vnext[t];
    }
#endif
#if ATTN_PREFETCH2
    if (P2) {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < KSTEPS; ++i) knext[t][i] = knext2[t][i];
#pragma unroll
      for (int t = 0; t < VT; ++t) vnext[t] = vnext2[t];
    }
#endif
  }
  }   // segments
#pragma unroll
  for (int b = 0; b < QB; ++b) {
    float ls = lsum[b];
    ls += __shfl_xor(ls, 16, WAVE);
    ls += __shfl_xor(ls, 32, WAVE);
    const float inv = 1.0f / ls;
    if (store_col[b]) {
#pragma unroll
      for (int t = 0; t < VT; ++t) {
        u32x2 w;
        uint16_t* dst = a.out + kblk_off(qrow[b], qhead * HD + 16 * t + 4 * g, a.out_rows);
        if constexpr (PR) {
          u32x2 wl;
          SPLIT_BF16X2(o[b][t][0] * inv, o[b][t][1] * inv, w[0], wl[0]);
          SPLIT_BF16X2(o[b][t][2] * inv, o[b][t][3] * inv, w[1], wl[1]);
          *(u32x2*)(dst + a.out_lo_off) = wl;
        } else {
          w[0] = pack_f16x2(o[b][t][0] * inv, o[b][t][1] * inv);
          w[1] = pack_f16x2(o[b][t][2] * inv, o[b][t][3] * inv);
        }
        *(u32x2*)dst = w;
      }
    }
  }
}

template <bool DECODE, int QB>
hipError_t dispatch(const AttnArgs& a, int jobs, hipStream_t s) {
  if (jobs <= 0) return hipSuccess;
  dim3 grid((jobs + 3) / 4), block(256);
  if (a.precise) {
    switch (a.lay.h) {
#define CASE(H) case H: hipLaunchKernelGGL((attention_kernel<H, DECODE, (QB > 1 && H > 80) ? 1 : QB, true>), grid, block, 0, s, a); break;
      CASE(16) CASE(32) CASE(48) CASE(64) CASE(80) CASE(96) CASE(112) CASE(128)
#undef CASE
      default: return hipErrorInvalidValue;     // head size 256 would not fit the register file with two planes
    }
    return hipGetLastError();
  }
  switch (a.lay.h) {
#define CASE(H) case H: hipLaunchKernelGGL((attention_kernel<H, DECODE, (QB > 1 && H > 80) ? 1 : QB>), grid, block, 0, s, a); break;
    CASE(16) CASE(32) CASE(48) CASE(64) CASE(80) CASE(96) CASE(112) CASE(128) CASE(256)
#undef CASE
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t rl_attention_decode(const AttnArgs& a, hipStream_t s) {
  if (a.share_k && (a.S % a.share_k != 0 || a.share_k * (a.Hq / a.lay.Hkv) > 16)) return hipErrorInvalidValue;
  return dispatch<true, 1>(a, (a.share_k ? a.S / a.share_k : a.S) * a.lay.Hkv, s);
}
// a.jobs: 16-token blocks; every sequence must contribute a multiple of rl_attention_prefill_qb(h) of them (blocks
// past its end are allowed), since a wave takes that many consecutive blocks
int rl_attention_prefill_qb(int h) { return h <= 80 ? 2 : 1; }
hipError_t rl_attention_prefill(const AttnArgs& a, hipStream_t s) {
  const int qb = rl_attention_prefill_qb(a.lay.h);
  if (a.njobs % qb != 0) return hipErrorInvalidValue;
  return dispatch<false, 2>(a, a.njobs / qb * a.Hq, s);
}
