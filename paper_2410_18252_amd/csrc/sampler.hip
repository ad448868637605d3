// Second phase of the fused LM-head sampler and scorer.  The LM-head GEMM (EPI_LMHEAD) leaves, per
// row and per group of 64 vocabulary columns, the max and the sum of exp of the tempered logits --
// never the logits or the probabilities.  Here one wave per row combines them into log Z, walks
// the group sums in ascending vocabulary order (fp64) to find the group in which the CDF crosses
// u, recomputes that group's 64 logits and finishes the scan inside it (one column per lane).
#include "kernels.h"

namespace {

__device__ __forceinline__ double wave_incl_scan(double v, int lane) {
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double t = __shfl_up(v, o, WAVE);
    if (lane >= o) v += t;
  }
  return v;
}

// log Z of one row from its partials; also returns the reference max M.  All lanes get the result.
__device__ __forceinline__ void row_logz(const float2* p, int ngroups, int lane, float& M, double& Z) {
  float mx = -INFINITY;
  for (int g = lane; g < ngroups; g += 64) mx = fmaxf(mx, p[g].x);
  M = wave_max(mx);
  double z = 0.0;
  const int per = (ngroups + 63) / 64;
  const int g0 = lane * per, g1 = min(g0 + per, ngroups);
  for (int g = g0; g < g1; ++g) z += (double)(p[g].y * __expf(p[g].x - M));
  Z = wave_incl_scan(z, lane);   // inclusive prefix; lane 63 holds the total
}

__global__ __launch_bounds__(256) void sample_kernel(SampleArgs a) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.R) return;
  const size_t idx = (size_t)(a.io_index ? a.io_index[row] : row) * a.io_stride + a.io_add;
  if (a.finished && a.finished[row]) {            // the completion ended at an earlier step
    if (lane == 0) {
      a.tokens[idx] = a.eos;
      a.logprobs[idx] = 0.f;
      if (a.next_token) a.next_token[row] = a.eos;
    }
    return;
  }
  float u = a.greedy ? 0.f : a.uniforms[idx];
  if (!(u >= 0.f && u < 1.f)) {
    if (lane == 0) atomicOr(a.status, RLGEN_FAULT_UNIFORM);
    u = (u >= 1.f) ? 0.99999994f : 0.f;
  }
  int forced = a.forced ? a.forced[idx] : -1;
  if (forced >= a.vocab) {
    if (lane == 0) atomicOr(a.status, RLGEN_FAULT_TOKEN);
    forced = a.vocab - 1;
  }
  const float2* p = a.partial + (size_t)row * a.ngroups;
  float M;
  double incl;
  row_logz(p, a.ngroups, lane, M, incl);
  const double Z = __shfl(incl, 63, WAVE);
  const double logZ = (double)M + log(Z);
  const double target = (double)u * Z;

  // locate the group: lanes own contiguous runs of groups, in ascending order
  const int per = (a.ngroups + 63) / 64;
  const int g0 = lane * per, g1 = min(g0 + per, a.ngroups);
  double run = incl;
  {
    double own = 0.0;
    for (int g = g0; g < g1; ++g) own += (double)(p[g].y * __expf(p[g].x - M));
    run = incl - own;   // exclusive prefix of this lane
  }
  int gsel = 0x7fffffff;
  double base = 0.0;
  {
    double r = run;
    for (int g = g0; g < g1; ++g) {
      const double w = (double)(p[g].y * __expf(p[g].x - M));
      if (r + w > target && gsel == 0x7fffffff) {
        gsel = g;
        base = r;
      }
      r += w;
    }
  }
  int gmin = gsel;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) gmin = min(gmin, __shfl_xor(gmin, o, WAVE));
  if (gmin == 0x7fffffff) gmin = a.ngroups - 1;                 // cannot happen for u < 1; stay in bounds
  const int owner = min(gmin / per, 63);
  base = __shfl(gsel == gmin ? base : run, owner, WAVE);
  if (a.greedy) {
    // the first group that holds the largest logit: M is the largest group maximum
    int gbest = 0x7fffffff;
    for (int g = g0; g < g1; ++g)
      if (p[g].x == M) { gbest = g; break; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) gbest = min(gbest, __shfl_xor(gbest, o, WAVE));
    gmin = gbest == 0x7fffffff ? 0 : gbest;
  }
  if (forced >= 0) gmin = forced >> 6;

  // Recompute the 64 tempered logits of group gmin.  Both operands are K-block major (a column's 64 K values are one
  // 128-byte line), so the lanes work in groups of eight: lane l reads the 16-byte chunk l % 8 of the lines of columns
  // l / 8 + 8 j, j = 0..7 -- every wave-wide load is eight whole lines -- and the eight partial sums of a column are
  // added across its lane group at the end.
  const int chunk = lane & 7, cgroup = lane >> 3;
  float part[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) part[j] = 0.f;
  // Two K blocks per trip: their 18 loads are requested before the first product, so a trip waits for memory once.
  // (One block per trip left the wave waiting out a memory latency 40-64 times; four per trip are faster still for this
  // kernel alone but measured slower over the two-stream decode phase, beside the other half's attention.)  The products
  // are added in the same order whatever the trip length.
  constexpr int KB = 2;
  for (int kb = 0; kb < a.d; kb += 64 * KB) {
    u32x4 hv[KB], hl[KB], wv[KB][8];
    bool live[KB];
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      const int k = kb + 64 * q + 8 * chunk;
      live[q] = k < a.d;                   // d is a multiple of 32: the last K block may be half full
      if (!live[q]) continue;
      hv[q] = *(const u32x4*)(a.hfin + kblk_off(row, k, a.R));
      if (a.precise) hl[q] = *(const u32x4*)(a.hfin + a.hfin_lo_off + kblk_off(row, k, a.R));
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int c = gmin * 64 + cgroup + 8 * j;
        if (c < a.vocab) wv[q][j] = *(const u32x4*)(a.lm_head + kblk_off(c, k, a.vocab));
      }
    }
#pragma unroll
    for (int q = 0; q < KB; ++q) {
      if (!live[q]) continue;
      float h[8];
      if (a.precise) {
        // the normalised row as bf16 hi/lo pairs: their sum is formed in fp32, where it is exact
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          h[2 * e] = __uint_as_float(hv[q][e] << 16) + __uint_as_float(hl[q][e] << 16);
          h[2 * e + 1] = __uint_as_float(hv[q][e] & 0xffff0000u) + __uint_as_float(hl[q][e] & 0xffff0000u);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          h[2 * e] = f16_bits_to_f32((uint16_t)(hv[q][e] & 0xffffu));
          h[2 * e + 1] = f16_bits_to_f32((uint16_t)(hv[q][e] >> 16));
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int c = gmin * 64 + cgroup + 8 * j;
        if (c >= a.vocab) continue;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (a.precise) {                    // bf16 weights
            part[j] += __uint_as_float(wv[q][j][e] << 16) * h[2 * e];
            part[j] += __uint_as_float(wv[q][j][e] & 0xffff0000u) * h[2 * e + 1];
          } else {
            part[j] += f16_bits_to_f32((uint16_t)(wv[q][j][e] & 0xffffu)) * h[2 * e];
            part[j] += f16_bits_to_f32((uint16_t)(wv[q][j][e] >> 16)) * h[2 * e + 1];
          }
        }
      }
    }
  }
  // lane L ends up with column 64 gmin + L = cgroup' + 8 j' for cgroup' = L % 8, j' = L / 8: the sum of lane group cgroup'
  float acc = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float v = part[j];
    v += __shfl_xor(v, 1, WAVE);
    v += __shfl_xor(v, 2, WAVE);
    v += __shfl_xor(v, 4, WAVE);
    const float t = __shfl(v, 8 * (lane & 7), WAVE);
    if ((lane >> 3) == j) acc = t;
  }
  const int col = gmin * 64 + lane;
  const float logit = col < a.vocab ? acc / a.temperature : -INFINITY;
  int tok;
  if (forced >= 0) {
    tok = forced;
  } else if (a.greedy) {
    const float best = wave_max(logit);
    const unsigned long long at = __ballot(logit == best);
    tok = min(gmin * 64 + (at ? __ffsll((long long)at) - 1 : 0), a.vocab - 1);
  } else {
    const double e = (logit == -INFINITY) ? 0.0 : (double)__expf(logit - M);
    const double cum = base + wave_incl_scan(e, lane);
    const unsigned long long hit = __ballot(cum > target && e > 0.0);
    const unsigned long long pos = __ballot(e > 0.0);
    int j;
    if (hit) j = __ffsll((long long)hit) - 1;
    else if (pos) j = 63 - __clzll((long long)pos);   // rounding left the crossing outside: last positive column
    else j = 0;
    tok = min(gmin * 64 + j, a.vocab - 1);
  }
  const float ltok = __shfl(logit, tok & 63, WAVE);
  if (lane == 0) {
    a.tokens[idx] = tok;
    a.logprobs[idx] = (float)((double)ltok - logZ);
    if (a.next_token) a.next_token[row] = tok;
    if (a.finished && tok == a.eos) a.finished[row] = 1;
  }
}

__global__ __launch_bounds__(256) void score_finalize_kernel(const float2* partial, int ngroups, const float* target_logit,
                                                            const int* out_index, float* out, int R) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= R) return;
  float M;
  double incl;
  row_logz(partial + (size_t)row * ngroups, ngroups, lane, M, incl);
  if (lane == 63) out[out_index[row]] = (float)((double)target_logit[row] - ((double)M + log(incl)));
}

}  // namespace

hipError_t rl_sample(const SampleArgs& a, hipStream_t s) {
  if (a.R <= 0) return hipSuccess;
  hipLaunchKernelGGL(sample_kernel, dim3((a.R + 3) / 4), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t rl_score_finalize(const float2* partial, int ngroups, const float* target_logit, const int* out_index,
                             float* out, int R, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  hipLaunchKernelGGL(score_finalize_kernel, dim3((R + 3) / 4), dim3(256), 0, s, partial, ngroups, target_logit, out_index, out, R);
  return hipGetLastError();
}
