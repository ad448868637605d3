// Small memory-bound kernels around the GEMMs: weight conversion, embedding gather, LayerNorm /
// RMSNorm, rotary embedding + KV-cache write, and the consumers of the log-probs.
#include "kernels.h"

namespace {

constexpr int TPB = 256;
inline int blocks_for(size_t n, int per = TPB) { return (int)((n + per - 1) / per); }

__global__ void to_bf16_kernel(uint16_t* dst, const void* src, int src_is_bf16, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride)
    dst[i] = src_is_bf16 ? ((const uint16_t*)src)[i] : f32_to_bf16_bits(((const float*)src)[i]);
}
// as_bf16: the bf16 bit patterns themselves are stored (precise mode) instead of their fp16 equivalents
__global__ void to_f16w_kernel(uint16_t* dst, const void* src, int src_is_bf16, int rows, int K, int rows_total, int row0,
                               int perm_h, int perm_r, int as_bf16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)rows * K, stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const uint16_t b = src_is_bf16 ? ((const uint16_t*)src)[i] : f32_to_bf16_bits(((const float*)src)[i]);
    int row = (int)(i / K);
    if (perm_h > 0) row = row / perm_h * perm_h + qkv_packed_pos(row % perm_h, perm_r);
    dst[kblk_off(row0 + row, (int)(i % K), rows_total)] = as_bf16 ? b : f32_to_f16_bits(bf16_bits_to_f32(b));
  }
}
__global__ void to_f32_kernel(float* dst, const void* src, int src_is_bf16, size_t n, int perm_h, int perm_r) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const float v = src_is_bf16 ? bf16_bits_to_f32(((const uint16_t*)src)[i]) : ((const float*)src)[i];
    const size_t o = perm_h > 0 ? i / perm_h * perm_h + qkv_packed_pos((int)(i % perm_h), perm_r) : i;
    dst[o] = v;
  }
}
__global__ void pack_gate_up_kernel(uint16_t* dst, const void* gate, const void* up, int src_is_bf16, int F, int d, int as_bf16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)2 * F * d, stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const int row = (int)(i / d), col = (int)(i % d);
    const int blk = row >> 5, in = row & 31;
    const void* src = (blk & 1) ? up : gate;
    const size_t si = (size_t)((blk >> 1) * 32 + in) * d + col;
    const uint16_t b = src_is_bf16 ? ((const uint16_t*)src)[si] : f32_to_bf16_bits(((const float*)src)[si]);
    dst[kblk_off(row, col, 2 * F)] = as_bf16 ? b : f32_to_f16_bits(bf16_bits_to_f32(b));
  }
}
__global__ void rope_table_kernel(float2* tab, int max_pos, int r, double theta) {
  const int half = r / 2;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= max_pos * half) return;
  const int pos = i / half, k = i % half;
  const double ang = (double)pos * pow(theta, -2.0 * (double)k / (double)r);
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}
__global__ void fill_zero_kernel(u32x4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = u32x4{0, 0, 0, 0};
}

__global__ void fill_random_f16_kernel(uint16_t* p, size_t n, unsigned seed, int as_bf16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    unsigned x = (unsigned)i * 2654435761u + seed;
    x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13;
    const float v = (x & 0xffff) / 65536.0f - 0.5f;
    p[i] = as_bf16 ? f32_to_bf16_bits(v) : f32_to_f16_bits(v);
  }
}

__global__ void embed_kernel(float* x, const uint16_t* E, const int* tokens, const int* tok_index, int rows, int d,
                             int vocab, unsigned* status) {
  const int row = blockIdx.x;
  int tok = tokens[tok_index ? tok_index[row] : row];
  if (tok < 0 || tok >= vocab) {
    if (threadIdx.x == 0) atomicOr(status, RLGEN_FAULT_TOKEN);
    tok = min(max(tok, 0), vocab - 1);
  }
  const uint16_t* e = E + (size_t)tok * d;
  float* xr = x + (size_t)row * d;
  for (int i = threadIdx.x * 8; i < d; i += blockDim.x * 8) {
    const u32x4 v = *(const u32x4*)(e + i);
    f32x4 lo, hi;
    lo[0] = __uint_as_float(v[0] << 16); lo[1] = __uint_as_float(v[0] & 0xffff0000u);
    lo[2] = __uint_as_float(v[1] << 16); lo[3] = __uint_as_float(v[1] & 0xffff0000u);
    hi[0] = __uint_as_float(v[2] << 16); hi[1] = __uint_as_float(v[2] & 0xffff0000u);
    hi[2] = __uint_as_float(v[3] << 16); hi[3] = __uint_as_float(v[3] & 0xffff0000u);
    *(f32x4*)(xr + i) = lo;
    *(f32x4*)(xr + i + 4) = hi;
  }
}

// One wave per row; the row lives in registers (d <= 64 * 4 * NV).  Mean, then variance of the
// centred values (two passes over registers), all in fp32; the normalised row is stored as fp16.
template <int NV>
__global__ __launch_bounds__(256) void norm_kernel(const float* x, const int* row_index, int rows, int d, float eps,
                                                   const float* g1, const float* b1, uint16_t* out1,
                                                   const float* g2, const float* b2, uint16_t* out2,
                                                   int out_rows, int out_row0, unsigned* status, size_t lo_off) {
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const float* xr = x + (size_t)(row_index ? row_index[row] : row) * d;
  f32x4 v[NV];
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int col = (i * 64 + lane) * 4;
    v[i] = col < d ? *(const f32x4*)(xr + col) : f32x4{0.f, 0.f, 0.f, 0.f};
    sum += v[i][0] + v[i][1] + v[i][2] + v[i][3];
  }
  const bool rms = (b1 == nullptr);
  const float mean = rms ? 0.f : wave_sum(sum) / (float)d;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int col = (i * 64 + lane) * 4;
    if (col < d) {
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[i][e] -= mean;
        sq += v[i][e] * v[i][e];
      }
    }
  }
  const float rstd = rsqrtf(wave_sum(sq) / (float)d + eps);
  bool sat = false;                 // did a value leave fp16's range (it is clamped; the context's status word records it)
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int col = (i * 64 + lane) * 4;
    if (col >= d) continue;
    const f32x4 ga = *(const f32x4*)(g1 + col);
    f32x4 ba = f32x4{0.f, 0.f, 0.f, 0.f};
    if (!rms) ba = *(const f32x4*)(b1 + col);
    f32x4 y;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      y[e] = v[i][e] * rstd * ga[e] + ba[e];
      sat |= f16_out_of_range(y[e]);
    }
    u32x2 w;
    if (lo_off) {          // precise mode: bf16 hi/lo pairs, the lo halves lo_off elements behind the hi halves
      u32x2 wl;
      SPLIT_BF16X2(y[0], y[1], w[0], wl[0]);
      SPLIT_BF16X2(y[2], y[3], w[1], wl[1]);
      *(u32x2*)(out1 + lo_off + kblk_off(out_row0 + row, col, out_rows)) = wl;
    } else {
      w[0] = pack_f16x2(y[0], y[1]);
      w[1] = pack_f16x2(y[2], y[3]);
    }
    *(u32x2*)(out1 + kblk_off(out_row0 + row, col, out_rows)) = w;
    if (out2) {
      const f32x4 gb = *(const f32x4*)(g2 + col);
      f32x4 bb = f32x4{0.f, 0.f, 0.f, 0.f};
      if (b2) bb = *(const f32x4*)(b2 + col);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        y[e] = v[i][e] * rstd * gb[e] + bb[e];
        sat |= f16_out_of_range(y[e]);
      }
      if (lo_off) {
        u32x2 wl;
        SPLIT_BF16X2(y[0], y[1], w[0], wl[0]);
        SPLIT_BF16X2(y[2], y[3], w[1], wl[1]);
        *(u32x2*)(out2 + lo_off + kblk_off(out_row0 + row, col, out_rows)) = wl;
      } else {
        w[0] = pack_f16x2(y[0], y[1]);
        w[1] = pack_f16x2(y[2], y[3]);
      }
      *(u32x2*)(out2 + kblk_off(out_row0 + row, col, out_rows)) = w;
    }
  }
  flag_f16_range(sat && lo_off == 0, status);        // bf16 pairs have fp32's range
}

// One thread per (row, head slot, 8-dim chunk).  Head slots: Hq query heads, Hkv key heads, Hkv
// value heads.  The pair (i, i + r/2) of the first r dims is rotated by the row's position.
__global__ void rope_kv_kernel(RopeArgs a) {
  const int nch = a.h >> 3;
  const int slots = a.Hq + 2 * a.Hkv;
  const int done = a.v_by_blocks ? a.Hq + a.Hkv : slots;     // head slots this kernel handles
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t total = (size_t)a.rows * done * nch;
  if (idx >= total) return;
  const int chunk = (int)(idx % nch);
  const int slot = (int)((idx / nch) % done);
  const int row = (int)(idx / ((size_t)nch * done));
  const float* src = a.qkv + (size_t)row * slots * a.h + (size_t)slot * a.h;
  const int pos = a.pos[row] + a.pos_add;
  const int half = a.r >> 1;
  float v[8];
  const bool is_v = slot >= a.Hq + a.Hkv;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int dim = chunk * 8 + e;
    float x = src[dim];
    if (!is_v && dim < a.r) {
      const int i = dim < half ? dim : dim - half;
      const float2 cs = a.table[(size_t)pos * half + i];
      const float partner = src[dim < half ? dim + half : dim - half];
      x = dim < half ? x * cs.x - partner * cs.y : x * cs.x + partner * cs.y;
    }
    v[e] = x;
  }
  if (slot < a.Hq) {
    u32x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = pack_f16x2(v[2 * e], v[2 * e + 1]);
    *(u32x4*)(a.q + (size_t)row * a.Hq * a.h + slot * a.h + chunk * 8) = w;
    return;
  }
  const int s0 = a.dst_seq[row];
  const int slotpos = pos - (a.slot_sub ? a.slot_sub[row] : 0);     // where in the stream the token goes
  for (int cpy = 0; cpy < a.ncopy; ++cpy) {
    const int s = s0 + cpy;
    const long long off = a.kv_off[s];
    const int cap = a.kv_cap[s];
    if (!is_v) {
      uint16_t* st = a.kv + a.lay.stream(off, cap, slot - a.Hq);
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
      *(u32x4*)(st + a.lay.k_elem(slotpos, chunk * 8)) = w;
    } else {
      uint16_t* st = a.kv + a.lay.stream(off, cap, slot - a.Hq - a.Hkv);
#pragma unroll
      for (int e = 0; e < 8; ++e) st[a.lay.v_elem(slotpos, chunk * 8 + e)] = f32_to_bf16_bits(v[e]);
    }
  }
}

// Prompt pass: values of 8 consecutive tokens of one sequence and one head dim form one 16-byte unit of
// the cache layout, so one thread gathers them (coalesced across head dims) and writes the unit whole, to
// every copy.  One block per 16-token job; slots past the prompt's end are written as zero (the decode
// steps fill them later).
__global__ __launch_bounds__(256) void rope_v_prefill_kernel(RopeArgs a) {
  const AttnJob jb = a.jobs[blockIdx.x];
  const int slots = a.Hq + 2 * a.Hkv;
  const int per_group = a.Hkv * a.h;
  const size_t ld = (size_t)slots * a.h;
  for (int item = threadIdx.x; item < 2 * per_group; item += blockDim.x) {
    const int grp = item / per_group, rem = item - grp * per_group;
    const int head = rem / a.h, dim = rem - head * a.h;
    const int pos0 = jb.qblock * 16 + grp * 8;
    if (pos0 >= jb.len) continue;
    const float* src = a.qkv + (size_t)(jb.row0 + pos0) * ld + (size_t)(a.Hq + a.Hkv + head) * a.h + dim;
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = pos0 + i < jb.len ? src[(size_t)i * ld] : 0.f;
    u32x4 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(v[2 * e], v[2 * e + 1]);
    for (int cpy = 0; cpy < a.ncopy; ++cpy) {
      const int s = jb.cache_seq + cpy;
      uint16_t* st = a.kv + a.lay.stream(a.kv_off[s], a.kv_cap[s], head);
      *(u32x4*)(st + a.lay.v_elem(pos0, dim)) = w;
    }
  }
}

// The same from staged bf16 rows [k heads | v heads] (fused QKV projection): keys move as 16-byte units of 8 head
// dims, values are gathered over 8 tokens as above.
__global__ __launch_bounds__(256) void kv_prefill_kernel(RopeArgs a) {
  const AttnJob jb = a.jobs[blockIdx.x];
  const int per_group = a.Hkv * a.h;
  const size_t ld = (size_t)2 * per_group;
  const int ntok = min(16, jb.len - jb.qblock * 16);
  const int nch = per_group >> 3;                       // 16-byte units of one token's keys (or values)
  const float inv_h = 1.0f / (float)a.h;
  const uint16_t* stage = a.kvstage + (size_t)(jb.row0 + jb.qblock * 16) * ld;
  // the job's items are spread over gridDim.y blocks: the copies are latency-bound, so more blocks in flight
  const int first = threadIdx.x + blockDim.x * blockIdx.y, step = blockDim.x * gridDim.y;
  // keys: items ordered as the cache stores them -- (head, 8-dim chunk, t, row) with 8 rows of a 16-token job
  // contiguous -- so that eight lanes write one 128-byte line; the staged rows are read in 16-byte pieces
#pragma unroll 2
  for (int item = first; item < 16 * nch; item += step) {
    const int r8 = item & 7, t = (item >> 3) & 1, unit = item >> 4;
    const int tok = 8 * (r8 >> 2) + 4 * t + (r8 & 3);
    if (tok >= ntok) continue;
    const int head = (int)(((float)(unit << 3) + 0.5f) * inv_h), dim = (unit << 3) - head * a.h;
    const u32x4 w = *(const u32x4*)(stage + (size_t)tok * ld + (unit << 3));
    const long long o = a.lay.k_elem(jb.qblock * 16 + tok, dim);
    for (int cpy = 0; cpy < a.ncopy; ++cpy) {
      const int s = jb.cache_seq + cpy;
      *(u32x4*)(a.kv + a.lay.stream(a.kv_off[s], a.kv_cap[s], head) + o) = w;
    }
  }
  // values: a thread takes 8 head dims of 8 consecutive tokens (8 row-contiguous 16-byte loads), transposes them
  // in registers and writes the 8 units (one per head dim, 8 keys each), which are 128 contiguous bytes
  for (int item = first; item < 2 * nch; item += step) {
    const int grp = item / nch, unit = item - grp * nch;
    if (grp * 8 >= ntok) continue;
    const int head = (int)(((float)(unit << 3) + 0.5f) * inv_h), dim = (unit << 3) - head * a.h;
    u32x4 b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
      b[i] = grp * 8 + i < ntok ? *(const u32x4*)(stage + (size_t)(grp * 8 + i) * ld + per_group + (unit << 3)) : u32x4{0, 0, 0, 0};
    u32x4 w[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t lo = b[2 * e][j >> 1], hi = b[2 * e + 1][j >> 1];
        w[j][e] = (j & 1) ? ((lo >> 16) | (hi & 0xffff0000u)) : ((lo & 0xffffu) | (hi << 16));
      }
    const long long o = a.lay.v_elem(jb.qblock * 16 + grp * 8, dim);
    for (int cpy = 0; cpy < a.ncopy; ++cpy) {
      const int s = jb.cache_seq + cpy;
      u32x4* dst = (u32x4*)(a.kv + a.lay.stream(a.kv_off[s], a.kv_cap[s], head) + o);
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[j] = w[j];
    }
  }
}

__global__ void sequence_logprob_kernel(const float* tlp, const int* from, const int* lens, int N, int stride, float* out) {
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (n >= N) return;
  float acc = 0.f;
  for (int t = max(from[n], 0) + lane; t < min(lens[n], stride); t += 64) acc += tlp[(size_t)n * stride + t];
  acc = wave_sum(acc);
  if (lane == 0) out[n] = acc;
}
__global__ void select_pairs_kernel(const float* rewards, int B, int k, int* idx_pos, int* idx_neg) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const float* r = rewards + (size_t)b * k;
  int pos = 0, neg = 0;
  for (int j = 1; j < k; ++j) {
    if (r[j] > r[pos]) pos = j;        // first of the highest
    if (r[j] <= r[neg]) neg = j;       // last of the lowest
  }
  idx_pos[b] = pos;
  idx_neg[b] = neg;
}
__global__ void dpo_loss_kernel(const float* pp, const float* rp, const float* pn, const float* rn, int P, float beta, float* loss) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= P) return;
  const float x = beta * ((pp[i] - rp[i]) - (pn[i] - rn[i]));
  // -log sigmoid(x) = max(-x, 0) + log1p(exp(-|x|))
  loss[i] = fmaxf(-x, 0.f) + log1pf(expf(-fabsf(x)));
}

// One thread per completion; its baseline is the mean reward of the prompt's other k - 1 completions.
__global__ void proximal_rloo_kernel(const float* lp_pol, const float* lp_old, const float* rewards, int B, int k, float eps,
                                     float* objective) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * k) return;
  const float* r = rewards + (size_t)(i / k) * k;
  float others = 0.f;
  for (int j = 0; j < k; ++j) others += (j == i % k) ? 0.f : r[j];
  const float adv = rewards[i] - others / (float)(k - 1);
  const float ratio = expf(lp_pol[i] - lp_old[i]);
  const float clipped = fminf(fmaxf(ratio, 1.f - eps), 1.f + eps);
  objective[i] = fminf(ratio * adv, clipped * adv);
}

}  // namespace

hipError_t rl_to_bf16(uint16_t* dst, const void* src, int src_is_bf16, size_t n, hipStream_t s) {
  if (!n) return hipSuccess;
  hipLaunchKernelGGL(to_bf16_kernel, dim3(min(blocks_for(n), 65536)), dim3(TPB), 0, s, dst, src, src_is_bf16, n);
  return hipGetLastError();
}
hipError_t rl_to_f16w(uint16_t* dst, const void* src, int src_is_bf16, int rows, int K, int rows_total, int row0, hipStream_t s,
                      int perm_h, int perm_r, int as_bf16) {
  if (perm_h > 0 && (rows % perm_h != 0 || perm_r % 4 != 0 || perm_r > perm_h)) return hipErrorInvalidValue;
  const size_t n = (size_t)rows * K;
  if (!n) return hipSuccess;
  hipLaunchKernelGGL(to_f16w_kernel, dim3(min(blocks_for(n), 65536)), dim3(TPB), 0, s, dst, src, src_is_bf16, rows, K, rows_total, row0,
                     perm_h, perm_r, as_bf16);
  return hipGetLastError();
}
hipError_t rl_to_f32(float* dst, const void* src, int src_is_bf16, size_t n, hipStream_t s, int perm_h, int perm_r) {
  if (!n) return hipSuccess;
  if (perm_h > 0 && (n % perm_h != 0 || perm_r % 4 != 0 || perm_r > perm_h)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(to_f32_kernel, dim3(min(blocks_for(n), 65536)), dim3(TPB), 0, s, dst, src, src_is_bf16, n, perm_h, perm_r);
  return hipGetLastError();
}
hipError_t rl_pack_gate_up(uint16_t* dst, const void* gate, const void* up, int src_is_bf16, int F, int d, hipStream_t s, int as_bf16) {
  hipLaunchKernelGGL(pack_gate_up_kernel, dim3(min(blocks_for((size_t)2 * F * d), 65536)), dim3(TPB), 0, s, dst, gate, up,
                     src_is_bf16, F, d, as_bf16);
  return hipGetLastError();
}
hipError_t rl_rope_table(float2* tab, int max_pos, int rotary_dim, float theta, hipStream_t s) {
  const int n = max_pos * (rotary_dim / 2);
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(rope_table_kernel, dim3(blocks_for(n)), dim3(TPB), 0, s, tab, max_pos, rotary_dim, (double)theta);
  return hipGetLastError();
}
hipError_t rl_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (!bytes) return hipSuccess;
  if (bytes % 16 != 0 || ((uintptr_t)p) % 16 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(min(blocks_for(bytes / 16), 262144)), dim3(TPB), 0, s, (u32x4*)p, bytes / 16);
  return hipGetLastError();
}
hipError_t rl_fill_random_f16(uint16_t* p, size_t n, unsigned seed, hipStream_t s, int as_bf16) {
  if (!n) return hipSuccess;
  hipLaunchKernelGGL(fill_random_f16_kernel, dim3(min(blocks_for(n), 65536)), dim3(TPB), 0, s, p, n, seed, as_bf16);
  return hipGetLastError();
}
hipError_t rl_embed(float* x, const uint16_t* E, const int* tokens, const int* tok_index, int rows, int d, int vocab,
                    unsigned* status, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(embed_kernel, dim3(rows), dim3(128), 0, s, x, E, tokens, tok_index, rows, d, vocab, status);
  return hipGetLastError();
}
hipError_t rl_norm(const float* x, const int* row_index, int rows, int d, float eps, const float* g1, const float* b1,
                   uint16_t* out1, const float* g2, const float* b2, uint16_t* out2, int out_rows, int out_row0,
                   unsigned* status, hipStream_t s, size_t lo_off) {
  if (rows <= 0) return hipSuccess;
  const dim3 grid((rows + 3) / 4), block(256);
  const int nv = (d + 255) / 256;
#define NORM(NV) hipLaunchKernelGGL((norm_kernel<NV>), grid, block, 0, s, x, row_index, rows, d, eps, g1, b1, out1, g2, b2, out2, out_rows, out_row0, status, lo_off)
  if (nv <= 1) NORM(1);
  else if (nv <= 2) NORM(2);
  else if (nv <= 4) NORM(4);
  else if (nv <= 8) NORM(8);
  else if (nv <= 16) NORM(16);
  else if (nv <= 32) NORM(32);
  else return hipErrorInvalidValue;
#undef NORM
  return hipGetLastError();
}
hipError_t rl_rope_kv(const RopeArgs& a, hipStream_t s) {
  const size_t total = (size_t)a.rows * (a.v_by_blocks ? a.Hq + a.Hkv : a.Hq + 2 * a.Hkv) * (a.h >> 3);
  if (!total) return hipSuccess;
  hipLaunchKernelGGL(rope_kv_kernel, dim3(blocks_for(total)), dim3(TPB), 0, s, a);
  if (a.v_by_blocks && a.njobs > 0) hipLaunchKernelGGL(rope_v_prefill_kernel, dim3(a.njobs), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t rl_kv_prefill(const RopeArgs& a, hipStream_t s) {
  if (a.njobs <= 0) return hipSuccess;
  if (!a.kvstage || !a.jobs || a.h % 8 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kv_prefill_kernel, dim3(a.njobs, 8), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t rl_sequence_logprob(const float* tlp, const int* from, const int* lens, int N, int stride, float* out, hipStream_t s) {
  if (N <= 0) return hipSuccess;
  hipLaunchKernelGGL(sequence_logprob_kernel, dim3((N + 3) / 4), dim3(256), 0, s, tlp, from, lens, N, stride, out);
  return hipGetLastError();
}
hipError_t rl_select_pairs(const float* rewards, int B, int k, int* idx_pos, int* idx_neg, hipStream_t s) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_pairs_kernel, dim3(blocks_for(B)), dim3(TPB), 0, s, rewards, B, k, idx_pos, idx_neg);
  return hipGetLastError();
}
hipError_t rl_dpo_loss(const float* pp, const float* rp, const float* pn, const float* rn, int P, float beta, float* loss, hipStream_t s) {
  if (P <= 0) return hipSuccess;
  hipLaunchKernelGGL(dpo_loss_kernel, dim3(blocks_for(P)), dim3(TPB), 0, s, pp, rp, pn, rn, P, beta, loss);
  return hipGetLastError();
}
hipError_t rl_proximal_rloo(const float* lp_pol, const float* lp_old, const float* rewards, int B, int k, float eps, float* objective,
                            hipStream_t s) {
  if (B <= 0) return hipSuccess;
  hipLaunchKernelGGL(proximal_rloo_kernel, dim3(blocks_for((size_t)B * k)), dim3(TPB), 0, s, lp_pol, lp_old, rewards, B, k, eps,
                     objective);
  return hipGetLastError();
}
