// fp16 x fp16 -> fp32 GEMM on the gfx950 matrix cores, C[M,N] = A[M,K] . W[N,K]^T, with the
// epilogues the decoder needs fused in.  (Weights are the caller's bf16 values held in fp16, which
// represents them exactly; activations are fp16, whose 11 significant bits keep the logits within
// the parity bound where bf16 activations do not.)  Both operands are K-contiguous, so every MFMA operand
// fragment is one 16-byte load.  256 threads = 4 waves in a 2x2 arrangement; each wave owns a
// (BM/2)x(BN/2) sub-tile built from 32x32x16 MFMAs; A and W tiles of depth 64 are staged through
// LDS (16-byte chunks, XOR-swizzled by row so that fragment reads spread over all banks) with
// register prefetch of the next tile and one barrier per K step.
#include "kernels.h"

namespace {

constexpr int BK = 64;            // bf16 elements of K per LDS stage (128 bytes per row)

// Blocks are handed to the 8 XCDs round-robin by the hardware.  Renumber them so that each XCD
// (one L2) works on a contiguous range of logical tile ids, then walk tiles M-fastest inside groups
// of 8 M-tiles: the blocks that share a weight tile run on the same L2 at the same time.
__device__ __forceinline__ void tile_of_block(int tiles_m, int tiles_n, int& tm, int& tn) {
  const int nb = gridDim.x, bid = blockIdx.x;
  const int per = (nb + 7) >> 3;
  const int full = (nb & 7) == 0 ? 8 : (nb & 7);
  const int xcd = bid & 7, slot = bid >> 3;
  const int logical = xcd < full ? xcd * per + slot : full * per + (xcd - full) * (per - 1) + slot;
  constexpr int GROUP_M = 8;
  const int per_group = GROUP_M * tiles_n;
  const int group = logical / per_group;
  const int first_m = group * GROUP_M;
  const int gsz = min(tiles_m - first_m, GROUP_M);
  const int in_group = logical - group * per_group;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

__device__ __forceinline__ float gelu_erf(float v) { return 0.5f * v * (1.0f + erff(v * 0.70710678118654752f)); }
__device__ __forceinline__ float silu(float v) { return v / (1.0f + __expf(-v)); }

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_f16_kernel(GemmArgs g) {
  constexpr int TM = BM / 64, TN = BN / 64;      // 32x32 MFMA tiles per wave in each direction
  __shared__ __attribute__((aligned(16))) uint16_t lds[2][(BM + BN) * BK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  int tile_m, tile_n;
  tile_of_block(tiles_m, tiles_n, tile_m, tile_n);
  const int row0 = tile_m * BM, col0 = tile_n * BN;

  // ---- global -> register staging: thread t covers chunk (t % 8) of rows (t / 8) + 32 i
  const int ld_chunk = tid & 7, ld_row = tid >> 3;
  const uint16_t* __restrict__ A = (const uint16_t*)g.A;
  const uint16_t* __restrict__ W = (const uint16_t*)g.W;
  u32x4 ra[BM / 32], rb[BN / 32];
  const uint16_t* pa[BM / 32];
  const uint16_t* pb[BN / 32];
#pragma unroll
  for (int i = 0; i < BM / 32; ++i) {
    int r = min(row0 + ld_row + 32 * i, g.M - 1);
    pa[i] = A + (size_t)r * g.lda + ld_chunk * 8;
  }
#pragma unroll
  for (int i = 0; i < BN / 32; ++i) {
    int r = min(col0 + ld_row + 32 * i, g.N - 1);
    pb[i] = W + (size_t)r * g.ldw + ld_chunk * 8;
  }
  auto load_global = [&](int k0) {
    const bool ok = k0 + ld_chunk * 8 < g.K;
#pragma unroll
    for (int i = 0; i < BM / 32; ++i) ra[i] = ok ? *(const u32x4*)(pa[i] + k0) : u32x4{0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < BN / 32; ++i) rb[i] = ok ? *(const u32x4*)(pb[i] + k0) : u32x4{0, 0, 0, 0};
  };
  auto store_lds = [&](int buf) {
    uint16_t* la = lds[buf];
    uint16_t* lb = lds[buf] + BM * BK;
#pragma unroll
    for (int i = 0; i < BM / 32; ++i) {
      int r = ld_row + 32 * i;
      *(u32x4*)(la + r * BK + ((ld_chunk ^ (r & 7)) * 8)) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < BN / 32; ++i) {
      int r = ld_row + 32 * i;
      *(u32x4*)(lb + r * BK + ((ld_chunk ^ (r & 7)) * 8)) = rb[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = (g.K + BK - 1) / BK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  const int frow = lane & 31, fhalf = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_global((kt + 1) * BK);
    const uint16_t* la = lds[cur] + (wm * (BM / 2)) * BK;
    const uint16_t* lb = lds[cur] + BM * BK + (wn * (BN / 2)) * BK;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      f16x8 fa[TM], fb[TN];
      const int chunk = kk * 2 + fhalf;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        int r = i * 32 + frow;
        fa[i] = *(const f16x8*)(la + r * BK + ((chunk ^ (r & 7)) * 8));
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        int r = j * 32 + frow;
        fb[j] = *(const f16x8*)(lb + r * BK + ((chunk ^ (r & 7)) * 8));
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_lds(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][e]: row = 8 (e / 4) + 4 (lane / 32) + e % 4, col = lane % 32 of the 32x32 tile
  const int wrow0 = row0 + wm * (BM / 2), wcol0 = col0 + wn * (BN / 2);
  if constexpr (EPI == EPI_LMHEAD) {
    // per row and per 64-column group: max and sum of exp of the tempered logits; optional capture
    // of the target column's tempered logit.  Nothing of size [M, N] is written.
    static_assert(BN == 128, "one wave must own one 64-column group");
    const int group = wcol0 >> 6;
    const int ngroups = (g.N + 63) >> 6;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = wrow0 + i * 32 + 8 * (e >> 2) + 4 * fhalf + (e & 3);
        float l[TN];
        float mx = -INFINITY;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = wcol0 + j * 32 + frow;
          l[j] = col < g.N ? acc[i][j][e] / g.temperature : -INFINITY;
          mx = fmaxf(mx, l[j]);
          if (g.target != nullptr && row < g.M && col < g.N && g.target[row] == col) g.target_logit[row] = l[j];
        }
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, WAVE));
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < TN; ++j) s += (l[j] == -INFINITY) ? 0.f : __expf(l[j] - mx);
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o, WAVE);
        if (frow == 0 && row < g.M && group < ngroups)
          g.partial[(size_t)row * ngroups + group] = make_float2(mx, s);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = wcol0 + j * 32 + frow;
        if (col >= g.N) continue;
        const float b = g.bias ? g.bias[col] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = wrow0 + i * 32 + 8 * (e >> 2) + 4 * fhalf + (e & 3);
          if (row >= g.M) continue;
          float v = acc[i][j][e] + b;
          if constexpr (EPI == EPI_F32) {
            ((float*)g.out)[(size_t)row * g.ldo + col] = v;
          } else if constexpr (EPI == EPI_RESID) {
            float* p = (float*)g.out + (size_t)row * g.ldo + col;
            *p = *p + v;
          } else if constexpr (EPI == EPI_GELU_F16) {
            ((uint16_t*)g.out)[(size_t)row * g.ldo + col] = f32_to_f16_bits(gelu_erf(v));
          } else if constexpr (EPI == EPI_SWIGLU_F16) {
            // weight rows come in blocks of 32: block 2b = gate rows [32b, 32b+32), block 2b+1 = the
            // matching up rows, so tile j (even) and tile j+1 hold gate and up of the same features.
            if ((j & 1) == 0) {
              const float up = acc[i][j + 1 < TN ? j + 1 : j][e];
              const int f = ((wcol0 + j * 32) >> 1) + frow;
              ((uint16_t*)g.out)[(size_t)row * g.ldo + f] = f32_to_f16_bits(silu(v) * up);
            }
          }
        }
      }
    }
  }
}

template <int BM, int BN, int EPI>
hipError_t launch(const GemmArgs& g, hipStream_t s) {
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  hipLaunchKernelGGL((gemm_f16_kernel<BM, BN, EPI>), dim3(tiles), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace

hipError_t rl_gemm(const GemmArgs& g, int epi, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.K % 8 != 0 || g.lda % 8 != 0 || g.ldw % 8 != 0) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_F32: return launch<128, 128, EPI_F32>(g, s);
    case EPI_RESID: return launch<128, 128, EPI_RESID>(g, s);
    case EPI_GELU_F16: return launch<128, 128, EPI_GELU_F16>(g, s);
    case EPI_SWIGLU_F16:
      if (g.N % 64 != 0) return hipErrorInvalidValue;
      return launch<128, 128, EPI_SWIGLU_F16>(g, s);
    case EPI_LMHEAD: return launch<128, 128, EPI_LMHEAD>(g, s);
  }
  return hipErrorInvalidValue;
}
