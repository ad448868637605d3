// Host-callable launchers of the rlgen kernels.  Everything here is internal to librlgen.so.
#pragma once
#include "common.h"

// ------------------------------------------------------------------ KV cache layout
// One contiguous stream per (layer, sequence, kv head): `cap` keys (a multiple of 32), cut into
// super-blocks of 32 keys; each super-block holds its 32 keys (32 h bf16) followed by its 32 values, so a
// decode step reads the stream front to back.  Inside a super-block the elements are ordered so
// that every MFMA operand fragment the attention kernel needs is one 16-byte unit and every
// wave-wide load instruction reads one contiguous kilobyte:
//   K super-block: [t = 0..1][chunk = 0..h/8-1][r = 0..15][8 head dims]
//                  holding key 8 (r / 4) + 4 t + r % 4, head dims 8 chunk .. 8 chunk + 7
//   V super-block: [tile = 0..h/16-1][g = 0..3][r = 0..15][8 keys]
//                  holding head dim 16 tile + r, keys 8 g .. 8 g + 7
// Streams of a sequence: head 0..Hkv-1; sequences follow each other at token offsets kv_off[s];
// layers are max_kv_tokens * Hkv * h * 2 elements apart.
struct KvLayout {
  int Hkv, h;
  long long layer_stride;  // elements between layers
  __host__ __device__ long long seq_base(long long kv_off) const { return 2LL * kv_off * Hkv * h; }
  __host__ __device__ long long stream(long long kv_off, int cap, int head) const {
    return seq_base(kv_off) + (long long)head * 2 * cap * h;
  }
  // element offset of key / value (key, dim) inside a stream
  __host__ __device__ long long k_elem(int key, int dim) const {
    const int sb = key >> 5, kk = key & 31;
    const int r = 4 * (kk >> 3) + (kk & 3), t = (kk >> 2) & 1;
    return (long long)sb * 64 * h + (((t * (h >> 3) + (dim >> 3)) * 16 + r) << 3) + (dim & 7);
  }
  __host__ __device__ long long v_elem(int key, int dim) const {
    const int sb = key >> 5, kk = key & 31;
    return (long long)sb * 64 * h + 32 * h + (((((dim >> 4) * 4 + (kk >> 3)) * 16) + (dim & 15)) << 3) + (kk & 7);
  }
};

// ------------------------------------------------------------------ GEMM
enum { EPI_F32 = 0, EPI_RESID = 1, EPI_GELU_F16 = 2, EPI_SWIGLU_F16 = 3, EPI_LMHEAD = 4, EPI_PARTIAL = 5, EPI_QKV = 6 };

// Epilogue of the fused QKV projection (EPI_QKV): bias, rotary embedding and the writes of q (fp16) and of k, v
// (bf16, into the cache) happen on the accumulators.  For that the weight rows of every query and key head are
// stored in the order qkv_packed_dim() gives: the rotary pairs (i, i + r/2), (i + 1, i + 1 + r/2) of a head sit
// in four consecutive output columns, which one lane holds.  Requires r % 4 == 0.
struct QkvEpi {
  int Hq, Hkv, h, r;
  // precise mode: q is written as fp32 [M, Hq h] (q points at floats); keys and values as bf16 hi/lo pairs, the lo
  // halves kv_lo_off elements behind the hi halves in the cache and stage_lo_off elements behind them in the staging rows
  long long kv_lo_off, stage_lo_off;
  float inv_h;                   // 1 / h
  const float2* table;           // [max_pos, r/2] cos, sin
  const int* pos; int pos_add;   // position of row i = pos[i] + pos_add
  uint16_t* q;                   // out: fp16 [M, Hq h], head dims in natural order
  // prompt pass: k (rotated) and v as bf16 [M, 2 Hkv h] (k heads, then v heads) for rl_kv_prefill
  uint16_t* kvstage;
  // decode (kvstage null): k, v straight into the cache of sequence dst_seq[i] at slot position - slot_sub[i]
  const int* dst_seq; const int* slot_sub;   // slot_sub nullable
  uint16_t* kv; KvLayout lay; const int* kv_off; const int* kv_cap;
};
// head dim held by packed position p of a query / key head (identity for p >= r)
__host__ __device__ __forceinline__ int qkv_packed_dim(int p, int r) {
  return p >= r ? p : 2 * (p >> 2) + (p & 1) + ((p & 2) ? (r >> 1) : 0);
}
// and its inverse: packed position of head dim `dim`
__host__ __device__ __forceinline__ int qkv_packed_pos(int dim, int r) {
  if (dim >= r) return dim;
  const int half = r >> 1, i = dim < half ? dim : dim - half;
  return 4 * (i >> 1) + (i & 1) + (dim < half ? 0 : 2);
}

struct GemmArgs {
  const void* A;                // [M, K] fp16, K-block major (kblk_off with rows = M)
  const void* W;                // [N, K] fp16, K-block major (rows = N)
  int M, N, K;
  // Precise mode (precise = 1): W holds bf16 bit patterns; A is a bf16 hi/lo pair per element, stored as a matrix of
  // twice the K blocks (the hi blocks, then the lo blocks: kblk_elems(M, K) elements apart), and the product is
  // A_hi W^T + A_lo W^T on the bf16 matrix instructions: 16 significant bits of every activation instead of fp16's 11.
  // The *_F16 epilogues then write bf16 hi/lo pairs too, the lo halves out_lo_off elements behind the hi halves.
  int precise; size_t out_lo_off;
  const float* bias;            // [N] or null
  void* out; int ldo;           // EPI_F32 / EPI_RESID: fp32 [M, N] row-major, leading dim ldo;
                                // *_F16: fp16 K-block major with rows = M (ldo unused)
  // EPI_LMHEAD only
  float temperature;
  float2* partial;              // [M, ceil(N/64)] (max, sum exp) of the tempered logits per 64 columns
  const int* target;            // nullable [M]: column whose tempered logit is captured
  float* target_logit;          // [M]
  // split-K scratch (nullable: no split-K): fp32 [splits, M, N], ws_elems floats available
  float* ws; size_t ws_elems; int splits;
  QkvEpi qe;                    // EPI_QKV only (out / ldo unused)
  unsigned* status;             // nullable: receives RLGEN_FAULT_RANGE when an fp16 (or cached bf16, later read as fp16)
                                // output of the epilogue exceeds fp16's range and is clamped
};
// tile shape chosen from the problem size; g.splits >= 2 (with g.ws) cuts K into that many parts (rl_gemm_splitk)
hipError_t rl_gemm(const GemmArgs& g, int epi, hipStream_t s);
// the same with an explicit tile shape (tuning and tests): 0 = 128x128, 1 = 256x128, 2 = 256x256, ...
hipError_t rl_gemm_variant(const GemmArgs& g, int epi, int variant, hipStream_t s);
hipError_t rl_gemm_splitk(const GemmArgs& g, int epi, int variant, hipStream_t s);   // needs g.ws, g.splits >= 2

// ------------------------------------------------------------------ attention
// prefill: 16 queries [16 qblock, 16 qblock + 16) of one sequence.  pre_len > 0: the sequence continues a prefix held
// by cache sequence pre_seq (pre_len keys, all visible to every query) -- the shared prompt of grouped scoring
struct AttnJob { int cache_seq, row0, len, qblock, pre_seq, pre_len; };
struct AttnArgs {
  const uint16_t* q; int q_ld;        // fp16 [rows, Hq * h], rotated
  uint16_t* out; int out_rows;        // fp16 [out_rows, Hq * h], K-block major (input of the O projection)
  // precise mode: q points at fp32 [rows, Hq * h]; the cache holds bf16 hi/lo pairs, the lo halves kv_lo_off elements
  // behind the hi halves; the output is bf16 hi/lo pairs, the lo halves out_lo_off elements behind the hi halves
  int precise; long long kv_lo_off; size_t out_lo_off;
  const uint16_t* kv;                 // this layer's cache base
  KvLayout lay;
  const int* kv_off; const int* kv_cap;  // per cache sequence
  int Hq;
  float scale;
  // decode: one query row per sequence, keys 0 .. ctx_base[s] + ctx_add - 1
  const int* ctx_base; int ctx_add; int S;
  const int* order;                   // nullable [S] (or [prompts] when share_k): unit handled by slot i
  // shared prompt cache: 0 = off.  K = samples per prompt: sequence s = prompt * K + j; cache sequence `prompt`
  // holds the prompt's keys (ctx_base[prompt * K] of them), cache sequence sfx_first + s the ctx_add new tokens of s
  int share_k, sfx_first;
  const int* cache_seq_of;            // nullable [S] (not with share_k): cache sequence of row i, default i (kv_off / kv_cap index)
  const int* finished;                // nullable [S]: sequences whose completion has ended are skipped (their output rows keep
                                      // whatever they held; nothing downstream of an ended sequence is used)
  // prefill
  const AttnJob* jobs; int njobs;
};
hipError_t rl_attention_decode(const AttnArgs& a, hipStream_t s);
hipError_t rl_attention_prefill(const AttnArgs& a, hipStream_t s);
// 16-token blocks a prompt-pass attention wave takes at once for head size h; a.jobs must list a multiple of it per sequence
int rl_attention_prefill_qb(int h);

// ------------------------------------------------------------------ element-wise and small kernels
// dst bf16 <- src (fp32 rounded to nearest even, or bf16 copied); n elements
hipError_t rl_to_bf16(uint16_t* dst, const void* src, int src_is_bf16, size_t n, hipStream_t s);
// dst fp16 K-block major [rows_total, K] <- the bf16 values of src [rows, K] row-major placed at rows
// row0 .. row0 + rows - 1 (fp32 sources are first rounded to bf16, nearest even)
// perm_h > 0: source row head * perm_h + dim lands at row head * perm_h + qkv_packed_pos(dim, perm_r)
// as_bf16: store the bf16 bit patterns themselves (the weight format of precise mode)
hipError_t rl_to_f16w(uint16_t* dst, const void* src, int src_is_bf16, int rows, int K, int rows_total, int row0, hipStream_t s,
                      int perm_h = 0, int perm_r = 0, int as_bf16 = 0);
// dst fp32 <- src (fp32 copied, or bf16 expanded); n elements
// perm_h > 0: element head * perm_h + dim lands at head * perm_h + qkv_packed_pos(dim, perm_r)
hipError_t rl_to_f32(float* dst, const void* src, int src_is_bf16, size_t n, hipStream_t s, int perm_h = 0, int perm_r = 0);
// gate/up rows interleaved in blocks of 32 rows: dst [2F, d] fp16 (bf16 values), K-block major
hipError_t rl_pack_gate_up(uint16_t* dst, const void* gate, const void* up, int src_is_bf16, int F, int d, hipStream_t s, int as_bf16 = 0);
// cos/sin table [max_pos, r/2] (float2), angles pos * theta^(-2i/r) evaluated in fp64
hipError_t rl_rope_table(float2* tab, int max_pos, int rotary_dim, float theta, hipStream_t s);
hipError_t rl_fill_zero(void* p, size_t bytes, hipStream_t s);
// n pseudo-random fp16 values in [-0.5, 0.5) (inputs for timing runs)
hipError_t rl_fill_random_f16(uint16_t* p, size_t n, unsigned seed, hipStream_t s, int as_bf16 = 0);

// x[row, :] = float(E[tok[row]]), tok gathered as tokens[tok_index[row]] ; flags a bad id
hipError_t rl_embed(float* x, const uint16_t* E, const int* tokens, const int* tok_index, int rows, int d,
                    int vocab, unsigned* status, hipStream_t s);
// LayerNorm / RMSNorm of fp32 rows into fp16.  out2/g2/b2 nullable (second normalisation of the same
// row with other gains, NeoX); b1 null selects RMSNorm.  row_index nullable: source row of output row i.
// Outputs are K-block major matrices of out_rows rows; output row i goes to row out_row0 + i.
// status (nullable): receives RLGEN_FAULT_RANGE if a normalised value does not fit fp16 (it is clamped).
// lo_off > 0 (precise mode): outputs are bf16 hi/lo pairs, the lo halves lo_off elements behind the hi halves.
hipError_t rl_norm(const float* x, const int* row_index, int rows, int d, float eps, const float* g1,
                   const float* b1, uint16_t* out1, const float* g2, const float* b2, uint16_t* out2,
                   int out_rows, int out_row0, unsigned* status, hipStream_t s, size_t lo_off = 0);

// Rotary + KV write.  qkv fp32 [rows, (Hq + 2 Hkv) h] (bias already added) ->
//   q fp16 [rows, Hq h] rotated; k (rotated) and v written as bf16 to the cache of `ncopy` consecutive cache
//   sequences starting at dst_seq[row].
struct RopeArgs {
  const float* qkv; int rows;
  int Hq, Hkv, h, r;
  const float2* table;           // [max_pos, r/2]
  const int* pos;                // [rows] position of each row in its sequence
  const int* dst_seq;            // [rows] first cache sequence receiving the row's k, v
  int ncopy;
  int pos_add;                   // added to pos[] (decode step)
  const int* slot_sub;           // nullable [rows]: cache slot = position - slot_sub[row] (shared prompt cache)
  uint16_t* q;                   // out
  uint16_t* kv; KvLayout lay; const int* kv_off; const int* kv_cap;
  // prompt pass: V is written by a second kernel, one block per 16-token job (dst_seq[row] == jobs[].cache_seq)
  int v_by_blocks; const AttnJob* jobs; int njobs;
  const uint16_t* kvstage;       // rl_kv_prefill: bf16 [rows, 2 Hkv h], rotated k heads then v heads
};
// Moves the staged keys and values of a prompt pass into the cache layout, to every copy; one block per 16-token job.
hipError_t rl_kv_prefill(const RopeArgs& a, hipStream_t s);
hipError_t rl_rope_kv(const RopeArgs& a, hipStream_t s);

// Sampling phase 2 (after the EPI_LMHEAD GEMM): per row, combine the per-64-column partials into
// log Z, find the column group where the CDF crosses u, recompute that group's 64 logits from hfin and
// the LM head, scan it, and emit token and log-prob.  forced nullable.  Output index out_index[row].
struct SampleArgs {
  int precise;                          // hfin holds bf16 hi/lo pairs (lo halves hfin_lo_off elements behind), lm_head bf16
  size_t hfin_lo_off;
  const float2* partial; int ngroups;
  const uint16_t* hfin; int d;          // fp16 [R, d] rows fed to the LM head GEMM (K-block major)
  const uint16_t* lm_head; int vocab;   // fp16 [V, d] (K-block major)
  float temperature;
  const float* uniforms; const int* forced; const int* io_index;  // value index of row i: io_index[i] * io_stride + io_add
  int io_stride, io_add;
  int* tokens; float* logprobs;         // written at the same index
  int* next_token;                      // nullable [R]: copy of the emitted token for the next decode step
  int greedy;                           // 1: the token is the first index of the largest logit (uniforms unused)
  int eos; int* finished;               // eos >= 0 and finished [R] non-null: a row that has emitted eos keeps emitting
                                        // it at log-prob 0 (forced entries ignored)
  int R;
  unsigned* status;
};
hipError_t rl_sample(const SampleArgs& a, hipStream_t s);
// Scoring phase 2: out[out_index[i]] = target_logit[i] - log Z(i)
hipError_t rl_score_finalize(const float2* partial, int ngroups, const float* target_logit, const int* out_index,
                             float* out, int R, hipStream_t s);

hipError_t rl_sequence_logprob(const float* tlp, const int* from, const int* lens, int N, int stride, float* out, hipStream_t s);
hipError_t rl_select_pairs(const float* rewards, int B, int k, int* idx_pos, int* idx_neg, hipStream_t s);
hipError_t rl_dpo_loss(const float* pp, const float* rp, const float* pn, const float* rn, int P, float beta, float* loss, hipStream_t s);
hipError_t rl_proximal_rloo(const float* lp_pol, const float* lp_old, const float* rewards, int B, int k, float eps, float* objective,
                            hipStream_t s);
