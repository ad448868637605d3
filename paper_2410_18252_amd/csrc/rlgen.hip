// Host side of librlgen.so: configuration checks, workspace carving, weight packing and the
// scheduler that turns rlgen_generate / rlgen_score into kernel launches on the caller's stream.
// No device memory is allocated here (no hipMalloc, no hipFree); the host allocations are the context, two pinned
// buffers (per-call sequence metadata; the flags and index lists of EOS compaction), two internal streams and a few events.
#include "../../include/rlgen.h"
#include "kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

// ------------------------------------------------------------------ rlgen_sample_static's scratch
// The final-norm + LM-head + sampling stage needs three intermediate buffers: the normalised rows (16-bit, K-block
// major), the (max, sum exp) pair per row and 64 vocabulary columns, and one captured logit per row.  rlgen_sample_static
// keeps them here instead of in the caller's workspace, for at most STATIC_MAX_ROWS rows of a model with d_model <=
// STATIC_MAX_D and vocab <= 64 STATIC_MAX_GROUPS.  Every GPU the library runs on holds its own copy of the array (about
// 4.3 MB) until the process ends; its address on a device is asked for once, in rlgen_create, with that device current.
constexpr int STATIC_MAX_ROWS = 64, STATIC_MAX_D = 8192, STATIC_MAX_GROUPS = 4096;
constexpr size_t STATIC_HFIN_BYTES = (size_t)STATIC_MAX_ROWS * STATIC_MAX_D * 2 * 2;      // two 16-bit values per element at most
constexpr size_t STATIC_PARTIAL_BYTES = (size_t)STATIC_MAX_ROWS * STATIC_MAX_GROUPS * sizeof(float2);
constexpr size_t STATIC_TARGET_BYTES = 256;
static __device__ __align__(256) unsigned char scratch[STATIC_HFIN_BYTES + STATIC_PARTIAL_BYTES + STATIC_TARGET_BYTES];
static unsigned char* scratch_on_device[64];      // device address of `scratch` per device, null until rlgen_create ran there

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t v, size_t a = ALIGN) { return (v + a - 1) / a * a; }
inline int round32(int v) { return (v + 31) & ~31; }

struct SeqMeta {       // one per sequence of a call, consumed by expand_kernel
  int row0;            // first row of the sequence in its chunk's packed activations
  int len;             // tokens processed by the prompt / scoring pass
  int src_off;         // offset of the sequence's first token in the caller's token array
  int cache_seq;       // cache sequence that receives (the first copy of) its keys and values
  int job0;            // first attention job of the sequence within its chunk
  int lm0;             // first LM-head row of the sequence within its chunk (scoring)
  int score_from;      // first scored position
  int out_off;         // offset of the sequence's row in the output array (scoring)
  // grouped scoring: the sequence is the tail of a caller's sequence whose first pos0 tokens are processed once
  // for the whole group, as the sequence in cache stream pre_seq
  int pos0;            // position of the sequence's first token (0 unless it continues a shared prefix)
  int prev_row;        // row holding the last token of the shared prefix (-1: none): it predicts this sequence's first token
  int pre_seq;         // cache stream of the shared prefix
  int ref_off;         // offset, in the caller's token array, of the group's first sequence (prefixes are compared against it)
};

struct LayerW {
  float *n1g, *n1b, *n2g, *n2b, *bqkv, *bo, *bup, *bdown;
  uint16_t *wqkv, *wo, *wup, *wdown;
};

struct Carve {
  size_t off = 0;
  template <typename T> T* take(char* base, size_t count) {
    T* p = base ? (T*)(base + off) : nullptr;
    off = align_up(off + count * sizeof(T));
    return p;
  }
};

}  // namespace

struct rlgen_ctx {
  rlgen_model_cfg cfg;
  int R;          // activation rows
  int LM;         // rows per LM-head pass
  int ngroups;
  size_t need;
  char* ws;
  // weights
  uint16_t *embed, *lm_head;
  float *fng, *fnb;
  std::vector<LayerW> layers;
  float2* rope;
  uint16_t* kv;
  KvLayout lay;
  unsigned* status;
  // per-call metadata (device)
  SeqMeta* d_meta;
  int *d_kv_off, *d_kv_cap, *d_ctx_base, *d_iota, *d_lastrow, *d_order;
  bool use_order;
  bool fused_qkv;         // rotary_dim % 4 == 0: rotary embedding and cache writes run in the QKV GEMM's epilogue
  int score_groups;       // k > 1: rlgen_score treats every k consecutive sequences as one prompt with k completions
  int eos_token;          // -1: completions never end early (rlgen_set_eos)
  int* d_finished;        // [max_seqs] 1 once a sequence of the running call has emitted eos_token
  int eos_every;          // ended sequences are dropped from the batch every this many decode steps (0: never)
  int *d_cmp, *d_lists;   // compacted per-row arrays (2 sides x 4 x max_seqs) and uploaded index lists (3 x max_seqs)
  int *h_fin, *h_lists;   // pinned: downloaded flags [max_seqs], index lists [3 max_seqs]
  int share_k;            // samples per prompt of the running generate call when prompts share their cache, else 0
  int *d_tok_index, *d_pos, *d_dst_seq, *d_lm_row, *d_target, *d_out_index, *d_next_token;
  AttnJob* d_jobs;
  // activations: the set in use (see Bufs / use_set)
  float *x, *qkv, *target_logit, *splitk;
  size_t splitk_elems;
  uint16_t *n1, *n2, *q, *attn, *act, *hfin;
  float2* partial;
  // Set 0 serves the prompt pass, scoring and a decode of the whole batch.  A large decode batch is cut in two
  // halves that run on two internal streams with sets 1 and 2: while one half streams its KV cache (HBM-bound),
  // the other half's linear layers (matrix-core-bound) share the machine with it.
  struct Bufs {
    float *x, *qkv, *target_logit, *splitk;
    size_t splitk_elems;
    uint16_t *n1, *n2, *q, *attn, *act, *hfin;
    float2* partial;
  } set[3];
  int Sg;                 // rows of sets 1 and 2
  hipStream_t gstream[2];
  hipEvent_t ev_fork, ev_join[2];
  bool have_streams;
  int split_min_seqs;
  bool split_off;         // rlgen_set_decode_split(ctx, 0)
  // host staging (pinned)
  char* h_stage;
  size_t stage_bytes;
  hipEvent_t ev_meta;
  bool meta_pending;
  // timings
  hipEvent_t ev_start, ev_mid, ev_end;
  bool timed;
  int profiling;          // n > 0: every n-th decode-attention launch is bracketed with events
  std::vector<hipEvent_t> prof_events;
  size_t prof_used;
  // tile shape and K split of each linear layer, measured at creation: [decode | prompt pass][which GEMM]
  // [decode of max_seqs rows | prompt pass | decode of half of max_seqs rows][which GEMM]
  struct GemmChoice { int variant, splits; } tuned[3][5];
  bool half_rows;         // the decode steps being enqueued cover half of the batch
  // precise mode (cfg.precise): 16-bit activations and cached keys/values are bf16 hi/lo pairs.  pw = 2 then (else 1):
  // 16-bit values per activation element; kv_plane = elements between the hi and the lo plane of the cache
  int pw;
  long long kv_plane;
  int device;             // the device the context was created on
};

namespace {

int check_cfg(const rlgen_model_cfg* c) {
  if (!c) return RLGEN_ERR_NULL;
  if (c->arch != RLGEN_ARCH_NEOX && c->arch != RLGEN_ARCH_LLAMA) return RLGEN_ERR_BAD_CFG;
  if (c->n_layers < 1 || c->d_model < 32 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 16 ||
      c->d_ffn < 32 || c->vocab < 2)
    return RLGEN_ERR_BAD_CFG;
  if (c->d_model != c->n_q_heads * c->head_dim) return RLGEN_ERR_BAD_CFG;
  if (c->n_q_heads % c->n_kv_heads != 0 || c->n_q_heads / c->n_kv_heads > 16) return RLGEN_ERR_BAD_CFG;
  if (c->arch == RLGEN_ARCH_NEOX && c->n_kv_heads != c->n_q_heads) return RLGEN_ERR_BAD_CFG;
  const int h = c->head_dim;
  if (!(h == 256 || (h % 16 == 0 && h <= 128))) return RLGEN_ERR_BAD_CFG;
  if (c->d_model % 32 != 0 || c->d_ffn % 32 != 0 || c->d_model > 8192) return RLGEN_ERR_BAD_CFG;
  if (c->rotary_dim < 0 || c->rotary_dim % 2 != 0 || c->rotary_dim > h) return RLGEN_ERR_BAD_CFG;
  if (!(c->rope_theta > 0.f) || !std::isfinite(c->rope_theta)) return RLGEN_ERR_BAD_CFG;
  if (!(c->norm_eps > 0.f) || !std::isfinite(c->norm_eps)) return RLGEN_ERR_BAD_CFG;
  if (c->weight_dtype != RLGEN_DTYPE_F32 && c->weight_dtype != RLGEN_DTYPE_BF16) return RLGEN_ERR_BAD_CFG;
  if (c->max_seqs < 1 || c->max_seq_len < 2 || c->max_kv_tokens < round32(c->max_seq_len)) return RLGEN_ERR_BAD_CFG;
  if (c->max_kv_tokens > (1LL << 30) || c->max_seqs > (1 << 20) || c->max_seq_len > (1 << 20)) return RLGEN_ERR_BAD_CFG;
  if (c->max_batch_tokens != 0 && c->max_batch_tokens < c->max_seq_len) return RLGEN_ERR_BAD_CFG;
  if (c->max_batch_tokens > (1 << 22)) return RLGEN_ERR_BAD_CFG;
  if (c->share_prompt_kv != 0 && c->share_prompt_kv != 1) return RLGEN_ERR_BAD_CFG;
  // precise mode runs the fused QKV epilogue only and keeps two cache planes per attention wave in registers
  if (c->precise != 0 && (c->precise != 1 || c->rotary_dim % 4 != 0 || h > 128)) return RLGEN_ERR_BAD_CFG;
  return RLGEN_OK;
}

void use_set(rlgen_ctx* c, int i) {
  const rlgen_ctx::Bufs& b = c->set[i];
  c->x = b.x; c->qkv = b.qkv; c->target_logit = b.target_logit; c->splitk = b.splitk; c->splitk_elems = b.splitk_elems;
  c->n1 = b.n1; c->n2 = b.n2; c->q = b.q; c->attn = b.attn; c->act = b.act; c->hfin = b.hfin; c->partial = b.partial;
}

// Lays the workspace out; with base == nullptr only the size is computed.
size_t carve(rlgen_ctx* c, char* base) {
  const rlgen_model_cfg& m = c->cfg;
  const size_t d = m.d_model, F = m.d_ffn, V = m.vocab, h = m.head_dim;
  const size_t qd = (size_t)m.n_q_heads * h, kvd = (size_t)m.n_kv_heads * h, nqkv = qd + 2 * kvd;
  const bool llama = m.arch == RLGEN_ARCH_LLAMA;
  // default chunk: 32768 rows (128 row tiles of 256: the tile count of every linear layer is then a multiple of
  // the 256 CUs when its width is a multiple of 512), but no more than a call can ever hold
  int mbt = m.max_batch_tokens ? m.max_batch_tokens : (int)std::min<long long>(32768, (long long)m.max_seqs * m.max_seq_len);
  if (mbt < m.max_seq_len) mbt = m.max_seq_len;
  c->R = mbt > m.max_seqs ? mbt : m.max_seqs;
  c->LM = c->R < 4096 ? c->R : 4096;
  if (c->LM < m.max_seqs) c->LM = m.max_seqs;
  c->ngroups = (int)((V + 63) / 64);
  const size_t R = c->R, LM = c->LM, S = m.max_seqs;

  Carve k;
  c->status = k.take<unsigned>(base, 64);
  c->embed = k.take<uint16_t>(base, V * d);
  c->lm_head = k.take<uint16_t>(base, kblk_elems(V, d));
  c->fng = k.take<float>(base, d);
  c->fnb = k.take<float>(base, d);
  c->layers.resize(m.n_layers);
  for (auto& L : c->layers) {
    L.n1g = k.take<float>(base, d); L.n1b = k.take<float>(base, d);
    L.n2g = k.take<float>(base, d); L.n2b = k.take<float>(base, d);
    L.wqkv = k.take<uint16_t>(base, kblk_elems(nqkv, d)); L.bqkv = k.take<float>(base, nqkv);
    L.wo = k.take<uint16_t>(base, kblk_elems(d, qd)); L.bo = k.take<float>(base, d);
    L.wup = k.take<uint16_t>(base, kblk_elems((llama ? 2 : 1) * F, d)); L.bup = k.take<float>(base, F);
    L.wdown = k.take<uint16_t>(base, kblk_elems(d, F)); L.bdown = k.take<float>(base, d);
  }
  c->rope = k.take<float2>(base, (size_t)m.max_seq_len * (m.rotary_dim / 2 > 0 ? m.rotary_dim / 2 : 1));
  c->lay.Hkv = m.n_kv_heads;
  c->lay.h = m.head_dim;
  c->lay.layer_stride = 2LL * m.max_kv_tokens * m.n_kv_heads * m.head_dim;
  c->pw = m.precise ? 2 : 1;
  c->kv_plane = c->lay.layer_stride * m.n_layers;
  c->kv = k.take<uint16_t>(base, (size_t)c->kv_plane * c->pw);
  c->d_meta = k.take<SeqMeta>(base, 2 * S);       // grouped scoring adds one shared prefix per group
  c->d_kv_off = k.take<int>(base, 2 * S); c->d_kv_cap = k.take<int>(base, 2 * S);   // prompt + per-sequence streams
  c->d_ctx_base = k.take<int>(base, S); c->d_iota = k.take<int>(base, S);
  c->d_lastrow = k.take<int>(base, S); c->d_next_token = k.take<int>(base, S);
  c->d_order = k.take<int>(base, S);
  c->d_finished = k.take<int>(base, S + 4);
  c->d_cmp = k.take<int>(base, 8 * S); c->d_lists = k.take<int>(base, 3 * S);
  c->d_tok_index = k.take<int>(base, R); c->d_pos = k.take<int>(base, R); c->d_dst_seq = k.take<int>(base, R);
  c->d_lm_row = k.take<int>(base, R); c->d_target = k.take<int>(base, R); c->d_out_index = k.take<int>(base, R);
  c->d_jobs = k.take<AttnJob>(base, R / 16 + 4 * S + 2);
  c->Sg = (2 * m.max_seqs + 2) / 3 + 1;        // the larger half: ceil(B / 2) prompts of B >= 2, k samples each
  for (int i = 0; i < 3; ++i) {
    const size_t rows = i == 0 ? R : (size_t)c->Sg, lm = i == 0 ? LM : (size_t)c->Sg;
    rlgen_ctx::Bufs& b = c->set[i];
    b.x = k.take<float>(base, rows * d);
    const size_t pw = c->pw;                   // precise mode: hi and lo halves (q: fp32)
    b.n1 = k.take<uint16_t>(base, pw * kblk_elems(rows, d));
    b.n2 = k.take<uint16_t>(base, pw * kblk_elems(rows, d));
    b.qkv = k.take<float>(base, rows * nqkv);
    b.q = k.take<uint16_t>(base, pw * rows * qd);
    b.attn = k.take<uint16_t>(base, pw * kblk_elems(rows, qd));
    b.act = k.take<uint16_t>(base, pw * kblk_elems(rows, F));
    b.hfin = k.take<uint16_t>(base, pw * kblk_elems(lm, d));
    b.partial = k.take<float2>(base, lm * (size_t)c->ngroups);
    b.target_logit = k.take<float>(base, lm);
    b.splitk_elems = (size_t)12 << 20;          // 48 MB of split-K partial sums
    b.splitk = k.take<float>(base, b.splitk_elems);
  }
  use_set(c, 0);
  return k.off;
}

#define HIPCHK(expr) do { if ((expr) != hipSuccess) return RLGEN_ERR_DEVICE; } while (0)

int pack_weights(rlgen_ctx* c, const rlgen_weights* w, hipStream_t st) {
  const rlgen_model_cfg& m = c->cfg;
  const bool llama = m.arch == RLGEN_ARCH_LLAMA;
  const int bf = m.weight_dtype == RLGEN_DTYPE_BF16;
  const size_t d = m.d_model, F = m.d_ffn, V = m.vocab, h = m.head_dim;
  const size_t qd = (size_t)m.n_q_heads * h, kvd = (size_t)m.n_kv_heads * h;
  const int nqkv = (int)(qd + 2 * kvd);
  if (!w || !w->embed_in || !w->final_norm_g || !w->lm_head || !w->layers) return RLGEN_ERR_NULL;
  if (!llama && !w->final_norm_b) return RLGEN_ERR_NULL;
  for (int l = 0; l < m.n_layers; ++l) {
    const rlgen_layer_weights& s = w->layers[l];
    if (!s.norm1_g || !s.norm2_g || !s.wq || !s.wk || !s.wv || !s.wo || !s.w_up || !s.w_down) return RLGEN_ERR_NULL;
    if (llama ? !s.w_gate : (!s.norm1_b || !s.norm2_b || !s.bq || !s.bk || !s.bv || !s.bo || !s.b_up || !s.b_down))
      return RLGEN_ERR_NULL;
  }
  HIPCHK(rl_to_bf16(c->embed, w->embed_in, bf, V * d, st));
  const int pb = m.precise;           // precise mode keeps the bf16 bit patterns
  HIPCHK(rl_to_f16w(c->lm_head, w->lm_head, bf, (int)V, (int)d, (int)V, 0, st, 0, 0, pb));
  HIPCHK(rl_to_f32(c->fng, w->final_norm_g, bf, d, st));
  if (!llama) HIPCHK(rl_to_f32(c->fnb, w->final_norm_b, bf, d, st));
  for (int l = 0; l < m.n_layers; ++l) {
    const rlgen_layer_weights& s = w->layers[l];
    LayerW& L = c->layers[l];
    HIPCHK(rl_to_f32(L.n1g, s.norm1_g, bf, d, st));
    HIPCHK(rl_to_f32(L.n2g, s.norm2_g, bf, d, st));
    // fused QKV epilogue: query and key rows of a head in the order that puts rotary pairs side by side
    const int ph = c->fused_qkv ? (int)h : 0, pr = m.rotary_dim;
    HIPCHK(rl_to_f16w(L.wqkv, s.wq, bf, (int)qd, (int)d, nqkv, 0, st, ph, pr, pb));
    HIPCHK(rl_to_f16w(L.wqkv, s.wk, bf, (int)kvd, (int)d, nqkv, (int)qd, st, ph, pr, pb));
    HIPCHK(rl_to_f16w(L.wqkv, s.wv, bf, (int)kvd, (int)d, nqkv, (int)(qd + kvd), st, 0, 0, pb));
    HIPCHK(rl_to_f16w(L.wo, s.wo, bf, (int)d, (int)qd, (int)d, 0, st, 0, 0, pb));
    HIPCHK(rl_to_f16w(L.wdown, s.w_down, bf, (int)d, (int)F, (int)d, 0, st, 0, 0, pb));
    if (llama) {
      HIPCHK(rl_pack_gate_up(L.wup, s.w_gate, s.w_up, bf, (int)F, (int)d, st, pb));
    } else {
      HIPCHK(rl_to_f16w(L.wup, s.w_up, bf, (int)F, (int)d, (int)F, 0, st, 0, 0, pb));
      HIPCHK(rl_to_f32(L.n1b, s.norm1_b, bf, d, st));
      HIPCHK(rl_to_f32(L.n2b, s.norm2_b, bf, d, st));
      HIPCHK(rl_to_f32(L.bqkv, s.bq, bf, qd, st, ph, pr));
      HIPCHK(rl_to_f32(L.bqkv + qd, s.bk, bf, kvd, st, ph, pr));
      HIPCHK(rl_to_f32(L.bqkv + qd + kvd, s.bv, bf, kvd, st));
      HIPCHK(rl_to_f32(L.bo, s.bo, bf, d, st));
      HIPCHK(rl_to_f32(L.bup, s.b_up, bf, F, st));
      HIPCHK(rl_to_f32(L.bdown, s.b_down, bf, d, st));
    }
  }
  return RLGEN_OK;
}

// Expands per-sequence metadata into the per-row arrays the kernels index.  One block per sequence.
__global__ void expand_kernel(const SeqMeta* meta, int first, const int* tokens, int* tok_index, int* pos, int* dst_seq,
                              AttnJob* jobs, int* lm_row, int* target, int* out_index, int scoring, int job_mult,
                              unsigned* status) {
  const SeqMeta m = meta[first + blockIdx.x];
  for (int p = threadIdx.x; p < m.len; p += blockDim.x) {
    tok_index[m.row0 + p] = m.src_off + p;
    pos[m.row0 + p] = m.pos0 + p;
    dst_seq[m.row0 + p] = m.cache_seq;
  }
  // 16-token blocks, their count rounded up to a multiple of job_mult (the blocks past the end do nothing)
  const int nj = (m.len + 16 * job_mult - 1) / (16 * job_mult) * job_mult;
  for (int j = threadIdx.x; j < nj; j += blockDim.x)
    jobs[m.job0 + j] = AttnJob{m.cache_seq, m.row0, m.len, j, m.pre_seq, m.prev_row >= 0 ? m.pos0 : 0};
  if (scoring && m.prev_row >= 0) {
    // every token of the tail is scored; the first one from the shared prefix's last row
    for (int t = threadIdx.x; t < m.len; t += blockDim.x) {
      lm_row[m.lm0 + t] = t == 0 ? m.prev_row : m.row0 + t - 1;
      target[m.lm0 + t] = tokens[m.src_off + t];
      out_index[m.lm0 + t] = m.out_off + t;
    }
    // the caller declared the first pos0 tokens equal to those of the group's first sequence
    bool same = true;
    for (int p = threadIdx.x; p < m.pos0; p += blockDim.x) same &= tokens[m.src_off - m.pos0 + p] == tokens[m.ref_off + p];
    if (!same) atomicOr(status, RLGEN_FAULT_GROUP);
  } else if (scoring) {
    for (int t = m.score_from + threadIdx.x; t < m.len; t += blockDim.x) {
      const int i = m.lm0 + (t - m.score_from);
      lm_row[i] = m.row0 + t - 1;
      target[i] = tokens[m.src_off + t];
      out_index[i] = m.out_off + t;
    }
  }
}
// Row arrays for the timing runs of the fused QKV projection: consecutive rows belong to different cache sequences
// (as in a decode step), row i being slot (i / nseq) % npos of sequence i % nseq.
__global__ void tune_rows_kernel(int* pos, int* dst_seq, int* kv_off, int* kv_cap, int rows, int nseq, int npos) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < rows) {
    dst_seq[i] = i % nseq;
    pos[i] = (i / nseq) % npos;
  }
  if (i < nseq) {
    kv_off[i] = 32 * i;
    kv_cap[i] = 32;
  }
}
// Rows keep[0 .. n) of a decode batch become rows 0 .. n of the compacted one (none of them has ended).
__global__ void compact_rows_kernel(const int* keep, int n, const int* seq, const int* ctx, const int* next, int* seq2, int* ctx2,
                                    int* next2, int* fin2) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int r = keep[i];
  seq2[i] = seq[r]; ctx2[i] = ctx[r]; next2[i] = next[r]; fin2[i] = 0;
}
// Outputs of steps t .. T - 1 of sequences that ended before step t: the EOS id at log-prob 0.  One block per sequence.
__global__ void fill_tail_kernel(const int* seqs, int t, int T, int eos, int* tokens, float* logprobs) {
  const size_t o = (size_t)seqs[blockIdx.x] * T;
  for (int i = t + threadIdx.x; i < T; i += blockDim.x) { tokens[o + i] = eos; logprobs[o + i] = 0.f; }
}
__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}
__global__ void clamp_targets_kernel(int* target, int n, int vocab, unsigned* status) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int t = target[i];
  if (t < 0 || t >= vocab) {
    atomicOr(status, RLGEN_FAULT_TOKEN);
    target[i] = min(max(t, 0), vocab - 1);
  }
}

struct Chunk { int first, count, rows, jobs, lm_rows; };
// 16-token blocks of a sequence of `len` tokens in the job list: rounded up to what one attention wave takes
int jobs_of(const rlgen_ctx* c, int len) {
  const int per = 16 * rl_attention_prefill_qb(c->cfg.head_dim);
  return (len + per - 1) / per * (per / 16);
}

enum { G_QKV = 0, G_O = 1, G_UP = 2, G_DOWN = 3, G_LMHEAD = 4 };

// variant < 0: the tile shape follows from the problem size.  splits >= 2 needs g.ws.
hipError_t run_choice(const GemmArgs& g, int epi, int variant, int splits, hipStream_t st) {
  GemmArgs h = g;
  h.splits = (splits >= 2 && g.ws) ? splits : 1;
  if (variant < 0) return rl_gemm(h, epi, st);
  if (h.splits >= 2) return rl_gemm_splitk(h, epi, variant, st);
  return rl_gemm_variant(h, epi, variant, st);
}
hipError_t gemm(rlgen_ctx* c, int which, bool decode, const GemmArgs& g, int epi, hipStream_t st) {
  const int mode = decode ? (c->half_rows ? 2 : 0) : 1;
  // the K split is that of the mode's family (decode / prompt pass) even where a mode was not tuned
  return run_choice(g, epi, c->tuned[mode][which].variant, c->tuned[decode ? 0 : 1][which].splits, st);
}

QkvEpi qkv_epilogue(const rlgen_ctx* c, const RopeArgs& r, uint16_t* kvstage) {
  QkvEpi e{};
  e.kv_lo_off = c->kv_plane;                                    // used in precise mode only
  e.stage_lo_off = (long long)r.rows * 2 * r.Hkv * r.h;         // the lo staging rows follow the hi staging rows
  e.Hq = r.Hq; e.Hkv = r.Hkv; e.h = r.h; e.r = r.r; e.inv_h = 1.0f / (float)r.h;
  e.table = r.table; e.pos = r.pos; e.pos_add = r.pos_add; e.slot_sub = r.slot_sub; e.dst_seq = r.dst_seq;
  e.q = r.q; e.kv = r.kv; e.lay = r.lay; e.kv_off = r.kv_off; e.kv_cap = r.kv_cap; e.kvstage = kvstage;
  return e;
}

// One pass of all decoder blocks over `rows` packed rows held in c->x.
//  decode: rows are sequences 0..rows-1 at step t (the token drawn at step t-1 enters at position
//          ctx_base + t - 1); otherwise rows follow d_pos / d_dst_seq / d_jobs of the current chunk.
// A decode step covers sequences g0 .. g0 + rows - 1 (all of the call's, or one half); with a shared prompt cache
// these are the samples of prompts b0 .. of the call's B prompts.
struct DecView {
  int g0, b0, B;
  // compacted batch (after ended sequences were dropped): per-row arrays instead of the per-sequence ones at g0
  const int* row_seq = nullptr; const int* row_ctx = nullptr; int* row_next = nullptr; int* row_fin = nullptr;
  const int* row_order = nullptr;
};
// Below this many sequences a decode step is too short to gain from running as two concurrent halves.
constexpr int DECODE_SPLIT_MIN_SEQS = 256;     // rlgen_set_decode_split_min replaces it

int run_layers(rlgen_ctx* c, int rows, bool decode, int t, int ncopy, bool use_cache_layers, int njobs, hipStream_t st,
               DecView dv = DecView{0, 0, 0}) {
  const rlgen_model_cfg& m = c->cfg;
  const bool llama = m.arch == RLGEN_ARCH_LLAMA;
  const int d = m.d_model, F = m.d_ffn, h = m.head_dim;
  const int qd = m.n_q_heads * h, nqkv = qd + 2 * m.n_kv_heads * h;
  for (int l = 0; l < m.n_layers; ++l) {
    const LayerW& L = c->layers[l];
    uint16_t* kvl = c->kv + (use_cache_layers ? (size_t)c->lay.layer_stride * l : 0);
    const int pr = m.precise;
    // precise mode: distance between the hi and the lo halves of a 16-bit activation matrix of `rows` rows and K columns
    auto lo_off = [&](int K) { return pr ? kblk_elems(rows, K) : (size_t)0; };
    if (llama) HIPCHK(rl_norm(c->x, nullptr, rows, d, m.norm_eps, L.n1g, nullptr, c->n1, nullptr, nullptr, nullptr, rows, 0, c->status, st, lo_off(d)));
    else HIPCHK(rl_norm(c->x, nullptr, rows, d, m.norm_eps, L.n1g, L.n1b, c->n1, L.n2g, L.n2b, c->n2, rows, 0, c->status, st, lo_off(d)));
    GemmArgs g{};
    g.precise = pr;
    g.A = c->n1; g.W = L.wqkv; g.M = rows; g.N = nqkv; g.K = d;
    g.bias = llama ? nullptr : L.bqkv; g.out = c->qkv; g.ldo = nqkv; g.ws = c->splitk; g.ws_elems = c->splitk_elems;
    g.status = c->status;
    RopeArgs r{};
    r.qkv = c->qkv; r.rows = rows; r.Hq = m.n_q_heads; r.Hkv = m.n_kv_heads; r.h = h; r.r = m.rotary_dim;
    r.table = c->rope; r.q = c->q; r.kv = kvl; r.lay = c->lay; r.kv_off = c->d_kv_off; r.kv_cap = c->d_kv_cap;
    if (decode) {
      r.pos = dv.row_seq ? dv.row_ctx : c->d_ctx_base + dv.g0; r.pos_add = t - 1;
      r.dst_seq = dv.row_seq ? dv.row_seq : c->d_iota + dv.g0; r.ncopy = 1;
      r.slot_sub = c->share_k ? c->d_ctx_base + dv.g0 : nullptr;     // new tokens start at slot 0 of their own stream
    }
    else { r.pos = c->d_pos; r.pos_add = 0; r.dst_seq = c->d_dst_seq; r.ncopy = ncopy; r.v_by_blocks = 1; r.jobs = c->d_jobs; r.njobs = njobs; }
    if (c->fused_qkv) {
      // the prompt pass leaves k and v as bf16 rows in the (otherwise unused) fp32 qkv buffer for the block-wise writer
      g.qe = qkv_epilogue(c, r, decode ? nullptr : (uint16_t*)c->qkv);
      g.ws = nullptr;
      HIPCHK(gemm(c, G_QKV, decode, g, EPI_QKV, st));
      if (!decode) {
        r.kvstage = (const uint16_t*)c->qkv;
        HIPCHK(rl_kv_prefill(r, st));
        if (pr) {           // the lo halves: staged behind the hi rows, cached one plane further
          RopeArgs rl = r;
          rl.kvstage = r.kvstage + g.qe.stage_lo_off;
          rl.kv = r.kv + c->kv_plane;
          HIPCHK(rl_kv_prefill(rl, st));
        }
      }
    } else {
      HIPCHK(gemm(c, G_QKV, decode, g, EPI_F32, st));
      HIPCHK(rl_rope_kv(r, st));
    }
    AttnArgs a{};
    a.q = c->q; a.q_ld = qd; a.out = c->attn; a.out_rows = rows; a.kv = kvl; a.lay = c->lay;
    a.kv_off = c->d_kv_off; a.kv_cap = c->d_kv_cap; a.Hq = m.n_q_heads; a.scale = 1.0f / sqrtf((float)h);
    a.precise = pr; a.kv_lo_off = c->kv_plane; a.out_lo_off = lo_off(qd);
    if (decode) {
      // the kernel indexes sequences (prompts, if shared) from 0: hand it the arrays at this view's first entry
      const int u0 = c->share_k ? dv.b0 : dv.g0;
      a.kv_off = c->d_kv_off + u0; a.kv_cap = c->d_kv_cap + u0;
      a.ctx_base = c->d_ctx_base + dv.g0; a.ctx_add = t; a.S = rows; a.order = c->use_order ? c->d_order + u0 : nullptr;
      a.share_k = c->share_k; a.sfx_first = c->share_k ? dv.B + dv.g0 - dv.b0 : 0;
      a.finished = c->eos_token >= 0 ? c->d_finished + dv.g0 : nullptr;
      if (dv.row_seq) {
        a.kv_off = c->d_kv_off; a.kv_cap = c->d_kv_cap; a.cache_seq_of = dv.row_seq; a.ctx_base = dv.row_ctx;
        a.order = dv.row_order; a.finished = dv.row_fin;
      }
      hipEvent_t e0 = nullptr, e1 = nullptr;
      if (c->profiling > 0 && (l + t) % c->profiling == 0) {
        while (c->prof_events.size() < c->prof_used + 2) {
          hipEvent_t e;
          HIPCHK(hipEventCreate(&e));
          c->prof_events.push_back(e);
        }
        e0 = c->prof_events[c->prof_used++];
        e1 = c->prof_events[c->prof_used++];
        HIPCHK(hipEventRecord(e0, st));
      }
      HIPCHK(rl_attention_decode(a, st));
      if (e1) HIPCHK(hipEventRecord(e1, st));
    } else {
      a.jobs = c->d_jobs; a.njobs = njobs;
      HIPCHK(rl_attention_prefill(a, st));
    }
    g = GemmArgs{};
    g.precise = pr;
    g.A = c->attn; g.W = L.wo; g.M = rows; g.N = d; g.K = qd;
    g.bias = llama ? nullptr : L.bo; g.out = c->x; g.ldo = d; g.ws = c->splitk; g.ws_elems = c->splitk_elems;
    HIPCHK(gemm(c, G_O, decode, g, EPI_RESID, st));
    if (llama) HIPCHK(rl_norm(c->x, nullptr, rows, d, m.norm_eps, L.n2g, nullptr, c->n2, nullptr, nullptr, nullptr, rows, 0, c->status, st, lo_off(d)));
    g = GemmArgs{};
    g.precise = pr; g.out_lo_off = lo_off(F);
    g.A = c->n2; g.W = L.wup; g.M = rows; g.N = llama ? 2 * F : F; g.K = d;
    g.bias = llama ? nullptr : L.bup; g.out = c->act; g.ldo = F; g.ws = c->splitk; g.ws_elems = c->splitk_elems;
    g.status = c->status;
    HIPCHK(gemm(c, G_UP, decode, g, llama ? EPI_SWIGLU_F16 : EPI_GELU_F16, st));
    g = GemmArgs{};
    g.precise = pr;
    g.A = c->act; g.W = L.wdown; g.M = rows; g.N = d; g.K = F;
    g.bias = llama ? nullptr : L.bdown; g.out = c->x; g.ldo = d; g.ws = c->splitk; g.ws_elems = c->splitk_elems;
    HIPCHK(gemm(c, G_DOWN, decode, g, EPI_RESID, st));
  }
  return RLGEN_OK;
}

// Final norm of selected rows of c->x into rows out_row0.. of c->hfin (a K-block major matrix of out_rows rows).
int final_norm(rlgen_ctx* c, const int* row_index, int rows, int out_rows, int out_row0, hipStream_t st) {
  const rlgen_model_cfg& m = c->cfg;
  HIPCHK(rl_norm(c->x, row_index, rows, m.d_model, m.norm_eps, c->fng, m.arch == RLGEN_ARCH_LLAMA ? nullptr : c->fnb, c->hfin,
                 nullptr, nullptr, nullptr, out_rows, out_row0, c->status, st, m.precise ? kblk_elems(out_rows, m.d_model) : 0));
  return RLGEN_OK;
}

int lm_head_stats(rlgen_ctx* c, const uint16_t* hfin, int rows, float temperature, const int* target, hipStream_t st) {
  GemmArgs g{};
  g.A = hfin; g.W = c->lm_head;   g.M = rows; g.N = c->cfg.vocab; g.K = c->cfg.d_model;
  g.precise = c->cfg.precise;
  g.temperature = temperature; g.partial = c->partial; g.target = target; g.target_logit = c->target_logit;
  HIPCHK(gemm(c, G_LMHEAD, rows <= c->cfg.max_seqs, g, EPI_LMHEAD, st));
  return RLGEN_OK;
}

// temperature 0 selects greedy decoding: arg max of the logits, log-prob under softmax(z)
int sample_rows(rlgen_ctx* c, int rows, float temperature, const float* uniforms, const int* forced, int io_stride,
                int io_add, int* tokens, float* logprobs, int* next_token, hipStream_t st, int* finished = nullptr,
                const int* io_index = nullptr) {
  const bool greedy = temperature == 0.f;
  if (greedy) temperature = 1.f;
  int rc = lm_head_stats(c, c->hfin, rows, temperature, nullptr, st);
  if (rc) return rc;
  SampleArgs s{};
  s.precise = c->cfg.precise; s.hfin_lo_off = c->cfg.precise ? kblk_elems(rows, c->cfg.d_model) : 0;
  s.partial = c->partial; s.ngroups = c->ngroups; s.hfin = c->hfin; s.d = c->cfg.d_model;
  s.lm_head = c->lm_head; s.vocab = c->cfg.vocab; s.temperature = temperature;
  s.uniforms = uniforms; s.forced = forced; s.io_index = io_index; s.io_stride = io_stride; s.io_add = io_add;
  s.tokens = tokens; s.logprobs = logprobs; s.next_token = next_token; s.R = rows; s.status = c->status;
  s.greedy = greedy ? 1 : 0; s.eos = c->eos_token; s.finished = c->eos_token >= 0 ? finished : nullptr;
  HIPCHK(rl_sample(s, st));
  return RLGEN_OK;
}

// bytes of the weights a decode step reads (fp16 matrices: every layer's and the LM head)
double weight_bytes_of(const rlgen_model_cfg& m) {
  const double qd = (double)m.n_q_heads * m.head_dim, kvd = (double)m.n_kv_heads * m.head_dim;
  const double per_layer = (qd + 2 * kvd) * m.d_model + qd * m.d_model +
                           (m.arch == RLGEN_ARCH_LLAMA ? 3.0 : 2.0) * m.d_ffn * (double)m.d_model;
  return 2.0 * (per_layer * m.n_layers + (double)m.vocab * m.d_model);
}

// How the sum over a linear layer's inner dimension is cut (split-K): a function of the layer's shape and of the
// context's capacity alone, never of a timing, so that a sequence's sums are taken in the same order whichever tile
// shapes a context picked and whether a decode step covers the whole batch, half of it, or what EOS compaction left.
// `rows` is the row count the launches are sized for.  The cut pays when 64x128 tiles leave CUs idle: about two blocks
// per CU, every part keeping at least 4 K tiles, at most 8 parts, and the fp32 partial sums must fit the scratch.
// `beside_attention`: the launches are those of a two-stream decode, which run beside the other half's attention and
// share the path from L2 into the CUs with it; there the extra operand traffic of small tiles and the pass over the
// partial sums cost more than idle CUs do, so the cut stops at one block per CU (measured on the 2.8B shape: 3 parts
// for the 2560-wide projections of a 512-row half are 3 % slower over the decode phase than none).
int split_rule(int rows, int cap_rows, int N, int K, int epi, size_t ws_elems, bool beside_attention) {
  if (epi != EPI_F32 && epi != EPI_RESID && epi != EPI_GELU_F16) return 1;      // the other epilogues have no two-pass form
  const long long t = (long long)((rows + 63) / 64) * ((N + 127) / 128);
  const int nk = (K + 63) / 64;
  long long sp = beside_attention ? 256 / t : (512 + t / 2) / t;
  sp = std::min<long long>(sp, 8);
  sp = std::min<long long>(sp, nk / 4);
  sp = std::min<long long>(sp, (long long)(ws_elems / ((size_t)cap_rows * N)));
  return sp >= 2 ? (int)sp : 1;
}

struct Events3 {      // three timing events, destroyed on every path out of the tuner
  hipEvent_t e[3] = {nullptr, nullptr, nullptr};
  bool create() {
    for (auto& x : e) if (hipEventCreate(&x) != hipSuccess) return false;
    return true;
  }
  ~Events3() { for (auto x : e) if (x) (void)hipEventDestroy(x); }
};

// Is a half-batch decode worth preparing for: the context could hold a batch that decodes as two halves (see
// rlgen_generate), i.e. a full cache would outweigh the weights four times.
bool capacity_splits_decode(const rlgen_ctx* c) {
  const rlgen_model_cfg& m = c->cfg;
  if (!c->have_streams || m.max_seqs < DECODE_SPLIT_MIN_SEQS) return false;
  return 4.0 * m.n_kv_heads * m.head_dim * (double)m.max_kv_tokens * m.n_layers >= 4.0 * weight_bytes_of(m);
}

// Fixes the K split of every linear layer by split_rule, then times the tile shapes on each layer at the row counts it
// will see -- max_seqs rows (or half of them) for a decode step, a full chunk for the prompt pass -- and keeps the
// fastest.  Tile shape does not change the order of any sum.  Inputs are the activation scratch buffers filled with
// pseudo-random fp16; outputs land in scratch.
int tune_gemms(rlgen_ctx* c, hipStream_t st) {
  const rlgen_model_cfg& m = c->cfg;
  const bool llama = m.arch == RLGEN_ARCH_LLAMA;
  const int d = m.d_model, F = m.d_ffn, qd = m.n_q_heads * m.head_dim, nqkv = qd + 2 * m.n_kv_heads * m.head_dim;
  const int pr = m.precise;
  const size_t pw = c->pw;
  HIPCHK(rl_fill_random_f16(c->n1, pw * kblk_elems(c->R, d), 11, st, pr));
  HIPCHK(rl_fill_random_f16(c->n2, pw * kblk_elems(c->R, d), 12, st, pr));
  HIPCHK(rl_fill_random_f16(c->attn, pw * kblk_elems(c->R, qd), 13, st, pr));
  HIPCHK(rl_fill_random_f16(c->act, pw * kblk_elems(c->R, F), 14, st, pr));
  HIPCHK(rl_fill_random_f16(c->hfin, pw * kblk_elems(c->LM, d), 15, st, pr));
  if (pr) HIPCHK(rl_fill_zero(c->q, align_up((size_t)c->R * qd * 4, 16), st));      // fp32 queries of the neighbour attention
  HIPCHK(rl_fill_zero(c->x, align_up((size_t)c->R * d * 4, 16), st));
  {
    const int tseq = (int)std::min<long long>(m.max_seqs, m.max_kv_tokens / 32);
    hipLaunchKernelGGL(tune_rows_kernel, dim3((c->R + 255) / 256), dim3(256), 0, st, c->d_pos, c->d_dst_seq, c->d_kv_off,
                       c->d_kv_cap, c->R, tseq, std::min(32, m.max_seq_len));
    HIPCHK(hipGetLastError());
  }
  Events3 ev;
  if (!ev.create()) return RLGEN_ERR_DEVICE;
  hipEvent_t e0 = ev.e[0], e1 = ev.e[1], e2 = ev.e[2];
  const LayerW& L = c->layers[0];
  int rc = RLGEN_OK;
  const bool tune_half = capacity_splits_decode(c);
  // rows a decode launch is sized for
  const int dec_rows_eff = tune_half ? (m.max_seqs + 1) / 2 : m.max_seqs;
  for (int which = 0; which < 5; ++which) c->tuned[2][which] = {-1, 1};
  // The neighbour of the half-batch timing runs: the decode attention of the other half, over half a full batch of
  // sequences that each hold their share of the cache (all zeros), twice in a row.  Its three per-sequence arrays
  // live in the (idle) index area of EOS compaction and are uploaded from that feature's pinned buffer.
  AttnArgs nb{};
  float nb_ms = 0.f;
  if (tune_half) {
    const int Sh = (m.max_seqs + 1) / 2;
    const int cap = (int)std::min<long long>(m.max_kv_tokens / m.max_seqs, m.max_seq_len) / 32 * 32;
    if (cap >= 32 && (long long)Sh * cap * 2 * m.n_kv_heads * m.head_dim <= c->lay.layer_stride) {
      int* meta = c->h_fin;                       // 4 * max_seqs ints, pinned
      int* nb_meta = c->d_cmp;                    // 8 * max_seqs ints
      for (int i = 0; i < Sh; ++i) { meta[i] = i * cap; meta[Sh + i] = cap; meta[2 * Sh + i] = cap - 1; }
      bool ok = hipMemcpyAsync(nb_meta, meta, (size_t)3 * Sh * sizeof(int), hipMemcpyHostToDevice, st) == hipSuccess &&
                rl_fill_zero(c->kv, (size_t)Sh * cap * 2 * m.n_kv_heads * m.head_dim * 2, st) == hipSuccess;
      nb.q = c->q; nb.q_ld = qd; nb.out = (uint16_t*)c->qkv; nb.out_rows = Sh; nb.kv = c->kv; nb.lay = c->lay;
      nb.kv_off = nb_meta; nb.kv_cap = nb_meta + Sh; nb.ctx_base = nb_meta + 2 * Sh; nb.ctx_add = 1; nb.S = Sh;
      nb.Hq = m.n_q_heads; nb.scale = 1.0f / sqrtf((float)m.head_dim);
      nb.precise = pr; nb.kv_lo_off = c->kv_plane; nb.out_lo_off = pr ? kblk_elems(Sh, qd) : 0;
      if (pr && ok) ok = rl_fill_zero(c->kv + c->kv_plane, (size_t)Sh * cap * 2 * m.n_kv_heads * m.head_dim * 2, st) == hipSuccess;
      for (int r = 0; ok && r < 2; ++r) {          // the second pair is the timed one
        ok = hipEventRecord(e0, st) == hipSuccess && rl_attention_decode(nb, st) == hipSuccess &&
             rl_attention_decode(nb, st) == hipSuccess && hipEventRecord(e1, st) == hipSuccess &&
             hipEventSynchronize(e1) == hipSuccess && hipEventElapsedTime(&nb_ms, e0, e1) == hipSuccess;
      }
      if (!ok) return RLGEN_ERR_DEVICE;
    }
  }
  const int modes[3] = {2, 0, 1};
  for (int mi = tune_half ? 0 : 1; mi < 3 && rc == RLGEN_OK; ++mi) {
    const int mode = modes[mi];
    for (int which = 0; which < 5 && rc == RLGEN_OK; ++which) {
      GemmArgs g{};
      g.precise = pr;
      int epi = EPI_F32;
      // a decode step sees max_seqs rows, or about half of them when the batch is split in two
      const int dec_rows = mode == 2 ? (m.max_seqs + 1) / 2 : m.max_seqs;
      g.M = mode != 1 ? dec_rows : c->R;
      g.ws = c->splitk; g.ws_elems = c->splitk_elems;
      switch (which) {
        case G_QKV:
          g.A = c->n1; g.W = L.wqkv; g.N = nqkv; g.K = d; g.bias = llama ? nullptr : L.bqkv; g.out = c->qkv; g.ldo = nqkv; epi = EPI_F32;
          if (c->fused_qkv) {
            // rows spread over `tseq` cache sequences of 32 slots each, as tune_rows_kernel laid out
            RopeArgs r{};
            r.Hq = m.n_q_heads; r.Hkv = m.n_kv_heads; r.h = m.head_dim; r.r = m.rotary_dim; r.table = c->rope; r.q = c->q;
            r.kv = c->kv; r.lay = c->lay; r.kv_off = c->d_kv_off; r.kv_cap = c->d_kv_cap;
            r.pos = c->d_pos; r.dst_seq = c->d_dst_seq; r.ncopy = 1; r.rows = g.M;
            g.qe = qkv_epilogue(c, r, mode != 1 ? nullptr : (uint16_t*)c->qkv);
            g.ws = nullptr;          // the fused epilogue has no split-K form
            epi = EPI_QKV;
          }
          break;
        case G_O: g.A = c->attn; g.W = L.wo; g.N = d; g.K = qd; g.bias = llama ? nullptr : L.bo; g.out = c->x; g.ldo = d; epi = EPI_RESID; break;
        case G_UP: g.A = c->n2; g.W = L.wup; g.N = llama ? 2 * F : F; g.K = d; g.bias = llama ? nullptr : L.bup; g.out = c->act; g.ldo = F;
                   g.out_lo_off = pr ? kblk_elems(g.M, F) : 0;
                   epi = llama ? EPI_SWIGLU_F16 : EPI_GELU_F16; break;
        case G_DOWN: g.A = c->act; g.W = L.wdown; g.N = d; g.K = F; g.bias = llama ? nullptr : L.bdown; g.out = c->x; g.ldo = d; epi = EPI_RESID;
                     break;
        case G_LMHEAD: g.A = c->hfin; g.W = c->lm_head; g.M = mode != 1 ? dec_rows : c->LM; g.N = m.vocab; g.K = d; g.temperature = 1.f;
                       g.partial = c->partial; g.ws = nullptr; epi = EPI_LMHEAD; break;
      }
      const bool wide_only = epi == EPI_SWIGLU_F16 || epi == EPI_LMHEAD;
      // the K split: by rule, the same for every decode mode
      const int splits = !g.ws ? 1 : mode == 1 ? split_rule(c->R, c->R, g.N, g.K, epi, g.ws_elems, false)
                                               : split_rule(dec_rows_eff, m.max_seqs, g.N, g.K, epi, g.ws_elems, tune_half);
      std::vector<int> cands = {0, 5};
      if (splits == 1) { cands.push_back(3); if (!pr) cands.push_back(10); }
      if (mode == 2 && splits == 1 && !pr) { cands.push_back(1); cands.push_back(4); }     // beside attention other shapes can win
      if (!wide_only) {
        cands.push_back(7);
        // deeper load pipeline: pays on a long K with few tiles (precise mode is compiled for four tile shapes only)
        if (g.K % 64 == 0 && g.K >= 2048 * splits && g.M <= 2048 && !pr) { cands.push_back(8); cands.push_back(9); }
      }
      // clocks drift with load, so the candidates take turns: one warm-up each, then three rounds in which
      // every candidate is timed over two launches; the smallest total wins
      std::vector<float> total(cands.size(), 0.f);
      bool ok = true;
      for (size_t i = 0; ok && i < cands.size(); ++i) ok = run_choice(g, epi, cands[i], splits, st) == hipSuccess;
      for (int round = 0; ok && round < 3; ++round)
        for (size_t i = 0; ok && i < cands.size(); ++i) {
          ok = hipEventRecord(e0, st) == hipSuccess;
          for (int r = 0; ok && r < 2; ++r) ok = run_choice(g, epi, cands[i], splits, st) == hipSuccess;
          if (ok) ok = hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
          float ms = 0.f;
          if (ok) ok = hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
          total[i] += ms;
        }
      if (!ok) { rc = RLGEN_ERR_DEVICE; break; }
      // A half-batch GEMM runs beside the other half's attention, and both live on the path from L2 into the CUs:
      // what counts there is how much longer the neighbour takes, not the GEMM's time alone (on the 2.8B shape 256x128
      // tiles win for QKV and FFN-up although 64x128 tiles are 25 % faster alone: 6 % off the decode phase).  So the
      // half-batch candidates are timed again beside the attention of the other half: [two attention launches ||
      // `reps` GEMMs], with reps small enough that the GEMMs end first.  A candidate's cost is what it adds to the
      // attention's time plus its own time in that company (the two halves take turns, so both are on the clock).
      std::vector<float> score(total);
      // (only from 512 rows up: with fewer, the 256-row tiles that pay in company leave most CUs without a block, and
      // on the 1B shape with 256-row halves the joint choice was 0-5 % slower than the choice by time alone)
      if (mode == 2 && nb_ms > 0.f && which != G_LMHEAD && g.M >= 512 && ok) {
        float best_alone = total[0];
        for (float t : total) best_alone = std::min(best_alone, t);
        best_alone /= 6.f;                                       // ms per launch
        const int reps = std::max(1, std::min(8, (int)(nb_ms / (4.f * best_alone))));
        std::fill(score.begin(), score.end(), 0.f);
        auto joint = [&](size_t i) {
          ok = hipEventRecord(e0, st) == hipSuccess && hipEventRecord(c->ev_fork, st) == hipSuccess &&
               hipStreamWaitEvent(c->gstream[0], c->ev_fork, 0) == hipSuccess &&
               hipStreamWaitEvent(c->gstream[1], c->ev_fork, 0) == hipSuccess &&
               rl_attention_decode(nb, c->gstream[0]) == hipSuccess && rl_attention_decode(nb, c->gstream[0]) == hipSuccess;
          for (int r = 0; ok && r < reps; ++r)
            ok = run_choice(g, epi, cands[i], splits, c->gstream[1]) == hipSuccess;
          if (ok) ok = hipEventRecord(e2, c->gstream[1]) == hipSuccess;
          for (int gi = 0; ok && gi < 2; ++gi)
            ok = hipEventRecord(c->ev_join[gi], c->gstream[gi]) == hipSuccess &&
                 hipStreamWaitEvent(st, c->ev_join[gi], 0) == hipSuccess;
          if (ok) ok = hipEventRecord(e1, st) == hipSuccess && hipEventSynchronize(e1) == hipSuccess;
          float ms = 0.f, ms_gemms = 0.f;
          if (ok) ok = hipEventElapsedTime(&ms, e0, e1) == hipSuccess && hipEventElapsedTime(&ms_gemms, e0, e2) == hipSuccess;
          // per GEMM: what it adds to the neighbour's time, plus how long the half that runs it waits for it
          return ((ms - nb_ms) + ms_gemms) / (float)reps;
        };
        for (int round = 0; ok && round < 3; ++round)
          for (size_t i = 0; ok && i < cands.size(); ++i) score[i] += joint(i) / 3.f;
        // the leaders (and the candidate that is fastest alone) take turns again, often enough to tell them apart
        if (ok) {
          size_t alone_i = 0;
          for (size_t i = 1; i < cands.size(); ++i) if (total[i] < total[alone_i]) alone_i = i;
          std::vector<size_t> lead(cands.size());
          for (size_t i = 0; i < lead.size(); ++i) lead[i] = i;
          std::sort(lead.begin(), lead.end(), [&](size_t x, size_t y) { return score[x] < score[y]; });
          if (lead.size() > 3) lead.resize(3);
          if (std::find(lead.begin(), lead.end(), alone_i) == lead.end()) lead.push_back(alone_i);
          std::vector<float> fine(cands.size(), 0.f);
          for (int round = 0; ok && round < 12; ++round)
            for (size_t i : lead) { if (!ok) break; fine[i] += joint(i) / 12.f; }
          for (size_t i = 0; i < cands.size(); ++i)
            score[i] = std::find(lead.begin(), lead.end(), i) != lead.end() ? fine[i] : std::max(score[i], 1e30f);
        }
        if (!ok) { rc = RLGEN_ERR_DEVICE; break; }
      }
      size_t bi = 0, alone = 0;
      for (size_t i = 1; i < cands.size(); ++i) {
        if (score[i] < score[bi]) bi = i;
        if (total[i] < total[alone]) alone = i;
      }
      // the joint timing is the noisier one: the candidate that is fastest alone is kept unless another one is clearly
      // cheaper in company
      if (score[bi] > 0.985f * score[alone]) bi = alone;
      c->tuned[mode][which] = {cands[bi], splits};
    }
  }
  return rc;
}

// Waits until the previous call's metadata upload has left the staging buffer.
int stage_begin(rlgen_ctx* c) {
  if (c->meta_pending) {
    HIPCHK(hipEventSynchronize(c->ev_meta));
    c->meta_pending = false;
  }
  return RLGEN_OK;
}

struct Staged {
  SeqMeta* meta; int *kv_off, *kv_cap, *ctx_base, *iota, *lastrow, *order;
};
Staged stage_views(rlgen_ctx* c) {
  const size_t S = c->cfg.max_seqs;
  char* p = c->h_stage;
  Staged s;
  s.meta = (SeqMeta*)p; p += align_up(2 * S * sizeof(SeqMeta));
  s.kv_off = (int*)p; p += align_up(2 * S * 4);
  s.kv_cap = (int*)p; p += align_up(2 * S * 4);
  s.ctx_base = (int*)p; p += align_up(S * 4);
  s.iota = (int*)p; p += align_up(S * 4);
  s.lastrow = (int*)p; p += align_up(S * 4);
  s.order = (int*)p;
  return s;
}
int stage_upload(rlgen_ctx* c, const Staged& s, int nmeta, int nseq, int nstreams, hipStream_t st) {
  HIPCHK(hipMemcpyAsync(c->d_meta, s.meta, (size_t)nmeta * sizeof(SeqMeta), hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_kv_off, s.kv_off, (size_t)nstreams * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_kv_cap, s.kv_cap, (size_t)nstreams * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_ctx_base, s.ctx_base, (size_t)nseq * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_iota, s.iota, (size_t)nseq * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_lastrow, s.lastrow, (size_t)nseq * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipMemcpyAsync(c->d_order, s.order, (size_t)nseq * 4, hipMemcpyHostToDevice, st));
  HIPCHK(hipEventRecord(c->ev_meta, st));
  c->meta_pending = true;
  return RLGEN_OK;
}

int expand(rlgen_ctx* c, const Chunk& ch, const int* tokens, bool scoring, hipStream_t st) {
  hipLaunchKernelGGL(expand_kernel, dim3(ch.count), dim3(256), 0, st, c->d_meta, ch.first, tokens, c->d_tok_index, c->d_pos,
                     c->d_dst_seq, c->d_jobs, c->d_lm_row, c->d_target, c->d_out_index, scoring ? 1 : 0,
                     rl_attention_prefill_qb(c->cfg.head_dim), c->status);
  HIPCHK(hipGetLastError());
  return RLGEN_OK;
}

// Teacher-forced pass shared by rlgen_score (logits == nullptr) and rlgen_debug_logits.
int score_impl(rlgen_ctx* c, const int32_t* seqs, const int32_t* seq_lens, const int32_t* score_from, int N, int stride,
               float temperature, float* out, float* logits, hipStream_t st) {
  if (!c || !seqs || !seq_lens || (!out && !logits)) return RLGEN_ERR_NULL;
  const rlgen_model_cfg& m = c->cfg;
  if (N < 1 || stride < 1) return RLGEN_ERR_BAD_ARG;
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return RLGEN_ERR_BAD_ARG;
  if (N > m.max_seqs) return RLGEN_ERR_CAPACITY;
  if ((long long)N * stride > INT32_MAX) return RLGEN_ERR_BAD_ARG;          // token and output offsets are 32-bit
  for (int n = 0; n < N; ++n) {
    if (seq_lens[n] < 1 || seq_lens[n] > stride) return RLGEN_ERR_BAD_ARG;
    if (seq_lens[n] > m.max_seq_len) return RLGEN_ERR_CAPACITY;
  }
  // Grouped scoring (rlgen_set_score_groups): the k sequences of a group share their first score_from tokens, which
  // are processed once, as a sequence of their own whose keys and values every member's tail attends to.
  const int gk = (!logits && c->score_groups > 1) ? c->score_groups : 1;
  if (gk > 1) {
    if (N % gk != 0 || !score_from) return RLGEN_ERR_BAD_ARG;
    for (int n0 = 0; n0 < N; n0 += gk)
      for (int j = 0; j < gk; ++j)
        if (score_from[n0 + j] != score_from[n0] || score_from[n0] < 1 || score_from[n0] > seq_lens[n0 + j]) return RLGEN_ERR_BAD_ARG;
  }
  int rc = stage_begin(c);
  if (rc) return rc;
  Staged s = stage_views(c);
  std::vector<Chunk> chunks;
  int nmeta = 0;
  // (the separate rotary kernel of the unfused path places keys by position, not by position within the tail: there
  // the call scores plainly)
  bool grouped = gk > 1 && c->fused_qkv;
  if (grouped) {
    Chunk cur{0, 0, 0, 0, 0};
    long long kvtok = 0;
    int vs = 0;                               // virtual sequences: one shared prefix per group, one tail per member
    for (int n0 = 0; n0 < N && grouped; n0 += gk) {
      const int P = score_from[n0];
      long long rows_g = P, kv_g = round32(P);
      for (int j = 0; j < gk; ++j)
        if (seq_lens[n0 + j] > P) { rows_g += seq_lens[n0 + j] - P; kv_g += round32(seq_lens[n0 + j] - P); }
      if (rows_g > c->R || kv_g > m.max_kv_tokens) { grouped = false; break; }     // a group must fit one chunk: score plainly
      if (cur.count && (cur.rows + rows_g > c->R || kvtok + kv_g > m.max_kv_tokens)) {
        chunks.push_back(cur);
        cur = Chunk{vs, 0, 0, 0, 0};
        kvtok = 0;
      }
      auto add = [&](int len, int src_off, int out_off) -> SeqMeta& {
        SeqMeta& e = s.meta[vs];
        e = SeqMeta{};
        e.prev_row = -1;
        e.row0 = cur.rows; e.len = len; e.src_off = src_off; e.cache_seq = vs; e.job0 = cur.jobs; e.lm0 = cur.lm_rows;
        e.score_from = len; e.out_off = out_off;
        s.kv_off[vs] = (int)kvtok; s.kv_cap[vs] = round32(len);
        kvtok += round32(len);
        ++vs;
        cur.count++; cur.rows += len; cur.jobs += jobs_of(c, len);
        return e;
      };
      const int pre_vs = vs;
      add(P, n0 * stride, n0 * stride);
      const int last_prefix_row = cur.rows - 1;
      for (int j = 0; j < gk; ++j) {
        const int n = n0 + j, L = seq_lens[n] - P;
        if (L <= 0) continue;
        const int lm0 = cur.lm_rows;
        SeqMeta& e = add(L, n * stride + P, n * stride + P);
        e.lm0 = lm0; e.pos0 = P; e.prev_row = last_prefix_row; e.pre_seq = pre_vs; e.ref_off = n0 * stride;
        cur.lm_rows += L;
      }
    }
    if (grouped) {
      chunks.push_back(cur);
      nmeta = vs;
    } else {
      chunks.clear();
    }
  }
  if (!grouped) {
    Chunk cur{0, 0, 0, 0, 0};
    long long kvtok = 0;
    for (int n = 0; n < N; ++n) {
      const int len = seq_lens[n];
      const int from = logits ? len : std::max(1, score_from ? score_from[n] : 1);
      const int nlm = logits ? 1 : std::max(0, len - from);
      if (cur.count && (cur.rows + len > c->R || kvtok + round32(len) > m.max_kv_tokens)) {
        chunks.push_back(cur);
        cur = Chunk{n, 0, 0, 0, 0};
        kvtok = 0;
      }
      SeqMeta& e = s.meta[n];
      e = SeqMeta{};
      e.prev_row = -1;
      e.row0 = cur.rows; e.len = len; e.src_off = n * stride; e.cache_seq = n; e.job0 = cur.jobs;
      e.lm0 = cur.lm_rows; e.score_from = from; e.out_off = n * stride;
      s.kv_off[n] = (int)kvtok; s.kv_cap[n] = round32(len);
      s.ctx_base[n] = len; s.iota[n] = n; s.lastrow[n] = cur.rows + len - 1; s.order[n] = n;
      kvtok += round32(len);
      cur.count++; cur.rows += len; cur.jobs += jobs_of(c, len); cur.lm_rows += nlm;
    }
    chunks.push_back(cur);
    nmeta = N;
  }
  rc = stage_upload(c, s, nmeta, grouped ? 0 : N, nmeta, st);
  if (rc) return rc;
  if (c->timed) HIPCHK(hipEventRecord(c->ev_start, st));
  if (!logits) {
    hipLaunchKernelGGL(fill_f32_kernel, dim3(std::min<size_t>(((size_t)N * stride + 255) / 256, 65536)), dim3(256), 0, st, out,
                       (size_t)N * stride, 0.f);
    HIPCHK(hipGetLastError());
  }
  for (const Chunk& ch : chunks) {
    rc = expand(c, ch, seqs, !logits, st);
    if (rc) return rc;
    HIPCHK(rl_embed(c->x, c->embed, seqs, c->d_tok_index, ch.rows, m.d_model, m.vocab, c->status, st));
    rc = run_layers(c, ch.rows, false, 0, 1, false, ch.jobs, st);
    if (rc) return rc;
    if (logits) {
      rc = final_norm(c, c->d_lastrow + ch.first, ch.count, ch.count, 0, st);
      if (rc) return rc;
      GemmArgs g{};
      g.A = c->hfin; g.W = c->lm_head; g.M = ch.count; g.N = m.vocab; g.K = m.d_model; g.precise = m.precise;
      g.out = logits + (size_t)ch.first * m.vocab; g.ldo = m.vocab;
      HIPCHK(rl_gemm(g, EPI_F32, st));
    } else {
      if (ch.lm_rows > 0) {
        hipLaunchKernelGGL(clamp_targets_kernel, dim3((ch.lm_rows + 255) / 256), dim3(256), 0, st, c->d_target, ch.lm_rows,
                           m.vocab, c->status);
        HIPCHK(hipGetLastError());
      }
      for (int r0 = 0; r0 < ch.lm_rows; r0 += c->LM) {
        const int nr = std::min(c->LM, ch.lm_rows - r0);
        rc = final_norm(c, c->d_lm_row + r0, nr, nr, 0, st);
        if (rc) return rc;
        rc = lm_head_stats(c, c->hfin, nr, temperature, c->d_target + r0, st);
        if (rc) return rc;
        HIPCHK(rl_score_finalize(c->partial, c->ngroups, c->target_logit, c->d_out_index + r0, out, nr, st));
      }
    }
  }
  if (c->timed) {
    HIPCHK(hipEventRecord(c->ev_mid, st));
    HIPCHK(hipEventRecord(c->ev_end, st));
  }
  return RLGEN_OK;
}

}  // namespace

extern "C" {

size_t rlgen_workspace_bytes(const rlgen_model_cfg* cfg) {
  if (check_cfg(cfg) != RLGEN_OK) return 0;
  rlgen_ctx tmp{};
  tmp.cfg = *cfg;
  return carve(&tmp, nullptr);
}

int rlgen_create(const rlgen_model_cfg* cfg, const rlgen_weights* weights, void* workspace, size_t workspace_bytes,
                 void* hip_stream, rlgen_ctx** out) {
  if (!cfg || !weights || !workspace || !out) return RLGEN_ERR_NULL;
  int rc = check_cfg(cfg);
  if (rc) return rc;
  rlgen_ctx* c = new (std::nothrow) rlgen_ctx{};
  if (!c) return RLGEN_ERR_DEVICE;
  c->cfg = *cfg;
  c->need = carve(c, nullptr);
  if (workspace_bytes < c->need || ((uintptr_t)workspace) % ALIGN != 0) {
    delete c;
    return RLGEN_ERR_WORKSPACE;
  }
  c->ws = (char*)workspace;
  carve(c, c->ws);
  hipStream_t st = (hipStream_t)hip_stream;
  const size_t S = cfg->max_seqs;
  c->stage_bytes = align_up(2 * S * sizeof(SeqMeta)) + 4 * align_up(S * 4) + 2 * align_up(2 * S * 4);
  auto fail = [&](int code) {
    rlgen_destroy(c);
    return code;
  };
  if (hipHostMalloc((void**)&c->h_stage, c->stage_bytes, hipHostMallocDefault) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  if (hipEventCreateWithFlags(&c->ev_meta, hipEventDisableTiming) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  if (hipEventCreate(&c->ev_start) != hipSuccess || hipEventCreate(&c->ev_mid) != hipSuccess ||
      hipEventCreate(&c->ev_end) != hipSuccess)
    return fail(RLGEN_ERR_DEVICE);
  c->timed = true;
  c->eos_token = -1;
  c->eos_every = 8;
  if (hipHostMalloc((void**)&c->h_fin, (size_t)4 * S * sizeof(int), hipHostMallocDefault) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  c->h_lists = c->h_fin + S;
  // two internal streams (default priority) for the halves of a large decode batch
  if (hipStreamCreateWithFlags(&c->gstream[0], hipStreamNonBlocking) != hipSuccess ||
      hipStreamCreateWithFlags(&c->gstream[1], hipStreamNonBlocking) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_join[0], hipEventDisableTiming) != hipSuccess ||
      hipEventCreateWithFlags(&c->ev_join[1], hipEventDisableTiming) != hipSuccess)
    return fail(RLGEN_ERR_DEVICE);
  c->have_streams = true;
  c->split_min_seqs = DECODE_SPLIT_MIN_SEQS;
  c->fused_qkv = cfg->rotary_dim % 4 == 0;
  {
    // where this device keeps the scratch array of rlgen_sample_static (the array's name is no device address)
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(RLGEN_ERR_DEVICE);
    if (!scratch_on_device[dev]) {
      unsigned char* ptr = nullptr;
      if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return fail(RLGEN_ERR_DEVICE);
      scratch_on_device[dev] = ptr;
    }
    c->device = dev;
  }
  rc = pack_weights(c, weights, st);
  if (rc) return fail(rc);
  if (rl_rope_table(c->rope, cfg->max_seq_len, cfg->rotary_dim, cfg->rope_theta, st) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  for (auto& row : c->tuned) for (auto& ch : row) ch = {-1, 1};
  rc = tune_gemms(c, st);
  if (rc) return fail(rc);
  if (rl_fill_zero(c->status, 256, st) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  // The cache must hold finite values everywhere: a partly filled super-block is read whole and the
  // unused keys are masked to probability zero, which only cancels finite values.
  if (rl_fill_zero(c->kv, (size_t)c->kv_plane * c->pw * 2, st) != hipSuccess) return fail(RLGEN_ERR_DEVICE);
  *out = c;
  return RLGEN_OK;
}

int rlgen_update_weights(rlgen_ctx* ctx, const rlgen_weights* weights, void* hip_stream) {
  if (!ctx || !weights) return RLGEN_ERR_NULL;
  return pack_weights(ctx, weights, (hipStream_t)hip_stream);
}

int rlgen_generate(rlgen_ctx* c, const int32_t* prompts, const int32_t* prompt_lens, int32_t B, int32_t prompt_stride,
                   int32_t k, int32_t max_new, float temperature, const float* uniforms, const int32_t* forced,
                   int32_t* tokens, float* token_logprobs, void* hip_stream) {
  if (!c || !prompts || !prompt_lens || !uniforms || !tokens || !token_logprobs) return RLGEN_ERR_NULL;
  const rlgen_model_cfg& m = c->cfg;
  if (B < 1 || k < 1 || max_new < 1 || prompt_stride < 1) return RLGEN_ERR_BAD_ARG;
  if (!(temperature >= 0.f) || !std::isfinite(temperature)) return RLGEN_ERR_BAD_ARG;      // 0 = greedy
  if ((long long)B * k > m.max_seqs) return RLGEN_ERR_CAPACITY;
  if ((long long)B * prompt_stride > INT32_MAX || (long long)B * k * max_new > INT32_MAX) return RLGEN_ERR_BAD_ARG;   // 32-bit offsets
  // shared prompt cache: one stream per prompt plus one short stream of new tokens per sequence; the k samples
  // of a prompt and the query heads of a kv head share the 16 columns of the attention MFMA
  const bool share = m.share_prompt_kv != 0;
  if (share && (long long)k * (m.n_q_heads / m.n_kv_heads) > 16) return RLGEN_ERR_BAD_ARG;
  long long kvtok = 0;
  for (int b = 0; b < B; ++b) {
    if (prompt_lens[b] < 1 || prompt_lens[b] > prompt_stride) return RLGEN_ERR_BAD_ARG;
    if ((long long)prompt_lens[b] + max_new > m.max_seq_len) return RLGEN_ERR_CAPACITY;
    kvtok += share ? round32(prompt_lens[b]) + (long long)k * round32(max_new) : (long long)k * round32(prompt_lens[b] + max_new);
  }
  if (kvtok > m.max_kv_tokens) return RLGEN_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)hip_stream;
  const int S = B * k;
  int rc = stage_begin(c);
  if (rc) return rc;
  Staged s = stage_views(c);
  std::vector<Chunk> chunks;
  Chunk cur{0, 0, 0, 0, 0};
  long long off = 0;
  for (int b = 0; b < B; ++b) {
    const int len = prompt_lens[b];
    if (cur.count && cur.rows + len > c->R) {
      chunks.push_back(cur);
      cur = Chunk{b, 0, 0, 0, 0};
    }
    SeqMeta& e = s.meta[b];
    e = SeqMeta{};
    e.prev_row = -1;
    e.row0 = cur.rows; e.len = len; e.src_off = b * prompt_stride; e.cache_seq = share ? b : b * k; e.job0 = cur.jobs;
    e.lm0 = 0; e.score_from = len; e.out_off = 0;
    if (share) {
      s.kv_off[b] = (int)off; s.kv_cap[b] = round32(len);
      off += round32(len);
    }
    for (int j = 0; j < k; ++j) {
      const int q = b * k + j;
      s.ctx_base[q] = len; s.lastrow[q] = cur.rows + len - 1;
      if (share) {
        s.iota[q] = B + q;       // the stream that takes sequence q's new tokens
      } else {
        s.iota[q] = q;
        s.kv_off[q] = (int)off; s.kv_cap[q] = round32(len + max_new);
        off += round32(len + max_new);
      }
    }
    cur.count++; cur.rows += len; cur.jobs += jobs_of(c, len);
  }
  chunks.push_back(cur);
  if (share)
    for (int q = 0; q < S; ++q) {
      s.kv_off[B + q] = (int)off; s.kv_cap[B + q] = round32(max_new);
      off += round32(max_new);
    }
  // A large batch decodes as two halves (whole prompts each) on two streams.  Each half's attention launch takes
  // its sequences (prompts, if they share their cache) longest context first when there are few jobs per CU, so
  // that the launch does not end on a handful of long ones; the order is local to the half.
  // Splitting reads the weights twice per step, so it pays only when the cache traffic of a step dwarfs them.
  bool split = c->have_streams && !c->split_off && B >= 2 && S >= c->split_min_seqs;
  if (split && c->split_min_seqs == DECODE_SPLIT_MIN_SEQS) {
    const double kvd = (double)m.n_kv_heads * m.head_dim;
    const double weight_bytes = weight_bytes_of(m);
    double ctx = 0;
    for (int b = 0; b < B; ++b) ctx += (share ? 1.0 : (double)k) * prompt_lens[b] + (double)k * max_new * 0.5;
    const double kv_bytes = 4.0 * kvd * ctx * m.n_layers;
    split = kv_bytes >= 4.0 * weight_bytes;
  }
  // with EOS set and one cache per sequence, ended sequences leave the batch (single stream; see the decode loop)
  const bool compacting = c->eos_token >= 0 && !share && c->eos_every > 0 && max_new > 1;
  if (compacting) split = false;
  const int ngroups = split ? 2 : 1;
  const int Bh = ngroups == 2 ? (B + 1) / 2 : B;       // the larger half: at most 2/3 of B * k <= max_seqs rows (B >= 2)
  {
    const int unit_k = share ? 1 : k;                 // order entries per prompt
    for (int gi = 0; gi < ngroups; ++gi) {
      const int u0 = (gi == 0 ? 0 : Bh) * unit_k, n = (gi == 0 ? Bh : B - Bh) * unit_k;
      for (int i = 0; i < n; ++i) s.order[u0 + i] = i;
      std::stable_sort(s.order + u0, s.order + u0 + n, [&](int x, int y) {
        return prompt_lens[(u0 + x) / unit_k] > prompt_lens[(u0 + y) / unit_k];
      });
    }
    c->use_order = (long long)(share ? B : S) * m.n_kv_heads <= 8192 * ngroups;
  }
  c->share_k = share ? k : 0;
  rc = stage_upload(c, s, B, S, share ? B + S : S, st);
  if (rc) return rc;
  c->prof_used = 0;
  if (c->timed) HIPCHK(hipEventRecord(c->ev_start, st));
  // prompt pass: once per prompt; keys and values go to all k sequences of the prompt
  for (const Chunk& ch : chunks) {
    rc = expand(c, ch, prompts, false, st);
    if (rc) return rc;
    HIPCHK(rl_embed(c->x, c->embed, prompts, c->d_tok_index, ch.rows, m.d_model, m.vocab, c->status, st));
    rc = run_layers(c, ch.rows, false, 0, share ? 1 : k, true, ch.jobs, st);
    if (rc) return rc;
    rc = final_norm(c, c->d_lastrow + ch.first * k, ch.count * k, S, ch.first * k, st);
    if (rc) return rc;
  }
  if (c->timed) HIPCHK(hipEventRecord(c->ev_mid, st));
  if (c->eos_token >= 0) HIPCHK(rl_fill_zero(c->d_finished, align_up((size_t)S * 4, 16), st));
  rc = sample_rows(c, S, temperature, uniforms, forced, max_new, 0, tokens, token_logprobs, c->d_next_token, st, c->d_finished);
  if (rc) return rc;
  // one decode step of sequences g0 .. g0 + n - 1 on stream gs, with the activation set in use
  auto decode_step = [&](int t, DecView dv, int n, hipStream_t gs) -> int {
    HIPCHK(rl_embed(c->x, c->embed, dv.row_seq ? dv.row_next : c->d_next_token + dv.g0, nullptr, n, m.d_model, m.vocab, c->status, gs));
    int r2 = run_layers(c, n, true, t, 1, true, 0, gs, dv);
    if (r2) return r2;
    r2 = final_norm(c, nullptr, n, n, 0, gs);
    if (r2) return r2;
    if (dv.row_seq)       // row i reads and writes the entries of sequence row_seq[i]
      return sample_rows(c, n, temperature, uniforms, forced, max_new, t, tokens, token_logprobs, dv.row_next, gs, dv.row_fin, dv.row_seq);
    const size_t o = (size_t)dv.g0 * max_new;
    return sample_rows(c, n, temperature, uniforms + o, forced ? forced + o : nullptr, max_new, t, tokens + o, token_logprobs + o,
                       c->d_next_token + dv.g0, gs, c->d_finished + dv.g0);
  };
  if (ngroups == 2 && max_new > 1) {
    HIPCHK(hipEventRecord(c->ev_fork, st));
    for (int gi = 0; gi < 2; ++gi) HIPCHK(hipStreamWaitEvent(c->gstream[gi], c->ev_fork, 0));
    for (int t = 1; t < max_new && rc == RLGEN_OK; ++t)
      for (int gi = 0; gi < 2 && rc == RLGEN_OK; ++gi) {
        use_set(c, 1 + gi);
        c->half_rows = c->tuned[2][0].variant >= 0;
        const int b0 = gi == 0 ? 0 : Bh, nb = gi == 0 ? Bh : B - Bh;
        rc = decode_step(t, DecView{b0 * k, b0, B}, nb * k, c->gstream[gi]);
      }
    use_set(c, 0);
    c->half_rows = false;
    // join also after an error: the caller's stream must not run ahead of work already queued
    for (int gi = 0; gi < 2; ++gi) {
      HIPCHK(hipEventRecord(c->ev_join[gi], c->gstream[gi]));
      HIPCHK(hipStreamWaitEvent(st, c->ev_join[gi], 0));
    }
    if (rc) return rc;
  } else if (compacting) {
    // Completions end at EOS: every eos_every steps the host reads which sequences have ended (this waits for the
    // stream), fills the rest of their outputs and drops them from the batch; the rows that remain are gathered
    // into fresh per-row arrays.  The cache is addressed by sequence, so nothing in it moves.
    std::vector<int> row_seq(S);
    for (int q = 0; q < S; ++q) row_seq[q] = q;
    DecView dv{0, 0, B};
    dv.row_seq = c->d_iota; dv.row_ctx = c->d_ctx_base; dv.row_next = c->d_next_token; dv.row_fin = c->d_finished;
    dv.row_order = c->use_order ? c->d_order : nullptr;
    int rows = S, side = 0;
    for (int t = 1; t < max_new && rows > 0; ++t) {
      if (t % c->eos_every == 0) {
        HIPCHK(hipMemcpyAsync(c->h_fin, dv.row_fin, (size_t)rows * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        int kept = 0, gone = 0;
        int* keep = c->h_lists;             // [0, kept): rows that stay; then the sequence ids that leave; then the new order
        std::vector<int> left;
        for (int i = 0; i < rows; ++i)
          if (c->h_fin[i]) left.push_back(row_seq[i]);
          else { keep[kept] = i; row_seq[kept] = row_seq[i]; ++kept; }
        gone = (int)left.size();
        if (gone > 0) {
          int* h_left = keep + kept;
          int* h_order = h_left + gone;
          for (int i = 0; i < gone; ++i) h_left[i] = left[i];
          for (int i = 0; i < kept; ++i) h_order[i] = i;
          std::stable_sort(h_order, h_order + kept, [&](int x, int y) { return prompt_lens[row_seq[x] / k] > prompt_lens[row_seq[y] / k]; });
          HIPCHK(hipMemcpyAsync(c->d_lists, keep, (size_t)(2 * kept + gone) * 4, hipMemcpyHostToDevice, st));
          int* d_keep = c->d_lists;
          int* d_left = d_keep + kept;
          int* d_ord = d_left + gone;
          hipLaunchKernelGGL(fill_tail_kernel, dim3(gone), dim3(64), 0, st, d_left, t, max_new, c->eos_token, tokens, token_logprobs);
          HIPCHK(hipGetLastError());
          if (kept > 0) {
            int* base = c->d_cmp + (size_t)side * 4 * S;
            hipLaunchKernelGGL(compact_rows_kernel, dim3((kept + 255) / 256), dim3(256), 0, st, d_keep, kept, dv.row_seq, dv.row_ctx,
                               dv.row_next, base, base + S, base + 2 * S, base + 3 * S);
            HIPCHK(hipGetLastError());
            dv.row_seq = base; dv.row_ctx = base + S; dv.row_next = base + 2 * S; dv.row_fin = base + 3 * S;
            dv.row_order = (long long)kept * m.n_kv_heads <= 8192 ? d_ord : nullptr;
            side ^= 1;
          }
          rows = kept;
          if (rows == 0) break;
        }
      }
      rc = decode_step(t, dv, rows, st);
      if (rc) return rc;
    }
  } else {
    for (int t = 1; t < max_new; ++t) {
      rc = decode_step(t, DecView{0, 0, B}, S, st);
      if (rc) return rc;
    }
  }
  if (c->timed) HIPCHK(hipEventRecord(c->ev_end, st));
  return RLGEN_OK;
}

int rlgen_score(rlgen_ctx* ctx, const int32_t* seqs, const int32_t* seq_lens, const int32_t* score_from, int32_t N,
                int32_t stride, float temperature, float* token_logprobs, void* hip_stream) {
  if (!ctx || !token_logprobs) return RLGEN_ERR_NULL;
  return score_impl(ctx, seqs, seq_lens, score_from, N, stride, temperature, token_logprobs, nullptr, (hipStream_t)hip_stream);
}

int rlgen_debug_logits(rlgen_ctx* ctx, const int32_t* seqs, const int32_t* seq_lens, int32_t N, int32_t stride, float* logits,
                       void* hip_stream) {
  if (!ctx || !logits) return RLGEN_ERR_NULL;
  return score_impl(ctx, seqs, seq_lens, nullptr, N, stride, 1.0f, nullptr, logits, (hipStream_t)hip_stream);
}

int rlgen_debug_sample(rlgen_ctx* c, const float* hidden, int32_t R, float temperature, const float* uniforms,
                       const int32_t* forced, int32_t* tokens, float* token_logprobs, void* hip_stream) {
  if (!c || !hidden || !uniforms || !tokens || !token_logprobs) return RLGEN_ERR_NULL;
  if (R < 1) return RLGEN_ERR_BAD_ARG;
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return RLGEN_ERR_BAD_ARG;
  if (R > c->LM) return RLGEN_ERR_CAPACITY;
  hipStream_t st = (hipStream_t)hip_stream;
  const rlgen_model_cfg& m = c->cfg;
  HIPCHK(rl_norm(hidden, nullptr, R, m.d_model, m.norm_eps, c->fng, m.arch == RLGEN_ARCH_LLAMA ? nullptr : c->fnb, c->hfin,
                 nullptr, nullptr, nullptr, R, 0, c->status, st, m.precise ? kblk_elems(R, m.d_model) : 0));
  return sample_rows(c, R, temperature, uniforms, forced, 1, 0, tokens, token_logprobs, nullptr, st);
}

int rlgen_sample_static(rlgen_ctx* c, const float* hidden, int32_t R, float temperature, const float* uniforms,
                        const int32_t* forced, int32_t* tokens, float* token_logprobs, void* hip_stream) {
  if (!c || !hidden || !uniforms || !tokens || !token_logprobs) return RLGEN_ERR_NULL;
  if (R < 1) return RLGEN_ERR_BAD_ARG;
  if (!(temperature > 0.f) || !std::isfinite(temperature)) return RLGEN_ERR_BAD_ARG;
  const rlgen_model_cfg& m = c->cfg;
  if (R > STATIC_MAX_ROWS || m.d_model > STATIC_MAX_D || c->ngroups > STATIC_MAX_GROUPS) return RLGEN_ERR_CAPACITY;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != c->device) return RLGEN_ERR_DEVICE;      // the context's device must be current
  unsigned char* base = scratch_on_device[dev];
  if (!base) return RLGEN_ERR_DEVICE;
  hipStream_t st = (hipStream_t)hip_stream;
  // The stage's kernels take their intermediate buffers from the context's current activation set: point that at the
  // static array for the duration of the call.  Every element the kernels read is written earlier in this same call
  // (R normalised rows, R x ngroups partials), so nothing left over from a previous call is ever read and nothing needs
  // clearing.
  uint16_t* const keep_hfin = c->hfin;
  float2* const keep_partial = c->partial;
  float* const keep_target = c->target_logit;
  c->hfin = (uint16_t*)base;
  c->partial = (float2*)(base + STATIC_HFIN_BYTES);
  c->target_logit = (float*)(base + STATIC_HFIN_BYTES + STATIC_PARTIAL_BYTES);
  int rc = RLGEN_OK;
  if (rl_norm(hidden, nullptr, R, m.d_model, m.norm_eps, c->fng, m.arch == RLGEN_ARCH_LLAMA ? nullptr : c->fnb, c->hfin, nullptr,
              nullptr, nullptr, R, 0, c->status, st, m.precise ? kblk_elems(R, m.d_model) : 0) != hipSuccess)
    rc = RLGEN_ERR_DEVICE;
  if (rc == RLGEN_OK) rc = sample_rows(c, R, temperature, uniforms, forced, 1, 0, tokens, token_logprobs, nullptr, st);
  c->hfin = keep_hfin; c->partial = keep_partial; c->target_logit = keep_target;
  return rc;
}

int rlgen_sequence_logprob(const float* token_logprobs, const int32_t* from, const int32_t* lens, int32_t N, int32_t stride,
                           float* seq_logprob, void* hip_stream) {
  if (!token_logprobs || !from || !lens || !seq_logprob) return RLGEN_ERR_NULL;
  if (N < 1 || stride < 1) return RLGEN_ERR_BAD_ARG;
  HIPCHK(rl_sequence_logprob(token_logprobs, from, lens, N, stride, seq_logprob, (hipStream_t)hip_stream));
  return RLGEN_OK;
}

int rlgen_dpo_loss(const float* pol_pos, const float* ref_pos, const float* pol_neg, const float* ref_neg, int32_t P, float beta,
                   float* loss, void* hip_stream) {
  if (!pol_pos || !ref_pos || !pol_neg || !ref_neg || !loss) return RLGEN_ERR_NULL;
  if (P < 1 || !std::isfinite(beta)) return RLGEN_ERR_BAD_ARG;
  HIPCHK(rl_dpo_loss(pol_pos, ref_pos, pol_neg, ref_neg, P, beta, loss, (hipStream_t)hip_stream));
  return RLGEN_OK;
}

int rlgen_proximal_rloo(const float* pol_logprob, const float* old_logprob, const float* rewards, int32_t B, int32_t k,
                        float epsilon, float* objective, void* hip_stream) {
  if (!pol_logprob || !old_logprob || !rewards || !objective) return RLGEN_ERR_NULL;
  if (B < 1 || k < 2 || (int64_t)B * k > INT32_MAX || !std::isfinite(epsilon) || epsilon < 0.f) return RLGEN_ERR_BAD_ARG;
  HIPCHK(rl_proximal_rloo(pol_logprob, old_logprob, rewards, B, k, epsilon, objective, (hipStream_t)hip_stream));
  return RLGEN_OK;
}

int rlgen_select_pairs(const float* rewards, int32_t B, int32_t k, int32_t* idx_pos, int32_t* idx_neg, void* hip_stream) {
  if (!rewards || !idx_pos || !idx_neg) return RLGEN_ERR_NULL;
  if (B < 1 || k < 1) return RLGEN_ERR_BAD_ARG;
  HIPCHK(rl_select_pairs(rewards, B, k, idx_pos, idx_neg, (hipStream_t)hip_stream));
  return RLGEN_OK;
}

int rlgen_get_timings(rlgen_ctx* c, float* prefill_ms, float* decode_ms, float* decode_attn_ms, int32_t* decode_attn_launches) {
  if (!c) return RLGEN_ERR_NULL;
  HIPCHK(hipEventSynchronize(c->ev_end));
  float a = 0.f, b = 0.f;
  HIPCHK(hipEventElapsedTime(&a, c->ev_start, c->ev_mid));
  HIPCHK(hipEventElapsedTime(&b, c->ev_mid, c->ev_end));
  if (prefill_ms) *prefill_ms = a;
  if (decode_ms) *decode_ms = b;
  float tot = 0.f;
  for (size_t i = 0; i + 1 < c->prof_used; i += 2) {
    float t = 0.f;
    HIPCHK(hipEventElapsedTime(&t, c->prof_events[i], c->prof_events[i + 1]));
    tot += t;
  }
  if (decode_attn_ms) *decode_attn_ms = tot;
  if (decode_attn_launches) *decode_attn_launches = (int32_t)(c->prof_used / 2);
  return RLGEN_OK;
}

int rlgen_set_profiling(rlgen_ctx* c, int32_t on) {
  if (!c) return RLGEN_ERR_NULL;
  c->profiling = on > 0 ? on : 0;
  if (!on) c->prof_used = 0;
  return RLGEN_OK;
}

int rlgen_set_eos(rlgen_ctx* c, int32_t eos_token) {
  if (!c) return RLGEN_ERR_NULL;
  if (eos_token < -1 || eos_token >= c->cfg.vocab) return RLGEN_ERR_BAD_ARG;
  c->eos_token = eos_token;
  return RLGEN_OK;
}

int rlgen_set_score_groups(rlgen_ctx* c, int32_t k) {
  if (!c) return RLGEN_ERR_NULL;
  if (k < 1) return RLGEN_ERR_BAD_ARG;
  c->score_groups = k;
  return RLGEN_OK;
}

int rlgen_set_decode_split(rlgen_ctx* c, int32_t on) {
  if (!c) return RLGEN_ERR_NULL;
  c->split_off = on == 0;
  return RLGEN_OK;
}

int rlgen_status_bits(rlgen_ctx* c, void* hip_stream, uint32_t* faults) {
  if (!c) return RLGEN_ERR_NULL;
  unsigned v = 0;
  HIPCHK(hipMemcpyAsync(&v, c->status, sizeof(v), hipMemcpyDeviceToHost, (hipStream_t)hip_stream));
  HIPCHK(hipStreamSynchronize((hipStream_t)hip_stream));
  if (faults) *faults = v;
  return v ? RLGEN_ERR_DEVICE : RLGEN_OK;
}

int rlgen_status(rlgen_ctx* c, void* hip_stream) { return rlgen_status_bits(c, hip_stream, nullptr); }

int rlgen_set_eos_compaction(rlgen_ctx* c, int32_t every) {
  if (!c) return RLGEN_ERR_NULL;
  if (every < 0) return RLGEN_ERR_BAD_ARG;
  c->eos_every = every;
  return RLGEN_OK;
}

int rlgen_set_decode_split_min(rlgen_ctx* c, int32_t min_seqs) {
  if (!c) return RLGEN_ERR_NULL;
  if (min_seqs != 0 && min_seqs < 2) return RLGEN_ERR_BAD_ARG;
  c->split_min_seqs = min_seqs ? min_seqs : DECODE_SPLIT_MIN_SEQS;
  return RLGEN_OK;
}

int rlgen_debug_get_gemm(rlgen_ctx* c, int32_t mode, int32_t which, int32_t* variant, int32_t* splits) {
  if (!c) return RLGEN_ERR_NULL;
  if (mode < 0 || mode > 2 || which < 0 || which > 4) return RLGEN_ERR_BAD_ARG;
  if (variant) *variant = c->tuned[mode][which].variant;
  if (splits) *splits = c->tuned[mode == 1 ? 1 : 0][which].splits;
  return RLGEN_OK;
}

int rlgen_debug_set_gemm(rlgen_ctx* c, int32_t mode, int32_t which, int32_t variant) {
  if (!c) return RLGEN_ERR_NULL;
  if (mode < 0 || mode > 2 || which < 0 || which > 4 || variant < -1 || variant > 10) return RLGEN_ERR_BAD_ARG;
  // the fused gate/up and LM-head epilogues need a wave to own 64 columns: not the 64-column-per-wave-pair shapes
  const bool wide_only = which == G_LMHEAD || (which == G_UP && c->cfg.arch == RLGEN_ARCH_LLAMA);
  if (wide_only && variant >= 6 && variant <= 9) return RLGEN_ERR_BAD_ARG;
  if (c->cfg.precise && variant != -1 && variant != 0 && variant != 3 && variant != 5 && variant != 7) return RLGEN_ERR_BAD_ARG;
  c->tuned[mode][which].variant = variant;
  return RLGEN_OK;
}

const char* rlgen_strerror(int code) {
  switch (code) {
    case RLGEN_OK: return "ok";
    case RLGEN_ERR_NULL: return "a required pointer is null";
    case RLGEN_ERR_BAD_CFG: return "inconsistent or unsupported model configuration";
    case RLGEN_ERR_BAD_ARG: return "argument out of its domain";
    case RLGEN_ERR_CAPACITY: return "call exceeds the capacity the context was created with";
    case RLGEN_ERR_WORKSPACE: return "workspace too small or misaligned";
    case RLGEN_ERR_UNIMPLEMENTED: return "not implemented";
    case RLGEN_ERR_DEVICE: return "HIP call failed or a kernel flagged an out-of-range token id or uniform";
  }
  return "unknown error code";
}

void rlgen_destroy(rlgen_ctx* c) {
  if (!c) return;
  if (c->ev_meta) {
    if (c->meta_pending) (void)hipEventSynchronize(c->ev_meta);
    (void)hipEventDestroy(c->ev_meta);
  }
  if (c->ev_start) (void)hipEventDestroy(c->ev_start);
  if (c->ev_mid) (void)hipEventDestroy(c->ev_mid);
  if (c->ev_end) (void)hipEventDestroy(c->ev_end);
  for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
  if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
  for (int i = 0; i < 2; ++i) {
    if (c->ev_join[i]) (void)hipEventDestroy(c->ev_join[i]);
    if (c->gstream[i]) {
      (void)hipStreamSynchronize(c->gstream[i]);
      (void)hipStreamDestroy(c->gstream[i]);
    }
  }
  if (c->h_stage) (void)hipHostFree(c->h_stage);
  if (c->h_fin) (void)hipHostFree(c->h_fin);
  delete c;
}

}  // extern "C"
