// Host side of the stairs C ABI: context, weight upload and re-layout, the per-forward launch
// schedule, the propose / verify / accept loop.  All arithmetic of the method runs in the
// kernels of stairs_kernels.hip; this file only sequences them.
#include "../../include/stairs.h"
#include "stairs_kernels.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <new>
#include <string>
#include <vector>

using namespace stairs;

namespace {

struct Layer {
  const float* attn_norm = nullptr;
  const float* ffn_norm = nullptr;
  const void* wqkv = nullptr;   // [3d, d]
  const void* wo = nullptr;     // [d, d]
  const void* wgu = nullptr;    // [2f, d]
  const void* wdown = nullptr;  // [d, f]
};

// One layer of an encoder-decoder stack (decoder layers also hold the cross-attention block)
struct EdLayer {
  const float *attn_norm = nullptr, *cross_norm = nullptr, *ffn_norm = nullptr;
  const void* wqkv = nullptr;    // [3a, d]
  const void* wo = nullptr;      // [d, a]
  const void* cqkv = nullptr;    // [3a, d] cross-attention q | k | v: used whole once per source, for its k and v
  const void* cq = nullptr;      // [a, d] cross-attention query projection alone (every decoder forward)
  const void* co = nullptr;      // [d, a]
  const void* w_in = nullptr;    // [f, d]
  const void* w_out = nullptr;   // [d, f]
};

struct Model {
  stairs_model_cfg cfg{};
  bool bf16 = false;
  int hd = 0, cap = 0;
  // encoder-decoder models: cfg describes the decoder (n_layers = decoder layers, rope_theta = 0: no rotation)
  // matrices of one forward far beyond the 256 MB memory-side cache: read them with the streaming hint
  bool stream_weights = false;
  bool encdec = false;
  int da = 0;                       // attention width n_heads * head_dim (decoder-only models: d_model)
  int max_src = 0, cap_src = 0;     // source positions the encoder-side buffers hold
  std::vector<EdLayer> enc, dec;
  const float* enc_final_norm = nullptr;
  float* enc_bias = nullptr;        // [H][2 * max_src - 1]: bias by key position - query position + max_src - 1
  float* dec_bias = nullptr;        // [H][cap]: bias by key position - query position + cap - 1 (keys before the query)
  char *Ke = nullptr, *Ve = nullptr;   // encoder self-attention keys/values of the layer being run: [H][cap_src][hd]
  char *Kx = nullptr, *Vx = nullptr;   // cross-attention keys/values: [decoder layers][H][cap_src][hd]
  size_t kvx_layer_bytes = 0;
  const void* tok_emb = nullptr;    // row-major, cfg dtype
  const void* lm_head = nullptr;    // GEMM layout
  const float* final_norm = nullptr;
  std::vector<Layer> layers;
  char* Kc = nullptr;               // [slots][layers][H][cap][hd]
  char* Vc = nullptr;
  size_t kv_layer_bytes = 0;
  int valid = 0;                    // positions 0..valid-1 of the cache hold the current sequence
  size_t esz() const { return bf16 ? 2 : 4; }
};

}  // namespace

constexpr int kGemmCounters = 2048;   // >= column groups of the widest GEMM (N / 64)
constexpr int kAttnCounters = 4096;                    // one per (sequence slot, attention head)
constexpr int kCounters = kGemmCounters + kAttnCounters;

struct stairs_ctx {
  hipStream_t st = nullptr;
  int k_max = 0;
  bool have_draft = false;
  Model T, D;
  std::vector<void*> owned;                       // every device allocation, freed in stairs_free
  std::map<std::pair<const void*, int>, const void*> dedup;   // (first host ptr, kind) -> device copy
  // workspaces (sized for the larger of the two models)
  float *x = nullptr, *ssq = nullptr, *q_rot = nullptr, *attn_out = nullptr, *h = nullptr, *logits = nullptr;
  float *partial = nullptr, *part_o = nullptr, *part_ml = nullptr;
  float2* rope_cs = nullptr;
  // activation fragments of x, attn_out and h for forwards of more than 4 rows (bf16 models), see frag_bytes()
  uint4 *xf = nullptr, *af = nullptr, *hf = nullptr;
  // block prefill (bf16 models, env STAIRS_NO_BLOCK_PREFILL=1 turns it off): [kPfRows, .] workspaces
  bool block_prefill = false;
  float *pf_x = nullptr, *pf_y = nullptr, *pf_q = nullptr, *pf_attn = nullptr;
  uint4* pf_frag = nullptr;    // block fragments of the activation in front of the current projection
  float* pf_part = nullptr;    // k-split results of block GEMMs with few rows (short prompts, forwards of many sequences)
  size_t pf_part_floats = 0;
  float2* pf_cs = nullptr;
  // encoder-decoder contexts: source tokens and the encoder's activations [max_src, .]
  bool encdec = false;
  int start_token = 0, S = 0;   // S = length of the encoded source
  int* src_tok = nullptr;
  float *enc_x = nullptr, *enc_ssq = nullptr, *enc_q = nullptr;
  // sampling variant: parameters on the device, the assistant's logits rows of the pending proposal, log-sum-exps
  SampleParams* samp = nullptr;
  SampleWs* samp_ws = nullptr;
  float *dlogits = nullptr, *lse = nullptr;
  bool pending_sampled = false;
  int nchunk_cap = 0;
  int* tokens = nullptr;       // device copy of the sequence(s): [n_slots][tok_stride], capacity tok_cap each
  int tok_cap = 0, tok_stride = 0;
  int n_slots = 1;             // sequence slots the caches, token arrays and state hold (stairs_reserve_batch)
  int rows_cap = kMaxRows;     // rows logits, target tokens and attention partial results are sized for
  int fwd_rows = kMaxRows;     // rows one forward of the decode kernels takes (kMaxFwdRows once several sequences are reserved)
  int pf_rows = 0;             // rows the block workspaces (pf_*) hold
  int* counters = nullptr;     // [kCounters] split-K / attention hand-off tickets, zero between launches
  int* tgt_tok = nullptr;      // [kMaxRows]
  int* state = nullptr;        // per slot kSlotState ints: [0] = L, [1] = n of last iteration, [2] = constant 0, [3] = active
  int eos_id = -1;             // end token of the generation loops (stairs_set_eos); -1: none
  int* h_pinned = nullptr;     // pinned host: [0..1] state, [2..2+kMaxRows) target tokens; batch: [n_slots][kSlotState] state
  int h_pinned_ints = 0;
  // host mirror
  int L = 0, P = 0;
  bool prefilled = false;
  int pending_k = -1;          // draft length of the outstanding proposal, -1 = none
  hipEvent_t ev[8] = {};       // 0,1: general; 5,6,7: iteration start / after the proposal / after validation
  struct IterGraph { int half, k, nch, B; hipGraphExec_t exec; };   // B = 0: the single-sequence path, -1: its sampled variant
  std::vector<IterGraph> graphs;   // captured iterations, see iteration_graph()
  std::vector<hipEvent_t> probe_ev;   // stairs_time_kernel(8): event pairs around one projection inside a forward
  int probe_role = -1;               // role being timed in situ, -1 = none, kProbeEmptyPair = calibration
  bool own_stream = false;
  bool use_graphs = true;      // env STAIRS_NO_GRAPH=1 turns replay off
  bool sync_launches = false;  // env STAIRS_SYNC_LAUNCHES=1 or 2: wait after every kernel (for counter-collecting profilers)
  bool sync_blocks = false;    // =2: prompts still go through the block kernels (=1: through the decode kernels)
  std::string err;
};

namespace {

#define HIPCHK(c, expr)                                                               \
  do {                                                                                \
    hipError_t e_ = (expr);                                                           \
    if (e_ != hipSuccess) {                                                           \
      (c)->err = std::string(#expr) + ": " + hipGetErrorString(e_);                   \
      return STAIRS_EHIP;                                                             \
    }                                                                                 \
  } while (0)

int fail(stairs_ctx* c, int code, const char* msg) {
  if (c) c->err = msg;
  return code;
}

template <typename T>
int dev_alloc(stairs_ctx* c, T** out, size_t count) {
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, std::max<size_t>(count, 1) * sizeof(T));
  if (e != hipSuccess) {
    c->err = std::string("hipMalloc: ") + hipGetErrorString(e);
    (void)hipGetLastError();
    return STAIRS_ENOMEM;
  }
  c->owned.push_back(p);
  *out = static_cast<T*>(p);
  return STAIRS_OK;
}

const char* check_cfg(const stairs_model_cfg* m) {
  if (!m) return "model config is NULL";
  if (m->n_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->d_ffn < 1 || m->vocab < 1 || m->max_seq < 2)
    return "model dimensions must be positive (max_seq >= 2)";
  if (m->dtype != STAIRS_DTYPE_FP32 && m->dtype != STAIRS_DTYPE_BF16) return "unknown dtype";
  if (m->d_model % m->n_heads) return "d_model is not a multiple of n_heads";
  const int hd = m->d_model / m->n_heads;
  if (hd != 64 && hd != 128) return "head_dim must be 64 or 128";
  if (m->dtype == STAIRS_DTYPE_BF16) {
    if (m->d_model % 256 || m->d_ffn % 256) return "bf16 models need d_model and d_ffn to be multiples of 256";
    if (m->vocab % 16) return "bf16 models need vocab to be a multiple of 16";
  } else {
    if (m->d_model % 4 || m->d_ffn % 4 || m->vocab % 4) return "fp32 models need d_model, d_ffn, vocab multiples of 4";
  }
  if (!(m->rope_theta > 0.f) || !(m->rms_eps >= 0.f)) return "rope_theta must be > 0 and rms_eps >= 0";
  if (std::max({m->vocab, 3 * m->d_model, 2 * m->d_ffn}) / 64 + 1 > kGemmCounters || m->n_heads > kAttnCounters)
    return "model too wide for the hand-off counters";
  if (m->max_seq > 60000) return "max_seq above 60000 is not supported (attention merge table lives in LDS)";
  return nullptr;
}

const char* check_weights(const stairs_model_cfg* m, const stairs_weights* w) {
  if (!w) return "weights are NULL";
  if (!w->tok_emb || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
      !w->ffn_norm || !w->w_gate || !w->w_up || !w->w_down)
    return "a weight pointer is NULL";
  for (int l = 0; l < m->n_layers; ++l)
    if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate[l] ||
        !w->w_up[l] || !w->w_down[l])
      return "a per-layer weight pointer is NULL";
  return nullptr;
}

constexpr size_t kStreamHintBytes = 512u << 20;   // models streaming more than this per forward use the hint
constexpr int kProbeEmptyPair = 100;
constexpr int kProbeKernelEvents = 101;   // the gate/up launch records its own start / end events
enum { KIND_EMB = 0, KIND_HEAD, KIND_NORM, KIND_QKV, KIND_WO, KIND_GU, KIND_DOWN };

// Upload a matrix made of `nparts` row blocks (each [rows_each, K], host, model dtype) as one
// [nparts*rows_each, K] GEMM operand; bf16 goes through the operand re-layout kernel.
int upload_matrix(stairs_ctx* c, bool bf16, const void* const* parts, int nparts, int rows_each, int K, int kind,
                  int hd, char* staging, const void** out) {
  // gate/up and q/k rows are reordered so that SwiGLU and rotation pairs share a 16-row tile
  const int perm = (kind == KIND_GU) ? kPermGateUp : (kind == KIND_QKV) ? kPermQKV : kPermNone;
  auto key = std::make_pair(parts[0], kind);
  auto it = c->dedup.find(key);
  if (it != c->dedup.end()) {
    *out = it->second;
    return STAIRS_OK;
  }
  const size_t esz = bf16 ? 2 : 4;
  const size_t part_bytes = (size_t)rows_each * K * esz;
  char* dst = nullptr;
  int rc = dev_alloc(c, &dst, part_bytes * nparts);
  if (rc) return rc;
  char* raw = bf16 ? staging : dst;
  for (int p = 0; p < nparts; ++p)
    HIPCHK(c, hipMemcpyAsync(raw + p * part_bytes, parts[p], part_bytes, hipMemcpyHostToDevice, c->st));
  if (bf16) {
    launch_swizzle_bf16(reinterpret_cast<const uint16_t*>(staging), reinterpret_cast<uint4*>(dst), nparts * rows_each, K,
                        perm, rows_each, hd, c->st);
    HIPCHK(c, hipGetLastError());
  }
  HIPCHK(c, hipStreamSynchronize(c->st));   // staging and the host buffers are reused right away
  c->dedup[key] = dst;
  *out = dst;
  return STAIRS_OK;
}

int upload_plain(stairs_ctx* c, const void* host, size_t bytes, int kind, const void** out) {
  auto key = std::make_pair(host, kind);
  auto it = c->dedup.find(key);
  if (it != c->dedup.end()) {
    *out = it->second;
    return STAIRS_OK;
  }
  char* dst = nullptr;
  int rc = dev_alloc(c, &dst, bytes);
  if (rc) return rc;
  HIPCHK(c, hipMemcpyAsync(dst, host, bytes, hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));
  c->dedup[key] = dst;
  *out = dst;
  return STAIRS_OK;
}

int build_model(stairs_ctx* c, Model* m, const stairs_model_cfg* cfg, const stairs_weights* w, char* staging) {
  m->cfg = *cfg;
  m->bf16 = cfg->dtype == STAIRS_DTYPE_BF16;
  m->hd = cfg->d_model / cfg->n_heads;
  m->cap = (cfg->max_seq + 31) / 32 * 32;   // whole 32-position value blocks
  const int d = cfg->d_model, f = cfg->d_ffn, V = cfg->vocab;
  int rc;
  if ((rc = upload_plain(c, w->tok_emb, (size_t)V * d * m->esz(), KIND_EMB, &m->tok_emb))) return rc;
  const void* one[1] = {w->lm_head};
  if ((rc = upload_matrix(c, m->bf16, one, 1, V, d, KIND_HEAD, m->hd, staging, &m->lm_head))) return rc;
  const void* fn = nullptr;
  if ((rc = upload_plain(c, w->final_norm, (size_t)d * 4, KIND_NORM, &fn))) return rc;
  m->final_norm = static_cast<const float*>(fn);
  m->layers.resize(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l) {
    Layer& ly = m->layers[l];
    const void* p = nullptr;
    if ((rc = upload_plain(c, w->attn_norm[l], (size_t)d * 4, KIND_NORM, &p))) return rc;
    ly.attn_norm = static_cast<const float*>(p);
    if ((rc = upload_plain(c, w->ffn_norm[l], (size_t)d * 4, KIND_NORM, &p))) return rc;
    ly.ffn_norm = static_cast<const float*>(p);
    const void* qkv[3] = {w->wq[l], w->wk[l], w->wv[l]};
    if ((rc = upload_matrix(c, m->bf16, qkv, 3, d, d, KIND_QKV, m->hd, staging, &ly.wqkv))) return rc;
    one[0] = w->wo[l];
    if ((rc = upload_matrix(c, m->bf16, one, 1, d, d, KIND_WO, m->hd, staging, &ly.wo))) return rc;
    const void* gu[2] = {w->w_gate[l], w->w_up[l]};
    if ((rc = upload_matrix(c, m->bf16, gu, 2, f, d, KIND_GU, m->hd, staging, &ly.wgu))) return rc;
    one[0] = w->w_down[l];
    if ((rc = upload_matrix(c, m->bf16, one, 1, d, f, KIND_DOWN, m->hd, staging, &ly.wdown))) return rc;
  }
  m->stream_weights = m->bf16 && ((size_t)cfg->n_layers * (4 * (size_t)d * d + 3 * (size_t)d * f) + (size_t)V * d) * 2 > kStreamHintBytes;
  m->kv_layer_bytes = (size_t)cfg->n_heads * m->cap * m->hd * m->esz();
  if ((rc = dev_alloc(c, &m->Kc, m->kv_layer_bytes * cfg->n_layers))) return rc;
  if ((rc = dev_alloc(c, &m->Vc, m->kv_layer_bytes * cfg->n_layers))) return rc;
  // positions that were never written are multiplied by probability 0 in the value product: they must be finite
  HIPCHK(c, hipMemsetAsync(m->Kc, 0, m->kv_layer_bytes * cfg->n_layers, c->st));
  HIPCHK(c, hipMemsetAsync(m->Vc, 0, m->kv_layer_bytes * cfg->n_layers, c->st));
  return STAIRS_OK;
}

// ---- encoder-decoder models -----------------------------------------------------------------------------------
const char* check_encdec_cfg(const stairs_encdec_cfg* m) {
  if (!m) return "model config is NULL";
  if (m->n_enc_layers < 1 || m->n_dec_layers < 1 || m->d_model < 1 || m->n_heads < 1 || m->d_ffn < 1 || m->vocab < 1 ||
      m->max_seq < 2 || m->max_src < 1)
    return "model dimensions must be positive (max_seq >= 2)";
  if (m->head_dim != 64 && m->head_dim != 128) return "head_dim must be 64 or 128";
  const long a = (long)m->n_heads * m->head_dim;
  if (m->d_model % 256 || m->d_ffn % 256 || a % 256) return "d_model, n_heads * head_dim and d_ffn must be multiples of 256";
  if (m->vocab % 16) return "vocab must be a multiple of 16";
  if (!(m->rms_eps >= 0.f)) return "rms_eps must be >= 0";
  if (m->rel_buckets < 4 || m->rel_buckets % 4 || m->rel_max_distance <= m->rel_buckets / 2)
    return "rel_buckets must be a multiple of 4 and rel_max_distance above rel_buckets / 2";
  if (std::max<long>({(long)m->vocab, 3 * a, (long)m->d_ffn}) / 64 + 1 > kGemmCounters || m->n_heads > kAttnCounters)
    return "model too wide for the hand-off counters";
  if (m->max_seq > 60000) return "max_seq above 60000 is not supported (attention merge table lives in LDS)";
  if (m->max_src > 4096) return "max_src above 4096 is not supported";
  return nullptr;
}

const char* check_encdec_weights(const stairs_encdec_cfg* m, const stairs_encdec_weights* w) {
  if (!w) return "weights are NULL";
  if (!w->tok_emb || !w->lm_head || !w->enc_rel_bias || !w->dec_rel_bias || !w->enc_final_norm || !w->dec_final_norm ||
      !w->enc_attn_norm || !w->enc_ffn_norm || !w->enc_wq || !w->enc_wk || !w->enc_wv || !w->enc_wo || !w->enc_w_in ||
      !w->enc_w_out || !w->dec_attn_norm || !w->dec_cross_norm || !w->dec_ffn_norm || !w->dec_wq || !w->dec_wk ||
      !w->dec_wv || !w->dec_wo || !w->dec_cq || !w->dec_ck || !w->dec_cv || !w->dec_co || !w->dec_w_in || !w->dec_w_out)
    return "a weight pointer is NULL";
  for (int l = 0; l < m->n_enc_layers; ++l)
    if (!w->enc_attn_norm[l] || !w->enc_ffn_norm[l] || !w->enc_wq[l] || !w->enc_wk[l] || !w->enc_wv[l] || !w->enc_wo[l] ||
        !w->enc_w_in[l] || !w->enc_w_out[l])
      return "a per-layer weight pointer is NULL";
  for (int l = 0; l < m->n_dec_layers; ++l)
    if (!w->dec_attn_norm[l] || !w->dec_cross_norm[l] || !w->dec_ffn_norm[l] || !w->dec_wq[l] || !w->dec_wk[l] ||
        !w->dec_wv[l] || !w->dec_wo[l] || !w->dec_cq[l] || !w->dec_ck[l] || !w->dec_cv[l] || !w->dec_co[l] ||
        !w->dec_w_in[l] || !w->dec_w_out[l])
      return "a per-layer weight pointer is NULL";
  return nullptr;
}

// Bucket of a distance n >= 0 when one side of the query has `side` buckets: the distance itself below side / 2,
// then logarithmically spaced up to max_distance, the last bucket beyond (rule of the original T5).
int rel_bucket(int n, int side, int max_distance) {
  const int exact = side / 2;
  if (n < exact) return n;
  const double t = std::log((double)n / exact) / std::log((double)max_distance / exact) * (side - exact);
  return std::min(exact + (int)std::floor(t), side - 1);
}

// bucket of rel = key position - query position: two-sided (encoder; keys after the query take the upper half of the
// buckets) or one-sided (decoder; keys after the query count as distance 0)
int bias_bucket(int rel, bool two_sided, int buckets, int max_distance) {
  if (two_sided) return (rel > 0 ? buckets / 2 : 0) + rel_bucket(std::abs(rel), buckets / 2, max_distance);
  return rel_bucket(std::max(-rel, 0), buckets, max_distance);
}

// Bias tables by distance: dst[h][i] = table[bucket(rel)][h] with rel = i - zero (key position - query position).
int upload_bias(stairs_ctx* c, const float* table, int buckets, int max_distance, int H, int len, int zero, bool two_sided,
                float** out) {
  std::vector<float> host((size_t)H * len);
  for (int i = 0; i < len; ++i) {
    const int rel = i - zero;
    const int b = bias_bucket(rel, two_sided, buckets, max_distance);
    for (int h = 0; h < H; ++h) host[(size_t)h * len + i] = table[(size_t)b * H + h];
  }
  int rc = dev_alloc(c, out, host.size());
  if (rc) return rc;
  HIPCHK(c, hipMemcpyAsync(*out, host.data(), host.size() * sizeof(float), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));
  return STAIRS_OK;
}

int build_encdec_model(stairs_ctx* c, Model* m, const stairs_encdec_cfg* cfg, const stairs_encdec_weights* w, char* staging) {
  m->encdec = true;
  m->bf16 = true;
  m->cfg = stairs_model_cfg{cfg->n_dec_layers, cfg->d_model, cfg->n_heads, cfg->d_ffn, cfg->vocab, cfg->max_seq,
                            0.f /* no rotation */, cfg->rms_eps, STAIRS_DTYPE_BF16};
  m->hd = cfg->head_dim;
  m->da = cfg->n_heads * cfg->head_dim;
  m->cap = (cfg->max_seq + 31) / 32 * 32;
  m->max_src = cfg->max_src;
  m->cap_src = (cfg->max_src + 31) / 32 * 32;
  const int d = cfg->d_model, a = m->da, f = cfg->d_ffn, V = cfg->vocab, H = cfg->n_heads;
  int rc;
  if ((rc = upload_plain(c, w->tok_emb, (size_t)V * d * 2, KIND_EMB, &m->tok_emb))) return rc;
  const void* one[1] = {w->lm_head};
  if ((rc = upload_matrix(c, true, one, 1, V, d, KIND_HEAD, m->hd, staging, &m->lm_head))) return rc;
  auto gain = [&](const float* host, const float** out) {
    const void* p = nullptr;
    const int r = upload_plain(c, host, (size_t)d * 4, KIND_NORM, &p);
    *out = static_cast<const float*>(p);
    return r;
  };
  auto plain = [&](const void* host, int N, int K, const void** out) {     // a matrix whose rows keep their order
    const void* o[1] = {host};
    return upload_matrix(c, true, o, 1, N, K, KIND_WO, m->hd, staging, out);
  };
  if ((rc = gain(w->dec_final_norm, &m->final_norm)) || (rc = gain(w->enc_final_norm, &m->enc_final_norm))) return rc;
  m->enc.resize(cfg->n_enc_layers);
  for (int l = 0; l < cfg->n_enc_layers; ++l) {
    EdLayer& ly = m->enc[l];
    const void* qkv[3] = {w->enc_wq[l], w->enc_wk[l], w->enc_wv[l]};
    if ((rc = gain(w->enc_attn_norm[l], &ly.attn_norm)) || (rc = gain(w->enc_ffn_norm[l], &ly.ffn_norm)) ||
        (rc = upload_matrix(c, true, qkv, 3, a, d, KIND_QKV, m->hd, staging, &ly.wqkv)) ||
        (rc = plain(w->enc_wo[l], d, a, &ly.wo)) || (rc = plain(w->enc_w_in[l], f, d, &ly.w_in)) ||
        (rc = plain(w->enc_w_out[l], d, f, &ly.w_out)))
      return rc;
  }
  m->dec.resize(cfg->n_dec_layers);
  for (int l = 0; l < cfg->n_dec_layers; ++l) {
    EdLayer& ly = m->dec[l];
    const void* qkv[3] = {w->dec_wq[l], w->dec_wk[l], w->dec_wv[l]};
    const void* cqkv[3] = {w->dec_cq[l], w->dec_ck[l], w->dec_cv[l]};
    if ((rc = gain(w->dec_attn_norm[l], &ly.attn_norm)) || (rc = gain(w->dec_cross_norm[l], &ly.cross_norm)) ||
        (rc = gain(w->dec_ffn_norm[l], &ly.ffn_norm)) ||
        (rc = upload_matrix(c, true, qkv, 3, a, d, KIND_QKV, m->hd, staging, &ly.wqkv)) ||
        (rc = plain(w->dec_wo[l], d, a, &ly.wo)) ||
        (rc = upload_matrix(c, true, cqkv, 3, a, d, KIND_QKV, m->hd, staging, &ly.cqkv)) ||
        (rc = plain(w->dec_cq[l], a, d, &ly.cq)) || (rc = plain(w->dec_co[l], d, a, &ly.co)) ||
        (rc = plain(w->dec_w_in[l], f, d, &ly.w_in)) || (rc = plain(w->dec_w_out[l], d, f, &ly.w_out)))
      return rc;
  }
  if ((rc = upload_bias(c, w->enc_rel_bias, cfg->rel_buckets, cfg->rel_max_distance, H, 2 * m->max_src - 1, m->max_src - 1,
                        true, &m->enc_bias)) ||
      (rc = upload_bias(c, w->dec_rel_bias, cfg->rel_buckets, cfg->rel_max_distance, H, m->cap, m->cap - 1, false,
                        &m->dec_bias)))
    return rc;
  m->stream_weights = ((size_t)cfg->n_dec_layers * (8 * (size_t)d * a + 2 * (size_t)d * f) + (size_t)V * d) * 2 > kStreamHintBytes;
  m->kv_layer_bytes = (size_t)H * m->cap * m->hd * 2;
  m->kvx_layer_bytes = (size_t)H * m->cap_src * m->hd * 2;
  const size_t self_bytes = m->kv_layer_bytes * cfg->n_dec_layers, cross_bytes = m->kvx_layer_bytes * cfg->n_dec_layers;
  if ((rc = dev_alloc(c, &m->Kc, self_bytes)) || (rc = dev_alloc(c, &m->Vc, self_bytes)) ||
      (rc = dev_alloc(c, &m->Kx, cross_bytes)) || (rc = dev_alloc(c, &m->Vx, cross_bytes)) ||
      (rc = dev_alloc(c, &m->Ke, m->kvx_layer_bytes)) || (rc = dev_alloc(c, &m->Ve, m->kvx_layer_bytes)))
    return rc;
  // positions never written meet probability 0 in the value product: they must be finite
  HIPCHK(c, hipMemsetAsync(m->Kc, 0, self_bytes, c->st));
  HIPCHK(c, hipMemsetAsync(m->Vc, 0, self_bytes, c->st));
  HIPCHK(c, hipMemsetAsync(m->Kx, 0, cross_bytes, c->st));
  HIPCHK(c, hipMemsetAsync(m->Vx, 0, cross_bytes, c->st));
  HIPCHK(c, hipMemsetAsync(m->Ke, 0, m->kvx_layer_bytes, c->st));
  HIPCHK(c, hipMemsetAsync(m->Ve, 0, m->kvx_layer_bytes, c->st));
  return STAIRS_OK;
}

size_t max_matrix_bytes(const stairs_model_cfg* m) {
  const size_t esz = m->dtype == STAIRS_DTYPE_BF16 ? 2 : 4;
  const size_t d = m->d_model, f = m->d_ffn, V = m->vocab;
  return std::max({3 * d * d, 2 * f * d, V * d}) * esz;
}

size_t max_partial_floats(const stairs_model_cfg* m) {
  const int b = m->dtype == STAIRS_DTYPE_BF16;
  const size_t d = m->d_model, f = m->d_ffn, V = m->vocab;
  const size_t sd = gemm_slices(m->d_model, b), sf = gemm_slices(m->d_ffn, b);
  return kMaxRows * std::max({sd * 3 * d, sd * 2 * f, sf * d, sd * V});
}

// One forward of `M` rows at positions pos..pos+M-1 whose token ids are tokens[pos..pos+M-1].
// nchunk = attention chunks to launch: >= ceil((pos + M) / kAttnChunk); extra ones find no keys.
// logits_rows: 0 = no unembedding (prefill), 1 = last row only -> c->logits row 0,
//              M = every row -> c->logits rows 0..M-1.
// Several sequences: pos.rps > 0 rows per slot, M = rps * (number of slots), slots 0..M/rps-1; otherwise the
// rows belong to sequence slot `slot`.
int forward_ed(stairs_ctx* c, Model* m, PosRef pos, int nchunk, int M, int logits_rows, float* logits_dst);
int forward_block(stairs_ctx* c, Model* m, PosRef pos, int nchunk, int M, int logits_rows);

// logits_dst: where the logits rows go (nullptr: c->logits)
int forward(stairs_ctx* c, Model* m, PosRef pos, int nchunk, int M, int logits_rows, int slot = 0, float* logits_dst = nullptr) {
  if (m->encdec) {
    if (slot != 0 || pos.rps) return fail(c, STAIRS_EINVAL, "forward: encoder-decoder models take one sequence");
    return forward_ed(c, m, pos, nchunk, M, logits_rows, logits_dst);
  }
  if (M > c->fwd_rows) {                    // many sequences at once: the block kernels
    if (slot != 0 || logits_dst) return fail(c, STAIRS_EINVAL, "forward: launch shape outside the workspaces");
    return forward_block(c, m, pos, nchunk, M, logits_rows);
  }
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, f = g.d_ffn, H = g.n_heads, V = g.vocab;
  const int b = m->bf16 ? 1 : 0;
  const int sn = ssq_groups(d, b);
  hipStream_t st = c->st;
  if (nchunk < 1 || nchunk > c->nchunk_cap || M < 1 || M > c->fwd_rows || M > c->rows_cap || (M > kMaxRows && !b))
    return fail(c, STAIRS_EINVAL, "forward: launch shape outside the workspaces");
#define SYNCPOINT()                                             \
  do {                                                          \
    if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(st));  \
  } while (0)
  const int nslots = pos.rps ? M / pos.rps : 1;
  const int rows_per_slot = pos.rps ? pos.rps : M;
  const size_t slot_bytes = (size_t)g.n_layers * m->kv_layer_bytes;
  const size_t slot_off = pos.rps ? 0 : (size_t)slot * slot_bytes;
  if (slot < 0 || slot >= c->n_slots || nslots > c->n_slots || nslots * H > kAttnCounters || (pos.rps && (M % pos.rps || !b)))
    return fail(c, STAIRS_EINVAL, "forward: slots outside what the context holds");
  // more than 4 rows (bf16): every producer of an activation also leaves its MFMA operand fragments, with the gain of
  // the norm in front of the next projection folded in, and the projections take the hand-off-free kernel
  const bool fr = b && M > 4;
  // more than kMaxRows rows exist only on the hand-off-free GEMM: every projection must fit it
  if (M > kMaxRows && !(fr && gemm_takes_rows(M, std::max(d, f))))
    return fail(c, STAIRS_EINVAL, "forward: more rows than the weight-streaming kernels take for this model");
  launch_embed(m->tok_emb, b, c->tokens + (pos.rps ? 0 : (size_t)slot * c->tok_stride), pos.rps ? c->tok_stride : 0,
               c->tok_stride, V, pos, M, d, c->x, c->ssq, m->hd, g.rope_theta, c->rope_cs, st, fr ? c->xf : nullptr,
               m->layers[0].attn_norm);
  SYNCPOINT();
  const RowNorm none{nullptr, nullptr, 0, 0.f};
  AttnMode amode{0.f, nullptr, 0, 0, 0, fr ? c->af : nullptr};
  for (int l = 0; l < g.n_layers; ++l) {
    const Layer& ly = m->layers[l];
    char* Kl = m->Kc + slot_off + l * m->kv_layer_bytes;
    char* Vl = m->Vc + slot_off + l * m->kv_layer_bytes;
    GemmEpi e{};
    e.counters = c->counters;
    e.stream_weights = m->stream_weights;
    e.rope_cs = c->rope_cs;
    e.pos = pos;
    e.Kc = reinterpret_cast<_Float16*>(Kl);
    e.Vc = reinterpret_cast<_Float16*>(Vl);
    e.Kc32 = reinterpret_cast<float*>(Kl);
    e.Vc32 = reinterpret_cast<float*>(Vl);
    e.cap = m->cap;
    e.H = H;
    e.hd = m->hd;
    e.kv_slot_stride = slot_bytes / m->esz();
    e.ssq_out = c->ssq;
    e.out = c->q_rot;
    RowNorm an{ly.attn_norm, c->ssq, sn, g.rms_eps};
    launch_gemm(kRoleQKV, b, ly.wqkv, 3 * d, d, c->x, d, M, an, c->partial, e, st, fr ? c->xf : nullptr);
    SYNCPOINT();
    launch_attention(c->q_rot, Kl, Vl, b, m->cap, d, H, rows_per_slot, pos, nslots, slot_bytes / m->esz(), nchunk,
                     c->nchunk_cap, c->part_o, c->part_ml, c->counters + kGemmCounters, c->attn_out, st, amode);
    SYNCPOINT();
    e.out = c->x;
    e.frag_out = fr ? c->xf : nullptr;             // x after the attention block, for the gate/up projection
    e.frag_gain = ly.ffn_norm;
    launch_gemm(kRoleWo, b, ly.wo, d, d, c->attn_out, d, M, none, c->partial, e, st, fr ? c->af : nullptr);
    SYNCPOINT();
    e.out = c->h;
    e.frag_out = fr ? c->hf : nullptr;             // the SwiGLU output, for the down projection
    e.frag_gain = nullptr;
    if (c->probe_role == kProbeEmptyPair) {      // calibration: the pair with nothing between its two records
      HIPCHK(c, hipEventRecord(c->probe_ev[2 * l], st));
      HIPCHK(c, hipEventRecord(c->probe_ev[2 * l + 1], st));
    }
    if (c->probe_role == kRoleGateUp) HIPCHK(c, hipEventRecord(c->probe_ev[2 * l], st));
    if (c->probe_role == kProbeKernelEvents) set_gemm_launch_events(c->probe_ev[2 * l], c->probe_ev[2 * l + 1]);
    RowNorm fn{ly.ffn_norm, c->ssq, sn, g.rms_eps};
    launch_gemm(kRoleGateUp, b, ly.wgu, 2 * f, d, c->x, d, M, fn, c->partial, e, st, fr ? c->xf : nullptr);
    if (c->probe_role == kRoleGateUp) HIPCHK(c, hipEventRecord(c->probe_ev[2 * l + 1], st));
    SYNCPOINT();
    e.out = c->x;
    e.frag_out = fr ? c->xf : nullptr;             // x after the layer, for the next layer's QKV or the unembedding
    e.frag_gain = l + 1 < g.n_layers ? m->layers[l + 1].attn_norm : m->final_norm;
    launch_gemm(kRoleDown, b, ly.wdown, d, f, c->h, f, M, none, c->partial, e, st, fr ? c->hf : nullptr);
    SYNCPOINT();
  }
  if (logits_rows > 0) {
    const int r0 = M - logits_rows;
    GemmEpi e{};
    e.counters = c->counters;
    e.stream_weights = m->stream_weights;
    e.out = logits_dst ? logits_dst : c->logits;
    e.hd = m->hd;
    // (the fragments hold all M rows: usable when the unembedding takes them all)
    launch_gemm(kRoleHead, b, m->lm_head, V, d, c->x + (size_t)r0 * d, d, logits_rows,
                RowNorm{m->final_norm, c->ssq + r0 * sn, sn, g.rms_eps}, c->partial, e, st, (fr && r0 == 0) ? c->xf : nullptr);
    SYNCPOINT();
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
#undef SYNCPOINT
}

// A forward of 33 .. kMaxBlockRows rows of several sequences (pos.rps rows per slot) on the block kernels: the
// projections run on the MFMA-bound GEMM of the prompt ingestion over all rows at once, attention on the decode
// kernel (one grid slice per slot, each against its own cache), the rest is element-wise.  Every output has one order
// of additions whatever the number of rows, so a sequence's results do not depend on which others share the forward
// (they are not the bits of the decode kernels, whose additions go chunk by chunk).  All rows' logits -> c->logits.
int forward_block(stairs_ctx* c, Model* m, PosRef pos, int nchunk, int M, int logits_rows) {
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, f = g.d_ffn, H = g.n_heads, V = g.vocab;
  hipStream_t st = c->st;
  if (!c->block_prefill || !m->bf16 || m->encdec || !pos.rps || M % pos.rps || M > kMaxBlockRows || M > c->pf_rows || M > c->rows_cap ||
      (logits_rows != 0 && logits_rows != M))
    return fail(c, STAIRS_EINVAL, "forward: rows outside what the block workspaces hold");
  const int nslots = M / pos.rps;
  if (nchunk < 1 || nchunk > c->nchunk_cap || nslots > c->n_slots || nslots * H > kAttnCounters)
    return fail(c, STAIRS_EINVAL, "forward: launch shape outside the workspaces");
  const size_t slot_bytes = (size_t)g.n_layers * m->kv_layer_bytes;
  const size_t slot_stride = slot_bytes / m->esz();
  // (the gather also leaves sum-of-squares partials nobody needs here: into pf_y, which is scratch until the first GEMM)
  launch_embed(m->tok_emb, 1, c->tokens, c->tok_stride, c->tok_stride, V, pos, M, d, c->pf_x, c->pf_y, m->hd, g.rope_theta, c->pf_cs, st);
  const AttnMode amode{0.f, nullptr, 0, 0, 0, nullptr};
  for (int l = 0; l < g.n_layers; ++l) {
    const Layer& ly = m->layers[l];
    char* Kl = m->Kc + l * m->kv_layer_bytes;
    char* Vl = m->Vc + l * m->kv_layer_bytes;
    launch_pf_norm_split(c->pf_x, ly.attn_norm, g.rms_eps, M, d, c->pf_frag, st);
    launch_gemm_block(ly.wqkv, 3 * d, d, c->pf_frag, M, c->pf_y, 3 * d, kPermQKV, d, m->hd, 0, st, c->pf_part, c->pf_part_floats);
    launch_pf_rope_kv_rows(c->pf_y, M, d, H, pos, slot_stride, c->pf_cs, c->pf_q, reinterpret_cast<_Float16*>(Kl),
                           reinterpret_cast<_Float16*>(Vl), m->cap, st);
    launch_attention(c->pf_q, Kl, Vl, 1, m->cap, d, H, pos.rps, pos, nslots, slot_stride, nchunk, c->nchunk_cap, c->part_o,
                     c->part_ml, c->counters + kGemmCounters, c->pf_attn, st, amode);
    launch_pf_norm_split(c->pf_attn, nullptr, 0.f, M, d, c->pf_frag, st);
    launch_gemm_block(ly.wo, d, d, c->pf_frag, M, c->pf_x, d, kPermNone, 0, 0, 1, st, c->pf_part, c->pf_part_floats);
    launch_pf_norm_split(c->pf_x, ly.ffn_norm, g.rms_eps, M, d, c->pf_frag, st);
    launch_gemm_block(ly.wgu, 2 * f, d, c->pf_frag, M, c->pf_y, 2 * f, kPermGateUp, f, 0, 0, st, c->pf_part, c->pf_part_floats);
    launch_pf_swiglu_split(c->pf_y, M, f, c->pf_frag, st);
    launch_gemm_block(ly.wdown, d, f, c->pf_frag, M, c->pf_x, d, kPermNone, 0, 0, 1, st, c->pf_part, c->pf_part_floats);
    if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(st));
  }
  if (logits_rows > 0) {
    launch_pf_norm_split(c->pf_x, m->final_norm, g.rms_eps, M, d, c->pf_frag, st);
    launch_gemm_block(m->lm_head, V, d, c->pf_frag, M, c->logits, V, kPermNone, 0, 0, 0, st, c->pf_part, c->pf_part_floats);
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

PosRef abs_pos(const stairs_ctx* c, int p) { return PosRef{c->state + 2, p}; }   // state[2] == 0
PosRef rel_pos(const stairs_ctx* c, int off) { return PosRef{c->state, off}; }     // state[0] == L, kept on the device
int chunks_for(int kv_len) { return (std::max(kv_len, 1) + kAttnChunk - 1) / kAttnChunk; }

// The feed-forward block of an encoder-decoder layer on M rows of x (ssq = their sum-of-squares partials):
// x += W_out relu(W_in norm(x)); h = workspace [M, f].
// frags: x comes with its activation fragments in c->xf (gain of ffn_norm folded in), the hidden activations leave
// theirs in c->hf and the result its own in c->xf with next_gain folded in (forwards of more than 4 rows)
void launch_ed_ffn(stairs_ctx* c, const Model* m, const EdLayer& ly, float* x, float* ssq, int M, bool frags = false,
                   const float* next_gain = nullptr) {
  const int d = m->cfg.d_model, f = m->cfg.d_ffn, sn = ssq_groups(d, 1);
  const RowNorm none{nullptr, nullptr, 0, 0.f};
  GemmEpi e{};
  e.counters = c->counters;
  e.stream_weights = m->stream_weights;
  e.hd = m->hd;
  e.out = c->h;
  e.act = kActRelu;
  e.frag_out = frags ? c->hf : nullptr;
  RowNorm fn{ly.ffn_norm, ssq, sn, m->cfg.rms_eps};
  launch_gemm(kRoleHead, 1, ly.w_in, f, d, x, d, M, fn, c->partial, e, c->st, frags ? c->xf : nullptr);
  e.act = kActNone;
  e.out = x;
  e.ssq_out = ssq;
  e.frag_out = frags ? c->xf : nullptr;
  e.frag_gain = next_gain;
  launch_gemm(kRoleDown, 1, ly.w_out, d, f, c->h, f, M, none, c->partial, e, c->st, frags ? c->hf : nullptr);
}

// Decoder forward of an encoder-decoder model: M rows of the decoder sequence at pos.. (see forward()).  Per layer:
// self-attention over the decoder's cache with the one-sided position bias, cross-attention over the keys and
// values stairs_encode left for this layer (every row sees all c->S source positions), feed-forward.
int forward_ed(stairs_ctx* c, Model* m, PosRef pos, int nchunk, int M, int logits_rows, float* logits_dst) {
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, a = m->da, H = g.n_heads, V = g.vocab;
  const int sn = ssq_groups(d, 1);
  hipStream_t st = c->st;
  const int nch_src = chunks_for(c->S);
  if (nchunk < 1 || nchunk > c->nchunk_cap || nch_src > c->nchunk_cap || M < 1 || M > kMaxRows || c->S < 1)
    return fail(c, STAIRS_EINVAL, "forward: launch shape outside the workspaces");
#define SYNCPOINT()                                             \
  do {                                                          \
    if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(st));  \
  } while (0)
  // more than 4 rows: every producer of an activation also leaves its MFMA operand fragments (gain of the norm in
  // front of the next projection folded in) and the projections take the hand-off-free kernel, as in forward()
  const bool fr = M > 4;
  uint4* const xf = fr ? c->xf : nullptr;
  uint4* const af = fr ? c->af : nullptr;
  launch_embed(m->tok_emb, 1, c->tokens, 0, c->tok_stride, V, pos, M, d, c->x, c->ssq, m->hd, 0.f, c->rope_cs, st, xf,
               m->dec[0].attn_norm);
  SYNCPOINT();
  const RowNorm none{nullptr, nullptr, 0, 0.f};
  const AttnMode self_mode{1.f, m->dec_bias, m->cap, m->cap - 1, 0, af};
  const AttnMode cross_mode{1.f, nullptr, 0, 0, c->S, af};
  auto normed = [&](const float* gain) {
    RowNorm n{gain, c->ssq, sn, g.rms_eps};
    return n;
  };
  for (int l = 0; l < g.n_layers; ++l) {
    const EdLayer& ly = m->dec[l];
    char* Kl = m->Kc + l * m->kv_layer_bytes;
    char* Vl = m->Vc + l * m->kv_layer_bytes;
    GemmEpi e{};
    e.counters = c->counters;
    e.stream_weights = m->stream_weights;
    e.rope_cs = c->rope_cs;
    e.pos = pos;
    e.Kc = reinterpret_cast<_Float16*>(Kl);
    e.Vc = reinterpret_cast<_Float16*>(Vl);
    e.cap = m->cap;
    e.H = H;
    e.hd = m->hd;
    e.ssq_out = c->ssq;
    e.out = c->q_rot;
    launch_gemm(kRoleQKV, 1, ly.wqkv, 3 * a, d, c->x, d, M, normed(ly.attn_norm), c->partial, e, st, xf);
    SYNCPOINT();
    launch_attention(c->q_rot, Kl, Vl, 1, m->cap, a, H, M, pos, 1, 0, nchunk, c->nchunk_cap, c->part_o, c->part_ml,
                     c->counters + kGemmCounters, c->attn_out, st, self_mode);
    SYNCPOINT();
    e.out = c->x;
    e.frag_out = xf;                               // x after self-attention, for the cross-attention queries
    e.frag_gain = ly.cross_norm;
    launch_gemm(kRoleWo, 1, ly.wo, d, a, c->attn_out, a, M, none, c->partial, e, st, af);
    SYNCPOINT();
    e.out = c->q_rot;
    e.frag_out = nullptr;
    e.frag_gain = nullptr;
    launch_gemm(kRoleHead, 1, ly.cq, a, d, c->x, d, M, normed(ly.cross_norm), c->partial, e, st, xf);
    SYNCPOINT();
    launch_attention(c->q_rot, m->Kx + l * m->kvx_layer_bytes, m->Vx + l * m->kvx_layer_bytes, 1, m->cap_src, a, H, M, pos, 1, 0,
                     nch_src, c->nchunk_cap, c->part_o, c->part_ml, c->counters + kGemmCounters, c->attn_out, st, cross_mode);
    SYNCPOINT();
    e.out = c->x;
    e.frag_out = xf;                               // x after cross-attention, for the feed-forward block
    e.frag_gain = ly.ffn_norm;
    launch_gemm(kRoleWo, 1, ly.co, d, a, c->attn_out, a, M, none, c->partial, e, st, af);
    SYNCPOINT();
    launch_ed_ffn(c, m, ly, c->x, c->ssq, M, fr, l + 1 < g.n_layers ? m->dec[l + 1].attn_norm : m->final_norm);
    SYNCPOINT();
  }
  if (logits_rows > 0) {
    const int r0 = M - logits_rows;
    GemmEpi e{};
    e.counters = c->counters;
    e.stream_weights = m->stream_weights;
    e.out = logits_dst ? logits_dst : c->logits;
    e.hd = m->hd;
    launch_gemm(kRoleHead, 1, m->lm_head, V, d, c->x + (size_t)r0 * d, d, logits_rows,
                RowNorm{m->final_norm, c->ssq + r0 * sn, sn, g.rms_eps}, c->partial, e, st, r0 == 0 ? xf : nullptr);
    SYNCPOINT();
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

// Encoder of one model over the c->S source tokens in c->src_tok, 32 rows at a time through the decode kernels:
// per layer first the keys and values of all rows (every row attends to every source position), then attention
// with the two-sided position bias, output projection and feed-forward block by block.  Afterwards the
// cross-attention keys and values of every decoder layer are formed from the normalised encoder output.
int encode_model(stairs_ctx* c, Model* m) {
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, a = m->da, H = g.n_heads, S = c->S;
  const int sn = ssq_groups(d, 1);
  hipStream_t st = c->st;
  const int nch = chunks_for(S);
  if (S < 1 || S > m->max_src || nch > c->nchunk_cap) return fail(c, STAIRS_EINVAL, "encode: source outside the workspaces");
  const RowNorm none{nullptr, nullptr, 0, 0.f};
  const AttnMode mode{1.f, m->enc_bias, 2 * m->max_src - 1, m->max_src - 1, S};
  auto rows_of = [&](int b) { return std::min(kMaxRows, S - b); };
  auto epi_for = [&](int b, char* K, char* V, float* out) {
    GemmEpi e{};
    e.counters = c->counters;
    e.stream_weights = m->stream_weights;
    e.rope_cs = c->rope_cs;
    e.pos = abs_pos(c, b);
    e.Kc = reinterpret_cast<_Float16*>(K);
    e.Vc = reinterpret_cast<_Float16*>(V);
    e.cap = m->cap_src;
    e.H = H;
    e.hd = m->hd;
    e.ssq_out = c->enc_ssq + (size_t)b * sn;
    e.out = out;
    return e;
  };
  auto normed = [&](const float* gain, int b, int M) {
    RowNorm n{gain, c->enc_ssq + (size_t)b * sn, sn, g.rms_eps};
    return n;
  };
  for (int b = 0; b < S; b += kMaxRows)
    launch_embed(m->tok_emb, 1, c->src_tok, 0, S, g.vocab, abs_pos(c, b), rows_of(b), d, c->enc_x + (size_t)b * d,
                 c->enc_ssq + (size_t)b * sn, m->hd, 0.f, c->rope_cs, st);
  for (size_t l = 0; l < m->enc.size(); ++l) {
    const EdLayer& ly = m->enc[l];
    for (int b = 0; b < S; b += kMaxRows) {
      const int M = rows_of(b);
      launch_gemm(kRoleQKV, 1, ly.wqkv, 3 * a, d, c->enc_x + (size_t)b * d, d, M, normed(ly.attn_norm, b, M), c->partial,
                  epi_for(b, m->Ke, m->Ve, c->enc_q + (size_t)b * a), st);
    }
    for (int b = 0; b < S; b += kMaxRows) {
      const int M = rows_of(b);
      launch_attention(c->enc_q + (size_t)b * a, m->Ke, m->Ve, 1, m->cap_src, a, H, M, abs_pos(c, b), 1, 0, nch, c->nchunk_cap,
                       c->part_o, c->part_ml, c->counters + kGemmCounters, c->attn_out, st, mode);
      launch_gemm(kRoleWo, 1, ly.wo, d, a, c->attn_out, a, M, none, c->partial, epi_for(b, m->Ke, m->Ve, c->enc_x + (size_t)b * d), st);
      launch_ed_ffn(c, m, ly, c->enc_x + (size_t)b * d, c->enc_ssq + (size_t)b * sn, M);
    }
    if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(st));
  }
  for (size_t l = 0; l < m->dec.size(); ++l)
    for (int b = 0; b < S; b += kMaxRows) {
      const int M = rows_of(b);
      launch_gemm(kRoleQKV, 1, m->dec[l].cqkv, 3 * a, d, c->enc_x + (size_t)b * d, d, M, normed(m->enc_final_norm, b, M), c->partial,
                  epi_for(b, m->Kx + l * m->kvx_layer_bytes, m->Vx + l * m->kvx_layer_bytes, c->enc_q + (size_t)b * a), st);
    }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

// Positions [from, to) of sequence slot `slot` into a model's cache in blocks of up to kPfRows rows: the four
// projections of a layer run on the MFMA-bound block GEMM over the whole block (the residual additions inside it),
// attention on k_attn_flash (its keys include the block's own rows, appended just before), the rest is element-wise.
int ingest_blocks(stairs_ctx* c, Model* m, int from, int to, int slot) {
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, f = g.d_ffn, H = g.n_heads;
  hipStream_t st = c->st;
  const size_t slot_bytes = (size_t)g.n_layers * m->kv_layer_bytes;
  const int* tokens = c->tokens + (size_t)slot * c->tok_stride;
#define PF_SYNC()                                               \
  do {                                                          \
    if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(st));  \
  } while (0)
  for (int p0 = from; p0 < to; p0 += kPfRows) {
    const int R = std::min(kPfRows, to - p0);
    launch_pf_embed(static_cast<const uint16_t*>(m->tok_emb), tokens, p0, c->tok_stride, g.vocab, R, d, c->pf_x, st);
    PF_SYNC();
    launch_pf_rope_table(p0, R, m->hd, g.rope_theta, c->pf_cs, st);
    PF_SYNC();
    for (int l = 0; l < g.n_layers; ++l) {
      const Layer& ly = m->layers[l];
      char* Kl = m->Kc + (size_t)slot * slot_bytes + l * m->kv_layer_bytes;
      char* Vl = m->Vc + (size_t)slot * slot_bytes + l * m->kv_layer_bytes;
      launch_pf_norm_split(c->pf_x, ly.attn_norm, g.rms_eps, R, d, c->pf_frag, st);
      PF_SYNC();
      launch_gemm_block(ly.wqkv, 3 * d, d, c->pf_frag, R, c->pf_y, 3 * d, kPermQKV, d, m->hd, 0, st, c->pf_part, c->pf_part_floats);
      PF_SYNC();
      launch_pf_rope_kv(c->pf_y, R, d, H, p0, c->pf_cs, c->pf_q, reinterpret_cast<_Float16*>(Kl), reinterpret_cast<_Float16*>(Vl),
                        m->cap, st);
      PF_SYNC();
      launch_attention_flash(c->pf_q, Kl, Vl, m->cap, d, H, R, p0, c->pf_attn, st);
      PF_SYNC();
      launch_pf_norm_split(c->pf_attn, nullptr, 0.f, R, d, c->pf_frag, st);
      PF_SYNC();
      launch_gemm_block(ly.wo, d, d, c->pf_frag, R, c->pf_x, d, kPermNone, 0, 0, 1, st, c->pf_part, c->pf_part_floats);
      PF_SYNC();
      launch_pf_norm_split(c->pf_x, ly.ffn_norm, g.rms_eps, R, d, c->pf_frag, st);
      PF_SYNC();
      launch_gemm_block(ly.wgu, 2 * f, d, c->pf_frag, R, c->pf_y, 2 * f, kPermGateUp, f, 0, 0, st, c->pf_part, c->pf_part_floats);
      PF_SYNC();
      launch_pf_swiglu_split(c->pf_y, R, f, c->pf_frag, st);
      PF_SYNC();
      launch_gemm_block(ly.wdown, d, f, c->pf_frag, R, c->pf_x, d, kPermNone, 0, 0, 1, st, c->pf_part, c->pf_part_floats);
      PF_SYNC();
    }
    HIPCHK(c, hipGetLastError());
  }
#undef PF_SYNC
  return STAIRS_OK;
}

constexpr int kBlockPrefillMin = 64;   // fewer rows than this go through the decode kernels

// ingest positions [from, to) of sequence slot `slot` into a model's cache, no logits
int ingest(stairs_ctx* c, Model* m, int from, int to, int slot = 0) {
  // (STAIRS_SYNC_LAUNCHES=1, a wait after every launch for a counter-collecting profiler: the decode kernels
  // ingest the prompt; =2 keeps the block kernels)
  if (c->block_prefill && (!c->sync_launches || c->sync_blocks) && m->bf16 && !m->encdec && to - from >= kBlockPrefillMin) {
    int rc = ingest_blocks(c, m, from, to, slot);
    if (rc) return rc;
  } else {
    for (int p = from; p < to; p += kMaxRows) {
      const int M = std::min(kMaxRows, to - p);
      int rc = forward(c, m, abs_pos(c, p), chunks_for(p + M), M, 0, slot);
      if (rc) return rc;
    }
  }
  if (slot == 0 && to > m->valid) m->valid = to;
  return STAIRS_OK;
}

// Enqueue the draft's k greedy steps.  Positions are taken relative to the device-side sequence
// length (state[0] == L), so the same launches can be replayed for any L; nch = attention chunks to launch.
int enqueue_propose(stairs_ctx* c, int k, int nch) {
  Model* m = &c->D;
  const int V = m->cfg.vocab;
  // step 1: rows at L-2, L-1 (row L-2 is recomputed when it is already cached: same values);
  // its argmax is d_1 -> tokens[L].  Steps 2..k: one row each.
  int rc = forward(c, m, rel_pos(c, -2), nch, 2, 1);
  if (rc) return rc;
  launch_argmax(c->logits, V, V, 1, 0, 1, c->tokens, rel_pos(c, 0), 0, c->st);
  for (int j = 1; j < k; ++j) {
    rc = forward(c, m, rel_pos(c, j - 1), nch, 1, 1);
    if (rc) return rc;
    launch_argmax(c->logits, V, V, 1, 0, 1, c->tokens, rel_pos(c, j), 0, c->st);
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

// Enqueue the stair batch for the k draft tokens sitting in tokens[L..L+k), its per-row argmax and the validation.
int enqueue_verify(stairs_ctx* c, int k, int nch) {
  Model* m = &c->T;
  const int M = k + 1, V = m->cfg.vocab;
  int rc = forward(c, m, rel_pos(c, -1), nch, M, M);
  if (rc) return rc;
  launch_argmax(c->logits, V, V, M, 0, 1, c->tgt_tok, PosRef{nullptr, 0}, 0, c->st);
  launch_accept(c->tokens, c->tgt_tok, k, c->state, 1, 0, c->st);
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

// The two halves of a SAMPLED iteration: the assistant draws its k tokens one by one (its logits rows stay in
// c->dlogits for the validation), then the stair batch, the rows' log-sum-exps and the keep / replace walk.
int enqueue_propose_sampled(stairs_ctx* c, int k, int nch) {
  Model* m = &c->D;
  const int V = m->cfg.vocab;
  int rc = forward(c, m, rel_pos(c, -2), nch, 2, 1, 0, c->dlogits);
  if (rc) return rc;
  launch_sample(c->dlogits, V, c->samp, 0, c->tokens, rel_pos(c, 0), c->samp_ws, c->st);
  for (int j = 1; j < k; ++j) {
    rc = forward(c, m, rel_pos(c, j - 1), nch, 1, 1, 0, c->dlogits + (size_t)j * V);
    if (rc) return rc;
    launch_sample(c->dlogits + (size_t)j * V, V, c->samp, 0, c->tokens, rel_pos(c, j), c->samp_ws, c->st);
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

int enqueue_verify_sampled(stairs_ctx* c, int k, int nch) {
  Model* m = &c->T;
  const int M = k + 1, V = m->cfg.vocab;
  int rc = forward(c, m, rel_pos(c, -1), nch, M, M);
  if (rc) return rc;
  launch_row_lse(c->logits, M, c->dlogits, k, V, V, c->samp, c->lse, c->st);
  launch_accept_sampled(c->tokens, c->logits, c->dlogits, V, V, k, c->lse, c->samp, c->state, c->tgt_tok, c->samp_ws, c->st);
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

// temperature and seed of the sampled calls onto the device (buffers on first use)
int set_sampling(stairs_ctx* c, float temperature, uint64_t seed) {
  if (!(temperature > 0.f) || !(temperature < 1e6f)) return fail(c, STAIRS_EINVAL, "temperature must be positive");
  if (c->n_slots != 1) return fail(c, STAIRS_EINVAL, "sampling takes a context without reserved batch slots");
  int rc;
  if (!c->samp) {
    const size_t V = c->T.cfg.vocab;
    if ((rc = dev_alloc(c, &c->samp, 1)) || (rc = dev_alloc(c, &c->samp_ws, 1)) ||
        (rc = dev_alloc(c, &c->dlogits, (size_t)kMaxRows * V)) || (rc = dev_alloc(c, &c->lse, (size_t)2 * kMaxRows)))
      return rc;
    HIPCHK(c, hipMemsetAsync(c->samp_ws, 0, sizeof(SampleWs), c->st));
  }
  uint64_t z = seed + 0x9E3779B97F4A7C15ull;       // one splitmix64 step, forced odd
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  const SampleParams sp{1.0f / temperature, (z ^ (z >> 31)) | 1ull};
  HIPCHK(c, hipMemcpyAsync(c->samp, &sp, sizeof(sp), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));           // sp is on the stack
  return STAIRS_OK;
}

// The same two halves for B sequences at once: every forward holds the rows of all slots (2, then 1, then k+1 per
// slot), positions, token arrays and caches are looked up per slot on the device.
int enqueue_propose_batch(stairs_ctx* c, int B, int k, int nch) {
  Model* m = &c->D;
  const int V = m->cfg.vocab;
  int rc = forward(c, m, PosRef{c->state, -2, 2}, nch, 2 * B, 2 * B);
  if (rc) return rc;
  launch_argmax(c->logits, V, V, B, 1, 2, c->tokens, PosRef{c->state, 0, 1}, c->tok_stride, c->st);   // each slot's 2nd row
  for (int j = 1; j < k; ++j) {
    rc = forward(c, m, PosRef{c->state, j - 1, 1}, nch, B, B);
    if (rc) return rc;
    launch_argmax(c->logits, V, V, B, 0, 1, c->tokens, PosRef{c->state, j, 1}, c->tok_stride, c->st);
  }
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

int enqueue_verify_batch(stairs_ctx* c, int B, int k, int nch) {
  Model* m = &c->T;
  const int M = k + 1, V = m->cfg.vocab;
  int rc = forward(c, m, PosRef{c->state, -1, M}, nch, B * M, B * M);
  if (rc) return rc;
  launch_argmax(c->logits, V, V, B * M, 0, 1, c->tgt_tok, PosRef{nullptr, 0}, 0, c->st);
  launch_accept(c->tokens, c->tgt_tok, k, c->state, B, c->tok_stride, c->st);
  HIPCHK(c, hipGetLastError());
  return STAIRS_OK;
}

int do_propose(stairs_ctx* c, int k, bool sampled = false) {
  Model* m = &c->D;
  const int L = c->L;
  // the draft's cache must hold positions 0..L-3; the 2-row first step covers L-2 and L-1
  if (m->valid < L - 2) {
    int rc = ingest(c, m, m->valid, L - 2);
    if (rc) return rc;
  }
  int rc = sampled ? enqueue_propose_sampled(c, k, chunks_for(L + k - 1)) : enqueue_propose(c, k, chunks_for(L + k - 1));
  if (rc) return rc;
  m->valid = L + k - 1;      // tokens S, d_1..d_{k-1} are in the cache
  c->pending_k = k;
  c->pending_sampled = sampled;
  return STAIRS_OK;
}

// read back what the validation kernel decided and move the host's mirror of the state
int finish_verify(stairs_ctx* c, int k, int* n_out) {
  const int L = c->L, M = k + 1;
  HIPCHK(c, hipMemcpyAsync(c->h_pinned, c->state, 2 * sizeof(int), hipMemcpyDeviceToHost, c->st));
  HIPCHK(c, hipMemcpyAsync(c->h_pinned + 2, c->tgt_tok, M * sizeof(int), hipMemcpyDeviceToHost, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));
  const int n = c->h_pinned[1];
  if (c->h_pinned[0] != L + n + 1 || n < 0 || n > k) return fail(c, STAIRS_EHIP, "device state out of sync with host");
  c->L = L + n + 1;
  c->T.valid = L + n;                                 // positions L-1 .. L-1+n stay
  if (c->have_draft) c->D.valid = std::min(c->D.valid, L + n);
  c->pending_k = -1;
  *n_out = n;
  return STAIRS_OK;
}

int do_verify(stairs_ctx* c, int k, int* n_out, bool sampled = false) {
  int rc = sampled ? enqueue_verify_sampled(c, k, chunks_for(c->L + k)) : enqueue_verify(c, k, chunks_for(c->L + k));
  if (rc) return rc;
  return finish_verify(c, k, n_out);
}

// The two halves of an iteration -- (0) the k draft steps, (1) stair batch + argmax + validation -- as HIP
// graphs that are replayed while their launch shapes stay valid: positions come from the device, only the
// attention grid (nch chunks, padded to a multiple of 4) bounds the sequence length a graph can serve.
int iteration_graph(stairs_ctx* c, int half, int k, int nch, hipGraphExec_t* out, int B = 0) {
  for (auto& g : c->graphs)
    if (g.half == half && g.k == k && g.nch == nch && g.B == B) {
      *out = g.exec;
      return STAIRS_OK;
    }
  hipGraph_t graph = nullptr;
  HIPCHK(c, hipStreamBeginCapture(c->st, hipStreamCaptureModeThreadLocal));
  const int rc = B > 0 ? (half == 0 ? enqueue_propose_batch(c, B, k, nch) : enqueue_verify_batch(c, B, k, nch))
                 : B < 0 ? (half == 0 ? enqueue_propose_sampled(c, k, nch) : enqueue_verify_sampled(c, k, nch))
                         : (half == 0 ? enqueue_propose(c, k, nch) : enqueue_verify(c, k, nch));
  hipError_t e = hipStreamEndCapture(c->st, &graph);
  if (rc) {
    if (graph) (void)hipGraphDestroy(graph);
    return rc;
  }
  HIPCHK(c, e);
  hipGraphExec_t exec = nullptr;
  e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  HIPCHK(c, e);
  c->graphs.push_back({half, k, nch, B, exec});
  *out = exec;
  return STAIRS_OK;
}

int copy_out(stairs_ctx* c, void* dst, const void* src, size_t bytes) {
  HIPCHK(c, hipMemcpyAsync(dst, src, bytes, hipMemcpyDefault, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));
  return STAIRS_OK;
}

int capacity_ok(const stairs_ctx* c, int need) {
  if (need > c->T.cap) return 0;
  if (c->have_draft && need > c->D.cap) return 0;
  return need <= c->tok_cap;
}

}  // namespace

// =========================================================================================
extern "C" {

const char* stairs_strerror(int code) {
  switch (code) {
    case STAIRS_OK: return "ok";
    case STAIRS_EINVAL: return "invalid argument";
    case STAIRS_ECAPACITY: return "sequence exceeds max_seq";
    case STAIRS_ESTATE: return "call not allowed in this state";
    case STAIRS_ENOMEM: return "out of memory";
    case STAIRS_EHIP: return "HIP runtime error";
    default: return "unknown error";
  }
}

const char* stairs_last_error(const stairs_ctx* ctx) { return ctx ? ctx->err.c_str() : "context is NULL"; }

void stairs_free(stairs_ctx* c) {
  if (!c) return;
  (void)hipStreamSynchronize(c->st);
  for (auto& g : c->graphs) (void)hipGraphExecDestroy(g.exec);
  for (auto& e : c->probe_ev) (void)hipEventDestroy(e);
  for (void* p : c->owned) (void)hipFree(p);
  if (c->h_pinned) (void)hipHostFree(c->h_pinned);
  for (auto& e : c->ev)
    if (e) (void)hipEventDestroy(e);
  if (c->own_stream) (void)hipStreamDestroy(c->st);
  delete c;
}

// Sizes of the workspaces shared by the two models of a context
struct WsDims {
  int dmax, amax, fmax, Hmax, capmax, vocab;
  int srcmax;          // encoder-decoder contexts: most source positions, else 0
  size_t partial_floats;
};

// new context on the caller's stream (or one of its own), environment switches read
static stairs_ctx* new_ctx(void* hip_stream, int k_max, bool have_draft, bool block_prefill_ok, int* rc_out) {
  stairs_ctx* c = new (std::nothrow) stairs_ctx;
  if (!c) {
    *rc_out = STAIRS_ENOMEM;
    return nullptr;
  }
  c->st = static_cast<hipStream_t>(hip_stream);
  if (!c->st) {   // graph capture needs a real stream; default priority
    if (hipStreamCreateWithFlags(&c->st, hipStreamNonBlocking) != hipSuccess) {
      delete c;
      *rc_out = STAIRS_EHIP;
      return nullptr;
    }
    c->own_stream = true;
  }
  c->k_max = k_max;
  c->have_draft = have_draft;
  const char* e = getenv("STAIRS_SYNC_LAUNCHES");
  c->sync_launches = e && (e[0] == '1' || e[0] == '2');
  c->sync_blocks = e && e[0] == '2';
  e = getenv("STAIRS_NO_GRAPH");
  c->use_graphs = !(e && e[0] == '1') && !c->sync_launches;
  e = getenv("STAIRS_NO_BLOCK_PREFILL");
  c->block_prefill = block_prefill_ok && !(e && e[0] == '1');
  *rc_out = STAIRS_OK;
  return c;
}

static int alloc_workspaces(stairs_ctx* c, const WsDims& w);

int stairs_init(stairs_ctx** out, const stairs_model_cfg* tcfg, const stairs_weights* tw, const stairs_model_cfg* dcfg,
                const stairs_weights* dw, int32_t k_max, void* hip_stream) {
  if (!out) return STAIRS_EINVAL;
  *out = nullptr;
  if (check_cfg(tcfg) || check_weights(tcfg, tw)) return STAIRS_EINVAL;
  const bool have_draft = dcfg != nullptr;
  if (have_draft && (check_cfg(dcfg) || check_weights(dcfg, dw) || dcfg->vocab != tcfg->vocab)) return STAIRS_EINVAL;
  if (k_max < 0 || k_max >= STAIRS_MAX_ROWS) return STAIRS_EINVAL;
  if (!have_draft && k_max != 0) return STAIRS_EINVAL;
  int rc = STAIRS_OK;
  stairs_ctx* c = new_ctx(hip_stream, k_max, have_draft, tcfg->dtype == STAIRS_DTYPE_BF16, &rc);
  if (!c) return rc;
  auto bail = [&](int code) {
    if (code == STAIRS_EHIP || code == STAIRS_ENOMEM) fprintf(stderr, "stairs_init: %s\n", c->err.c_str());
    stairs_free(c);
    return code;
  };
  if (configure_kernels() != hipSuccess) return bail(STAIRS_EHIP);
  size_t stage_bytes = max_matrix_bytes(tcfg);
  if (have_draft) stage_bytes = std::max(stage_bytes, max_matrix_bytes(dcfg));
  char* staging = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&staging), stage_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return bail(STAIRS_ENOMEM);
  }
  rc = build_model(c, &c->T, tcfg, tw, staging);
  if (!rc && have_draft) rc = build_model(c, &c->D, dcfg, dw, staging);
  (void)hipFree(staging);
  if (rc) return bail(rc);

  WsDims w{};
  w.dmax = w.amax = std::max(tcfg->d_model, have_draft ? dcfg->d_model : 0);
  w.fmax = std::max(tcfg->d_ffn, have_draft ? dcfg->d_ffn : 0);
  w.Hmax = std::max(tcfg->n_heads, have_draft ? dcfg->n_heads : 0);
  w.capmax = std::max(tcfg->max_seq, have_draft ? dcfg->max_seq : 0);
  w.vocab = tcfg->vocab;
  w.partial_floats = max_partial_floats(tcfg);
  if (have_draft) w.partial_floats = std::max(w.partial_floats, max_partial_floats(dcfg));
  if ((rc = alloc_workspaces(c, w))) return bail(rc);
  *out = c;
  return STAIRS_OK;
}

// workspaces, token array, state, counters, pinned host mirror, events
static int alloc_workspaces(stairs_ctx* c, const WsDims& w) {
  int rc;
  auto bail = [&](int code) { return code; };
  const int dmax = w.dmax, fmax = w.fmax, Hmax = w.Hmax, capmax = w.capmax;
  const int wide = std::max(w.dmax, w.amax);
  c->nchunk_cap = (std::max(capmax, w.srcmax) + kAttnChunk - 1) / kAttnChunk;
  c->tok_cap = capmax;
  c->tok_stride = capmax + kMaxRows;
  if (w.srcmax > 0 &&
      ((rc = dev_alloc(c, &c->src_tok, (size_t)w.srcmax + kMaxRows)) || (rc = dev_alloc(c, &c->enc_x, (size_t)w.srcmax * dmax)) ||
       (rc = dev_alloc(c, &c->enc_ssq, (size_t)w.srcmax * ssq_groups(dmax, 1))) ||
       (rc = dev_alloc(c, &c->enc_q, (size_t)w.srcmax * w.amax))))
    return rc;
  // (activations and their fragments for kMaxFwdRows rows: a few MB; what grows with the context or the vocabulary
  // is sized for rows_cap rows and enlarged by stairs_reserve_batch)
  if (frag_bytes(std::max(wide, fmax)) > kFragHalfU4 * 16) return fail(c, STAIRS_EINVAL, "d_model / d_ffn too large for the activation fragment blocks");
  if ((rc = dev_alloc(c, &c->x, (size_t)kMaxFwdRows * dmax)) || (rc = dev_alloc(c, &c->ssq, (size_t)kMaxFwdRows * ssq_groups(dmax, 1))) ||
      (rc = dev_alloc(c, &c->q_rot, (size_t)kMaxFwdRows * wide)) || (rc = dev_alloc(c, &c->attn_out, (size_t)kMaxFwdRows * wide)) ||
      (rc = dev_alloc(c, &c->h, (size_t)kMaxFwdRows * fmax)) || (rc = dev_alloc(c, &c->logits, (size_t)kMaxRows * w.vocab)) ||
      (rc = dev_alloc(c, &c->partial, w.partial_floats)) ||
      (rc = dev_alloc(c, &c->xf, frag_alloc_bytes(dmax) / sizeof(uint4))) || (rc = dev_alloc(c, &c->af, frag_alloc_bytes(wide) / sizeof(uint4))) ||
      (rc = dev_alloc(c, &c->hf, frag_alloc_bytes(fmax) / sizeof(uint4))) ||
      (rc = dev_alloc(c, &c->part_o, (size_t)kMaxRows * Hmax * c->nchunk_cap * 128)) ||
      (rc = dev_alloc(c, &c->part_ml, (size_t)kMaxRows * Hmax * c->nchunk_cap * 2)) ||
      (rc = dev_alloc(c, &c->rope_cs, (size_t)kMaxFwdRows * 64)) || (rc = dev_alloc(c, &c->tokens, (size_t)c->tok_cap + kMaxRows)) ||
      (rc = dev_alloc(c, &c->tgt_tok, (size_t)kMaxRows)) || (rc = dev_alloc(c, &c->counters, (size_t)kCounters)) || (rc = dev_alloc(c, &c->state, 2 * kSlotState)))
    return bail(rc);
  if (c->block_prefill) {
    // rows per block: what the longest sequence needs, at most kPfRows
    const int rows = std::min(kPfRows, (capmax + kBlkRows - 1) / kBlkRows * kBlkRows);
    c->pf_rows = rows;
    const size_t wide = std::max<size_t>(3 * (size_t)dmax, 2 * (size_t)fmax), inner = std::max<size_t>(dmax, fmax);
    if ((rc = dev_alloc(c, &c->pf_x, (size_t)rows * dmax)) || (rc = dev_alloc(c, &c->pf_y, (size_t)rows * wide)) ||
        (rc = dev_alloc(c, &c->pf_q, (size_t)rows * dmax)) || (rc = dev_alloc(c, &c->pf_attn, (size_t)rows * dmax)) ||
        (rc = dev_alloc(c, &c->pf_frag, pf_frag_bytes(rows, (int)inner) / sizeof(uint4))) ||
        (rc = dev_alloc(c, &c->pf_cs, (size_t)rows * 64)))
      return bail(rc);
    // blocks of few rows have too few (feature, row) tiles for the chip: their GEMMs cut k and need room for the pieces
    c->pf_part_floats = (size_t)16 << 20;
    if ((rc = dev_alloc(c, &c->pf_part, c->pf_part_floats))) return bail(rc);
    // rows of a block past its last one are read by the GEMM (and their results dropped): they must hold numbers
    if (hipMemsetAsync(c->pf_frag, 0, pf_frag_bytes(rows, (int)inner), c->st) != hipSuccess) return bail(STAIRS_EHIP);
  }
  // every slot of the token array always holds a valid id: a diagnostic forward may run at positions the current
  // sequence has not reached, and the embedding gather takes whatever id it finds there
  if (hipMemsetAsync(c->tokens, 0, ((size_t)c->tok_cap + kMaxRows) * sizeof(int), c->st) != hipSuccess) return bail(STAIRS_EHIP);
  if (hipMemsetAsync(c->state, 0, 2 * kSlotState * sizeof(int), c->st) != hipSuccess) return bail(STAIRS_EHIP);
  if (hipMemsetAsync(c->counters, 0, kCounters * sizeof(int), c->st) != hipSuccess) return bail(STAIRS_EHIP);
  c->h_pinned_ints = 2 * kSlotState + kMaxRows;     // single sequence: 2 + rows; a batch of one slot: state + rows
  if (hipHostMalloc(reinterpret_cast<void**>(&c->h_pinned), c->h_pinned_ints * sizeof(int), hipHostMallocDefault) != hipSuccess) {
    c->h_pinned = nullptr;
    return bail(STAIRS_ENOMEM);
  }
  for (auto& e : c->ev)
    if (hipEventCreate(&e) != hipSuccess) return bail(STAIRS_EHIP);
  if (hipStreamSynchronize(c->st) != hipSuccess) return bail(STAIRS_EHIP);
  return STAIRS_OK;
}

static size_t ed_matrix_bytes(const stairs_encdec_cfg* m) {
  const size_t d = m->d_model, a = (size_t)m->n_heads * m->head_dim, f = m->d_ffn, V = m->vocab;
  return std::max({3 * a * d, f * d, V * d}) * 2;
}
static size_t ed_partial_floats(const stairs_encdec_cfg* m) {
  const size_t d = m->d_model, a = (size_t)m->n_heads * m->head_dim, f = m->d_ffn, V = m->vocab;
  const size_t sd = gemm_slices(m->d_model, 1), sa = gemm_slices((int)a, 1), sf = gemm_slices(m->d_ffn, 1);
  return kMaxRows * std::max({sd * 3 * a, sd * f, sd * V, sa * d, sf * d});
}

int stairs_encdec_init(stairs_ctx** out, const stairs_encdec_cfg* tcfg, const stairs_encdec_weights* tw,
                       const stairs_encdec_cfg* dcfg, const stairs_encdec_weights* dw, int32_t k_max, int32_t start_token,
                       void* hip_stream) {
  if (!out) return STAIRS_EINVAL;
  *out = nullptr;
  if (check_encdec_cfg(tcfg) || check_encdec_weights(tcfg, tw)) return STAIRS_EINVAL;
  const bool have_draft = dcfg != nullptr;
  if (have_draft && (check_encdec_cfg(dcfg) || check_encdec_weights(dcfg, dw) || dcfg->vocab != tcfg->vocab)) return STAIRS_EINVAL;
  if (k_max < 0 || k_max >= STAIRS_MAX_ROWS || (!have_draft && k_max != 0)) return STAIRS_EINVAL;
  if (start_token < 0 || start_token >= tcfg->vocab) return STAIRS_EINVAL;
  int rc = STAIRS_OK;
  stairs_ctx* c = new_ctx(hip_stream, k_max, have_draft, false, &rc);
  if (!c) return rc;
  c->encdec = true;
  c->start_token = start_token;
  auto bail = [&](int code) {
    if (code == STAIRS_EHIP || code == STAIRS_ENOMEM) fprintf(stderr, "stairs_encdec_init: %s\n", c->err.c_str());
    stairs_free(c);
    return code;
  };
  if (configure_kernels() != hipSuccess) return bail(STAIRS_EHIP);
  size_t stage_bytes = ed_matrix_bytes(tcfg);
  if (have_draft) stage_bytes = std::max(stage_bytes, ed_matrix_bytes(dcfg));
  char* staging = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&staging), stage_bytes) != hipSuccess) {
    (void)hipGetLastError();
    return bail(STAIRS_ENOMEM);
  }
  rc = build_encdec_model(c, &c->T, tcfg, tw, staging);
  if (!rc && have_draft) rc = build_encdec_model(c, &c->D, dcfg, dw, staging);
  (void)hipFree(staging);
  if (rc) return bail(rc);
  WsDims w{};
  w.dmax = std::max(tcfg->d_model, have_draft ? dcfg->d_model : 0);
  w.amax = std::max(c->T.da, have_draft ? c->D.da : 0);
  w.fmax = std::max(tcfg->d_ffn, have_draft ? dcfg->d_ffn : 0);
  w.Hmax = std::max(tcfg->n_heads, have_draft ? dcfg->n_heads : 0);
  w.capmax = std::max(tcfg->max_seq, have_draft ? dcfg->max_seq : 0);
  w.srcmax = std::max(tcfg->max_src, have_draft ? dcfg->max_src : 0);
  w.vocab = tcfg->vocab;
  w.partial_floats = ed_partial_floats(tcfg);
  if (have_draft) w.partial_floats = std::max(w.partial_floats, ed_partial_floats(dcfg));
  if ((rc = alloc_workspaces(c, w))) return bail(rc);
  *out = c;
  return STAIRS_OK;
}

int32_t stairs_rel_bucket(int32_t rel, int32_t two_sided, int32_t buckets, int32_t max_distance) {
  if (buckets < 4 || buckets % 4 || max_distance <= buckets / 2) return -1;
  return bias_bucket(rel, two_sided != 0, buckets, max_distance);
}

int stairs_encode(stairs_ctx* c, const int32_t* src, int32_t S) {
  if (!c) return STAIRS_EINVAL;
  if (!c->encdec) return fail(c, STAIRS_EINVAL, "stairs_encode needs an encoder-decoder context");
  if (!src || S < 1) return fail(c, STAIRS_EINVAL, "source is NULL or empty");
  if (S > c->T.max_src || (c->have_draft && S > c->D.max_src)) return fail(c, STAIRS_ECAPACITY, "source exceeds max_src");
  for (int i = 0; i < S; ++i)
    if (src[i] < 0 || src[i] >= c->T.cfg.vocab) return fail(c, STAIRS_EINVAL, "source token outside the vocabulary");
  if (!capacity_ok(c, 1 + c->k_max + 1)) return fail(c, STAIRS_ECAPACITY, "1 + k_max + 1 exceeds max_seq");
  c->prefilled = false;
  c->pending_k = -1;
  // captured iterations hold the source length: they stay valid only for a source of the same length
  HIPCHK(c, hipStreamSynchronize(c->st));
  if (S != c->S) {
    for (auto& g : c->graphs) (void)hipGraphExecDestroy(g.exec);
    c->graphs.clear();
  }
  HIPCHK(c, hipMemsetAsync(c->counters, 0, kCounters * sizeof(int), c->st));
  HIPCHK(c, hipMemcpyAsync(c->src_tok, src, (size_t)S * sizeof(int), hipMemcpyHostToDevice, c->st));
  const int st4[kSlotState] = {1, 0, 0, 1};
  HIPCHK(c, hipMemcpyAsync(c->state, st4, sizeof(st4), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipMemcpyAsync(c->tokens, &c->start_token, sizeof(int), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));     // st4 is on the stack
  c->S = S;
  c->L = c->P = 1;
  c->T.valid = c->D.valid = 0;
  int rc = encode_model(c, &c->T);
  if (!rc && c->have_draft) rc = encode_model(c, &c->D);
  if (rc) return rc;
  HIPCHK(c, hipStreamSynchronize(c->st));
  c->prefilled = true;
  return STAIRS_OK;
}

int stairs_prefill(stairs_ctx* c, const int32_t* prompt, int32_t P) {
  if (!c) return STAIRS_EINVAL;
  if (c->encdec) return fail(c, STAIRS_EINVAL, "encoder-decoder context: stairs_encode starts a sequence");
  if (!prompt || P < 1) return fail(c, STAIRS_EINVAL, "prompt is NULL or empty");
  if (!capacity_ok(c, P + c->k_max + 1)) return fail(c, STAIRS_ECAPACITY, "prompt + k_max + 1 exceeds max_seq");
  for (int i = 0; i < P; ++i)
    if (prompt[i] < 0 || prompt[i] >= c->T.cfg.vocab) return fail(c, STAIRS_EINVAL, "prompt token outside the vocabulary");
  c->prefilled = false;
  c->pending_k = -1;
  HIPCHK(c, hipMemsetAsync(c->counters, 0, kCounters * sizeof(int), c->st));
  HIPCHK(c, hipMemcpyAsync(c->tokens, prompt, (size_t)P * sizeof(int), hipMemcpyHostToDevice, c->st));
  const int st3[kSlotState] = {P, 0, 0, 1};
  HIPCHK(c, hipMemcpyAsync(c->state, st3, sizeof(st3), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));     // st3 is on the stack
  c->L = c->P = P;
  c->T.valid = c->D.valid = 0;
  int rc = ingest(c, &c->T, 0, P - 1);
  if (!rc && c->have_draft) rc = ingest(c, &c->D, 0, P - 1);
  if (rc) return rc;
  HIPCHK(c, hipStreamSynchronize(c->st));
  c->prefilled = true;
  return STAIRS_OK;
}

int draft_propose(stairs_ctx* c, int32_t k, int32_t* draft_out) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "draft_propose before stairs_prefill");
  if (!c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  if (c->pending_k >= 0) return fail(c, STAIRS_ESTATE, "a proposal is already pending");
  if (k < 1 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [1, k_max]");
  if (!capacity_ok(c, c->L + k + 1)) return fail(c, STAIRS_ECAPACITY, "L + k + 1 exceeds max_seq");
  int rc = do_propose(c, k);
  if (rc) return rc;
  if (draft_out) return copy_out(c, draft_out, c->tokens + c->L, (size_t)k * sizeof(int));
  HIPCHK(c, hipStreamSynchronize(c->st));
  return STAIRS_OK;
}

static int verify_common(stairs_ctx* c, int k, int32_t* target_tok_out, int32_t* n_accepted_out, float* logits_out) {
  int n = 0;
  int rc = do_verify(c, k, &n);
  if (rc) return rc;
  if (target_tok_out) memcpy(target_tok_out, c->h_pinned + 2, (size_t)(k + 1) * sizeof(int));
  if (n_accepted_out) *n_accepted_out = n;
  if (logits_out) return copy_out(c, logits_out, c->logits, (size_t)(k + 1) * c->T.cfg.vocab * sizeof(float));
  return STAIRS_OK;
}

int stairs_verify(stairs_ctx* c, int32_t k, int32_t* target_tok_out, int32_t* n_accepted_out, float* logits_out) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "stairs_verify before stairs_prefill");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && c->pending_k != k) return fail(c, STAIRS_ESTATE, "no pending proposal of this k");
  if (k == 0 && c->pending_k > 0) return fail(c, STAIRS_ESTATE, "a proposal of another k is pending");
  if (!capacity_ok(c, c->L + k + 1)) return fail(c, STAIRS_ECAPACITY, "L + k + 1 exceeds max_seq");
  return verify_common(c, k, target_tok_out, n_accepted_out, logits_out);
}

int stairs_verify_tokens(stairs_ctx* c, const int32_t* draft, int32_t k, int32_t* target_tok_out, int32_t* n_accepted_out,
                         float* logits_out) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "stairs_verify_tokens before stairs_prefill");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && !draft) return fail(c, STAIRS_EINVAL, "draft is NULL");
  for (int i = 0; i < k; ++i)
    if (draft[i] < 0 || draft[i] >= c->T.cfg.vocab) return fail(c, STAIRS_EINVAL, "draft token outside the vocabulary");
  if (!capacity_ok(c, c->L + k + 1)) return fail(c, STAIRS_ECAPACITY, "L + k + 1 exceeds max_seq");
  if (c->pending_k >= 0 && c->have_draft) c->D.valid = std::min(c->D.valid, c->L - 1);   // drop the proposal's rows
  c->pending_k = -1;
  if (k > 0) {
    HIPCHK(c, hipMemcpyAsync(c->tokens + c->L, draft, (size_t)k * sizeof(int), hipMemcpyHostToDevice, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    if (c->have_draft) c->D.valid = std::min(c->D.valid, c->L);   // whatever it held beyond S is not these tokens
  }
  return verify_common(c, k, target_tok_out, n_accepted_out, logits_out);
}

// The loop of stairs_decode.  adaptive: k is the first draft length and the next one follows from what was accepted
// (everything: one more, up to k_max; otherwise one more than the accepted count).
static int decode_loop(stairs_ctx* c, int32_t G, int32_t k, bool adaptive, int32_t* tokens_out, stairs_stats* stats,
                       bool sampled = false) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "stairs_decode before stairs_prefill");
  if (c->pending_k >= 0) return fail(c, STAIRS_ESTATE, "a proposal is pending");
  if (G < 0 || (G > 0 && !tokens_out)) return fail(c, STAIRS_EINVAL, "G < 0 or tokens_out is NULL");
  if (k < 0 || k > c->k_max || (adaptive && k < 1)) return fail(c, STAIRS_EINVAL, adaptive ? "k outside [1, k_max]" : "k outside [0, k_max]");
  if (k > 0 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  const int k_cap = adaptive ? c->k_max : k;   // longest draft the loop can reach
  if (!capacity_ok(c, c->L + G + k_cap + 1)) return fail(c, STAIRS_ECAPACITY, "L + G + k + 1 exceeds max_seq");
  stairs_stats s;
  memset(&s, 0, sizeof(s));
  const int L0 = c->L;
  int L_end = -1;                  // length of the sequence up to and including the end token, once it was emitted
  int rc;
  HIPCHK(c, hipEventRecord(c->ev[1], c->st));
  while (c->L - L0 < G) {
    int n = 0;
    if (k > 0 && c->D.valid < c->L - 2 && (rc = ingest(c, &c->D, c->D.valid, c->L - 2))) return rc;
    HIPCHK(c, hipEventRecord(c->ev[5], c->st));
    if (c->use_graphs) {
      const int nch = std::min((chunks_for(c->L + k) + 3) / 4 * 4, c->nchunk_cap);   // never past the partial buffers
      hipGraphExec_t gp = nullptr, gv = nullptr;
      const int gB = sampled ? -1 : 0;
      if (k > 0 && (rc = iteration_graph(c, 0, k, nch, &gp, gB))) return rc;
      if ((rc = iteration_graph(c, 1, k, nch, &gv, gB))) return rc;
      if (k > 0) HIPCHK(c, hipGraphLaunch(gp, c->st));
      HIPCHK(c, hipEventRecord(c->ev[6], c->st));
      HIPCHK(c, hipGraphLaunch(gv, c->st));
    } else {
      if (k > 0 && (rc = sampled ? enqueue_propose_sampled(c, k, chunks_for(c->L + k - 1))
                                 : enqueue_propose(c, k, chunks_for(c->L + k - 1))))
        return rc;
      HIPCHK(c, hipEventRecord(c->ev[6], c->st));
      if ((rc = sampled ? enqueue_verify_sampled(c, k, chunks_for(c->L + k)) : enqueue_verify(c, k, chunks_for(c->L + k)))) return rc;
    }
    HIPCHK(c, hipEventRecord(c->ev[7], c->st));
    if (k > 0) c->D.valid = c->L + k - 1;
    if ((rc = finish_verify(c, k, &n))) return rc;
    float a = 0.f, b = 0.f;
    HIPCHK(c, hipEventElapsedTime(&a, c->ev[5], c->ev[6]));
    HIPCHK(c, hipEventElapsedTime(&b, c->ev[6], c->ev[7]));
    s.ms_draft += a;
    s.ms_verify += b;
    s.iterations += 1;
    s.accepted += n;
    s.accept_hist[n] += 1;
    if (adaptive) k = (n == k) ? std::min(k + 1, c->k_max) : std::max(1, n + 1);
    // the end token closes the answer: what the iteration emitted after it is dropped (finish_verify left the
    // n + 1 emitted tokens in the pinned buffer)
    if (c->eos_id >= 0) {
      int j = 0;
      while (j <= n && c->h_pinned[2 + j] != c->eos_id) ++j;
      if (j <= n) {
        L_end = c->L - (n + 1) + j + 1;
        break;
      }
    }
  }
  HIPCHK(c, hipEventRecord(c->ev[0], c->st));
  HIPCHK(c, hipEventSynchronize(c->ev[0]));
  HIPCHK(c, hipEventElapsedTime(&s.ms_decode, c->ev[1], c->ev[0]));
  // the last iteration may have produced more than asked for (or tokens after the end token): the sequence is cut
  // back (the caches hold a prefix of what they held, which stays valid)
  const int L_keep = std::min(L0 + G, L_end >= 0 ? L_end : c->L);
  s.tokens = L_keep - L0;
  if (c->L > L_keep) {
    c->L = L_keep;
    c->T.valid = std::min(c->T.valid, c->L - 1);
    if (c->have_draft) c->D.valid = std::min(c->D.valid, c->L - 1);
    HIPCHK(c, hipMemcpyAsync(c->state, &c->L, sizeof(int), hipMemcpyHostToDevice, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
  }
  if (s.tokens > 0 && (rc = copy_out(c, tokens_out, c->tokens + L0, (size_t)s.tokens * sizeof(int)))) return rc;
  for (int i = s.tokens; i < G; ++i) tokens_out[i] = c->eos_id;
  if (stats) *stats = s;
  return STAIRS_OK;
}

int stairs_set_eos(stairs_ctx* c, int32_t eos_id) {
  if (!c) return STAIRS_EINVAL;
  if (eos_id < -1 || eos_id >= c->T.cfg.vocab) return fail(c, STAIRS_EINVAL, "end token outside [-1, vocab)");
  c->eos_id = eos_id;
  return STAIRS_OK;
}

int stairs_decode(stairs_ctx* c, int32_t G, int32_t k, int32_t* tokens_out, stairs_stats* stats) {
  return decode_loop(c, G, k, false, tokens_out, stats);
}

int stairs_decode_adaptive(stairs_ctx* c, int32_t G, int32_t k_first, int32_t* tokens_out, stairs_stats* stats) {
  return decode_loop(c, G, k_first, true, tokens_out, stats);
}

int stairs_decode_sampled(stairs_ctx* c, int32_t G, int32_t k, float temperature, uint64_t seed, int32_t* tokens_out,
                          stairs_stats* stats) {
  if (!c) return STAIRS_EINVAL;
  int rc = set_sampling(c, temperature, seed);
  if (rc) return rc;
  return decode_loop(c, G, k, false, tokens_out, stats, true);
}

int draft_propose_sampled(stairs_ctx* c, int32_t k, float temperature, uint64_t seed, int32_t* draft_out, float* draft_logits_out) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "draft_propose_sampled before a sequence was started");
  if (!c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  if (c->pending_k >= 0) return fail(c, STAIRS_ESTATE, "a proposal is already pending");
  if (k < 1 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [1, k_max]");
  if (!capacity_ok(c, c->L + k + 1)) return fail(c, STAIRS_ECAPACITY, "L + k + 1 exceeds max_seq");
  int rc = set_sampling(c, temperature, seed);
  if (rc) return rc;
  if ((rc = do_propose(c, k, true))) return rc;
  if (draft_logits_out &&
      (rc = copy_out(c, draft_logits_out, c->dlogits, (size_t)k * c->T.cfg.vocab * sizeof(float))))
    return rc;
  if (draft_out) return copy_out(c, draft_out, c->tokens + c->L, (size_t)k * sizeof(int));
  HIPCHK(c, hipStreamSynchronize(c->st));
  return STAIRS_OK;
}

int stairs_verify_sampled(stairs_ctx* c, int32_t k, float temperature, uint64_t seed, int32_t* emitted_out,
                          int32_t* n_accepted_out, float* logits_out) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "stairs_verify_sampled before a sequence was started");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && (c->pending_k != k || !c->pending_sampled)) return fail(c, STAIRS_ESTATE, "no pending sampled proposal of this k");
  if (k == 0 && c->pending_k > 0) return fail(c, STAIRS_ESTATE, "a proposal of another k is pending");
  if (!capacity_ok(c, c->L + k + 1)) return fail(c, STAIRS_ECAPACITY, "L + k + 1 exceeds max_seq");
  int rc = set_sampling(c, temperature, seed);
  if (rc) return rc;
  int n = 0;
  if ((rc = do_verify(c, k, &n, true))) return rc;
  if (emitted_out) memcpy(emitted_out, c->h_pinned + 2, (size_t)(n + 1) * sizeof(int));
  if (n_accepted_out) *n_accepted_out = n;
  if (logits_out) return copy_out(c, logits_out, c->logits, (size_t)(k + 1) * c->T.cfg.vocab * sizeof(float));
  return STAIRS_OK;
}

int stairs_generate_sampled(stairs_ctx* c, const int32_t* prompt, int32_t P, int32_t G, int32_t k, float temperature,
                            uint64_t seed, int32_t* tokens_out, stairs_stats* stats) {
  if (!c) return STAIRS_EINVAL;
  if (G < 0 || (G > 0 && !tokens_out)) return fail(c, STAIRS_EINVAL, "G < 0 or tokens_out is NULL");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  if (!prompt || P < 1) return fail(c, STAIRS_EINVAL, "prompt is NULL or empty");
  if (!capacity_ok(c, P + G + k + 1)) return fail(c, STAIRS_ECAPACITY, "P + G + k + 1 exceeds max_seq");
  int rc = stairs_prefill(c, prompt, P);
  if (rc) return rc;
  return stairs_decode_sampled(c, G, k, temperature, seed, tokens_out, stats);
}

int stairs_generate(stairs_ctx* c, const int32_t* prompt, int32_t P, int32_t G, int32_t k, int32_t* tokens_out,
                    stairs_stats* stats) {
  if (!c) return STAIRS_EINVAL;
  if (G < 0 || (G > 0 && !tokens_out)) return fail(c, STAIRS_EINVAL, "G < 0 or tokens_out is NULL");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  if (!prompt || P < 1) return fail(c, STAIRS_EINVAL, "prompt is NULL or empty");
  if (!capacity_ok(c, P + G + k + 1)) return fail(c, STAIRS_ECAPACITY, "P + G + k + 1 exceeds max_seq");
  float ms_prefill = 0.f;
  HIPCHK(c, hipEventRecord(c->ev[0], c->st));
  int rc = stairs_prefill(c, prompt, P);
  if (rc) return rc;
  HIPCHK(c, hipEventRecord(c->ev[1], c->st));
  HIPCHK(c, hipEventSynchronize(c->ev[1]));
  HIPCHK(c, hipEventElapsedTime(&ms_prefill, c->ev[0], c->ev[1]));
  stairs_stats s;
  if ((rc = stairs_decode(c, G, k, tokens_out, &s))) return rc;
  s.ms_prefill = ms_prefill;
  if (stats) *stats = s;
  return STAIRS_OK;
}

int stairs_encdec_generate(stairs_ctx* c, const int32_t* src, int32_t S, int32_t G, int32_t k, int32_t* tokens_out,
                           stairs_stats* stats) {
  if (!c) return STAIRS_EINVAL;
  if (!c->encdec) return fail(c, STAIRS_EINVAL, "stairs_encdec_generate needs an encoder-decoder context");
  if (G < 0 || (G > 0 && !tokens_out)) return fail(c, STAIRS_EINVAL, "G < 0 or tokens_out is NULL");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  if (!capacity_ok(c, 1 + G + k + 1)) return fail(c, STAIRS_ECAPACITY, "1 + G + k + 1 exceeds max_seq");
  float ms_encode = 0.f;
  HIPCHK(c, hipEventRecord(c->ev[0], c->st));
  int rc = stairs_encode(c, src, S);
  if (rc) return rc;
  HIPCHK(c, hipEventRecord(c->ev[1], c->st));
  HIPCHK(c, hipEventSynchronize(c->ev[1]));
  HIPCHK(c, hipEventElapsedTime(&ms_encode, c->ev[0], c->ev[1]));
  stairs_stats s;
  if ((rc = stairs_decode(c, G, k, tokens_out, &s))) return rc;
  s.ms_prefill = ms_encode;
  if (stats) *stats = s;
  return STAIRS_OK;
}

int stairs_reserve_batch(stairs_ctx* c, int32_t max_batch) {
  if (!c) return STAIRS_EINVAL;
  if (c->encdec) return fail(c, STAIRS_EINVAL, "encoder-decoder contexts take one sequence");
  if (max_batch < 1 || max_batch > STAIRS_MAX_BATCH) return fail(c, STAIRS_EINVAL, "max_batch outside [1, STAIRS_MAX_BATCH]");
  if (max_batch > kMaxRows / 2 && !c->block_prefill)
    return fail(c, STAIRS_EINVAL, "more than STAIRS_MAX_ROWS / 2 sequences need the block kernels (bf16 models, STAIRS_NO_BLOCK_PREFILL unset)");
  if (!c->T.bf16 || (c->have_draft && !c->D.bf16)) return fail(c, STAIRS_EINVAL, "several sequences need bf16 models");
  if (max_batch * std::max(c->T.cfg.n_heads, c->have_draft ? c->D.cfg.n_heads : 0) > kAttnCounters)
    return fail(c, STAIRS_EINVAL, "max_batch * n_heads exceeds the attention hand-off counters");
  HIPCHK(c, hipStreamSynchronize(c->st));
  c->prefilled = false;
  c->pending_k = -1;
  if (max_batch <= c->n_slots) return STAIRS_OK;
  // captured graphs hold the old pointers: they go first, so that no failure below can leave one that replays
  // launches on released memory
  for (auto& g : c->graphs) (void)hipGraphExecDestroy(g.exec);
  c->graphs.clear();
  // new, larger arrays; the old ones are released
  auto release = [&](void* p) {
    auto it = std::find(c->owned.begin(), c->owned.end(), p);
    if (it != c->owned.end()) c->owned.erase(it);
    (void)hipFree(p);
  };
  int rc;
  for (Model* m : {&c->T, &c->D}) {
    if (m == &c->D && !c->have_draft) continue;
    const size_t bytes = (size_t)max_batch * m->cfg.n_layers * m->kv_layer_bytes;
    char *K = nullptr, *V = nullptr;
    if ((rc = dev_alloc(c, &K, bytes)) || (rc = dev_alloc(c, &V, bytes))) return rc;
    HIPCHK(c, hipMemsetAsync(K, 0, bytes, c->st));
    HIPCHK(c, hipMemsetAsync(V, 0, bytes, c->st));
    release(m->Kc);
    release(m->Vc);
    m->Kc = K;
    m->Vc = V;
    m->valid = 0;
  }
  // several sequences: the decode kernels take forwards of up to kMaxFwdRows rows (the hand-off-free GEMM holds the
  // chunk sums of all rows in LDS: k up to 16384), the block kernels up to kMaxBlockRows: logits, target tokens and
  // attention partial results for that many rows
  const int want_rows = max_batch > kMaxRows / 2 ? kMaxBlockRows : max_batch >= 2 ? kMaxFwdRows : kMaxRows;
  if (c->rows_cap < want_rows) {
    const int Hmax = std::max(c->T.cfg.n_heads, c->have_draft ? c->D.cfg.n_heads : 0);
    float *lg = nullptr, *po = nullptr, *pm = nullptr;
    int* tt = nullptr;
    if (want_rows == kMaxBlockRows && !c->pf_part) {
      c->pf_part_floats = (size_t)16 << 20;
      if ((rc = dev_alloc(c, &c->pf_part, c->pf_part_floats))) return rc;
    }
    if ((rc = dev_alloc(c, &lg, (size_t)want_rows * c->T.cfg.vocab)) ||
        (rc = dev_alloc(c, &po, (size_t)want_rows * Hmax * c->nchunk_cap * 128)) ||
        (rc = dev_alloc(c, &pm, (size_t)want_rows * Hmax * c->nchunk_cap * 2)) || (rc = dev_alloc(c, &tt, (size_t)want_rows)))
      return rc;
    release(c->logits);
    release(c->part_o);
    release(c->part_ml);
    release(c->tgt_tok);
    c->logits = lg;
    c->part_o = po;
    c->part_ml = pm;
    c->tgt_tok = tt;
    c->rows_cap = want_rows;
  }
  if (max_batch >= 2) {
    int kmax = std::max(c->T.cfg.d_model, c->T.cfg.d_ffn);
    if (c->have_draft) kmax = std::max({kmax, c->D.cfg.d_model, c->D.cfg.d_ffn});
    if (gemm_takes_rows(kMaxFwdRows, kmax)) c->fwd_rows = kMaxFwdRows;
  }
  int *tok = nullptr, *state = nullptr;
  if ((rc = dev_alloc(c, &tok, (size_t)max_batch * c->tok_stride)) || (rc = dev_alloc(c, &state, (size_t)(max_batch + 1) * kSlotState)))
    return rc;
  HIPCHK(c, hipMemsetAsync(tok, 0, (size_t)max_batch * c->tok_stride * sizeof(int), c->st));
  HIPCHK(c, hipMemsetAsync(state, 0, (size_t)(max_batch + 1) * kSlotState * sizeof(int), c->st));
  release(c->tokens);
  release(c->state);
  c->tokens = tok;
  c->state = state;
  int* hp = nullptr;
  const int ints = std::max(2 + kMaxRows, max_batch * kSlotState + c->rows_cap);
  if (hipHostMalloc(reinterpret_cast<void**>(&hp), ints * sizeof(int), hipHostMallocDefault) != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, STAIRS_ENOMEM, "hipHostMalloc failed");
  }
  (void)hipHostFree(c->h_pinned);
  c->h_pinned = hp;
  c->h_pinned_ints = ints;
  HIPCHK(c, hipStreamSynchronize(c->st));
  c->n_slots = max_batch;
  return STAIRS_OK;
}

int stairs_generate_batch(stairs_ctx* c, const int32_t* const* prompts, const int32_t* P, int32_t B, int32_t G, int32_t k,
                          int32_t* tokens_out, stairs_stats* stats) {
  if (!c) return STAIRS_EINVAL;
  if (c->encdec) return fail(c, STAIRS_EINVAL, "encoder-decoder contexts take one sequence");
  if (B < 1 || B > c->n_slots) return fail(c, STAIRS_EINVAL, "B outside [1, reserved batch]");
  if (G < 0 || (G > 0 && !tokens_out)) return fail(c, STAIRS_EINVAL, "G < 0 or tokens_out is NULL");
  if (k < 0 || k > c->k_max) return fail(c, STAIRS_EINVAL, "k outside [0, k_max]");
  if (k > 0 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  const int rows_max = std::max(B * (k + 1), B * 2);
  if (rows_max > c->rows_cap || (rows_max > c->fwd_rows && rows_max > c->pf_rows))
    return fail(c, STAIRS_EINVAL, "B * (k + 1) exceeds the rows one forward takes (STAIRS_MAX_STREAM_ROWS, or STAIRS_MAX_BATCH_ROWS after a reservation of more than STAIRS_MAX_ROWS / 2 sequences)");
  if (!c->T.bf16 || (c->have_draft && !c->D.bf16)) return fail(c, STAIRS_EINVAL, "several sequences need bf16 models");
  if (!prompts || !P) return fail(c, STAIRS_EINVAL, "prompts or P is NULL");
  for (int b = 0; b < B; ++b) {
    if (!prompts[b] || P[b] < 1) return fail(c, STAIRS_EINVAL, "a prompt is NULL or empty");
    // a slot that has its G tokens stops, so it never goes past P + G + k
    if (!capacity_ok(c, P[b] + G + k + 1)) return fail(c, STAIRS_ECAPACITY, "P + G + k + 1 exceeds max_seq");
    for (int i = 0; i < P[b]; ++i)
      if (prompts[b][i] < 0 || prompts[b][i] >= c->T.cfg.vocab) return fail(c, STAIRS_EINVAL, "prompt token outside the vocabulary");
  }
  stairs_stats s;
  memset(&s, 0, sizeof(s));
  c->prefilled = false;            // the single-sequence state (slot 0) is overwritten
  c->pending_k = -1;
  int rc;
  HIPCHK(c, hipMemsetAsync(c->counters, 0, kCounters * sizeof(int), c->st));
  HIPCHK(c, hipEventRecord(c->ev[0], c->st));
  std::vector<int> L(B), L0(B), hstate((size_t)B * kSlotState);
  std::vector<char> active(B, 1), ended(B, 0);
  for (int b = 0; b < B; ++b) {
    HIPCHK(c, hipMemcpyAsync(c->tokens + (size_t)b * c->tok_stride, prompts[b], (size_t)P[b] * sizeof(int), hipMemcpyHostToDevice, c->st));
    L[b] = L0[b] = P[b];
    hstate[b * kSlotState + 0] = P[b];
    hstate[b * kSlotState + 1] = 0;
    hstate[b * kSlotState + 2] = 0;
    hstate[b * kSlotState + 3] = G > 0 ? 1 : 0;
    active[b] = G > 0;
  }
  HIPCHK(c, hipMemcpyAsync(c->state, hstate.data(), hstate.size() * sizeof(int), hipMemcpyHostToDevice, c->st));
  HIPCHK(c, hipStreamSynchronize(c->st));
  // prompt ingestion, one sequence at a time (rows of one slot per forward)
  for (int b = 0; b < B; ++b)
    for (Model* m : {&c->T, &c->D}) {
      if (m == &c->D && !c->have_draft) continue;
      if ((rc = ingest(c, m, 0, P[b] - 1, b))) return rc;
    }
  c->T.valid = c->D.valid = 0;     // nothing the single-sequence calls could rely on
  HIPCHK(c, hipEventRecord(c->ev[1], c->st));
  int n_active = G > 0 ? B : 0;
  while (n_active > 0) {
    int Lmax = 0;
    for (int b = 0; b < B; ++b)
      if (active[b]) Lmax = std::max(Lmax, L[b]);
    HIPCHK(c, hipEventRecord(c->ev[5], c->st));
    if (c->use_graphs) {
      const int nch = std::min((chunks_for(Lmax + k) + 3) / 4 * 4, c->nchunk_cap);
      hipGraphExec_t gp = nullptr, gv = nullptr;
      if (k > 0 && (rc = iteration_graph(c, 0, k, nch, &gp, B))) return rc;
      if ((rc = iteration_graph(c, 1, k, nch, &gv, B))) return rc;
      if (k > 0) HIPCHK(c, hipGraphLaunch(gp, c->st));
      HIPCHK(c, hipEventRecord(c->ev[6], c->st));
      HIPCHK(c, hipGraphLaunch(gv, c->st));
    } else {
      if (k > 0 && (rc = enqueue_propose_batch(c, B, k, chunks_for(Lmax + k - 1)))) return rc;
      HIPCHK(c, hipEventRecord(c->ev[6], c->st));
      if ((rc = enqueue_verify_batch(c, B, k, chunks_for(Lmax + k)))) return rc;
    }
    HIPCHK(c, hipEventRecord(c->ev[7], c->st));
    HIPCHK(c, hipMemcpyAsync(c->h_pinned, c->state, (size_t)B * kSlotState * sizeof(int), hipMemcpyDeviceToHost, c->st));
    int* emitted = c->h_pinned + (size_t)B * kSlotState;       // [B][k + 1] target tokens (with an end token only)
    if (c->eos_id >= 0)
      HIPCHK(c, hipMemcpyAsync(emitted, c->tgt_tok, (size_t)B * (k + 1) * sizeof(int), hipMemcpyDeviceToHost, c->st));
    HIPCHK(c, hipStreamSynchronize(c->st));
    bool any_done = false;
    for (int b = 0; b < B; ++b) {
      if (!active[b]) continue;
      const int n = c->h_pinned[b * kSlotState + 1];
      if (c->h_pinned[b * kSlotState] != L[b] + n + 1 || n < 0 || n > k) return fail(c, STAIRS_EHIP, "device state out of sync with host");
      L[b] += n + 1;
      s.accepted += n;
      s.accept_hist[n] += 1;
      if (c->eos_id >= 0) {                             // the end token closes this sequence's answer
        int j = 0;
        while (j <= n && emitted[b * (k + 1) + j] != c->eos_id) ++j;
        if (j <= n) {
          L[b] += j - n;
          ended[b] = 1;
        }
      }
      if (ended[b] || L[b] - L0[b] >= G) {
        active[b] = 0;
        --n_active;
        any_done = true;
      }
    }
    if (any_done) {                                   // finished slots stop: their rows get no position any more
      for (int b = 0; b < B; ++b) {
        hstate[b * kSlotState + 0] = L[b];
        hstate[b * kSlotState + 3] = active[b];
      }
      // only the active flags change on the device (L is already there)
      for (int b = 0; b < B; ++b)
        if (!active[b])
          HIPCHK(c, hipMemcpyAsync(c->state + b * kSlotState + 3, &hstate[b * kSlotState + 3], sizeof(int), hipMemcpyHostToDevice, c->st));
      HIPCHK(c, hipStreamSynchronize(c->st));
    }
    float a = 0.f, bms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&a, c->ev[5], c->ev[6]));
    HIPCHK(c, hipEventElapsedTime(&bms, c->ev[6], c->ev[7]));
    s.ms_draft += a;
    s.ms_verify += bms;
    s.iterations += 1;
  }
  HIPCHK(c, hipEventRecord(c->ev[2], c->st));
  HIPCHK(c, hipEventSynchronize(c->ev[2]));
  HIPCHK(c, hipEventElapsedTime(&s.ms_prefill, c->ev[0], c->ev[1]));
  HIPCHK(c, hipEventElapsedTime(&s.ms_decode, c->ev[1], c->ev[2]));
  s.tokens = 0;
  for (int b = 0; b < B && G > 0; ++b) {
    const int got = std::min(G, L[b] - L0[b]);
    s.tokens += got;
    HIPCHK(c, hipMemcpyAsync(tokens_out + (size_t)b * G, c->tokens + (size_t)b * c->tok_stride + L0[b], (size_t)got * sizeof(int),
                             hipMemcpyDeviceToHost, c->st));
    for (int i = got; i < G; ++i) tokens_out[(size_t)b * G + i] = c->eos_id;
  }
  HIPCHK(c, hipStreamSynchronize(c->st));
  if (stats) *stats = s;
  return STAIRS_OK;
}

int stairs_get_tokens(stairs_ctx* c, int32_t* out, int32_t cap, int32_t* len) {
  if (!c) return STAIRS_EINVAL;
  if (!c->prefilled) return fail(c, STAIRS_ESTATE, "no sequence yet");
  if (len) *len = c->L;
  const int n = std::min(cap, c->L);
  if (n > 0 && !out) return fail(c, STAIRS_EINVAL, "out is NULL");
  if (n > 0) return copy_out(c, out, c->tokens, (size_t)n * sizeof(int));
  return STAIRS_OK;
}

int stairs_gemm_host(int32_t dtype, const void* W, const float* X, float* Y, int32_t M, int32_t N, int32_t K, void* hip_stream) {
  if (!W || !X || !Y || M < 1 || M > kMaxRows || N < 1 || K < 1) return STAIRS_EINVAL;
  const bool b = dtype == STAIRS_DTYPE_BF16;
  if (!b && dtype != STAIRS_DTYPE_FP32) return STAIRS_EINVAL;
  if (b ? (K % 256 || N % 16 || N / 64 + 1 > kGemmCounters) : (K % 4 || N % 4)) return STAIRS_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (configure_kernels() != hipSuccess) return STAIRS_EHIP;
  const size_t wbytes = (size_t)N * K * (b ? 2 : 4);
  const int S = gemm_slices(K, b);
  char *dW = nullptr, *dWs = nullptr;
  float *dX = nullptr, *dP = nullptr, *dY = nullptr;
  int* dCnt = nullptr;
  uint4* dF = nullptr;                       // activation fragments (bf16, more than 4 rows)
  const bool fr = b && M > 4;
  int rc = STAIRS_OK;
  auto ok = [&](hipError_t e) {
    if (e != hipSuccess && rc == STAIRS_OK) {
      fprintf(stderr, "stairs_gemm_host: %s\n", hipGetErrorString(e));
      rc = STAIRS_EHIP;
    }
    return e == hipSuccess;
  };
  if (ok(hipMalloc((void**)&dW, wbytes)) && ok(hipMalloc((void**)&dX, (size_t)M * K * 4)) &&
      ok(hipMalloc((void**)&dP, (size_t)S * M * N * 4)) && ok(hipMalloc((void**)&dY, (size_t)M * N * 4)) &&
      ok(hipMalloc((void**)&dCnt, kGemmCounters * sizeof(int))) && (!b || ok(hipMalloc((void**)&dWs, wbytes))) &&
      (!fr || ok(hipMalloc((void**)&dF, frag_bytes(K))))) {
    ok(hipMemcpyAsync(dW, W, wbytes, hipMemcpyHostToDevice, st));
    ok(hipMemcpyAsync(dX, X, (size_t)M * K * 4, hipMemcpyHostToDevice, st));
    if (b) launch_swizzle_bf16(reinterpret_cast<const uint16_t*>(dW), reinterpret_cast<uint4*>(dWs), N, K, kPermNone, 0, 0, st);
    ok(hipMemsetAsync(dCnt, 0, kGemmCounters * sizeof(int), st));
    RowNorm none{nullptr, nullptr, 0, 0.f};
    GemmEpi e{};
    e.counters = dCnt;
    e.stream_weights = wbytes > kStreamHintBytes / 4;   // exercised by the larger test matrices
    e.out = dY;
    e.hd = 64;
    if (fr) launch_split_frag(dX, K, M, K, nullptr, dF, st);
    launch_gemm(kRoleHead, b, b ? dWs : dW, N, K, dX, K, M, none, dP, e, st, dF);
    ok(hipGetLastError());
    ok(hipMemcpyAsync(Y, dY, (size_t)M * N * 4, hipMemcpyDeviceToHost, st));
    ok(hipStreamSynchronize(st));
  }
  (void)hipFree(dW); (void)hipFree(dWs); (void)hipFree(dX); (void)hipFree(dP); (void)hipFree(dY); (void)hipFree(dCnt);
  (void)hipFree(dF);
  return rc;
}

// ---- stairs_gemm_device: stairs_gemm_host for callers that cannot allocate ---------------------------------------
// Everything stairs_gemm_host allocates per call lives in one file-scope device array instead; every GPU the library
// runs on holds its own copy at its own address until the process ends.  Layout (bytes): hand-off counters, split-K /
// fp32 partial sums, the re-laid-out bf16 weights, the activation fragments.
constexpr size_t kNaCounterBytes = (size_t)kGemmCounters * sizeof(int);
constexpr size_t kNaPartialBytes = (size_t)STAIRS_GEMM_DEVICE_MAX_PARTIAL;
constexpr size_t kNaWeightBytes = (size_t)STAIRS_GEMM_DEVICE_MAX_WEIGHT;
constexpr size_t kNaFragBytes = ((size_t)(STAIRS_GEMM_DEVICE_MAX_K / 32) * 256 + (size_t)(STAIRS_GEMM_DEVICE_MAX_K / 512 + 1) * kFragChunkPad) * 16;
constexpr size_t kNaPartialOff = kNaCounterBytes;
constexpr size_t kNaWeightOff = kNaPartialOff + kNaPartialBytes;
constexpr size_t kNaFragOff = kNaWeightOff + kNaWeightBytes;
constexpr size_t kNaScratchBytes = kNaFragOff + kNaFragBytes;
static_assert(kNaPartialOff % 256 == 0 && kNaWeightOff % 256 == 0 && kNaFragOff % 256 == 0, "scratch regions stay 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[kNaScratchBytes];

// `scratch` is a host-side stand-in in host code, not a device address: the address on the current device is looked
// up once per device and kept; everything below passes that pointer.
constexpr int kNaMaxDevices = 64;
static unsigned char* g_scratch_ptr[kNaMaxDevices] = {};

static __global__ __launch_bounds__(256) void k_fill_zero(int* p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

int stairs_gemm_device(int32_t dtype, const void* W, const float* X, float* Y, int32_t M, int32_t N, int32_t K, void* hip_stream) {
  if (!W || !X || !Y || M < 1 || M > kMaxRows || N < 1 || K < 1) return STAIRS_EINVAL;
  const bool b = dtype == STAIRS_DTYPE_BF16;
  if (!b && dtype != STAIRS_DTYPE_FP32) return STAIRS_EINVAL;
  if (b ? (K % 256 || N % 16 || N / 64 + 1 > kGemmCounters) : (K % 4 || N % 4)) return STAIRS_EINVAL;
  // limits of the fixed scratch array
  const size_t S = gemm_slices(K, b);
  if (K > STAIRS_GEMM_DEVICE_MAX_K || S * M * N * sizeof(float) > kNaPartialBytes || (b && (size_t)N * K * 2 > kNaWeightBytes)) {
    fprintf(stderr, "stairs_gemm_device: shape M=%d N=%d K=%d exceeds the fixed scratch (K <= %d, slices*M*N*4 <= %zu, bf16 N*K*2 <= %zu)\n",
            M, N, K, STAIRS_GEMM_DEVICE_MAX_K, kNaPartialBytes, kNaWeightBytes);
    return STAIRS_ECAPACITY;
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kNaMaxDevices) return STAIRS_EHIP;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fprintf(stderr, "stairs_gemm_device: hipGetSymbolAddress: %s\n", hipGetErrorString(e));
      return STAIRS_EHIP;
    }
    if (configure_kernels() != hipSuccess) return STAIRS_EHIP;      // (function attributes: no allocation)
    g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
  }
  unsigned char* base = g_scratch_ptr[dev];
  int* cnt = reinterpret_cast<int*>(base);
  float* partial = reinterpret_cast<float*>(base + kNaPartialOff);
  uint4* wsw = reinterpret_cast<uint4*>(base + kNaWeightOff);
  uint4* frag = reinterpret_cast<uint4*>(base + kNaFragOff);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // the array keeps the last call's contents: the counters must start at zero (a fill kernel, not a memset node, so
  // that a caller may capture the call)
  hipLaunchKernelGGL(k_fill_zero, dim3((kGemmCounters + 255) / 256), dim3(256), 0, st, cnt, kGemmCounters);
  if (b) launch_swizzle_bf16(static_cast<const uint16_t*>(W), wsw, N, K, kPermNone, 0, 0, st);
  const bool fr = b && M > 4;
  if (fr) launch_split_frag(X, K, M, K, nullptr, frag, st);
  RowNorm none{nullptr, nullptr, 0, 0.f};
  GemmEpi e{};
  e.counters = cnt;
  e.stream_weights = (size_t)N * K * (b ? 2 : 4) > kStreamHintBytes / 4;
  e.out = Y;
  e.hd = 64;
  launch_gemm(kRoleHead, b, b ? static_cast<const void*>(wsw) : W, N, K, X, K, M, none, partial, e, st, fr ? frag : nullptr);
  if (hipGetLastError() != hipSuccess) return STAIRS_EHIP;
  return STAIRS_OK;
}

int stairs_copy_probe(int64_t bytes, int32_t reps, float* ms_per_launch, void* hip_stream) {
  if (bytes < 16 || bytes % 16 || reps < 1) return STAIRS_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  char *src = nullptr, *dst = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  int rc = STAIRS_OK;
  if (hipMalloc((void**)&src, bytes) != hipSuccess || hipMalloc((void**)&dst, bytes) != hipSuccess) {
    (void)hipGetLastError();
    rc = STAIRS_ENOMEM;
  } else if (hipMemsetAsync(src, 1, bytes, st) != hipSuccess || hipEventCreate(&e0) != hipSuccess ||
             hipEventCreate(&e1) != hipSuccess) {
    rc = STAIRS_EHIP;
  } else {
    launch_copy_probe(src, dst, bytes, st);   // warm-up
    (void)hipEventRecord(e0, st);
    for (int r = 0; r < reps; ++r) launch_copy_probe(src, dst, bytes, st);
    (void)hipEventRecord(e1, st);
    float ms = 0.f;
    if (hipGetLastError() != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
        hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
      rc = STAIRS_EHIP;
    else if (ms_per_launch)
      *ms_per_launch = ms / reps;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(src);
  (void)hipFree(dst);
  return rc;
}

int stairs_time_kernel(stairs_ctx* c, int32_t which, int32_t M, int32_t ctx_len, int32_t reps, float* ms_per_launch,
                       double* bytes_per_launch) {
  if (!c) return STAIRS_EINVAL;
  if (which < 0 || which > 10 || M < 1 || M > kMaxRows || reps < 1 || !ms_per_launch)
    return fail(c, STAIRS_EINVAL, "bad argument to stairs_time_kernel");
  if (c->encdec) return fail(c, STAIRS_EINVAL, "stairs_time_kernel takes decoder-only contexts");
  if (c->pending_k >= 0) return fail(c, STAIRS_ESTATE, "a proposal is pending");
  if (which == 7 && !c->have_draft) return fail(c, STAIRS_ESTATE, "context has no draft model");
  Model* m = which == 7 ? &c->D : &c->T;
  const stairs_model_cfg& g = m->cfg;
  const int d = g.d_model, f = g.d_ffn, V = g.vocab, b = m->bf16 ? 1 : 0;
  const size_t esz = m->esz();
  if (which >= 5 && (ctx_len < M || ctx_len > m->cap)) return fail(c, STAIRS_EINVAL, "ctx_len outside [M, max_seq]");
  if (which == 1 && (ctx_len < M || ctx_len > m->cap)) return fail(c, STAIRS_EINVAL, "ctx_len outside [M, max_seq]");
  // the QKV projection appends keys and values, the whole forwards do too: the caches no longer hold the current
  // sequence afterwards, so it ends here (the generation calls then ask for stairs_prefill instead of using them)
  if (which == 1 || which >= 6) {
    c->prefilled = false;
    c->T.valid = c->D.valid = 0;
  }
  if (which == 8 || which == 9 || which == 10) {
    // the gate/up projection timed where it really runs: `reps` whole forwards of M rows ending at position
    // ctx_len-1, an event pair around each layer's gate/up launch, all other kernels untouched in between
    const int nl = g.n_layers;
    while ((int)c->probe_ev.size() < 2 * nl) {
      hipEvent_t e = nullptr;
      HIPCHK(c, hipEventCreate(&e));
      c->probe_ev.push_back(e);
    }
    double total_ms = 0;
    for (int r = 0; r <= reps; ++r) {              // r == 0: warm-up
      // 9: what an event pair reads with no kernel inside; 10: the launch's own start / end events
      c->probe_role = which == 8 ? kRoleGateUp : which == 9 ? kProbeEmptyPair : kProbeKernelEvents;
      int rc = forward(c, m, abs_pos(c, ctx_len - M), chunks_for(ctx_len), M, M);
      c->probe_role = -1;
      if (rc) return rc;
      HIPCHK(c, hipStreamSynchronize(c->st));
      for (int l = 0; l < nl && r > 0; ++l) {
        float ms1 = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms1, c->probe_ev[2 * l], c->probe_ev[2 * l + 1]));
        total_ms += ms1;
      }
    }
    *ms_per_launch = (float)(total_ms / ((double)reps * nl));
    if (bytes_per_launch) *bytes_per_launch = 2.0 * f * d * esz;
    return STAIRS_OK;
  }
  RowNorm none{nullptr, nullptr, 0, 0.f};
  double bytes = 0;
  const PosRef tpos = abs_pos(c, which == 1 ? ctx_len - M : 0);
  if (which == 1) launch_rope_table(tpos, M, m->hd, g.rope_theta, c->rope_cs, c->st);
  // more than 4 rows: the projections read activation fragments, as inside a forward (whatever the workspaces hold)
  const bool fr = b && M > 4 && which <= 4;
  if (fr) {
    launch_split_frag(c->x, d, M, d, nullptr, c->xf, c->st);
    launch_split_frag(c->attn_out, d, M, d, nullptr, c->af, c->st);
    launch_split_frag(c->h, f, M, f, nullptr, c->hf, c->st);
  }
  const uint4 *xf = fr ? c->xf : nullptr, *af = fr ? c->af : nullptr, *hf = fr ? c->hf : nullptr;
  for (int pass = 0; pass < 2; ++pass) {          // pass 0 = warm-up of one launch per layer
    const int n = pass ? reps : (which >= 6 ? 1 : g.n_layers);
    if (pass) HIPCHK(c, hipEventRecord(c->ev[0], c->st));
    for (int r = 0; r < n; ++r) {
      const int l = r % g.n_layers;
      const Layer& ly = m->layers[l];
      char* Kl = m->Kc + l * m->kv_layer_bytes;
      char* Vl = m->Vc + l * m->kv_layer_bytes;
      GemmEpi e{};
      e.counters = c->counters;
      e.stream_weights = m->stream_weights;
      e.rope_cs = c->rope_cs;
      e.pos = tpos;
      e.Kc = reinterpret_cast<_Float16*>(Kl);
      e.Vc = reinterpret_cast<_Float16*>(Vl);
      e.Kc32 = reinterpret_cast<float*>(Kl);
      e.Vc32 = reinterpret_cast<float*>(Vl);
      e.cap = m->cap;
      e.H = g.n_heads;
      e.hd = m->hd;
      e.ssq_out = c->ssq;
      switch (which) {
        case 0: e.out = c->h; launch_gemm(kRoleGateUp, b, ly.wgu, 2 * f, d, c->x, d, M, none, c->partial, e, c->st, xf); bytes = 2.0 * f * d * esz; break;
        case 1: e.out = c->q_rot; launch_gemm(kRoleQKV, b, ly.wqkv, 3 * d, d, c->x, d, M, none, c->partial, e, c->st, xf); bytes = 3.0 * d * d * esz; break;
        case 2: e.out = c->x; launch_gemm(kRoleWo, b, ly.wo, d, d, c->attn_out, d, M, none, c->partial, e, c->st, af); bytes = 1.0 * d * d * esz; break;
        case 3: e.out = c->x; launch_gemm(kRoleDown, b, ly.wdown, d, f, c->h, f, M, none, c->partial, e, c->st, hf); bytes = 1.0 * d * f * esz; break;
        case 4: e.out = c->logits; launch_gemm(kRoleHead, b, m->lm_head, V, d, c->x, d, M, none, c->partial, e, c->st, xf); bytes = 1.0 * V * d * esz; break;
        case 6:
        case 7: {
          // a whole forward of M rows ending at position ctx_len-1 (all rows' logits for the
          // target, last row's for the draft); it overwrites those rows of the cache
          int rc = forward(c, m, abs_pos(c, ctx_len - M), chunks_for(ctx_len), M, which == 6 ? M : 1);
          if (rc) return rc;
          const double np_ = (double)g.n_layers * (4.0 * d * d + 3.0 * d * f) + (double)V * d;
          bytes = np_ * esz + 2.0 * g.n_layers * (double)ctx_len * d * esz;
          break;
        }
        default: {
          const size_t off = (size_t)(r % g.n_layers) * m->kv_layer_bytes;
          launch_attention(c->q_rot, m->Kc + off, m->Vc + off, b, m->cap, d, g.n_heads, M, abs_pos(c, ctx_len - M), 1, 0,
                           (ctx_len + kAttnChunk - 1) / kAttnChunk, c->nchunk_cap, c->part_o, c->part_ml,
                           c->counters + kGemmCounters, c->attn_out, c->st);
          bytes = 2.0 * ctx_len * d * esz;
        }
      }
      if (c->sync_launches) HIPCHK(c, hipStreamSynchronize(c->st));
    }
    if (pass) HIPCHK(c, hipEventRecord(c->ev[1], c->st));
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->st));
  }
  float ms = 0.f;
  HIPCHK(c, hipEventElapsedTime(&ms, c->ev[0], c->ev[1]));
  *ms_per_launch = ms / reps;
  if (bytes_per_launch) *bytes_per_launch = bytes;
  return STAIRS_OK;
}

}  // extern "C"
