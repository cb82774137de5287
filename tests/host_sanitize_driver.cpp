// Host-sanitizer driver for the C ABI of include/stairs.h.
//
// Built together with the library's two sources as ONE executable whose host code is instrumented with
// AddressSanitizer and UndefinedBehaviorSanitizer (device code is not instrumented; build line in
// tests/test_host_sanitizers.py).  Part 1 needs no GPU: the argument checks and host-only routines of every entry
// point.  Part 2 runs when a GPU is visible: a tiny random bf16 model pair through every kind of call (prefill in
// blocks and in rows, stairs generation, adaptive length, sampling, end token, batches on the decode and on the
// block kernels, encoder-decoder, the diagnostics) and their error paths on a live context, so that the host side
// of all of them (weight re-layout, workspace sizing, cache bookkeeping, graph bookkeeping, copies to the caller's
// buffers) runs under the sanitizers.  Results are also checked where the method fixes them (stairs == plain
// greedy, same seed same run).  Exit status 0 = no check failed; a sanitizer report aborts the process.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/stairs.h"

static int g_failed = 0;
#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "CHECK failed, line %d: %s\n", __LINE__, #cond);  \
      ++g_failed;                                                            \
    }                                                                        \
  } while (0)

struct Rng {
  uint64_t s;
  uint32_t next() {
    s = s * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(s >> 33);
  }
  float uniform() { return (float)(next() & 0xFFFFFF) / 16777216.0f - 0.5f; }
};

static uint16_t to_bf16(float v) {
  uint32_t u;
  std::memcpy(&u, &v, 4);
  u += 0x7FFF + ((u >> 16) & 1);
  return (uint16_t)(u >> 16);
}

static std::vector<uint16_t> matrix(Rng& r, size_t n, float scale) {
  std::vector<uint16_t> m(n);
  for (auto& x : m) x = to_bf16(r.uniform() * scale);
  return m;
}

// ---- a decoder-only model in host memory; the draft shares the target's first layers ----------------------------
struct HostModel {
  stairs_model_cfg cfg{};
  std::vector<uint16_t> tok_emb, lm_head;
  std::vector<float> final_norm;
  std::vector<std::vector<uint16_t>> wq, wk, wv, wo, wg, wu, wd;
  std::vector<std::vector<float>> an, fn;
  std::vector<const void*> pq, pk, pv, po, pg, pu, pd;
  std::vector<const float*> pan, pfn;
  stairs_weights w{};
  void build(Rng& r, int L, int d, int H, int f, int V, int max_seq) {
    cfg = {L, d, H, f, V, max_seq, 10000.f, 1e-5f, STAIRS_DTYPE_BF16};
    tok_emb = matrix(r, (size_t)V * d, 0.08f);
    lm_head = matrix(r, (size_t)V * d, 0.08f);
    final_norm.assign(d, 1.f);
    for (int l = 0; l < L; ++l) {
      const float deep = l == 0 ? 1.f : 0.3f;
      wq.push_back(matrix(r, (size_t)d * d, 0.08f));
      wk.push_back(matrix(r, (size_t)d * d, 0.08f));
      wv.push_back(matrix(r, (size_t)d * d, 0.08f));
      wo.push_back(matrix(r, (size_t)d * d, 0.08f * deep));
      wg.push_back(matrix(r, (size_t)f * d, 0.08f));
      wu.push_back(matrix(r, (size_t)f * d, 0.08f));
      wd.push_back(matrix(r, (size_t)d * f, 0.08f * deep));
      an.emplace_back(d, 1.f);
      fn.emplace_back(d, 1.f);
    }
    point(L);
  }
  void point(int L) {
    pq.clear(); pk.clear(); pv.clear(); po.clear(); pg.clear(); pu.clear(); pd.clear(); pan.clear(); pfn.clear();
    for (int l = 0; l < L; ++l) {
      pq.push_back(wq[l].data()); pk.push_back(wk[l].data()); pv.push_back(wv[l].data()); po.push_back(wo[l].data());
      pg.push_back(wg[l].data()); pu.push_back(wu[l].data()); pd.push_back(wd[l].data());
      pan.push_back(an[l].data()); pfn.push_back(fn[l].data());
    }
    w.tok_emb = tok_emb.data();
    w.lm_head = lm_head.data();
    w.final_norm = final_norm.data();
    w.attn_norm = pan.data();
    w.wq = pq.data(); w.wk = pk.data(); w.wv = pv.data(); w.wo = po.data();
    w.ffn_norm = pfn.data();
    w.w_gate = pg.data(); w.w_up = pu.data(); w.w_down = pd.data();
  }
};

// ---- part 1: no GPU -------------------------------------------------------------------------------------------------
static void part1_without_gpu() {
  for (int code = 1; code >= -8; --code) CHECK(stairs_strerror(code) != nullptr && std::strlen(stairs_strerror(code)) > 0);
  CHECK(stairs_last_error(nullptr) != nullptr);
  // the bucket rule: table shapes the library rejects, range and monotonicity of what it accepts
  CHECK(stairs_rel_bucket(0, 1, 30, 128) == -1);
  CHECK(stairs_rel_bucket(0, 1, 32, 16) == -1);
  for (int two = 0; two < 2; ++two) {
    int prev = -1;
    for (int rel = 0; rel >= -5000; --rel) {               // keys before the query, farther and farther
      const int b = stairs_rel_bucket(rel, two, 32, 128);
      CHECK(b >= 0 && b < 32 && b >= prev);
      prev = b;
    }
    for (int rel = 1; rel < 5000; rel += 7) {
      const int b = stairs_rel_bucket(rel, two, 32, 128);
      CHECK(two ? (b >= 16 && b < 32) : b == 0);
    }
  }
  // every entry point refuses a NULL context without touching anything
  int32_t buf[8] = {0};
  stairs_stats st;
  int32_t n = 0;
  CHECK(stairs_prefill(nullptr, buf, 4) == STAIRS_EINVAL);
  CHECK(draft_propose(nullptr, 1, buf) == STAIRS_EINVAL);
  CHECK(stairs_verify(nullptr, 1, buf, &n, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_verify_tokens(nullptr, buf, 1, buf, &n, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_generate(nullptr, buf, 4, 4, 0, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_decode(nullptr, 4, 0, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_decode_adaptive(nullptr, 4, 1, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_set_eos(nullptr, 1) == STAIRS_EINVAL);
  CHECK(stairs_reserve_batch(nullptr, 2) == STAIRS_EINVAL);
  const int32_t* pp[1] = {buf};
  int32_t P1[1] = {4};
  CHECK(stairs_generate_batch(nullptr, pp, P1, 1, 4, 0, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_decode_sampled(nullptr, 4, 0, 1.f, 1, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_generate_sampled(nullptr, buf, 4, 4, 0, 1.f, 1, buf, &st) == STAIRS_EINVAL);
  CHECK(draft_propose_sampled(nullptr, 1, 1.f, 1, buf, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_verify_sampled(nullptr, 1, 1.f, 1, buf, &n, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_encode(nullptr, buf, 4) == STAIRS_EINVAL);
  CHECK(stairs_encdec_generate(nullptr, buf, 4, 4, 0, buf, &st) == STAIRS_EINVAL);
  CHECK(stairs_get_tokens(nullptr, buf, 8, &n) == STAIRS_EINVAL);
  stairs_free(nullptr);
  // stairs_init: NULLs and shapes are rejected before any device work
  stairs_ctx* ctx = reinterpret_cast<stairs_ctx*>(buf);
  CHECK(stairs_init(&ctx, nullptr, nullptr, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  Rng r{5};
  HostModel m;
  m.build(r, 1, 256, 4, 512, 512, 64);
  stairs_model_cfg bad = m.cfg;
  bad.d_model = 250;
  CHECK(stairs_init(&ctx, &bad, &m.w, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  bad = m.cfg;
  bad.n_heads = 3;
  CHECK(stairs_init(&ctx, &bad, &m.w, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  bad = m.cfg;
  bad.vocab = 500;
  CHECK(stairs_init(&ctx, &bad, &m.w, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  bad = m.cfg;
  bad.dtype = 7;
  CHECK(stairs_init(&ctx, &bad, &m.w, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  CHECK(stairs_init(&ctx, &m.cfg, &m.w, nullptr, nullptr, STAIRS_MAX_ROWS, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  CHECK(stairs_init(&ctx, &m.cfg, &m.w, nullptr, nullptr, -1, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  stairs_weights wn = m.w;
  wn.lm_head = nullptr;
  CHECK(stairs_init(&ctx, &m.cfg, &wn, nullptr, nullptr, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  CHECK(stairs_encdec_init(&ctx, nullptr, nullptr, nullptr, nullptr, 0, 0, nullptr) == STAIRS_EINVAL && ctx == nullptr);
  // the diagnostics check their shapes on the host
  float x[4] = {0}, y[4] = {0};
  CHECK(stairs_gemm_host(STAIRS_DTYPE_BF16, nullptr, x, y, 1, 16, 256, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_gemm_host(STAIRS_DTYPE_BF16, buf, x, y, 1, 16, 100, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_gemm_host(STAIRS_DTYPE_BF16, buf, x, y, 0, 16, 256, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_gemm_host(9, buf, x, y, 1, 16, 256, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_gemm_device(STAIRS_DTYPE_BF16, nullptr, x, y, 1, 16, 256, nullptr) == STAIRS_EINVAL);
  CHECK(stairs_gemm_device(STAIRS_DTYPE_BF16, buf, x, y, 1, 16, 100, nullptr) == STAIRS_EINVAL);
}

// ---- part 2: with a GPU ---------------------------------------------------------------------------------------------
static std::vector<int32_t> prompt_of(Rng& r, int P, int V) {
  std::vector<int32_t> p(P);
  for (auto& t : p) t = (int32_t)(r.next() % (uint32_t)V);
  return p;
}

static void part2_decoder_only() {
  Rng r{11};
  const int V = 512, d = 256, H = 4, f = 512, cap = 400;
  HostModel T;
  T.build(r, 3, d, H, f, V, cap);
  HostModel D = T;                      // same tensors, first layer only (the library keeps shared tensors once)
  D.cfg.n_layers = 1;
  D.point(1);
  D.w = T.w;                            // same host addresses as the target's
  stairs_ctx* c = nullptr;
  CHECK(stairs_init(&c, &T.cfg, &T.w, &D.cfg, &T.w, 8, nullptr) == STAIRS_OK && c != nullptr);
  if (!c) return;
  const int G = 40;
  stairs_stats st;
  {
    int32_t tmp[8];
    CHECK(stairs_decode(c, 4, 2, tmp, &st) == STAIRS_ESTATE);               // no sequence yet
    CHECK(draft_propose(c, 2, tmp) == STAIRS_ESTATE);
  }
  for (int P : {1, 2, 70, 200}) {        // rows-only prefill, and prompts that take the block prefill
    std::vector<int32_t> p = prompt_of(r, P, V);
    std::vector<int32_t> base(G), got(G);
    CHECK(stairs_generate(c, p.data(), P, G, 0, base.data(), &st) == STAIRS_OK);
    CHECK(st.tokens == G && st.iterations == G);
    for (int k : {1, 3, 8}) {
      CHECK(stairs_generate(c, p.data(), P, G, k, got.data(), &st) == STAIRS_OK);
      CHECK(got == base);
      CHECK(st.tokens == G && st.iterations <= G && st.accepted + st.iterations >= G);
    }
    CHECK(stairs_prefill(c, p.data(), P) == STAIRS_OK);
    CHECK(stairs_decode_adaptive(c, G, 2, got.data(), &st) == STAIRS_OK);
    CHECK(got == base);
    // step by step, with the tokens and logits copied out
    CHECK(stairs_prefill(c, p.data(), P) == STAIRS_OK);
    std::vector<int32_t> dr(3), tg(4);
    std::vector<float> logits((size_t)4 * V);
    int32_t n = -1;
    CHECK(stairs_verify(c, 3, tg.data(), &n, nullptr) == STAIRS_ESTATE);
    CHECK(draft_propose(c, 3, dr.data()) == STAIRS_OK);
    CHECK(draft_propose(c, 3, dr.data()) == STAIRS_ESTATE);
    CHECK(stairs_verify(c, 3, tg.data(), &n, logits.data()) == STAIRS_OK);
    CHECK(n >= 0 && n <= 3 && tg[0] == base[0]);
    CHECK(stairs_verify_tokens(c, base.data() + n + 1, 2, tg.data(), &n, logits.data()) == STAIRS_OK);
    CHECK(n == 2);
    std::vector<int32_t> seq(P + 16);
    int32_t len = 0;
    CHECK(stairs_get_tokens(c, seq.data(), (int32_t)seq.size(), &len) == STAIRS_OK && len > P);
    // end token
    CHECK(stairs_set_eos(c, base[9]) == STAIRS_OK);
    CHECK(stairs_generate(c, p.data(), P, G, 3, got.data(), &st) == STAIRS_OK);
    CHECK(st.tokens >= 1 && st.tokens <= 10 && got[st.tokens - 1] == base[9]);
    for (int i = 0; i < st.tokens; ++i) CHECK(got[i] == base[i]);
    for (int i = st.tokens; i < G; ++i) CHECK(got[i] == base[9]);
    CHECK(stairs_set_eos(c, V) == STAIRS_EINVAL);
    CHECK(stairs_set_eos(c, -1) == STAIRS_OK);
    // sampling: same seed, same run
    std::vector<int32_t> s1(G), s2(G);
    CHECK(stairs_generate_sampled(c, p.data(), P, G, 3, 0.7f, 99, s1.data(), &st) == STAIRS_OK);
    CHECK(stairs_generate_sampled(c, p.data(), P, G, 3, 0.7f, 99, s2.data(), &st) == STAIRS_OK);
    CHECK(s1 == s2);
    CHECK(stairs_generate_sampled(c, p.data(), P, G, 3, 0.f, 99, s2.data(), &st) == STAIRS_EINVAL);
  }
  // error paths on a live context
  std::vector<int32_t> p = prompt_of(r, cap, V), out(64);
  CHECK(stairs_prefill(c, p.data(), cap) == STAIRS_ECAPACITY);
  p[7] = V;
  CHECK(stairs_prefill(c, p.data(), 30) == STAIRS_EINVAL);
  p[7] = 3;
  CHECK(stairs_prefill(c, p.data(), 30) == STAIRS_OK);
  CHECK(stairs_decode(c, -1, 2, out.data(), &st) == STAIRS_EINVAL);
  CHECK(stairs_decode(c, 8, 9, out.data(), &st) == STAIRS_EINVAL);
  CHECK(stairs_decode(c, cap, 2, out.data(), &st) == STAIRS_ECAPACITY);
  CHECK(stairs_decode(c, 0, 2, nullptr, &st) == STAIRS_OK);
  CHECK(std::strlen(stairs_last_error(c)) > 0);
  // several sequences: on the decode kernels, then (more than 16 reserved) on the block kernels
  std::vector<std::vector<int32_t>> ps;
  for (int P : {40, 1, 129, 70, 64, 3}) ps.push_back(prompt_of(r, P, V));
  std::vector<const int32_t*> pp;
  std::vector<int32_t> PP;
  for (auto& q : ps) {
    pp.push_back(q.data());
    PP.push_back((int32_t)q.size());
  }
  std::vector<int32_t> alone((size_t)ps.size() * G), both((size_t)ps.size() * G);
  for (size_t b = 0; b < ps.size(); ++b) CHECK(stairs_generate(c, pp[b], PP[b], G, 3, alone.data() + b * G, &st) == STAIRS_OK);
  CHECK(stairs_generate_batch(c, pp.data(), PP.data(), 2, G, 3, both.data(), &st) == STAIRS_EINVAL);   // nothing reserved
  CHECK(stairs_reserve_batch(c, 6) == STAIRS_OK);
  CHECK(stairs_generate_batch(c, pp.data(), PP.data(), 6, G, 3, both.data(), &st) == STAIRS_OK);
  CHECK(both == alone && st.tokens == 6 * G);
  CHECK(stairs_generate_batch(c, pp.data(), PP.data(), 7, G, 3, both.data(), &st) == STAIRS_EINVAL);
  CHECK(stairs_reserve_batch(c, STAIRS_MAX_BATCH + 1) == STAIRS_EINVAL);
  CHECK(stairs_reserve_batch(c, 24) == STAIRS_OK);
  std::vector<const int32_t*> pp24;
  std::vector<int32_t> PP24;
  for (int b = 0; b < 24; ++b) {
    pp24.push_back(pp[b % 6]);
    PP24.push_back(PP[b % 6]);
  }
  std::vector<int32_t> wide((size_t)24 * G);
  CHECK(stairs_generate_batch(c, pp24.data(), PP24.data(), 24, G, 3, wide.data(), &st) == STAIRS_OK);   // 96 rows
  CHECK(st.tokens == 24 * G);
  for (int b = 6; b < 24; ++b)          // the same prompt in another slot of the same forward: the same tokens
    CHECK(std::memcmp(wide.data() + (size_t)b * G, wide.data() + (size_t)(b % 6) * G, G * sizeof(int32_t)) == 0);
  CHECK(stairs_set_eos(c, wide[4]) == STAIRS_OK);
  CHECK(stairs_generate_batch(c, pp24.data(), PP24.data(), 24, G, 3, wide.data(), &st) == STAIRS_OK);
  CHECK(st.tokens < 24 * G);
  CHECK(stairs_set_eos(c, -1) == STAIRS_OK);
  // diagnostics
  float ms = -1.f;
  double bytes = 0.;
  CHECK(stairs_time_kernel(c, 2, 3, 64, 2, &ms, &bytes) == STAIRS_OK && ms > 0.f && bytes > 0.);
  CHECK(stairs_time_kernel(c, 99, 3, 64, 2, &ms, &bytes) == STAIRS_EINVAL);
  stairs_free(c);
  CHECK(stairs_copy_probe(1 << 20, 2, &ms, nullptr) == STAIRS_OK && ms > 0.f);
  CHECK(stairs_copy_probe(100, 2, &ms, nullptr) == STAIRS_EINVAL);

  // the GEMM entry points: host buffers, and caller-owned device buffers without allocation
  const int M = 5, N = 64, K = 512;
  std::vector<uint16_t> W = matrix(r, (size_t)N * K, 1.f);
  std::vector<float> X((size_t)M * K), Y1((size_t)M * N), Y2((size_t)M * N);
  for (auto& v : X) v = r.uniform();
  CHECK(stairs_gemm_host(STAIRS_DTYPE_BF16, W.data(), X.data(), Y1.data(), M, N, K, nullptr) == STAIRS_OK);
  void *dW = nullptr, *dX = nullptr, *dY = nullptr;
  CHECK(hipMalloc(&dW, W.size() * 2) == hipSuccess && hipMalloc(&dX, X.size() * 4) == hipSuccess &&
        hipMalloc(&dY, Y2.size() * 4) == hipSuccess);
  CHECK(hipMemcpy(dW, W.data(), W.size() * 2, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemcpy(dX, X.data(), X.size() * 4, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(stairs_gemm_device(STAIRS_DTYPE_BF16, dW, (const float*)dX, (float*)dY, M, N, K, nullptr) == STAIRS_OK);
  CHECK(hipDeviceSynchronize() == hipSuccess);
  CHECK(hipMemcpy(Y2.data(), dY, Y2.size() * 4, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(Y1 == Y2);
  CHECK(stairs_gemm_device(STAIRS_DTYPE_BF16, dW, (const float*)dX, (float*)dY, M, N, 16384, nullptr) == STAIRS_ECAPACITY);
  (void)hipFree(dW);
  (void)hipFree(dX);
  (void)hipFree(dY);
}

static void part2_encoder_decoder() {
  Rng r{23};
  const int V = 512, d = 256, H = 4, hd = 64, f = 512, Le = 2, Ld = 2, a = H * hd;
  stairs_encdec_cfg cfg = {Le, Ld, d, H, hd, f, V, 64, 96, 32, 128, 1e-6f};
  std::vector<uint16_t> emb = matrix(r, (size_t)V * d, 0.8f), head = matrix(r, (size_t)V * d, 0.08f);
  std::vector<float> eb(32 * H), db(32 * H), ones(d, 1.f);
  for (auto& v : eb) v = r.uniform();
  for (auto& v : db) v = r.uniform();
  std::vector<std::vector<uint16_t>> mats;
  auto mk = [&](size_t n) {
    mats.push_back(matrix(r, n, 0.08f));
    return (const void*)mats.back().data();
  };
  mats.reserve(64);
  std::vector<const void*> ewq, ewk, ewv, ewo, ein, eout, dwq, dwk, dwv, dwo, dcq, dck, dcv, dco, din, dout;
  std::vector<const float*> norms_e(Le, ones.data()), norms_d(Ld, ones.data());
  for (int l = 0; l < Le; ++l) {
    ewq.push_back(mk((size_t)a * d)); ewk.push_back(mk((size_t)a * d)); ewv.push_back(mk((size_t)a * d));
    ewo.push_back(mk((size_t)d * a)); ein.push_back(mk((size_t)f * d)); eout.push_back(mk((size_t)d * f));
  }
  for (int l = 0; l < Ld; ++l) {
    dwq.push_back(mk((size_t)a * d)); dwk.push_back(mk((size_t)a * d)); dwv.push_back(mk((size_t)a * d));
    dwo.push_back(mk((size_t)d * a)); dcq.push_back(mk((size_t)a * d)); dck.push_back(mk((size_t)a * d));
    dcv.push_back(mk((size_t)a * d)); dco.push_back(mk((size_t)d * a)); din.push_back(mk((size_t)f * d));
    dout.push_back(mk((size_t)d * f));
  }
  stairs_encdec_weights w{};
  w.tok_emb = emb.data(); w.lm_head = head.data();
  w.enc_rel_bias = eb.data(); w.dec_rel_bias = db.data();
  w.enc_final_norm = ones.data(); w.dec_final_norm = ones.data();
  w.enc_attn_norm = norms_e.data(); w.enc_ffn_norm = norms_e.data();
  w.enc_wq = ewq.data(); w.enc_wk = ewk.data(); w.enc_wv = ewv.data(); w.enc_wo = ewo.data();
  w.enc_w_in = ein.data(); w.enc_w_out = eout.data();
  w.dec_attn_norm = norms_d.data(); w.dec_cross_norm = norms_d.data(); w.dec_ffn_norm = norms_d.data();
  w.dec_wq = dwq.data(); w.dec_wk = dwk.data(); w.dec_wv = dwv.data(); w.dec_wo = dwo.data();
  w.dec_cq = dcq.data(); w.dec_ck = dck.data(); w.dec_cv = dcv.data(); w.dec_co = dco.data();
  w.dec_w_in = din.data(); w.dec_w_out = dout.data();
  stairs_encdec_cfg dcfg = cfg;          // assistant: the first encoder and decoder layer of the same model
  dcfg.n_enc_layers = dcfg.n_dec_layers = 1;
  stairs_ctx* c = nullptr;
  CHECK(stairs_encdec_init(&c, &cfg, &w, &dcfg, &w, 4, 0, nullptr) == STAIRS_OK && c != nullptr);
  if (!c) return;
  const int G = 30;
  stairs_stats st;
  for (int S : {1, 33, 64}) {
    std::vector<int32_t> src = prompt_of(r, S, V), base(G), got(G);
    CHECK(stairs_encdec_generate(c, src.data(), S, G, 0, base.data(), &st) == STAIRS_OK);
    CHECK(stairs_encdec_generate(c, src.data(), S, G, 4, got.data(), &st) == STAIRS_OK);
    CHECK(got == base && st.tokens == G);
    CHECK(stairs_encode(c, src.data(), S) == STAIRS_OK);
    CHECK(stairs_decode_sampled(c, G, 2, 0.5f, 7, got.data(), &st) == STAIRS_OK);
  }
  std::vector<int32_t> src = prompt_of(r, 65, V), got(G);
  CHECK(stairs_encode(c, src.data(), 65) == STAIRS_ECAPACITY);
  CHECK(stairs_prefill(c, src.data(), 10) == STAIRS_EINVAL);
  CHECK(stairs_reserve_batch(c, 2) == STAIRS_EINVAL);
  CHECK(stairs_encdec_generate(c, src.data(), 10, 200, 2, got.data(), &st) == STAIRS_ECAPACITY);
  stairs_free(c);
}

int main() {
  part1_without_gpu();
  std::printf("part 1 (no GPU): %d failed checks\n", g_failed);
  std::fflush(stdout);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) {
    (void)hipGetLastError();
    std::printf("no GPU visible: part 2 skipped\n");
    return g_failed ? 1 : 0;
  }
  part2_decoder_only();
  std::printf("part 2 (decoder-only): %d failed checks so far\n", g_failed);
  std::fflush(stdout);
  part2_encoder_decoder();
  std::printf("part 2 (encoder-decoder): %d failed checks in all\n", g_failed);
  return g_failed ? 1 : 0;
}
