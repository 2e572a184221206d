// Driver of the host-only sanitizer build: every entry point of the C ABI is run over exactly sized host allocations
// standing in for device memory (workspaces of precisely *_workspace_bytes bytes), at small ragged shapes and at the
// benchmark's shapes.  The kernel launchers are stubs that touch the ends of every operand (stub_launch.cpp), so an
// offset, extent or workspace-size mistake in the host layer is an address-sanitizer report; undefined behaviour in
// the host arithmetic (overflowing 32-bit products of sizes, misaligned access) is an UBSan report.
#include "../../include/streambp.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

namespace sbp { long long stub_touches(); }

static void* dmalloc(size_t bytes) {             // "device" memory: 256-byte aligned like a real allocation
  void* p = nullptr;
  if (posix_memalign(&p, 256, bytes ? bytes : 1) != 0) { std::perror("posix_memalign"); std::exit(2); }
  std::memset(p, 0, bytes < 4096 ? bytes : 4096);
  return p;
}
#define CHECK(expr) do { int32_t rc__ = (expr); if (rc__ != 0) { std::printf("FAIL %s -> %d (%s)\n", #expr, rc__, streambp_last_error()); return 1; } } while (0)

static int run_layer(int dtype, int B, int T, int chunk, int d, int Hq, int Hkv, int dh, int F, int window, bool pad, int rank) {
  const size_t es = dtype == SBP_BF16 ? 2 : 4, qd = (size_t)Hq * dh, kd = (size_t)Hkv * dh;
  sbp_layer_cfg c{};
  c.dtype = dtype; c.batch = B; c.seq_len = T; c.chunk = chunk; c.hidden = d; c.n_q_heads = Hq; c.n_kv_heads = Hkv; c.head_dim = dh;
  c.mlp_width = F; c.rms_eps = 1e-6f; c.rope_theta = 1e4f; c.window = window;
  std::vector<int32_t> first(B, 0);
  if (pad) { for (int b = 0; b < B; ++b) first[b] = (b * 37 + 5) % (T + 1); c.seq_first = first.data(); }
  const size_t msz[7] = {qd * d, kd * d, kd * d, d * qd, (size_t)F * d, (size_t)F * d, (size_t)d * F};
  void* wm[9]; void* gm[9];
  for (int i = 0; i < 7; ++i) { wm[i] = dmalloc(msz[i] * es); gm[i] = dmalloc(msz[i] * 4); }
  for (int i = 7; i < 9; ++i) { wm[i] = dmalloc(d * es); gm[i] = dmalloc((size_t)d * 4); }
  sbp_layer_weights w{wm[0], wm[1], wm[2], wm[3], wm[4], wm[5], wm[6], wm[7], wm[8]};
  sbp_layer_grads g{gm[0], gm[1], gm[2], gm[3], gm[4], gm[5], gm[6], (float*)gm[7], (float*)gm[8]};
  const size_t act = (size_t)B * T * d * es;
  void *x = dmalloc(act), *dy = dmalloc(act), *dx = dmalloc(act), *y = dmalloc(act);
  const size_t need = streambp_layer_workspace_bytes(&c);
  if (!need) { std::printf("FAIL workspace_bytes: %s\n", streambp_last_error()); return 1; }
  void* ws = dmalloc(need);
  CHECK(streambp_layer_backward(&c, &w, x, dy, dx, &g, ws, need, nullptr));
  CHECK(streambp_layer_forward(&c, &w, x, y, ws, need, nullptr));
  if (streambp_layer_backward(&c, &w, x, dy, dx, &g, ws, need - 1, nullptr) != SBP_ERR_WORKSPACE) { std::printf("FAIL: short workspace accepted\n"); return 1; }
  std::free(ws);
  if (rank > 0) {
    sbp_lora_adapters ad{}; sbp_lora_grads dg{};
    ad.rank = rank; ad.scale = 2.0f;
    const size_t outs[7] = {qd, kd, kd, (size_t)d, (size_t)F, (size_t)F, (size_t)d}, ins[7] = {(size_t)d, (size_t)d, (size_t)d, qd, (size_t)d, (size_t)d, (size_t)F};
    std::vector<void*> owned;
    for (int i = 0; i < 7; ++i) {
      if (i == 1) continue;                      // one matrix without an adapter
      void* a = dmalloc(rank * ins[i] * es); void* b = dmalloc(outs[i] * rank * es);
      void* da = dmalloc(rank * ins[i] * 4); void* db = dmalloc(outs[i] * rank * 4);
      ad.a[i] = a; ad.b[i] = b; dg.da[i] = (float*)da; dg.db[i] = (float*)db;
      owned.insert(owned.end(), {a, b, da, db});
    }
    const size_t need_l = streambp_layer_lora_workspace_bytes(&c, &ad);
    if (!need_l) { std::printf("FAIL lora workspace_bytes: %s\n", streambp_last_error()); return 1; }
    void* wl = dmalloc(need_l);
    CHECK(streambp_layer_lora_backward(&c, &w, &ad, x, dy, dx, &dg, wl, need_l, nullptr));
    std::free(wl);
    for (void* p : owned) std::free(p);
  }
  for (int i = 0; i < 9; ++i) { std::free(wm[i]); std::free(gm[i]); }
  std::free(x); std::free(dy); std::free(dx); std::free(y);
  return 0;
}

static int run_head(int dtype, int B, int T, int chunk, int d, int V, int objective, int grad_dtype) {
  const size_t es = dtype == SBP_BF16 ? 2 : 4, ges = grad_dtype == SBP_BF16 ? 2 : 4;
  sbp_head_cfg c{};
  c.dtype = dtype; c.batch = B; c.seq_len = T; c.chunk = chunk; c.hidden = d; c.vocab = V; c.objective = objective;
  c.loss_scale = 1.0f; c.clip_eps = 0.2f; c.kl_beta = 0.04f; c.grad_dtype = grad_dtype;
  const size_t rows = (size_t)B * T;
  void *w = dmalloc((size_t)V * d * es), *h = dmalloc(rows * d * es), *dh = dmalloc(rows * d * es), *dw = dmalloc((size_t)V * d * ges);
  int32_t* tg = (int32_t*)dmalloc(rows * 4);
  float *oldp = (float*)dmalloc(rows * 4), *refp = (float*)dmalloc(rows * 4), *adv = (float*)dmalloc((size_t)B * 4), *loss = (float*)dmalloc(4);
  int64_t* na = (int64_t*)dmalloc(8);
  const size_t need = streambp_lmhead_workspace_bytes(&c);
  if (!need) { std::printf("FAIL head workspace_bytes: %s\n", streambp_last_error()); return 1; }
  void* ws = dmalloc(need);
  CHECK(streambp_lmhead_ce_backward(&c, w, h, tg, oldp, refp, adv, dh, dw, loss, na, ws, need, nullptr));
  if (streambp_lmhead_ce_backward(&c, w, h, tg, oldp, refp, adv, dh, dw, loss, na, ws, need - 1, nullptr) != SBP_ERR_WORKSPACE) { std::printf("FAIL: short head workspace accepted\n"); return 1; }
  for (void* p : {w, h, dh, dw, (void*)tg, (void*)oldp, (void*)refp, (void*)adv, (void*)loss, (void*)na, ws}) std::free(p);
  return 0;
}

static int run_attn(int dtype, int Hq, int Hkv, int dh, int s, int cq, int window, int kv_first) {
  const size_t es = dtype == SBP_BF16 ? 2 : 4, qn = (size_t)cq * Hq * dh, kn = (size_t)(s + cq) * Hkv * dh;
  sbp_attn_cfg c{dtype, Hq, Hkv, dh, s, cq, 0.1f, window, kv_first};
  void *q = dmalloc(qn * es), *k = dmalloc(kn * es), *v = dmalloc(kn * es), *o = dmalloc(qn * es), *d_o = dmalloc(qn * es), *dq = dmalloc(qn * es);
  float *lse = (float*)dmalloc((size_t)Hq * cq * 4), *dk = (float*)dmalloc(kn * 4), *dv = (float*)dmalloc(kn * 4);
  const size_t need = streambp_attn_workspace_bytes(&c);
  void* ws = dmalloc(need);
  CHECK(streambp_attn_chunk_forward(&c, q, k, v, o, lse, nullptr));
  CHECK(streambp_attn_chunk_backward(&c, q, k, v, o, lse, d_o, dq, dk, dv, ws, need, nullptr));
  CHECK(streambp_attn_chunk_backward_noalloc(&c, q, k, v, o, lse, d_o, dq, dk, dv, nullptr));
  for (void* p : {q, k, v, o, d_o, dq, (void*)lse, (void*)dk, (void*)dv, ws}) std::free(p);
  return 0;
}

static int run_stack(int dtype, int L, int B, int T, int chunk, int d, int Hq, int Hkv, int dh, int F, int V, int head_chunk) {
  const size_t es = dtype == SBP_BF16 ? 2 : 4, qd = (size_t)Hq * dh, kd = (size_t)Hkv * dh, rows = (size_t)B * T;
  sbp_stack_cfg c{};
  c.layer.dtype = dtype; c.layer.batch = B; c.layer.seq_len = T; c.layer.chunk = chunk; c.layer.hidden = d; c.layer.n_q_heads = Hq;
  c.layer.n_kv_heads = Hkv; c.layer.head_dim = dh; c.layer.mlp_width = F; c.layer.rms_eps = 1e-6f; c.layer.rope_theta = 1e4f;
  c.n_layers = L; c.vocab = V; c.head_chunk = head_chunk; c.objective = SBP_OBJ_SFT; c.loss_scale = 1.0f; c.final_eps = 1e-6f;
  const size_t msz[7] = {qd * d, kd * d, kd * d, d * qd, (size_t)F * d, (size_t)F * d, (size_t)d * F};
  std::vector<sbp_layer_weights> ws(L); std::vector<sbp_layer_grads> gs(L); std::vector<void*> owned;
  auto own = [&](size_t b) { void* p = dmalloc(b); owned.push_back(p); return p; };
  for (int l = 0; l < L; ++l) {
    void* wm[9]; void* gm[9];
    for (int i = 0; i < 7; ++i) { wm[i] = own(msz[i] * es); gm[i] = own(msz[i] * 4); }
    for (int i = 7; i < 9; ++i) { wm[i] = own(d * es); gm[i] = own((size_t)d * 4); }
    ws[l] = sbp_layer_weights{wm[0], wm[1], wm[2], wm[3], wm[4], wm[5], wm[6], wm[7], wm[8]};
    gs[l] = sbp_layer_grads{gm[0], gm[1], gm[2], gm[3], gm[4], gm[5], gm[6], (float*)gm[7], (float*)gm[8]};
  }
  std::vector<void*> ckpt(L + 1);
  for (auto& p : ckpt) p = own(rows * d * es);
  void *emb = own((size_t)V * d * es), *w_head = own((size_t)V * d * es), *g_final = own(d * es), *dw_head = own((size_t)V * d * 4);
  void *demb = own((size_t)V * d * 4), *dg_final = own((size_t)d * 4), *dx0 = own(rows * d * es), *ids = own(rows * 4), *tg = own(rows * 4);
  void *loss = own(4), *na = own(8);
  const size_t need = streambp_stack_workspace_bytes(&c);
  if (!need) { std::printf("FAIL stack workspace_bytes: %s\n", streambp_last_error()); return 1; }
  void* wsp = own(need);
  CHECK(streambp_stack_forward(&c, ws.data(), emb, (const int32_t*)ids, ckpt.data(), wsp, need, nullptr));
  CHECK(streambp_stack_backward(&c, ws.data(), g_final, w_head, ckpt.data(), (const int32_t*)ids, (const int32_t*)tg, nullptr, nullptr, nullptr,
                                gs.data(), (float*)dg_final, dw_head, (float*)demb, dx0, (float*)loss, (int64_t*)na, wsp, need, nullptr));
  for (void* p : owned) std::free(p);
  return 0;
}

// A planted mistake, to show that the harness sees one: the caller's dx is one element short, as if the host layer had
// computed the last chunk's row offset one row too far.  Must end in an address-sanitizer report.
static int run_planted() {
  sbp_layer_cfg c{};
  c.dtype = SBP_F32; c.batch = 1; c.seq_len = 100; c.chunk = 32; c.hidden = 64; c.n_q_heads = 4; c.n_kv_heads = 4; c.head_dim = 16;
  c.mlp_width = 172; c.rms_eps = 1e-6f; c.rope_theta = 1e4f;
  const size_t msz[7] = {64 * 64, 64 * 64, 64 * 64, 64 * 64, 172 * 64, 172 * 64, 64 * 172};
  void* wm[9]; void* gm[9];
  for (int i = 0; i < 7; ++i) { wm[i] = dmalloc(msz[i] * 4); gm[i] = dmalloc(msz[i] * 4); }
  for (int i = 7; i < 9; ++i) { wm[i] = dmalloc(64 * 4); gm[i] = dmalloc(64 * 4); }
  sbp_layer_weights w{wm[0], wm[1], wm[2], wm[3], wm[4], wm[5], wm[6], wm[7], wm[8]};
  sbp_layer_grads g{gm[0], gm[1], gm[2], gm[3], gm[4], gm[5], gm[6], (float*)gm[7], (float*)gm[8]};
  void *x = dmalloc(100 * 64 * 4), *dy = dmalloc(100 * 64 * 4), *dx = std::malloc(100 * 64 * 4 - 4);
  const size_t need = streambp_layer_workspace_bytes(&c);
  void* ws = dmalloc(need);
  return streambp_layer_backward(&c, &w, x, dy, dx, &g, ws, need, nullptr);
}

int main(int argc, char** argv) {
  const bool big = argc > 1 && std::strcmp(argv[1], "big") == 0;
  if (argc > 1 && std::strcmp(argv[1], "planted") == 0) return run_planted();
  int bad = 0;
  // small ragged shapes, both storage types, every mask option, adapter mode
  bad += run_layer(SBP_F32, 1, 256, 64, 64, 4, 4, 16, 172, 0, false, 3);
  bad += run_layer(SBP_F32, 3, 97, 40, 64, 4, 2, 16, 172, 16, true, 0);
  bad += run_layer(SBP_BF16, 2, 333, 100, 256, 4, 2, 128, 512, 0, true, 8);
  bad += run_layer(SBP_BF16, 1, 1100, 128, 1024, 8, 2, 128, 4096, 200, false, 32);
  bad += run_layer(SBP_BF16, 1, 1, 1, 256, 4, 2, 128, 512, 0, false, 1);
  bad += run_layer(SBP_BF16, 1, 5, 1000000, 72, 6, 2, 24, 172, 0, false, 5);
  for (int obj = 0; obj < 3; ++obj) {
    bad += run_head(SBP_F32, 2, 50, 24, 64, 512, obj, SBP_F32);
    bad += run_head(SBP_BF16, 2, 300, 128, 256, 1024, obj, obj == 1 ? SBP_BF16 : SBP_F32);
  }
  bad += run_head(SBP_BF16, 1, 1, 1, 256, 1, SBP_OBJ_SFT, SBP_F32);
  bad += run_attn(SBP_BF16, 8, 2, 128, 300, 77, 0, 0);
  bad += run_attn(SBP_BF16, 8, 2, 128, 1000, 256, 300, 990);
  bad += run_attn(SBP_F32, 6, 2, 24, 0, 1, 0, 0);
  bad += run_stack(SBP_F32, 3, 1, 256, 64, 64, 4, 4, 16, 172, 512, 100);
  bad += run_stack(SBP_BF16, 2, 2, 300, 128, 256, 4, 2, 128, 512, 1024, 128);
  if (big) {   // the benchmark's shapes: sizes whose products pass 2^31
    bad += run_layer(SBP_BF16, 1, 32768, 2048, 3584, 28, 4, 128, 18944, 0, false, 32);
    bad += run_layer(SBP_BF16, 1, 70001, 4096, 256, 4, 2, 128, 512, 0, false, 0);
    bad += run_head(SBP_BF16, 1, 32768, 2048, 3584, 152064, SBP_OBJ_SFT, SBP_F32);
    bad += run_head(SBP_BF16, 8, 16384, 2048, 3584, 152064, SBP_OBJ_GRPO, SBP_F32);
  }
  std::printf("%s: %d failing cases, %lld operand extents touched\n", bad ? "FAILED" : "OK", bad, sbp::stub_touches());
  return bad ? 1 : 0;
}
