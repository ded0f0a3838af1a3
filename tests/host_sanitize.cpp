// Native driver for the host side of the C ABI, built with AddressSanitizer + UndefinedBehaviorSanitizer on the host
// pass only (tests/test_host_sanitizers.py). It needs no GPU: it walks the host arithmetic, the argument checks that
// must refuse a call before anything is launched, and the feed's queue with real threads.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <chrono>
#include <thread>
#include <vector>

#include "qp.h"
#include "qp_feed.h"
#include "qp_layer.h"

static int failures = 0;
#define CHECK(cond)                                                   \
  do {                                                                \
    if (!(cond)) {                                                    \
      printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);        \
      ++failures;                                                     \
    }                                                                 \
  } while (0)

static void host_arithmetic() {
  CHECK(qp_keep_count(100, 0.07) == 7 && qp_keep_count(2048, 0.1) == 205 && qp_keep_count(0, 0.5) == 0);
  CHECK(qp_keep_count(10, 0.0) == -1 && qp_keep_count(10, 1.5) == -1);
  CHECK(qp_cache_capacity(3600, 128, 64, 0.1) == 46125 && qp_cache_capacity(0, 1, 1, 0.5) == -1);
  qp_layout L{28, 4, 128, QP_BF16, 0.f};
  CHECK(qp_workspace_bytes(&L, 2048, 64) > 0 && qp_workspace_bytes(nullptr, 2048, 64) == 0);
  const int n_gs[] = {1, 7, 64, 500, 512, 1024, 2048, 8192};
  const int cs[] = {0, 1, 63, 257, 5000, 9840, 46125, 200000};
  for (int n_g : n_gs)
    for (int c : cs) {
      qp_attend_plan_info p;
      CHECK(qp_attend_plan(&L, n_g, c, (size_t)32 << 20, &p) == QP_OK);
      CHECK(p.key_chunks >= 1 && p.workgroups >= 1 && p.scratch_bytes <= ((size_t)32 << 20));
      if (p.key_chunks > 1 && p.kernel == QP_ATTEND_MFMA) {
        const int n_ct = (c + 63) / 64;
        CHECK((p.key_chunks - 1) * p.tiles_per_chunk < n_ct && n_ct <= p.key_chunks * p.tiles_per_chunk);
      }
    }
  CHECK(qp_attend_plan(&L, 0, 10, 0, nullptr) != QP_OK);
  const int ms[] = {1, 64, 129, 2048, 8192};
  const int nk[][2] = {{3584, 3584}, {4608, 3584}, {3584, 18944}, {8, 64}, {8192, 29568}};
  for (int m : ms)
    for (auto& s : nk) {
      qp_linear_plan_info p;
      CHECK(qp_linear_plan(m, s[0], s[1], (size_t)32 << 20, &p) == QP_OK);
      CHECK((p.k_chunks - 1) * p.k_steps_per_chunk < s[1] / 64 && s[1] / 64 <= p.k_chunks * p.k_steps_per_chunk);
    }
  qp_linear_plan_info lp;
  CHECK(qp_linear_plan(4, 8, 72, 0, &lp) == QP_ERR_UNSUPPORTED && qp_linear_plan(4, 8, 64, 0, nullptr) == QP_ERR_INVALID_ARG);
  qp_layer_shape S{3584, 18944, 1e-6f, 1e6f, {16, 24, 24}};
  CHECK(qp_layer_workspace_bytes(&L, &S, 2048, 64) > qp_workspace_bytes(&L, 2048, 64));
  qp_layer_shape bad = S;
  bad.mrope_section[2] = 20;
  CHECK(qp_layer_workspace_bytes(&L, &bad, 2048, 64) == 0 && qp_layer_workspace_bytes(&L, nullptr, 2048, 64) == 0);
  CHECK(strlen(qp_status_string(QP_ERR_CAPACITY)) > 0 && strlen(qp_status_string((qp_status)77)) > 0);
  CHECK(strncmp(qp_version(), "quickprefill", 12) == 0);
  CHECK(qp_select_attend_kernel(99) == QP_ERR_INVALID_ARG && qp_select_attend_kernel(QP_ATTEND_AUTO) == QP_OK);
  CHECK(qp_select_linear_tile(64) == QP_ERR_INVALID_ARG && qp_select_linear_tile(0) == QP_OK);
}

// every call below must be refused by the host-side checks (nothing may reach a launch: there is no GPU here)
static void argument_errors() {
  qp_layout L{28, 4, 128, QP_BF16, 0.f};
  alignas(256) static unsigned char buf[4096];
  void* p = buf;
  void* odd = buf + 2;
  float* f = (float*)buf;
  int32_t pos3[3] = {0, 0, 0};
  qp_cache cache{p, p, (int32_t*)p, 16, 0};
  CHECK(qp_group_attend(nullptr, p, p, p, 4, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_group_attend(&L, nullptr, p, p, 4, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_group_attend(&L, odd, p, p, 4, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_group_attend(&L, p, p, p, 0, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_group_attend(&L, p, p, p, QP_MAX_GROUP_TOKENS + 1, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_UNSUPPORTED);
  qp_layout odd_heads{7, 4, 128, QP_BF16, 0.f};
  CHECK(qp_group_attend(&odd_heads, p, p, p, 4, &cache, p, nullptr, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_score_kv(&L, (qp_score_rule)9, p, p, 4, nullptr, 0, f, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_score_kv(&L, QP_SCORE_WINDOW_ATTN, p, p, 4, nullptr, 0, f, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_score_kv(&L, QP_SCORE_KEY_NORM_SMALL, nullptr, p, 4, nullptr, 0, f, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_topk_compact(&L, f, p, p, 4, 0, 0, &cache, nullptr, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_topk_compact(&L, f, p, p, 4, 5, 0, &cache, nullptr, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  qp_cache full{p, p, (int32_t*)p, 16, 15};
  CHECK(qp_topk_compact(&L, f, p, p, 4, 2, 0, &full, nullptr, p, 4096, nullptr) == QP_ERR_CAPACITY);
  CHECK(full.len == 15);
  CHECK(qp_prefill_video(&L, 8, 16, 2, 0.5, QP_SCORE_KEY_NORM_SMALL, p, p, p, nullptr, 0, &cache, p, p, 16, nullptr) == QP_ERR_CAPACITY);
  CHECK(qp_prefill_video(&L, 8, 16, 2, 1.5, QP_SCORE_KEY_NORM_SMALL, p, p, p, nullptr, 0, &cache, p, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(cache.len == 0);
  CHECK(qp_rms_norm(p, p, p, 4, 72 + 4, 1e-6f, nullptr) == QP_ERR_UNSUPPORTED);
  CHECK(qp_rms_norm(p, nullptr, p, 4, 64, 1e-6f, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_linear(p, p, nullptr, nullptr, p, 4, 8, 72, nullptr, 0, nullptr) == QP_ERR_UNSUPPORTED);
  CHECK(qp_linear(p, p, odd, nullptr, p, 4, 8, 64, nullptr, 0, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_linear(p, p, nullptr, nullptr, p, 4, 8, 64, odd, 64, nullptr) == QP_ERR_INVALID_ARG);
  const int32_t sec_bad[3] = {16, 24, 20}, sec[3] = {16, 24, 24};
  CHECK(qp_rope_table(pos3, 1, 1, 1e6f, sec_bad, f, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_rope_table(nullptr, 1, 1, 1e6f, sec, f, nullptr) == QP_ERR_INVALID_ARG);
  qp_layout d64{4, 2, 64, QP_BF16, 0.f};
  CHECK(qp_qkv_rope(&d64, p, p, p, f, 4, 64, p, p, p, nullptr, 0, nullptr) == QP_ERR_UNSUPPORTED);
  CHECK(qp_swiglu_gate_up(p, p, p, 4, 64, 64, nullptr) == QP_ERR_UNSUPPORTED);
  qp_layer_shape S{256, 384, 1e-6f, 1e6f, {16, 24, 24}};
  qp_layout small{4, 2, 128, QP_BF16, 0.f};
  qp_layer_weights W{p, p, p, p, p, p, p};
  CHECK(qp_layer_group(&small, &S, &W, p, pos3, 1, 4, 0, nullptr, 0, QP_SCORE_KEY_NORM_SMALL, 2, &cache, p, nullptr, p, 4096, nullptr) == QP_ERR_CAPACITY);
  CHECK(qp_layer_group(&small, &S, nullptr, p, pos3, 1, 4, 0, nullptr, 0, QP_SCORE_KEY_NORM_SMALL, 2, &cache, p, nullptr, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_layer_group(&small, &S, &W, p, pos3, 1, 4, 0, nullptr, 0, QP_SCORE_WINDOW_ATTN, 2, &cache, p, nullptr, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_layer_group(&small, &S, &W, p, pos3, 1, 4, 0, nullptr, 0, QP_SCORE_KEY_NORM_SMALL, 5, &cache, p, nullptr, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(cache.len == 0);
  CHECK(qp_layer_window_queries(&small, &S, &W, p, pos3, 1, 0, p, p, 4096, nullptr) == QP_ERR_INVALID_ARG);
  CHECK(qp_layer_window_queries(&small, &S, &W, p, pos3, 1, 4, p, p, 4096, nullptr) == QP_ERR_CAPACITY);
}

static void feed_queue() {
  qp_feed* f = nullptr;
  CHECK(qp_feed_create(1, 64, QP_FEED_PAGEABLE, &f) == QP_ERR_INVALID_ARG && f == nullptr);
  CHECK(qp_feed_create(3, 64, QP_FEED_PAGEABLE, &f) == QP_OK && f != nullptr);
  const int n_groups = 200;
  std::thread producer([&] {
    for (int i = 0; i < n_groups; ++i) {
      void* slot = nullptr;
      if (qp_feed_begin_write(f, &slot) != QP_OK) return;
      memset(slot, i & 0xff, 64);
      if (i % 17 == 0) std::this_thread::sleep_for(std::chrono::microseconds(300));
      if (qp_feed_publish(f, 8 + (size_t)(i % 7) * 8) != QP_OK) return;
    }
    qp_feed_close(f);
  });
  int seen = 0;
  for (;;) {
    const void* slot = nullptr;
    size_t bytes = 0;
    int32_t g = -1;
    qp_status st = qp_feed_next(f, 2000, &slot, &bytes, &g);
    if (st == QP_FEED_END) break;
    CHECK(st == QP_OK);
    if (st != QP_OK) break;
    CHECK(g == seen && bytes == 8 + (size_t)(g % 7) * 8);
    for (size_t b = 0; b < bytes; ++b) CHECK(((const unsigned char*)slot)[b] == (unsigned char)(g & 0xff));
    CHECK(qp_feed_release(f, g) == QP_OK);
    CHECK(qp_feed_release(f, g) == QP_ERR_INVALID_ARG);  // twice
    ++seen;
  }
  producer.join();
  CHECK(seen == n_groups);
  void* slot = nullptr;
  CHECK(qp_feed_begin_write(f, &slot) == QP_ERR_INVALID_ARG);  // closed
  qp_feed_destroy(f);

  // the stand-in producer, its sizes checked against the slots
  CHECK(qp_feed_create(2, 16, QP_FEED_PAGEABLE, &f) == QP_OK);
  std::vector<unsigned char> src(48);
  for (size_t i = 0; i < src.size(); ++i) src[i] = (unsigned char)i;
  const size_t too_big[1] = {17}, sizes[3] = {16, 16, 16};
  CHECK(qp_feed_stub_producer(f, src.data(), too_big, 1, 0, 0) == QP_ERR_CAPACITY);
  CHECK(qp_feed_stub_producer(f, src.data(), sizes, 3, 1000, 500) == QP_OK);
  CHECK(qp_feed_stub_producer(f, src.data(), sizes, 3, 1000, 500) == QP_ERR_INVALID_ARG);  // one stub per feed
  for (int g = 0; g < 3; ++g) {
    const void* s2 = nullptr;
    size_t bytes = 0;
    int32_t gi = -1;
    CHECK(qp_feed_next(f, -1, &s2, &bytes, &gi) == QP_OK && gi == g && bytes == 16);
    CHECK(memcmp(s2, src.data() + 16 * g, 16) == 0);
    CHECK(qp_feed_release(f, g) == QP_OK);
  }
  const void* s3 = nullptr;
  size_t b3 = 0;
  int32_t g3 = -1;
  CHECK(qp_feed_next(f, -1, &s3, &b3, &g3) == QP_FEED_END);
  double ms = 0;
  CHECK(qp_feed_stub_join(f, &ms) == QP_OK && ms >= 1.9);
  qp_feed_destroy(f);
  qp_feed_destroy(nullptr);
}

int main() {
  host_arithmetic();
  argument_errors();
  feed_queue();
  if (failures == 0) printf("ALL OK\n");
  return failures == 0 ? 0 : 1;
}
