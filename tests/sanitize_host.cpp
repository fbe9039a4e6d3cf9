// Host-side stress of the chunk store and the two-stage saver through the C ABI, meant to be
// built with -fsanitize=thread or -fsanitize=address (host code only; tests/test_sanitizers.py
// does that and runs it where there is no GPU).  Several threads use ONE store at the same
// time, each on its own contexts, as include/hcache.h allows: a saver producer (daemon threads
// behind it), plain appenders, readers of the index, and a dropper.  At the end every stored
// byte is compared with what was appended.  Exit status 0 and "sanitize_host ok" on success.
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "hcache.h"

#define CHECK(call)                                                                 \
  do {                                                                              \
    hc_status s_ = (call);                                                          \
    if (s_ != HC_OK) {                                                              \
      std::fprintf(stderr, "%s -> %d: %s\n", #call, (int)s_, hc_last_error());       \
      std::exit(2);                                                                 \
    }                                                                               \
  } while (0)

static const int L = 3, D = 64, CT = 8;              // layers, row width (bf16), rows per chunk

// row r of (context, layer): a recognisable pattern
static void fill_row(uint16_t* dst, int64_t seq, int layer, int r) {
  for (int c = 0; c < D; ++c) dst[c] = (uint16_t)(seq * 131 + layer * 17 + r * 3 + c);
}

static void verify(hc_store* st, int64_t seq, int n_tok) {
  std::vector<uint16_t> want(D);
  for (int l = 0; l < L; ++l) {
    if (hc_store_tokens(st, seq, l) != n_tok) { std::fprintf(stderr, "token count of %lld/%d\n", (long long)seq, l); std::exit(3); }
    for (int r = 0; r < n_tok; ++r) {
      const void* p = nullptr;
      int32_t rows = 0;
      CHECK(hc_store_chunk(st, seq, l, r / CT, &p, &rows));
      fill_row(want.data(), seq, l, r);
      if (r % CT >= rows || std::memcmp(static_cast<const uint16_t*>(p) + (size_t)(r % CT) * D, want.data(), D * 2) != 0) {
        std::fprintf(stderr, "row %d of %lld/%d differs\n", r, (long long)seq, l);
        std::exit(3);
      }
    }
  }
}

int main() {
  hc_store* st = nullptr;
  CHECK(hc_store_create_ex(L, D, CT, 4096, /*pinned=*/0, &st));
  hc_saver* sv = nullptr;
  CHECK(hc_saver_create(st, /*max_rows=*/64, /*n_slots=*/3, /*n_threads=*/4, &sv));
  std::atomic<bool> stop{false};

  // producer: continuous batching through the saver, contexts 100..103, rows of several
  // contexts per step, layer by layer
  const int saver_tokens = 90;
  std::thread producer([&] {
    std::vector<uint16_t> batch((size_t)64 * D);
    std::vector<int64_t> row_seq(64);
    for (int r = 0; r < saver_tokens; r += 5) {
      const int n = r + 5 <= saver_tokens ? 5 : saver_tokens - r;
      for (int l = 0; l < L; ++l) {
        int k = 0;
        for (int64_t seq = 100; seq < 104; ++seq)
          for (int i = 0; i < n; ++i, ++k) {
            fill_row(batch.data() + (size_t)k * D, seq, l, r + i);
            row_seq[k] = seq;
          }
        CHECK(hc_saver_save_layer_host(sv, l, batch.data(), k, row_seq.data()));
      }
    }
    CHECK(hc_saver_flush(sv));
  });
  // appenders: plain appends, two threads, disjoint contexts
  const int app_tokens = 70;
  auto appender = [&](int64_t first) {
    std::vector<uint16_t> rows((size_t)7 * D);
    for (int64_t seq = first; seq < first + 3; ++seq)
      for (int r = 0; r < app_tokens; r += 7)
        for (int l = 0; l < L; ++l) {
          for (int i = 0; i < 7; ++i) fill_row(rows.data() + (size_t)i * D, seq, l, r + i);
          CHECK(hc_store_append(st, seq, l, rows.data(), 7));
        }
  };
  std::thread app1(appender, 200), app2(appender, 300);
  // dropper: short-lived contexts come and go, returning chunks to the free list
  std::thread dropper([&] {
    std::vector<uint16_t> rows((size_t)CT * D);
    for (int it = 0; it < 200; ++it) {
      const int64_t seq = 900 + it % 5;
      for (int l = 0; l < L; ++l) {
        for (int i = 0; i < CT; ++i) fill_row(rows.data() + (size_t)i * D, seq, l, i);
        CHECK(hc_store_append(st, seq, l, rows.data(), CT));
      }
      CHECK(hc_store_drop(st, seq));
    }
  });
  // reader: polls the index of contexts other threads are appending to (counts only: rows of a
  // context that is still being written must not be read)
  std::thread reader([&] {
    int64_t seen = 0;
    while (!stop.load()) {
      for (int64_t seq : {100, 101, 200, 300, 302, 901})
        for (int l = 0; l < L; ++l) seen += hc_store_tokens(st, seq, l);
    }
    if (seen < 0) std::exit(4);
  });
  producer.join();
  app1.join();
  app2.join();
  dropper.join();
  stop.store(true);
  reader.join();

  for (int64_t seq = 100; seq < 104; ++seq) verify(st, seq, saver_tokens);
  for (int64_t seq : {200, 201, 202, 300, 301, 302}) verify(st, seq, app_tokens);
  CHECK(hc_saver_destroy(sv));
  CHECK(hc_store_destroy(st));
  std::puts("sanitize_host ok");
  return 0;
}
