// CPU exercise of the staging pool's slot state machine (paper_2509_21841_amd/csrc/zp_pool.h) with a fake backend:
// several threads reserve, fill and submit slots at once while "copies" complete in the background. A slot handed to
// two threads at the same time, or handed out while the copy that reads it is still pending, is an error.
// Like the HIP runtime, the fake reports a never-recorded event as complete -- the case the RESERVED state exists for.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <thread>
#include <vector>

#include "../paper_2509_21841_amd/csrc/zp_pool.h"

struct FakeEvent {
  std::atomic<long> done_at{0};  // 0: never recorded; else the tick at which the copy behind it completes
};
static std::atomic<long> g_tick{1};
static std::atomic<int> g_errors{0};

struct Header {  // lives at the start of every host buffer
  std::atomic<int> owner;        // thread that is filling the buffer, 0 if none
  std::atomic<long> busy_until;  // tick until which a pending copy still reads the buffer
};

struct FakeBackend {
  typedef FakeEvent *event_t;
  typedef int stream_t;
  static int alloc(void **p, size_t bytes) {
    *p = std::calloc(1, bytes);
    return *p ? 0 : 1;
  }
  static void release(void *p) { std::free(p); }
  static int event_create(event_t *e) {
    *e = new FakeEvent();
    return 0;
  }
  static int event_record(event_t e, stream_t) {
    e->done_at.store(g_tick.load() + 40);  // the copy completes 40 ticks from now
    return 0;
  }
  static bool event_done(event_t e) { return g_tick.load() >= e->done_at.load(); }
};

int main() {
  zp_staging_pool<FakeBackend> pool;
  const int n_threads = 4, iters = 20000;
  std::atomic<bool> stop{false};
  std::thread clock([&] {
    while (!stop.load()) {
      g_tick.fetch_add(1);
      std::this_thread::yield();
    }
  });
  std::vector<std::thread> th;
  for (int t = 1; t <= n_threads; t++)
    th.emplace_back([&, t] {
      for (int i = 0; i < iters; i++) {
        int slot;
        void *host;
        if (pool.acquire(sizeof(Header) + 64 + (size_t)(i % 3) * 1000, &slot, &host)) { g_errors++; return; }
        Header *h = (Header *)host;
        int expect = 0;
        if (!h->owner.compare_exchange_strong(expect, t)) g_errors++;      // another thread is filling this buffer
        if (g_tick.load() < h->busy_until.load()) g_errors++;              // a pending copy still reads it
        char *payload = (char *)host + sizeof(Header);
        std::memset(payload, t, 64);
        std::this_thread::yield();
        for (int b = 0; b < 64; b++)
          if (payload[b] != (char)t) { g_errors++; break; }
        h->owner.store(0);
        if (i % 7 == 3) {
          pool.abandon(slot);                                              // an upload that failed before the copy
        } else {
          h->busy_until.store(g_tick.load() + 40);
          if (pool.submitted(slot, 0)) g_errors++;
        }
      }
    });
  for (auto &x : th) x.join();
  stop.store(true);
  clock.join();
  std::printf("slots %zu errors %d\n", pool.size(), g_errors.load());
  return g_errors.load() ? 1 : 0;
}
