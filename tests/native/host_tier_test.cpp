// CPU-only exercise of the pinned-unit ring and its drain threads (built with a thread sanitizer by
// the test that runs it).  A "copy engine" thread stands in for the GPU: it fills ring units some time
// after they are handed to it, and the job's ready() waits for that, as the library waits for an event.
#include <cstdio>
#include <algorithm>
#include <cstdlib>
#include <random>

#include "host_tier.hpp"

namespace {

struct Engine {  // fills units asynchronously, in order, like copies queued on a stream
  struct Op {
    char *dst;
    int64_t bytes;
    uint32_t seed;
    std::shared_ptr<std::atomic<bool>> done;
  };
  std::mutex m;
  std::condition_variable cv;
  std::deque<Op> q;
  bool quit = false;
  std::thread th;
  Engine() : th([this] { run(); }) {}
  ~Engine() {
    {
      std::lock_guard<std::mutex> g(m);
      quit = true;
    }
    cv.notify_all();
    th.join();
  }
  static void fill(char *p, int64_t n, uint32_t seed) {
    uint32_t x = seed * 2654435761u + 12345u;
    for (int64_t i = 0; i < n; ++i) {
      x = x * 1664525u + 1013904223u;
      p[i] = (char)(x >> 24);
    }
  }
  void push(Op op) {
    {
      std::lock_guard<std::mutex> g(m);
      q.push_back(std::move(op));
    }
    cv.notify_one();
  }
  void run() {
    for (;;) {
      Op op;
      {
        std::unique_lock<std::mutex> lk(m);
        cv.wait(lk, [this] { return quit || !q.empty(); });
        if (q.empty()) return;
        op = std::move(q.front());
        q.pop_front();
      }
      fill(op.dst, op.bytes, op.seed);
      op.done->store(true, std::memory_order_release);
    }
  }
};

int check(bool ok, const char *what) {
  if (!ok) std::fprintf(stderr, "FAILED: %s\n", what);
  return ok ? 0 : 1;
}

}  // namespace

int main(int argc, char **argv) {
  const int threads = argc > 1 ? std::atoi(argv[1]) : 3;
  const int units = argc > 2 ? std::atoi(argv[2]) : 3;
  const int64_t unit_bytes = 4096;
  const int layers = 24;
  int bad = 0;
  std::vector<char> ring((size_t)(units * unit_bytes));
  lkv::HostTier tier;
  tier.start(ring.data(), unit_bytes, units, threads, layers);
  Engine engine;
  std::mt19937 rng(7);

  // offload direction: engine fills a unit, a worker drains it into the layer's pageable image
  std::vector<std::vector<char>> image((size_t)layers), want((size_t)layers);
  for (int l = 0; l < layers; ++l) {
    int64_t bytes = 1 + (int64_t)(rng() % (5 * unit_bytes));
    if (l == 3) bytes = 0;
    if (l == 4) bytes = 2 * unit_bytes;  // whole units, no tail
    image[(size_t)l].assign((size_t)bytes, 0);
    want[(size_t)l].assign((size_t)bytes, 0);
    for (int64_t off = 0; off < bytes; off += unit_bytes) {
      int64_t m = bytes - off < unit_bytes ? bytes - off : unit_bytes;
      uint32_t seed = (uint32_t)(l * 1000 + off / unit_bytes);
      Engine::fill(want[(size_t)l].data() + off, m, seed);
      int u = tier.acquire();
      bad += check(u >= 0 && u < units, "unit index in range");
      auto done = std::make_shared<std::atomic<bool>>(false);
      engine.push({tier.unit_ptr(u), m, seed, done});
      lkv::HostTier::Job j;
      j.ready = [done] {
        while (!done->load(std::memory_order_acquire)) std::this_thread::yield();
        return true;
      };
      j.dst = image[(size_t)l].data() + off;
      j.src = tier.unit_ptr(u);
      j.bytes = m;
      j.unit = u;
      j.key = l;
      tier.submit(std::move(j));
    }
    if (l % 5 == 0) {  // a reader that waits for one layer only sees that layer complete
      bad += check(tier.wait_key(l), "wait_key reports success");
      bad += check(image[(size_t)l] == want[(size_t)l], "layer image complete after wait_key");
    }
  }
  bad += check(tier.wait_all(), "wait_all reports success");
  for (int l = 0; l < layers; ++l) bad += check(image[(size_t)l] == want[(size_t)l], "layer image after wait_all");
  bad += check(!tier.busy_key(0), "nothing pending after wait_all");

  // every unit is back: they can all be taken without blocking
  std::vector<int> got;
  for (int i = 0; i < units; ++i) got.push_back(tier.acquire());
  std::sort(got.begin(), got.end());
  for (int i = 0; i < units; ++i) bad += check(got[(size_t)i] == i, "all units returned exactly once");
  for (int u : got) tier.release(u);

  // split memcpy: sizes around the piece size, odd tails, small and empty
  for (int64_t bytes : {(int64_t)0, (int64_t)1, (int64_t)4097, ((int64_t)4 << 20) - 1, ((int64_t)9 << 20) + 13,
                        (int64_t)33 << 20}) {
    std::vector<char> a((size_t)bytes), b((size_t)bytes + 64, 0x5a);
    Engine::fill(a.data(), bytes, (uint32_t)bytes);
    tier.copy_parallel(b.data(), a.data(), bytes);
    bad += check(std::memcmp(a.data(), b.data(), (size_t)bytes) == 0, "copy_parallel copies every byte");
    bool tail_ok = true;
    for (int i = 0; i < 64; ++i) tail_ok &= b[(size_t)bytes + i] == 0x5a;
    bad += check(tail_ok, "copy_parallel writes nothing past the end");
  }

  // a failed wait is reported, the unit still comes back, and later jobs still run
  {
    int u = tier.acquire();
    lkv::HostTier::Job j;
    j.ready = [] { return false; };
    j.unit = u;
    j.key = 1;
    tier.submit(std::move(j));
    bad += check(!tier.wait_key(1), "failed wait is reported by wait_key");
    bad += check(tier.failed(), "failure is sticky");
    int v = tier.acquire();
    tier.release(v);
  }
  tier.stop();
  tier.stop();  // idempotent
  std::printf("host_tier_test: %s (threads %d, units %d, drained %lld bytes)\n", bad ? "FAILED" : "ok", threads, units,
              (long long)tier.copied_bytes());
  return bad ? 1 : 0;
}
