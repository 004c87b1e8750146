// chain_table_check.cpp -- the bookkeeping of run-time compiled chains (csrc/nfad_chain_table.hpp)
// exercised on the host with a stand-in kernel type: slot reuse, the capacity counting LIVE chains
// only, kernels shared between chains that differ in constants and destroyed with their last user.
// Plain C++, no GPU.  Exit status 0 = all checks passed.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <thread>

#include "../../paper_2209_10778_amd/csrc/nfad_chain_table.hpp"

static std::atomic<int> g_alive{0};   // stand-in kernels currently loaded
struct FakeKernel {
  int uid;
  explicit FakeKernel(int u) : uid(u) { ++g_alive; }
  ~FakeKernel() { --g_alive; }
};
struct FakeArgs {
  float c[4];
};
using Table = nfad::jit::ChainTable<FakeKernel, FakeArgs>;

static int g_failures = 0;
#define CHECK(cond)                                                     \
  do {                                                                  \
    if (!(cond)) {                                                      \
      std::printf("%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      ++g_failures;                                                     \
    }                                                                   \
  } while (0)

static std::shared_ptr<FakeKernel> kernel_for(Table& t, const std::string& key, int* compiles) {
  std::shared_ptr<FakeKernel> k = t.find_kernel(key);
  if (!k) {
    ++*compiles;
    k = t.adopt(key, std::make_shared<FakeKernel>(*compiles));
  }
  return k;
}

int main() {
  {
    Table t(3);   // the capacity hook: three live chains
    int compiles = 0;
    // a loop that compiles and releases far more chains than the capacity never fills the table
    for (int step = 0; step < 10000; ++step) {
      CHECK(t.has_room());
      const int slot = t.insert("x c *", "Mul<X, Arg<0>>", kernel_for(t, "Mul<X, Arg<0>>", &compiles), FakeArgs{{(float)step}});
      CHECK(slot == 0);                       // the freed slot is handed out again
      Table::Chain c;
      CHECK(t.get(slot, c) && c.args.c[0] == (float)step && c.name == "jit:0");
      CHECK(t.release(slot));
      CHECK(!t.release(slot));                // a dead id stays dead
    }
    CHECK(t.live() == 0 && g_alive == 0);     // the kernel went with its last chain each time

    // chains that differ only in constants share one kernel; it survives until the last one goes
    compiles = 0;
    const int a = t.insert("x 0.1 *", "K1", kernel_for(t, "K1", &compiles), FakeArgs{{0.1f}});
    const int b = t.insert("x 0.2 *", "K1", kernel_for(t, "K1", &compiles), FakeArgs{{0.2f}});
    const int c = t.insert("x tanh", "K2", kernel_for(t, "K2", &compiles), FakeArgs{});
    CHECK(a == 0 && b == 1 && c == 2 && compiles == 2 && g_alive == 2 && t.live_kernels() == 2);
    CHECK(!t.has_room());
    CHECK(t.insert("x exp", "K3", std::make_shared<FakeKernel>(99), FakeArgs{}) == -1);   // full: live chains count
    CHECK(g_alive == 2);                      // ... and the rejected kernel is gone
    Table::Chain ca, cb;
    CHECK(t.get(a, ca) && t.get(b, cb) && ca.kernel == cb.kernel && ca.args.c[0] != cb.args.c[0]);
    ca = Table::Chain();
    cb = Table::Chain();
    CHECK(t.release(a) && g_alive == 2);      // b still uses K1
    CHECK(t.has_room());
    const int d = t.insert("x 0.3 *", "K1", kernel_for(t, "K1", &compiles), FakeArgs{{0.3f}});
    CHECK(d == 0 && compiles == 2);           // lowest free slot, no new compile
    CHECK(t.release(b) && t.release(d) && g_alive == 1 && t.live_kernels() == 1);
    CHECK(t.find_kernel("K1") == nullptr);

    // a call in flight (a copy of the chain) keeps the kernel loaded across a release
    Table::Chain in_flight;
    CHECK(t.get(c, in_flight));
    CHECK(t.release(c) && g_alive == 1 && t.live() == 0);
    CHECK(t.peek(c) == nullptr);
    in_flight = Table::Chain();
    CHECK(g_alive == 0);
  }
  {
    // concurrent compile / launch / release of the same structure from several threads
    Table t(64);
    std::vector<std::thread> threads;
    for (int w = 0; w < 8; ++w)
      threads.emplace_back([&t, w] {
        for (int i = 0; i < 2000; ++i) {
          std::shared_ptr<FakeKernel> k = t.find_kernel("K");
          if (!k) k = t.adopt("K", std::make_shared<FakeKernel>(w));
          const int slot = t.insert("p", "K", k, FakeArgs{{(float)i}});
          if (slot < 0) continue;
          Table::Chain c;
          if (t.get(slot, c) && c.kernel == nullptr) std::abort();
          t.release(slot);
        }
      });
    for (auto& th : threads) th.join();
    CHECK(t.live() == 0);
  }
  CHECK(g_alive == 0);
  std::printf(g_failures ? "FAILED: %d check(s)\n" : "all checks passed\n", g_failures);
  return g_failures ? 1 : 0;
}
