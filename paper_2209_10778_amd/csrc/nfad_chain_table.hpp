// nfad_chain_table.hpp -- the table of run-time compiled chains: the one stateful part of
// libnfad.  Plain C++ (no HIP): the compiled kernel is a payload type whose destructor releases
// it, so the bookkeeping can be exercised on a machine without a GPU.
//
// A CHAIN is what a caller holds an id for: a program text, the values of its run-time
// constants, and a reference to a KERNEL.  A kernel is one compiled forward kernel, identified
// by the program's structure with its constants left open (the key), and shared by every live
// chain whose program differs only in those constants.  Ids are slot numbers: a released
// chain's slot is handed out again, so the capacity bounds LIVE chains, however many were
// compiled and released before.  A kernel dies with its last chain (or with the last call that
// still holds a reference to it).  Every method takes the table's lock; nothing is handed out
// by pointer.
#pragma once
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <vector>

namespace nfad {
namespace jit {

template <class Kernel, class Args>
class ChainTable {
 public:
  struct Chain {
    std::string program, name, key;
    std::shared_ptr<Kernel> kernel;
    Args args{};
  };

  explicit ChainTable(int capacity) : capacity_(capacity) {}

  int capacity() const { return capacity_; }
  int live() {
    std::lock_guard<std::mutex> lock(mu_);
    return live_;
  }
  bool has_room() {
    std::lock_guard<std::mutex> lock(mu_);
    return live_ < capacity_;
  }

  // The live kernel compiled for `key`, or null.
  std::shared_ptr<Kernel> find_kernel(const std::string& key) {
    std::lock_guard<std::mutex> lock(mu_);
    auto it = kernels_.find(key);
    return it == kernels_.end() ? nullptr : it->second.lock();
  }

  // Registers a freshly compiled kernel under `key` and returns the kernel to use: `fresh`, or
  // the one another thread registered for the same key in the meantime (`fresh` is then dropped).
  std::shared_ptr<Kernel> adopt(const std::string& key, std::shared_ptr<Kernel> fresh) {
    std::lock_guard<std::mutex> lock(mu_);
    auto it = kernels_.find(key);
    if (it != kernels_.end()) {
      if (std::shared_ptr<Kernel> old = it->second.lock()) return old;
    }
    kernels_[key] = fresh;
    return fresh;
  }

  // A new chain in the lowest free slot; -1 if `capacity` chains are live.
  int insert(const std::string& program, const std::string& key, std::shared_ptr<Kernel> kernel, const Args& args) {
    std::lock_guard<std::mutex> lock(mu_);
    if (live_ >= capacity_) return -1;
    size_t slot = 0;
    while (slot < slots_.size() && slots_[slot]) ++slot;
    if (slot == slots_.size()) slots_.emplace_back();
    slots_[slot].reset(new Chain{program, "jit:" + std::to_string(slot), key, std::move(kernel), args});
    ++live_;
    return (int)slot;
  }

  // Frees a slot; false if the slot is not live.  The kernel goes with its last chain -- or, if a
  // call in flight still holds a reference, when that call returns.
  bool release(int slot) {
    std::shared_ptr<Kernel> last;   // destroyed after the lock is dropped: unloading may be slow
    std::lock_guard<std::mutex> lock(mu_);
    if (slot < 0 || slot >= (int)slots_.size() || !slots_[slot]) return false;
    last = std::move(slots_[slot]->kernel);
    if (last.use_count() == 1) kernels_.erase(slots_[slot]->key);   // no other chain, no call: forget the key
    slots_[slot].reset();
    --live_;
    return true;
  }

  // Number of distinct kernels that are alive (diagnostics and tests).
  int live_kernels() {
    std::lock_guard<std::mutex> lock(mu_);
    int n = 0;
    for (auto& kv : kernels_) n += kv.second.expired() ? 0 : 1;
    return n;
  }

  // A copy of a live chain (the copy's kernel reference keeps the kernel loaded while it is used).
  bool get(int slot, Chain& out) {
    std::lock_guard<std::mutex> lock(mu_);
    if (slot < 0 || slot >= (int)slots_.size() || !slots_[slot]) return false;
    out = *slots_[slot];
    return true;
  }

  // The address of a live chain's strings stays valid until the chain is released.
  const Chain* peek(int slot) {
    std::lock_guard<std::mutex> lock(mu_);
    return (slot < 0 || slot >= (int)slots_.size()) ? nullptr : slots_[slot].get();
  }

 private:
  std::mutex mu_;
  const int capacity_;
  int live_ = 0;
  std::vector<std::unique_ptr<Chain>> slots_;
  std::map<std::string, std::weak_ptr<Kernel>> kernels_;
};

}  // namespace jit
}  // namespace nfad
