// Host-side bookkeeping of the per-kernel opt-in for large dynamic LDS: which (kernel function, device)
// pairs have had their attribute set.  Plain C++ with no GPU dependency, so it can be unit-tested on a
// machine without a GPU.
#pragma once
#include <mutex>
#include <set>
#include <utility>

namespace aa {

class LdsOptInRegistry {
 public:
  // true until done() has been called for this (function, device): the caller then sets the attribute
  bool needs(const void* fn, int device) {
    std::lock_guard<std::mutex> lock(mu_);
    return done_.find(std::make_pair(fn, device)) == done_.end();
  }
  void done(const void* fn, int device) {
    std::lock_guard<std::mutex> lock(mu_);
    done_.insert(std::make_pair(fn, device));
  }
  size_t size() {
    std::lock_guard<std::mutex> lock(mu_);
    return done_.size();
  }

 private:
  std::mutex mu_;
  std::set<std::pair<const void*, int>> done_;
};

// one registry per process image (inline function: its static is shared by every translation unit)
inline LdsOptInRegistry& lds_optin_registry() {
  static LdsOptInRegistry r;
  return r;
}

}  // namespace aa
