// Plans of recent one-shot calls (lc_copy, lc_gemm), keyed by everything a plan depends on: the layouts' text, the element
// type, the pointers' alignment and the tuning settings in force.  Planning is pure host work, so a hit changes nothing
// but the time of the call.  Thread-safe; bounded: when full it is emptied (callers with many distinct layouts should
// hold plan handles themselves).
#pragma once
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>

namespace lc {

template <typename Plan>
class PlanCache {
 public:
  std::shared_ptr<const Plan> find(const std::string& key) {
    std::lock_guard<std::mutex> hold(lock_);
    auto it = plans_.find(key);
    return it == plans_.end() ? nullptr : it->second;
  }
  void insert(const std::string& key, std::shared_ptr<const Plan> plan) {
    std::lock_guard<std::mutex> hold(lock_);
    if (plans_.size() >= kCapacity) plans_.clear();
    plans_[key] = std::move(plan);
  }

 private:
  static constexpr size_t kCapacity = 256;
  std::mutex lock_;
  std::unordered_map<std::string, std::shared_ptr<const Plan>> plans_;
};

}  // namespace lc
