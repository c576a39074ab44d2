// Host-side bookkeeping of the cacheless decode: which expert sits in which HBM slot, and in
// which order loads, evictions and computations are issued.  Pure C++ (no HIP), so the state
// machine can be driven on a CPU with a fake copy engine.
//
// Paper background (Section 3.1): worker groups alternate between loading the experts of a
// future layer (EL_l) and computing the current one (EC_l); an expert is evicted right after
// use; when the router disagrees with the prediction the computation waits for a reload.
// On one GPU the "groups" are groups of k slots: S slots hold floor(S/k) layers' experts.
#pragma once
#include <cstdint>
#include <cstddef>
#include <deque>
#include <vector>

namespace odmoe {

class SlotPool {
 public:
  struct Slot {
    int32_t layer = -1, expert = -1;
    bool occupied = false;
  };

  explicit SlotPool(int n) : slots_(n) {
    for (int i = 0; i < n; ++i) free_.push_back(i);
  }
  int size() const { return (int)slots_.size(); }
  int n_free() const { return (int)free_.size(); }
  const Slot& at(int s) const { return slots_[s]; }

  int find(int32_t layer, int32_t expert) const {
    for (int s = 0; s < (int)slots_.size(); ++s)
      if (slots_[s].occupied && slots_[s].layer == layer && slots_[s].expert == expert) return s;
    return -1;
  }
  // Oldest-released free slot first, so a new copy rarely has to wait for the kernels that
  // read the slot's previous tenant.  -1 when every slot is occupied.
  int acquire(int32_t layer, int32_t expert) {
    if (free_.empty()) return -1;
    int s = free_.front();
    free_.pop_front();
    slots_[s].layer = layer;
    slots_[s].expert = expert;
    slots_[s].occupied = true;
    return s;
  }
  bool release(int s) {
    if (s < 0 || s >= (int)slots_.size() || !slots_[s].occupied) return false;
    slots_[s] = Slot();
    free_.push_back(s);
    return true;
  }
  // Every occupied slot becomes free (a call failed part-way: what it had loaded is not kept).
  void release_all() {
    for (int s = 0; s < (int)slots_.size(); ++s)
      if (slots_[s].occupied) release(s);
  }

 private:
  std::vector<Slot> slots_;
  std::deque<int> free_;
};

struct Action {
  enum Kind { LOAD = 0, DROP = 1, RELEASE = 2 };
  // LOAD: copy (layer, expert) into slot.   DROP: a wrongly predicted expert leaves its slot
  // unused.   RELEASE: a used expert leaves its slot after the layer's kernels (eviction).
  int32_t kind, layer, expert, slot;
};

// Order of loads / evictions for one decode token through L layers with S slots.
class DecodeScheduler {
 public:
  DecodeScheduler(int L, int E, int k, SlotPool* pool) : L_(L), E_(E), k_(k), pool_(pool) {}

  uint64_t loads = 0, reloads = 0, hint_hits = 0;

  void begin_token(const int32_t* pred) {
    pred_ = pred;
    next_issue_ = 0;
    loads = reloads = hint_hits = 0;
  }

  // Before layer l is routed: issue predicted loads for layers l, l+1, ... while a whole group
  // of k slots is free (round-robin over slot groups).  At most floor(S/k) layers are in
  // flight, so the layer being routed can always obtain k slots for reloads, whatever the
  // hints of later layers occupy.
  void before_route(int l, std::vector<Action>& out) {
    if (!pred_) return;
    if (next_issue_ < l) next_issue_ = l;
    const int ahead = pool_->size() / k_;
    while (next_issue_ < L_ && next_issue_ < l + ahead && pool_->n_free() >= k_) {
      const int32_t* p = pred_ + (size_t)next_issue_ * k_;
      for (int i = 0; i < k_; ++i) {
        int32_t e = p[i];
        if (e < 0 || e >= E_) continue;                     // unusable hint
        if (pool_->find(next_issue_, e) >= 0) continue;     // duplicate hint
        int s = pool_->acquire(next_issue_, e);
        out.push_back(Action{Action::LOAD, next_issue_, e, s});
        ++loads;
      }
      ++next_issue_;
    }
  }

  // After layer l is routed.  `actual` = the k experts the router chose.  Wrong predictions are
  // dropped, missing experts loaded.  slot_of_rank[i] receives the slot of actual[i].
  // Returns false if a slot could not be found (cannot happen when S >= k).
  bool after_route(int l, const int32_t* actual, std::vector<Action>& out, int32_t* slot_of_rank) {
    const bool hinted = pred_ && next_issue_ > l;
    // drop every expert of layer l that sits in a slot but was not chosen
    for (int s = 0; s < pool_->size(); ++s) {
      const SlotPool::Slot& sl = pool_->at(s);
      if (!sl.occupied || sl.layer != l) continue;
      bool used = false;
      for (int i = 0; i < k_; ++i) used |= (actual[i] == sl.expert);
      if (!used) {
        out.push_back(Action{Action::DROP, l, sl.expert, s});
        pool_->release(s);
      }
    }
    for (int i = 0; i < k_; ++i) {
      int s = pool_->find(l, actual[i]);
      if (s >= 0) {
        if (hinted) ++hint_hits;
      } else {
        s = pool_->acquire(l, actual[i]);
        if (s < 0) return false;
        out.push_back(Action{Action::LOAD, l, actual[i], s});
        ++loads;
        if (hinted) ++reloads;
      }
      slot_of_rank[i] = s;
    }
    return true;
  }

  // After the kernels of layer l are enqueued: evict its experts.
  void after_compute(int l, const int32_t* actual, std::vector<Action>& out) {
    for (int i = 0; i < k_; ++i) {
      int s = pool_->find(l, actual[i]);
      if (s >= 0) {
        out.push_back(Action{Action::RELEASE, l, actual[i], s});
        pool_->release(s);
      }
    }
  }

 private:
  int L_, E_, k_;
  SlotPool* pool_;
  const int32_t* pred_ = nullptr;
  int next_issue_ = 0;
};

}  // namespace odmoe
