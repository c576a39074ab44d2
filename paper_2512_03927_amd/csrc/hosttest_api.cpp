// Host-only C entry points that drive the slot pool and the decode scheduler without a GPU
// (used by the CPU tests; not part of the product boundary).
#include <cstdint>
#include <vector>

#include "sched.hpp"

using namespace odmoe;

struct HostSim {
  SlotPool pool;
  DecodeScheduler sched;
  std::vector<Action> acts;
  HostSim(int L, int E, int k, int S) : pool(S), sched(L, E, k, &pool) {}
};

static int flush(HostSim* s, int32_t* out, int cap) {
  int n = 0;
  for (const Action& a : s->acts) {
    if (n + 4 > cap) break;
    out[n++] = a.kind; out[n++] = a.layer; out[n++] = a.expert; out[n++] = a.slot;
  }
  s->acts.clear();
  return n / 4;
}

extern "C" {
void* odmoe_sim_new(int L, int E, int k, int S) { return new HostSim(L, E, k, S); }
void odmoe_sim_del(void* p) { delete static_cast<HostSim*>(p); }
void odmoe_sim_begin(void* p, const int32_t* pred) { static_cast<HostSim*>(p)->sched.begin_token(pred); }
// Each call appends actions as (kind, layer, expert, slot) quadruples into out; returns the count.
int odmoe_sim_before_route(void* p, int l, int32_t* out, int cap) {
  HostSim* s = static_cast<HostSim*>(p);
  s->sched.before_route(l, s->acts);
  return flush(s, out, cap);
}
int odmoe_sim_after_route(void* p, int l, const int32_t* actual, int32_t* slot_of_rank, int32_t* out, int cap) {
  HostSim* s = static_cast<HostSim*>(p);
  if (!s->sched.after_route(l, actual, s->acts, slot_of_rank)) return -1;
  return flush(s, out, cap);
}
int odmoe_sim_after_compute(void* p, int l, const int32_t* actual, int32_t* out, int cap) {
  HostSim* s = static_cast<HostSim*>(p);
  s->sched.after_compute(l, actual, s->acts);
  return flush(s, out, cap);
}
void odmoe_sim_counters(void* p, uint64_t* loads, uint64_t* reloads, uint64_t* hits) {
  HostSim* s = static_cast<HostSim*>(p);
  *loads = s->sched.loads; *reloads = s->sched.reloads; *hits = s->sched.hint_hits;
}
int odmoe_sim_n_free(void* p) { return static_cast<HostSim*>(p)->pool.n_free(); }
int odmoe_sim_pool_acquire(void* p, int layer, int expert) { return static_cast<HostSim*>(p)->pool.acquire(layer, expert); }
int odmoe_sim_pool_find(void* p, int layer, int expert) { return static_cast<HostSim*>(p)->pool.find(layer, expert); }
int odmoe_sim_pool_release(void* p, int slot) { return static_cast<HostSim*>(p)->pool.release(slot) ? 0 : -1; }
void odmoe_sim_pool_release_all(void* p) { static_cast<HostSim*>(p)->pool.release_all(); }
}
