// Hierarchical load balancing of rollout requests (Section 5.2 of the paper) as a host-side,
// step-driven simulation: it decides which requests decode together on which inference
// instance at every decode step, i.e. the batch composition that the decode-attention plan
// is then given.  No GPU code in this file.
//
//   intra-agent: every agent owns some inference instances; a min-heap over (load, instance)
//     yields the least-loaded instance for each new request (load = unfinished requests
//     assigned to the instance);
//   inter-agent: every poll_interval steps the waiting-queue lengths of the agents are
//     compared; when the largest exceeds the smallest by more than delta, instances of the
//     agent with the shortest queue move to the one with the longest (the donor keeps at least
//     one), are offline for migration_delay steps (weight transfer) and then serve the
//     receiver's new requests.
// The exact rules (tie-breaks, the number of instances moved, what happens to a moved
// instance's requests) are stated at marl_balancer_step in marl_decode.h; where the paper
// leaves them open the choices are listed there.
#include <algorithm>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "marl_decode.h"

namespace {

struct Request {
  int32_t id, agent, remaining, generated, instance;
  int64_t done_step;   // -1 while unfinished
};

// Binary min-heap over the active instances of one agent, keyed (load, instance id), with
// positions tracked so that a key can be changed or an instance removed in O(log n).
class LoadHeap {
 public:
  explicit LoadHeap(const std::vector<std::vector<int32_t>>* lists) : lists_(lists) {}
  bool empty() const { return heap_.empty(); }
  size_t size() const { return heap_.size(); }
  int32_t top() const { return heap_[0]; }
  const std::vector<int32_t>& members() const { return heap_; }
  void push(int32_t inst) {
    if ((size_t)inst >= pos_.size()) pos_.resize(inst + 1, -1);
    pos_[inst] = (int32_t)heap_.size();
    heap_.push_back(inst);
    up(heap_.size() - 1);
  }
  void remove(int32_t inst) {
    const size_t p = pos_[inst];
    pos_[inst] = -1;
    const int32_t last = heap_.back();
    heap_.pop_back();
    if (p < heap_.size()) {
      heap_[p] = last;
      pos_[last] = (int32_t)p;
      up(p);
      down(pos_[last]);
    }
  }
  void changed(int32_t inst) {   // the instance's load went up or down
    up(pos_[inst]);
    down(pos_[inst]);
  }

 private:
  bool less(int32_t a, int32_t b) const {
    const size_t la = (*lists_)[a].size(), lb = (*lists_)[b].size();
    return la != lb ? la < lb : a < b;
  }
  void up(size_t p) {
    while (p > 0) {
      const size_t parent = (p - 1) / 2;
      if (!less(heap_[p], heap_[parent])) break;
      swap_at(p, parent);
      p = parent;
    }
  }
  void down(size_t p) {
    for (;;) {
      size_t best = p;
      const size_t l = 2 * p + 1, r = l + 1;
      if (l < heap_.size() && less(heap_[l], heap_[best])) best = l;
      if (r < heap_.size() && less(heap_[r], heap_[best])) best = r;
      if (best == p) break;
      swap_at(p, best);
      p = best;
    }
  }
  void swap_at(size_t a, size_t b) {
    std::swap(heap_[a], heap_[b]);
    pos_[heap_[a]] = (int32_t)a;
    pos_[heap_[b]] = (int32_t)b;
  }
  const std::vector<std::vector<int32_t>>* lists_;
  std::vector<int32_t> heap_, pos_;
};

}  // namespace

struct marl_balancer {
  marl_balancer_config cfg;
  int64_t now = 0, completed = 0, migrations = 0;
  std::vector<Request> requests;                 // by submission order
  std::unordered_map<int32_t, int32_t> slot_of_id;   // request id -> index in `requests` (ids may be sparse)
  std::vector<std::vector<int32_t>> lists;       // per instance: indices into `requests`, FIFO
  std::vector<int32_t> owner, target;            // per instance: agent, or -1 while in transit
  std::vector<int64_t> arrive;                   // per instance in transit: step at which it joins `target`
  std::vector<LoadHeap> heaps;                   // per agent

  int32_t dispatch(int32_t req_index) {
    Request& r = requests[req_index];
    const int32_t inst = heaps[r.agent].top();
    lists[inst].push_back(req_index);
    r.instance = inst;
    heaps[r.agent].changed(inst);
    return inst;
  }
  int64_t waiting(int32_t agent) const {
    int64_t q = 0;
    for (int32_t inst : heaps[agent].members())
      q += std::max<int64_t>(0, (int64_t)lists[inst].size() - cfg.slots_per_instance);
    return q;
  }
};

// No exception may cross the C boundary: a failed host allocation becomes a status code.
template <class F>
int guarded(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return MARL_OUT_OF_MEMORY;
  } catch (...) {
    return MARL_INVALID_ARG;
  }
}

extern "C" {

int marl_balancer_create(const marl_balancer_config* cfg, const int32_t* instances_per_agent,
                         marl_balancer** out) {
  if (!cfg || !instances_per_agent || !out) return MARL_INVALID_ARG;
  if (cfg->num_agents < 1 || cfg->delta < 0 || cfg->slots_per_instance < 1 || cfg->poll_interval < 1 ||
      cfg->migration_delay < 0)
    return MARL_INVALID_ARG;
  long total = 0;
  for (int a = 0; a < cfg->num_agents; ++a) {
    if (instances_per_agent[a] < 1) return MARL_INVALID_ARG;   // every agent keeps one instance alive
    total += instances_per_agent[a];
    if (total > (1 << 24)) return MARL_UNSUPPORTED;
  }
  marl_balancer* b = new (std::nothrow) marl_balancer;
  if (!b) return MARL_OUT_OF_MEMORY;
  const int rc = guarded([&] {
    b->cfg = *cfg;
    b->lists.resize(total);
    b->owner.resize(total);
    b->target.assign(total, -1);
    b->arrive.assign(total, 0);
    b->heaps.reserve(cfg->num_agents);
    int32_t inst = 0;
    for (int a = 0; a < cfg->num_agents; ++a) {
      b->heaps.emplace_back(&b->lists);
      for (int k = 0; k < instances_per_agent[a]; ++k, ++inst) {
        b->owner[inst] = a;
        b->heaps[a].push(inst);
      }
    }
    return (int)MARL_OK;
  });
  if (rc != MARL_OK) {
    delete b;
    return rc;
  }
  *out = b;
  return MARL_OK;
}

void marl_balancer_destroy(marl_balancer* b) { delete b; }

int marl_balancer_submit(marl_balancer* b, int32_t agent, int32_t request_id, int32_t gen_len,
                         int32_t* instance) {
  if (!b || agent < 0 || agent >= b->cfg.num_agents || request_id < 0 || gen_len < 1) return MARL_INVALID_ARG;
  if (b->requests.size() >= (size_t)INT32_MAX) return MARL_UNSUPPORTED;
  return guarded([&] {
    if (!b->slot_of_id.emplace(request_id, (int32_t)b->requests.size()).second) return (int)MARL_INVALID_ARG;   // ids are unique
    b->requests.push_back(Request{request_id, agent, gen_len, 0, -1, -1});
    const int32_t inst = b->dispatch((int32_t)b->requests.size() - 1);
    if (instance) *instance = inst;
    return (int)MARL_OK;
  });
}

int marl_balancer_step(marl_balancer* b, marl_balancer_stats* stats) {
  if (!b) return MARL_INVALID_ARG;
  return guarded([&] {
  const int32_t I = (int32_t)b->lists.size(), A = b->cfg.num_agents, slots = b->cfg.slots_per_instance;
  // 1. instances whose weight transfer has finished join their new agent
  for (int32_t inst = 0; inst < I; ++inst)
    if (b->owner[inst] < 0 && b->arrive[inst] <= b->now) {
      b->owner[inst] = b->target[inst];
      b->target[inst] = -1;
      b->heaps[b->owner[inst]].push(inst);
    }
  // 2. one decode step: the first `slots` requests of every active instance emit a token
  for (int32_t inst = 0; inst < I; ++inst) {
    if (b->owner[inst] < 0) continue;
    std::vector<int32_t>& list = b->lists[inst];
    const size_t running = std::min<size_t>(list.size(), (size_t)slots);
    size_t keep = 0;
    for (size_t k = 0; k < list.size(); ++k) {
      Request& r = b->requests[list[k]];
      if (k < running) {
        ++r.generated;
        if (--r.remaining == 0) {
          r.done_step = b->now;
          r.instance = -1;
          ++b->completed;
          continue;
        }
      }
      list[keep++] = list[k];
    }
    if (keep != list.size()) {
      list.resize(keep);
      b->heaps[b->owner[inst]].changed(inst);
    }
  }
  ++b->now;
  // 3. inter-agent poll
  if (b->now % b->cfg.poll_interval == 0 && A > 1) {
    int32_t hi = 0, lo = 0;
    int64_t qhi = -1, qlo = -1;
    for (int32_t a = 0; a < A; ++a) {
      const int64_t q = b->waiting(a);
      if (q > qhi) { qhi = q; hi = a; }
      // the donor: shortest queue, among those the most active instances, then the lowest id
      if (qlo < 0 || q < qlo || (q == qlo && b->heaps[a].size() > b->heaps[lo].size())) { qlo = q; lo = a; }
    }
    const int64_t diff = qhi - qlo;
    if (diff > b->cfg.delta && hi != lo) {
      const int64_t want = (diff + slots - 1) / slots;
      const int64_t can = (int64_t)b->heaps[lo].size() - 1;
      for (int64_t m = std::min(want, can); m > 0; --m) {
        const int32_t inst = b->heaps[lo].top();        // the donor's least-loaded instance
        b->heaps[lo].remove(inst);
        b->owner[inst] = -1;
        b->target[inst] = hi;
        b->arrive[inst] = b->now + b->cfg.migration_delay;
        ++b->migrations;
        std::vector<int32_t> orphans;
        orphans.swap(b->lists[inst]);
        for (int32_t req : orphans) b->dispatch(req);   // re-queued on the donor's other instances
      }
    }
  }
  if (stats) {
    stats->now = b->now;
    stats->completed = b->completed;
    stats->submitted = (int64_t)b->requests.size();
    stats->migrations = b->migrations;
  }
  return (int)MARL_OK;
  });
}

int marl_balancer_agent_state(const marl_balancer* b, int32_t agent, int32_t* active_instances,
                              int64_t* waiting_requests, int64_t* assigned_requests) {
  if (!b || agent < 0 || agent >= b->cfg.num_agents) return MARL_INVALID_ARG;
  if (active_instances) *active_instances = (int32_t)b->heaps[agent].size();
  if (waiting_requests) *waiting_requests = b->waiting(agent);
  if (assigned_requests) {
    int64_t n = 0;
    for (int32_t inst : b->heaps[agent].members()) n += (int64_t)b->lists[inst].size();
    *assigned_requests = n;
  }
  return MARL_OK;
}

int marl_balancer_instance_batch(const marl_balancer* b, int32_t instance, int32_t* owner,
                                 int32_t* request_ids, int32_t* generated, int32_t capacity,
                                 int32_t* count) {
  if (!b || instance < 0 || (size_t)instance >= b->lists.size() || !count || capacity < 0) return MARL_INVALID_ARG;
  if (owner) *owner = b->owner[instance];
  const std::vector<int32_t>& list = b->lists[instance];
  const int32_t running = b->owner[instance] < 0 ? 0
                          : (int32_t)std::min<size_t>(list.size(), (size_t)b->cfg.slots_per_instance);
  *count = running;
  if (running > capacity) return MARL_WORKSPACE_TOO_SMALL;
  for (int32_t k = 0; k < running; ++k) {
    const Request& r = b->requests[list[k]];
    if (request_ids) request_ids[k] = r.id;
    if (generated) generated[k] = r.generated;
  }
  return MARL_OK;
}

int marl_balancer_request_state(const marl_balancer* b, int32_t request_id, int32_t* instance,
                                int32_t* generated, int64_t* done_step) {
  if (!b || request_id < 0) return MARL_INVALID_ARG;
  const auto it = b->slot_of_id.find(request_id);
  if (it == b->slot_of_id.end()) return MARL_INVALID_ARG;
  const Request& r = b->requests[it->second];
  if (instance) *instance = r.instance;
  if (generated) *generated = r.generated;
  if (done_step) *done_step = r.done_step;
  return MARL_OK;
}

}  // extern "C"
