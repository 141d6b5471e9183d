// Host-side phase-aware scheduler (paper Section IV): instance selection for
// reasoning requests (Algorithm 1) and for answering requests (Algorithm 2),
// the adaptive-migration rule, and the two-level round-robin queues of the
// intra-instance scheduler.  Produces batches and block tables in the layout of
// the pkv kernels and ordered data-movement orders; touches no GPU itself.
#include "../../include/pascal_sched.h"

#include <algorithm>
#include <cmath>
#include <new>
#include <vector>

namespace {

struct Request {
  int instance = 0;
  int phase = PASCAL_REASONING;
  int state = PASCAL_QUEUED;
  int level = 0;                // 0: high-priority queue, 1: low-priority queue
  int prompt = 0;
  int kv_tokens = 0;
  int reasoning_tokens = 0;
  int quantum_used = 0;
  int quanta_done = 0;          // quanta completed in the current queue
  int host_blocks = 0;          // size of the image in the host store while offloaded
  int preemptions = 0;
  int migrations = 0;
  double arrival = 0.0;
  double finish = -1.0;
  std::vector<int32_t> blocks;       // GPU blocks in table order
  std::vector<double> answer_times;  // when each answering token was produced
};

struct Instance {
  std::vector<int32_t> free_blocks;  // stack; back() is handed out next
  std::vector<int> queue[2];         // [0] reasoning (high priority), [1] answering (low)
  std::vector<int> selected;
  std::vector<pascal_op> ops;
  std::vector<int32_t> op_blocks;
  bool awaiting_commit = false;
};

}  // namespace

struct pascal_sched {
  pascal_config cfg;
  std::vector<Instance> inst;
  std::vector<Request> req;

  int blocks_for(int tokens) const { return (tokens + cfg.block_tokens - 1) / cfg.block_tokens; }

  // ---- the signals of Section IV-B -------------------------------------------------
  // t_i: the token pacer of every answering request still holds tokens, i.e. by `now`
  // the reader (one token per target_tpot_s since the first) expects no more than exist.
  bool slo_ok(int i, double now) const {
    for (int rid : inst[i].queue[1]) {
      const Request& q = req[rid];
      if (q.phase != PASCAL_ANSWERING || q.answer_times.empty()) continue;
      const double expected = 1.0 + std::floor((now - q.answer_times[0]) / cfg.target_tpot_s);
      if ((double)q.answer_times.size() < expected) return false;
    }
    return true;
  }
  // m_i: KV memory on the GPU and in the host store, plus prompts not yet started.
  int64_t footprint(int i) const {
    int64_t total = 0;
    for (int lvl = 0; lvl < 2; ++lvl)
      for (int rid : inst[i].queue[lvl]) {
        const Request& q = req[rid];
        if (q.state == PASCAL_QUEUED) total += blocks_for(q.prompt);
        else if (q.state == PASCAL_RESIDENT) total += (int64_t)q.blocks.size();
        else total += q.host_blocks;
      }
    return total;
  }
  int reasoning_count(int i) const { return (int)inst[i].queue[0].size(); }
  // a_i: answering requests that have not used up their first quantum.
  int fresh_answering(int i) const {
    int n = 0;
    for (int rid : inst[i].queue[1]) n += req[rid].quanta_done == 0;
    return n;
  }

  // ---- Algorithm 1 ---------------------------------------------------------------------
  int select_for_reasoning(double now) const {
    const int n = cfg.num_instances;
    bool any_ok = false;
    std::vector<char> ok(n);
    for (int i = 0; i < n; ++i) any_ok |= (ok[i] = slo_ok(i, now));
    int best = -1;
    int64_t best_m = 0;
    for (int i = 0; i < n; ++i) {
      if (any_ok && !ok[i]) continue;          // E = compliant instances, or all of them
      const int64_t m = footprint(i);
      if (best < 0 || m < best_m) { best = i; best_m = m; }
    }
    return best;
  }

  // ---- Algorithm 2 ---------------------------------------------------------------------
  int select_for_answering(double now, int current) const {
    const int n = cfg.num_instances;
    bool any_ok = false;
    std::vector<char> ok(n);
    for (int i = 0; i < n; ++i) any_ok |= (ok[i] = slo_ok(i, now));
    std::vector<int> key(n);
    for (int i = 0; i < n; ++i)
      key[i] = reasoning_count(i) + (any_ok ? 0 : fresh_answering(i));
    int best = -1;
    for (int i = 0; i < n; ++i) {
      if (any_ok && !ok[i]) continue;
      if (best < 0 || key[i] < key[best]) best = i;
    }
    // among equal minima the instance the request is on wins: no transfer for nothing
    if ((!any_ok || ok[current]) && key[current] == key[best]) best = current;
    return best;
  }

  // ---- order bookkeeping -----------------------------------------------------------------
  static void remove_from(std::vector<int>& q, int rid) {
    const auto it = std::find(q.begin(), q.end(), rid);
    if (it != q.end()) q.erase(it);
  }

  void push_op(Instance& at, int kind, int instance, int rid, const std::vector<int32_t>& blocks,
               int other = -1, const std::vector<int32_t>* other_blocks = nullptr) {
    pascal_op op{};
    op.kind = kind;
    op.instance = instance;
    op.request = rid;
    op.other_instance = other;
    op.first_block = (int32_t)at.op_blocks.size();
    op.n_blocks = (int32_t)blocks.size();
    at.op_blocks.insert(at.op_blocks.end(), blocks.begin(), blocks.end());
    if (other_blocks) {
      op.n_other_blocks = (int32_t)other_blocks->size();
      at.op_blocks.insert(at.op_blocks.end(), other_blocks->begin(), other_blocks->end());
    }
    at.ops.push_back(op);
  }

  std::vector<int32_t> take_blocks(Instance& ins, int n) {
    std::vector<int32_t> got(n);
    for (int k = 0; k < n; ++k) { got[k] = ins.free_blocks.back(); ins.free_blocks.pop_back(); }
    return got;
  }

  // ---- one iteration of an instance -------------------------------------------------------
  void plan(int i) {
    Instance& ins = inst[i];
    ins.ops.clear();
    ins.op_blocks.clear();
    ins.selected.clear();
    std::vector<int> order(ins.queue[0]);
    order.insert(order.end(), ins.queue[1].begin(), ins.queue[1].end());
    std::vector<char> evicted_now(order.size(), 0);
    // blocks held by resident requests behind the current position: what evictions could free
    int64_t resident_behind = 0;
    for (int rid : order)
      if (req[rid].state == PASCAL_RESIDENT) resident_behind += (int64_t)req[rid].blocks.size();
    for (size_t pos = 0; pos < order.size(); ++pos) {
      const int rid = order[pos];
      Request& q = req[rid];
      if (q.state == PASCAL_RESIDENT) resident_behind -= (int64_t)q.blocks.size();
      if (evicted_now[pos]) continue;
      const int after = q.state == PASCAL_QUEUED ? q.prompt : q.kv_tokens + 1;
      const int extra = blocks_for(after) - (int)q.blocks.size();
      // evict only when that makes the request fit
      if (extra > (int64_t)ins.free_blocks.size() + resident_behind) continue;
      for (size_t b = order.size(); extra > (int)ins.free_blocks.size() && b-- > pos + 1;) {
        Request& v = req[order[b]];
        if (v.state != PASCAL_RESIDENT) continue;
        push_op(ins, PASCAL_OP_OFFLOAD, i, order[b], v.blocks);
        ins.free_blocks.insert(ins.free_blocks.end(), v.blocks.begin(), v.blocks.end());
        resident_behind -= (int64_t)v.blocks.size();
        v.host_blocks = (int)v.blocks.size();
        v.blocks.clear();
        v.state = PASCAL_OFFLOADED;
        ++v.preemptions;
        evicted_now[b] = 1;
      }
      std::vector<int32_t> got = take_blocks(ins, extra);
      if (q.state == PASCAL_QUEUED) {
        push_op(ins, PASCAL_OP_PREFILL, i, rid, got);
      } else if (q.state == PASCAL_OFFLOADED) {
        const int n_old = q.host_blocks;
        push_op(ins, PASCAL_OP_RELOAD, i, rid, std::vector<int32_t>(got.begin(), got.begin() + n_old));
        if (extra > n_old)
          push_op(ins, PASCAL_OP_GROW, i, rid, std::vector<int32_t>(got.begin() + n_old, got.end()));
        q.host_blocks = 0;
        q.state = PASCAL_RESIDENT;
      } else if (extra > 0) {
        push_op(ins, PASCAL_OP_GROW, i, rid, got);
      }
      q.blocks.insert(q.blocks.end(), got.begin(), got.end());
      ins.selected.push_back(rid);
      if (cfg.max_batch && (int)ins.selected.size() == cfg.max_batch) break;
    }
    ins.awaiting_commit = true;
  }

  int context_len_after(const Request& q) const {
    return q.state == PASCAL_QUEUED ? q.prompt : q.kv_tokens + 1;
  }

  // ---- the iteration's tokens ---------------------------------------------------------------
  void phase_transition(Instance& log, int rid, double now) {
    Request& q = req[rid];
    const int cur = q.instance;
    const int sel = (cfg.flags & PASCAL_FLAG_NO_MIGRATION) ? cur : select_for_answering(now, cur);
    int dst = sel;
    if (sel != cur && !(cfg.flags & PASCAL_FLAG_NOT_ADAPTIVE)) {
      // adaptive migration: stay when there is room here and none there
      const bool room_here = (int)inst[cur].free_blocks.size() >= cfg.headroom_blocks;
      const bool room_there =
          (int)inst[sel].free_blocks.size() >= (int)q.blocks.size() + cfg.headroom_blocks;
      if (room_here && !room_there) dst = cur;
    }
    q.phase = PASCAL_ANSWERING;
    q.level = 1;
    q.quantum_used = 0;
    q.quanta_done = 0;
    if (dst != cur) {
      const std::vector<int32_t> src = q.blocks;
      Instance& from = inst[cur];
      Instance& to = inst[dst];
      from.free_blocks.insert(from.free_blocks.end(), src.begin(), src.end());
      if (to.free_blocks.size() >= src.size()) {
        const std::vector<int32_t> got = take_blocks(to, (int)src.size());
        push_op(log, PASCAL_OP_MIGRATE, cur, rid, src, dst, &got);
        q.blocks = got;
      } else {
        push_op(log, PASCAL_OP_MIGRATE_HOST, cur, rid, src, dst);
        q.host_blocks = (int)src.size();
        q.blocks.clear();
        q.state = PASCAL_OFFLOADED;
      }
      q.instance = dst;
      ++q.migrations;
    }
    inst[dst].queue[1].push_back(rid);
  }

  void commit(int i, double now, const int32_t* kinds) {
    Instance& ins = inst[i];
    ins.ops.clear();
    ins.op_blocks.clear();
    for (size_t k = 0; k < ins.selected.size(); ++k) {
      const int rid = ins.selected[k];
      Request& q = req[rid];
      if (q.state == PASCAL_QUEUED) { q.state = PASCAL_RESIDENT; q.kv_tokens = q.prompt; }
      else ++q.kv_tokens;
      if (q.phase == PASCAL_REASONING) ++q.reasoning_tokens;
      else q.answer_times.push_back(now);
      std::vector<int>& queue = ins.queue[q.level];
      if (++q.quantum_used >= cfg.quantum_tokens) {   // quantum used up: to the back of the queue
        q.quantum_used = 0;
        ++q.quanta_done;
        remove_from(queue, rid);
        queue.push_back(rid);
      }
      if (kinds[k] == PASCAL_END_OF_SEQUENCE) {
        remove_from(queue, rid);
        push_op(ins, PASCAL_OP_FREE, i, rid, q.blocks);
        ins.free_blocks.insert(ins.free_blocks.end(), q.blocks.begin(), q.blocks.end());
        q.blocks.clear();
        q.state = PASCAL_FINISHED;
        q.finish = now;
      } else if (kinds[k] == PASCAL_END_OF_REASONING && q.phase == PASCAL_REASONING) {
        remove_from(queue, rid);
        phase_transition(ins, rid, now);
      } else if (q.phase == PASCAL_REASONING && q.level == 0 && q.kv_tokens > cfg.demote_tokens) {
        remove_from(ins.queue[0], rid);           // conditional demotion, Section IV-C
        ins.queue[1].push_back(rid);
        q.level = 1;
        q.quantum_used = 0;
        q.quanta_done = 0;
      }
    }
    ins.selected.clear();
    ins.awaiting_commit = false;
  }

  // Section II-C measure from TPOT alone: token k is read at d_k = max(g_k, d_{k-1} + pace);
  // score = area under the read curve / area under the expected curve up to d_last.
  double qoe(const Request& q) const {
    const std::vector<double>& g = q.answer_times;
    if (g.size() <= 1) return 1.0;
    std::vector<double> d(g.size());
    for (size_t k = 0; k < g.size(); ++k)
      d[k] = k == 0 ? g[0] : std::max(g[k], d[k - 1] + cfg.target_tpot_s);
    const double T = d.back();
    double digested = 0.0, expected = 0.0;
    for (size_t k = 0; k < g.size(); ++k) digested += T - d[k];
    for (size_t k = 0; k < g.size(); ++k) expected += T - (g[0] + (double)k * cfg.target_tpot_s);
    return expected > 0.0 ? digested / expected : 1.0;
  }
};

extern "C" {

const char* pascal_status_string(int status) {
  switch (status) {
    case PASCAL_OK: return "ok";
    case PASCAL_ERR_NULL: return "a required pointer is NULL";
    case PASCAL_ERR_ARG: return "a value is out of range";
    case PASCAL_ERR_STATE: return "plan and commit must alternate on an instance";
    case PASCAL_ERR_CAPACITY: return "an output array is too small, or the prompt cannot fit an instance";
    default: return "unknown status";
  }
}

int pascal_create(const pascal_config* c, pascal_sched** out) {
  if (!c || !out) return PASCAL_ERR_NULL;
  if (c->num_instances < 1 || c->num_instances > 4096 || c->gpu_blocks < 1 || c->block_tokens < 1 ||
      c->quantum_tokens < 1 || c->demote_tokens < 1 || c->headroom_blocks < 0 || c->max_batch < 0 ||
      !(c->target_tpot_s > 0.0) || (c->flags & ~(PASCAL_FLAG_NO_MIGRATION | PASCAL_FLAG_NOT_ADAPTIVE)))
    return PASCAL_ERR_ARG;
  pascal_sched* s = new (std::nothrow) pascal_sched();
  if (!s) return PASCAL_ERR_CAPACITY;
  try {
    s->cfg = *c;
    s->inst.resize(c->num_instances);
    for (Instance& ins : s->inst) {
      ins.free_blocks.resize(c->gpu_blocks);
      for (int b = 0; b < c->gpu_blocks; ++b) ins.free_blocks[b] = c->gpu_blocks - 1 - b;  // lowest id first
    }
  } catch (const std::bad_alloc&) {   // no C++ exception may cross the C boundary
    delete s;
    return PASCAL_ERR_CAPACITY;
  }
  *out = s;
  return PASCAL_OK;
}

void pascal_destroy(pascal_sched* s) { delete s; }

int pascal_submit(pascal_sched* s, int32_t prompt_tokens, double now, int32_t* request,
                  int32_t* instance) {
  if (!s || !request || !instance) return PASCAL_ERR_NULL;
  if (prompt_tokens < 1) return PASCAL_ERR_ARG;
  if (s->blocks_for(prompt_tokens) > s->cfg.gpu_blocks) return PASCAL_ERR_CAPACITY;
  try {
    const int i = s->select_for_reasoning(now);
    Request q;
    q.instance = i;
    q.prompt = prompt_tokens;
    q.arrival = now;
    s->inst[i].queue[0].reserve(s->inst[i].queue[0].size() + 1);
    s->req.push_back(q);
    const int rid = (int)s->req.size() - 1;
    s->inst[i].queue[0].push_back(rid);
    *request = rid;
    *instance = i;
  } catch (const std::bad_alloc&) {
    return PASCAL_ERR_CAPACITY;
  }
  return PASCAL_OK;
}

static bool bad_instance(const pascal_sched* s, int32_t i) { return i < 0 || i >= s->cfg.num_instances; }

int pascal_plan(pascal_sched* s, int32_t instance, int32_t* n_selected, int32_t* n_ops,
                int32_t* n_op_blocks) {
  if (!s || !n_selected || !n_ops || !n_op_blocks) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance)) return PASCAL_ERR_ARG;
  if (s->inst[instance].awaiting_commit) return PASCAL_ERR_STATE;
  try {
    s->plan(instance);
  } catch (const std::bad_alloc&) {   // host memory exhausted: the scheduler state is no longer usable
    return PASCAL_ERR_CAPACITY;
  }
  const Instance& ins = s->inst[instance];
  *n_selected = (int32_t)ins.selected.size();
  *n_ops = (int32_t)ins.ops.size();
  *n_op_blocks = (int32_t)ins.op_blocks.size();
  return PASCAL_OK;
}

int pascal_plan_batch(const pascal_sched* s, int32_t instance, int32_t* requests,
                      int32_t* context_lens, int32_t capacity) {
  if (!s) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance)) return PASCAL_ERR_ARG;
  const Instance& ins = s->inst[instance];
  if (!ins.awaiting_commit) return PASCAL_ERR_STATE;
  if ((int)ins.selected.size() > capacity) return PASCAL_ERR_CAPACITY;
  if (!ins.selected.empty() && (!requests || !context_lens)) return PASCAL_ERR_NULL;
  for (size_t k = 0; k < ins.selected.size(); ++k) {
    requests[k] = ins.selected[k];
    context_lens[k] = s->context_len_after(s->req[ins.selected[k]]);
  }
  return PASCAL_OK;
}

int pascal_plan_block_tables(const pascal_sched* s, int32_t instance, int32_t* block_tables,
                             int32_t max_blocks_per_seq, int32_t fill) {
  if (!s) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance) || max_blocks_per_seq < 1) return PASCAL_ERR_ARG;
  const Instance& ins = s->inst[instance];
  if (!ins.awaiting_commit) return PASCAL_ERR_STATE;
  if (!ins.selected.empty() && !block_tables) return PASCAL_ERR_NULL;
  for (int rid : ins.selected)
    if ((int)s->req[rid].blocks.size() > max_blocks_per_seq) return PASCAL_ERR_CAPACITY;
  for (size_t k = 0; k < ins.selected.size(); ++k) {
    const std::vector<int32_t>& b = s->req[ins.selected[k]].blocks;
    int32_t* row = block_tables + (size_t)k * max_blocks_per_seq;
    std::copy(b.begin(), b.end(), row);
    std::fill(row + b.size(), row + max_blocks_per_seq, fill);
  }
  return PASCAL_OK;
}

int pascal_ops(const pascal_sched* s, int32_t instance, pascal_op* ops, int32_t op_capacity,
               int32_t* blocks, int32_t block_capacity) {
  if (!s) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance)) return PASCAL_ERR_ARG;
  const Instance& ins = s->inst[instance];
  if ((int)ins.ops.size() > op_capacity || (int)ins.op_blocks.size() > block_capacity)
    return PASCAL_ERR_CAPACITY;
  if ((!ins.ops.empty() && !ops) || (!ins.op_blocks.empty() && !blocks)) return PASCAL_ERR_NULL;
  std::copy(ins.ops.begin(), ins.ops.end(), ops);
  std::copy(ins.op_blocks.begin(), ins.op_blocks.end(), blocks);
  return PASCAL_OK;
}

int pascal_commit(pascal_sched* s, int32_t instance, double now, const int32_t* token_kinds,
                  int32_t n, int32_t* n_ops, int32_t* n_op_blocks) {
  if (!s || !n_ops || !n_op_blocks) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance)) return PASCAL_ERR_ARG;
  Instance& ins = s->inst[instance];
  if (!ins.awaiting_commit) return PASCAL_ERR_STATE;
  if (n != (int32_t)ins.selected.size()) return PASCAL_ERR_ARG;
  if (n > 0 && !token_kinds) return PASCAL_ERR_NULL;
  for (int32_t k = 0; k < n; ++k)
    if (token_kinds[k] < PASCAL_TOKEN || token_kinds[k] > PASCAL_END_OF_SEQUENCE) return PASCAL_ERR_ARG;
  try {
    s->commit(instance, now, token_kinds);
  } catch (const std::bad_alloc&) {
    return PASCAL_ERR_CAPACITY;
  }
  *n_ops = (int32_t)ins.ops.size();
  *n_op_blocks = (int32_t)ins.op_blocks.size();
  return PASCAL_OK;
}

int pascal_instance_signals(const pascal_sched* s, int32_t instance, double now, int32_t* t,
                            int64_t* m, int32_t* r, int32_t* a, int32_t* free_blocks) {
  if (!s) return PASCAL_ERR_NULL;
  if (bad_instance(s, instance)) return PASCAL_ERR_ARG;
  if (t) *t = s->slo_ok(instance, now) ? 1 : 0;
  if (m) *m = s->footprint(instance);
  if (r) *r = s->reasoning_count(instance);
  if (a) *a = s->fresh_answering(instance);
  if (free_blocks) *free_blocks = (int32_t)s->inst[instance].free_blocks.size();
  return PASCAL_OK;
}

int pascal_request(const pascal_sched* s, int32_t request, pascal_request_info* out) {
  if (!s || !out) return PASCAL_ERR_NULL;
  if (request < 0 || request >= (int32_t)s->req.size()) return PASCAL_ERR_ARG;
  const Request& q = s->req[request];
  pascal_request_info o{};
  o.instance = q.instance;
  o.phase = q.phase;
  o.state = q.state;
  o.level = q.level;
  o.prompt_tokens = q.prompt;
  o.kv_tokens = q.kv_tokens;
  o.reasoning_tokens = q.reasoning_tokens;
  o.answering_tokens = (int32_t)q.answer_times.size();
  o.n_blocks = (int32_t)q.blocks.size();
  o.preemptions = q.preemptions;
  o.migrations = q.migrations;
  o.arrival = q.arrival;
  o.finish = q.finish;
  o.ttft = q.answer_times.empty() ? -1.0 : q.answer_times[0] - q.arrival;
  o.qoe = s->qoe(q);
  *out = o;
  return PASCAL_OK;
}

int pascal_request_visible_tokens(const pascal_sched* s, int32_t request, double now,
                                  int32_t* visible) {
  if (!s || !visible) return PASCAL_ERR_NULL;
  if (request < 0 || request >= (int32_t)s->req.size()) return PASCAL_ERR_ARG;
  const std::vector<double>& g = s->req[request].answer_times;
  int32_t n = 0;
  double d = 0.0;
  for (size_t k = 0; k < g.size(); ++k) {
    d = k == 0 ? g[0] : std::max(g[k], d + s->cfg.target_tpot_s);
    if (d > now) break;   // the release times only grow
    ++n;
  }
  *visible = n;
  return PASCAL_OK;
}

int pascal_request_blocks(const pascal_sched* s, int32_t request, int32_t* blocks, int32_t capacity) {
  if (!s) return PASCAL_ERR_NULL;
  if (request < 0 || request >= (int32_t)s->req.size()) return PASCAL_ERR_ARG;
  const std::vector<int32_t>& b = s->req[request].blocks;
  if ((int)b.size() > capacity) return PASCAL_ERR_CAPACITY;
  if (!b.empty() && !blocks) return PASCAL_ERR_NULL;
  std::copy(b.begin(), b.end(), blocks);
  return (int)b.size();
}

}  // extern "C"
